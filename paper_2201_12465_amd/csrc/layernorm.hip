// LayerNorm forward and backward over the last dimension, one wavefront per row.
//
// A normalisation layer is one of the paper's neural-network primitives
// (Section 4.2), composed from elementwise and reduction tensor primitives
// (Section 4.1.1) that its backend fuses to raise arithmetic intensity; here
// the whole operator is one kernel per direction.  HBM traffic is the
// algorithmic minimum: forward reads x and writes y (+ 8 bytes of statistics
// per row); backward reads dy, x (and the skip gradient if there is one) and
// writes dx, with the three column reductions (dgamma, dbeta, and the column
// sums of dx that form the bias gradient of the linear layer feeding x) kept
// in registers across the rows a wavefront walks and folded through LDS to
// one partial row per workgroup.
//
// Lane l owns the 16-byte column chunks l, l+64, l+128, ... of a row, so
// every global access is a coalesced 1 KiB line per wavefront and a lane's
// columns never change from row to row.
#include "devutil.h"
#include "kernels.h"

namespace fl {
namespace {

// 16 raw bytes of a row: VEC elements of either type, converted only when the row's turn comes.
template <typename T> __device__ __forceinline__ void unpack16(const uint4 &r, float *v);
template <> __device__ __forceinline__ void unpack16<float>(const uint4 &r, float *v) {
  v[0] = __uint_as_float(r.x); v[1] = __uint_as_float(r.y); v[2] = __uint_as_float(r.z); v[3] = __uint_as_float(r.w);
}
template <> __device__ __forceinline__ void unpack16<bf16_t>(const uint4 &r, float *v) {
  const bf16x8_t t = __builtin_bit_cast(bf16x8_t, r);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = static_cast<float>(t[e]);
}

// Wave w of the grid takes rows w, w + nwaves, ...: the next row's chunks are requested before the
// current row is reduced, so that a wave always has a row in flight.
template <typename T, int NCH>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T *__restrict__ x, const T *__restrict__ gamma,
                                                     const T *__restrict__ beta, float eps, int M, int D, int nwaves,
                                                     T *__restrict__ y, float *__restrict__ mean,
                                                     float *__restrict__ rstd) {
  constexpr int VEC = Elem<T>::VEC;
  const int lane = threadIdx.x & 63;
  int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= nwaves) return;
  const int nchunks = D / VEC;
  const float invD = 1.0f / D;
  uint4 nxt[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    nxt[i] = make_uint4(0, 0, 0, 0);
    if (c < nchunks) nxt[i] = *reinterpret_cast<const uint4 *>(x + (size_t)m * D + c * VEC);
  }
  float g[NCH][VEC], b[NCH][VEC];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
#pragma unroll
    for (int e = 0; e < VEC; ++e) g[i][e] = 0.f, b[i][e] = 0.f;
    if (c < nchunks) {
      VecIO<T, VEC>::load(gamma + c * VEC, g[i]);
      VecIO<T, VEC>::load(beta + c * VEC, b[i]);
    }
  }
  for (; m < M; m += nwaves) {
    float v[NCH][VEC];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      unpack16<T>(nxt[i], v[i]);   // zeros beyond the row
#pragma unroll
      for (int e = 0; e < VEC; ++e) s += v[i][e];
    }
    const int mn = m + nwaves;
    if (mn < M) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = lane + 64 * i;
        if (c < nchunks) nxt[i] = *reinterpret_cast<const uint4 *>(x + (size_t)mn * D + c * VEC);
      }
    }
    const float mu = wave_sum(s) * invD;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      if (lane + 64 * i < nchunks) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          float d = v[i][e] - mu;
          q += d * d;
        }
      }
    }
    const float rs = rsqrtf(wave_sum(q) * invD + eps);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunks) {
        float o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = (v[i][e] - mu) * rs * g[i][e] + b[i][e];
        VecIO<T, VEC>::store(y + (size_t)m * D + c * VEC, o);
      }
    }
    if (lane == 0) {
      mean[m] = mu;
      rstd[m] = rs;
    }
  }
}

// Workgroup b walks rows b*rows_per_wg .. ; wave w takes rows w, w+nw, ... of that range, two at a
// time so that twice as many loads are in flight.  The three column partials live in registers and
// are folded across the waves through LDS, one quantity at a time, by all threads.
// Rows wider than 1024 elements (ln_bwd_wide) run with four wavefronts per workgroup and one row per
// wavefront in flight: a lane then holds up to 64 elements of each of seven row-length quantities, which
// needs the register budget of one wavefront per SIMD.
template <typename T, int NCH> constexpr bool ln_bwd_wide() { return NCH * Elem<T>::VEC > 16; }

template <typename T, int NCH>
__global__ __launch_bounds__((NCH * Elem<T>::VEC > 16) ? 256 : 512) void ln_bwd_kernel(const T *__restrict__ dy, const T *__restrict__ x,
                                                     const float *__restrict__ mean, const float *__restrict__ rstd,
                                                     const T *__restrict__ gamma, const T *__restrict__ add, int M,
                                                     int D, int rows_per_wg, T *__restrict__ dx,
                                                     float *__restrict__ ws) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int R = ln_bwd_wide<T, NCH>() ? 1 : 2;
  extern __shared__ float red[];  // [nw][D]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int nchunks = D / VEC;
  const float invD = 1.0f / D;
  float gam[NCH][VEC], pg[NCH][VEC], pb[NCH][VEC], px[NCH][VEC];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
#pragma unroll
    for (int e = 0; e < VEC; ++e) gam[i][e] = 0.f, pg[i][e] = 0.f, pb[i][e] = 0.f, px[i][e] = 0.f;
    if (c < nchunks) VecIO<T, VEC>::load(gamma + c * VEC, gam[i]);
  }
  const int m0 = blockIdx.x * rows_per_wg, m1 = min(M, m0 + rows_per_wg);
  for (int mb = m0 + wave; mb < m1; mb += R * nw) {
    float d[R][NCH][VEC], xv[R][NCH][VEC], av[R][NCH][VEC], mu[R], rs[R];
    bool ok[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      const int m = mb + rr * nw;
      ok[rr] = m < m1;
      mu[rr] = ok[rr] ? mean[m] : 0.f;
      rs[rr] = ok[rr] ? rstd[m] : 0.f;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = lane + 64 * i;
        if (ok[rr] && c < nchunks) {
          VecIO<T, VEC>::load(dy + (size_t)m * D + c * VEC, d[rr][i]);
          VecIO<T, VEC>::load(x + (size_t)m * D + c * VEC, xv[rr][i]);
          if (add) VecIO<T, VEC>::load(add + (size_t)m * D + c * VEC, av[rr][i]);
        } else {
#pragma unroll
          for (int e = 0; e < VEC; ++e) d[rr][i][e] = 0.f, xv[rr][i][e] = mu[rr];
        }
        if (!add || !(ok[rr] && c < nchunks)) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) av[rr][i][e] = 0.f;
        }
      }
    }
    float s1[R], s2[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      s1[rr] = 0.f, s2[rr] = 0.f;
#pragma unroll
      for (int i = 0; i < NCH; ++i)
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float xh = (xv[rr][i][e] - mu[rr]) * rs[rr];
          const float g = d[rr][i][e] * gam[i][e];
          xv[rr][i][e] = xh;   // keep xhat
          s1[rr] += g;
          s2[rr] += g * xh;
          pg[i][e] += d[rr][i][e] * xh;
          pb[i][e] += d[rr][i][e];
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
#pragma unroll
      for (int rr = 0; rr < R; ++rr) {
        s1[rr] += __shfl_xor(s1[rr], o, 64);
        s2[rr] += __shfl_xor(s2[rr], o, 64);
      }
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      const int m = mb + rr * nw;
      const float a1 = s1[rr] * invD, a2 = s2[rr] * invD;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = lane + 64 * i;
        float o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          o[e] = rs[rr] * (d[rr][i][e] * gam[i][e] - a1 - xv[rr][i][e] * a2) + av[rr][i][e];
          px[i][e] += o[e];
        }
        if (ok[rr] && c < nchunks) VecIO<T, VEC>::store(dx + (size_t)m * D + c * VEC, o);
      }
    }
  }
  // fold the waves' partial rows through LDS: wave w writes row w, then every thread sums columns
  float *out = ws + (size_t)blockIdx.x * 3 * D;
#pragma unroll
  for (int qn = 0; qn < 3; ++qn) {
    float(*p)[VEC] = qn == 0 ? pg : (qn == 1 ? pb : px);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunks)
#pragma unroll
        for (int e = 0; e < VEC; ++e) red[(size_t)wave * D + c * VEC + e] = p[i][e];
    }
    __syncthreads();
    for (int col = threadIdx.x; col < D; col += blockDim.x) {
      float a = 0.f;
      for (int w = 0; w < nw; ++w) a += red[(size_t)w * D + col];
      out[(size_t)qn * D + col] = a;
    }
    __syncthreads();
  }
}

// Rows of at most 1024 elements: 8 wavefronts per workgroup, wave w takes rows w, w + 8, ... of the
// workgroup's range, one row per turn.  The raw 16-byte chunks of the next PF rows (dy, x, the skip
// gradient, and the two row statistics) are requested before the current row is reduced, so that a
// wavefront always has PF rows in flight while it computes; a lane holds at most 16 elements of a row.
template <typename T, int NCH, bool ADD>
__global__ __launch_bounds__(512) void ln_bwd_rows_kernel(const T *__restrict__ dy, const T *__restrict__ x,
                                                          const float *__restrict__ mean,
                                                          const float *__restrict__ rstd, const T *__restrict__ gamma,
                                                          const T *__restrict__ add, int M, int D, int rows_per_wg,
                                                          T *__restrict__ dx, float *__restrict__ ws) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int PF = 3, NW = 8;
  extern __shared__ float red[];  // [NW][3][D]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nchunks = D / VEC;
  const float invD = 1.0f / D;
  float gam[NCH][VEC], pg[NCH][VEC], pb[NCH][VEC], px[NCH][VEC];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
#pragma unroll
    for (int e = 0; e < VEC; ++e) gam[i][e] = 0.f, pg[i][e] = 0.f, pb[i][e] = 0.f, px[i][e] = 0.f;
    if (c < nchunks) VecIO<T, VEC>::load(gamma + c * VEC, gam[i]);
  }
  const int m0 = blockIdx.x * rows_per_wg, m1 = min(M, m0 + rows_per_wg);
  uint4 rdy[PF][NCH], rx[PF][NCH], radd[PF][ADD ? NCH : 1];
  float rmu[PF], rrs[PF];
  auto request = [&](int slot, int m) {
    const bool ok = m < m1;
    rmu[slot] = ok ? mean[m] : 0.f;
    rrs[slot] = ok ? rstd[m] : 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      rdy[slot][i] = make_uint4(0, 0, 0, 0);
      rx[slot][i] = make_uint4(0, 0, 0, 0);
      if (ADD) radd[slot][i] = make_uint4(0, 0, 0, 0);
      if (ok && c < nchunks) {
        const size_t off = (size_t)m * D + c * VEC;
        rdy[slot][i] = *reinterpret_cast<const uint4 *>(dy + off);
        rx[slot][i] = *reinterpret_cast<const uint4 *>(x + off);
        if (ADD) radd[slot][i] = *reinterpret_cast<const uint4 *>(add + off);
      }
    }
  };
#pragma unroll
  for (int k = 0; k < PF; ++k) request(k, m0 + wave + k * NW);
  for (int m = m0 + wave; m < m1; m += NW) {
    // take the oldest row out of the queue, move the others up, ask for the row PF turns ahead
    float d[NCH][VEC], xh[NCH][VEC], av[NCH][VEC];
    const float mu = rmu[0], rs = rrs[0];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      unpack16<T>(rdy[0][i], d[i]);
      unpack16<T>(rx[0][i], xh[i]);
      if (ADD) unpack16<T>(radd[0][i], av[i]);
    }
#pragma unroll
    for (int k = 0; k + 1 < PF; ++k) {
      rmu[k] = rmu[k + 1];
      rrs[k] = rrs[k + 1];
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        rdy[k][i] = rdy[k + 1][i];
        rx[k][i] = rx[k + 1][i];
        if (ADD) radd[k][i] = radd[k + 1][i];
      }
    }
    request(PF - 1, m + PF * NW);
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const bool in = lane + 64 * i < nchunks;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float h = in ? (xh[i][e] - mu) * rs : 0.f;   // zero beyond the row: its raw chunk reads as 0, not as the mean
        const float g = d[i][e] * gam[i][e];
        xh[i][e] = h;
        s1 += g;
        s2 += g * h;
        pg[i][e] += d[i][e] * h;
        pb[i][e] += d[i][e];
      }
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    const float a1 = s1 * invD, a2 = s2 * invD;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      float o[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        o[e] = rs * (d[i][e] * gam[i][e] - a1 - xh[i][e] * a2) + (ADD ? av[i][e] : 0.f);
        if (c >= nchunks) o[e] = 0.f;
        px[i][e] += o[e];
      }
      if (c < nchunks) VecIO<T, VEC>::store(dx + (size_t)m * D + c * VEC, o);
    }
  }
  // fold the waves' partial rows through LDS in one pass: wave w writes its three rows (16-byte pieces:
  // no two lanes of a quarter-wave on one bank), then every thread sums columns of [3][D]
  float *out = ws + (size_t)blockIdx.x * 3 * D;
#pragma unroll
  for (int qn = 0; qn < 3; ++qn) {
    float(*p)[VEC] = qn == 0 ? pg : (qn == 1 ? pb : px);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunks)
#pragma unroll
        for (int e = 0; e < VEC; e += 4)
          *reinterpret_cast<float4 *>(red + ((size_t)wave * 3 + qn) * D + c * VEC + e) =
              make_float4(p[i][e], p[i][e + 1], p[i][e + 2], p[i][e + 3]);
    }
  }
  __syncthreads();
  for (int col = threadIdx.x; col < 3 * D; col += NW * 64) {
    float a = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) a += red[(size_t)w * 3 * D + col];
    out[col] = a;
  }
}

int ln_waves(int D) { return D <= 1024 ? 8 : 4; }  // must match ln_bwd_wide: 256 threads for wide rows

template <typename T>
hipError_t ln_fwd_t(const void *x, const void *g, const void *b, float eps, int M, int D, void *y, float *mean,
                    float *rstd, hipStream_t s) {
  constexpr int VEC = Elem<T>::VEC;
  const int nch = (D / VEC + 63) / 64;
  // as many waves as the chip holds at once (8 per SIMD), every wave the same number of rows
  const int rows_per_wave = (M + 8191) / 8192;
  const int nwaves = (M + rows_per_wave - 1) / rows_per_wave;
  dim3 grid((nwaves + 3) / 4), block(256);
#define FL_LN_FWD(N)                                                                                        \
  hipLaunchKernelGGL((ln_fwd_kernel<T, N>), grid, block, 0, s, static_cast<const T *>(x),                   \
                     static_cast<const T *>(g), static_cast<const T *>(b), eps, M, D, nwaves,              \
                     static_cast<T *>(y), mean, rstd)
  if (nch <= 1) FL_LN_FWD(1);
  else if (nch <= 2) FL_LN_FWD(2);
  else if (nch <= 4) FL_LN_FWD(4);
  else if (nch <= 8) FL_LN_FWD(8);
  else if (nch <= 16) FL_LN_FWD(16);
  else return hipErrorInvalidValue;
#undef FL_LN_FWD
  return hipGetLastError();
}

template <typename T>
hipError_t ln_bwd_t(const void *dy, const void *x, const float *mean, const float *rstd, const void *g,
                    const void *add, int M, int D, void *dx, float *ws, hipStream_t s) {
  constexpr int VEC = Elem<T>::VEC;
  const int nch = (D / VEC + 63) / 64;
  const int nw = ln_waves(D);
  const int parts = ln_bwd_parts(M, D);
  const int rows_per_wg = (M + parts - 1) / parts;
  dim3 grid(parts), block(64 * nw);
  const size_t lds = (size_t)nw * D * sizeof(float) * (nch * VEC <= 16 ? 3 : 1);  // the pipelined kernel folds all three sums at once
#define FL_LN_ROWS(N, A)                                                                                      \
  do {                                                                                                        \
    auto kern = ln_bwd_rows_kernel<T, N, A>;                                                                  \
    static bool raised = false;                                                                               \
    if (lds > 64 * 1024 && !raised) { /* more dynamic LDS than the default limit: allow the CU's 160 KB */    \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                                \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);             \
      if (e != hipSuccess) return e;                                                                          \
      raised = true;                                                                                          \
    }                                                                                                         \
    hipLaunchKernelGGL(kern, grid, block, lds, s, static_cast<const T *>(dy), static_cast<const T *>(x),      \
                       mean, rstd, static_cast<const T *>(g), static_cast<const T *>(add), M, D, rows_per_wg, \
                       static_cast<T *>(dx), ws);                                                             \
  } while (0)
#define FL_LN_BWD(N)                                                                                          \
  hipLaunchKernelGGL((ln_bwd_kernel<T, N>), grid, block, lds, s, static_cast<const T *>(dy),                  \
                     static_cast<const T *>(x), mean, rstd, static_cast<const T *>(g),                        \
                     static_cast<const T *>(add), M, D, rows_per_wg, static_cast<T *>(dx), ws)
  if (nch * VEC <= 16) {  // at most 16 elements of a row per lane: the pipelined kernel
    if (nch <= 1) { if (add) FL_LN_ROWS(1, true); else FL_LN_ROWS(1, false); }
    else if (nch <= 2) { if (add) FL_LN_ROWS(2, true); else FL_LN_ROWS(2, false); }
    else if constexpr (VEC == 4) { if (add) FL_LN_ROWS(4, true); else FL_LN_ROWS(4, false); }
  }
  else if (nch <= 4) FL_LN_BWD(4);
  else if (nch <= 8) FL_LN_BWD(8);
  else if (nch <= 16) FL_LN_BWD(16);
  else return hipErrorInvalidValue;
#undef FL_LN_BWD
#undef FL_LN_ROWS
  return hipGetLastError();
}

}  // namespace

int ln_bwd_parts(int M, int D) {
  const int nw = ln_waves(D);
  int parts = (M + 2 * nw - 1) / (2 * nw);  // at least two rows per wave
  // At most 160 workgroups, not one per CU: alone the kernel is 3 % slower with them (11.9 against 11.5 us on
  // 4096 x 768), but inside the backward pass it runs beside a weight-gradient GEMM of the other stream, and
  // leaving that kernel 96 CUs to itself is worth more (BERT-base step 0.381 -> 0.375 ms with 128-160, speech
  // and ViT shapes -0.7 % and -0.9 % with 144-192; 512 workgroups: +0.8 % on those two).
  if (parts > 160) parts = 160;
  const int rows = (M + parts - 1) / parts;
  return (M + rows - 1) / rows;  // no empty workgroup
}

hipError_t launch_layernorm_fwd(int dt, const void *x, const void *gamma, const void *beta, float eps, int M, int D,
                                void *y, float *mean, float *rstd, hipStream_t stream) {
  if (!x || !gamma || !beta || !y || !mean || !rstd || M < 1 || D < 8 || D % 8 || D > 4096)
    return hipErrorInvalidValue;
  return dt == DT_F32 ? ln_fwd_t<float>(x, gamma, beta, eps, M, D, y, mean, rstd, stream)
                      : ln_fwd_t<bf16_t>(x, gamma, beta, eps, M, D, y, mean, rstd, stream);
}

hipError_t launch_layernorm_bwd(int dt, const void *dy, const void *x, const float *mean, const float *rstd,
                                const void *gamma, const void *add, int M, int D, void *dx, float *ws,
                                hipStream_t stream) {
  if (!dy || !x || !mean || !rstd || !gamma || !dx || !ws || M < 1 || D < 8 || D % 8 || D > 4096)
    return hipErrorInvalidValue;
  return dt == DT_F32 ? ln_bwd_t<float>(dy, x, mean, rstd, gamma, add, M, D, dx, ws, stream)
                      : ln_bwd_t<bf16_t>(dy, x, mean, rstd, gamma, add, M, D, dx, ws, stream);
}

}  // namespace fl
