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

template <typename T, int NCH>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T *__restrict__ x, const T *__restrict__ gamma,
                                                     const T *__restrict__ beta, float eps, int M, int D,
                                                     T *__restrict__ y, float *__restrict__ mean,
                                                     float *__restrict__ rstd) {
  constexpr int VEC = Elem<T>::VEC;
  const int lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= M) return;
  const int nchunks = D / VEC;
  float v[NCH][VEC];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < nchunks) {
      VecIO<T, VEC>::load(x + (size_t)m * D + c * VEC, v[i]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) s += v[i][e];
    }
  }
  const float mu = wave_sum(s) / D;
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
  const float rs = rsqrtf(wave_sum(q) / D + eps);
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < nchunks) {
      float g[VEC], b[VEC], o[VEC];
      VecIO<T, VEC>::load(gamma + c * VEC, g);
      VecIO<T, VEC>::load(beta + c * VEC, b);
#pragma unroll
      for (int e = 0; e < VEC; ++e) o[e] = (v[i][e] - mu) * rs * g[e] + b[e];
      VecIO<T, VEC>::store(y + (size_t)m * D + c * VEC, o);
    }
  }
  if (lane == 0) {
    mean[m] = mu;
    rstd[m] = rs;
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

int ln_waves(int D) { return D <= 1024 ? 8 : 4; }  // must match ln_bwd_wide: 256 threads for wide rows

template <typename T>
hipError_t ln_fwd_t(const void *x, const void *g, const void *b, float eps, int M, int D, void *y, float *mean,
                    float *rstd, hipStream_t s) {
  constexpr int VEC = Elem<T>::VEC;
  const int nch = (D / VEC + 63) / 64;
  dim3 grid((M + 3) / 4), block(256);
#define FL_LN_FWD(N)                                                                                        \
  hipLaunchKernelGGL((ln_fwd_kernel<T, N>), grid, block, 0, s, static_cast<const T *>(x),                   \
                     static_cast<const T *>(g), static_cast<const T *>(b), eps, M, D, static_cast<T *>(y), \
                     mean, rstd)
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
  const size_t lds = (size_t)nw * D * sizeof(float);
#define FL_LN_BWD(N)                                                                                          \
  hipLaunchKernelGGL((ln_bwd_kernel<T, N>), grid, block, lds, s, static_cast<const T *>(dy),                  \
                     static_cast<const T *>(x), mean, rstd, static_cast<const T *>(g),                        \
                     static_cast<const T *>(add), M, D, rows_per_wg, static_cast<T *>(dx), ws)
  if (nch <= 1) FL_LN_BWD(1);
  else if (nch <= 2) FL_LN_BWD(2);
  else if (nch <= 4) FL_LN_BWD(4);
  else if (nch <= 8) FL_LN_BWD(8);
  else if (nch <= 16) FL_LN_BWD(16);
  else return hipErrorInvalidValue;
#undef FL_LN_BWD
  return hipGetLastError();
}

}  // namespace

int ln_bwd_parts(int M, int D) {
  const int nw = ln_waves(D);
  int parts = (M + 2 * nw - 1) / (2 * nw);  // at least two rows per wave
  if (parts > 256) parts = 256;
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
