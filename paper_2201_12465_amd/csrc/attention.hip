// Masked scaled-dot-product attention, forward and backward, with the score and
// probability matrices kept on chip (never written to HBM).
//
// In the paper's terms this is a chain of tensor primitives -- two matmuls, a
// scale, a max/exp/sum softmax (Section 4.1.1) -- fused into one operator with a
// hand-written gradient function (Section 4.2; Section 5.2.1 "pre-fused gradient
// computation for common sequences").  The softmax is computed online over key
// tiles of 64 (running row maximum and row sum), so any sequence length fits;
// masked keys (j >= length; with the causal mask also j > i) are never visited or
// get probability exactly 0.  The backward pass recomputes the probabilities from
// the saved log-sum-exp:  P = exp(S - LSE), dV = P^T dO, dP = dO V^T,
// dS = P (dP - delta), delta_i = sum_d dO_i O_i, dQ = dS K / sqrt(dh),
// dK = dS^T Q / sqrt(dh).
//
// This file holds the general kernels (any element type and head size, fp32 arithmetic on
// the vector ALUs; the matrix-core kernels of attention_mfma*.hip take the common cases): one wavefront per query row (forward, dQ) or per key row (dK, dV).
#include "devutil.h"
#include "kernels.h"
#include "philox.h"

namespace fl {
namespace {

constexpr int ROWS_PER_WG = 16;  // rows a workgroup of 4 waves walks (4 per wave)
constexpr int MAX_DH = 256;

template <typename T>
__device__ __forceinline__ float dot_row(const float *__restrict__ s, const T *__restrict__ g, int dh) {
  constexpr int VEC = Elem<T>::VEC;
  float a = 0.f;
  for (int d = 0; d < dh; d += VEC) {
    float v[VEC];
    VecIO<T, VEC>::load(g + d, v);
#pragma unroll
    for (int e = 0; e < VEC; ++e) a += s[d + e] * v[e];
  }
  return a;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_rows(const T *__restrict__ qkv, const int32_t *__restrict__ lengths,
                                                     int causal, DropSpec drop, int Tn, int H, int dh, float scale,
                                                     T *__restrict__ o, float *__restrict__ lse) {
  __shared__ float sq[4][MAX_DH];
  __shared__ float sp[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.z, h = blockIdx.y;
  const int D = H * dh, ld = 3 * D;
  const int len = lengths ? min(max(lengths[b], 1), Tn) : Tn;  // a length outside 1..T is treated as the nearest valid one
  const T *base = qkv + (size_t)b * Tn * ld;
  for (int r = 0; r < ROWS_PER_WG / 4; ++r) {
    const int iw = blockIdx.x * ROWS_PER_WG + r * 4 + wave;
    const bool active = iw < Tn;
    const int i = active ? iw : Tn - 1;
    __syncthreads();
    for (int d = lane; d < dh; d += 64) sq[wave][d] = to_f32(base[(size_t)i * ld + h * dh + d]) * scale;
    __syncthreads();
    float mrun = -INFINITY, lrun = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
    // keys this row may see, and the (workgroup-uniform) end of the key loop for the four rows of this round
    const int lim = causal ? min(len, i + 1) : len;
    const int jend = causal ? min(len, min(Tn, blockIdx.x * ROWS_PER_WG + r * 4 + 4)) : len;
    for (int j0 = 0; j0 < jend; j0 += 64) {
      const int j = j0 + lane;
      float s = -INFINITY;
      if (j < lim) s = dot_row<T>(sq[wave], base + (size_t)j * ld + D + h * dh, dh);
      // the first tile holds key 0, which every row may see: mnew is finite from then on
      const float mnew = fmaxf(mrun, wave_max(s));
      const float p = j < lim ? __expf(s - mnew) : 0.f;
      const float corr = __expf(mrun - mnew);
      lrun = lrun * corr + wave_sum(p);   // the softmax denominator ignores dropout
      mrun = mnew;
      sp[wave][lane] = (drop.thr && j < lim) ? p * drop_keep1(drop, j, i, b * H + h) : p;
      __syncthreads();
      const int nj = min(64, jend - j0);
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[c] *= corr;
      for (int jj = 0; jj < nj; ++jj) {
        const float pj = sp[wave][jj];
        const T *vrow = base + (size_t)(j0 + jj) * ld + 2 * D + h * dh;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int d = lane + 64 * c;
          if (d < dh) acc[c] += pj * to_f32(vrow[d]);
        }
      }
      __syncthreads();
    }
    if (active) {
      const float inv = 1.0f / lrun;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int d = lane + 64 * c;
        if (d < dh) o[((size_t)b * Tn + i) * D + h * dh + d] = from_f32<T>(acc[c] * inv);
      }
      if (lane == 0) lse[((size_t)b * H + h) * Tn + i] = mrun + __logf(lrun);
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_rows(const T *__restrict__ qkv, const T *__restrict__ o,
                                                        const T *__restrict__ dout, const float *__restrict__ lse,
                                                        const int32_t *__restrict__ lengths, int causal,
                                                        DropSpec drop, int Tn, int H, int dh, float scale,
                                                        T *__restrict__ dqkv, const float *__restrict__ delta) {
  __shared__ float sq[4][MAX_DH];
  __shared__ float sdo[4][MAX_DH];
  __shared__ float sp[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.z, h = blockIdx.y;
  const int D = H * dh, ld = 3 * D;
  const int len = lengths ? min(max(lengths[b], 1), Tn) : Tn;  // a length outside 1..T is treated as the nearest valid one
  const T *base = qkv + (size_t)b * Tn * ld;
  for (int r = 0; r < ROWS_PER_WG / 4; ++r) {
    const int iw = blockIdx.x * ROWS_PER_WG + r * 4 + wave;
    const bool active = iw < Tn;
    const int i = active ? iw : Tn - 1;
    const size_t orow = ((size_t)b * Tn + i) * D + h * dh;
    __syncthreads();
    for (int d = lane; d < dh; d += 64) {
      sq[wave][d] = to_f32(base[(size_t)i * ld + h * dh + d]) * scale;
      sdo[wave][d] = to_f32(dout[orow + d]);
    }
    const float L = lse[((size_t)b * H + h) * Tn + i];
    const float dl = delta[((size_t)b * H + h) * Tn + i];
    __syncthreads();
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const int lim = causal ? min(len, i + 1) : len;
    const int jend = causal ? min(len, min(Tn, blockIdx.x * ROWS_PER_WG + r * 4 + 4)) : len;
    for (int j0 = 0; j0 < jend; j0 += 64) {
      const int j = j0 + lane;
      float ds = 0.f;
      if (j < lim) {
        const float s = dot_row<T>(sq[wave], base + (size_t)j * ld + D + h * dh, dh);
        float dp = dot_row<T>(sdo[wave], base + (size_t)j * ld + 2 * D + h * dh, dh);
        if (drop.thr) dp *= drop_keep1(drop, j, i, b * H + h);
        ds = __expf(s - L) * (dp - dl);
      }
      sp[wave][lane] = ds;
      __syncthreads();
      const int nj = min(64, jend - j0);
      for (int jj = 0; jj < nj; ++jj) {
        const float dj = sp[wave][jj];
        const T *krow = base + (size_t)(j0 + jj) * ld + D + h * dh;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int d = lane + 64 * c;
          if (d < dh) acc[c] += dj * to_f32(krow[d]);
        }
      }
      __syncthreads();
    }
    if (active) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int d = lane + 64 * c;
        if (d < dh) dqkv[((size_t)b * Tn + i) * ld + h * dh + d] = from_f32<T>(acc[c] * scale);
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_rows(const T *__restrict__ qkv, const T *__restrict__ dout,
                                                         const float *__restrict__ lse,
                                                         const float *__restrict__ delta,
                                                         const int32_t *__restrict__ lengths, int causal,
                                                         DropSpec drop, int Tn, int H, int dh, float scale,
                                                         T *__restrict__ dqkv) {
  __shared__ float sk[4][MAX_DH];
  __shared__ float sv[4][MAX_DH];
  __shared__ float sp[4][64];
  __shared__ float sds[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.z, h = blockIdx.y;
  const int D = H * dh, ld = 3 * D;
  const int len = lengths ? min(max(lengths[b], 1), Tn) : Tn;  // a length outside 1..T is treated as the nearest valid one
  const T *base = qkv + (size_t)b * Tn * ld;
  for (int r = 0; r < ROWS_PER_WG / 4; ++r) {
    const int jw = blockIdx.x * ROWS_PER_WG + r * 4 + wave;
    const bool active = jw < Tn;
    const int j = active ? jw : Tn - 1;
    const bool masked = j >= len;
    __syncthreads();
    for (int d = lane; d < dh; d += 64) {
      sk[wave][d] = to_f32(base[(size_t)j * ld + D + h * dh + d]) * scale;
      sv[wave][d] = to_f32(base[(size_t)j * ld + 2 * D + h * dh + d]);
    }
    __syncthreads();
    float ak[4] = {0.f, 0.f, 0.f, 0.f}, av[4] = {0.f, 0.f, 0.f, 0.f};
    // with the causal mask only queries i >= j see key j; start at the tile of the workgroup's first key
    const int ibeg = causal ? (blockIdx.x * ROWS_PER_WG) / 64 * 64 : 0;
    for (int i0 = ibeg; i0 < Tn; i0 += 64) {
      const int i = i0 + lane;
      float p = 0.f, ds = 0.f;
      if (i < Tn && !masked && (!causal || i >= j)) {
        const float s = dot_row<T>(sk[wave], base + (size_t)i * ld + h * dh, dh);
        float dp = dot_row<T>(sv[wave], dout + ((size_t)b * Tn + i) * D + h * dh, dh);
        const size_t st = ((size_t)b * H + h) * Tn + i;
        p = __expf(s - lse[st]);
        const float keep = drop.thr ? drop_keep1(drop, j, i, b * H + h) : 1.f;
        ds = p * (dp * keep - delta[st]);
        p *= keep;   // dV sees the dropped-out probabilities
      }
      sp[wave][lane] = p;
      sds[wave][lane] = ds;
      __syncthreads();
      const int ni = min(64, Tn - i0);
      for (int ii = 0; ii < ni; ++ii) {
        const float pi = sp[wave][ii], di = sds[wave][ii];
        const T *qrow = base + (size_t)(i0 + ii) * ld + h * dh;
        const T *grow = dout + ((size_t)b * Tn + i0 + ii) * D + h * dh;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int d = lane + 64 * c;
          if (d < dh) {
            av[c] += pi * to_f32(grow[d]);
            ak[c] += di * to_f32(qrow[d]);
          }
        }
      }
      __syncthreads();
    }
    if (active) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int d = lane + 64 * c;
        if (d < dh) {
          dqkv[((size_t)b * Tn + j) * ld + D + h * dh + d] = from_f32<T>(masked ? 0.f : ak[c] * scale);
          dqkv[((size_t)b * Tn + j) * ld + 2 * D + h * dh + d] = from_f32<T>(masked ? 0.f : av[c]);
        }
      }
    }
  }
}

// delta[b, h, t] = sum_d dO[b, t, h*dh + d] * O[b, t, h*dh + d]: one wavefront per token row; a lane's
// VEC consecutive elements lie in one head (dh is a multiple of 16); the lanes of a head meet in LDS.
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_rows(const T *__restrict__ o, const T *__restrict__ dout, int rows,
                                                       int Tn, int H, int dh, float *__restrict__ delta) {
  constexpr int VEC = Elem<T>::VEC;
  __shared__ float sp[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * 4 + wave;
  if (row >= rows) return;  // whole wavefronts leave; no workgroup barrier below
  const int b = row / Tn, t = row - b * Tn, D = H * dh;
  const int lph = dh / VEC;                    // lanes per head
  const int chunk = (64 * VEC / dh) * dh;      // elements per step: as many whole heads as 64 lanes hold
  for (int c0 = 0; c0 < D; c0 += chunk) {
    const int col = c0 + lane * VEC;
    float part = 0.f;
    if (lane * VEC < chunk && col < D) {
      float a[VEC], g[VEC];
      VecIO<T, VEC>::load(o + (size_t)row * D + col, a);
      VecIO<T, VEC>::load(dout + (size_t)row * D + col, g);
#pragma unroll
      for (int e = 0; e < VEC; ++e) part += a[e] * g[e];
    }
    sp[wave][lane] = part;  // LDS operations of one wavefront complete in order
    const int heads_here = min(chunk, D - c0) / dh;
    if (lane < heads_here) {
      float sum = 0.f;
      for (int k = 0; k < lph; ++k) sum += sp[wave][lane * lph + k];
      delta[((size_t)b * H + (c0 / dh + lane)) * Tn + t] = sum;
    }
  }
}

bool attn_shape_ok(int B, int T, int H, int dh) {
  return B >= 1 && T >= 1 && H >= 1 && dh >= 16 && dh % 16 == 0 && dh <= MAX_DH && H <= 65535 && B <= 65535;
}

}  // namespace

hipError_t launch_attention_fwd(int dt, const void *qkv, const int32_t *lengths, int causal, const DropSpec &drop,
                                int B, int T, int H, int dh, void *o, float *lse, hipStream_t stream) {
  if (!qkv || !o || !lse || !attn_shape_ok(B, T, H, dh)) return hipErrorInvalidValue;
  if (dt == DT_BF16 && !forced_general_attention() && attention_mfma_supported(dh))
    return launch_attention_fwd_mfma(qkv, lengths, causal, drop, B, T, H, dh, o, lse, stream);
  if (dt == DT_F32 && !forced_general_attention() && attention_mfma_f32_supported(dh))
    return launch_attention_fwd_mfma_f32(qkv, lengths, causal, drop, B, T, H, dh, o, lse, stream);
  const float scale = 1.0f / sqrtf((float)dh);
  dim3 grid((T + ROWS_PER_WG - 1) / ROWS_PER_WG, H, B), block(256);
  if (dt == DT_F32)
    hipLaunchKernelGGL(attn_fwd_rows<float>, grid, block, 0, stream, static_cast<const float *>(qkv), lengths,
                       causal, drop, T, H, dh, scale, static_cast<float *>(o), lse);
  else
    hipLaunchKernelGGL(attn_fwd_rows<bf16_t>, grid, block, 0, stream, static_cast<const bf16_t *>(qkv), lengths,
                       causal, drop, T, H, dh, scale, static_cast<bf16_t *>(o), lse);
  return hipGetLastError();
}

bool attention_bwd_parts_independent(int dt, int dh) {
  if (forced_general_attention()) return true;
  return !(dt == DT_BF16 ? attention_mfma_supported(dh) : attention_mfma_f32_supported(dh));
}

hipError_t launch_attention_bwd(int dt, const void *qkv, const void *o, const void *do_, const float *lse,
                                const int32_t *lengths, int causal, const DropSpec &drop, int B, int T, int H, int dh,
                                void *dqkv, float *delta, hipStream_t stream, int parts) {
  if (!qkv || !o || !do_ || !lse || !dqkv || !delta || !attn_shape_ok(B, T, H, dh) || !(parts & ATTN_BWD_ALL))
    return hipErrorInvalidValue;
  if (!attention_bwd_parts_independent(dt, dh)) {  // matrix cores: delta is produced by the dQ kernel
    if (!(parts & (ATTN_BWD_DQ | ATTN_BWD_DKV))) return hipSuccess;
    if (dt == DT_F32)
      return launch_attention_bwd_mfma_f32(qkv, o, do_, lse, lengths, causal, drop, B, T, H, dh, dqkv, delta, stream,
                                           parts);
    return launch_attention_bwd_mfma(qkv, o, do_, lse, lengths, causal, drop, B, T, H, dh, dqkv, delta, stream, parts);
  }
  if (parts & ATTN_BWD_DELTA) {
    const int rows = B * T;
    dim3 grid((rows + 3) / 4), block(256);
    if (dt == DT_F32)
      hipLaunchKernelGGL(attn_delta_rows<float>, grid, block, 0, stream, static_cast<const float *>(o),
                         static_cast<const float *>(do_), rows, T, H, dh, delta);
    else
      hipLaunchKernelGGL(attn_delta_rows<bf16_t>, grid, block, 0, stream, static_cast<const bf16_t *>(o),
                         static_cast<const bf16_t *>(do_), rows, T, H, dh, delta);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (!(parts & (ATTN_BWD_DQ | ATTN_BWD_DKV))) return hipSuccess;
  const float scale = 1.0f / sqrtf((float)dh);
  dim3 grid((T + ROWS_PER_WG - 1) / ROWS_PER_WG, H, B), block(256);
  if (dt == DT_F32) {
    if (parts & ATTN_BWD_DQ)
      hipLaunchKernelGGL(attn_bwd_dq_rows<float>, grid, block, 0, stream, static_cast<const float *>(qkv),
                         static_cast<const float *>(o), static_cast<const float *>(do_), lse, lengths, causal, drop, T,
                         H, dh, scale, static_cast<float *>(dqkv), delta);
    if (parts & ATTN_BWD_DKV)
      hipLaunchKernelGGL(attn_bwd_dkv_rows<float>, grid, block, 0, stream, static_cast<const float *>(qkv),
                         static_cast<const float *>(do_), lse, delta, lengths, causal, drop, T, H, dh, scale,
                         static_cast<float *>(dqkv));
  } else {
    if (parts & ATTN_BWD_DQ)
      hipLaunchKernelGGL(attn_bwd_dq_rows<bf16_t>, grid, block, 0, stream, static_cast<const bf16_t *>(qkv),
                         static_cast<const bf16_t *>(o), static_cast<const bf16_t *>(do_), lse, lengths, causal, drop,
                         T, H, dh, scale, static_cast<bf16_t *>(dqkv), delta);
    if (parts & ATTN_BWD_DKV)
      hipLaunchKernelGGL(attn_bwd_dkv_rows<bf16_t>, grid, block, 0, stream, static_cast<const bf16_t *>(qkv),
                         static_cast<const bf16_t *>(do_), lse, delta, lengths, causal, drop, T, H, dh, scale,
                         static_cast<bf16_t *>(dqkv));
  }
  return hipGetLastError();
}

}  // namespace fl
