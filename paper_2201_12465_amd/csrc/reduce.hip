// Column reductions: second stage of every two-stage reduction (split-k GEMM
// partials, LayerNorm-backward partials) and the stand-alone bias gradient
// db[n] = sum_m dy[m,n] of a linear layer (the gradient function of the paper's
// add primitive with a broadcast operand; Section 4.1.1 / Section 4.2).
// Both stages are deterministic: fixed summation order, no atomics.
#include "devutil.h"
#include "kernels.h"

namespace fl {
namespace {

// out_s[n..n+3] = sum_p partial[p*stride + s*seglen + n..n+3]
template <typename T>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ partial, int P, size_t stride,
                                                              size_t seglen, T *out0, T *out1, T *out2, int accumulate) {
  const size_t n = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (n >= seglen) return;
  const int s = blockIdx.y;
  const float *src = partial + (size_t)s * seglen + n;
  float a[4] = {0.f, 0.f, 0.f, 0.f};
  for (int p = 0; p < P; ++p) {
    float4 t = *reinterpret_cast<const float4 *>(src + (size_t)p * stride);
    a[0] += t.x; a[1] += t.y; a[2] += t.z; a[3] += t.w;
  }
  T *out = s == 0 ? out0 : (s == 1 ? out1 : out2);
  if (out) {
    if (accumulate) {
      float o[4];
      VecIO<T, 4>::load(out + n, o);
      a[0] += o[0]; a[1] += o[1]; a[2] += o[2]; a[3] += o[3];
    }
    VecIO<T, 4>::store(out + n, a);
  }
}

// Same sums when there are many partial rows and few columns: a workgroup of 16 waves owns 64
// float4 columns, wave w adds rows w, w+16, ..., and the 16 running sums meet in LDS.
template <typename T>
__global__ __launch_bounds__(1024) void reduce_partials_tall_kernel(const float *__restrict__ partial, int P,
                                                                    size_t stride, size_t seglen, T *out0, T *out1,
                                                                    T *out2, int accumulate) {
  __shared__ float4 red[16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t n = ((size_t)blockIdx.x * 64 + lane) * 4;
  const int s = blockIdx.y;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  if (n < seglen) {
    const float *src = partial + (size_t)s * seglen + n;
    for (int p = wave; p < P; p += 16) {
      float4 t = *reinterpret_cast<const float4 *>(src + (size_t)p * stride);
      a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
    }
  }
  red[wave][lane] = a;
  __syncthreads();
  if (wave == 0 && n < seglen) {
    float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      float4 t = red[w][lane];
      v[0] += t.x; v[1] += t.y; v[2] += t.z; v[3] += t.w;
    }
    T *out = s == 0 ? out0 : (s == 1 ? out1 : out2);
    if (out) {
      if (accumulate) {
        float o[4];
        VecIO<T, 4>::load(out + n, o);
        v[0] += o[0]; v[1] += o[1]; v[2] += o[2]; v[3] += o[3];
      }
      VecIO<T, 4>::store(out + n, v);
    }
  }
}

// Several such reductions in one launch (the second stages a backward pass has collected).  A workgroup
// of 16 waves serves one job: "flat" jobs (few partial rows) give every thread one float4 column and let it
// walk the P rows; "tall" jobs (many partial rows, few columns) work as reduce_partials_tall_kernel.  Both
// add in the order of the single-job kernels above, so the sums are bit-identical to theirs.
struct ReduceTable {
  ReduceJob job[REDUCE_MAX_JOBS];
  int first_block[REDUCE_MAX_JOBS + 1];  // job j owns workgroups first_block[j] .. first_block[j+1]-1
  int blocks_per_seg[REDUCE_MAX_JOBS];
  int n;
};
template <typename T>
__global__ __launch_bounds__(1024) void reduce_batch_kernel(ReduceTable tb, int accumulate) {
  __shared__ float4 red[16][64];
  int j = 0;
  while (j + 1 < tb.n && (int)blockIdx.x >= tb.first_block[j + 1]) ++j;
  const ReduceJob &J = tb.job[j];
  const int local = blockIdx.x - tb.first_block[j];
  const int s = local / tb.blocks_per_seg[j], blk = local - s * tb.blocks_per_seg[j];
  T *out = static_cast<T *>(J.out[s]);
  const float *src0 = J.partial + (size_t)s * J.seglen;
  if (J.P < 32) {
    const size_t n = ((size_t)blk * 1024 + threadIdx.x) * 4;
    if (n >= J.seglen || !out) return;
    float a[4] = {0.f, 0.f, 0.f, 0.f};
    for (int p = 0; p < J.P; ++p) {
      float4 t = *reinterpret_cast<const float4 *>(src0 + n + (size_t)p * J.stride);
      a[0] += t.x; a[1] += t.y; a[2] += t.z; a[3] += t.w;
    }
    if (accumulate) {
      float o[4];
      VecIO<T, 4>::load(out + n, o);
      a[0] += o[0]; a[1] += o[1]; a[2] += o[2]; a[3] += o[3];
    }
    VecIO<T, 4>::store(out + n, a);
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t n = ((size_t)blk * 64 + lane) * 4;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  if (n < J.seglen) {
    for (int p = wave; p < J.P; p += 16) {
      float4 t = *reinterpret_cast<const float4 *>(src0 + n + (size_t)p * J.stride);
      a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
    }
  }
  red[wave][lane] = a;
  __syncthreads();
  if (wave == 0 && n < J.seglen && out) {
    float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      float4 t = red[w][lane];
      v[0] += t.x; v[1] += t.y; v[2] += t.z; v[3] += t.w;
    }
    if (accumulate) {
      float o[4];
      VecIO<T, 4>::load(out + n, o);
      v[0] += o[0]; v[1] += o[1]; v[2] += o[2]; v[3] += o[3];
    }
    VecIO<T, 4>::store(out + n, v);
  }
}

constexpr int CS_ROWS = 32;   // rows per first-stage block

// ws[rb][n] = sum over the rows of block rb of in[m][n]; 64 lanes x VEC columns, 4 waves interleave rows
template <typename T>
__global__ __launch_bounds__(256) void colsum_stage1_kernel(const T *__restrict__ in, int M, int N, float *ws) {
  constexpr int VEC = Elem<T>::VEC;
  __shared__ float red[4][64 * VEC];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = (blockIdx.x * 64 + lane) * VEC;
  const int m0 = blockIdx.y * CS_ROWS, m1 = min(M, m0 + CS_ROWS);
  float a[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) a[e] = 0.f;
  if (n < N) {
    for (int m = m0 + wave; m < m1; m += 4) {
      float v[VEC];
      VecIO<T, VEC>::load(in + (size_t)m * N + n, v);
#pragma unroll
      for (int e = 0; e < VEC; ++e) a[e] += v[e];
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) red[wave][lane * VEC + e] = a[e];
  __syncthreads();
  if (wave == 0 && n < N) {
#pragma unroll
    for (int e = 0; e < VEC; ++e)
      ws[(size_t)blockIdx.y * N + n + e] = red[0][lane * VEC + e] + red[1][lane * VEC + e] +
                                           red[2][lane * VEC + e] + red[3][lane * VEC + e];
  }
}

}  // namespace

hipError_t launch_reduce_partials(int dt, const float *partial, int P, size_t stride, size_t seglen, int nseg,
                                  void *out0, void *out1, void *out2, hipStream_t stream, bool accumulate) {
  const int acc = accumulate ? 1 : 0;
  if (!partial || P < 1 || nseg < 1 || nseg > 3 || seglen == 0 || seglen % 4 || stride % 4)
    return hipErrorInvalidValue;
  if ((size_t)nseg * seglen > stride && P > 1) return hipErrorInvalidValue;
  if (P >= 32) {
    dim3 tgrid((unsigned)((seglen / 4 + 63) / 64), nseg);
    if (dt == DT_F32)
      hipLaunchKernelGGL(reduce_partials_tall_kernel<float>, tgrid, dim3(1024), 0, stream, partial, P, stride, seglen,
                         static_cast<float *>(out0), static_cast<float *>(out1), static_cast<float *>(out2), acc);
    else
      hipLaunchKernelGGL(reduce_partials_tall_kernel<bf16_t>, tgrid, dim3(1024), 0, stream, partial, P, stride,
                         seglen, static_cast<bf16_t *>(out0), static_cast<bf16_t *>(out1),
                         static_cast<bf16_t *>(out2), acc);
    return hipGetLastError();
  }
  dim3 grid((unsigned)((seglen / 4 + 255) / 256), nseg);
  if (dt == DT_F32)
    hipLaunchKernelGGL(reduce_partials_kernel<float>, grid, dim3(256), 0, stream, partial, P, stride, seglen,
                       static_cast<float *>(out0), static_cast<float *>(out1), static_cast<float *>(out2), acc);
  else
    hipLaunchKernelGGL(reduce_partials_kernel<bf16_t>, grid, dim3(256), 0, stream, partial, P, stride, seglen,
                       static_cast<bf16_t *>(out0), static_cast<bf16_t *>(out1), static_cast<bf16_t *>(out2), acc);
  return hipGetLastError();
}

hipError_t launch_reduce_batch(int dt, const ReduceJob *jobs, int n, hipStream_t stream, bool accumulate) {
  if (!jobs || n < 1 || n > REDUCE_MAX_JOBS) return hipErrorInvalidValue;
  ReduceTable tb;
  tb.n = n;
  int total = 0;
  for (int j = 0; j < n; ++j) {
    const ReduceJob &J = jobs[j];
    if (!J.partial || J.P < 1 || J.nseg < 1 || J.nseg > 3 || J.seglen == 0 || J.seglen % 4 || J.stride % 4)
      return hipErrorInvalidValue;
    if ((size_t)J.nseg * J.seglen > J.stride && J.P > 1) return hipErrorInvalidValue;
    tb.job[j] = J;
    const size_t cols4 = J.seglen / 4;
    tb.blocks_per_seg[j] = (int)(J.P < 32 ? (cols4 + 1023) / 1024 : (cols4 + 63) / 64);
    tb.first_block[j] = total;
    total += tb.blocks_per_seg[j] * J.nseg;
  }
  tb.first_block[n] = total;
  if (dt == DT_F32)
    hipLaunchKernelGGL(reduce_batch_kernel<float>, dim3(total), dim3(1024), 0, stream, tb, accumulate ? 1 : 0);
  else
    hipLaunchKernelGGL(reduce_batch_kernel<bf16_t>, dim3(total), dim3(1024), 0, stream, tb, accumulate ? 1 : 0);
  return hipGetLastError();
}

size_t colsum_ws_floats(int M, int N) { return (size_t)((M + CS_ROWS - 1) / CS_ROWS) * N; }

int colsum_stage1_rows(int M) { return (M + CS_ROWS - 1) / CS_ROWS; }

hipError_t launch_colsum_stage1(int dt, const void *in, int M, int N, float *ws, hipStream_t stream) {
  if (!in || !ws || M < 1 || N < 1 || N % 8) return hipErrorInvalidValue;
  const int rb = colsum_stage1_rows(M);
  const int vec = dt == DT_F32 ? 4 : 8;
  dim3 grid((N + 64 * vec - 1) / (64 * vec), rb);
  if (dt == DT_F32)
    hipLaunchKernelGGL(colsum_stage1_kernel<float>, grid, dim3(256), 0, stream, static_cast<const float *>(in), M, N, ws);
  else
    hipLaunchKernelGGL(colsum_stage1_kernel<bf16_t>, grid, dim3(256), 0, stream, static_cast<const bf16_t *>(in), M, N, ws);
  return hipGetLastError();
}

hipError_t launch_colsum(int dt, const void *in, int M, int N, float *ws, void *out, hipStream_t stream,
                         bool accumulate) {
  if (!out) return hipErrorInvalidValue;
  hipError_t e = launch_colsum_stage1(dt, in, M, N, ws, stream);
  if (e != hipSuccess) return e;
  return launch_reduce_partials(dt, ws, colsum_stage1_rows(M), (size_t)N, (size_t)N, 1, out, nullptr, nullptr, stream,
                                accumulate);
}

// Plain copy of nbytes (a multiple of 16; 16-byte aligned): the reference for what one read plus one
// write of a buffer costs, and the known-size kernel the HBM byte counters are calibrated against.
namespace {
__global__ __launch_bounds__(256) void copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16) {
  const size_t step = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += step) dst[i] = src[i];
}
}  // namespace

hipError_t launch_copy(const void *src, void *dst, size_t nbytes, hipStream_t stream) {
  if (!src || !dst || nbytes % 16 || ((uintptr_t)src | (uintptr_t)dst) % 16) return hipErrorInvalidValue;
  if (nbytes == 0) return hipSuccess;
  const size_t n16 = nbytes / 16;
  const size_t want = (n16 + 256 * 4 - 1) / (256 * 4);  // about four 16-byte pieces per lane
  const int grid = (int)(want < 1 ? 1 : (want > 256 * 32 ? 256 * 32 : want));
  copy_kernel<<<grid, 256, 0, stream>>>(static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n16);
  return hipGetLastError();
}

// Matrix-core ceiling of the GPU this runs on: every wavefront issues `iters` rounds of eight independent
// 32x32 MFMAs (bf16: k = 16, fp32: k = 2) on operands that stay in registers, so nothing but the MFMA
// pipes limits it.  One float per thread is written so that the loop cannot be dropped.
namespace {
constexpr int PROBE_MFMAS = 8;
template <bool BF16> __global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, float *out) {
  f32x16_t acc[PROBE_MFMAS];
#pragma unroll
  for (int j = 0; j < PROBE_MFMAS; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  const float seed = 1.f / (float)(1 + (threadIdx.x & 63));
  bf16x8_t a8, b8;
#pragma unroll
  for (int e = 0; e < 8; ++e) a8[e] = (__bf16)(seed + (float)e * 0.125f), b8[e] = (__bf16)(0.5f - seed);
  const float a1 = seed, b1 = 0.5f - seed;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int j = 0; j < PROBE_MFMAS; ++j) {
      if constexpr (BF16) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a8, b8, acc[j], 0, 0, 0);
      else acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[j], 0, 0, 0);
    }
  }
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < PROBE_MFMAS; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += acc[j][r];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = sum;
}
}  // namespace

hipError_t launch_mfma_probe(int dt, int workgroups, int iters, float *out, double *flops, hipStream_t stream) {
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || !out) return hipErrorInvalidValue;
  if (dt == DT_BF16) mfma_probe_kernel<true><<<workgroups, 256, 0, stream>>>(iters, out);
  else mfma_probe_kernel<false><<<workgroups, 256, 0, stream>>>(iters, out);
  if (flops) *flops = (double)workgroups * 4 * iters * PROBE_MFMAS * 2.0 * 32 * 32 * (dt == DT_BF16 ? 16 : 2);
  return hipGetLastError();
}

}  // namespace fl
