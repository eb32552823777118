// Fused parameter update over a list of tensors: one launch for all of a layer's parameters.
//
// The paper's optimizers are first-order methods written on tensor operations (Section 4.2
// "Optimizers"); its training loop ends an iteration with opt.step(); opt.zeroGrad().  Executed
// primitive by primitive, an Adam step is about ten elementwise kernels per tensor; here the whole
// update of every tensor is one HBM-bound kernel: each element's parameter, gradient and state are
// read once and written once.
//   SGD   g' = g + wd*p;  buf = mu*buf + g';  p -= lr*buf
//   Adam  g' = g + wd*p;  m = b1*m + (1-b1)*g';  v = b2*v + (1-b2)*g'^2;
//         p -= lr * (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps)
// Parameters and gradients have the storage type; the state (buf / m, v) is fp32; arithmetic is
// fp32 and the parameter is rounded once on the way out.
#include "devutil.h"
#include "kernels.h"

namespace fl {
namespace {

struct OptTable {
  float *master[OPT_MAX_TENSORS];  // fp32 copy of the parameter that carries the update (or nullptr)
  void *p[OPT_MAX_TENSORS];
  const void *g[OPT_MAX_TENSORS];
  float *m[OPT_MAX_TENSORS];
  float *v[OPT_MAX_TENSORS];
  long long n[OPT_MAX_TENSORS];
};

template <typename T, int KIND>
__global__ __launch_bounds__(256) void opt_step_kernel(OptTable tb, OptHyper h) {
  constexpr int VEC = Elem<T>::VEC;
  const int t = blockIdx.y;
  const long long n = tb.n[t];
  T *p = static_cast<T *>(tb.p[t]);
  const T *g = static_cast<const T *>(tb.g[t]);
  float *m = tb.m[t], *v = tb.v[t], *w = tb.master[t];
  for (long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * VEC; i < n; i += (long long)gridDim.x * 256 * VEC) {
    float pv[VEC], gv[VEC], mv[VEC], vv[VEC];
    if (w) {  // the full-precision copy is the parameter; p only receives its rounded value
#pragma unroll
      for (int e = 0; e < VEC; e += 4) VecIO<float, 4>::load(w + i + e, pv + e);
    } else {
      VecIO<T, VEC>::load(p + i, pv);
    }
    VecIO<T, VEC>::load(g + i, gv);
    if (KIND == 1 || h.momentum != 0.f) {
#pragma unroll
      for (int e = 0; e < VEC; e += 4) VecIO<float, 4>::load(m + i + e, mv + e);
    }
    if (KIND == 1) {
#pragma unroll
      for (int e = 0; e < VEC; e += 4) VecIO<float, 4>::load(v + i + e, vv + e);
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const float gp = gv[e] + h.weight_decay * pv[e];
      if (KIND == 0) {
        float step = gp;
        if (h.momentum != 0.f) {
          mv[e] = h.momentum * mv[e] + gp;
          step = mv[e];
        }
        pv[e] -= h.lr * step;
      } else {
        mv[e] = h.beta1 * mv[e] + (1.f - h.beta1) * gp;
        vv[e] = h.beta2 * vv[e] + (1.f - h.beta2) * gp * gp;
        pv[e] -= h.lr * (mv[e] * h.inv_bias1) / (sqrtf(vv[e] * h.inv_bias2) + h.eps);
      }
    }
    VecIO<T, VEC>::store(p + i, pv);
    if (w) {
#pragma unroll
      for (int e = 0; e < VEC; e += 4) VecIO<float, 4>::store(w + i + e, pv + e);
    }
    if (KIND == 1 || h.momentum != 0.f) {
#pragma unroll
      for (int e = 0; e < VEC; e += 4) VecIO<float, 4>::store(m + i + e, mv + e);
    }
    if (KIND == 1) {
#pragma unroll
      for (int e = 0; e < VEC; e += 4) VecIO<float, 4>::store(v + i + e, vv + e);
    }
  }
}

struct ZeroTable {
  void *p[OPT_MAX_TENSORS];
  long long bytes[OPT_MAX_TENSORS];
};
__global__ __launch_bounds__(256) void zero_tensors_kernel(ZeroTable tb) {
  const int t = blockIdx.y;
  uint4 *p = static_cast<uint4 *>(tb.p[t]);
  const long long n = tb.bytes[t] / 16;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256)
    p[i] = make_uint4(0, 0, 0, 0);
}

__global__ __launch_bounds__(256) void fill_words_kernel(uint4 *p, long long n, unsigned w) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256)
    p[i] = make_uint4(w, w, w, w);
}

}  // namespace

hipError_t launch_fill_words(void *p, size_t bytes, unsigned word, hipStream_t stream) {
  if (!p || bytes < 16 || bytes % 16 || (reinterpret_cast<uintptr_t>(p) & 15)) return hipErrorInvalidValue;
  long long n = (long long)(bytes / 16), blocks = (n + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(fill_words_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, static_cast<uint4 *>(p), n, word);
  return hipGetLastError();
}

hipError_t launch_opt_step(int dt, int kind, const OptHyper &h, int n, void *const *params, const void *const *grads,
                           float *const *m, float *const *v, const long long *numel, hipStream_t stream,
                           float *const *master) {
  if (n < 1 || n > OPT_MAX_TENSORS || !params || !grads || !numel || (kind != 0 && kind != 1))
    return hipErrorInvalidValue;
  const bool need_m = kind == 1 || h.momentum != 0.f;
  if ((need_m && !m) || (kind == 1 && !v)) return hipErrorInvalidValue;
  OptTable tb;
  long long maxn = 0;
  for (int i = 0; i < n; ++i) {
    // whole 8-element vectors and 16-byte aligned pointers
    if (!params[i] || !grads[i] || numel[i] < 8 || numel[i] % 8 || (need_m && !m[i]) || (kind == 1 && !v[i]))
      return hipErrorInvalidValue;
    if ((reinterpret_cast<uintptr_t>(params[i]) | reinterpret_cast<uintptr_t>(grads[i]) |
         (need_m ? reinterpret_cast<uintptr_t>(m[i]) : 0) | (kind == 1 ? reinterpret_cast<uintptr_t>(v[i]) : 0)) & 15)
      return hipErrorInvalidValue;
    tb.master[i] = master ? master[i] : nullptr;
    if (tb.master[i] && (reinterpret_cast<uintptr_t>(tb.master[i]) & 15)) return hipErrorInvalidValue;
    tb.p[i] = params[i]; tb.g[i] = grads[i];
    tb.m[i] = need_m ? m[i] : nullptr; tb.v[i] = kind == 1 ? v[i] : nullptr;
    tb.n[i] = numel[i];
    if (numel[i] > maxn) maxn = numel[i];
  }
  const int vec = dt == DT_F32 ? 4 : 8;
  long long blocks = (maxn / vec + 255) / 256;
  if (blocks > 1024) blocks = 1024;  // grid-stride beyond that: 4 workgroups per CU
  dim3 grid((unsigned)blocks, n);
  if (dt == DT_F32) {
    if (kind == 0) hipLaunchKernelGGL((opt_step_kernel<float, 0>), grid, dim3(256), 0, stream, tb, h);
    else hipLaunchKernelGGL((opt_step_kernel<float, 1>), grid, dim3(256), 0, stream, tb, h);
  } else {
    if (kind == 0) hipLaunchKernelGGL((opt_step_kernel<bf16_t, 0>), grid, dim3(256), 0, stream, tb, h);
    else hipLaunchKernelGGL((opt_step_kernel<bf16_t, 1>), grid, dim3(256), 0, stream, tb, h);
  }
  return hipGetLastError();
}

hipError_t launch_zero_tensors(int n, void *const *ptrs, const long long *bytes, hipStream_t stream) {
  if (n < 1 || n > OPT_MAX_TENSORS || !ptrs || !bytes) return hipErrorInvalidValue;
  ZeroTable tb;
  long long maxb = 0;
  for (int i = 0; i < n; ++i) {
    if (!ptrs[i] || bytes[i] < 16 || bytes[i] % 16 || (reinterpret_cast<uintptr_t>(ptrs[i]) & 15)) return hipErrorInvalidValue;
    tb.p[i] = ptrs[i];
    tb.bytes[i] = bytes[i];
    if (bytes[i] > maxb) maxb = bytes[i];
  }
  long long blocks = (maxb / 16 + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(zero_tensors_kernel, dim3((unsigned)blocks, n), dim3(256), 0, stream, tb);
  return hipGetLastError();
}

}  // namespace fl
