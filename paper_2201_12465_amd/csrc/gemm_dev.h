// Device-side argument block and epilogue shared by the GEMM kernels.
#pragma once
#include "devutil.h"

namespace fl {

struct GemmDev {
  const void *A, *B;
  void *C;
  int M, N, K, lda, ldb, ldc;
  const void *bias, *residual, *aux;
  void *preact;
  int act, dact;
  float *partial;
  int k_per_split, tiles_m, tiles_n;
};


// Epilogue on four consecutive outputs C[m, n0..n0+3] (see GemmArgs for the order of the steps).
template <typename T>
__device__ __forceinline__ void gemm_epilogue_quad(const GemmDev &p, int m, int n0, float (&v)[4]) {
  if (p.partial) {
    float *dst = p.partial + ((size_t)blockIdx.z * p.M + m) * p.N + n0;
    *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
    return;
  }
  const size_t off = (size_t)m * p.ldc + n0;
  float t[4];
  if (p.bias) {
    VecIO<T, 4>::load(static_cast<const T *>(p.bias) + n0, t);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += t[e];
  }
  if (p.preact) VecIO<T, 4>::store(static_cast<T *>(p.preact) + off, v);
  if (p.act == 1) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
  } else if (p.act == 2) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = gelu_f(v[e]);
  }
  if (p.residual) {
    VecIO<T, 4>::load(static_cast<const T *>(p.residual) + off, t);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += t[e];
  }
  if (p.dact) {
    VecIO<T, 4>::load(static_cast<const T *>(p.aux) + off, t);
    if (p.dact == 1) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = t[e] > 0.f ? v[e] : 0.f;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] *= gelu_grad_f(t[e]);
    }
  }
  VecIO<T, 4>::store(static_cast<T *>(p.C) + off, v);
}

// The same steps on eight consecutive outputs C[m, n0..n0+7] (bf16 storage): 16-byte accesses.
__device__ __forceinline__ void gemm_epilogue_oct(const GemmDev &p, int m, int n0, float (&v)[8]) {
  if (p.partial) {
    float *dst = p.partial + ((size_t)blockIdx.z * p.M + m) * p.N + n0;
    *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
    return;
  }
  const size_t off = (size_t)m * p.ldc + n0;
  float t[8];
  if (p.bias) {
    VecIO<bf16_t, 8>::load(static_cast<const bf16_t *>(p.bias) + n0, t);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += t[e];
  }
  if (p.preact) VecIO<bf16_t, 8>::store(static_cast<bf16_t *>(p.preact) + off, v);
  if (p.act == 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
  } else if (p.act == 2) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = gelu_f(v[e]);
  }
  if (p.residual) {
    VecIO<bf16_t, 8>::load(static_cast<const bf16_t *>(p.residual) + off, t);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += t[e];
  }
  if (p.dact) {
    VecIO<bf16_t, 8>::load(static_cast<const bf16_t *>(p.aux) + off, t);
    if (p.dact == 1) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = t[e] > 0.f ? v[e] : 0.f;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f(t[e]);
    }
  }
  VecIO<bf16_t, 8>::store(static_cast<bf16_t *>(p.C) + off, v);
}

// The 8 XCDs receive workgroup ids round-robin; give each a contiguous range of tiles.
__device__ __forceinline__ int xcd_tile_order(int bid, int nb) {
  const int xcd = bid & 7, idx = bid >> 3, per = nb >> 3, rem = nb & 7;
  return (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
}

}  // namespace fl
