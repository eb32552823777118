// Device-side helpers shared by the kernels: element types, 16-byte vector
// access, bf16 <-> fp32 conversion, wavefront reductions (64 lanes).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace fl {

typedef __bf16 bf16_t;
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int VEC = 4; };   // elements per 16 bytes
template <> struct Elem<bf16_t> { static constexpr int VEC = 8; };

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return static_cast<float>(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return static_cast<bf16_t>(v); }  // RNE

// Loads / stores of N consecutive elements as fp32 (N*sizeof(T) bytes, naturally aligned).
template <typename T, int N> struct VecIO;
template <> struct VecIO<float, 4> {
  static __device__ __forceinline__ void load(const float *p, float *v) {
    float4 t = *reinterpret_cast<const float4 *>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  static __device__ __forceinline__ void store(float *p, const float *v) {
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct VecIO<bf16_t, 4> {
  static __device__ __forceinline__ void load(const bf16_t *p, float *v) {
    bf16x4_t t = *reinterpret_cast<const bf16x4_t *>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = static_cast<float>(t[i]);
  }
  static __device__ __forceinline__ void store(bf16_t *p, const float *v) {
    bf16x4_t t;
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = static_cast<bf16_t>(v[i]);
    *reinterpret_cast<bf16x4_t *>(p) = t;
  }
};
template <> struct VecIO<bf16_t, 8> {
  static __device__ __forceinline__ void load(const bf16_t *p, float *v) {
    bf16x8_t t = *reinterpret_cast<const bf16x8_t *>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = static_cast<float>(t[i]);
  }
  static __device__ __forceinline__ void store(bf16_t *p, const float *v) {
    bf16x8_t t;
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = static_cast<bf16_t>(v[i]);
    *reinterpret_cast<bf16x8_t *>(p) = t;
  }
};

// Wavefront-wide reductions (every lane receives the result).  Inside a row of 16 lanes the partners come
// through the data-parallel-primitive lane selects of the ALU (no LDS round trip as with a shuffle):
// quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror; after them every lane of a row
// holds its row's result, and the four rows meet through scalar reads of one lane each.
template <int CTRL> __device__ __forceinline__ float dpp_lane(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float lane_value(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
// The value of lane l and the value of lane l ^ 32, in the vector ALU (a shuffle goes through LDS and
// costs its round trip).  v_permlane32_swap exchanges the upper half of one register with the lower half
// of another; given the same value twice, one register ends up with the lower half's values in both of its
// halves and the other with the upper half's: any symmetric combination of the two is the pair's result.
// (Inline assembly: through the compiler's builtin the two results of one value given twice came back
// as one and the same register.  The two wait states in front cover a vector-ALU write of either operand
// by the instruction just before.)
__device__ __forceinline__ void half_pair(float v, float &a, float &b) {
  a = v;
  b = v;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float half_pair_sum(float v) {
  float a, b;
  half_pair(v, a, b);
  return a + b;
}
__device__ __forceinline__ float half_pair_max(float v) {
  float a, b;
  half_pair(v, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_lane<0xB1>(v);
  v += dpp_lane<0x4E>(v);
  v += dpp_lane<0x141>(v);
  v += dpp_lane<0x140>(v);
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_lane<0xB1>(v));
  v = fmaxf(v, dpp_lane<0x4E>(v));
  v = fmaxf(v, dpp_lane<0x141>(v));
  v = fmaxf(v, dpp_lane<0x140>(v));
  return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}

// erf(x) and E = exp(-x^2) without branches: the rational approximation 7.1.26 of Abramowitz & Stegun,
// erf(|x|) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p |x|), absolute error below 1.5e-7
// (the spacing of fp32 numbers near 1).  The library's erff costs several times as much inside a
// GEMM epilogue, where nothing overlaps it.
__device__ __forceinline__ float erf_exp_f(float x, float &E) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  E = __expf(-ax * ax);
  float q = fmaf(t, 1.061405429f, -1.453152027f);
  q = fmaf(t, q, 1.421413741f);
  q = fmaf(t, q, -0.284496736f);
  q = fmaf(t, q, 0.254829592f);
  const float r = fmaf(-q * t, E, 1.0f);
  return copysignf(r, x);
}
// Exact (erf-based) GELU and its derivative:  gelu(u) = u Phi(u),  gelu'(u) = Phi(u) + u phi(u).
__device__ __forceinline__ float gelu_f(float u) {
  float E;
  return 0.5f * u * (1.0f + erf_exp_f(u * 0.70710678118654752f, E));
}
__device__ __forceinline__ float gelu_grad_f(float u) {
  float E;  // exp(-u^2 / 2), shared by the two terms
  const float cdf = 0.5f * (1.0f + erf_exp_f(u * 0.70710678118654752f, E));
  return fmaf(u * 0.39894228040143268f, E, cdf);
}

// The 8 XCDs (each with an L2 of its own) receive workgroup ids round-robin: position of workgroup `bid` of `nb`
// in an order that gives every XCD one contiguous range, so that neighbours in the order share an L2.
__device__ __forceinline__ int xcd_contiguous_order(int bid, int nb) {
  const int xcd = bid & 7, idx = bid >> 3, per = nb >> 3, rem = nb & 7;
  return (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
}
// (row block, head, batch) of a workgroup of an attention kernel's grid (row blocks, heads, batch): the row blocks
// of one (batch, head) are neighbours in that order, so they pull its K/V (Q/dO) rows through ONE L2 -- with the
// grid's own coordinates they land on all eight XCDs, and a sequence of 8 row blocks is fetched from the memory
// side eight times (speech shape, forward: 186 MB per launch for 49 MB of tensors).
struct AttnBlock { int rb, hd, b; };
__device__ __forceinline__ AttnBlock attn_block() {
  const int nrb = gridDim.x, H = gridDim.y;
  const int bid = blockIdx.x + nrb * (blockIdx.y + H * blockIdx.z);
  const int id = xcd_contiguous_order(bid, nrb * H * gridDim.z);
  AttnBlock a;
  a.rb = id % nrb;
  a.hd = (id / nrb) % H;
  a.b = id / (nrb * H);
  return a;
}

}  // namespace fl
