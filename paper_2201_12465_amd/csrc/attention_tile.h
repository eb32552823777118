// Whole-sequence attention tiles in LDS for head size 64: the layout, the fragment reads and the
// load/wait primitives of the one-kernel backward (attention_bwd_fused.hip).
//
// A tile is row-major [row][64] bf16 (128-byte rows) and serves both the 16-byte row-fragment reads and
// the transposing reads (ds_read_b64_tr_b16): 16-byte chunk c of row r sits at position c ^ swz(r), where
// swz permutes bits 1..3 of r so that 16 consecutive rows of one chunk, and 4 consecutive rows of 4
// consecutive chunks, both touch each of the 64 banks once.  Tiles are filled by direct-to-LDS loads
// (lds_dma16): a wave-level load covers 8 rows, lane l fetching the chunk that belongs at position l.
#pragma once
#include "devutil.h"
#include "lds_dma.h"
#include <type_traits>
#include <utility>

namespace fl {
namespace attn64 {

constexpr int DH = 64, ROWB = DH * 2;   // head size, bytes of a tile row
constexpr float LOG2E = 1.4426950408889634f;

typedef __attribute__((address_space(3))) s16x4_t *lds_s16x4_ptr;
typedef short s16x8_t __attribute__((ext_vector_type(8)));

__device__ __forceinline__ int swz(int row) {
  const int t = row >> 1;
  return ((t & 1) << 2) | ((t >> 1) & 3);
}

// Fragment reads.  Everything that depends on the lane is computed once per kernel (the functions
// *_lane below return a byte offset inside a tile); a query block, a k-step or a column block then only
// adds a constant, which travels in the instruction's offset field.
//
// Row fragment: tile row (lane%32), elements kk*16 + (lane/32)*8 .. +7 of a 32-row block; + r0*ROWB for the block at row r0
// (r0 a multiple of 16: the swizzle only looks at bits 1..3 of the row).
__device__ __forceinline__ unsigned row_frag_lane(int kk, int lane) {
  const int r = lane & 31;
  return (unsigned)(r * ROWB + (((kk * 2 + (lane >> 5)) ^ swz(r)) << 4));
}
__device__ __forceinline__ bf16x8_t row_frag_at(const unsigned char *p) { return *reinterpret_cast<const bf16x8_t *>(p); }

__device__ __forceinline__ bf16x8_t join_halves(s16x4_t lo, s16x4_t hi) {
  s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8_t, v);
}

// Fragment of the transposed tile: its rows are COLUMNS c0 .. c0+31 of the LDS tile, the 8 k-values of
// lane half h are tile rows klo + h*4 + {0..3} and klo + 8 + h*4 + {0..3} (the order in which a lane
// half holds a 32x32 accumulator block's rows, so that such a block packs straight into the other operand).
// half = 0: the address of the first four k-values, 1: of the other four; + klo*ROWB for the k-step at
// tile row klo (a multiple of 16).
__device__ __forceinline__ unsigned tr_frag_lane(int c0, int half, int lane) {
  const int g = lane >> 4, s = lane & 15;
  const int col = c0 + (g & 1) * 16 + 4 * (s & 3);
  const int k0 = (g >> 1) * 4 + (s >> 2) + 8 * half;
  return (unsigned)(k0 * ROWB + (((col >> 3) ^ swz(k0)) << 4) + (col & 7) * 2);
}
// The same inside an unswizzled tile with a row pitch of `pitch` bytes (pitch = 64 mod 128); the second
// half lies 8*pitch further on.
__device__ __forceinline__ unsigned tr_plain_lane(int pitch, int c0, int lane) {
  const int g = lane >> 4, s = lane & 15;
  return (unsigned)(((g >> 1) * 4 + (s >> 2)) * pitch + (c0 + (g & 1) * 16 + 4 * (s & 3)) * 2);
}
__device__ __forceinline__ bf16x8_t tr_frag_at(const unsigned char *lo, const unsigned char *hi) {
  return join_halves(__builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)lo),
                     __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)hi));
}

__device__ __forceinline__ bf16x8_t pack8(const f32x16_t &v, int s) {
  bf16x8_t o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = static_cast<bf16_t>(v[8 * s + e]);
  return o;
}
__device__ __forceinline__ bf16x8_t zero_frag() {
  bf16x8_t z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = static_cast<bf16_t>(0.f);
  return z;
}
__device__ __forceinline__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

// Loads whose results the kernel waits for itself (the compiler does not know they are in flight: it
// must not be given a reason to wait for ALL outstanding loads, the younger query blocks included).
__device__ __forceinline__ void async_load16(f32x4_t &dst, const void *p) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void async_load4(float &dst, const void *p) {
  asm volatile("global_load_dword %0, %1, off" : "=v"(dst) : "v"(p) : "memory");
}
// Placed after the wait that covers an asynchronous load: the value may be read from here on.
__device__ __forceinline__ void arrived(f32x4_t &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void arrived(float &v) { asm volatile("" : "+v"(v)); }
// LDS writes of this wavefront are visible to the workgroup after the barrier.  No fence: a fence makes
// the compiler wait for every outstanding global access as well.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
template <int N> __device__ __forceinline__ void wait_loads_le() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("" ::: "memory");
  FL_WAIT_VMCNT(N);
  asm volatile("" ::: "memory");
}

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ...: a loop whose index is a constant in every pass
template <int... I, typename F> __device__ __forceinline__ void unrolled(std::integer_sequence<int, I...>, F &&f) {
  (f(std::integral_constant<int, I>{}), ...);
}

}  // namespace attn64
}  // namespace fl
