// Fused masked attention on the matrix cores (bf16 in, fp32 accumulate), forward
// and backward, for head sizes up to 256 that are multiples of 16 (kernel instances exist for 32, 64, 96,
// 128, 192 and 256; a smaller size runs on the next instance with the missing columns read as zeros and
// never stored).
//
// Same operator as attention.hip (the paper's matmul / exp / max / sum primitives,
// Section 4.1.1, fused into one operator with a pre-fused gradient function,
// Section 5.2.1), with the two contractions of each step on v_mfma_f32_32x32x16_bf16
// and the softmax statistics in fp32 registers.  Scores and probabilities never
// leave the wavefront.
//
// A wavefront owns 32 query rows (forward, dQ) or 32 key rows (dK/dV) and walks
// the other sequence dimension in LDS tiles of 64 rows.  The MFMA that produces a
// score block is oriented so that the index contracted NEXT ends up in a lane's
// registers and the surviving index on the lanes:
//   forward / dQ:  S^T[key, q] = K Q^T      -> lane = q, registers = 16 keys;
//                  row max / sum = in-lane reduction + one exchange with lane^32;
//                  O^T[d, q] += V^T[d, key] P^T[key, q] takes P straight from registers
//   dK / dV:       S[q, key] = Q K^T        -> lane = key, registers = 16 queries;
//                  dV^T[d, key] += dO^T[d, q] P[q, key],  dK^T[d, key] += Q^T[d, q] dS[q, key]
// The "transposed" A operands (V^T, K^T, Q^T, dO^T) are read from row-major LDS
// tiles with the transposing LDS load (ds_read_b64_tr_b16); tiles that are read in
// both orientations are kept twice, each with the row padding that keeps its access
// pattern free of bank conflicts.
//
// exp is evaluated as exp2 with log2(e) folded into the scale.  Masked keys
// (j >= length) get probability exactly 0, so their dK / dV rows are exact zeros.
#include "devutil.h"
#include "kernels.h"
#include "philox.h"
#include <type_traits>
#include <utility>

namespace fl {
namespace {

constexpr int NT = 256;        // threads per workgroup (4 wavefronts)
constexpr int ROWS_WG = 128;   // rows owned by a workgroup (32 per wavefront)
constexpr int TILE = 64;       // rows of the walked dimension per LDS tile
constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;
constexpr float RESCALE_SLACK = 8.f;  // see attn_fwd_mfma

// Row stride (elements) of a tile read with 16-byte row-fragment loads: 16 bytes of padding.
constexpr int kc_stride(int dh) { return dh + 8; }
// Row stride of a tile read with transposing loads: bytes = 64 (mod 128).
constexpr int tr_stride(int dh) { return (((dh * 2 - 64 + 127) / 128) * 128 + 64) / 2; }

typedef __attribute__((address_space(3))) s16x4_t *lds_s16x4_ptr;

// A-operand fragment of the transposed tile: rows r0..r0+31 are COLUMNS of the LDS tile,
// the 8 k-values of lane half h are tile rows klo + h*4 + {0..3} and klo + 8 + h*4 + {0..3}.
__device__ __forceinline__ bf16x8_t tr_frag(const bf16_t *lds, int stride, int r0, int klo, int lane) {
  const int g = lane >> 4, s = lane & 15;
  const int col = r0 + (g & 1) * 16 + 4 * (s & 3);
  const int k0 = klo + (g >> 1) * 4 + (s >> 2);
  s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + k0 * stride + col));
  s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + (k0 + 8) * stride + col));
  typedef short s16x8_t __attribute__((ext_vector_type(8)));
  s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8_t, v);
}

// Row fragment: tile row r0 + lane%32, elements kk*16 + (lane/32)*8 .. +7.
__device__ __forceinline__ bf16x8_t kc_frag(const bf16_t *lds, int stride, int r0, int kk, int lane) {
  return *reinterpret_cast<const bf16x8_t *>(lds + (r0 + (lane & 31)) * stride + kk * 16 + (lane >> 5) * 8);
}

__device__ __forceinline__ bf16x8_t zero_frag() {
  bf16x8_t z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = static_cast<bf16_t>(0.f);
  return z;
}

// Same layout straight from global memory (row pointer of this lane's row, or nullptr -> zeros).
__device__ __forceinline__ bf16x8_t g_frag(const bf16_t *row, int kk, int lane, int dh) {
  if (!row || kk * 16 >= dh) return zero_frag();   // dh is a multiple of 16: both lane halves agree
  return *reinterpret_cast<const bf16x8_t *>(row + kk * 16 + (lane >> 5) * 8);
}

// Marks the point by which two fragments must be in registers.  Placed after a run of LDS reads it keeps
// the compiler from sinking each read to just in front of the MFMA that uses it (which it does under
// register pressure, and which makes every MFMA wait out an LDS round trip of its own).
__device__ __forceinline__ void keep_requested(bf16x8_t &a, bf16x8_t &b) { asm volatile("" : "+v"(a), "+v"(b)); }
// Memory operations written before this point are issued before it: LDS reads requested early stay early.
__device__ __forceinline__ void issue_fence() { asm volatile("" ::: "memory"); }

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ...: a loop whose index is a constant in every pass
template <int... I, typename F> __device__ __forceinline__ void unrolled(std::integer_sequence<int, I...>, F &&f) {
  (f(std::integral_constant<int, I>{}), ...);
}
// N batches of LDS fragment reads, each followed by the MFMAs that consume it, with the reads of batch
// i+1 issued BEFORE the MFMAs of batch i (two sets of fragment registers, picked by the slot argument).
// Left alone the compiler gives consecutive batches the same registers, and every batch then waits out
// its own LDS round trip with the matrix core idle -- which a kernel that runs one wavefront per SIMD
// cannot hide behind another wavefront.  load(i, slot) and compute(i, slot) get integral constants.
// AHEAD = false keeps one set of registers: batch after batch, for the instances that have none to spare.
template <int N, bool AHEAD = true, typename L, typename C>
__device__ __forceinline__ void pipelined(L &&load, C &&compute, bool first_loaded = false) {
  if (!first_loaded) load(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
  unrolled(std::make_integer_sequence<int, N>{}, [&](auto i) {
    constexpr int I = decltype(i)::value;
    if constexpr (AHEAD) {
      if constexpr (I + 1 < N) load(std::integral_constant<int, I + 1>{}, std::integral_constant<int, (I + 1) & 1>{});
      __builtin_amdgcn_sched_barrier(0);
      compute(i, std::integral_constant<int, I & 1>{});
      __builtin_amdgcn_sched_barrier(0);
    } else {
      if constexpr (I > 0) load(i, std::integral_constant<int, 0>{});
      compute(i, std::integral_constant<int, 0>{});
    }
  });
}

// 2^x as the bare v_exp_f32: the arguments here are at most RESCALE_SLACK and results below the smallest
// normal number may become 0 (probabilities under 1e-38), so the library function's range handling
// (four more instructions per value) buys nothing.
__device__ __forceinline__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

// registers 8s..8s+7 of a score block, rounded to bf16: the B operand of the next MFMA
__device__ __forceinline__ bf16x8_t pack8(const f32x16_t &v, int s) {
  bf16x8_t o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = static_cast<bf16_t>(v[8 * s + e]);
  return o;
}

// A tile of up to TILE rows of DH elements on its way from global memory to LDS.  load() only
// issues the global reads (into registers); store() writes them to one or two LDS tiles.  The
// kernels load tile t+1 right after storing tile t, so the reads are in flight during the MFMAs.
// Rows >= nvalid are zero.
template <int DH, int NTH = NT> struct TileRegs {
  static constexpr int CPR = DH / 8, N = TILE * CPR / NTH;  // 16-byte chunks per row, per thread
  static_assert(TILE * CPR % NTH == 0, "a tile is a whole number of 16-byte chunks per thread");
  uint4 r[N];
  __device__ __forceinline__ void load(const bf16_t *src, size_t ld, int nvalid, int dh) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + NTH * i, row = c / CPR, ch = c % CPR;
      r[i] = row < nvalid && ch * 8 < dh ? *reinterpret_cast<const uint4 *>(src + (size_t)row * ld + ch * 8)
                                         : make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(bf16_t *dst0, int stride0, bf16_t *dst1, int stride1) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + NTH * i, row = c / CPR, ch = c % CPR;
      *reinterpret_cast<uint4 *>(dst0 + row * stride0 + ch * 8) = r[i];
      if (dst1) *reinterpret_cast<uint4 *>(dst1 + row * stride1 + ch * 8) = r[i];
    }
  }
};

// index (within a 32-block) of accumulator register r for lane half h
__device__ __forceinline__ int acc_row(int r, int h) { return (r >> 2) * 8 + h * 4 + (r & 3); }

// Wavefronts per SIMD the compiler is asked to make room for (second argument of __launch_bounds__).
// With the thread count alone it budgets registers for one wavefront per SIMD and spends them on
// unrolling; small heads do not need that many, and a second to fourth resident wavefront hides the
// LDS and exp latencies of the first (head size 64, B*H*T/128 = 384 workgroups: dK/dV 23.7 -> 15.7 us).
// The values are the largest that compile without scratch.
// Large heads: the two 32-row blocks of a tile are NOT unrolled into one body (the `#pragma unroll (...)`
// in front of the block loops).  Unrolled, the scheduler keeps both blocks' fragments and scores live,
// runs out of the 512 registers and spills (head size 192: 136-232 bytes per lane in the dK pass, head
// size 256: up to 720); rolled, every instance compiles without scratch (dK pass at head size 192 and
// T = 1000: 150 -> 99 us).
// dK and dV in one pass up to head size 192 (rolled, that fits the register file); above, two passes.
constexpr bool dkv_two_passes(int dh) { return dh > 192; }
// key groups of the forward kernel (see attn_fwd_mfma): large heads, where one group leaves one wavefront per SIMD
constexpr int fwd_key_groups(int dh, bool drop) { return dh > 128 && dh <= 192 ? 2 : 1; }   // head size 256 does not fit 256 registers
constexpr int fwd_waves(int dh, bool drop) { return dh <= 64 ? (drop ? 3 : 4) : dh <= 128 ? 2 : 1; }
constexpr int dq_waves(int dh, bool drop) { return dh <= 64 ? (drop ? 2 : 3) : dh <= 96 ? 2 : dh <= 128 ? (drop ? 1 : 2) : 1; }
constexpr int dkv_waves(int dh) { return dh <= 64 ? 2 : 1; }

// ------------------------------------------------------------------------------------------ forward
// KG = 2: eight wavefronts; wavefronts w and w + 4 own the same 32 queries and take the first / second 32-key
// block of every tile, each with its own running maximum, denominator and output accumulators, which group 0
// merges at the end (the usual rescaling to the common maximum).  For large heads this puts two wavefronts
// on every SIMD -- each within 256 registers -- so that one's softmax arithmetic and LDS waits run under the
// other's MFMAs, with the same LDS traffic per key as four wavefronts that walk both blocks.
template <int DH, bool CAUSAL, bool DROP, int KG = 1>
__global__ __launch_bounds__(NT * KG, KG > 1 ? 1 : fwd_waves(DH, DROP)) void attn_fwd_mfma(const bf16_t *__restrict__ qkv, const int32_t *__restrict__ lengths,
                                                    DropSpec drop, int Tn, int H, int dh, float scale,
                                                    bf16_t *__restrict__ o, float *__restrict__ lse) {
  constexpr int KS = kc_stride(DH), VS = tr_stride(DH), NK = DH / 16, NB = DH / 32;
  // K fragments in flight at one time (4 registers each); small heads run several wavefronts per SIMD
  // instead and have no registers to spare
  constexpr int KBATCH = DH <= 64 ? 1 : KG > 1 ? 4 : DH > 192 ? NK / 2 : NK;
  static_assert(NK % KBATCH == 0 && (KBATCH == 1 || KBATCH % 2 == 0), "K fragments are pinned in pairs");
  constexpr bool LAZY = DH > 64;   // rescale the output accumulators only when a row's reference maximum moves
  // V^T fragments requested BEFORE the softmax arithmetic of a block, so that their LDS round trip runs
  // under it (48 registers at head size 192; the largest head has none to spare)
  constexpr int VEARLY = DH <= 64 || DH > 192 || KG > 1 ? 0 : NB;
  // K tile, V tile.  KG > 1: two such stages (and the merge at the end reuses them) -- a wavefront that is done
  // with tile t stores its part of tile t+1 into the other stage while the others still compute, and one
  // barrier per tile is enough.
  constexpr int STG = KG > 1 ? 2 : 1, STAGE = TILE * (KS + VS);
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t *const smem = reinterpret_cast<bf16_t *>(smem_raw);
  const int lane = threadIdx.x & 63, h2 = lane >> 5;
  const int wave = (threadIdx.x >> 6) % 4, kgrp = (threadIdx.x >> 6) / 4;   // position among the query rows, key block
  const AttnBlock blk = attn_block();
  const int b = blk.b, hd = blk.hd, rb = blk.rb;
  const int D = H * dh;
  const size_t ld = (size_t)3 * D;
  const int len = lengths ? min(max(lengths[b], 1), Tn) : Tn;  // a length outside 1..T is treated as the nearest valid one
  const bf16_t *base = qkv + (size_t)b * Tn * ld + hd * dh;
  const int q = rb * ROWS_WG + wave * 32 + (lane & 31);
  const bf16_t *qrow = q < Tn ? base + (size_t)q * ld : nullptr;
  bf16x8_t qf[NK];
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) qf[kk] = g_frag(qrow, kk, lane, dh);
  const float c = scale * LOG2E;
  float m = -INFINITY, l = 0.f;
  f32x16_t oacc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;

  // With the causal mask the workgroup needs keys up to its last query only, and a wavefront keys up
  // to the last of its 32 queries.  Wavefront rows and key blocks are both aligned to 32, so every key
  // block a wavefront visits holds at least one allowed key for each of its queries.
  const int kend = CAUSAL ? min(len, (int)(rb * ROWS_WG + ROWS_WG)) : len;
  const int wend = CAUSAL ? min(len, (int)(rb * ROWS_WG + wave * 32 + 32)) : len;
  TileRegs<DH, NT * KG> tk, tv;
  tk.load(base + D, ld, min(TILE, Tn), dh);
  tv.load(base + 2 * D, ld, min(TILE, Tn), dh);
  auto load_tile = [&](int kt) {   // issue the global reads of the tile that starts at key kt
    tk.load(base + (size_t)kt * ld + D, ld, min(TILE, Tn - kt), dh);
    tv.load(base + (size_t)kt * ld + 2 * D, ld, min(TILE, Tn - kt), dh);
  };
  if constexpr (STG == 2) {
    tk.store(smem, KS, nullptr, 0);
    tv.store(smem + TILE * KS, VS, nullptr, 0);
    __syncthreads();
    if (TILE < kend) load_tile(TILE);
  }
  for (int k0 = 0, it = 0; k0 < kend; k0 += TILE, ++it) {
    bf16_t *const sK = smem + (STG == 2 ? (it & 1) * STAGE : 0), *const sV = sK + TILE * KS;
    if constexpr (STG == 1) {
      __syncthreads();
      tk.store(sK, KS, nullptr, 0);
      tv.store(sV, VS, nullptr, 0);
      __syncthreads();
      if (k0 + TILE < kend) load_tile(k0 + TILE);
    }
#pragma unroll (DH >= 192 ? 1 : 2)
    for (int kb = (KG > 1 ? kgrp : 0); kb < (KG > 1 ? kgrp + 1 : 2); ++kb) {
      if (k0 + kb * 32 >= wend) break;
      f32x16_t s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
      // The K fragments are requested in batches ahead of the MFMAs that consume them: one at a time,
      // every MFMA of the chain would wait out an LDS round trip of its own.
#pragma unroll
      for (int kh = 0; kh < NK; kh += KBATCH) {
        bf16x8_t kf[KBATCH];
#pragma unroll
        for (int kk = 0; kk < KBATCH; ++kk) kf[kk] = kc_frag(sK, KS, kb * 32, kh + kk, lane);
        if constexpr (KBATCH > 1) {
#pragma unroll
          for (int kk = 0; kk < KBATCH; kk += 2) keep_requested(kf[kk], kf[kk + 1]);
        }
#pragma unroll
        for (int kk = 0; kk < KBATCH; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kh + kk], s, 0, 0, 0);
      }
      bf16x8_t vt[VEARLY ? VEARLY : 1][2];
      if constexpr (VEARLY > 0) {
#pragma unroll
        for (int db = 0; db < VEARLY; ++db)
#pragma unroll
          for (int st = 0; st < 2; ++st) vt[db][st] = tr_frag(sV, VS, db * 32, kb * 32 + 16 * st, lane);
        issue_fence();
      }
      // Masked scores become -inf; a block wholly inside the sequence (and, with the causal mask, wholly at or
      // before the wavefront's first query) has none, which is the common case and a wavefront-uniform test.
      // The scale is applied inside the exponent's fused multiply-add, so the maximum is taken over raw scores.
      const int kbase = k0 + kb * 32;
      if (!(kbase + 32 <= len && (!CAUSAL || kbase + 31 <= (int)(rb * ROWS_WG + wave * 32)))) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kbase + acc_row(r, h2);
          if (!(key < len && (!CAUSAL || key <= q))) s[r] = -INFINITY;
        }
      }
      float mloc = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[r]);
      mloc = half_pair_max(mloc) * c;   // c > 0
      // The reference maximum m moves only when a block's maximum exceeds it by more than RESCALE_SLACK
      // (in units of log2): probabilities are then at most 2^RESCALE_SLACK instead of 1, which changes
      // neither O / l nor the log-sum-exp, and the accumulators are rescaled only in the blocks where some
      // row's reference moved (the first block, and rarely again) instead of in every block.
      // Heads up to 64 keep the plain rule (32 multiplications per block, and no registers for this).
      const bool moved = !LAZY || mloc > m + RESCALE_SLACK;   // first block: m = -inf
      const float mnew = LAZY ? (moved ? mloc : m) : fmaxf(m, mloc);
      float rs = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[r] = exp2_raw(fmaf(s[r], c, -mnew));   // -inf stays -inf: mnew is finite (every visited block has an allowed key per query)
        rs += s[r];
      }
      rs = half_pair_sum(rs);
      const bool rescale = !LAZY || __any(moved);    // wave-uniform
      const float corr = (LAZY && !moved) ? 1.f : exp2_raw(m - mnew);
      l = l * corr + rs;   // the softmax denominator ignores dropout
      m = mnew;
      if constexpr (DROP) {  // registers 4g..4g+3 hold four consecutive keys: one generator call
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float kp[4];
          drop_keep4(drop, (uint32_t)(k0 + kb * 32 + g * 8 + h2 * 4) >> 2, (uint32_t)q, (uint32_t)(b * H + hd), kp);
#pragma unroll
          for (int e = 0; e < 4; ++e) s[g * 4 + e] *= kp[e];
        }
      }
      bf16x8_t pf[2] = {pack8(s, 0), pack8(s, 1)};
      if (rescale) {
#pragma unroll
        for (int db = 0; db < NB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][r] *= corr;
      }
      if constexpr (VEARLY > 0) {
#pragma unroll
        for (int db = 0; db < VEARLY; ++db) keep_requested(vt[db][0], vt[db][1]);
      }
#pragma unroll
      for (int db = 0; db < NB; ++db) {
#pragma unroll
        for (int st = 0; st < 2; ++st)
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              db < VEARLY ? vt[db][st] : tr_frag(sV, VS, db * 32, kb * 32 + 16 * st, lane), pf[st], oacc[db], 0, 0, 0);
      }
    }
    if constexpr (STG == 2) {
      // the other stage was last read in the previous pass, which every wavefront left through the barrier below
      if (k0 + TILE < kend) {
        bf16_t *const nK = smem + ((it + 1) & 1) * STAGE;
        tk.store(nK, KS, nullptr, 0);
        tv.store(nK + TILE * KS, VS, nullptr, 0);
      }
      __syncthreads();
      if (k0 + 2 * TILE < kend) load_tile(k0 + 2 * TILE);
    }
  }
  if constexpr (KG > 1) {
    // group 1 parks (m, l) and its accumulators, CH 32-column blocks at a time, in the K/V tiles' LDS
    // ([wave][register][lane]: lane-contiguous); group 0 folds them in.  Group 0 has seen key 0, so its
    // maximum is finite; a group 1 that saw no block has m = -inf, l = 0 and weight 2^(-inf) = 0.
    float *red = reinterpret_cast<float *>(smem);
    constexpr int FLOATS = STG * STAGE / 2, STATS = 4 * 2 * 64;
    constexpr int CH = (FLOATS - STATS) / (4 * 16 * 64) < NB ? (FLOATS - STATS) / (4 * 16 * 64) : NB;
    static_assert(CH >= 1, "the tiles' LDS holds at least one accumulator block per wavefront");
    float *stat = red + 4 * CH * 16 * 64 + wave * 128 + lane;
    float *blk0 = red + wave * CH * 16 * 64 + lane;
    float a0 = 1.f, a1 = 0.f;
#pragma unroll
    for (int d0 = 0; d0 < NB; d0 += CH) {
      __syncthreads();   // the tiles (first pass) or the previous chunk are no longer being read
      if (kgrp == 1) {
        if (d0 == 0) stat[0] = m, stat[64] = l;
#pragma unroll
        for (int db = d0; db < NB && db < d0 + CH; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) blk0[((db - d0) * 16 + r) * 64] = oacc[db][r];
      }
      __syncthreads();
      if (kgrp == 0) {
        if (d0 == 0) {
          const float m1 = stat[0], l1 = stat[64];
          const float mstar = fmaxf(m, m1);
          a0 = exp2_raw(m - mstar);
          a1 = exp2_raw(m1 - mstar);
          l = l * a0 + l1 * a1;
          m = mstar;
        }
#pragma unroll
        for (int db = d0; db < NB && db < d0 + CH; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][r] = oacc[db][r] * a0 + blk0[((db - d0) * 16 + r) * 64] * a1;
      }
    }
    if (kgrp != 0) return;   // no barrier follows
  }
  if (q < Tn) {
    const float inv = 1.0f / l;
    bf16_t *orow = o + ((size_t)b * Tn + q) * D + hd * dh;
#pragma unroll
    for (int db = 0; db < NB; ++db)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        float v[4] = {oacc[db][qd * 4] * inv, oacc[db][qd * 4 + 1] * inv, oacc[db][qd * 4 + 2] * inv,
                      oacc[db][qd * 4 + 3] * inv};
        if (db * 32 + qd * 8 + h2 * 4 < dh) VecIO<bf16_t, 4>::store(orow + db * 32 + qd * 8 + h2 * 4, v);
      }
    if (h2 == 0) lse[((size_t)b * H + hd) * Tn + q] = (m + log2f(l)) * LN2;
  }
}

// ------------------------------------------------------------------------------------------ dQ (+ delta)
template <int DH, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(NT, dq_waves(DH, DROP)) void attn_bwd_dq_mfma(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ o,
                                                       const bf16_t *__restrict__ dout,
                                                       const float *__restrict__ lse,
                                                       const int32_t *__restrict__ lengths, DropSpec drop, int Tn,
                                                       int H, int dh, float scale, bf16_t *__restrict__ dqkv,
                                                       float *__restrict__ delta) {
  constexpr int KS = kc_stride(DH), TS = tr_stride(DH), NK = DH / 16, NB = DH / 32;
  __shared__ __attribute__((aligned(16))) bf16_t sK[TILE * KS];   // K rows for S^T = K Q^T
  __shared__ __attribute__((aligned(16))) bf16_t sKt[TILE * TS];  // K again, for K^T in dQ^T = K^T dS^T
  __shared__ __attribute__((aligned(16))) bf16_t sV[TILE * KS];   // V rows for dP^T = V dO^T
  constexpr int KBATCH = DH <= 128 ? 1 : 2;   // K and V fragments of a batch (8 registers per step, two batches in flight)
  constexpr int TBATCH = DH <= 64 ? 1 : NB % 2 == 0 ? 2 : 3;   // K^T fragment pairs of a batch
  static_assert(NK % KBATCH == 0 && NB % TBATCH == 0, "batches must divide the head size");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h2 = lane >> 5;
  const AttnBlock blk = attn_block();
  const int b = blk.b, hd = blk.hd, rb = blk.rb;
  const int D = H * dh;
  const size_t ld = (size_t)3 * D;
  const int len = lengths ? min(max(lengths[b], 1), Tn) : Tn;  // a length outside 1..T is treated as the nearest valid one
  const bf16_t *base = qkv + (size_t)b * Tn * ld + hd * dh;
  const int q = rb * ROWS_WG + wave * 32 + (lane & 31);
  const bool qok = q < Tn;
  const bf16_t *qrow = qok ? base + (size_t)q * ld : nullptr;
  const bf16_t *dorow = qok ? dout + ((size_t)b * Tn + q) * D + hd * dh : nullptr;
  const bf16_t *orow = qok ? o + ((size_t)b * Tn + q) * D + hd * dh : nullptr;
  bf16x8_t qf[NK], dof[NK];
  float dl = 0.f;
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) {
    qf[kk] = g_frag(qrow, kk, lane, dh);
    dof[kk] = g_frag(dorow, kk, lane, dh);
    bf16x8_t of = g_frag(orow, kk, lane, dh);
#pragma unroll
    for (int e = 0; e < 8; ++e) dl += static_cast<float>(dof[kk][e]) * static_cast<float>(of[e]);
  }
  dl = half_pair_sum(dl);
  const size_t st_idx = ((size_t)b * H + hd) * Tn + (qok ? q : 0);
  const float L2 = qok ? lse[st_idx] * LOG2E : 0.f;
  if (qok && h2 == 0) delta[st_idx] = dl;
  const float c = scale * LOG2E;
  f32x16_t acc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  const int kend = CAUSAL ? min(len, (int)(rb * ROWS_WG + ROWS_WG)) : len;       // as in the forward kernel
  const int wend = CAUSAL ? min(len, (int)(rb * ROWS_WG + wave * 32 + 32)) : len;
  TileRegs<DH> tk, tv;
  tk.load(base + D, ld, min(TILE, Tn), dh);
  tv.load(base + 2 * D, ld, min(TILE, Tn), dh);
  for (int k0 = 0; k0 < kend; k0 += TILE) {
    __syncthreads();
    tk.store(sK, KS, sKt, TS);
    tv.store(sV, KS, nullptr, 0);
    __syncthreads();
    if (k0 + TILE < kend) {
      tk.load(base + (size_t)(k0 + TILE) * ld + D, ld, min(TILE, Tn - k0 - TILE), dh);
      tv.load(base + (size_t)(k0 + TILE) * ld + 2 * D, ld, min(TILE, Tn - k0 - TILE), dh);
    }
#pragma unroll (DH >= 256 || DH == 128 ? 1 : 2)
    for (int kb = 0; kb < 2; ++kb) {
      if (k0 + kb * 32 >= wend) break;
      f32x16_t s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f, dp[r] = 0.f;
      // K and V row fragments in batches, the next batch requested before the MFMAs of this one
      bf16x8_t kfr[2][KBATCH], vfr[2][KBATCH];
      pipelined<NK / KBATCH>(
          [&](auto bi, auto sl) {
            constexpr int kh = decltype(bi)::value * KBATCH, S = decltype(sl)::value;
#pragma unroll
            for (int kk = 0; kk < KBATCH; ++kk) {
              kfr[S][kk] = kc_frag(sK, KS, kb * 32, kh + kk, lane);
              vfr[S][kk] = kc_frag(sV, KS, kb * 32, kh + kk, lane);
            }
          },
          [&](auto bi, auto sl) {
            constexpr int kh = decltype(bi)::value * KBATCH, S = decltype(sl)::value;
#pragma unroll
            for (int kk = 0; kk < KBATCH; ++kk) {
              s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[S][kk], qf[kh + kk], s, 0, 0, 0);
              dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[S][kk], dof[kh + kk], dp, 0, 0, 0);
            }
          });
      // the first K^T fragments are requested before the dS arithmetic, so that their LDS round trip runs under it
      // (not with dropout at the large heads: the mask generator needs the registers)
      constexpr bool EARLY = !(DROP && DH >= 192);
      bf16x8_t tf[2][TBATCH][2];
      auto load_t = [&](auto bi, auto sl) {
        constexpr int d0 = decltype(bi)::value * TBATCH, S = decltype(sl)::value;
#pragma unroll
        for (int db = 0; db < TBATCH; ++db)
#pragma unroll
          for (int st = 0; st < 2; ++st) tf[S][db][st] = tr_frag(sKt, TS, (d0 + db) * 32, kb * 32 + 16 * st, lane);
      };
      if constexpr (EARLY) {
        load_t(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        issue_fence();
      }
      if constexpr (DROP) {  // dP = (dO V^T) * keep
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float kp[4];
          drop_keep4(drop, (uint32_t)(k0 + kb * 32 + g * 8 + h2 * 4) >> 2, (uint32_t)q, (uint32_t)(b * H + hd), kp);
#pragma unroll
          for (int e = 0; e < 4; ++e) dp[g * 4 + e] *= kp[e];
        }
      }
      // masked scores become -inf (probability 2^-inf = 0) only in blocks that reach the sequence end or the
      // diagonal: a wavefront-uniform test, as in the forward kernel
      const int kbase = k0 + kb * 32;
      if (!(kbase + 32 <= len && (!CAUSAL || kbase + 31 <= (int)(rb * ROWS_WG + wave * 32)))) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kbase + acc_row(r, h2);
          if (!(key < len && (!CAUSAL || key <= q))) s[r] = -INFINITY;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = exp2_raw(fmaf(s[r], c, -L2)) * (dp[r] - dl);   // dS^T
      const bf16x8_t dsf[2] = {pack8(s, 0), pack8(s, 1)};
      pipelined<NB / TBATCH>(
          load_t,
          [&](auto bi, auto sl) {
            constexpr int d0 = decltype(bi)::value * TBATCH, S = decltype(sl)::value;
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
              for (int db = 0; db < TBATCH; ++db)
                acc[d0 + db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf[S][db][st], dsf[st], acc[d0 + db], 0, 0, 0);
          },
          EARLY);
    }
  }
  if (qok) {
    bf16_t *drow = dqkv + ((size_t)b * Tn + q) * ld + hd * dh;
#pragma unroll
    for (int db = 0; db < NB; ++db)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        float v[4] = {acc[db][qd * 4] * scale, acc[db][qd * 4 + 1] * scale, acc[db][qd * 4 + 2] * scale,
                      acc[db][qd * 4 + 3] * scale};
        if (db * 32 + qd * 8 + h2 * 4 < dh) VecIO<bf16_t, 4>::store(drow + db * 32 + qd * 8 + h2 * 4, v);
      }
  }
}

// ------------------------------------------------------------------------------------------ dK, dV
// MODE 0 computes both; MODE 1 only dV, MODE 2 only dK.  Head size 256 runs it twice (1 then 2): two
// accumulator sets of DH/32 x 16 registers plus the K and V fragments do not fit the register file.
template <int DH, int MODE, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(NT, dkv_waves(DH)) void attn_bwd_dkv_mfma(const bf16_t *__restrict__ qkv,
                                                        const bf16_t *__restrict__ dout,
                                                        const float *__restrict__ lse,
                                                        const float *__restrict__ delta,
                                                        const int32_t *__restrict__ lengths, DropSpec drop, int Tn,
                                                        int H, int dh, float scale, bf16_t *__restrict__ dqkv) {
  constexpr bool DO_DV = MODE != 2, DO_DK = MODE != 1;
  constexpr int KS = kc_stride(DH), TS = tr_stride(DH), NK = DH / 16, NB = DH / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t *sQ = reinterpret_cast<bf16_t *>(smem_raw);   // Q rows for S = Q K^T
  bf16_t *sQt = sQ + TILE * KS;                        // Q again, for Q^T in dK^T = Q^T dS
  bf16_t *sDO = sQt + TILE * TS;                       // dO rows for dP = dO V^T
  bf16_t *sDOt = sDO + TILE * KS;                      // dO again, for dO^T in dV^T = dO^T P
  float *sL = reinterpret_cast<float *>(sDOt + TILE * TS);  // lse*log2(e) of the tile's queries
  float *sDl = sL + TILE;                                   // delta of the tile's queries
  constexpr int KBATCH = DH <= 64 ? 1 : 2;   // Q and dO fragments in flight (8 registers per step)
  constexpr int TBATCH = DH <= 64 ? 1 : (NB % 3 == 0 && DH < 192) ? 3 : 2;   // transposed dO / Q fragment pairs in flight
  static_assert(NK % KBATCH == 0 && NB % TBATCH == 0, "batches must divide the head size");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h2 = lane >> 5;
  const AttnBlock blk = attn_block();
  const int b = blk.b, hd = blk.hd, rb = blk.rb;
  const int D = H * dh;
  const size_t ld = (size_t)3 * D;
  const int len = lengths ? min(max(lengths[b], 1), Tn) : Tn;  // a length outside 1..T is treated as the nearest valid one
  const bf16_t *base = qkv + (size_t)b * Tn * ld + hd * dh;
  const int key = rb * ROWS_WG + wave * 32 + (lane & 31);
  const bool kok = key < Tn;
  const bf16_t *krow = kok ? base + (size_t)key * ld + D : nullptr;
  const bf16_t *vrow = kok ? base + (size_t)key * ld + 2 * D : nullptr;
  bf16x8_t kf[NK], vf[DO_DK ? NK : 1];
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) {
    kf[kk] = g_frag(krow, kk, lane, dh);
    if constexpr (DO_DK) vf[kk] = g_frag(vrow, kk, lane, dh);
  }
  const float c = scale * LOG2E;
  const bool live = key < len;   // a masked key has probability 0 against every query
  f32x16_t dk[DO_DK ? NB : 1], dv[DO_DV ? NB : 1];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      if constexpr (DO_DK) dk[i][r] = 0.f;
      if constexpr (DO_DV) dv[i][r] = 0.f;
    }
  // a workgroup whose keys are all masked only writes zeros
  const bool wg_live = rb * ROWS_WG < len;
  const size_t stat0 = ((size_t)b * H + hd) * Tn;
  const bf16_t *dobase = dout + (size_t)b * Tn * D + hd * dh;

  TileRegs<DH> tq, tdo;
  float rl = INFINITY, rd = 0.f;   // this thread's lse / delta entry of the tile (threads < TILE)
  auto load_tile = [&](int q0) {
    const int nvalid = min(TILE, Tn - q0);
    tq.load(base + (size_t)q0 * ld, ld, nvalid, dh);
    tdo.load(dobase + (size_t)q0 * D, (size_t)D, nvalid, dh);
    if (threadIdx.x < TILE) {
      const bool ok = (int)threadIdx.x < nvalid;
      rl = ok ? lse[stat0 + q0 + threadIdx.x] * LOG2E : INFINITY;   // exp2(-inf) = 0 beyond T
      rd = ok ? delta[stat0 + q0 + threadIdx.x] : 0.f;
    }
  };
  // with the causal mask only queries at or after a key see it: start at the tile of the workgroup's
  // first key (ROWS_WG is a multiple of TILE) and let a wavefront skip query blocks before its keys
  const int qbeg = CAUSAL ? (int)(rb * ROWS_WG) : 0;
  const int wkey0 = rb * ROWS_WG + wave * 32;
  if (wg_live) load_tile(qbeg);
  for (int q0 = qbeg; wg_live && q0 < Tn; q0 += TILE) {
    __syncthreads();
    tq.store(sQ, KS, DO_DK ? sQt : nullptr, TS);
    if constexpr (DO_DK) tdo.store(sDO, KS, DO_DV ? sDOt : nullptr, TS);
    else tdo.store(sDOt, TS, nullptr, 0);
    if (threadIdx.x < TILE) {
      sL[threadIdx.x] = rl;
      sDl[threadIdx.x] = rd;
    }
    __syncthreads();
    if (q0 + TILE < Tn) load_tile(q0 + TILE);
#pragma unroll (DH >= 128 ? 1 : 2)
    for (int qb = 0; qb < 2; ++qb) {
      if (q0 + qb * 32 >= Tn) break;
      if (CAUSAL && q0 + qb * 32 + 31 < wkey0) continue;
      f32x16_t s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f, dp[r] = 0.f;
      // Q and dO row fragments in batches, the next batch requested before the MFMAs of this one
      constexpr bool SAHEAD = !(DROP && DH >= 192);   // statistics one group ahead: not where the mask generator needs the registers
      bf16x8_t qfr[2][KBATCH], dofr[2][KBATCH];
      pipelined<NK / KBATCH>(
          [&](auto bi, auto sl) {
            constexpr int kh = decltype(bi)::value * KBATCH, S = decltype(sl)::value;
#pragma unroll
            for (int kk = 0; kk < KBATCH; ++kk) {
              qfr[S][kk] = kc_frag(sQ, KS, qb * 32, kh + kk, lane);
              dofr[S][kk] = DO_DK ? kc_frag(sDO, KS, qb * 32, kh + kk, lane) : qfr[S][kk];
            }
          },
          [&](auto bi, auto sl) {
            constexpr int kh = decltype(bi)::value * KBATCH, S = decltype(sl)::value;
#pragma unroll
            for (int kk = 0; kk < KBATCH; ++kk) {
              s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfr[S][kk], kf[kh + kk], s, 0, 0, 0);
              if (DO_DK) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dofr[S][kk], vf[kh + kk], dp, 0, 0, 0);
            }
          });
      // dV^T += dO^T P, then dK^T += Q^T dS: one sequence of batches of transposed fragments; the first
      // batch is requested before the dS arithmetic (not with dropout: the mask generator needs the registers)
      constexpr int NBV = DO_DV ? NB / TBATCH : 0, NBK = DO_DK ? NB / TBATCH : 0;
      bf16x8_t tf[2][TBATCH][2];
      auto load_t = [&](auto bi, auto sl) {
        constexpr int J = decltype(bi)::value, S = decltype(sl)::value;
        constexpr bool V = J < NBV;
        constexpr int d0 = (V ? J : J - NBV) * TBATCH;
#pragma unroll
        for (int db = 0; db < TBATCH; ++db)
#pragma unroll
          for (int st = 0; st < 2; ++st)
            tf[S][db][st] = tr_frag(V ? sDOt : sQt, TS, (d0 + db) * 32, qb * 32 + 16 * st, lane);
      };
      constexpr bool EARLY = !DROP;
      if constexpr (EARLY) {
        load_t(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        issue_fence();
      }
      // The statistics of the block's queries are read as whole 16-byte groups (registers 4g..4g+3 of a
      // lane half hold four consecutive queries), one group ahead of their use, and pinned: read where they
      // are used, each sits behind the `live` test in a branch of its own and costs a full LDS round trip,
      // sixteen times per block.
      auto stats = [&](int g, float4 &l4, float4 &d4) {
        l4 = *reinterpret_cast<const float4 *>(sL + qb * 32 + g * 8 + h2 * 4);
        d4 = *reinterpret_cast<const float4 *>(sDl + qb * 32 + g * 8 + h2 * 4);
        asm volatile("" : "+v"(l4.x), "+v"(l4.y), "+v"(l4.z), "+v"(l4.w), "+v"(d4.x), "+v"(d4.y), "+v"(d4.z), "+v"(d4.w));
      };
      float4 l4n, d4n;
      if constexpr (SAHEAD) stats(0, l4n, d4n);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float lq[4], dq[4];
        if constexpr (SAHEAD) {
          const float4 l4 = l4n, d4 = d4n;
          if (g < 3) stats(g + 1, l4n, d4n);   // one group ahead
          lq[0] = l4.x, lq[1] = l4.y, lq[2] = l4.z, lq[3] = l4.w;
          dq[0] = d4.x, dq[1] = d4.y, dq[2] = d4.z, dq[3] = d4.w;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            lq[e] = sL[qb * 32 + g * 8 + h2 * 4 + e];
            dq[e] = sDl[qb * 32 + g * 8 + h2 * 4 + e];
          }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = g * 4 + e, qi = qb * 32 + acc_row(r, h2);
          const float ex = exp2_raw(s[r] * c - lq[e]);
          const float p = (live && (!CAUSAL || q0 + qi >= key)) ? ex : 0.f;
          float keep = 1.f;   // this lane's key against sixteen different queries: one generator call each
          if constexpr (DROP) keep = drop_keep1(drop, (uint32_t)key, (uint32_t)(q0 + qi), (uint32_t)(b * H + hd));
          if constexpr (DO_DK) dp[r] = p * (dp[r] * keep - dq[e]);   // dS
          s[r] = p * keep;   // dV sees the dropped-out probabilities
        }
      }
      const bf16x8_t pf[2] = {pack8(s, 0), pack8(s, 1)}, dsf[2] = {pack8(dp, 0), pack8(dp, 1)};
      pipelined<NBV + NBK>(
          load_t,
          [&](auto bi, auto sl) {
            constexpr int J = decltype(bi)::value, S = decltype(sl)::value;
            constexpr bool V = J < NBV;
            constexpr int d0 = (V ? J : J - NBV) * TBATCH;
#pragma unroll
            for (int db = 0; db < TBATCH; ++db)
#pragma unroll
              for (int st = 0; st < 2; ++st) {
                if constexpr (V) dv[d0 + db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf[S][db][st], pf[st], dv[d0 + db], 0, 0, 0);
                else dk[d0 + db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf[S][db][st], dsf[st], dk[d0 + db], 0, 0, 0);
              }
          },
          EARLY);
    }
  }
  if (kok) {
    bf16_t *dkrow = dqkv + ((size_t)b * Tn + key) * ld + D + hd * dh;
    bf16_t *dvrow = dkrow + D;
#pragma unroll
    for (int db = 0; db < NB; ++db)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        if constexpr (DO_DK) {
          float a[4] = {dk[db][qd * 4] * scale, dk[db][qd * 4 + 1] * scale, dk[db][qd * 4 + 2] * scale,
                        dk[db][qd * 4 + 3] * scale};
          if (db * 32 + qd * 8 + h2 * 4 < dh) VecIO<bf16_t, 4>::store(dkrow + db * 32 + qd * 8 + h2 * 4, a);
        }
        if constexpr (DO_DV) {
          float v[4] = {dv[db][qd * 4], dv[db][qd * 4 + 1], dv[db][qd * 4 + 2], dv[db][qd * 4 + 3]};
          if (db * 32 + qd * 8 + h2 * 4 < dh) VecIO<bf16_t, 4>::store(dvrow + db * 32 + qd * 8 + h2 * 4, v);
        }
      }
  }
}

template <int DH> size_t dkv_lds_bytes() {
  return (size_t)2 * TILE * (kc_stride(DH) + tr_stride(DH)) * sizeof(bf16_t) + 2 * TILE * sizeof(float);
}

template <int DH, bool CAUSAL, bool DROP>
hipError_t fwd_t(const void *qkv, const int32_t *lengths, const DropSpec &drop, int B, int T, int H, int dh, float scale,
                 void *o, float *lse, hipStream_t s) {
  dim3 grid((T + ROWS_WG - 1) / ROWS_WG, H, B);
  constexpr int KG = fwd_key_groups(DH, DROP);
  constexpr size_t lds = (size_t)(KG > 1 ? 2 : 1) * TILE * (kc_stride(DH) + tr_stride(DH)) * sizeof(bf16_t);
  static_assert(lds <= 160 * 1024, "the tiles fit in LDS");
  if (lds > 64 * 1024) {
    static bool raised = false;   // allow more than the default 64 KiB of dynamic LDS, once
    if (!raised) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(attn_fwd_mfma<DH, CAUSAL, DROP, KG>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      raised = true;
    }
  }
  hipLaunchKernelGGL((attn_fwd_mfma<DH, CAUSAL, DROP, KG>), grid, dim3(NT * KG), lds, s, static_cast<const bf16_t *>(qkv),
                     lengths, drop, T, H, dh, scale, static_cast<bf16_t *>(o), lse);
  return hipGetLastError();
}

template <int DH, int MODE, bool CAUSAL, bool DROP>
hipError_t launch_dkv(dim3 grid, size_t lds, const void *qkv, const void *dout, const float *lse, const float *delta,
                      const int32_t *lengths, const DropSpec &drop, int T, int H, int dh, float scale, void *dqkv,
                      hipStream_t s) {
  if (lds > 64 * 1024) {
    static bool raised = false;   // allow more than the default 64 KiB of dynamic LDS, once
    if (!raised) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(attn_bwd_dkv_mfma<DH, MODE, CAUSAL, DROP>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      raised = true;
    }
  }
  hipLaunchKernelGGL((attn_bwd_dkv_mfma<DH, MODE, CAUSAL, DROP>), grid, dim3(NT), lds, s,
                     static_cast<const bf16_t *>(qkv), static_cast<const bf16_t *>(dout), lse, delta, lengths, drop, T, H,
                     dh, scale, static_cast<bf16_t *>(dqkv));
  return hipGetLastError();
}

template <int DH, bool CAUSAL, bool DROP>
hipError_t bwd_t(const void *qkv, const void *o, const void *dout, const float *lse, const int32_t *lengths,
                 const DropSpec &drop, int B, int T, int H, int dh, float scale, void *dqkv, float *delta, hipStream_t s, int parts) {
  dim3 grid((T + ROWS_WG - 1) / ROWS_WG, H, B);
  hipError_t e = hipSuccess;
  if (parts & ATTN_BWD_DQ) {
    hipLaunchKernelGGL((attn_bwd_dq_mfma<DH, CAUSAL, DROP>), grid, dim3(NT), 0, s, static_cast<const bf16_t *>(qkv),
                       static_cast<const bf16_t *>(o), static_cast<const bf16_t *>(dout), lse, lengths, drop, T, H,
                       dh, scale, static_cast<bf16_t *>(dqkv), delta);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (!(parts & ATTN_BWD_DKV)) return e;
  const size_t lds = dkv_lds_bytes<DH>();
  e = launch_dkv<DH, dkv_two_passes(DH) ? 1 : 0, CAUSAL, DROP>(grid, lds, qkv, dout, lse, delta, lengths, drop, T, H, dh, scale, dqkv,
                                                      s);
  if (e != hipSuccess || !dkv_two_passes(DH)) return e;
  return launch_dkv<DH, 2, CAUSAL, DROP>(grid, lds, qkv, dout, lse, delta, lengths, drop, T, H, dh, scale, dqkv, s);
}

// the four (causal, dropout) instances of one head size
template <int DH>
hipError_t fwd_pick(int causal, const void *qkv, const int32_t *lengths, const DropSpec &drop, int B, int T, int H,
                    int dh, float scale, void *o, float *lse, hipStream_t s) {
  if (causal) return drop.thr ? fwd_t<DH, true, true>(qkv, lengths, drop, B, T, H, dh, scale, o, lse, s)
                              : fwd_t<DH, true, false>(qkv, lengths, drop, B, T, H, dh, scale, o, lse, s);
  return drop.thr ? fwd_t<DH, false, true>(qkv, lengths, drop, B, T, H, dh, scale, o, lse, s)
                  : fwd_t<DH, false, false>(qkv, lengths, drop, B, T, H, dh, scale, o, lse, s);
}
template <int DH>
hipError_t bwd_pick(int causal, const void *qkv, const void *o, const void *dout, const float *lse,
                    const int32_t *lengths, const DropSpec &drop, int B, int T, int H, int dh, float scale, void *dqkv,
                    float *delta, hipStream_t s, int parts) {
  if (causal)
    return drop.thr ? bwd_t<DH, true, true>(qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts)
                    : bwd_t<DH, true, false>(qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts);
  return drop.thr ? bwd_t<DH, false, true>(qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts)
                  : bwd_t<DH, false, false>(qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts);
}

}  // namespace

bool attention_mfma_supported(int dh) { return dh >= 16 && dh <= 256 && dh % 16 == 0; }

namespace {
// the kernel instance a head size runs on
int instance_of(int dh) { return dh <= 128 ? (dh + 31) / 32 * 32 : dh <= 192 ? 192 : 256; }
}  // namespace

hipError_t launch_attention_fwd_mfma(const void *qkv, const int32_t *lengths, int causal, const DropSpec &drop, int B,
                                     int T, int H, int dh, void *o, float *lse, hipStream_t s) {
  const float scale = 1.0f / sqrtf((float)dh);
  if (!attention_mfma_supported(dh)) return hipErrorInvalidValue;
  switch (instance_of(dh)) {
    case 32: return fwd_pick<32>(causal, qkv, lengths, drop, B, T, H, dh, scale, o, lse, s);
    case 64: return fwd_pick<64>(causal, qkv, lengths, drop, B, T, H, dh, scale, o, lse, s);
    case 96: return fwd_pick<96>(causal, qkv, lengths, drop, B, T, H, dh, scale, o, lse, s);
    case 128: return fwd_pick<128>(causal, qkv, lengths, drop, B, T, H, dh, scale, o, lse, s);
    case 192: return fwd_pick<192>(causal, qkv, lengths, drop, B, T, H, dh, scale, o, lse, s);
    case 256: return fwd_pick<256>(causal, qkv, lengths, drop, B, T, H, dh, scale, o, lse, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_attention_bwd_mfma(const void *qkv, const void *o, const void *dout, const float *lse,
                                     const int32_t *lengths, int causal, const DropSpec &drop, int B, int T, int H,
                                     int dh, void *dqkv, float *delta, hipStream_t s, int parts) {
  const float scale = 1.0f / sqrtf((float)dh);
  if (!attention_mfma_supported(dh)) return hipErrorInvalidValue;
  if ((parts & (ATTN_BWD_DQ | ATTN_BWD_DKV)) == (ATTN_BWD_DQ | ATTN_BWD_DKV) && attention_bwd_fused_applies(T, dh))
    return launch_attention_bwd_fused(qkv, o, dout, lse, lengths, causal, drop, B, T, H, dh, dqkv, s);
  switch (instance_of(dh)) {
    case 32: return bwd_pick<32>(causal, qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts);
    case 64: return bwd_pick<64>(causal, qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts);
    case 96: return bwd_pick<96>(causal, qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts);
    case 128: return bwd_pick<128>(causal, qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts);
    case 192: return bwd_pick<192>(causal, qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts);
    case 256: return bwd_pick<256>(causal, qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts);
  }
  return hipErrorInvalidValue;
}

}  // namespace fl
