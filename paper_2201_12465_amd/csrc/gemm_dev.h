// Device-side argument block and epilogue shared by the GEMM kernels.
#pragma once
#include "devutil.h"
#include "philox.h"

namespace fl {

struct GemmDev {
  const void *A, *B;
  void *C;
  int M, N, K, lda, ldb, ldc;
  const void *bias, *residual, *aux;
  void *preact;
  int act, dact;
  float *partial;
  int k_per_split, tiles_m, tiles_n, splits;
  int drop_where;  // 0 none, 1 = after the activation (forward), 2 = with the activation derivative (backward)
  DropSpec drop;
};


// The epilogue steps (see GemmArgs for their order) on eight consecutive outputs C[m, n0..n0+7]:
// 16-byte (bf16) / 32-byte (fp32) accesses.
template <typename T> struct Oct;
template <> struct Oct<bf16_t> {
  static __device__ __forceinline__ void load(const bf16_t *p, float *v) { VecIO<bf16_t, 8>::load(p, v); }
  static __device__ __forceinline__ void store(bf16_t *p, const float *v) { VecIO<bf16_t, 8>::store(p, v); }
};
template <> struct Oct<float> {
  static __device__ __forceinline__ void load(const float *p, float *v) {
    VecIO<float, 4>::load(p, v);
    VecIO<float, 4>::load(p + 4, v + 4);
  }
  static __device__ __forceinline__ void store(float *p, const float *v) {
    VecIO<float, 4>::store(p, v);
    VecIO<float, 4>::store(p + 4, v + 4);
  }
};

// What of the epilogue an instance of a kernel carries.  The steps a launch does not use are dead code, but
// straight-line code that every workgroup walks once (the epilogue is unrolled over a wavefront's 32-row blocks
// and passes) is fetched all the same, and the GELU / GELU' evaluations are most of it: a plain 4096 x 768 x 768
// GEMM is 0.6-1.4 us shorter without them.
constexpr int EPI_PARTIAL = 0;   // fp32 partial sums of a k-range only
constexpr int EPI_LIGHT = 1;     // everything but GELU and its derivative
constexpr int EPI_FULL = 2;
constexpr int EPI_GELU_FWD = 3;  // GELU as the activation, no activation derivative
constexpr int EPI_GELU_BWD = 4;  // GELU' as the activation derivative, no activation
constexpr int EPI_PLAIN = 5;     // bias and residual only
__host__ __device__ constexpr int gemm_epi_kind(bool partial, int act, int dact, bool preact = true) {
  return partial ? EPI_PARTIAL
         : act == 2 ? (dact ? EPI_FULL : EPI_GELU_FWD)
         : dact == 2 ? (act ? EPI_FULL : EPI_GELU_BWD)
         : (act == 0 && dact == 0 && !preact) ? EPI_PLAIN : EPI_LIGHT;
}

// PRE: the eight residual / aux values were already loaded by the caller (pre_res, pre_aux; bf16 only).
template <typename T, bool DROP, bool PRE = false, int EPI = EPI_FULL>
__device__ __forceinline__ void gemm_epilogue_oct(const GemmDev &p, int m, int n0, float (&v)[8],
                                                  const float (&bias8)[8], bf16x8_t pre_res = bf16x8_t{},
                                                  bf16x8_t pre_aux = bf16x8_t{}) {
  if (EPI == EPI_PARTIAL || p.partial) {
    Oct<float>::store(p.partial + (size_t)m * p.N + n0, v);
    return;
  }
  const size_t off = (size_t)m * p.ldc + n0;
  float t[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] += bias8[e];  // zeros without a bias
  if (EPI != EPI_PLAIN && p.preact) Oct<T>::store(static_cast<T *>(p.preact) + off, v);
  if (EPI == EPI_GELU_FWD || (EPI == EPI_FULL && p.act == 2)) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = gelu_f(v[e]);
  } else if (EPI != EPI_GELU_BWD && EPI != EPI_PLAIN && p.act == 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
  }
  if (DROP && p.drop_where == 1) {
    float k0[4], k1[4];
    drop_keep4(p.drop, (uint32_t)n0 >> 2, (uint32_t)m, 0u, k0);
    drop_keep4(p.drop, ((uint32_t)n0 >> 2) + 1, (uint32_t)m, 0u, k1);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] *= k0[e], v[e + 4] *= k1[e];
  }
  if (p.residual) {
    if constexpr (PRE) {
#pragma unroll
      for (int e = 0; e < 8; ++e) t[e] = static_cast<float>(pre_res[e]);
    } else {
      Oct<T>::load(static_cast<const T *>(p.residual) + off, t);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += t[e];
  }
  if (EPI != EPI_GELU_FWD && EPI != EPI_PLAIN && p.dact) {
    if constexpr (PRE) {
#pragma unroll
      for (int e = 0; e < 8; ++e) t[e] = static_cast<float>(pre_aux[e]);
    } else {
      Oct<T>::load(static_cast<const T *>(p.aux) + off, t);
    }
    if (EPI == EPI_LIGHT || (EPI == EPI_FULL && p.dact == 1)) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = t[e] > 0.f ? v[e] : 0.f;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f(t[e]);
    }
  }
  if (DROP && p.drop_where == 2) {
    float k0[4], k1[4];
    drop_keep4(p.drop, (uint32_t)n0 >> 2, (uint32_t)m, 0u, k0);
    drop_keep4(p.drop, ((uint32_t)n0 >> 2) + 1, (uint32_t)m, 0u, k1);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] *= k0[e], v[e + 4] *= k1[e];
  }
  Oct<T>::store(static_cast<T *>(p.C) + off, v);
}

// Epilogue of a wavefront's (TM*32) x (TN*32) accumulator block through LDS.  acc[i][j] is the
// 32x32 MFMA tile (i, j) in the "D = B_frag x A_frag" orientation: register q*4+e of a lane holds
// C[i*32 + lane%32, j*32 + q*8 + (lane/32)*4 + e].  Thirty-two rows at a time are parked in the
// wave's own LDS region (rows padded by 4 floats: the 16-byte writes and the reads below touch
// every bank once) and walked row-wise, so that every global access is 16 or 32 bytes per lane and
// a row's TN*32 outputs form one contiguous segment.  `cw` must hold 32*(TN*32+4) floats per wave.
// The caller has made sure (barrier) that nobody still reads the LDS this overwrites.
template <typename T, int TM, int TN, bool DROP, int EPI = EPI_FULL>
__device__ __forceinline__ void gemm_staged_epilogue(const GemmDev &p, const f32x16_t (&acc)[TM][TN], float *cw,
                                                     int mbase, int nbase, int lane) {
  constexpr int WC = TN * 32, CS = WC + 4;
  constexpr int LPR = WC / 8, RPP = 64 / LPR;  // lanes per row, rows per pass (lanes beyond LPR*RPP idle)
  constexpr int PASSES = (32 + RPP - 1) / RPP;
  // bf16: 4 registers per prefetched oct; the large wavefront tiles have no registers to spare
  constexpr bool PRE = sizeof(T) == 2 && TM * TN <= 4 && EPI != EPI_PARTIAL;
  const int rl = lane / LPR, c8 = lane % LPR;
  const int n0 = nbase + c8 * 8;
  const bool lane_ok = rl < RPP && n0 < p.N;
  // The residual and the activation-derivative operand of every pass are requested up front: inside
  // the pass loop each load would be waited for on its own, one memory latency per pass, with
  // nothing left to overlap it at the end of the kernel.
  float bias8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // a lane's eight columns are the same in every pass
  if (EPI != EPI_PARTIAL && p.bias && !p.partial && lane_ok) Oct<T>::load(static_cast<const T *>(p.bias) + n0, bias8);
  bf16x8_t pre_res[PRE ? TM : 1][PRE ? PASSES : 1], pre_aux[PRE ? TM : 1][PRE ? PASSES : 1];
  if constexpr (PRE) {
    const bool has_res = p.residual && !p.partial, has_aux = EPI != EPI_PLAIN && EPI != EPI_GELU_FWD && p.dact && !p.partial;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int k = 0; k < PASSES; ++k) {
        const int r = rl + k * RPP, m = mbase + i * 32 + r;
        const bool ok = lane_ok && r < 32 && m < p.M;
        const size_t off = (size_t)m * p.ldc + n0;
        pre_res[i][k] = bf16x8_t{};
        pre_aux[i][k] = bf16x8_t{};
        if (has_res && ok) pre_res[i][k] = *reinterpret_cast<const bf16x8_t *>(static_cast<const bf16_t *>(p.residual) + off);
        if (has_aux && ok) pre_aux[i][k] = *reinterpret_cast<const bf16x8_t *>(static_cast<const bf16_t *>(p.aux) + off);
      }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4 *>(cw + (lane & 31) * CS + j * 32 + q * 8 + (lane >> 5) * 4) =
            make_float4(acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]);
    // the wave reads what its own lanes wrote: LDS operations of one wave complete in order.
    // Without prefetched operands (register arrays indexed by the pass) the passes stay a loop: less code to fetch.
#pragma unroll (PRE ? PASSES : 1)
    for (int k = 0; k < PASSES; ++k) {
      const int r = rl + k * RPP;
      const int m = mbase + i * 32 + r;
      if (lane_ok && r < 32 && m < p.M) {
        const float4 lo = *reinterpret_cast<const float4 *>(cw + r * CS + c8 * 8);
        const float4 hi = *reinterpret_cast<const float4 *>(cw + r * CS + c8 * 8 + 4);
        float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        if constexpr (PRE) gemm_epilogue_oct<T, DROP, true, EPI>(p, m, n0, v, bias8, pre_res[i][k], pre_aux[i][k]);
        else gemm_epilogue_oct<T, DROP, false, EPI>(p, m, n0, v, bias8);
      }
    }
  }
}

// The 8 XCDs receive workgroup ids round-robin; give each a contiguous range of tiles.
__device__ __forceinline__ int xcd_tile_order(int bid, int nb) { return xcd_contiguous_order(bid, nb); }

// Work item (k-range `split`, tile (tm, tn)) of workgroup `bid` of a one-dimensional grid of
// splits * tiles_m * tiles_n workgroups.  Each XCD has its own L2 and takes a contiguous range of an
// order in which neighbours share operands: k-range first (so that an XCD reads one k-slice of both
// operands rather than all of them), then row-tiles in groups of `gm`, and inside a group down the
// group's rows before moving to the next column, so the tiles an XCD works on at one time share few
// operand panels and those stay in its L2.
__device__ __forceinline__ void xcd_work_coords(int bid, int tiles_m, int tiles_n, int splits, int gm, int &split,
                                                int &tm, int &tn) {
  const int tiles = tiles_m * tiles_n;
  int id = xcd_tile_order(bid, tiles * splits);
  split = id / tiles;
  id -= split * tiles;
  const int per_group = gm * tiles_n;
  const int g = id / per_group, r = id - g * per_group;
  const int rows = min(gm, tiles_m - g * gm);  // the last group may be shorter
  tn = r / rows;
  tm = g * gm + (r - tn * rows);
}

}  // namespace fl
