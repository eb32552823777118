// Fused masked attention in fp32 on the matrix cores (v_mfma_f32_32x32x2_f32), forward and
// backward, for head sizes up to 128 (multiples of 16; a kernel instance is built for each multiple of
// 32 and the next smaller size runs on it with its upper 16 columns read as zeros and never stored).
//
// Same operator, same decomposition and same orientation of the score blocks as the bf16 kernels
// in attention_mfma.hip (the paper's matmul / exp / max / sum primitives, Section 4.1.1, fused with
// a pre-fused gradient function, Section 5.2.1): a wavefront owns 32 query rows (forward, dQ) or
// 32 key rows (dK/dV) and walks the other sequence dimension in LDS tiles; the MFMA that produces
// a score block leaves the index contracted NEXT in a lane's registers, so probabilities go from
// accumulator registers straight into the next MFMA.
//
// The fp32 MFMA contracts two k per instruction: lanes 0..31 supply k = 0, lanes 32..63 k = 1, one
// value per lane for each operand.  With fp32 there is nothing to pack and nothing to transpose:
//   "row" fragments  (contraction along the head dimension): lane reads tile[row0 + lane%32][2*kk + lane/32]
//   "column" fragments (contraction along the walked rows): lane reads tile[krow][col0 + lane%32],
//       where krow is the tile row whose score sits in register t of THIS lane half -- the two
//       halves of a wavefront hold different rows in the same register, and the instruction only
//       needs both operands to agree on which row is "k = lane/32".
// Tiles are row-major fp32 with four floats of padding per row.
#include "devutil.h"
#include "kernels.h"
#include "philox.h"

namespace fl {
namespace {

constexpr int NT = 256;        // threads per workgroup (4 wavefronts)
constexpr int ROWS_WG = 128;   // rows owned by a workgroup (32 per wavefront)
constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;

constexpr int tile_rows(int dh) { return dh <= 64 ? 64 : 32; }   // rows of the walked dimension per LDS tile
constexpr int row_stride(int dh) { return dh + 4; }

__device__ __forceinline__ int acc_row(int r, int h) { return (r >> 2) * 8 + h * 4 + (r & 3); }

__device__ __forceinline__ f32x16_t mfma2(float a, float b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ void zero16(f32x16_t &v) {
#pragma unroll
  for (int r = 0; r < 16; ++r) v[r] = 0.f;
}

// A tile of up to TILE rows of DH floats on its way from global memory to LDS (rows >= nvalid are zero):
// load() issues the global reads, store() writes the tile; the kernels load tile t+1 right after storing
// tile t so that the reads are in flight during the MFMAs.
template <int DH> struct TileRegsF {
  static constexpr int TILE = tile_rows(DH), CPR = DH / 4, N = TILE * CPR / NT;
  static_assert(TILE * CPR % NT == 0, "tile must divide among the threads");
  float4 r[N];
  __device__ __forceinline__ void load(const float *src, size_t ld, int nvalid, int dh) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + NT * i, row = c / CPR, ch = c % CPR;
      r[i] = row < nvalid && ch * 4 < dh ? *reinterpret_cast<const float4 *>(src + (size_t)row * ld + ch * 4)
                                         : make_float4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(float *dst) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + NT * i, row = c / CPR, ch = c % CPR;
      *reinterpret_cast<float4 *>(dst + row * row_stride(DH) + ch * 4) = r[i];
    }
  }
};

// this lane's operand values of its own row: element 2*kk + lane/32 for every k-step kk (zeros without a row)
template <int DH> __device__ __forceinline__ void own_row(const float *row, int h2, int dh, float (&f)[DH / 2]) {
#pragma unroll
  for (int kk = 0; kk < DH / 2; ++kk) f[kk] = row && 2 * kk < dh ? row[2 * kk + h2] : 0.f;
}

// ------------------------------------------------------------------------------------------ forward
template <int DH, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(NT) void attn_fwd_mfma_f32(const float *__restrict__ qkv, const int32_t *__restrict__ lengths,
                                                        DropSpec drop, int Tn, int H, int dh, float scale,
                                                        float *__restrict__ o, float *__restrict__ lse) {
  constexpr int TILE = tile_rows(DH), ST = row_stride(DH), NB = DH / 32;
  __shared__ __attribute__((aligned(16))) float sK[TILE * ST];
  __shared__ __attribute__((aligned(16))) float sV[TILE * ST];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h2 = lane >> 5, l32 = lane & 31;
  const AttnBlock blk = attn_block();
  const int b = blk.b, hd = blk.hd, rb = blk.rb;
  const int D = H * dh;
  const size_t ld = (size_t)3 * D;
  const int len = lengths ? min(max(lengths[b], 1), Tn) : Tn;  // a length outside 1..T is treated as the nearest valid one
  const float *base = qkv + (size_t)b * Tn * ld + hd * dh;
  const int q = rb * ROWS_WG + wave * 32 + l32;
  float qf[DH / 2];
  own_row<DH>(q < Tn ? base + (size_t)q * ld : nullptr, h2, dh, qf);
  const float c = scale * LOG2E;
  float m = -INFINITY, l = 0.f;
  f32x16_t oacc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) zero16(oacc[i]);

  // causal: the workgroup needs keys up to its last query, a wavefront up to the last of its 32 queries
  const int kend = CAUSAL ? min(len, (int)(rb * ROWS_WG + ROWS_WG)) : len;
  const int wend = CAUSAL ? min(len, (int)(rb * ROWS_WG + wave * 32 + 32)) : len;
  TileRegsF<DH> tk, tv;
  tk.load(base + D, ld, min(TILE, Tn), dh);
  tv.load(base + 2 * D, ld, min(TILE, Tn), dh);
  for (int k0 = 0; k0 < kend; k0 += TILE) {
    __syncthreads();
    tk.store(sK);
    tv.store(sV);
    __syncthreads();
    if (k0 + TILE < kend) {
      tk.load(base + (size_t)(k0 + TILE) * ld + D, ld, min(TILE, Tn - k0 - TILE), dh);
      tv.load(base + (size_t)(k0 + TILE) * ld + 2 * D, ld, min(TILE, Tn - k0 - TILE), dh);
    }
#pragma unroll
    for (int kb = 0; kb < TILE / 32; ++kb) {
      if (k0 + kb * 32 >= wend) break;
      f32x16_t s;
      zero16(s);
      const float *krow = sK + (kb * 32 + l32) * ST + h2;
#pragma unroll
      for (int kk = 0; kk < DH / 2; ++kk) s = mfma2(krow[2 * kk], qf[kk], s);   // S^T[key, q]
      float mloc = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = k0 + kb * 32 + acc_row(r, h2);
        s[r] = (key < len && (!CAUSAL || key <= q)) ? s[r] * c : -INFINITY;
        mloc = fmaxf(mloc, s[r]);
      }
      mloc = half_pair_max(mloc);
      const float mnew = fmaxf(m, mloc);
      float rs = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[r] = exp2f(s[r] - mnew);
        rs += s[r];
      }
      rs = half_pair_sum(rs);
      const float corr = exp2f(m - mnew);
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
#pragma unroll
      for (int db = 0; db < NB; ++db) {
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= corr;
#pragma unroll
        for (int t = 0; t < 16; ++t)   // O^T[d, q] += V^T[d, key] P^T[key, q], key = the one register t holds
          oacc[db] = mfma2(sV[(kb * 32 + acc_row(t, h2)) * ST + db * 32 + l32], s[t], oacc[db]);
      }
    }
  }
  if (q < Tn) {
    const float inv = 1.0f / l;
    float *orow = o + ((size_t)b * Tn + q) * D + hd * dh;
#pragma unroll
    for (int db = 0; db < NB; ++db)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        float v[4] = {oacc[db][qd * 4] * inv, oacc[db][qd * 4 + 1] * inv, oacc[db][qd * 4 + 2] * inv,
                      oacc[db][qd * 4 + 3] * inv};
        if (db * 32 + qd * 8 + h2 * 4 < dh) VecIO<float, 4>::store(orow + db * 32 + qd * 8 + h2 * 4, v);
      }
    if (h2 == 0) lse[((size_t)b * H + hd) * Tn + q] = (m + log2f(l)) * LN2;
  }
}

// ------------------------------------------------------------------------------------------ dQ (+ delta)
template <int DH, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(NT) void attn_bwd_dq_mfma_f32(const float *__restrict__ qkv, const float *__restrict__ o,
                                                           const float *__restrict__ dout,
                                                           const float *__restrict__ lse,
                                                           const int32_t *__restrict__ lengths, DropSpec drop, int Tn,
                                                           int H, int dh, float scale, float *__restrict__ dqkv,
                                                           float *__restrict__ delta) {
  constexpr int TILE = tile_rows(DH), ST = row_stride(DH), NB = DH / 32;
  __shared__ __attribute__((aligned(16))) float sK[TILE * ST];
  __shared__ __attribute__((aligned(16))) float sV[TILE * ST];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h2 = lane >> 5, l32 = lane & 31;
  const AttnBlock blk = attn_block();
  const int b = blk.b, hd = blk.hd, rb = blk.rb;
  const int D = H * dh;
  const size_t ld = (size_t)3 * D;
  const int len = lengths ? min(max(lengths[b], 1), Tn) : Tn;  // a length outside 1..T is treated as the nearest valid one
  const float *base = qkv + (size_t)b * Tn * ld + hd * dh;
  const int q = rb * ROWS_WG + wave * 32 + l32;
  const bool qok = q < Tn;
  float qf[DH / 2], dof[DH / 2];
  own_row<DH>(qok ? base + (size_t)q * ld : nullptr, h2, dh, qf);
  own_row<DH>(qok ? dout + ((size_t)b * Tn + q) * D + hd * dh : nullptr, h2, dh, dof);
  float dl = 0.f;
  {
    float of[DH / 2];
    own_row<DH>(qok ? o + ((size_t)b * Tn + q) * D + hd * dh : nullptr, h2, dh, of);
#pragma unroll
    for (int kk = 0; kk < DH / 2; ++kk) dl += dof[kk] * of[kk];
  }
  dl = half_pair_sum(dl);
  const size_t st_idx = ((size_t)b * H + hd) * Tn + (qok ? q : 0);
  const float L2 = qok ? lse[st_idx] * LOG2E : 0.f;
  if (qok && h2 == 0) delta[st_idx] = dl;
  const float c = scale * LOG2E;
  f32x16_t acc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) zero16(acc[i]);

  const int kend = CAUSAL ? min(len, (int)(rb * ROWS_WG + ROWS_WG)) : len;       // as in the forward kernel
  const int wend = CAUSAL ? min(len, (int)(rb * ROWS_WG + wave * 32 + 32)) : len;
  TileRegsF<DH> tk, tv;
  tk.load(base + D, ld, min(TILE, Tn), dh);
  tv.load(base + 2 * D, ld, min(TILE, Tn), dh);
  for (int k0 = 0; k0 < kend; k0 += TILE) {
    __syncthreads();
    tk.store(sK);
    tv.store(sV);
    __syncthreads();
    if (k0 + TILE < kend) {
      tk.load(base + (size_t)(k0 + TILE) * ld + D, ld, min(TILE, Tn - k0 - TILE), dh);
      tv.load(base + (size_t)(k0 + TILE) * ld + 2 * D, ld, min(TILE, Tn - k0 - TILE), dh);
    }
#pragma unroll
    for (int kb = 0; kb < TILE / 32; ++kb) {
      if (k0 + kb * 32 >= wend) break;
      f32x16_t s, dp;
      zero16(s);
      zero16(dp);
      const float *krow = sK + (kb * 32 + l32) * ST + h2;
      const float *vrow = sV + (kb * 32 + l32) * ST + h2;
#pragma unroll
      for (int kk = 0; kk < DH / 2; ++kk) {
        s = mfma2(krow[2 * kk], qf[kk], s);      // S^T[key, q]
        dp = mfma2(vrow[2 * kk], dof[kk], dp);   // dP^T[key, q]
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
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = k0 + kb * 32 + acc_row(r, h2);
        const float p = (key < len && (!CAUSAL || key <= q)) ? exp2f(s[r] * c - L2) : 0.f;
        s[r] = p * (dp[r] - dl);   // dS^T
      }
#pragma unroll
      for (int db = 0; db < NB; ++db)
#pragma unroll
        for (int t = 0; t < 16; ++t)   // dQ^T[d, q] += K^T[d, key] dS^T[key, q]
          acc[db] = mfma2(sK[(kb * 32 + acc_row(t, h2)) * ST + db * 32 + l32], s[t], acc[db]);
    }
  }
  if (qok) {
    float *drow = dqkv + ((size_t)b * Tn + q) * ld + hd * dh;
#pragma unroll
    for (int db = 0; db < NB; ++db)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        float v[4] = {acc[db][qd * 4] * scale, acc[db][qd * 4 + 1] * scale, acc[db][qd * 4 + 2] * scale,
                      acc[db][qd * 4 + 3] * scale};
        if (db * 32 + qd * 8 + h2 * 4 < dh) VecIO<float, 4>::store(drow + db * 32 + qd * 8 + h2 * 4, v);
      }
  }
}

// ------------------------------------------------------------------------------------------ dK, dV
template <int DH, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(NT) void attn_bwd_dkv_mfma_f32(const float *__restrict__ qkv,
                                                            const float *__restrict__ dout,
                                                            const float *__restrict__ lse,
                                                            const float *__restrict__ delta,
                                                            const int32_t *__restrict__ lengths, DropSpec drop, int Tn,
                                                            int H, int dh, float scale, float *__restrict__ dqkv) {
  constexpr int TILE = tile_rows(DH), ST = row_stride(DH), NB = DH / 32;
  __shared__ __attribute__((aligned(16))) float sQ[TILE * ST];
  __shared__ __attribute__((aligned(16))) float sDO[TILE * ST];
  __shared__ float sL[TILE], sDl[TILE];   // lse*log2(e) and delta of the tile's queries
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h2 = lane >> 5, l32 = lane & 31;
  const AttnBlock blk = attn_block();
  const int b = blk.b, hd = blk.hd, rb = blk.rb;
  const int D = H * dh;
  const size_t ld = (size_t)3 * D;
  const int len = lengths ? min(max(lengths[b], 1), Tn) : Tn;  // a length outside 1..T is treated as the nearest valid one
  const float *base = qkv + (size_t)b * Tn * ld + hd * dh;
  const int key = rb * ROWS_WG + wave * 32 + l32;
  const bool kok = key < Tn;
  float kf[DH / 2], vf[DH / 2];
  own_row<DH>(kok ? base + (size_t)key * ld + D : nullptr, h2, dh, kf);
  own_row<DH>(kok ? base + (size_t)key * ld + 2 * D : nullptr, h2, dh, vf);
  const float c = scale * LOG2E;
  const bool live = key < len;   // a masked key has probability 0 against every query
  f32x16_t dk[NB], dv[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    zero16(dk[i]);
    zero16(dv[i]);
  }
  const bool wg_live = rb * ROWS_WG < len;   // a workgroup whose keys are all masked only writes zeros
  const size_t stat0 = ((size_t)b * H + hd) * Tn;
  const float *dobase = dout + (size_t)b * Tn * D + hd * dh;

  TileRegsF<DH> tq, tdo;
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
  // causal: only queries at or after a key see it (ROWS_WG is a multiple of TILE)
  const int qbeg = CAUSAL ? (int)(rb * ROWS_WG) : 0;
  const int wkey0 = rb * ROWS_WG + wave * 32;
  if (wg_live) load_tile(qbeg);
  for (int q0 = qbeg; wg_live && q0 < Tn; q0 += TILE) {
    __syncthreads();
    tq.store(sQ);
    tdo.store(sDO);
    if (threadIdx.x < TILE) {
      sL[threadIdx.x] = rl;
      sDl[threadIdx.x] = rd;
    }
    __syncthreads();
    if (q0 + TILE < Tn) load_tile(q0 + TILE);
#pragma unroll
    for (int qb = 0; qb < TILE / 32; ++qb) {
      if (q0 + qb * 32 >= Tn) break;
      if (CAUSAL && q0 + qb * 32 + 31 < wkey0) continue;
      f32x16_t s, dp;
      zero16(s);
      zero16(dp);
      const float *qrow = sQ + (qb * 32 + l32) * ST + h2;
      const float *dorow = sDO + (qb * 32 + l32) * ST + h2;
#pragma unroll
      for (int kk = 0; kk < DH / 2; ++kk) {
        s = mfma2(qrow[2 * kk], kf[kk], s);       // S[q, key]
        dp = mfma2(dorow[2 * kk], vf[kk], dp);    // dP[q, key]
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qi = qb * 32 + acc_row(r, h2);
        const float p = (live && (!CAUSAL || q0 + qi >= key)) ? exp2f(s[r] * c - sL[qi]) : 0.f;
        float keep = 1.f;   // this lane's key against sixteen different queries: one generator call each
        if constexpr (DROP) keep = drop_keep1(drop, (uint32_t)key, (uint32_t)(q0 + qi), (uint32_t)(b * H + hd));
        dp[r] = p * (dp[r] * keep - sDl[qi]);   // dS
        s[r] = p * keep;                        // dV sees the dropped-out probabilities
      }
#pragma unroll
      for (int db = 0; db < NB; ++db)
#pragma unroll
        for (int t = 0; t < 16; ++t) {
          const int row = (qb * 32 + acc_row(t, h2)) * ST + db * 32 + l32;
          dv[db] = mfma2(sDO[row], s[t], dv[db]);    // dV^T[d, key] += dO^T[d, q] P[q, key]
          dk[db] = mfma2(sQ[row], dp[t], dk[db]);    // dK^T[d, key] += Q^T[d, q] dS[q, key]
        }
    }
  }
  if (kok) {
    float *dkrow = dqkv + ((size_t)b * Tn + key) * ld + D + hd * dh;
    float *dvrow = dkrow + D;
#pragma unroll
    for (int db = 0; db < NB; ++db)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        float a[4] = {dk[db][qd * 4] * scale, dk[db][qd * 4 + 1] * scale, dk[db][qd * 4 + 2] * scale,
                      dk[db][qd * 4 + 3] * scale};
        float v[4] = {dv[db][qd * 4], dv[db][qd * 4 + 1], dv[db][qd * 4 + 2], dv[db][qd * 4 + 3]};
        if (db * 32 + qd * 8 + h2 * 4 < dh) {
          VecIO<float, 4>::store(dkrow + db * 32 + qd * 8 + h2 * 4, a);
          VecIO<float, 4>::store(dvrow + db * 32 + qd * 8 + h2 * 4, v);
        }
      }
  }
}

template <int DH, bool CAUSAL, bool DROP>
hipError_t fwd_t(const float *qkv, const int32_t *lengths, const DropSpec &drop, int B, int T, int H, int dh, float scale,
                 float *o, float *lse, hipStream_t s) {
  dim3 grid((T + ROWS_WG - 1) / ROWS_WG, H, B);
  hipLaunchKernelGGL((attn_fwd_mfma_f32<DH, CAUSAL, DROP>), grid, dim3(NT), 0, s, qkv, lengths, drop, T, H, dh, scale, o, lse);
  return hipGetLastError();
}

template <int DH, bool CAUSAL, bool DROP>
hipError_t bwd_t(const float *qkv, const float *o, const float *dout, const float *lse, const int32_t *lengths,
                 const DropSpec &drop, int B, int T, int H, int dh, float scale, float *dqkv, float *delta,
                 hipStream_t s, int parts) {
  dim3 grid((T + ROWS_WG - 1) / ROWS_WG, H, B);
  if (parts & ATTN_BWD_DQ) {
    hipLaunchKernelGGL((attn_bwd_dq_mfma_f32<DH, CAUSAL, DROP>), grid, dim3(NT), 0, s, qkv, o, dout, lse, lengths, drop,
                       T, H, dh, scale, dqkv, delta);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (parts & ATTN_BWD_DKV) {
    hipLaunchKernelGGL((attn_bwd_dkv_mfma_f32<DH, CAUSAL, DROP>), grid, dim3(NT), 0, s, qkv, dout, lse, delta, lengths,
                       drop, T, H, dh, scale, dqkv);
    return hipGetLastError();
  }
  return hipSuccess;
}

template <int DH>
hipError_t fwd_pick(int causal, const float *qkv, const int32_t *lengths, const DropSpec &drop, int B, int T, int H,
                    int dh, float scale, float *o, float *lse, hipStream_t s) {
  if (causal)
    return drop.thr ? fwd_t<DH, true, true>(qkv, lengths, drop, B, T, H, dh, scale, o, lse, s)
                    : fwd_t<DH, true, false>(qkv, lengths, drop, B, T, H, dh, scale, o, lse, s);
  return drop.thr ? fwd_t<DH, false, true>(qkv, lengths, drop, B, T, H, dh, scale, o, lse, s)
                  : fwd_t<DH, false, false>(qkv, lengths, drop, B, T, H, dh, scale, o, lse, s);
}

template <int DH>
hipError_t bwd_pick(int causal, const float *qkv, const float *o, const float *dout, const float *lse,
                    const int32_t *lengths, const DropSpec &drop, int B, int T, int H, int dh, float scale,
                    float *dqkv, float *delta, hipStream_t s, int parts) {
  if (causal)
    return drop.thr ? bwd_t<DH, true, true>(qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts)
                    : bwd_t<DH, true, false>(qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts);
  return drop.thr ? bwd_t<DH, false, true>(qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts)
                  : bwd_t<DH, false, false>(qkv, o, dout, lse, lengths, drop, B, T, H, dh, scale, dqkv, delta, s, parts);
}

}  // namespace

bool attention_mfma_f32_supported(int dh) { return dh >= 16 && dh <= 128 && dh % 16 == 0; }

hipError_t launch_attention_fwd_mfma_f32(const void *qkv, const int32_t *lengths, int causal, const DropSpec &drop,
                                         int B, int T, int H, int dh, void *o, float *lse, hipStream_t s) {
  const float scale = 1.0f / sqrtf((float)dh);
  const float *x = static_cast<const float *>(qkv);
  float *y = static_cast<float *>(o);
  if (!attention_mfma_f32_supported(dh)) return hipErrorInvalidValue;
  switch ((dh + 31) / 32) {
    case 1: return fwd_pick<32>(causal, x, lengths, drop, B, T, H, dh, scale, y, lse, s);
    case 2: return fwd_pick<64>(causal, x, lengths, drop, B, T, H, dh, scale, y, lse, s);
    case 3: return fwd_pick<96>(causal, x, lengths, drop, B, T, H, dh, scale, y, lse, s);
    case 4: return fwd_pick<128>(causal, x, lengths, drop, B, T, H, dh, scale, y, lse, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_attention_bwd_mfma_f32(const void *qkv, const void *o, const void *dout, const float *lse,
                                         const int32_t *lengths, int causal, const DropSpec &drop, int B, int T, int H,
                                         int dh, void *dqkv, float *delta, hipStream_t s, int parts) {
  const float scale = 1.0f / sqrtf((float)dh);
  const float *x = static_cast<const float *>(qkv), *oo = static_cast<const float *>(o);
  const float *g = static_cast<const float *>(dout);
  float *dx = static_cast<float *>(dqkv);
  if (!attention_mfma_f32_supported(dh)) return hipErrorInvalidValue;
  switch ((dh + 31) / 32) {
    case 1: return bwd_pick<32>(causal, x, oo, g, lse, lengths, drop, B, T, H, dh, scale, dx, delta, s, parts);
    case 2: return bwd_pick<64>(causal, x, oo, g, lse, lengths, drop, B, T, H, dh, scale, dx, delta, s, parts);
    case 3: return bwd_pick<96>(causal, x, oo, g, lse, lengths, drop, B, T, H, dh, scale, dx, delta, s, parts);
    case 4: return bwd_pick<128>(causal, x, oo, g, lse, lengths, drop, B, T, H, dh, scale, dx, delta, s, parts);
  }
  return hipErrorInvalidValue;
}

}  // namespace fl
