// Attention backward in ONE kernel for bf16 heads of size 64 whose whole sequence fits a workgroup's
// LDS (T <= 224): dQ, dK and dV of a (sequence, head) pair from one pass over the scores.
//
// Same operator as the two-kernel path of attention_mfma.hip (the gradient function of the fused
// attention operator: Section 4.1.1 primitives fused, Section 5.2.1), with these differences:
//   * S and dP are computed once (5 contractions instead of 7) and Q, K, V, dO are read once;
//   * delta_i = sum_d dO_i O_i is computed in the kernel and never leaves LDS.
//
// One workgroup per (b, h); wavefront w owns keys 32w .. 32w+31 (K and V fragments in registers) and
// walks the query blocks of 32: S = Q K^T and dP = dO V^T with lane = key and registers = queries,
// then dV^T += dO^T P and dK^T += Q^T dS.  dQ needs dS of ALL keys for a query block, i.e. of all
// wavefronts: every wavefront parks its dS^T block in LDS ([key][query], bf16), and after a barrier
// wavefront w computes one 32x32 tile of dQ^T = K^T dS^T over all keys.  That exchange runs in two
// rounds of R = (wavefronts / 2) query blocks, so that a round has exactly one dQ tile per wavefront
// (R query blocks x two 32-wide halves of the head) and the parked dS needs R*32 columns only.
// Nothing is accumulated with atomics: results do not depend on timing.
//
// Q, dO, K and V travel to LDS with direct-to-LDS loads.  Every load of the kernel is issued at its
// start, in the order of need -- the wavefront's own K and V rows, then Q, dO, O and the log-sum-exp of
// query block 0, 1, ... -- and loads complete in order, so "at most n loads outstanding" tells a
// wavefront that a given block has landed: block q is computed while blocks q+1.. are still on their
// way.  (With every workgroup of a launch resident at once there is no other workgroup to hide a load
// phase behind.)  A tile is row-major [row][64] (128-byte rows) and serves both the 16-byte
// row-fragment reads and the transposing reads (ds_read_b64_tr_b16): 16-byte chunk c of row r sits at
// position c ^ swz(r), where swz permutes bits 1..3 of r so that 16 consecutive rows of one chunk, and
// 4 consecutive rows of 4 consecutive chunks, both touch every bank once.  Rows beyond T repeat row
// T-1 (finite values; their probabilities are exact zeros), so no lane reads out of bounds and no
// 0 * NaN can arise.  A wavefront's V rows are only needed until they are in registers: they land in
// the wavefront's own rows of the parked-dS area.  Results leave through LDS too, so that every
// global store writes whole rows.
#include "attention_tile.h"
#include "kernels.h"
#include "philox.h"

namespace fl {
namespace {
using namespace attn64;

constexpr int MAX_T = 224;              // 3 tiles + parked dS + statistics = 159,488 bytes of LDS

// Row pitch (bytes) of the parked dS^T blocks: R*32 queries of 2 bytes, 64 mod 128 so that the
// transposing reads touch every bank once, and at least 128 so that a wavefront's 32 rows also hold
// its V rows (4 KiB) until they are in registers.
__host__ __device__ constexpr int parked_pitch(int R) { return R <= 3 ? 192 : 320; }

// NW wavefronts (2, 4, 6 or 8) for sequences of up to NW*32 rows; the sequence has NW-1 or NW blocks of 32.
template <int NW, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(NW * 64, 2) void attn_bwd_fused64(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ o,
                                                              const bf16_t *__restrict__ dout, const float *__restrict__ lse,
                                                              const int32_t *__restrict__ lengths, DropSpec drop, int Tn,
                                                              int H, float scale, bf16_t *__restrict__ dqkv) {
  constexpr int R = NW / 2, PITCH = parked_pitch(R);   // query blocks per round
  constexpr int PER = (8 + NW - 1) / NW;   // a block of Q and dO is 8 wave-level loads: this many per wavefront
  constexpr int PO = NW == 2 ? 2 : 1;      // (row, chunk) pairs of a block's delta step per thread (256 per block)
  constexpr int LB = PER + 2 * PO;         // loads a wavefront issues per query block
  static_assert(8 + NW * LB < 64, "every load of a wavefront is in flight at once");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int nqb = (Tn + 31) >> 5, rows = nqb * 32;   // blocks of 32 queries / keys that exist: NW-1 or NW
  unsigned char *sQ = smem, *sDO = sQ + rows * ROWB, *sK = sDO + rows * ROWB, *sdS = sK + rows * ROWB;
  float *sL = reinterpret_cast<float *>(sdS + rows * PITCH), *sDl = sL + rows;
  const int lane = threadIdx.x & 63, h2 = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int hd = blockIdx.x, b = blockIdx.y;
  const int D = H * DH;
  const size_t ld = (size_t)3 * D;
  const int len = lengths ? min(max(lengths[b], 1), Tn) : Tn;  // a length outside 1..T is treated as the nearest valid one
  const bf16_t *base = qkv + (size_t)b * Tn * ld + hd * DH;
  const bf16_t *dobase = dout + (size_t)b * Tn * D + hd * DH;
  const bf16_t *obase = o + (size_t)b * Tn * D + hd * DH;
  const float *lsebase = lse + ((size_t)b * H + hd) * Tn;
  const bool full = nqb == NW;

  // ---- every load of the kernel is issued here, in the order in which the data is needed:
  // the wavefront's own K and V rows, then query block after query block (Q, dO; O and the
  // log-sum-exp for the delta step).  Loads complete in order, so "at most n still in flight"
  // means everything but the youngest n has arrived.
  const unsigned lds0 = lds_address(smem);
  unsigned char *myV = sdS + wave * 32 * PITCH;   // this wavefront's rows of the parked area: V until it is in registers
  if (wave < nqb) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = wave * 32 + i * 8 + (lane >> 3);
      const int c = (lane & 7) ^ swz(row);        // the chunk that belongs at this lane's position
      const bf16_t *src = base + (size_t)min(row, Tn - 1) * ld + D + c * 8;
      lds_dma16(src, lds0 + (unsigned)(2 * rows * ROWB + (wave * 4 + i) * 1024));
      lds_dma16(src + D, lds0 + (unsigned)(3 * rows * ROWB + wave * 32 * PITCH + i * 1024));
    }
  }
  f32x4_t oreg[NW][PO];
  float lreg[NW][PO];
#pragma unroll
  for (int qb = 0; qb < NW; ++qb) {
    if (qb < nqb) {
#pragma unroll
      for (int k = 0; k < PER; ++k) {
        const int inst = (wave * PER + k) & 7;   // 0..3: Q rows 8*inst.., 4..7: dO rows 8*(inst-4)..
        const int row = qb * 32 + (inst & 3) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ swz(row);
        const int rg = min(row, Tn - 1);
        const bf16_t *src = inst < 4 ? base + (size_t)rg * ld + c * 8 : dobase + (size_t)rg * D + c * 8;
        lds_dma16(src, lds0 + (unsigned)((inst < 4 ? 0 : rows * ROWB) + (qb * 4 + (inst & 3)) * 1024));
      }
#pragma unroll
      for (int k = 0; k < PO; ++k) {
        const int id = (threadIdx.x + k * 64 * NW) & 255, rg = min(qb * 32 + (id >> 3), Tn - 1);
        async_load16(oreg[qb][k], obase + (size_t)rg * D + (id & 7) * 8);
        async_load4(lreg[qb][k], lsebase + rg);
      }
    }
  }

  // delta and log-sum-exp of query block qb into LDS: eight lanes share a row (16 bytes of O from its
  // register, of dO from LDS); every (row, chunk) pair may be computed by more than one thread
  const unsigned char *pdelta[PO];   // this thread's 16 bytes of dO for the delta step, in block 0
  int drow[PO];
#pragma unroll
  for (int k = 0; k < PO; ++k) {
    const int id = (threadIdx.x + k * 64 * NW) & 255;
    drow[k] = id >> 3;
    pdelta[k] = sDO + (id >> 3) * ROWB + (((id & 7) ^ swz(id >> 3)) << 4);
  }
  auto delta_step = [&](auto qb_c) {
    constexpr int qb = decltype(qb_c)::value;
#pragma unroll
    for (int k = 0; k < PO; ++k) {
      arrived(oreg[qb][k]);
      arrived(lreg[qb][k]);
      const bf16x8_t dov = *reinterpret_cast<const bf16x8_t *>(pdelta[k] + qb * 32 * ROWB);
      const bf16x8_t ov = __builtin_bit_cast(bf16x8_t, oreg[qb][k]);
      float dl = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) dl += static_cast<float>(ov[e]) * static_cast<float>(dov[e]);
      dl += dpp_lane<0xB1>(dl);    // the eight lanes of a row: lane ^ 1, lane ^ 2, then the other quad
      dl += dpp_lane<0x4E>(dl);
      dl += dpp_lane<0x141>(dl);
      if ((threadIdx.x & 7) == 0) {
        const int row = qb * 32 + drow[k];
        sDl[row] = dl;
        sL[row] = row < Tn ? lreg[qb][k] * LOG2E : INFINITY;   // exp2(-inf) = 0 beyond T
      }
    }
  };

  const int key = wave * 32 + (lane & 31);
  const float c = scale * LOG2E;
  const bool wave_live = wave < nqb && wave * 32 < len;   // a wavefront whose keys are all masked has nothing to add
  const bool live = key < len;
  f32x16_t dk[2], dv[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dk[i][r] = 0.f, dv[i][r] = 0.f;

  // own K and V rows have arrived (all query-block loads may still be in flight)
  if (full) wait_loads_le<NW * LB>(); else wait_loads_le<(NW - 1) * LB>();
  // lane addresses of the fragment reads in block 0 of each tile
  const unsigned char *qrow[4], *dorow[4], *qtr[2][2], *dotr[2][2];
  bf16x8_t kf[4], vf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const unsigned off = row_frag_lane(kk, lane);
    qrow[kk] = sQ + off;
    dorow[kk] = sDO + off;
    kf[kk] = wave < nqb ? row_frag_at(sK + wave * 32 * ROWB + off) : zero_frag();
    vf[kk] = wave < nqb ? row_frag_at(myV + off) : zero_frag();
  }
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const unsigned off = tr_frag_lane(db * 32, half, lane);
      qtr[db][half] = sQ + off;
      dotr[db][half] = sDO + off;
    }
  unsigned char *const park = sdS + key * PITCH + h2 * 8;   // this lane's key row of the parked blocks
  const float *const pl = sL + h2 * 4, *const pdl = sDl + h2 * 4;
  if (full) wait_loads_le<(NW - 1) * LB>(); else wait_loads_le<(NW - 2) * LB>();
  wg_barrier();
  delta_step(std::integral_constant<int, 0>{});

  // One query block: waits for the NEXT block's data (its delta step runs here, one block ahead), then
  // S, dP, dS, the dV and dK updates, and the parked dS^T block.
  auto step = [&](auto qb_c) {
    constexpr int qb = decltype(qb_c)::value, j = qb % R;
    if (qb + 1 < nqb) {
      if (full) wait_loads_le<(NW - 2 - qb > 0 ? NW - 2 - qb : 0) * LB>();
      else wait_loads_le<(NW - 3 - qb > 0 ? NW - 3 - qb : 0) * LB>();
    }
    wg_barrier();   // the next block's Q and dO are in LDS; this block's delta is visible
    if (qb + 1 < nqb) delta_step(std::integral_constant<int, (qb + 1 < NW ? qb + 1 : qb)>{});
    // with the causal mask a key is seen by the queries at or after it only
    if (!wave_live || (CAUSAL && qb < wave)) return;
    f32x16_t s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f, dp[r] = 0.f;
    bf16x8_t qfr[4], dofr[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      qfr[kk] = row_frag_at(qrow[kk] + qb * 32 * ROWB);
      dofr[kk] = row_frag_at(dorow[kk] + qb * 32 * ROWB);
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfr[kk], kf[kk], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dofr[kk], vf[kk], dp, 0, 0, 0);
    }
    // the transposed fragments of the next two contractions are requested before the dS arithmetic
    // (not with dropout: the mask generator needs the registers)
    bf16x8_t tdo[2][2], tq[2][2];
    auto request_transposed = [&] {
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          tdo[db][st] = tr_frag_at(dotr[db][0] + (qb * 32 + 16 * st) * ROWB, dotr[db][1] + (qb * 32 + 16 * st) * ROWB);
          tq[db][st] = tr_frag_at(qtr[db][0] + (qb * 32 + 16 * st) * ROWB, qtr[db][1] + (qb * 32 + 16 * st) * ROWB);
        }
    };
    if constexpr (!DROP) request_transposed();
    // register 4g+e of a lane half h holds query qb*32 + 8g + 4h + e
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float4 l4 = *reinterpret_cast<const float4 *>(pl + qb * 32 + g * 8);
      float4 d4 = *reinterpret_cast<const float4 *>(pdl + qb * 32 + g * 8);
      // pinned: otherwise the reads sink behind the `live` test, one LDS round trip per branch
      asm volatile("" : "+v"(l4.x), "+v"(l4.y), "+v"(l4.z), "+v"(l4.w), "+v"(d4.x), "+v"(d4.y), "+v"(d4.z), "+v"(d4.w));
      const float lq[4] = {l4.x, l4.y, l4.z, l4.w}, dq[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = g * 4 + e, qi = qb * 32 + g * 8 + h2 * 4 + e;
        const float ex = exp2_raw(s[r] * c - lq[e]);
        const float p = (live && (!CAUSAL || qi >= key)) ? ex : 0.f;
        float keep = 1.f;
        if constexpr (DROP) keep = drop_keep1(drop, (uint32_t)key, (uint32_t)qi, (uint32_t)(b * H + hd));
        dp[r] = p * (dp[r] * keep - dq[e]);   // dS
        s[r] = p * keep;                      // dV sees the dropped-out probabilities
      }
    }
    const bf16x8_t pf[2] = {pack8(s, 0), pack8(s, 1)}, dsf[2] = {pack8(dp, 0), pack8(dp, 1)};
    if constexpr (DROP) request_transposed();
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tdo[db][st], pf[st], dv[db], 0, 0, 0);
        dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq[db][st], dsf[st], dk[db], 0, 0, 0);
      }
    // dS^T[key][query] for the dQ step: this lane's key row, four consecutive queries per store
    unsigned char *wr = park + j * 64;
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      const s16x8_t v = __builtin_bit_cast(s16x8_t, dsf[st]);
      *reinterpret_cast<s16x4_t *>(wr + (2 * st) * 16) = __builtin_shufflevector(v, v, 0, 1, 2, 3);
      *reinterpret_cast<s16x4_t *>(wr + (2 * st + 1) * 16) = __builtin_shufflevector(v, v, 4, 5, 6, 7);
    }
  };

  // dQ^T[d, q] = sum over keys K^T[d, key] dS^T[key, q]: one 32 x 32 tile per wavefront and round
  const int tj = wave % R, tdb = wave / R;
  const unsigned char *const ktr0 = sK + tr_frag_lane(tdb * 32, 0, lane), *const ktr1 = sK + tr_frag_lane(tdb * 32, 1, lane);
  const unsigned char *const str0 = sdS + tr_plain_lane(PITCH, tj * 32, lane);
  auto dq_tile = [&](int round, f32x16_t &acc) {
    const int qb = round * R + tj;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    if (qb >= nqb) return;
    int kend = (len + 31) & ~31;                 // keys of the wavefronts that parked a block
    if (CAUSAL) kend = min(kend, qb * 32 + 32);
#pragma unroll
    for (int k0 = 0; k0 < NW * 32; k0 += 64) {   // four k-steps of fragments in flight
      if (k0 >= kend) break;
      const bool two = k0 + 32 < kend;
      bf16x8_t fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (i < 2 || two) {
          fa[i] = tr_frag_at(ktr0 + (k0 + 16 * i) * ROWB, ktr1 + (k0 + 16 * i) * ROWB);
          fb[i] = tr_frag_at(str0 + (k0 + 16 * i) * PITCH, str0 + (k0 + 16 * i + 8) * PITCH);
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i < 2 || two) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[i], acc, 0, 0, 0);
    }
  };
  // Results leave through LDS so that a global store instruction writes whole rows (16 bytes per lane,
  // 128 or 64 contiguous bytes per row) instead of 8-byte pieces of 32 different rows.  A parked tile is
  // [32 rows][8 chunks of 16 bytes], chunk c of row r at position c ^ (r & 7).
  auto park_block = [&](unsigned char *tile, const f32x16_t &v, int db, float f) {   // v^T: lane = row, registers = columns db*32 ..
    unsigned char *rowp = tile + (lane & 31) * ROWB + h2 * 8;
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
      bf16x4_t t;
#pragma unroll
      for (int e = 0; e < 4; ++e) t[e] = static_cast<bf16_t>(v[qd * 4 + e] * f);
      *reinterpret_cast<bf16x4_t *>(rowp + (((db * 4 + qd) ^ (lane & 7)) << 4)) = t;
    }
  };

  unrolled(std::make_integer_sequence<int, R>{}, [&](auto i) { step(i); });
  wg_barrier();
  f32x16_t acc0, acc1;
  dq_tile(0, acc0);
  wg_barrier();       // the next round overwrites the parked blocks
  unrolled(std::make_integer_sequence<int, R>{}, [&](auto i) {
    constexpr int qb = R + decltype(i)::value;
    if (qb < nqb) step(std::integral_constant<int, qb>{});
  });
  wg_barrier();
  dq_tile(1, acc1);
  wg_barrier();       // nobody reads the tiles any more: they become the staging area of the results
  // dQ: a wavefront's two tiles (32 queries x 32 columns each) through the K tile's rows of their query blocks
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    const int qb = round * R + tj;
    if (qb >= nqb) continue;
    unsigned char *tile = sK + qb * 32 * ROWB;
    park_block(tile, round == 0 ? acc0 : acc1, tdb, scale);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int r = i * 16 + (lane >> 2), lc = tdb * 4 + (lane & 3), q = qb * 32 + r;
      const uint4 v = *reinterpret_cast<const uint4 *>(tile + r * ROWB + ((lc ^ (r & 7)) << 4));
      if (q < Tn) *reinterpret_cast<uint4 *>(dqkv + ((size_t)b * Tn + q) * ld + hd * DH + lc * 8) = v;
    }
  }
  // dK and dV: the wavefront's 32 key rows through its own rows of the Q and dO tiles
  if (wave < nqb) {
    unsigned char *tk = sQ + wave * 32 * ROWB, *tv = sDO + wave * 32 * ROWB;
#pragma unroll
    for (int db = 0; db < 2; ++db) {
      park_block(tk, dk[db], db, scale);
      park_block(tv, dv[db], db, 1.f);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = i * 8 + (lane >> 3), lc = (lane & 7) ^ (r & 7), krow = wave * 32 + r;
      const uint4 vk = *reinterpret_cast<const uint4 *>(tk + r * ROWB + ((lane & 7) << 4));
      const uint4 vv = *reinterpret_cast<const uint4 *>(tv + r * ROWB + ((lane & 7) << 4));
      if (krow < Tn) {
        bf16_t *g = dqkv + ((size_t)b * Tn + krow) * ld + D + hd * DH + lc * 8;
        *reinterpret_cast<uint4 *>(g) = vk;
        *reinterpret_cast<uint4 *>(g + D) = vv;
      }
    }
  }
}

template <int NW, bool CAUSAL, bool DROP>
hipError_t launch_nw(const void *qkv, const void *o, const void *dout, const float *lse, const int32_t *lengths,
                     const DropSpec &drop, int B, int T, int H, void *dqkv, hipStream_t s) {
  const int rows = (T + 31) / 32 * 32;
  const size_t lds = (size_t)3 * rows * ROWB + (size_t)rows * parked_pitch(NW / 2) + (size_t)2 * rows * sizeof(float);
  static bool raised = false;   // allow more than the default 64 KiB of dynamic LDS, once
  if (!raised) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(attn_bwd_fused64<NW, CAUSAL, DROP>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    raised = true;
  }
  hipLaunchKernelGGL((attn_bwd_fused64<NW, CAUSAL, DROP>), dim3(H, B), dim3(64 * NW), lds, s,
                     static_cast<const bf16_t *>(qkv), static_cast<const bf16_t *>(o), static_cast<const bf16_t *>(dout),
                     lse, lengths, drop, T, H, 1.0f / sqrtf((float)DH), static_cast<bf16_t *>(dqkv));
  return hipGetLastError();
}

template <bool CAUSAL, bool DROP>
hipError_t launch_t(const void *qkv, const void *o, const void *dout, const float *lse, const int32_t *lengths,
                    const DropSpec &drop, int B, int T, int H, void *dqkv, hipStream_t s) {
  switch ((T + 63) / 64) {
    case 1: return launch_nw<2, CAUSAL, DROP>(qkv, o, dout, lse, lengths, drop, B, T, H, dqkv, s);
    case 2: return launch_nw<4, CAUSAL, DROP>(qkv, o, dout, lse, lengths, drop, B, T, H, dqkv, s);
    case 3: return launch_nw<6, CAUSAL, DROP>(qkv, o, dout, lse, lengths, drop, B, T, H, dqkv, s);
    case 4: return launch_nw<8, CAUSAL, DROP>(qkv, o, dout, lse, lengths, drop, B, T, H, dqkv, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

bool attention_bwd_fused_applies(int T, int dh) { return dh == DH && T >= 1 && T <= MAX_T && !forced_unfused_attention_bwd(); }

hipError_t launch_attention_bwd_fused(const void *qkv, const void *o, const void *dout, const float *lse,
                                      const int32_t *lengths, int causal, const DropSpec &drop, int B, int T, int H,
                                      int dh, void *dqkv, hipStream_t s) {
  if (!attention_bwd_fused_applies(T, dh) || B > 65535) return hipErrorInvalidValue;
  if (causal)
    return drop.thr ? launch_t<true, true>(qkv, o, dout, lse, lengths, drop, B, T, H, dqkv, s)
                    : launch_t<true, false>(qkv, o, dout, lse, lengths, drop, B, T, H, dqkv, s);
  return drop.thr ? launch_t<false, true>(qkv, o, dout, lse, lengths, drop, B, T, H, dqkv, s)
                  : launch_t<false, false>(qkv, o, dout, lse, lengths, drop, B, T, H, dqkv, s);
}

}  // namespace fl
