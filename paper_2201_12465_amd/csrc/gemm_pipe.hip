// Pipelined bf16 MFMA GEMM for gfx950 (same contraction and epilogue as gemm.hip;
// this is the kernel the layer's large GEMMs run on).
//
//   C[M,N] = sum_k A(m,k) B(n,k),  k-range a multiple of 64.
//
// * Operand tiles travel HBM/L2 -> LDS with the direct-to-LDS load
//   (global_load_lds_dwordx4): no VGPRs and no LDS-write instructions are spent on
//   staging, so NS stages (k-tiles) can be in flight; one workgroup barrier per k-tile.
//   A wave-level load writes 64 consecutive 16-byte chunks of LDS; WHICH global chunk a
//   lane fetches is free, and that is where the bank-conflict swizzle is applied:
//     k-contiguous tile  [rows][64 k]   : chunk c of row r sits at position c ^ ((r>>1)&7)
//     k-major tile       [64 k][rows]   : chunk c of k-row k sits at position c ^ ((k&3)<<2)
//   Both make the MFMA fragment reads (16-byte row reads, and the transposing
//   ds_read_b64_tr_b16 for k-major tiles) touch every bank once per 32 lanes.
// * Rows past the end of an operand are clamped to the last valid row (their products land in
//   output rows/columns that are never stored), so no lane ever reads out of bounds.
// * 256 threads = 4 wavefronts in a 2x2 grid over a BM x BN tile (other grids: see the instances in
//   launch_layout); each wavefront owns
//   (BM/2) x (BN/2) = TM x TN MFMA tiles of 32x32 (v_mfma_f32_32x32x16_bf16), issued as
//   D = B_frag x A_frag so that a lane ends with four consecutive n of one m.
#include "devutil.h"
#include "gemm_dev.h"
#include "kernels.h"
#include "lds_dma.h"

namespace fl {
namespace {

constexpr int KT = 64;

typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *glb_void_ptr;
typedef __attribute__((address_space(3))) s16x4_t *lds_s16x4_ptr;

template <int N> __device__ __forceinline__ void wait_vmcnt_le() { FL_WAIT_VMCNT(N); }

// One operand's staging plan for this wave: element offsets (from the operand base) of the chunks
// its lanes fetch, for each of its NOPS wave-level loads per k-tile.
template <bool KC, int R, int NW> struct Stager {
  static constexpr int NOPS = R / (8 * NW);  // R*128 bytes per stage / 1 KiB per load / NW waves
  int off[NOPS];
  int kstep;  // element offset from one k-tile to the next
  __device__ __forceinline__ void init(int ld, int row0, int nrows, int kbeg, int lane, int wave) {
#pragma unroll
    for (int j = 0; j < NOPS; ++j) {
      const int P = (wave + NW * j) * 64 + lane;  // chunk position inside the stage
      if (KC) {
        const int r = P >> 3, c = (P & 7) ^ ((r >> 1) & 7);
        off[j] = min(row0 + r, nrows - 1) * ld + kbeg + c * 8;
      } else {
        constexpr int CPR = R / 8;
        const int k = P / CPR, c = (P % CPR) ^ ((k & 3) << 2);
        off[j] = (kbeg + k) * ld + min(row0 + c * 8, nrows - 8);
      }
    }
    kstep = KC ? KT : KT * ld;
  }
  // stage_lds: LDS byte address of the stage's first byte; wave: wave-uniform (a scalar)
  __device__ __forceinline__ void issue(const bf16_t *base, int kt, unsigned stage_lds, int wave) const {
#pragma unroll
    for (int j = 0; j < NOPS; ++j) {
      const bf16_t *src = base + (size_t)off[j] + (size_t)kt * kstep;
      lds_dma16(src, stage_lds + (unsigned)(wave + NW * j) * 1024u);
    }
  }
};

// Fragment (32 rows starting at tile row r0, k-step kk) out of a swizzled stage.
template <bool KC, int R>
__device__ __forceinline__ bf16x8_t frag(const unsigned char *stage, int r0, int kk, int lane) {
  if (KC) {
    const int r = r0 + (lane & 31);
    const int c = (kk * 2 + (lane >> 5)) ^ ((r >> 1) & 7);
    return *reinterpret_cast<const bf16x8_t *>(stage + r * 128 + c * 16);
  } else {
    const int g = lane >> 4, s = lane & 15;
    const int kb = kk * 16 + (g >> 1) * 8 + (s >> 2);
    const int rowpos = r0 + (g & 1) * 16 + 4 * (s & 3);
    const int c = (rowpos >> 3) ^ ((kb & 3) << 2);
    const unsigned char *a = stage + kb * (R * 2) + c * 16 + (rowpos & 7) * 2;
    s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)a);
    s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(a + 4 * R * 2));
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
  }
}

// WM x WN wavefronts share a BM x BN tile; each owns TM x TN MFMA tiles of 32x32.  KG > 1: KG such
// groups of wavefronts work on the same tile, group g taking the g-th part of every k-tile, and their
// accumulators are added through LDS at the end.  For outputs with few tiles (one workgroup per CU)
// this puts two wavefronts on every SIMD, so that one's LDS reads overlap the other's MFMAs.
template <bool AKC, bool BKC, int BM, int BN, int NS, int WM, int WN, bool DROP, int KG, int EPI = EPI_FULL>
__global__ __launch_bounds__(WM *WN *KG * 64) void gemm_bf16_pipe(GemmDev p) {
  constexpr int NW = WM * WN * KG;
  constexpr int KKS = KT / 16 / KG;  // 16-wide k-steps of a k-tile per group
  static_assert(KKS >= 1 && KKS * KG * 16 == KT, "k-groups must divide the k-tile");
  constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);
  constexpr int A_BYTES = BM * 128, STAGE = (BM + BN) * 128;
  constexpr int OPS = Stager<AKC, BM, NW>::NOPS + Stager<BKC, BN, NW>::NOPS;  // loads per wave per k-tile
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  int split, tile_m, tile_n;
  xcd_work_coords(blockIdx.x, p.tiles_m, p.tiles_n, p.splits, 1024 / BM, split, tile_m, tile_n);
  const int row0 = tile_m * BM, col0 = tile_n * BN;
  const int kbeg = split * p.k_per_split;
  if (p.partial) p.partial += (size_t)split * p.M * p.N;
  const int kend = min(p.K, kbeg + p.k_per_split);
  const int nk = (kend - kbeg) / KT;
  const bf16_t *A = static_cast<const bf16_t *>(p.A);
  const bf16_t *B = static_cast<const bf16_t *>(p.B);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // in a scalar register: LDS addresses below are scalars too
  const unsigned smem_lds = lds_address(smem);
  const int kg = wave / (WM * WN), wpos = wave % (WM * WN);  // k-group, position in the tile
  const int wm = wpos / WN, wn = wpos % WN;

  Stager<AKC, BM, NW> sa;
  Stager<BKC, BN, NW> sb;
  sa.init(p.lda, row0, p.M, kbeg, lane, wave);
  sb.init(p.ldb, col0, p.N, kbeg, lane, wave);

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // prologue: NS-1 k-tiles in flight
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) {
    if (s < nk) {
      sa.issue(A, s, smem_lds + s * STAGE, wave);
      sb.issue(B, s, smem_lds + s * STAGE + A_BYTES, wave);
    }
  }
  for (int kt = 0; kt < nk; ++kt) {
    // k-tile kt must have landed: allow the loads of the (up to NS-2) younger k-tiles to stay in flight
    const int younger = min(NS - 2, nk - 1 - kt);
    if (NS >= 4 && younger >= 2) wait_vmcnt_le<2 * OPS>();
    else if (NS >= 3 && younger == 1) wait_vmcnt_le<OPS>();
    else wait_vmcnt_le<0>();
    // every wave's part of k-tile kt is in LDS; everyone is done reading k-tile kt-1.  A bare
    // s_barrier: __syncthreads() would add a fence that waits for ALL loads, younger k-tiles included.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (kt + NS - 1 < nk) {
      const unsigned st = smem_lds + ((kt + NS - 1) % NS) * STAGE;
      sa.issue(A, kt + NS - 1, st, wave);
      sb.issue(B, kt + NS - 1, st + A_BYTES, wave);
    }
    const unsigned char *sA = smem + (kt % NS) * STAGE, *sB = sA + A_BYTES;
    // fragments of k-step kk+1 are requested before the MFMAs of k-step kk are issued.  Left to itself the
    // scheduler sinks those reads behind the MFMAs and into the registers the MFMAs have just read, so that
    // every k-step waits out a full LDS round trip; the scheduling barriers keep the two groups apart where
    // the wavefront tile is small enough for the second fragment set to cost no occupancy.
    constexpr bool PIN = TM * TN <= 4;
    bf16x8_t fa[2][TM], fb[2][TN];
    const int kk0 = kg * KKS;
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = frag<AKC, BM>(sA, wm * (BM / WM) + i * 32, kk0, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = frag<BKC, BN>(sB, wn * (BN / WN) + j * 32, kk0, lane);
#pragma unroll
    for (int kk = 0; kk < KKS; ++kk) {
      if (kk + 1 < KKS) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
          fa[(kk + 1) & 1][i] = frag<AKC, BM>(sA, wm * (BM / WM) + i * 32, kk0 + kk + 1, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          fb[(kk + 1) & 1][j] = frag<BKC, BN>(sB, wn * (BN / WN) + j * 32, kk0 + kk + 1, lane);
      }
      if constexpr (PIN) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk & 1][j], fa[kk & 1][i], acc[i][j], 0, 0, 0);
      if constexpr (PIN) __builtin_amdgcn_sched_barrier(0);
    }
  }

  // Epilogue through LDS (see gemm_staged_epilogue): the operand stages are reused.
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();  // every wave is done reading the operand stages
  asm volatile("" ::: "memory");
  if constexpr (KG > 1) {
    // groups 1.. park their accumulators in LDS ([group-1][position][register][lane]: lane-contiguous,
    // no bank conflicts), group 0 adds them up and goes on alone
    float *red = reinterpret_cast<float *>(smem);
    constexpr int PER_WAVE = TM * TN * 16 * 64;
    if (kg > 0) {
      float *dst = red + ((size_t)(kg - 1) * (WM * WN) + wpos) * PER_WAVE + lane;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) dst[((i * TN + j) * 16 + r) * 64] = acc[i][j][r];
    }
    __syncthreads();
#pragma unroll
    for (int g = 1; g < KG && kg == 0; ++g) {
      const float *src = red + ((size_t)(g - 1) * (WM * WN) + wpos) * PER_WAVE + lane;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] += src[((i * TN + j) * 16 + r) * 64];
    }
    __syncthreads();  // the epilogue's staging area overlaps what other wavefronts have just read
    if (kg > 0) return;  // no barrier follows: group 0 finishes alone
  }
  float *cw = reinterpret_cast<float *>(smem) + (size_t)wpos * 32 * (TN * 32 + 4);
  gemm_staged_epilogue<bf16_t, TM, TN, DROP, EPI>(p, acc, cw, row0 + wm * (BM / WM), col0 + wn * (BN / WN), lane);
}

template <bool AKC, bool BKC, int BM, int BN, int NS, int WM, int WN, bool DROP, int KG, int EPI = EPI_FULL>
hipError_t launch_cfg_d(GemmDev d, int splits, hipStream_t s) {
  constexpr size_t stage_lds = (size_t)NS * (BM + BN) * 128;
  constexpr size_t epi_lds = (size_t)WM * WN * 32 * (BN / WN + 4) * sizeof(float);
  constexpr size_t red_lds = (size_t)(KG - 1) * BM * BN * sizeof(float);
  constexpr size_t lds0 = stage_lds > epi_lds ? stage_lds : epi_lds;
  constexpr size_t lds = lds0 > red_lds ? lds0 : red_lds;
  static_assert(lds <= 160 * 1024, "stages do not fit in LDS");
  auto kern = gemm_bf16_pipe<AKC, BKC, BM, BN, NS, WM, WN, DROP, KG, EPI>;
  if (lds > 64 * 1024) {
    static bool raised = false;
    if (!raised) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      raised = true;
    }
  }
  d.tiles_m = (d.M + BM - 1) / BM;
  d.tiles_n = (d.N + BN - 1) / BN;
  d.splits = splits;
  dim3 grid(d.tiles_m * d.tiles_n * splits);
  hipLaunchKernelGGL(kern, grid, dim3(WM * WN * KG * 64), lds, s, d);
  return hipGetLastError();
}

// Dropout in the epilogue exists for the 128x128 / 2-stage variant (the forward GEMMs in training mode).
template <bool AKC, bool BKC, int BM, int BN, int NS, int WM = 2, int WN = 2, int KG = 1>
hipError_t launch_cfg(const GemmDev &d, int splits, hipStream_t s) {
  if (d.drop_where) {
    if constexpr (AKC && BKC && NS == 2 && BM == 128 && BN == 128)
      return launch_cfg_d<AKC, BKC, BM, BN, NS, WM, WN, true, KG>(d, splits, s);
    else
      return hipErrorInvalidValue;
  }
  // the instances the layer runs on carry only the epilogue steps of their launch (see gemm_epi_kind)
  constexpr bool specialised = (BM == 128 && BN == 128 && WM == 2 && WN == 2 && ((NS == 2 && KG == 1) || (NS == 3 && KG == 2))) ||
                               (BM == 256 && BN == 192) || (BN == 128 && (BM == 160 || BM == 96));
  if constexpr (specialised) {
    const int kind = gemm_epi_kind(d.partial != nullptr, d.act, d.dact, d.preact != nullptr);
    if (kind == EPI_PLAIN) return launch_cfg_d<AKC, BKC, BM, BN, NS, WM, WN, false, KG, EPI_PLAIN>(d, splits, s);
    if (kind == EPI_PARTIAL) return launch_cfg_d<AKC, BKC, BM, BN, NS, WM, WN, false, KG, EPI_PARTIAL>(d, splits, s);
    if (kind == EPI_LIGHT) return launch_cfg_d<AKC, BKC, BM, BN, NS, WM, WN, false, KG, EPI_LIGHT>(d, splits, s);
    if (kind == EPI_GELU_FWD) return launch_cfg_d<AKC, BKC, BM, BN, NS, WM, WN, false, KG, EPI_GELU_FWD>(d, splits, s);
    if (kind == EPI_GELU_BWD) return launch_cfg_d<AKC, BKC, BM, BN, NS, WM, WN, false, KG, EPI_GELU_BWD>(d, splits, s);
  }
  return launch_cfg_d<AKC, BKC, BM, BN, NS, WM, WN, false, KG>(d, splits, s);
}

template <bool AKC, bool BKC>
hipError_t launch_layout(const GemmDev &d, int splits, int variant, hipStream_t s) {
  switch (variant) {
    case 0: return launch_cfg<AKC, BKC, 128, 128, 2>(d, splits, s);
    case 1: return launch_cfg<AKC, BKC, 128, 128, 4>(d, splits, s);
    case 2: return launch_cfg<AKC, BKC, 256, 128, 3>(d, splits, s);
    case 3: return launch_cfg<AKC, BKC, 256, 128, 2>(d, splits, s);
    case 4: return launch_cfg<AKC, BKC, 256, 256, 2>(d, splits, s);
    case 5: return launch_cfg<AKC, BKC, 256, 256, 2, 2, 4>(d, splits, s);
    case 6: return launch_cfg<AKC, BKC, 256, 128, 3, 4, 2>(d, splits, s);
    case 8: return launch_cfg<AKC, BKC, 128, 128, 2, 2, 2, 2>(d, splits, s);
    case 9: return launch_cfg<AKC, BKC, 128, 128, 3, 2, 2, 2>(d, splits, s);
    case 10:  // 160 rows: the same restriction for a k-major A operand
      if constexpr (AKC) return launch_cfg<AKC, BKC, 160, 128, 2, 1, 4>(d, splits, s);
      else return hipErrorInvalidValue;
    case 11:  // 96 rows: likewise
      if constexpr (AKC) return launch_cfg<AKC, BKC, 96, 128, 2, 1, 4>(d, splits, s);
      else return hipErrorInvalidValue;
    case 7:  // 192 columns: the k-major swizzle needs a power-of-two row length, so k-contiguous operands only
      if constexpr (AKC && BKC) return launch_cfg<AKC, BKC, 256, 192, 2, 4, 2>(d, splits, s);
      else return hipErrorInvalidValue;
  }
  return hipErrorInvalidValue;
}

}  // namespace

bool gemm_pipe_eligible(const GemmArgs &a, int kps) {
  // whole k-tiles only; operands must hold at least one full 8-element chunk per clamped row
  return kps % KT == 0 && a.K % KT == 0 && a.M >= 8 && a.N >= 8 && (long)a.M * a.lda < (1l << 31) &&
         (long)a.N * a.ldb < (1l << 31) && (long)a.K * (a.a_kc ? 1 : a.lda) < (1l << 31) &&
         (long)a.K * (a.b_kc ? 1 : a.ldb) < (1l << 31);
}

void gemm_pipe_tile(int variant, int *bm, int *bn) {
  static const int t[12][2] = {{128, 128}, {128, 128}, {256, 128}, {256, 128}, {256, 256}, {256, 256}, {256, 128}, {256, 192}, {128, 128}, {128, 128}, {160, 128}, {96, 128}};
  *bm = t[variant][0];
  *bn = t[variant][1];
}

int gemm_pipe_pick_variant(bool a_kc, bool b_kc, int M, int N, int K, bool alone) {
  const int forced = forced_gemm_pipe_variant();
  if (forced != -1) return (forced == 7 && !(a_kc && b_kc)) || ((forced == 10 || forced == 11) && !a_kc) ? -2 : forced;
  (void)K;
  // Measured inside the layer (whole training steps, same box, libraries alternating), since a loop over one
  // launch flatters whatever profits most from warm caches.
  // dy^T x (both operands k-major, split over the tokens) and dy W (one k-major operand, used where forward
  // left no transposed weights behind): 128x128 tiles, 2 stages, two workgroups per CU.  2-3 % of a step
  // against the register-staged kernel in gemm.hip on the BERT-base, speech and ViT shapes (0.404 -> 0.394,
  // 0.799 -> 0.779, 12.03 -> 11.68 ms for dy^T x; 12.07 -> 11.75 ms for dy W); the variants with three
  // stages or two wavefront groups per tile hold more LDS and slow the kernels they run beside.
  if (!a_kc && !b_kc) return 0;
  // More 128x128 tiles than the chip holds at two workgroups per CU, but not with 160x128 tiles: one round
  // instead of one and a bit (12608 x 768 outputs: 594 tiles against 474; dy W at k = 3072 / 2304 / 768 alone:
  // 83 -> 66, 64 -> 51, 28 -> 22 us).
  const long slots = 512, tiles128 = (long)((M + 127) / 128) * ((N + 127) / 128);
  const bool one_round_160 = tiles128 > slots && (long)((M + 159) / 160) * ((N + 127) / 128) <= slots;
  // One round of 128x128 tiles that leaves a quarter of the places empty, where 96x128 tiles fill them (8000 x 768
  // outputs: 378 tiles against 504; on their own 57 -> 48, 42 -> 38, 20 -> 17.5 us at k = 3072 / 2304 / 768).  Only with
  // more tiles than CUs (below that the two-k-group variant is ahead), and only for a launch that has the chip to
  // itself: in the backward pass the places that 128x128 tiles leave empty take the weight-gradient workgroups of
  // the other lane, and whole steps of the speech shape are slower with the rule there (0.725 -> 0.738 ms).
  const bool one_round_96 = alone && tiles128 > 256 && 5 * tiles128 <= 4 * slots && (long)((M + 95) / 96) * ((N + 127) / 128) <= slots;
  if (a_kc && !b_kc) return one_round_160 ? 10 : one_round_96 ? 11 : 0;
  if (!(a_kc && b_kc)) return -2;
  // the same for k-contiguous operands, ahead of one 75-78 %-full round of 256x192 tiles (ViT stack, libraries
  // alternating: 10.64 ms per step -> 10.58 with the rule for dy W alone -> 10.46 with both; BERT-base shape,
  // where it takes the fused projection: 0.3703 -> 0.3682 ms)
  if (one_round_160) return 10;
  // Both operands k-contiguous:
  // 256x192 tiles on 8 wavefronts halve the L1 and LDS traffic per flop and win when they fill the
  // chip in whole rounds (one workgroup per CU); otherwise 128x128 / 2 stages, two workgroups per CU.
  if (N % 192 == 0) {
    const long tiles = (long)((M + 255) / 256) * (N / 192);
    const long rounds = (tiles + 255) / 256;
    // one round of tiles: worth it from 160 tiles up; several rounds: only if the last one is nearly full
    // (12608 x 3072, 800 tiles = 3.1 rounds: 88 us against 81 with 128x128 tiles; 8000 x 3072, 512 tiles: 47.5
    // against 51)
    if (tiles >= 160 && 100 * tiles >= (rounds == 1 ? 74 : 90) * rounds * 256) return 7;
  }
  // at most one 128x128 tile per CU: three stages and two k-groups of wavefronts per tile (eight wavefronts on
  // the CU instead of four) keep more loads in flight.  Long k-loops (FFN2: 35 -> 32 us), and short ones as
  // well: the 4096 x 768 x 768 problems of the attention projection, whole steps on the BERT-base shape
  // 0.3835 -> 0.3756 ms (four stages, or one k-group with three stages: 0.379 / 0.380).  With more tiles than
  // CUs the two-workgroups-per-CU variant is ahead (speech shape, 378 tiles: 0.765 against 0.835 ms).
  if ((long)((M + 127) / 128) * ((N + 127) / 128) <= 256) return 9;
  return one_round_96 ? 11 : 0;
}

hipError_t launch_gemm_bf16_pipe(const GemmArgs &a, const void *dev, int splits, int variant, hipStream_t s) {
  const GemmDev &d = *static_cast<const GemmDev *>(dev);
  if (a.a_kc && a.b_kc) return launch_layout<true, true>(d, splits, variant, s);
  if (a.a_kc && !a.b_kc) return launch_layout<true, false>(d, splits, variant, s);
  if (!a.a_kc && !a.b_kc) return launch_layout<false, false>(d, splits, variant, s);
  return launch_layout<false, true>(d, splits, variant, s);
}

}  // namespace fl
