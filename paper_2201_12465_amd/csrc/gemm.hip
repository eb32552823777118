// MFMA GEMM for gfx950: C[M,N] = sum_k A(m,k) B(n,k), fp32 accumulation.
//
// These are the layer's dense contractions -- the paper's matmul primitive
// (Section 4.1.1, TensorBackend listing) that its reference backend hands to a
// vendor library; here it is written out for CDNA4.  One kernel template serves
// the three operand layouts of a linear layer and its two gradients:
//   y  = x W^T   A = x  [M,K] k-contiguous,  B = W [N,K] k-contiguous
//   dx = dy W    A = dy [M,K] k-contiguous,  B = W [K,N] k-major (n contiguous)
//   dW = dy^T x  A = dy [K,M] k-major,       B = x [K,N] k-major   (k = tokens)
//
// Work decomposition: a workgroup of 256 threads (4 wavefronts, 2x2) owns a
// 128x128 output tile; each wavefront owns 64x64 = 2x2 MFMA tiles of 32x32.
// (A 64x128 variant -- wavefront tile 32x64 -- doubles the workgroup count for
// outputs too small to give every CU more than one 128x128 tile.)
// Per k-tile (64 bf16 / 32 fp32 values) both operand tiles are staged in LDS:
//   k-contiguous operand: LDS [128 rows][k], rows padded by 16 bytes; a bf16 MFMA
//     fragment is one 16-byte LDS read per lane;
//   k-major operand: LDS [k][128 rows] copied as it lies in memory; bf16 fragments
//     are gathered with the transposing LDS read (ds_read_b64_tr_b16), which hands
//     each lane four consecutive-k values of one row; rows padded so that the four
//     k-rows a 16-lane group touches fall in different banks.
// fp32 uses v_mfma_f32_32x32x2_f32 with one LDS word per lane per operand.
// The MFMA is issued as D = B_frag x A_frag, so each lane ends up with four
// consecutive n for one m: the epilogue works on 4-element vectors along the
// contiguous output dimension.
//
// Workgroup ids are remapped so that each of the 8 XCDs (which receive ids
// round-robin) works on a contiguous range of tiles and its L2 sees few panels.
#include "devutil.h"
#include "gemm_dev.h"
#include "kernels.h"

namespace fl {
namespace {

constexpr int BM = 128, BN = 128, NTHREADS = 256;
// k-major LDS row stride in elements for a tile of ROWS rows (both types): ROWS + 32 keeps the
// transposing reads and the fp32 word reads free of bank conflicts
constexpr int ldr(int rows) { return rows + 32; }
constexpr int OPERAND_LDS_BYTES = 20480;

template <typename T> struct Tile;
template <> struct Tile<float> { static constexpr int KT = 32; static constexpr int LDK = 36; };
template <> struct Tile<bf16_t> { static constexpr int KT = 64; static constexpr int LDK = 72; };

__device__ __forceinline__ uint4 ld16(const void *p, bool ok) {
  return ok ? *reinterpret_cast<const uint4 *>(p) : make_uint4(0, 0, 0, 0);
}

// Global -> registers for one operand tile of ROWS rows: ROWS/32 chunks of 16 bytes per thread.
template <typename T, bool KC, int ROWS>
__device__ __forceinline__ void load_tile(const T *base, int ld, int row0, int nrows, int k0, int kend,
                                          uint4 (&r)[ROWS / 32]) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int KT = Tile<T>::KT;
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < ROWS / 32; ++i) {
    int c = tid + NTHREADS * i;
    if (KC) {
      constexpr int CPR = KT / VEC;  // chunks per row (8)
      int row = row0 + c / CPR, k = k0 + (c % CPR) * VEC;
      r[i] = ld16(base + (size_t)row * ld + k, row < nrows && k < kend);
    } else {
      constexpr int CPR = ROWS / VEC;  // chunks per k-row
      int k = k0 + c / CPR, row = row0 + (c % CPR) * VEC;
      r[i] = ld16(base + (size_t)k * ld + row, k < kend && row < nrows);
    }
  }
}

template <typename T, bool KC, int ROWS>
__device__ __forceinline__ void store_tile(T *lds, const uint4 (&r)[ROWS / 32]) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int KT = Tile<T>::KT;
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < ROWS / 32; ++i) {
    int c = tid + NTHREADS * i;
    if (KC) {
      constexpr int CPR = KT / VEC;
      *reinterpret_cast<uint4 *>(lds + (c / CPR) * Tile<T>::LDK + (c % CPR) * VEC) = r[i];
    } else {
      constexpr int CPR = ROWS / VEC;
      *reinterpret_cast<uint4 *>(lds + (c / CPR) * ldr(ROWS) + (c % CPR) * VEC) = r[i];
    }
  }
}

// bf16 fragment of the 32 rows starting at r0 for k-step kk (16 values of k).
template <bool KC, int LDR>
__device__ __forceinline__ bf16x8_t frag_bf16(const bf16_t *lds, int r0, int kk, int lane) {
  if (KC) {
    return *reinterpret_cast<const bf16x8_t *>(lds + (r0 + (lane & 31)) * Tile<bf16_t>::LDK + kk * 16 + (lane >> 5) * 8);
  } else {
    // 16-lane group g serves rows r0 + (g&1)*16 .. +15 and k-half g>>1; within the group lane s
    // points at k-row s/4 and the 4-row chunk s%4; the read returns, for lane s, row s of the
    // group and the four consecutive k of the addressed k-rows.
    int g = lane >> 4, s = lane & 15;
    int row = r0 + (g & 1) * 16 + 4 * (s & 3);
    int kb = kk * 16 + (g >> 1) * 8 + (s >> 2);
    typedef __attribute__((address_space(3))) s16x4_t *lds_ptr;
    s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds + kb * LDR + row));
    s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds + (kb + 4) * LDR + row));
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
  }
}

template <bool KC, int LDR>
__device__ __forceinline__ float frag_f32(const float *lds, int r0, int kk, int lane) {
  if (KC) return lds[(r0 + (lane & 31)) * Tile<float>::LDK + kk * 2 + (lane >> 5)];
  return lds[(kk * 2 + (lane >> 5)) * LDR + r0 + (lane & 31)];
}

template <typename T, bool AKC, bool BKC, int TMW, bool DROP>
__global__ __launch_bounds__(NTHREADS) void gemm_kernel(GemmDev p) {
  constexpr int KT = Tile<T>::KT;
  constexpr int BMT = 64 * TMW;  // tile height: TMW MFMA tiles per wavefront in m
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * OPERAND_LDS_BYTES];
  T *ldsA = reinterpret_cast<T *>(smem);
  T *ldsB = reinterpret_cast<T *>(smem + OPERAND_LDS_BYTES);

  int split, tile_m, tile_n;
  xcd_work_coords(blockIdx.x, p.tiles_m, p.tiles_n, p.splits, 1024 / BMT, split, tile_m, tile_n);
  const int row0 = tile_m * BMT, col0 = tile_n * BN;

  const int kbeg = split * p.k_per_split;
  if (p.partial) p.partial += (size_t)split * p.M * p.N;
  const int kend = min(p.K, kbeg + p.k_per_split);
  const T *A = static_cast<const T *>(p.A);
  const T *B = static_cast<const T *>(p.B);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  f32x16_t acc[TMW][2];
#pragma unroll
  for (int i = 0; i < TMW; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[BMT / 32], rb[4];
  if (kbeg < kend) {
    load_tile<T, AKC, BMT>(A, p.lda, row0, p.M, kbeg, kend, ra);
    load_tile<T, BKC, BN>(B, p.ldb, col0, p.N, kbeg, kend, rb);
  }
  for (int k0 = kbeg; k0 < kend; k0 += KT) {
    store_tile<T, AKC, BMT>(ldsA, ra);
    store_tile<T, BKC, BN>(ldsB, rb);
    __syncthreads();
    if (k0 + KT < kend) {  // next tile's loads stay in flight during the MFMAs
      load_tile<T, AKC, BMT>(A, p.lda, row0, p.M, k0 + KT, kend, ra);
      load_tile<T, BKC, BN>(B, p.ldb, col0, p.N, k0 + KT, kend, rb);
    }
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int kk = 0; kk < KT / 16; ++kk) {
        bf16x8_t fa[TMW], fb[2];
#pragma unroll
        for (int i = 0; i < TMW; ++i)
          fa[i] = frag_bf16<AKC, ldr(BMT)>(reinterpret_cast<const bf16_t *>(ldsA), wm * 32 * TMW + i * 32, kk, lane);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          fb[j] = frag_bf16<BKC, ldr(BN)>(reinterpret_cast<const bf16_t *>(ldsB), wn * 64 + j * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < TMW; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < KT / 2; ++kk) {
        float fa[TMW], fb[2];
#pragma unroll
        for (int i = 0; i < TMW; ++i)
          fa[i] = frag_f32<AKC, ldr(BMT)>(reinterpret_cast<const float *>(ldsA), wm * 32 * TMW + i * 32, kk, lane);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          fb[j] = frag_f32<BKC, ldr(BN)>(reinterpret_cast<const float *>(ldsB), wn * 64 + j * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < TMW; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fb[j], fa[i], acc[i][j], 0, 0, 0);
      }
    }
    __syncthreads();
  }

  // Epilogue through LDS (see gemm_staged_epilogue); the last __syncthreads() of the loop has
  // made the operand tiles free, and 4 waves x 32 x 68 floats fit in them.
  static_assert(4 * 32 * 68 * sizeof(float) <= 2 * OPERAND_LDS_BYTES, "epilogue staging does not fit");
  float *cw = reinterpret_cast<float *>(smem) + (size_t)wave * 32 * 68;
  gemm_staged_epilogue<T, TMW, 2, DROP>(p, acc, cw, row0 + wm * 32 * TMW, col0 + wn * 64, lane);
}

template <typename T, int TMW, bool DROP>
hipError_t launch_ttd(const GemmArgs &a, const GemmDev &d, dim3 grid, hipStream_t s) {
  if (a.a_kc && a.b_kc)
    hipLaunchKernelGGL((gemm_kernel<T, true, true, TMW, DROP>), grid, dim3(NTHREADS), 0, s, d);
  else if (a.a_kc && !a.b_kc)
    hipLaunchKernelGGL((gemm_kernel<T, true, false, TMW, DROP>), grid, dim3(NTHREADS), 0, s, d);
  else if (!a.a_kc && !a.b_kc)
    hipLaunchKernelGGL((gemm_kernel<T, false, false, TMW, DROP>), grid, dim3(NTHREADS), 0, s, d);
  else
    hipLaunchKernelGGL((gemm_kernel<T, false, true, TMW, DROP>), grid, dim3(NTHREADS), 0, s, d);
  return hipGetLastError();
}
// the instances with the dropout steps in their epilogue are separate kernels
template <typename T, int TMW>
hipError_t launch_tt(const GemmArgs &a, const GemmDev &d, dim3 grid, hipStream_t s) {
  return d.drop_where ? launch_ttd<T, TMW, true>(a, d, grid, s) : launch_ttd<T, TMW, false>(a, d, grid, s);
}

// tmw = 2: 128x128 tiles; tmw = 1: 64x128 tiles
template <typename T>
hipError_t launch_t(const GemmArgs &a, GemmDev d, int tmw, int splits, hipStream_t s) {
  d.tiles_m = (a.M + 64 * tmw - 1) / (64 * tmw);
  d.splits = splits;
  dim3 grid(d.tiles_m * d.tiles_n * splits);
  return tmw == 1 ? launch_tt<T, 1>(a, d, grid, s) : launch_tt<T, 2>(a, d, grid, s);
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

int gemm_pick_splits(int dt, int M, int N, int K) {
  const int KT = dt == DT_F32 ? Tile<float>::KT : Tile<bf16_t>::KT;
  long tiles = (long)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  int want, maxs = (K + 4 * KT - 1) / (4 * KT);  // at least four k-tiles per range
  if (dt == DT_BF16) {
    // measured on the dW shapes of the layer (k = 4096 tokens; 36, 108 and 144 tiles): about 430
    // workgroups are the best trade between filling the chip and the fp32 partial sums' traffic
    want = (int)((432 + tiles / 2) / tiles);
    if (want > 6) want = 6;
  } else if (gemm_f32_small_applies(M, N)) {
    // 32 x 32 tiles with k split inside the workgroup: a wavefront's chain is K/8 MFMAs of 64 clocks
    // (3.4 us at K = 1024), less than a second-stage launch costs, until K gets long
    want = (K + 4095) / 4096;
  } else {
    want = (int)((512 + tiles - 1) / tiles);
  }
  int s = want < maxs ? want : maxs;
  if (s > 32) s = 32;
  if (s < 1) s = 1;
  // ranges are whole k-tiles; drop ranges that rounding would leave empty
  int kps = ((K + s - 1) / s + KT - 1) / KT * KT;
  return (K + kps - 1) / kps;
}

hipError_t launch_gemm(int dt, const GemmArgs &a, hipStream_t stream) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0 || !a.A || !a.B) return hipErrorInvalidValue;
  const int KT = dt == DT_F32 ? Tile<float>::KT : Tile<bf16_t>::KT;
  const int splits = a.splits < 1 ? 1 : a.splits;
  // vector accesses: every contiguous dimension and leading dimension in units of 8 elements
  if (a.N % 8 || a.lda % 8 || a.ldb % 8) return hipErrorInvalidValue;
  if ((a.a_kc ? a.K : a.M) % 8 || (a.b_kc ? a.K : a.N) % 8) return hipErrorInvalidValue;
  if (!aligned16(a.A) || !aligned16(a.B)) return hipErrorInvalidValue;
  if (splits > 1) {
    if (!a.partial || a.bias || a.residual || a.preact || a.act || a.dact || a.drop_where || !aligned16(a.partial))
      return hipErrorInvalidValue;
  } else {
    if (!a.C || a.ldc % 8 || !aligned16(a.C) || !aligned16(a.bias) || !aligned16(a.residual) ||
        !aligned16(a.aux) || !aligned16(a.preact) || (a.dact && !a.aux))
      return hipErrorInvalidValue;
  }
  GemmDev d;
  d.A = a.A; d.B = a.B; d.C = a.C;
  d.M = a.M; d.N = a.N; d.K = a.K; d.lda = a.lda; d.ldb = a.ldb; d.ldc = a.ldc;
  d.bias = a.bias; d.residual = a.residual; d.aux = a.aux; d.preact = a.preact;
  d.act = a.act; d.dact = a.dact;
  d.drop_where = a.drop.thr ? a.drop_where : 0;
  d.drop = a.drop;
  d.partial = splits > 1 ? a.partial : nullptr;
  int kps = (a.K + splits - 1) / splits;
  kps = (kps + KT - 1) / KT * KT;
  d.k_per_split = kps;
  d.tiles_m = (a.M + BM - 1) / BM;
  d.tiles_n = (a.N + BN - 1) / BN;
  // every k-range must be non-empty, or its partial slab would stay unwritten
  if ((long)(splits - 1) * kps >= a.K) return hipErrorInvalidValue;
  if (dt == DT_BF16 && gemm_pipe_eligible(a, kps)) {
    int variant = gemm_pipe_pick_variant(a.a_kc, a.b_kc, a.M, a.N, a.K, a.alone);
    if (variant > 0 && d.drop_where) variant = 0;  // the dropout steps exist in the 128x128 / 2-stage instance only,
    if (d.drop_where && !(a.a_kc && a.b_kc)) variant = -2;  // and there for k-contiguous operands only
    if (variant >= 0) return launch_gemm_bf16_pipe(a, &d, splits, variant, stream);
  }
  const int force_tmw = forced_gemm_tile_height();
  if (dt == DT_F32 && !force_tmw && gemm_f32_small_applies(a.M, a.N)) return launch_gemm_f32_small(a, &d, splits, stream);
  // fewer than 1.5 full tiles per CU: halve the tile height so that twice as many workgroups run
  int tmw = (long)d.tiles_m * d.tiles_n * splits < 384 && a.M > 64 ? 1 : 2;
  if (force_tmw) tmw = force_tmw;
  return dt == DT_F32 ? launch_t<float>(a, d, tmw, splits, stream) : launch_t<bf16_t>(a, d, tmw, splits, stream);
}

}  // namespace fl
