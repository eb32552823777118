// fp32 GEMM for outputs with few tiles: C[M,N] = sum_k A(m,k) B(n,k), same contraction, operand
// layouts, k-range splitting and epilogue as gemm.hip (the paper's matmul primitive, Section 4.1.1).
//
// The fp32 MFMA (v_mfma_f32_32x32x2_f32) takes 64 clocks for two k, so a wavefront that owns a
// 64 x 64 block of the output needs K * 64 clocks for it, whatever else the kernel does, and a small
// problem cut into 128 x 128 tiles leaves most SIMDs without a wavefront (1024 x 256 x 1024: 32
// workgroups, 27 us of dependent MFMAs).  Here a workgroup owns a 32 x 32 tile and its four
// wavefronts split every k-tile among themselves (16 of 64 k each), so that the same problem runs on
// 256 workgroups with a chain of K/8 MFMAs per wavefront; the four accumulators meet in LDS, where
// the epilogue picks the sums up row-wise, eight columns per lane.
#include "devutil.h"
#include "gemm_dev.h"
#include "kernels.h"

namespace fl {
namespace {

constexpr int SM = 32, SN = 32, SKT = 64, NTHR = 256;
constexpr int KC_STRIDE = SKT + 4;   // [32 rows][64 k] floats, rows padded by 16 bytes
constexpr int KM_STRIDE = 32 + 4;    // [64 k][32 rows] floats
constexpr int OPERAND_FLOATS = SKT * KM_STRIDE > 32 * KC_STRIDE ? SKT * KM_STRIDE : 32 * KC_STRIDE;
constexpr int C_STRIDE = SN + 4;     // the wavefronts' accumulators as [4][32][36] floats

// one operand tile (32 rows x 64 k) on its way to LDS: two 16-byte chunks per thread
template <bool KC>
__device__ __forceinline__ void load_small(const float *base, int ld, int row0, int nrows, int k0, int kend,
                                           float4 (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = threadIdx.x + NTHR * i;
    bool ok;
    const float *src;
    if (KC) {
      const int row = row0 + c / 16, k = k0 + (c % 16) * 4;
      ok = row < nrows && k < kend;
      src = base + (size_t)row * ld + k;
    } else {
      const int k = k0 + c / 8, row = row0 + (c % 8) * 4;
      ok = k < kend && row < nrows;
      src = base + (size_t)k * ld + row;
    }
    r[i] = ok ? *reinterpret_cast<const float4 *>(src) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
}
template <bool KC> __device__ __forceinline__ void store_small(float *lds, const float4 (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = threadIdx.x + NTHR * i;
    if (KC) *reinterpret_cast<float4 *>(lds + (c / 16) * KC_STRIDE + (c % 16) * 4) = r[i];
    else *reinterpret_cast<float4 *>(lds + (c / 8) * KM_STRIDE + (c % 8) * 4) = r[i];
  }
}
// operand value of row lane%32 at tile-k `k`
template <bool KC> __device__ __forceinline__ float frag_small(const float *lds, int k, int lane) {
  return KC ? lds[(lane & 31) * KC_STRIDE + k] : lds[k * KM_STRIDE + (lane & 31)];
}

template <bool AKC, bool BKC, bool DROP>
__global__ __launch_bounds__(NTHR) void gemm_f32_small(GemmDev p) {
  __shared__ __attribute__((aligned(16))) float sA[OPERAND_FLOATS];
  __shared__ __attribute__((aligned(16))) float sB[OPERAND_FLOATS];
  __shared__ __attribute__((aligned(16))) float sC[4 * SM * C_STRIDE];
  int split, tile_m, tile_n;
  xcd_work_coords(blockIdx.x, p.tiles_m, p.tiles_n, p.splits, 32, split, tile_m, tile_n);
  const int row0 = tile_m * SM, col0 = tile_n * SN;
  const int kbeg = split * p.k_per_split;
  if (p.partial) p.partial += (size_t)split * p.M * p.N;
  const int kend = min(p.K, kbeg + p.k_per_split);
  const float *A = static_cast<const float *>(p.A);
  const float *B = static_cast<const float *>(p.B);
  const int lane = threadIdx.x & 63, kg = threadIdx.x >> 6, h2 = lane >> 5;

  f32x16_t acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  float4 ra[2], rb[2];
  if (kbeg < kend) {
    load_small<AKC>(A, p.lda, row0, p.M, kbeg, kend, ra);
    load_small<BKC>(B, p.ldb, col0, p.N, kbeg, kend, rb);
  }
  for (int k0 = kbeg; k0 < kend; k0 += SKT) {
    store_small<AKC>(sA, ra);
    store_small<BKC>(sB, rb);
    __syncthreads();
    if (k0 + SKT < kend) {  // the next tile's loads stay in flight during the MFMAs
      load_small<AKC>(A, p.lda, row0, p.M, k0 + SKT, kend, ra);
      load_small<BKC>(B, p.ldb, col0, p.N, k0 + SKT, kend, rb);
    }
#pragma unroll
    for (int kk = 0; kk < SKT / 8; ++kk) {  // this wavefront's quarter of the k-tile, two k per MFMA
      const int k = kg * (SKT / 4) + kk * 2 + h2;
      // D = B_frag x A_frag: register q*4+e of a lane ends up as C[lane%32, q*8 + (lane/32)*4 + e]
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(frag_small<BKC>(sB, k, lane), frag_small<AKC>(sA, k, lane), acc, 0, 0, 0);
    }
    __syncthreads();
  }
  // the four partial tiles, row-major
  float *mine = sC + kg * SM * C_STRIDE + (lane & 31) * C_STRIDE + h2 * 4;
#pragma unroll
  for (int q = 0; q < 4; ++q)
    *reinterpret_cast<float4 *>(mine + q * 8) = make_float4(acc[q * 4], acc[q * 4 + 1], acc[q * 4 + 2], acc[q * 4 + 3]);
  __syncthreads();
  if (threadIdx.x < SM * (SN / 8)) {
    const int m = row0 + threadIdx.x / (SN / 8), n0 = col0 + (threadIdx.x % (SN / 8)) * 8;
    if (m < p.M && n0 < p.N) {
      const float *src = sC + (threadIdx.x / (SN / 8)) * C_STRIDE + (threadIdx.x % (SN / 8)) * 8;
      float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int g = 0; g < 4; ++g) {   // fixed order: the result does not depend on timing
        const float4 lo = *reinterpret_cast<const float4 *>(src + g * SM * C_STRIDE);
        const float4 hi = *reinterpret_cast<const float4 *>(src + g * SM * C_STRIDE + 4);
        v[0] += lo.x; v[1] += lo.y; v[2] += lo.z; v[3] += lo.w;
        v[4] += hi.x; v[5] += hi.y; v[6] += hi.z; v[7] += hi.w;
      }
      float bias8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if (p.bias && !p.partial) Oct<float>::load(static_cast<const float *>(p.bias) + n0, bias8);
      gemm_epilogue_oct<float, DROP>(p, m, n0, v, bias8);
    }
  }
}

template <bool DROP> hipError_t launch_d(const GemmArgs &a, const GemmDev &d, dim3 grid, hipStream_t s) {
  if (a.a_kc && a.b_kc) hipLaunchKernelGGL((gemm_f32_small<true, true, DROP>), grid, dim3(NTHR), 0, s, d);
  else if (a.a_kc && !a.b_kc) hipLaunchKernelGGL((gemm_f32_small<true, false, DROP>), grid, dim3(NTHR), 0, s, d);
  else if (!a.a_kc && !a.b_kc) hipLaunchKernelGGL((gemm_f32_small<false, false, DROP>), grid, dim3(NTHR), 0, s, d);
  else hipLaunchKernelGGL((gemm_f32_small<false, true, DROP>), grid, dim3(NTHR), 0, s, d);
  return hipGetLastError();
}

}  // namespace

// Fewer than one 64 x 128 tile per CU: the tiles of gemm.hip would leave most of the chip idle.
bool gemm_f32_small_applies(int M, int N) { return (long)((M + 63) / 64) * ((N + 127) / 128) < 256; }

// `dev` is launch_gemm's filled GemmDev; the tile counts are recomputed for 32 x 32 tiles.
hipError_t launch_gemm_f32_small(const GemmArgs &a, const void *dev, int splits, hipStream_t s) {
  GemmDev d = *static_cast<const GemmDev *>(dev);
  d.tiles_m = (a.M + SM - 1) / SM;
  d.tiles_n = (a.N + SN - 1) / SN;
  d.splits = splits;
  dim3 grid(d.tiles_m * d.tiles_n * splits);
  return d.drop_where ? launch_d<true>(a, d, grid, s) : launch_d<false>(a, d, grid, s);
}

}  // namespace fl
