// Out-of-place transposes of up to TRANSPOSE_MAX row-major bf16 matrices in one launch.
//
// The layer keeps a transposed copy of its four weight matrices for the backward pass: the input
// gradient dx = dy W contracts over W's ROW index, and with W^T in memory that contraction runs along
// contiguous elements of both operands, which is the layout the pipelined GEMM kernel is fastest on.
// (The paper leaves the layout of a matmul's operands to the backend, Section 4.1.1.)
//
// A workgroup moves one 64 x 64 tile through LDS: 16-byte row chunks in, 16-byte row chunks of the
// transposed tile out.  Rows and columns are multiples of 8, so every chunk is whole.
#include "devutil.h"
#include "kernels.h"

namespace fl {
namespace {

constexpr int TT = 64;          // tile edge
constexpr int TP = TT + 2;      // LDS row pitch in elements: 33 words, so a column walk touches every bank once

struct TransposeJobs {
  const bf16_t *src[TRANSPOSE_MAX];
  bf16_t *dst[TRANSPOSE_MAX];
  int rows[TRANSPOSE_MAX], cols[TRANSPOSE_MAX];
  int tiles_c[TRANSPOSE_MAX];   // tiles along the columns of src
  int first[TRANSPOSE_MAX + 1]; // first workgroup of each job; first[n] = grid size
  int n;
};

__global__ __launch_bounds__(256) void transpose_tiles_kernel(TransposeJobs jobs) {
  __shared__ bf16_t tile[TT * TP];
  int j = 0;
  while (j + 1 < jobs.n && (int)blockIdx.x >= jobs.first[j + 1]) ++j;
  const int t = blockIdx.x - jobs.first[j];
  const int R = jobs.rows[j], C = jobs.cols[j];
  const int r0 = (t / jobs.tiles_c[j]) * TT, c0 = (t % jobs.tiles_c[j]) * TT;
  const bf16_t *src = jobs.src[j];
  bf16_t *dst = jobs.dst[j];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int ch = threadIdx.x + 256 * i, r = ch >> 3, c = (ch & 7) * 8;
    bf16x8_t v = bf16x8_t{};
    if (r0 + r < R && c0 + c < C) v = *reinterpret_cast<const bf16x8_t *>(src + (size_t)(r0 + r) * C + c0 + c);
    const uint4 u = __builtin_bit_cast(uint4, v);
    uint32_t *w = reinterpret_cast<uint32_t *>(&tile[r * TP + c]);  // 4-byte writes: the pitch is not a multiple of 16 bytes
    w[0] = u.x, w[1] = u.y, w[2] = u.z, w[3] = u.w;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int ch = threadIdx.x + 256 * i, c = ch >> 3, r = (ch & 7) * 8;  // output row c0 + c, columns r0 + r ..
    if (c0 + c < C && r0 + r < R) {
      bf16x8_t v;
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = tile[(r + e) * TP + c];
      *reinterpret_cast<bf16x8_t *>(dst + (size_t)(c0 + c) * R + r0 + r) = v;
    }
  }
}

}  // namespace

hipError_t launch_transpose_bf16(int n, const void *const *src, void *const *dst, const int *rows, const int *cols,
                                 hipStream_t stream) {
  if (n < 1 || n > TRANSPOSE_MAX || !src || !dst || !rows || !cols) return hipErrorInvalidValue;
  TransposeJobs jobs;
  jobs.n = n;
  int total = 0;
  for (int j = 0; j < n; ++j) {
    if (!src[j] || !dst[j] || rows[j] < 8 || cols[j] < 8 || rows[j] % 8 || cols[j] % 8 ||
        ((uintptr_t)src[j] | (uintptr_t)dst[j]) % 16)
      return hipErrorInvalidValue;
    jobs.src[j] = static_cast<const bf16_t *>(src[j]);
    jobs.dst[j] = static_cast<bf16_t *>(dst[j]);
    jobs.rows[j] = rows[j];
    jobs.cols[j] = cols[j];
    jobs.tiles_c[j] = (cols[j] + TT - 1) / TT;
    jobs.first[j] = total;
    const long tiles = (long)jobs.tiles_c[j] * ((rows[j] + TT - 1) / TT);
    if (total + tiles > (1l << 30)) return hipErrorInvalidValue;
    total += (int)tiles;
  }
  for (int j = n; j <= TRANSPOSE_MAX; ++j) jobs.first[j] = total;
  for (int j = n; j < TRANSPOSE_MAX; ++j) {
    jobs.src[j] = nullptr; jobs.dst[j] = nullptr; jobs.rows[j] = jobs.cols[j] = 0; jobs.tiles_c[j] = 1;
  }
  transpose_tiles_kernel<<<total, 256, 0, stream>>>(jobs);
  return hipGetLastError();
}

}  // namespace fl
