// out[m, n] = in[m, n] * keep(m, n): the gradient that enters a dropped-out branch whose output was
// added to a residual stream (the residual sum's gradient goes on unchanged on the identity branch,
// and masked into the branch).  Also the plain way to look at a mask: apply it to ones.
#include "devutil.h"
#include "kernels.h"
#include "philox.h"

namespace fl {
namespace {

template <typename T>
__global__ __launch_bounds__(256) void dropout_mul_kernel(const T *__restrict__ in, T *__restrict__ out, int M, int N,
                                                          DropSpec d) {
  const int quads = N >> 2;
  const size_t total = (size_t)M * quads;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int m = (int)(i / quads), q = (int)(i - (size_t)m * quads);
    float v[4], k[4];
    VecIO<T, 4>::load(in + (size_t)m * N + q * 4, v);
    drop_keep4(d, (uint32_t)q, (uint32_t)m, 0u, k);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] *= k[e];
    VecIO<T, 4>::store(out + (size_t)m * N + q * 4, v);
  }
}

}  // namespace

hipError_t launch_dropout_mul(int dt, const void *in, void *out, int M, int N, const DropSpec &d, hipStream_t stream) {
  if (!in || !out || M < 1 || N < 4 || N % 4 || d.thr == 0) return hipErrorInvalidValue;
  const size_t total = (size_t)M * (N / 4);
  const size_t want = (total + 255) / 256;
  const int grid = (int)(want > 256 * 16 ? 256 * 16 : want);
  if (dt == DT_F32)
    hipLaunchKernelGGL(dropout_mul_kernel<float>, dim3(grid), dim3(256), 0, stream, static_cast<const float *>(in),
                       static_cast<float *>(out), M, N, d);
  else
    hipLaunchKernelGGL(dropout_mul_kernel<bf16_t>, dim3(grid), dim3(256), 0, stream, static_cast<const bf16_t *>(in),
                       static_cast<bf16_t *>(out), M, N, d);
  return hipGetLastError();
}

}  // namespace fl
