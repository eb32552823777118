// Launchers of the gfx950 kernels.  Every launcher validates what its kernel and
// grid assume, enqueues on `stream`, never synchronises, and returns hipError_t.
// Element type: dt = 0 -> float, 1 -> bfloat16 (storage; all arithmetic in fp32).
#pragma once
#include <hip/hip_runtime_api.h>
#include <cstddef>
#include <cstdint>
#include "philox.h"

namespace fl {

enum { DT_F32 = 0, DT_BF16 = 1 };
static inline size_t dt_size(int dt) { return dt == DT_F32 ? 4 : 2; }

// ---------------------------------------------------------------------------
// GEMM  C[M,N] = sum_k A(m,k) * B(n,k), fp32 accumulation on MFMA.
//   a_kc:  A(m,k) = A[m*lda + k]  (k contiguous)   else  A[k*lda + m]
//   b_kc:  B(n,k) = B[n*ldb + k]  (k contiguous)   else  B[k*ldb + n]
// so  y = x W^T is (a_kc, b_kc);  dx = dy W is (a_kc, !b_kc);  dW = dy^T x is
// (!a_kc, !b_kc) with k running over tokens.
// Epilogue, in this order, on v = accumulator:
//   v += bias[n];  preact[m,n] = v (if preact);  v = act(v);  v += residual[m,n];
//   v *= act'(aux[m,n]) (dact: 1 = aux > 0, 2 = exact-GELU derivative at aux);  C[m,n] = v
// Dropout (drop_where, drop): 1 multiplies v by the keep mask of element (m, n) right after the
// activation (before the residual is added); 2 multiplies it at the very end (the backward of a
// dropped-out activation output: mask and activation derivative commute).
// With splits > 1 (k is cut into `splits` ranges) the raw partial sums go to
// `partial` (fp32 [splits][M][N]) and the epilogue must be empty; the caller then
// runs reduce_partials.
// Requirements (checked): N % 8 == 0; the contiguous dimension of each operand
// % 8 == 0; lda/ldb/ldc % 8 == 0; pointers 16-byte aligned.
struct GemmArgs {
  const void *A = nullptr, *B = nullptr;
  void *C = nullptr;
  int M = 0, N = 0, K = 0, lda = 0, ldb = 0, ldc = 0;
  bool a_kc = true, b_kc = true;
  bool alone = false;  // nothing else is expected on the chip beside this launch (the forward pass): tiles that fill every place
  const void *bias = nullptr, *residual = nullptr, *aux = nullptr;
  void *preact = nullptr;
  int act = 0, dact = 0;
  float *partial = nullptr;
  int splits = 1;
  int drop_where = 0;
  DropSpec drop;
};
hipError_t launch_gemm(int dt, const GemmArgs &a, hipStream_t stream);
// Number of k-ranges launch_gemm should use so that a small output still fills the chip.
int gemm_pick_splits(int dt, int M, int N, int K);
// Kernel-selection overrides (select.cpp).  The getters are constants in the library that ships; the
// setters exist only in the test build (FL_TEST_EXPORTS).
int forced_gemm_pipe_variant();   // -1 = automatic; >= 0 forces a tile/stage variant; -2 = never use the pipelined kernel
int forced_gemm_tile_height();    // gemm.hip kernel: 0 automatic, 1 = 64x128 tiles, 2 = 128x128 tiles
bool forced_general_attention();  // general (vector-ALU) attention kernels for every head size
bool forced_unfused_attention_bwd();  // never the one-kernel attention backward
#ifdef FL_TEST_EXPORTS
void gemm_pipe_force_variant(int v);
void gemm_force_tile_height(int tmw);
void attention_force_general(bool on);
void attention_force_unfused_bwd(bool on);
#endif

// fp32 outputs with few tiles (gemm_f32_small.hip): 32 x 32 tiles, the four wavefronts of a workgroup
// split k.  launch_gemm uses it when gemm_f32_small_applies and no tile height is forced.
bool gemm_f32_small_applies(int M, int N);
hipError_t launch_gemm_f32_small(const GemmArgs &a, const void *gemm_dev, int splits, hipStream_t s);

// The pipelined bf16 kernel (gemm_pipe.hip); launch_gemm uses it whenever the problem is eligible.
bool gemm_pipe_eligible(const GemmArgs &a, int k_per_split);
int gemm_pipe_pick_variant(bool a_kc, bool b_kc, int M, int N, int K, bool alone = false);  // < 0: use the kernel in gemm.hip
hipError_t launch_gemm_bf16_pipe(const GemmArgs &a, const void *gemm_dev, int splits, int variant, hipStream_t s);

// out_s[n] = sum_p partial[p*stride + s*seglen + n]  for s < nseg (<= 3), n < seglen;
// out_s has element type dt.  seglen % 4 == 0.
hipError_t launch_reduce_partials(int dt, const float *partial, int P, size_t stride, size_t seglen,
                                  int nseg, void *out0, void *out1, void *out2, hipStream_t stream,
                                  bool accumulate = false);  // accumulate: out_s += the sums

// Up to REDUCE_MAX_JOBS such reductions in one launch, with the same summation order (bit-identical sums).
constexpr int REDUCE_MAX_JOBS = 8;
struct ReduceJob {
  const float *partial;
  int P, nseg;
  size_t stride, seglen;
  void *out[3];
};
hipError_t launch_reduce_batch(int dt, const ReduceJob *jobs, int n, hipStream_t stream, bool accumulate = false);

// Column sums of in[M,N] (type dt) -> out[N] (type dt); ws must hold colsum_ws_floats(M,N) floats.
// launch_colsum_stage1 runs the first stage alone: ws then holds colsum_stage1_rows(M) partial rows of N
// floats, for a reduction the caller batches with others.
size_t colsum_ws_floats(int M, int N);
int colsum_stage1_rows(int M);
hipError_t launch_colsum_stage1(int dt, const void *in, int M, int N, float *ws, hipStream_t stream);
hipError_t launch_colsum(int dt, const void *in, int M, int N, float *ws, void *out, hipStream_t stream,
                         bool accumulate = false);

// out[m,n] = in[m,n] * keep(m,n) for the hidden-state site in d (in == out allowed); N % 4 == 0.
hipError_t launch_dropout_mul(int dt, const void *in, void *out, int M, int N, const DropSpec &d, hipStream_t stream);

// dst[0..nbytes) = src[0..nbytes): nbytes % 16 == 0, both pointers 16-byte aligned.
hipError_t launch_copy(const void *src, void *dst, size_t nbytes, hipStream_t stream);

// `workgroups` x 4 wavefronts each issue iters x 8 independent 32x32 MFMAs of type dt on register operands;
// out receives workgroups * 256 floats; *flops (host, may be null) = the floating-point operations launched.
hipError_t launch_mfma_probe(int dt, int workgroups, int iters, float *out, double *flops, hipStream_t stream);

// ---------------------------------------------------------------------------
// LayerNorm over the last dimension D of x[M,D] (biased variance, eps inside the
// square root).  Forward writes y and the per-row mean / reciprocal std (fp32).
// D % 8 == 0, D <= 4096.
hipError_t launch_layernorm_fwd(int dt, const void *x, const void *gamma, const void *beta, float eps,
                                int M, int D, void *y, float *mean, float *rstd, hipStream_t stream);
// Backward:  g = dy*gamma;  dx = rstd*(g - mean_D(g) - xhat*mean_D(g*xhat)) (+ add[m,:] if add);
// partial sums over rows of dy*xhat, dy and the final dx go to ws
// ([ln_bwd_parts(M, D)][3][D] floats); reduce_partials turns them into dgamma, dbeta
// and (if wanted) the bias gradient of the producer of x.
int ln_bwd_parts(int M, int D);
hipError_t launch_layernorm_bwd(int dt, const void *dy, const void *x, const float *mean, const float *rstd,
                                const void *gamma, const void *add, int M, int D, void *dx, float *ws,
                                hipStream_t stream);

// ---------------------------------------------------------------------------
// Masked scaled-dot-product attention on the fused projection buffer
// qkv[B*T, 3D] (q | k | v slabs, head h = columns h*dh..).  lengths: device
// int32[B] or nullptr (key j of sequence b is masked iff j >= lengths[b]); causal != 0
// additionally masks key j for query i iff j > i.  Forward writes o[B*T, D] and
// lse[B,H,T] (log-sum-exp of the scaled, masked scores; fp32).  dh % 16 == 0, dh <= 256.
// drop (site 1; thr == 0 = off): the probabilities are multiplied by the keep mask on their way to P V.
hipError_t launch_attention_fwd(int dt, const void *qkv, const int32_t *lengths, int causal, const DropSpec &drop,
                                int B, int T, int H, int dh, void *o, float *lse, hipStream_t stream);
// Backward: dqkv[B*T, 3D] from do_[B*T, D]; delta is fp32 scratch [B,H,T]
// (delta_i = sum_d dO_i O_i).  Rows of dk, dv at masked keys are written as 0.
// `parts` selects the steps: ATTN_BWD_DELTA writes delta, ATTN_BWD_DQ the q slab of dqkv, ATTN_BWD_DKV
// the k and v slabs (both read delta).  With the general kernels dQ and dK/dV do not depend on each
// other, so a caller may enqueue them on different streams once ATTN_BWD_DELTA is complete
// (attention_bwd_parts_independent says whether that holds); on the matrix-core path delta comes out of
// the dQ kernel and the parts must run in order on one stream.
enum { ATTN_BWD_DELTA = 1, ATTN_BWD_DQ = 2, ATTN_BWD_DKV = 4, ATTN_BWD_ALL = 7 };
hipError_t launch_attention_bwd(int dt, const void *qkv, const void *o, const void *do_, const float *lse,
                                const int32_t *lengths, int causal, const DropSpec &drop, int B, int T, int H, int dh,
                                void *dqkv, float *delta, hipStream_t stream, int parts = ATTN_BWD_ALL);
bool attention_bwd_parts_independent(int dt, int dh);


// bf16 attention on the matrix cores (attention_mfma.hip); the launchers above pick it when dt is
// bf16 and the head size is at most 256 (multiples of 16), unless the general kernels are forced.
bool attention_mfma_supported(int dh);
hipError_t launch_attention_fwd_mfma(const void *qkv, const int32_t *lengths, int causal, const DropSpec &drop, int B,
                                     int T, int H, int dh, void *o, float *lse, hipStream_t s);
hipError_t launch_attention_bwd_mfma(const void *qkv, const void *o, const void *dout, const float *lse,
                                     const int32_t *lengths, int causal, const DropSpec &drop, int B, int T, int H,
                                     int dh, void *dqkv, float *delta, hipStream_t s, int parts);

// bf16 attention backward in one kernel (attention_bwd_fused.hip): head size 64 and T <= 224, where a
// (sequence, head) pair fits one workgroup's LDS.  launch_attention_bwd_mfma hands it every such problem
// whose dQ and dK/dV parts are requested together; delta stays inside the kernel.
bool attention_bwd_fused_applies(int T, int dh);
hipError_t launch_attention_bwd_fused(const void *qkv, const void *o, const void *dout, const float *lse,
                                      const int32_t *lengths, int causal, const DropSpec &drop, int B, int T, int H,
                                      int dh, void *dqkv, hipStream_t s);

// fp32 attention on the matrix cores (attention_mfma_f32.hip), picked for dt fp32 and head sizes up
// to 128 (multiples of 16) unless the general kernels are forced.  As on the bf16 path, delta comes out of the
// dQ kernel: ATTN_BWD_DQ before ATTN_BWD_DKV on one stream.
bool attention_mfma_f32_supported(int dh);
hipError_t launch_attention_fwd_mfma_f32(const void *qkv, const int32_t *lengths, int causal, const DropSpec &drop,
                                         int B, int T, int H, int dh, void *o, float *lse, hipStream_t s);
hipError_t launch_attention_bwd_mfma_f32(const void *qkv, const void *o, const void *dout, const float *lse,
                                         const int32_t *lengths, int causal, const DropSpec &drop, int B, int T, int H,
                                         int dh, void *dqkv, float *delta, hipStream_t s, int parts);

// ---------------------------------------------------------------------------
// dst[j] [cols, rows] = transpose of src[j] [rows, cols] (row-major bf16; rows, cols multiples of 8;
// 16-byte aligned; src and dst do not overlap) for j < n <= TRANSPOSE_MAX, in one launch (transpose.hip).
constexpr int TRANSPOSE_MAX = 4;
hipError_t launch_transpose_bf16(int n, const void *const *src, void *const *dst, const int *rows, const int *cols,
                                 hipStream_t stream);

// ---------------------------------------------------------------------------
// Fused optimizer step over up to OPT_MAX_TENSORS tensors in one launch (optimizer.hip).
// kind 0 = SGD (momentum buffer m used iff momentum != 0), 1 = Adam (m, v).  params/grads have
// type dt, state is fp32; numel % 8 == 0; every pointer 16-byte aligned.  inv_bias1/2 are
// 1/(1-beta^t) computed on the host.
constexpr int OPT_MAX_TENSORS = 16;
struct OptHyper {
  float lr, momentum, weight_decay, beta1, beta2, eps, inv_bias1, inv_bias2;
};
// master (may be null, and so may any entry): fp32 copies of the parameters; where given, the update is
// applied to the copy and params[i] receives its rounded value.
hipError_t launch_opt_step(int dt, int kind, const OptHyper &h, int n, void *const *params, const void *const *grads,
                           float *const *m, float *const *v, const long long *numel, hipStream_t stream,
                           float *const *master = nullptr);
// Fills `bytes` (a multiple of 16; p 16-byte aligned) with copies of the 32-bit `word`.
hipError_t launch_fill_words(void *p, size_t bytes, unsigned word, hipStream_t stream);
// Zero-fills n buffers (byte counts multiples of 16) with one kernel.
hipError_t launch_zero_tensors(int n, void *const *ptrs, const long long *bytes, hipStream_t stream);

}  // namespace fl
