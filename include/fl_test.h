/*
 * fl_test.h -- test-only entry points of the library.
 *
 * Each hot-path kernel on its own (so that a parity test can compare it with the
 * matching step of the CPU oracle), the caching allocator over a caller-supplied
 * backing store, and the tape with stub operators (so that the host logic can be
 * tested without a GPU).  Nothing here is needed to run a layer.
 *
 * dtype is fl_dtype_t.  Pointers named A, B, C, x, y, ... are DEVICE pointers,
 * 16-byte aligned; hip_stream is a hipStream_t.  Return value: fl_status_t
 * (0 = ok; fl_last_error() has the message).  Nothing synchronises.
 */
#ifndef FL_TEST_H
#define FL_TEST_H
#include <stddef.h>
#include <stdint.h>
#include "fl_layer.h"
#ifdef __cplusplus
extern "C" {
#endif

/* C[M,N] = sum_k A(m,k) B(n,k) with the epilogue of the layer's GEMMs, in this order:
 * v += bias[n]; preact = v; v = act(v) (1 relu, 2 gelu); v += residual; v *= act'(aux)
 * (dact 1: aux > 0, dact 2: GELU derivative at aux).  a_kc: A is [M,K] (k contiguous) else
 * [K,M]; b_kc: B is [N,K] else [K,N].  splits: 0 = library's choice, 1 = none, >1 = that many
 * k-ranges (then `partial` must hold splits*M*N floats and the epilogue must be empty).
 * This is the matmul primitive of the paper's tensor interface (Section 4.1.1). */
int32_t fl_test_gemm(int32_t dtype, int32_t a_kc, int32_t b_kc, const void *A, const void *B, void *C, int32_t M,
                     int32_t N, int32_t K, const void *bias, const void *residual, int32_t act, void *preact,
                     int32_t dact, const void *aux, int32_t splits, float *partial, void *hip_stream);
/* Mean milliseconds (host pointer ms) of `iters` back-to-back launches of the plain GEMM. */
int32_t fl_test_gemm_time(int32_t dtype, int32_t a_kc, int32_t b_kc, const void *A, const void *B, void *C, int32_t M,
                          int32_t N, int32_t K, int32_t splits, float *partial, int32_t iters, float *ms,
                          void *hip_stream);
int32_t fl_test_gemm_splits(int32_t dtype, int32_t M, int32_t N, int32_t K);
/* Host-side selection rules (no GPU work): the pipelined bf16 kernel's tile variant for a problem
 * (-2 = the register-staged kernel; operand flags as in fl_test_gemm; _forward: y = x W^T as the forward
 * pass launches it, with the chip to itself), whether an fp32 output runs on
 * the 32 x 32-tile kernel, and which attention kernels serve a head size (0 general, 1 bf16 matrix-core,
 * 2 fp32 matrix-core). */
int32_t fl_test_gemm_variant(int32_t a_kc, int32_t b_kc, int32_t M, int32_t N, int32_t K);
int32_t fl_test_gemm_variant_forward(int32_t M, int32_t N, int32_t K);
int32_t fl_test_gemm_f32_small(int32_t M, int32_t N);
int32_t fl_test_attention_path(int32_t dtype, int32_t dh);
/* Tile/stage variant of the pipelined bf16 GEMM: -1 automatic, 0..3 forced, -2 use the plain kernel. */
void fl_test_gemm_force_variant(int32_t v);
/* Tile height of the plain GEMM kernel: 0 automatic, 1 = 64x128 tiles, 2 = 128x128 tiles. */
void fl_test_gemm_force_tile_height(int32_t tmw);

/* LayerNorm (a normalisation primitive, Section 4.2) over the last dimension of x[M,D]. */
int32_t fl_test_layernorm_fwd(int32_t dtype, const void *x, const void *gamma, const void *beta, float eps, int32_t M,
                              int32_t D, void *y, float *mean, float *rstd, void *hip_stream);
int32_t fl_test_layernorm_bwd_ws_floats(int32_t M, int32_t D);
/* dx = LN'(dy) (+ add if non-null); dgamma, dbeta; dxsum (may be NULL) = column sums of dx. */
int32_t fl_test_layernorm_bwd(int32_t dtype, const void *dy, const void *x, const float *mean, const float *rstd,
                              const void *gamma, const void *add, int32_t M, int32_t D, void *dx, void *dgamma,
                              void *dbeta, void *dxsum, float *ws, void *hip_stream);

/* out[n] = sum_m in[m,n]: the bias gradient of a linear layer. */
int64_t fl_test_colsum_ws_floats(int32_t M, int32_t N);
int32_t fl_test_colsum(int32_t dtype, const void *in, int32_t M, int32_t N, float *ws, void *out, void *hip_stream);

/* dst = src for nbytes (a multiple of 16): a plain copy kernel of known traffic (nbytes read, nbytes
 * written), against which the HBM byte counters are calibrated and copy bandwidth is measured. */
int32_t fl_test_copy(const void *src, void *dst, uint64_t nbytes, void *hip_stream);

/* Matrix-core ceiling of this GPU: `workgroups` x 4 wavefronts issue iters x 8 independent 32x32 MFMAs of
 * `dtype` (fl_dtype_t) on register operands.  out: device, workgroups * 256 floats (written, content
 * irrelevant); *flops: host, receives the floating-point operations one launch performs (may be NULL).
 * The caller times the launch; the benchmark reports the rate beside the datasheet peak. */
int32_t fl_test_mfma_probe(int32_t dtype, int32_t workgroups, int32_t iters, float *out, double *flops, void *hip_stream);

/* dst[j] [cols[j], rows[j]] = transpose of src[j] [rows[j], cols[j]] for j < n <= 4: row-major bf16
 * device matrices, sizes multiples of 8, 16-byte aligned, no overlap; src/dst/rows/cols are HOST arrays.
 * The kernel that makes the layer's transposed weight copies. */
int32_t fl_test_transpose_bf16(int32_t n, const void *const *src, void *const *dst, const int32_t *rows,
                               const int32_t *cols, void *hip_stream);

/* Masked scaled-dot-product attention on qkv[B*T, 3*H*dh]; lse and delta are fp32 [B,H,T];
 * causal != 0 adds the mask j > i; p_drop > 0 drops probabilities out (site 1 of fl_layer_set_dropout). */
int32_t fl_test_attention_fwd(int32_t dtype, const void *qkv, const int32_t *lengths, int32_t causal, float p_drop,
                              uint64_t seed, int32_t B, int32_t T, int32_t H, int32_t dh, void *o, float *lse,
                              void *hip_stream);
int32_t fl_test_attention_bwd(int32_t dtype, const void *qkv, const void *o, const void *dout, const float *lse,
                              const int32_t *lengths, int32_t causal, float p_drop, uint64_t seed, int32_t B,
                              int32_t T, int32_t H, int32_t dh, void *dqkv, float *delta, void *hip_stream);
/* out[m,n] = in[m,n] * keep(m,n) for a hidden-state site (2, 3 or 4) of fl_layer_set_dropout; p > 0. */
int32_t fl_test_dropout_mul(int32_t dtype, const void *in, void *out, int32_t M, int32_t N, int32_t site, float p,
                            uint64_t seed, void *hip_stream);

/* on != 0: bf16 attention uses the general (vector-ALU) kernels instead of the MFMA ones. */
void fl_test_attention_force_general(int32_t on);
/* on != 0: bf16 attention backward always runs as the dQ kernel followed by the dK/dV kernel(s), also where
 * the one-kernel backward (head size 64, T <= 224) would apply. */
void fl_test_attention_force_unfused_bwd(int32_t on);

/* Copies the value that the recorded forward's `lin`-th linear operator produced (0 fused QKV projection,
 * 1 attention projection + residual, 2 first feed-forward linear after its activation and dropout,
 * 3 second feed-forward linear + residual) into dst (device, cap_bytes large) on hip_stream; *bytes (host)
 * receives its size.  Valid between a forward and its backward.  With ReLU the sign pattern of value 2 is
 * the set of decisions u > 0 that the backward pass will use (a decision taken in floating point: a parity
 * test hands the same decisions to the oracle). */
int32_t fl_test_layer_peek_linear(fl_layer_t *layer, int32_t lin, void *dst, uint64_t cap_bytes, uint64_t *bytes,
                                  void *hip_stream);

/* The caching allocator (Section 4.1.2, Section 5.2.2) over a HOST-side backing store:
 * the two callbacks stand in for the device allocator; pointers are never dereferenced. */
typedef int (*fl_test_backing_malloc_fn)(void **ptr, size_t bytes); /* 0 = ok */
typedef int (*fl_test_backing_free_fn)(void *ptr);
void *fl_test_alloc_create(fl_test_backing_malloc_fn m, fl_test_backing_free_fn f);
void fl_test_alloc_destroy(void *a);
void *fl_test_alloc_alloc(void *a, uint64_t bytes, const void *stream);
int32_t fl_test_alloc_release(void *a, void *ptr);
void fl_test_alloc_trim(void *a);
void fl_test_alloc_set_split_limit(void *a, uint64_t bytes);
void fl_test_alloc_stats(void *a, fl_alloc_stats_t *out);
void *fl_test_alloc_alloc_tagged(void *a, uint64_t bytes, const void *stream, int32_t tag);
void fl_test_alloc_trace_enable(void *a, int32_t capacity);
int32_t fl_test_alloc_trace_read(void *a, fl_alloc_event_t *out, int32_t cap);

/* The tape (Section 4.2) with stub gradient functions: see the definition for the arguments. */
int32_t fl_test_tape_replay(int32_t n, const int32_t *in0, const int32_t *in1, int32_t n_input_slots, int32_t fail_at,
                            int32_t *order, int32_t *n_ran, int32_t *first_consumer, int32_t n_slots);

#ifdef __cplusplus
}
#endif
#endif
