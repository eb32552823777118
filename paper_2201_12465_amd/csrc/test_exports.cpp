// Test-only entry points (declared in include/fl_test.h): each kernel launcher on
// its own, the allocator over a caller-supplied backing store, and the tape with
// stub operators.  They let the parity tests compare every kernel with the
// corresponding oracle step, and the CPU tests exercise the host logic without
// a GPU.  None of them is needed to run a layer.
#include <hip/hip_runtime_api.h>

#include <vector>

#include "../../include/fl_layer.h"
#include "../../include/fl_test.h"
#include "allocator.h"
#include "kernels.h"
#include "runtime.h"
#include "tape.h"

using namespace fl;

namespace {
int hip_status(hipError_t e, const char *what) {
  if (e == hipSuccess) return FL_OK;
  return set_error(e == hipErrorInvalidValue ? FL_ERR_UNSUPPORTED : FL_ERR_DEVICE, "%s: %s", what,
                   hipGetErrorString(e));
}
struct TapeLog {
  int32_t *order;
  int cap, n;
};
int stub_backward(void *ctx, Tape *tape, const Node *self) {
  TapeLog *log = static_cast<TapeLog *>(ctx);
  if (self->flags == 2) return 77;  // a failing gradient function
  if (log->n < log->cap) log->order[log->n] = tape->index_of(self);
  log->n++;
  return 0;
}
}  // namespace

extern "C" {

int32_t fl_test_gemm(int32_t dtype, int32_t a_kc, int32_t b_kc, const void *A, const void *B, void *C, int32_t M,
                     int32_t N, int32_t K, const void *bias, const void *residual, int32_t act, void *preact,
                     int32_t dact, const void *aux, int32_t splits, float *partial, void *hip_stream) {
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  GemmArgs a;
  a.A = A; a.B = B; a.C = C; a.M = M; a.N = N; a.K = K;
  a.a_kc = a_kc != 0; a.b_kc = b_kc != 0;
  a.lda = a.a_kc ? K : M; a.ldb = a.b_kc ? K : N; a.ldc = N;
  a.bias = bias; a.residual = residual; a.act = act; a.preact = preact; a.dact = dact; a.aux = aux;
  const int dt = dtype == FL_F32 ? DT_F32 : DT_BF16;
  a.splits = splits > 0 ? splits : gemm_pick_splits(dt, M, N, K);
  if (a.splits > 1) {
    if (!partial) return set_error(FL_ERR_INVALID_ARG, "split GEMM needs a partial buffer");
    a.partial = partial;
    int rc = hip_status(launch_gemm(dt, a, st), "launch_gemm");
    if (rc) return rc;
    return hip_status(launch_reduce_partials(dt, partial, a.splits, (size_t)M * N, (size_t)M * N, 1, C, nullptr,
                                             nullptr, st),
                      "launch_reduce_partials");
  }
  return hip_status(launch_gemm(dt, a, st), "launch_gemm");
}

// Times `iters` back-to-back launches of one GEMM (no epilogue) with HIP events on the stream;
// *ms receives the mean milliseconds per launch.  Synchronises the stream.
int32_t fl_test_gemm_time(int32_t dtype, int32_t a_kc, int32_t b_kc, const void *A, const void *B, void *C, int32_t M,
                          int32_t N, int32_t K, int32_t splits, float *partial, int32_t iters, float *ms,
                          void *hip_stream) {
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
    return set_error(FL_ERR_DEVICE, "hipEventCreate failed");
  int rc = 0;
  for (int it = -2; it < iters && !rc; ++it) {
    if (it == 0) (void)hipEventRecord(e0, st);
    rc = fl_test_gemm(dtype, a_kc, b_kc, A, B, C, M, N, K, nullptr, nullptr, 0, nullptr, 0, nullptr, splits, partial,
                      hip_stream);
  }
  (void)hipEventRecord(e1, st);
  hipError_t e = hipEventSynchronize(e1);
  float t = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc) return rc;
  if (e != hipSuccess) return hip_status(e, "event timing");
  *ms = t / (iters > 0 ? iters : 1);
  return FL_OK;
}

void fl_test_gemm_force_variant(int32_t v) { gemm_pipe_force_variant(v); }
void fl_test_gemm_force_tile_height(int32_t tmw) { gemm_force_tile_height(tmw); }

int32_t fl_test_gemm_variant(int32_t a_kc, int32_t b_kc, int32_t M, int32_t N, int32_t K) {
  return gemm_pipe_pick_variant(a_kc != 0, b_kc != 0, M, N, K, false);
}
int32_t fl_test_gemm_variant_forward(int32_t M, int32_t N, int32_t K) {
  return gemm_pipe_pick_variant(true, true, M, N, K, true);
}
int32_t fl_test_gemm_f32_small(int32_t M, int32_t N) { return gemm_f32_small_applies(M, N) ? 1 : 0; }
int32_t fl_test_attention_path(int32_t dtype, int32_t dh) {
  if (dtype == FL_BF16) return attention_mfma_supported(dh) ? 1 : 0;
  return attention_mfma_f32_supported(dh) ? 2 : 0;
}

int32_t fl_test_gemm_splits(int32_t dtype, int32_t M, int32_t N, int32_t K) {
  return gemm_pick_splits(dtype == FL_F32 ? DT_F32 : DT_BF16, M, N, K);
}

int32_t fl_test_layernorm_fwd(int32_t dtype, const void *x, const void *gamma, const void *beta, float eps, int32_t M,
                              int32_t D, void *y, float *mean, float *rstd, void *hip_stream) {
  return hip_status(launch_layernorm_fwd(dtype == FL_F32 ? DT_F32 : DT_BF16, x, gamma, beta, eps, M, D, y, mean, rstd,
                                         static_cast<hipStream_t>(hip_stream)),
                    "launch_layernorm_fwd");
}

int32_t fl_test_layernorm_bwd_ws_floats(int32_t M, int32_t D) { return ln_bwd_parts(M, D) * 3 * D; }

int32_t fl_test_layernorm_bwd(int32_t dtype, const void *dy, const void *x, const float *mean, const float *rstd,
                              const void *gamma, const void *add, int32_t M, int32_t D, void *dx, void *dgamma,
                              void *dbeta, void *dxsum, float *ws, void *hip_stream) {
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int dt = dtype == FL_F32 ? DT_F32 : DT_BF16;
  int rc = hip_status(launch_layernorm_bwd(dt, dy, x, mean, rstd, gamma, add, M, D, dx, ws, st),
                      "launch_layernorm_bwd");
  if (rc) return rc;
  return hip_status(launch_reduce_partials(dt, ws, ln_bwd_parts(M, D), (size_t)3 * D, (size_t)D, dxsum ? 3 : 2,
                                           dgamma, dbeta, dxsum, st),
                    "launch_reduce_partials");
}

int32_t fl_test_copy(const void *src, void *dst, uint64_t nbytes, void *hip_stream) {
  return hip_status(launch_copy(src, dst, (size_t)nbytes, static_cast<hipStream_t>(hip_stream)), "launch_copy");
}

int32_t fl_test_mfma_probe(int32_t dtype, int32_t workgroups, int32_t iters, float *out, double *flops, void *hip_stream) {
  if (dtype != DT_F32 && dtype != DT_BF16) return set_error(FL_ERR_INVALID_ARG, "fl_test_mfma_probe: unknown dtype %d", dtype);
  return hip_status(launch_mfma_probe(dtype, workgroups, iters, out, flops, static_cast<hipStream_t>(hip_stream)),
                    "launch_mfma_probe");
}

int32_t fl_test_transpose_bf16(int32_t n, const void *const *src, void *const *dst, const int32_t *rows,
                               const int32_t *cols, void *hip_stream) {
  return hip_status(launch_transpose_bf16(n, src, dst, rows, cols, static_cast<hipStream_t>(hip_stream)),
                    "launch_transpose_bf16");
}

int64_t fl_test_colsum_ws_floats(int32_t M, int32_t N) { return (int64_t)colsum_ws_floats(M, N); }

int32_t fl_test_colsum(int32_t dtype, const void *in, int32_t M, int32_t N, float *ws, void *out, void *hip_stream) {
  return hip_status(launch_colsum(dtype == FL_F32 ? DT_F32 : DT_BF16, in, M, N, ws, out,
                                  static_cast<hipStream_t>(hip_stream)),
                    "launch_colsum");
}

int32_t fl_test_attention_fwd(int32_t dtype, const void *qkv, const int32_t *lengths, int32_t causal, float p_drop,
                              uint64_t seed, int32_t B, int32_t T, int32_t H, int32_t dh, void *o, float *lse,
                              void *hip_stream) {
  return hip_status(launch_attention_fwd(dtype == FL_F32 ? DT_F32 : DT_BF16, qkv, lengths, causal,
                                         make_drop_spec(p_drop, seed, 1), B, T, H, dh, o, lse,
                                         static_cast<hipStream_t>(hip_stream)),
                    "launch_attention_fwd");
}

int32_t fl_test_attention_bwd(int32_t dtype, const void *qkv, const void *o, const void *dout, const float *lse,
                              const int32_t *lengths, int32_t causal, float p_drop, uint64_t seed, int32_t B,
                              int32_t T, int32_t H, int32_t dh, void *dqkv, float *delta, void *hip_stream) {
  return hip_status(launch_attention_bwd(dtype == FL_F32 ? DT_F32 : DT_BF16, qkv, o, dout, lse, lengths, causal,
                                         make_drop_spec(p_drop, seed, 1), B, T, H, dh, dqkv, delta,
                                         static_cast<hipStream_t>(hip_stream)),
                    "launch_attention_bwd");
}

int32_t fl_test_dropout_mul(int32_t dtype, const void *in, void *out, int32_t M, int32_t N, int32_t site, float p,
                            uint64_t seed, void *hip_stream) {
  return hip_status(launch_dropout_mul(dtype == FL_F32 ? DT_F32 : DT_BF16, in, out, M, N,
                                       make_drop_spec(p, seed, (uint32_t)site), static_cast<hipStream_t>(hip_stream)),
                    "launch_dropout_mul");
}

void fl_test_attention_force_general(int32_t on) { attention_force_general(on != 0); }
void fl_test_attention_force_unfused_bwd(int32_t on) { attention_force_unfused_bwd(on != 0); }

// ---- allocator over a caller-supplied backing store -------------------------------------
void *fl_test_alloc_create(fl_test_backing_malloc_fn m, fl_test_backing_free_fn f) {
  return new CachingAllocator(m, f);
}
void fl_test_alloc_destroy(void *a) { delete static_cast<CachingAllocator *>(a); }
void *fl_test_alloc_alloc(void *a, uint64_t bytes, const void *stream) {
  return static_cast<CachingAllocator *>(a)->alloc((size_t)bytes, stream);
}
int32_t fl_test_alloc_release(void *a, void *ptr) { return static_cast<CachingAllocator *>(a)->release(ptr) ? 0 : 1; }
void fl_test_alloc_trim(void *a) { static_cast<CachingAllocator *>(a)->trim(); }
void fl_test_alloc_set_split_limit(void *a, uint64_t bytes) {
  static_cast<CachingAllocator *>(a)->set_split_limit((size_t)bytes);
}
void fl_test_alloc_stats(void *a, fl_alloc_stats_t *out) {
  AllocStats s = static_cast<CachingAllocator *>(a)->stats();
  out->backing_mallocs = s.backing_mallocs; out->backing_bytes = s.backing_bytes;
  out->cache_hits = s.cache_hits; out->cache_misses = s.cache_misses;
  out->live_bytes = s.live_bytes; out->peak_bytes = s.peak_bytes;
  out->cached_bytes = s.cached_bytes; out->split_count = s.split_count;
  out->requested_bytes = s.requested_bytes; out->largest_free_block = s.largest_free_block;
  out->free_blocks = s.free_blocks;
}
void *fl_test_alloc_alloc_tagged(void *a, uint64_t bytes, const void *stream, int32_t tag) {
  return static_cast<CachingAllocator *>(a)->alloc((size_t)bytes, stream, tag);
}
void fl_test_alloc_trace_enable(void *a, int32_t capacity) {
  static_cast<CachingAllocator *>(a)->trace_enable(capacity > 0 ? (size_t)capacity : 0);
}
int32_t fl_test_alloc_trace_read(void *a, fl_alloc_event_t *out, int32_t cap) {
  static_assert(sizeof(fl_alloc_event_t) == sizeof(AllocEvent), "the two event records must have one layout");
  return (int32_t)static_cast<CachingAllocator *>(a)->trace_read(reinterpret_cast<AllocEvent *>(out), cap > 0 ? (size_t)cap : 0);
}

// ---- tape with stub operators -------------------------------------------------------------
// Records n nodes; node i reads slots in0[i], in1[i] (-1 = none) and writes a fresh slot.
// Replays in reverse; order[] receives the node indices in the order their gradient
// functions ran; first_consumer[] (n_slots entries) the recorded first consumer of each
// slot.  fail_at >= 0 makes that node's gradient function fail.  Returns the replay's code.
int32_t fl_test_tape_replay(int32_t n, const int32_t *in0, const int32_t *in1, int32_t n_input_slots, int32_t fail_at,
                            int32_t *order, int32_t *n_ran, int32_t *first_consumer, int32_t n_slots) {
  Tape tape;
  for (int i = 0; i < n_input_slots; ++i) tape.new_slot();
  for (int i = 0; i < n; ++i) {
    Node nd;
    nd.backward = stub_backward;
    nd.in0 = in0[i];
    nd.in1 = in1[i];
    nd.flags = i == fail_at ? 2 : 0;
    if (nd.in0 >= (int)tape.slots.size() || nd.in1 >= (int)tape.slots.size()) return -1;
    nd.out = tape.new_slot();
    tape.record(nd);
  }
  TapeLog log{order, n, 0};
  int rc = tape.replay_reverse(&log);
  *n_ran = log.n;
  for (int s = 0; s < n_slots && s < (int)tape.slots.size(); ++s) first_consumer[s] = tape.slots[s].first_consumer;
  return rc;
}

}  // extern "C"
