/*
 * fl_layer.h -- C ABI of the MI355X-native Transformer encoder layer.
 *
 * One encoder layer's forward and backward pass, executed the way the paper's
 * tensor / autograd stack dispatches it (Flashlight, arXiv 2201.12465):
 * a module's forward() calls tensor primitives (Section 4.1.1, Section 4.2
 * "Neural Network Primitives"), each call is recorded on a dynamic tape together
 * with a gradient function (Section 4.2 "Automatic Differentiation", the
 * cosine-operator listing), backward() replays the tape in reverse, and every
 * intermediate buffer comes from a caching memory manager (Section 4.1.2 and its
 * CachingMemoryManager listing; Section 5.2.2).  Here all of it is native to one
 * gfx950 GPU: hand-written HIP kernels behind the calls below.
 *
 * Conventions
 *   - All pointers named X, Y, dY, dX, params.*, grads.*, lengths are DEVICE
 *     pointers owned by the caller.  Config / stats / handle pointers are HOST.
 *   - Activations are contiguous row-major [B, T, d_model].  Weights are
 *     [out, in] row-major, y = x W^T + b.  Wqkv = rows [Wq; Wk; Wv] ([3D, D]);
 *     head h owns columns h*dh .. (h+1)*dh of each D-wide slab (dh = D / heads).
 *   - Element type of every activation, parameter and gradient is `dtype`
 *     (FL_F32: float; FL_BF16: bfloat16 storage, fp32 accumulation and fp32
 *     softmax / LayerNorm statistics).  Device pointers must be 16-byte aligned.
 *   - `hip_stream` is the caller's hipStream_t (0 = the null stream).  All work
 *     is ordered on it: kernels are enqueued there or on library-owned streams
 *     that wait for it and that it waits for (see fl_set_grad_overlap), so work
 *     the caller enqueues afterwards sees every result.  forward/backward never
 *     synchronise the device.
 *   - Every call returns fl_status_t; no exception or abort crosses this ABI.
 *     fl_last_error() returns a thread-local message for the last failure.
 *     After an error outputs are unspecified; the handle stays destroyable.
 *   - A handle is not thread-safe; distinct handles may be used from distinct
 *     threads.  The caching allocator is process-wide and locked internally.
 */
#ifndef FL_LAYER_H
#define FL_LAYER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fl_layer fl_layer_t; /* opaque: tape + saved activations */

typedef enum {
  FL_OK = 0,
  FL_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, B > max_B, T > max_T, D % heads != 0 */
  FL_ERR_UNSUPPORTED = 2, /* shape outside what the kernels handle, misaligned pointer */
  FL_ERR_OOM = 3,         /* device allocation failed (handle stays usable)            */
  FL_ERR_DEVICE = 4,      /* a HIP call failed                                         */
  FL_ERR_STATE = 5        /* backward without a recorded forward, or on another stream */
} fl_status_t;

typedef enum { FL_F32 = 0, FL_BF16 = 1 } fl_dtype_t;
typedef enum { FL_ACT_RELU = 0, FL_ACT_GELU = 1 } fl_act_t; /* GELU = exact erf form */
typedef enum { FL_NORM_POST = 0, FL_NORM_PRE = 1 } fl_norm_t;

/* Host struct.  Supported shapes: d_model % 8 == 0, d_ffn % 8 == 0,
 * head size dh = d_model / n_heads with dh % 16 == 0 and dh <= 256,
 * d_model <= 4096.  ln_eps <= 0 selects the default 1e-5.
 * causal != 0: query i attends to keys j <= i only (the autoregressive
 * language-model task of Section 4.3 "Text"), on top of the key-padding mask. */
typedef struct {
  int32_t max_B, max_T, d_model, n_heads, d_ffn;
  fl_act_t act;
  fl_norm_t norm;
  fl_dtype_t dtype;
  float ln_eps;
  int32_t causal;
} fl_layer_config_t;

/* Host structs of device pointers; all 12 must be non-null.  Parameters are
 * read during forward AND backward; the library keeps no copy of them beyond
 * one backward pass (forward may leave transposed copies of the four weight
 * matrices behind for its own backward).  Keep them allocated and unchanged
 * from a forward call until the backward call that belongs to it has been
 * enqueued -- or, when no backward follows, until the next forward call on the
 * handle or fl_layer_destroy: the copies are made on a library-owned stream, and
 * those calls are the points at which that stream is joined (joining at the
 * end of forward was measured and costs 4 % of a training step). */
typedef struct {
  const void *Wqkv, *bqkv, *Wo, *bo, *W1, *b1, *W2, *b2, *ln1_g, *ln1_b, *ln2_g, *ln2_b;
} fl_layer_params_t;
typedef struct {
  void *Wqkv, *bqkv, *Wo, *bo, *W1, *b1, *W2, *b2, *ln1_g, *ln1_b, *ln2_g, *ln2_b;
} fl_layer_grads_t;

/* Creates a layer (the paper's Module, Section 4.2).  Allocates no device memory. */
fl_status_t fl_layer_create(const fl_layer_config_t *cfg, fl_layer_t **out);

/* Forward pass (Module::forward, Section 4.2 / the Dropout-module listing's
 * forward()): records one tape node per fused operator.
 *   post-LN:  Y1 = LN1(X + Attn(X)),  Y = LN2(Y1 + FFN(Y1))
 *   pre-LN :  R1 = X + Attn(LN1(X)),  Y = R1 + FFN(LN2(R1))
 *   Attn(x) = softmax(mask(QK^T / sqrt(dh))) V Wo^T + bo,  FFN(x) = act(x W1^T + b1) W2^T + b2.
 * X [B,T,D] is read here and again by backward (it is not copied: keep it
 * unchanged until backward has been enqueued and has run).  `lengths` is a
 * device int32[B] of key-padding lengths (key j of sequence b is masked iff
 * j >= lengths[b]) or NULL for no mask.  1 <= lengths[b] <= T is a precondition:
 * checking it would need a device synchronisation, so forward does not; the
 * kernels use the nearest valid value instead of a length outside that range
 * (never a read past a sequence, never an empty row).  With FL_DEBUG=1 in the
 * environment forward copies the lengths to the host, waits for the stream, and
 * returns FL_ERR_INVALID_ARG for a length outside the range; in that mode every
 * buffer taken from the caching allocator is also filled with NaN bit patterns
 * first, so that a read of memory nobody wrote shows up in the results.  Y [B,T,D] is written.  Any earlier recording on the handle
 * is discarded and its buffers go back to the cache. */
fl_status_t fl_layer_forward(fl_layer_t *layer, const fl_layer_params_t *params, const void *X,
                             const int32_t *lengths, int32_t B, int32_t T, void *Y, void *hip_stream);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The forward pass of fl_layer_forward in evaluation mode (no dropout,
 * nothing recorded or kept for a backward pass), same kernels, same results bit for bit, with every
 * intermediate (projections, attention output and row statistics, residual sums, LayerNorm outputs and
 * statistics, the feed-forward hidden activation) placed in a fixed device array of 128 MiB that each GPU
 * holds from the moment the library's code is loaded on it until the process ends.  The call allocates
 * nothing: no hipMalloc / hipFree, no stream or event creation, not through the caching allocator either
 * (fl_alloc_get_stats does not move).  Arguments, layouts and preconditions as for fl_layer_forward; every
 * kernel runs on hip_stream.
 * Limit: the intermediates alive at one time must fit the array,
 *   max(2*M*D + M*F, 4*M*D) * sizeof(element) + small change <= 128 MiB,   M = B*T
 * (all five benchmark shapes do; 12608 tokens of d_model 768, d_ffn 3072 in bf16 need 116 MB).  Beyond it
 * the call returns FL_ERR_UNSUPPORTED and enqueues nothing.  FL_ERR_STATE if the handle holds a recorded
 * forward whose backward has not run.
 * Every call on one GPU uses the same array and leaves its contents behind: two calls that may overlap on
 * a GPU (different streams without an event between them, different threads) race on it.  Calls on one
 * stream are ordered and safe.  Nothing in the array needs to start at zero. */
fl_status_t fl_layer_forward_static(fl_layer_t *layer, const fl_layer_params_t *params, const void *X,
                                    const int32_t *lengths, int32_t B, int32_t T, void *Y, void *hip_stream);

/* Backward pass (Variable::backward(), Section 4.2; the training-loop listing's
 * loss.backward()): replays the tape of the last forward in reverse order.
 * dY [B,T,D] is the upstream gradient; dX [B,T,D] and all 12 gradient tensors
 * are OVERWRITTEN (each parameter is used once per layer, so this equals the
 * paper's addGrad after zeroGrad).  `params` must hold the same values as in
 * the forward call.  Saved activations are released to the cache as their
 * nodes are replayed; a second backward without a new forward is FL_ERR_STATE. */
fl_status_t fl_layer_backward(fl_layer_t *layer, const fl_layer_params_t *params, const void *dY,
                              void *dX, fl_layer_grads_t *grads, void *hip_stream);

/* As fl_layer_backward, but with accumulate != 0 the 12 parameter gradients are ADDED to what
 * `grads` already holds -- the paper's addGrad semantics (Section 4.2, cosine-operator listing),
 * used to sum the gradients of several micro-batches before one optimizer step.  dX is always
 * overwritten. */
fl_status_t fl_layer_backward_accumulate(fl_layer_t *layer, const fl_layer_params_t *params, const void *dY,
                                         void *dX, fl_layer_grads_t *grads, int32_t accumulate, void *hip_stream);

/* Dropout for the forward passes that follow (training mode; the paper's Transformer workloads train
 * with it, Section 4.2 shows the module).  Four sites, as in the usual encoder layer: the attention
 * probabilities (rate p_attn) and, with rate p_hidden, the output of the attention projection and of
 * the second feed-forward linear right before their residual adds, and the output of the
 * feed-forward activation.  Kept elements are multiplied by 1/(1-p).  Every decision is a pure
 * function of (seed, site, element position) through the counter-based generator Philox4x32-10
 * (Salmon et al., SC'11): key = (seed mod 2^32, seed div 2^32); counter = (column div 4, row, site, c3),
 * the element uses word (column mod 4); kept iff word >= min(2^32-1, floor(p * 2^32)).
 * Site 1 (attention): row = query, column = key, c3 = b*H + h.  Sites 2 (projection), 3 (activation),
 * 4 (second linear): row = b*T + t, column = feature, c3 = 0.  A backward pass uses the settings of
 * the forward pass it belongs to.  Rates of 0 (the default) switch dropout off; pass a new seed per
 * step.  Rates must be in [0, 1). */
fl_status_t fl_layer_set_dropout(fl_layer_t *layer, float p_attn, float p_hidden, uint64_t seed);

/* Releases the handle and returns its buffers to the cache.  NULL is a no-op. */
fl_status_t fl_layer_destroy(fl_layer_t *layer);

/* Thread-local text of the last error returned on this thread ("" if none). */
const char *fl_last_error(void);

/* Backward passes started after this call do (non-zero, the default) or do not (0) run the
 * parameter-gradient kernels -- bias sums, the dW contractions and the second stages of their
 * reductions -- on a library-owned side stream beside the input-gradient chain (Section 4.1.3: the
 * backward pass is a reverse replay of the recorded graph; kernels of independent branches of that
 * graph may run at the same time).  The side stream waits, through events, for the gradients it
 * reads, and the caller's stream waits for it before fl_layer_backward returns control of dX and
 * the gradient buffers to work enqueued later on that stream: the caller sees the same ordering
 * either way, and the results are bit-identical.  Small problems (B*T*d_model < 2^18) always stay on
 * one stream.  The same switch decides where forward writes the transposed weight copies it leaves for
 * its backward (bf16 layers of middling size): on the side stream, or in order on the caller's.
 * Process-wide; a call that is already inside forward or backward when the switch changes may see
 * either setting for its remaining operators (both are correct).
 *
 * Graph capture: once calls with the same sizes have warmed the allocator's cache (so that no device
 * allocation happens), fl_layer_forward + fl_layer_backward on a capturing stream record a valid
 * graph -- the side streams enter the capture through the fork events and leave it at the join --
 * and replays reproduce the eager results bit for bit.  Timing (fl_prof_enable) must be off. */
fl_status_t fl_set_grad_overlap(int32_t enabled);

/* Deferred join, for stacks of layers (Section 4.2: a model is a sequence of modules whose backward
 * passes run one after the other).  With it enabled (non-zero; default 0) fl_layer_backward no longer
 * makes the caller's stream wait for the side stream before it returns: dX is complete in stream order
 * as always (the input-gradient chain never leaves the caller's stream), so the backward pass of the
 * layer below can start while this layer's last parameter-gradient kernels still run, but the buffers
 * in `grads` are complete only after fl_layer_join(layer, stream), which makes `stream` (and the stream
 * the layer ran on) wait for them.  The next fl_layer_forward on the handle and fl_layer_destroy join
 * by themselves.  Until the join, the layer keeps the activations its side-stream kernels read, and the
 * caller keeps X unchanged (a post-LN layer's last weight-gradient kernel reads it).  dY is free for reuse
 * in stream order as soon as fl_layer_backward has returned: the caller's stream waits for the side-stream
 * kernels that read it (the first ones of the pass), so a stack may alternate between two gradient buffers.
 * Without a side stream (small problems, fl_set_grad_overlap(0)) nothing is deferred and the join is a
 * no-op.  Results are bit-identical either way.  Do not enable it under graph capture unless the
 * captured region contains the join. */
fl_status_t fl_layer_set_deferred_join(fl_layer_t *layer, int32_t enabled);
fl_status_t fl_layer_join(fl_layer_t *layer, void *hip_stream);

/* Caching device allocator telemetry (Section 4.1.2; Section 5.2.2 describes
 * size-bucketed caches, block splitting and allocation telemetry).
 * backing_mallocs / backing_bytes: calls to and bytes obtained from the device
 * allocator so far; cache_hits / cache_misses: requests served from / not from
 * cached blocks; live_bytes: bytes handed out now; peak_bytes: its maximum;
 * cached_bytes: bytes held in free blocks; split_count: blocks split so far;
 * requested_bytes: what the live blocks were asked for before rounding, so
 * 1 - requested_bytes/live_bytes is the internal fragmentation;
 * largest_free_block / free_blocks: size of the largest and number of cached
 * blocks, so 1 - largest_free_block/cached_bytes is the share of the cache that
 * no single request can use (external fragmentation). */
typedef struct {
  uint64_t backing_mallocs, backing_bytes, cache_hits, cache_misses;
  uint64_t live_bytes, peak_bytes, cached_bytes, split_count;
  uint64_t requested_bytes, largest_free_block, free_blocks;
} fl_alloc_stats_t;
fl_status_t fl_alloc_get_stats(fl_alloc_stats_t *out);

/* Allocation trace (Section 5.2.2: telemetry that ties individual tensor
 * operations to specific allocations).  While enabled, every request to and
 * release into the allocator is recorded in a ring of `capacity` events
 * (the oldest are overwritten; capacity 0 switches the trace off; at most 2^20).
 * tag = (position of the operator on the layer's tape << 8) | fl_op_kind_t; the
 * release of a block carries the tag it was allocated with.
 * fl_alloc_trace_read moves up to cap of the oldest events into the host array
 * `out` and stores their number in *n. */
typedef enum {
  FL_OP_NONE = 0,
  FL_OP_LINEAR_FWD = 1,
  FL_OP_ATTENTION_FWD = 2,
  FL_OP_LAYERNORM_FWD = 3,
  FL_OP_LINEAR_BWD = 4,
  FL_OP_ATTENTION_BWD = 5,
  FL_OP_LAYERNORM_BWD = 6
} fl_op_kind_t;
typedef enum { FL_ALLOC_FROM_CACHE = 0, FL_ALLOC_FROM_DEVICE = 1, FL_ALLOC_RELEASE = 2 } fl_alloc_event_kind_t;
typedef struct {
  uint64_t seq;       /* running number of the event                          */
  uint64_t ptr;       /* device address handed out / given back               */
  uint64_t requested; /* bytes asked for (0 for a release)                    */
  uint64_t granted;   /* size of the block                                    */
  int32_t tag;        /* see above                                            */
  int32_t kind;       /* fl_alloc_event_kind_t                                */
} fl_alloc_event_t;
fl_status_t fl_alloc_trace_enable(int32_t capacity);
fl_status_t fl_alloc_trace_read(fl_alloc_event_t *out, int32_t cap, int32_t *n);

/* Returns every cached (free) slab to the device.  Synchronises the device. */
fl_status_t fl_alloc_trim(void);

/* Blocks larger than `bytes` are never split to serve a smaller request
 * (Section 5.2.2: restricting the splitting of large cache blocks reduced
 * fragmentation).  0 restores the default (no limit). */
fl_status_t fl_alloc_set_split_limit(uint64_t bytes);

/* ---- optimizer step (Section 4.2 "Optimizers"; the training-loop listing's opt.step() and
 * opt.zeroGrad()).  One fused kernel updates up to 16 tensors:
 *   SGD   g' = g + wd*p;  buf = momentum*buf + g';  p -= lr*buf      (momentum == 0: p -= lr*g')
 *   Adam  g' = g + wd*p;  m = b1*m + (1-b1)*g';  v = b2*v + (1-b2)*g'^2;
 *         p -= lr * (m/(1-b1^step)) / (sqrt(v/(1-b2^step)) + eps),   step = 1 for the first update
 * params[i] / grads[i]: device tensors of `dtype` with numel[i] elements (numel % 8 == 0, pointers
 * 16-byte aligned).  state_m[i] (SGD momentum buffer / Adam m) and state_v[i] (Adam v) are device
 * fp32 buffers of numel[i] elements owned by the caller, zero before the first step; state_m may
 * be NULL for SGD without momentum, state_v for SGD.  The pointer arrays themselves are HOST
 * arrays.  Arithmetic is fp32; a bf16 parameter is rounded once when it is written back, and no
 * higher-precision copy is kept: over many small steps that rounding accumulates (see fl_opt_step_master). */
typedef enum { FL_OPT_SGD = 0, FL_OPT_ADAM = 1 } fl_opt_kind_t;
typedef struct {
  fl_opt_kind_t kind;
  float lr, momentum, weight_decay, beta1, beta2, eps;
  int32_t step;
} fl_opt_config_t;
fl_status_t fl_opt_step(const fl_opt_config_t *cfg, fl_dtype_t dtype, int32_t n, void *const *params,
                        const void *const *grads, float *const *state_m, float *const *state_v, const int64_t *numel,
                        void *hip_stream);
/* The same step with full-precision master copies (Section 4.2: the optimizers act on the parameters' tensors;
 * with bf16 storage a parameter of magnitude 0.02 has a spacing of 6e-5, so updates of the order lr = 1e-4 and
 * below are largely rounded away when the bf16 value itself carries them).  master[i]: device fp32 buffer
 * of numel[i] elements owned by the caller, initialised with the parameter's values, or NULL for a tensor
 * without one (`master` itself may be NULL: then this is fl_opt_step).  Where given, the update reads and
 * writes the master copy and params[i] receives its value rounded to `dtype`; 8 more bytes of traffic per
 * element. */
fl_status_t fl_opt_step_master(const fl_opt_config_t *cfg, fl_dtype_t dtype, int32_t n, void *const *params,
                               float *const *master, const void *const *grads, float *const *state_m,
                               float *const *state_v, const int64_t *numel, void *hip_stream);
/* Sets n gradient tensors to zero with one kernel (safe inside a captured graph). */
fl_status_t fl_zero_grad(fl_dtype_t dtype, int32_t n, void *const *grads, const int64_t *numel, void *hip_stream);

/* ---- per-kernel timing telemetry (host-side; used by the benchmark) -------------
 * While enabled, launches of the selected kernel classes are bracketed by HIP
 * events on the caller's stream.  fl_prof_collect() synchronises those events
 * and fills `out` (host array of `cap` entries) with one entry per kernel class
 * seen: launches, total milliseconds, algorithmic flops and bytes summed over
 * the launches, and empty_bracket_ms: what a pair of events reads on that stream
 * with no kernel between them (the same figure in every entry; each bracket's
 * reading exceeds its kernel's duration by about this much).  Returns the number
 * of entries through *n. */
typedef enum {
  FL_K_GEMM_NT = 0,   /* y = x W^T (+bias, +activation, +residual); also dx  */
                      /* where forward left a transposed copy of W behind    */
  FL_K_GEMM_NN = 1,   /* dx = dy W (+activation derivative, +skip gradient)  */
  FL_K_GEMM_TN = 2,   /* dW = dy^T x (split over the token dimension)        */
  FL_K_SPLITK_REDUCE = 3,
  FL_K_ATTN_FWD = 4,
  FL_K_ATTN_BWD = 5,
  FL_K_LN_FWD = 6,
  FL_K_LN_BWD = 7,
  FL_K_COLSUM = 8,    /* bias gradients and second-stage column reductions   */
  FL_K_TRANSPOSE = 9, /* transposed weight copies made by forward            */
  FL_K_CLASS_COUNT = 10
} fl_kernel_class_t;
typedef struct {
  int32_t kernel_class;
  int32_t launches;
  double total_ms, flops, bytes, empty_bracket_ms;
} fl_prof_entry_t;
fl_status_t fl_prof_enable(uint32_t class_mask); /* bit i = class i; 0 disables and drops pending events */
fl_status_t fl_prof_collect(fl_prof_entry_t *out, int32_t cap, int32_t *n);

#ifdef __cplusplus
}
#endif
#endif /* FL_LAYER_H */
