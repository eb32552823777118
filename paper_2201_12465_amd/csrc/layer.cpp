// Encoder-layer orchestration and the C ABI declared in include/fl_layer.h.
//
// forward() is the paper's Module::forward (Section 4.2): it runs the fused
// operators in order, takes every intermediate buffer from the caching allocator
// (Section 4.1.2) and records one tape node per operator.  backward() is the
// paper's Variable::backward(): the tape is replayed in reverse and each node's
// gradient function adds into its inputs' gradients (Section 4.2, the
// cosine-operator listing).  Adding is fused into the producing kernel's
// epilogue wherever two gradient contributions meet (the residual connections),
// and requests attached to a slot let the kernel that finishes a gradient also
// apply the activation derivative or emit a bias gradient (Section 5.2.1,
// pre-fused gradient computation for common sequences).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/fl_layer.h"
#include "allocator.h"
#include "kernels.h"
#include "runtime.h"
#include "static_scratch.h"
#include "tape.h"

using namespace fl;

// ------------------------------------------------------------------ errors
namespace {
thread_local char g_err[512] = "";
}
namespace fl {
int set_error(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
}  // namespace fl

// ------------------------------------------------------------------ allocator instance
namespace {
// What the device allocator answered the last time it refused a request on this thread: the
// out-of-memory message of the layer carries it, so that a log tells a full device from a failed call.
thread_local hipError_t g_backing_error = hipSuccess;
thread_local size_t g_backing_bytes = 0;
int hip_backing_malloc(void **p, size_t bytes) {
  hipError_t e = hipMalloc(p, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();  // clear the sticky out-of-memory code
    g_backing_error = e;
    g_backing_bytes = bytes;
    *p = nullptr;
    return 1;
  }
  return 0;
}
int hip_backing_free(void *p) { return hipFree(p) == hipSuccess ? 0 : 1; }
}  // namespace
namespace fl {
CachingAllocator &device_allocator() {
  static CachingAllocator *a = new CachingAllocator(hip_backing_malloc, hip_backing_free);  // never destroyed
  return *a;
}
}  // namespace fl

// ------------------------------------------------------------------ per-kernel timing
namespace {
struct ProfEvent {
  hipEvent_t a, b;
  int cls;
  double flops, bytes;
};
struct Prof {
  std::mutex mu;
  uint32_t mask = 0;
  std::vector<ProfEvent> pending;
  std::vector<hipEvent_t> pool;
  hipStream_t last_stream = nullptr;
  hipEvent_t get() {
    if (!pool.empty()) {
      hipEvent_t e = pool.back();
      pool.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};
Prof &prof() {
  static Prof *p = new Prof();
  return *p;
}
}  // namespace

namespace fl {
// Set while this thread runs the allocation-free forward: nothing may create an event or take device memory.
thread_local bool g_no_alloc = false;
// Runs `launch` (which enqueues one kernel class on `s`), bracketed by events when that class is selected.
template <typename F>
hipError_t timed(int cls, double flops, double bytes, hipStream_t s, F &&launch) {
  Prof &P = prof();
  if (g_no_alloc || !(P.mask & (1u << cls))) return launch();
  std::lock_guard<std::mutex> g(P.mu);
  ProfEvent ev{P.get(), P.get(), cls, flops, bytes};
  if (!ev.a || !ev.b) return hipErrorOutOfMemory;
  hipError_t e = hipEventRecord(ev.a, s);
  if (e != hipSuccess) return e;
  e = launch();
  if (e != hipSuccess) return e;
  e = hipEventRecord(ev.b, s);
  if (e != hipSuccess) return e;
  P.pending.push_back(ev);
  P.last_stream = s;
  return hipSuccess;
}
}  // namespace fl

// ------------------------------------------------------------------ the layer
enum ParamId { P_WQKV, P_BQKV, P_WO, P_BO, P_W1, P_B1, P_W2, P_B2, P_LN1G, P_LN1B, P_LN2G, P_LN2B, P_COUNT };
enum OpId { OP_LINEAR = 1, OP_ATTN = 2, OP_LN = 3 };

struct fl_layer {
  fl_layer_config_t cfg;
  float eps;
  int dt;
  Tape tape;
  // state of the recorded forward
  int B = 0, T = 0, M = 0;
  hipStream_t stream = nullptr;
  const int32_t *lengths = nullptr;
  int slot_x = -1, slot_y = -1;
  // dropout: what the next forward will use, and what the recorded forward used (its backward needs the same)
  float p_attn = 0.f, p_hidden = 0.f;
  uint64_t seed = 0;
  float rec_p_attn = 0.f, rec_p_hidden = 0.f;
  uint64_t rec_seed = 0;
  // valid during backward
  bool accumulate = false;  // parameter gradients are added to what the caller's buffers hold
  // Parameter-gradient work (bias sums, dW GEMMs, second-stage reductions) is enqueued on a side
  // stream so that it runs beside the input-gradient chain; see side_mark(), side_begin(), side_join().
  hipStream_t side = nullptr;          // non-null while this backward uses the side stream
  std::vector<hipEvent_t> fork_events; // one per fork, reused by the next backward
  size_t forks = 0;
  hipEvent_t join_event = nullptr;
  hipEvent_t attn_join_event = nullptr;  // dK/dV kernels on the second side stream -> layer's stream
  std::vector<Buf *> held;             // buffers the side stream reads: released after the join
  bool defer_join = false;             // backward leaves the join to fl_layer_join() / the next call on the layer
  bool join_pending = false;           // a backward has ended without the join: join_event marks its side-stream work
  // Deferred join: side-stream kernels that read the CALLER's dY.  The layer's stream waits for them before
  // backward returns (they are the first parameter-gradient kernels of the pass and long done by then), so
  // that the caller may reuse dY's memory in stream order as soon as backward has returned.
  hipEvent_t caller_read_event = nullptr;
  bool caller_read_pending = false;
  // Transposed copies of Wqkv, Wo, W1, W2 (in kLinear order), made by forward for the input-gradient
  // GEMMs of its backward; see wt_make(), wt_acquire(), wt_release().
  Buf *wt[4] = {nullptr, nullptr, nullptr, nullptr};
  hipEvent_t wt_fork_event = nullptr, wt_event = nullptr;
  bool wt_on_side = false;             // made on the side stream, and the layer's stream has not waited yet
  // Second stages of the backward pass's two-stage reductions (split weight gradients, LayerNorm sums, bias
  // sums): collected while the tape is replayed and run as ONE launch at the end of the parameter-gradient
  // lane; the partial buffers are kept until then.
  std::vector<ReduceJob> reduce_jobs;
  std::vector<Buf *> reduce_bufs;
  std::vector<char> reduce_job_main;   // per job: its partial sums were written on the layer's stream
  // The pass's last linear operator (see linear_backward): where the side stream stood when its work began.
  int tail_node = -1;                  // tape index of that operator; -1 = the pass does not split its tail
  bool tail_split = false;
  size_t tail_jobs = 0;                // second stages collected before that point
  hipEvent_t tail_event = nullptr;     // recorded on the side stream at that point
  hipStream_t reduce_stream = nullptr;
  bool reduce_has_side = false;        // some collected job's partial sums were written on the side stream
  bool reduce_from_main = false;       // some collected job's partial sums were written on the layer's stream
                                       // after the last fork: the side stream has not been told to wait for them
  // Every fork puts a barrier on the layer's stream (the recorded event), a few microseconds in which the
  // input-gradient chain stands still.  The first linear operator replayed therefore does not fork: its
  // parameter-gradient work waits here for the next operator's fork and runs in front of that one's.
  std::vector<std::function<int(hipStream_t)>> pending_side;
  bool inference = false;              // forward keeps nothing for a backward pass (no pre-activation copy)
  const void *params[P_COUNT];
  void *grads[P_COUNT];
};

namespace {

#define FL_HIP(expr)                                                                      \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess)                                                                 \
      return set_error(e_ == hipErrorInvalidValue ? FL_ERR_UNSUPPORTED : FL_ERR_DEVICE,   \
                       "%s failed: %s", #expr, hipGetErrorString(e_));                    \
  } while (0)
// First-fit allocator over the static scratch array, host-side bookkeeping only.  It lives for one call of
// the allocation-free forward: every kernel of that call runs on one stream, so a range may be handed out
// again as soon as its last reader has been enqueued.
struct Arena {
  struct Range {
    size_t off, size;
    bool free;
  };
  unsigned char *base = nullptr;
  std::vector<Range> ranges;
  size_t live = 0, peak = 0;
  Arena(void *b, size_t bytes) : base(static_cast<unsigned char *>(b)) { ranges.push_back({0, bytes, true}); }
  void *alloc(size_t bytes) {
    const size_t need = (bytes + 255) / 256 * 256;
    for (size_t i = 0; i < ranges.size(); ++i) {
      if (!ranges[i].free || ranges[i].size < need) continue;
      const size_t rest = ranges[i].size - need;
      ranges[i].size = need;
      ranges[i].free = false;
      if (rest) ranges.insert(ranges.begin() + i + 1, Range{ranges[i].off + need, rest, true});
      live += need;
      if (live > peak) peak = live;
      return base + ranges[i].off;
    }
    return nullptr;
  }
  void release(void *p) {
    const size_t off = static_cast<unsigned char *>(p) - base;
    for (size_t i = 0; i < ranges.size(); ++i) {
      if (ranges[i].off != off || ranges[i].free) continue;
      ranges[i].free = true;
      live -= ranges[i].size;
      if (i + 1 < ranges.size() && ranges[i + 1].free) {
        ranges[i].size += ranges[i + 1].size;
        ranges.erase(ranges.begin() + i + 1);
      }
      if (i > 0 && ranges[i - 1].free) {
        ranges[i - 1].size += ranges[i].size;
        ranges.erase(ranges.begin() + i);
      }
      return;
    }
  }
};
thread_local Arena *g_arena = nullptr;  // non-null while this thread runs the allocation-free forward

// A request for device memory failed: says what was asked for and what the device allocator answered.
int oom_error(size_t bytes) {
  if (g_arena)
    return set_error(FL_ERR_UNSUPPORTED,
                     "the intermediates of this forward pass do not fit the static scratch: %zu more bytes wanted with "
                     "%zu of %zu in use; use fl_layer_forward, or fewer tokens per call",
                     bytes, g_arena->live, (size_t)kStaticScratchBytes);
  if (g_backing_error != hipSuccess) {
    const hipError_t e = g_backing_error;
    g_backing_error = hipSuccess;
    return set_error(FL_ERR_OOM, "device allocation of %zu bytes failed: hipMalloc(%zu) returned %s (%s)", bytes,
                     g_backing_bytes, hipGetErrorName(e), hipGetErrorString(e));
  }
  return set_error(FL_ERR_OOM, "device allocation of %zu bytes failed", bytes);
}
#define FL_TRY(expr)        \
  do {                      \
    int rc_ = (expr);       \
    if (rc_) return rc_;    \
  } while (0)

// Operator on whose behalf this thread allocates right now: (tape position << 8) | fl_op_kind_t.
thread_local int g_op_tag = 0;
struct OpTag {
  int saved;
  OpTag(int kind, int node) : saved(g_op_tag) { g_op_tag = (node << 8) | kind; }
  ~OpTag() { g_op_tag = saved; }
};

// FL_DEBUG=1 in the environment (read at every forward call) switches on the validating mode: key-padding
// lengths are copied to the host and checked (this synchronises the stream), and every block the allocator
// hands out is first filled with NaN bit patterns, so that a kernel reading what nobody wrote, or a block
// reused too early, shows up as NaN in the results instead of as plausible stale numbers.
bool g_debug = false;
bool debug_from_env() {
  const char *v = getenv("FL_DEBUG");
  return v && v[0] && !(v[0] == '0' && !v[1]);
}

Buf *buf_new(size_t bytes, hipStream_t s) {
  if (g_arena) {
    void *p = g_arena->alloc(bytes);
    Buf *b = p ? new (std::nothrow) Buf() : nullptr;
    if (!b) {
      if (p) g_arena->release(p);
      return nullptr;
    }
    b->ptr = p;
    b->bytes = bytes;
    b->refs = 1;
    b->from_arena = true;
    return b;
  }
  void *p = device_allocator().alloc(bytes, s, g_op_tag);
  if (!p) return nullptr;
  if (g_debug) {  // blocks are handed out in units of 512 bytes: rounding up to 16 stays inside the block
    if (launch_fill_words(p, (bytes + 15) / 16 * 16, 0xFFFFFFFFu, s) != hipSuccess) {
      device_allocator().release(p);
      return nullptr;
    }
  }
  Buf *b = new (std::nothrow) Buf();
  if (!b) {
    device_allocator().release(p);
    return nullptr;
  }
  b->ptr = p;
  b->bytes = bytes;
  b->refs = 1;
  return b;
}
void buf_unref(Buf *&b) {
  if (b && --b->refs == 0) {
    if (b->from_arena) {
      if (g_arena) g_arena->release(b->ptr);  // the arena is gone with its call otherwise
    } else {
      device_allocator().release(b->ptr);
    }
    delete b;
  }
  b = nullptr;
}
// Scratch that lives for the kernels enqueued in one scope: released to the cache at scope
// exit, which is safe because the cache only hands it out again for later work on this stream.
struct Scratch {
  Buf *b = nullptr;
  ~Scratch() { buf_unref(b); }
  int get(size_t bytes, hipStream_t s) {
    b = buf_new(bytes, s);
    return b ? 0 : oom_error(bytes);
  }
  float *f32() { return static_cast<float *>(b->ptr); }
};

// ---- side stream ---------------------------------------------------------------------------
// One stream per process, default priority, never destroyed.  It has no implicit ordering with
// any other stream: every dependency is an event.
std::atomic<bool> g_overlap{true};
// Events that order this library's streams among themselves on one device: no timing and no
// system-scope fence.  By default a recorded event also makes device memory visible to the host and to
// other devices, and that cache write-back delays the kernels behind every record; kernel boundaries
// already order memory within the device, which is all these events are for (the caller's own
// synchronisation with the host is untouched).  Measured: 0.429 -> 0.419 ms per step.
constexpr unsigned kEventFlags = hipEventDisableTiming | hipEventDisableSystemFence;
hipStream_t make_side_stream() {
  hipStream_t t = nullptr;
  if (hipStreamCreateWithFlags(&t, hipStreamNonBlocking) != hipSuccess) t = nullptr;
  return t;
}
hipStream_t side_stream() {
  static hipStream_t s = make_side_stream();
  return s;
}
// A second one for the dK/dV kernels of the attention backward, which run beside the dQ kernel: on the
// first side stream they would queue up behind the weight-gradient GEMMs.
hipStream_t side_stream2() {
  static hipStream_t s = make_side_stream();
  return s;
}
// Fork in two steps, so that the host can enqueue the next kernel of the critical path on the layer's
// stream BETWEEN them (enqueueing costs the host a few microseconds per call, and the GPU would wait):
// side_mark() records "everything enqueued on the layer's stream so far" in an event; side_begin()
// makes the side stream wait for that point and returns the stream to launch the parameter-gradient
// kernels on (the layer's own stream when overlap is off).
int side_mark(fl_layer *L, hipEvent_t *ev) {
  *ev = nullptr;
  if (!L->side) return 0;
  if (L->forks == L->fork_events.size()) {
    hipEvent_t e = nullptr;
    FL_HIP(hipEventCreateWithFlags(&e, kEventFlags));
    L->fork_events.push_back(e);
  }
  *ev = L->fork_events[L->forks++];
  FL_HIP(hipEventRecord(*ev, L->stream));
  return 0;
}
int side_begin(fl_layer *L, hipEvent_t ev, hipStream_t *out) {
  *out = L->stream;
  if (!L->side) return 0;
  FL_HIP(hipStreamWaitEvent(L->side, ev, 0));
  *out = L->side;
  L->reduce_from_main = false;  // whatever the layer's stream wrote before the event is ordered now
  return 0;
}
// A buffer that kernels on the side stream read must not go back to the cache of the layer's stream
// (where later kernels could overwrite it) before the join.
void side_hold(fl_layer *L, Buf *b) {
  if (!L->side || !b) return;
  b->refs++;
  L->held.push_back(b);
}
// The layer's stream waits for the side stream; afterwards the held buffers may be reused.
// wait_host: on an error path, where the order of what was enqueued is no longer known.
int side_join(fl_layer *L, bool wait_host, bool defer = false) {
  int rc = 0;
  const bool caller_read = L->caller_read_pending;
  L->caller_read_pending = false;
  if (defer && !wait_host && L->side && L->forks) {
    // Only mark the end of this backward's side-stream work; the held buffers stay held until
    // finish_pending_join().  (A failure to record falls through to the immediate join.)
    hipError_t e = hipSuccess;
    if (!L->join_event) e = hipEventCreateWithFlags(&L->join_event, kEventFlags);
    if (e == hipSuccess) e = hipEventRecord(L->join_event, L->side);
    if (e == hipSuccess && caller_read) e = hipStreamWaitEvent(L->stream, L->caller_read_event, 0);
    if (e == hipSuccess) {
      L->join_pending = true;
      L->forks = 0;
      L->side = nullptr;
      return 0;
    }
  }
  if (L->side && L->forks) {
    if (wait_host) {
      hipStreamSynchronize(L->side);
    } else {
      hipError_t e = hipSuccess;
      if (!L->join_event) e = hipEventCreateWithFlags(&L->join_event, kEventFlags);
      if (e == hipSuccess) e = hipEventRecord(L->join_event, L->side);
      if (e == hipSuccess) e = hipStreamWaitEvent(L->stream, L->join_event, 0);
      if (e != hipSuccess) {
        hipStreamSynchronize(L->side);
        rc = set_error(FL_ERR_DEVICE, "joining the side stream failed: %s", hipGetErrorString(e));
      }
    }
  }
  for (Buf *&b : L->held) buf_unref(b);
  L->held.clear();
  L->forks = 0;
  L->side = nullptr;
  return rc;
}

// Completes a join that backward left open: the layer's stream (whose cache the held buffers return to)
// waits for the marked point of the side stream, and so does `also` when it is another stream.  Where a
// stream cannot wait (wait_host: destroy and error paths; or the caller has destroyed the stream since),
// the host waits instead, as wt_release() does.
int finish_pending_join(fl_layer *L, hipStream_t also, bool wait_host) {
  if (L->join_pending) {
    bool ordered = !wait_host && hipStreamWaitEvent(L->stream, L->join_event, 0) == hipSuccess &&
                   (also == L->stream || hipStreamWaitEvent(also, L->join_event, 0) == hipSuccess);
    if (!ordered) {
      (void)hipGetLastError();
      if (hipEventSynchronize(L->join_event) != hipSuccess) hipStreamSynchronize(side_stream());
    }
    L->join_pending = false;
  }
  for (Buf *&b : L->held) buf_unref(b);
  L->held.clear();
  return 0;
}

// The transposed weights go back to the cache of the layer's stream: if they were written on the side
// stream and nobody has waited for that yet, the layer's stream (or, when it may no longer exist, the
// host) waits first, so that whatever the cache hands the memory to next is ordered after the writes.
void wt_release(fl_layer *L, bool host_wait) {
  if (L->wt_on_side) {
    if (host_wait || hipStreamWaitEvent(L->stream, L->wt_event, 0) != hipSuccess) hipEventSynchronize(L->wt_event);
    L->wt_on_side = false;
  }
  for (Buf *&b : L->wt) buf_unref(b);
}

void release_tape(fl_layer *L, bool host_wait = false) {
  wt_release(L, host_wait);
  for (Slot &s : L->tape.slots) {
    buf_unref(s.value_buf);
    buf_unref(s.grad_buf);
  }
  for (Node &n : L->tape.nodes)
    for (Buf *&b : n.saved) buf_unref(b);
  L->tape.clear();
}

size_t esize(const fl_layer *L) { return dt_size(L->dt); }

// Replaces a slot's accumulated gradient.
void set_grad(Slot &s, void *ptr, Buf *buf) {
  buf_unref(s.grad_buf);
  s.grad = ptr;
  s.grad_buf = buf;
}

struct LinearShape {
  int w, b;  // parameter ids
};
const LinearShape kLinear[4] = {{P_WQKV, P_BQKV}, {P_WO, P_BO}, {P_W1, P_B1}, {P_W2, P_B2}};

// ---- transposed weight copies ----------------------------------------------------------------
// dx = dy W contracts over the rows of W [out, in].  With bf16 operands the GEMM kernels are fastest
// when the contraction index is contiguous in both operands (direct-to-LDS staging, 16-byte fragment
// reads), so forward leaves W^T [in, out] of the four weight matrices behind for its backward: one
// launch, on the side stream while that is idle (forward has no other use for it), else on the layer's
// stream.  Small problems, very large ones (see below) and fp32 keep the general path.
int wt_make(fl_layer *L) {
  const int D = L->cfg.d_model, F = L->cfg.d_ffn;
  if (L->dt != DT_BF16 || (long)L->M * D < (1l << 18) || D % 64 || F % 64) return 0;
  // Measured: with more than about 512 output tiles of 128 x 128 in the d_model-wide gradients the general
  // kernel is as fast on W as the pipelined one on W^T, and the copies only cost their own time.
  if ((long)((L->M + 127) / 128) * ((D + 127) / 128) > 512) return 0;
  OpTag tag(FL_OP_LINEAR_FWD, 0);
  const int rows[4] = {3 * D, D, F, D}, cols[4] = {D, D, D, F};
  const void *src[4];
  void *dst[4];
  double bytes = 0;
  for (int i = 0; i < 4; ++i) {
    const size_t nb = (size_t)rows[i] * cols[i] * esize(L);
    L->wt[i] = buf_new(nb, L->stream);
    if (!L->wt[i]) {
      wt_release(L, false);
      return oom_error(nb);
    }
    src[i] = L->params[kLinear[i].w];
    dst[i] = L->wt[i]->ptr;
    bytes += 2.0 * nb;
  }
  hipStream_t s = L->stream;
  hipStream_t side = g_overlap ? side_stream() : nullptr;
  hipError_t he = hipSuccess;
  if (side) {  // the parameters (and the memory just taken from the cache) are ready at this point of the layer's stream
    if (!L->wt_fork_event) he = hipEventCreateWithFlags(&L->wt_fork_event, kEventFlags);
    if (he == hipSuccess && !L->wt_event) he = hipEventCreateWithFlags(&L->wt_event, kEventFlags);
    if (he == hipSuccess) he = hipEventRecord(L->wt_fork_event, L->stream);
    if (he == hipSuccess) he = hipStreamWaitEvent(side, L->wt_fork_event, 0);
    s = side;
  }
  if (he == hipSuccess)
    he = timed(FL_K_TRANSPOSE, 0, bytes, s, [&] { return launch_transpose_bf16(4, src, dst, rows, cols, s); });
  if (he == hipSuccess && side) {
    he = hipEventRecord(L->wt_event, side);
    L->wt_on_side = he == hipSuccess;
  }
  if (he != hipSuccess) {
    if (side) hipStreamSynchronize(side);
    wt_release(L, false);
    FL_HIP(he);
  }
  return 0;
}
// Before the layer's stream reads the copies.
int wt_acquire(fl_layer *L) {
  if (L->wt_on_side) {
    FL_HIP(hipStreamWaitEvent(L->stream, L->wt_event, 0));
    L->wt_on_side = false;
  }
  return 0;
}

// ---- batched second stages ---------------------------------------------------------------
// Every job's partial sums are produced on `ps` (or, for the LayerNorm sums, made visible to it by a fork)
// before anything enqueued later on `ps`: the batch launched at the end of the pass is ordered after them.
int reduce_flush(fl_layer *L) {
  int rc = 0;
  if (!L->reduce_jobs.empty()) {
    hipStream_t ps = L->reduce_stream;
    if (L->reduce_from_main && ps != L->stream) {
      if (!L->reduce_has_side) {
        ps = L->stream;  // every partial sum was written on the layer's stream: reduce there, in order
      } else {           // make the side stream wait for what the layer's stream wrote
        hipEvent_t ev;
        rc = side_mark(L, &ev);
        if (!rc) rc = side_begin(L, ev, &ps);
      }
    }
    if (!rc) {
      double bytes = 0;
      for (const ReduceJob &j : L->reduce_jobs) bytes += (double)(j.P * 4 + esize(L)) * j.seglen * j.nseg;
      hipError_t he = timed(FL_K_SPLITK_REDUCE, 0, bytes, ps, [&] {
        return launch_reduce_batch(L->dt, L->reduce_jobs.data(), (int)L->reduce_jobs.size(), ps, L->accumulate);
      });
      if (he != hipSuccess)
        rc = set_error(FL_ERR_DEVICE, "the batched second-stage reduction failed: %s", hipGetErrorString(he));
    }
  }
  for (Buf *&b : L->reduce_bufs) buf_unref(b);   // back to the cache of the stream that has just read them
  L->reduce_bufs.clear();
  L->reduce_jobs.clear();
  L->reduce_job_main.clear();
  L->reduce_from_main = false;
  L->reduce_has_side = false;
  L->tail_split = false;   // a flush in the middle of the pass: the tail is no longer what was counted
  return rc;
}
// The end of a pass whose last linear operator marked the side stream (tail_split): the second stages
// collected before the mark, and those whose partial sums the layer's stream wrote itself, run on the
// LAYER's stream -- which has nothing left to do while the side stream still works on that operator's
// weight gradient -- and only the rest behind that weight gradient on the side stream.  Same kernel,
// same summation order: which launch a job is part of does not change its result.
int reduce_flush_split(fl_layer *L) {
  std::vector<ReduceJob> on_main, on_side;
  for (size_t i = 0; i < L->reduce_jobs.size(); ++i)
    (i < L->tail_jobs || L->reduce_job_main[i] ? on_main : on_side).push_back(L->reduce_jobs[i]);
  int rc = 0;
  auto launch = [&](std::vector<ReduceJob> &jobs, hipStream_t ps) {
    for (size_t at = 0; at < jobs.size() && !rc; at += REDUCE_MAX_JOBS) {
      const int n = (int)std::min<size_t>(REDUCE_MAX_JOBS, jobs.size() - at);
      double bytes = 0;
      for (int k = 0; k < n; ++k) bytes += (double)(jobs[at + k].P * 4 + esize(L)) * jobs[at + k].seglen * jobs[at + k].nseg;
      hipError_t he = timed(FL_K_SPLITK_REDUCE, 0, bytes, ps,
                            [&] { return launch_reduce_batch(L->dt, jobs.data() + at, n, ps, L->accumulate); });
      if (he != hipSuccess)
        rc = set_error(FL_ERR_DEVICE, "the batched second-stage reduction failed: %s", hipGetErrorString(he));
    }
  };
  if (!on_main.empty()) {
    hipError_t he = hipStreamWaitEvent(L->stream, L->tail_event, 0);
    if (he != hipSuccess) rc = set_error(FL_ERR_DEVICE, "waiting for the side stream failed: %s", hipGetErrorString(he));
    if (!rc) launch(on_main, L->stream);
  }
  if (!rc) launch(on_side, L->side);
  // the partial sums came from either stream's cache and were read on either stream: they go back after the join
  for (Buf *&b : L->reduce_bufs) L->held.push_back(b);
  L->reduce_bufs.clear();
  L->reduce_jobs.clear();
  L->reduce_job_main.clear();
  L->reduce_from_main = false;
  L->reduce_has_side = false;
  L->tail_split = false;
  return rc;
}
// ps: the stream the batch will run on (the side stream while there is one).  from_main: the partial sums were
// written by a kernel on the layer's stream that no fork has covered yet.
int reduce_later(fl_layer *L, hipStream_t ps, bool from_main, Buf *partial, int P, size_t stride, size_t seglen,
                 int nseg, void *o0, void *o1, void *o2) {
  if (!L->reduce_jobs.empty() && (L->reduce_stream != ps || (int)L->reduce_jobs.size() == REDUCE_MAX_JOBS))
    FL_TRY(reduce_flush(L));
  L->reduce_stream = ps;
  if (from_main && ps != L->stream) L->reduce_from_main = true;
  if (!from_main && ps != L->stream) L->reduce_has_side = true;
  ReduceJob j;
  j.partial = static_cast<const float *>(partial->ptr);
  j.P = P; j.nseg = nseg; j.stride = stride; j.seglen = seglen;
  j.out[0] = o0; j.out[1] = o1; j.out[2] = o2;
  L->reduce_jobs.push_back(j);
  L->reduce_job_main.push_back(from_main ? 1 : 0);
  partial->refs++;
  L->reduce_bufs.push_back(partial);
  return 0;
}
int run_pending_side(fl_layer *L, hipStream_t ps) {
  int rc = 0;
  for (auto &f : L->pending_side)
    if (!rc) rc = f(ps);
  L->pending_side.clear();
  return rc;
}

// ---- gradient functions ---------------------------------------------------------------


// y = x W^T + b (+act) (+residual):  db = colsum(gy), dW = gy^T x, dx += gy W, dresidual += gy.
int linear_backward(void *ctx, Tape *tape, const Node *n) {
  fl_layer *L = static_cast<fl_layer *>(ctx);
  const int self = tape->index_of(n);
  OpTag tag(FL_OP_LINEAR_BWD, self);
  hipStream_t st = L->stream;
  Slot &ys = tape->slots[n->out];
  const int M = n->rows, K = n->n_in, N = n->n_out, dt = L->dt;
  const size_t e = esize(L);
  if (!ys.grad) return set_error(FL_ERR_STATE, "linear node %d: no gradient reached its output", self);
  if (ys.xform != XF_NONE && !ys.xform_done)
    return set_error(FL_ERR_STATE, "linear node %d: activation derivative was not applied upstream", self);
  const void *gy = ys.grad;
  const void *W = L->params[kLinear[n->param].w];
  // The linear output was dropped out before it was added to the residual stream: the identity branch
  // (below) passes the sum's gradient on as it is, the linear layer sees it times the keep mask.
  Buf *gm = nullptr;
  if (n->flags && L->rec_p_hidden > 0.f) {
    gm = buf_new((size_t)M * N * e, st);
    if (!gm) return oom_error((size_t)M * N * e);
    hipError_t he = launch_dropout_mul(dt, gy, gm->ptr, M, N, make_drop_spec(L->rec_p_hidden, L->rec_seed, n->flags), st);
    if (he != hipSuccess) {
      buf_unref(gm);
      FL_HIP(he);
    }
    gy = gm->ptr;
  }
  struct Unref {  // gm lives until this function returns (the side stream holds its own reference)
    Buf *&b;
    ~Unref() { buf_unref(b); }
  } unref_gm{gm};
  // The first linear operator of the replay leaves its parameter-gradient work to the next fork (see pending_side).
  const bool defer_side = L->side && L->forks == 0 && L->pending_side.empty() && self > 1;
  hipEvent_t forked = nullptr;
  if (!defer_side) FL_TRY(side_mark(L, &forked));   // gy is complete at this point of the layer's stream
  // input gradient: dx[M,K] = gy W (+ what other consumers of x already contributed)
  {
    Slot &xs = tape->slots[n->in0];
    const bool fin = tape->finishes(self, n->in0);
    GemmArgs a;
    a.A = gy; a.lda = N; a.a_kc = true;
    a.B = W; a.ldb = K; a.b_kc = false;
    a.M = M; a.N = K; a.K = N; a.ldc = K;
    int cls = FL_K_GEMM_NN;
    if (const Buf *wt = L->wt[n->param]) {  // W^T [K, N]: the contraction index is contiguous in both operands
      FL_TRY(wt_acquire(L));
      a.B = wt->ptr; a.ldb = N; a.b_kc = true;
      cls = FL_K_GEMM_NT;
    }
    a.residual = xs.grad;
    if (fin && xs.xform != XF_NONE) {
      a.dact = xs.xform;
      a.aux = xs.xform_aux;
      if (xs.xform_drop_site && L->rec_p_hidden > 0.f) {
        a.drop_where = 2;
        a.drop = make_drop_spec(L->rec_p_hidden, L->rec_seed, xs.xform_drop_site);
      }
    }
    Buf *nb = nullptr;
    if (fin && xs.grad_dst) {
      a.C = xs.grad_dst;
    } else {
      nb = buf_new((size_t)M * K * e, st);
      if (!nb) return oom_error((size_t)M * K * e);
      a.C = nb->ptr;
    }
    hipError_t he = timed(cls, 2.0 * M * N * K, ((double)M * N + (double)M * K + (double)N * K) * e, st,
                          [&] { return launch_gemm(dt, a, st); });
    if (he != hipSuccess) {
      buf_unref(nb);
      FL_HIP(he);
    }
    set_grad(xs, a.C, nb);
    if (a.dact) xs.xform_done = true;
  }
  // The parameter gradients need gy and the saved input only and nobody waits for them before the
  // backward pass ends: they go to the side stream, beside the input-gradient chain (whose GEMM is
  // already enqueued above).
  side_hold(L, gm ? gm : ys.grad_buf);
  side_hold(L, tape->slots[n->in0].value_buf);
  // The pass's last linear operator: nothing follows its input gradient on the layer's stream, while the
  // side stream still has this operator's weight gradient and every second stage ahead of it.  So its
  // bias sums run on the layer's stream behind the input gradient, and the second stages split (see
  // reduce_flush_split).  Measured on the BERT-base shape: the side stream used to end 45 us after the
  // layer's stream.
  const bool tail = L->side && !defer_side && self == L->tail_node;
  const bool need_colsum = !ys.colsum_done;
  const bool colsum_here = need_colsum && !tail;
  const bool reads_callers_dy = L->side && L->defer_join && !gm && !ys.grad_buf;
  const void *x_saved = n->s0;
  const int lin = n->param;
  auto side_work = [=](hipStream_t ps) -> int {
    OpTag tag2(FL_OP_LINEAR_BWD, self);
    // bias gradient, unless the kernel that finished gy already produced it: first stage here, second stage
    // batched with the others
    if (colsum_here) {
      Scratch ws;
      FL_TRY(ws.get(colsum_ws_floats(M, N) * sizeof(float), ps));
      FL_HIP(timed(FL_K_COLSUM, 0, (double)M * N * e, ps,
                   [&] { return launch_colsum_stage1(dt, gy, M, N, ws.f32(), ps); }));
      FL_TRY(reduce_later(L, ps, false, ws.b, colsum_stage1_rows(M), (size_t)N, (size_t)N, 1,
                          L->grads[kLinear[lin].b], nullptr, nullptr));
    }
    // weight gradient: dW[N,K] = sum_m gy[m,n] x[m,k]
    GemmArgs a;
    a.A = gy; a.lda = N; a.a_kc = false;
    a.B = x_saved; a.ldb = K; a.b_kc = false;
    a.M = N; a.N = K; a.K = M;
    a.C = L->grads[kLinear[lin].w]; a.ldc = K;
    a.splits = gemm_pick_splits(dt, a.M, a.N, a.K);
    const double fl = 2.0 * M * N * K, by = ((double)M * N + (double)M * K + (double)N * K) * e;
    if (a.splits > 1) {
      Scratch ws;
      FL_TRY(ws.get((size_t)a.splits * N * K * sizeof(float), ps));
      a.partial = ws.f32();
      FL_HIP(timed(FL_K_GEMM_TN, fl, by, ps, [&] { return launch_gemm(dt, a, ps); }));
      FL_TRY(reduce_later(L, ps, false, ws.b, a.splits, (size_t)N * K, (size_t)N * K, 1, a.C, nullptr, nullptr));
    } else {
      if (L->accumulate) a.residual = a.C;  // in place: each lane reads the elements it then writes
      FL_HIP(timed(FL_K_GEMM_TN, fl, by, ps, [&] { return launch_gemm(dt, a, ps); }));
    }
    if (reads_callers_dy) {  // gy is the caller's dY, and these were its readers
      if (!L->caller_read_event) FL_HIP(hipEventCreateWithFlags(&L->caller_read_event, kEventFlags));
      FL_HIP(hipEventRecord(L->caller_read_event, L->side));
      L->caller_read_pending = true;
    }
    return 0;
  };
  // The parameter gradients need gy and the saved input only and nobody waits for them before the
  // backward pass ends: they go to the side stream, beside the input-gradient chain (whose GEMM is
  // already enqueued above).
  if (defer_side) {
    L->pending_side.push_back(side_work);
  } else {
    hipStream_t ps;
    FL_TRY(side_begin(L, forked, &ps));
    FL_TRY(run_pending_side(L, ps));
    if (tail) {
      if (!L->tail_event) FL_HIP(hipEventCreateWithFlags(&L->tail_event, kEventFlags));
      FL_HIP(hipEventRecord(L->tail_event, ps));
      L->tail_jobs = L->reduce_jobs.size();
      L->tail_split = true;
      if (need_colsum) {   // on the layer's stream, behind the input gradient enqueued above
        Scratch ws;
        FL_TRY(ws.get(colsum_ws_floats(M, N) * sizeof(float), st));
        FL_HIP(timed(FL_K_COLSUM, 0, (double)M * N * e, st,
                     [&] { return launch_colsum_stage1(dt, gy, M, N, ws.f32(), st); }));
        FL_TRY(reduce_later(L, ps, true, ws.b, colsum_stage1_rows(M), (size_t)N, (size_t)N, 1,
                            L->grads[kLinear[lin].b], nullptr, nullptr));
      }
    }
    FL_TRY(side_work(ps));
    // (the second stages stay collected until the end of the pass: one launch there measured better than a
    // launch after every operator, 0.408 against 0.413 ms per step on the BERT-base shape)
  }
  // residual input: the identity branch passes gy through unchanged
  if (n->in1 >= 0) {
    Slot &rs = tape->slots[n->in1];
    if (rs.grad || tape->finishes(self, n->in1))
      return set_error(FL_ERR_UNSUPPORTED, "linear node %d: residual gradient would need a separate add", self);
    rs.grad = ys.grad;
    rs.grad_buf = ys.grad_buf;
    if (rs.grad_buf) rs.grad_buf->refs++;
  }
  set_grad(ys, nullptr, nullptr);
  buf_unref(ys.value_buf);
  for (Buf *b : n->saved) {
    Buf *t = b;
    buf_unref(t);
  }
  const_cast<Node *>(n)->saved[0] = const_cast<Node *>(n)->saved[1] = const_cast<Node *>(n)->saved[2] = nullptr;
  return 0;
}

int attention_backward(void *ctx, Tape *tape, const Node *n) {
  fl_layer *L = static_cast<fl_layer *>(ctx);
  const int self = tape->index_of(n);
  OpTag tag(FL_OP_ATTENTION_BWD, self);
  hipStream_t st = L->stream;
  Slot &os = tape->slots[n->out], &qs = tape->slots[n->in0];
  const int D = L->cfg.d_model, H = L->cfg.n_heads, dh = D / H, M = L->M;
  const size_t e = esize(L);
  if (!os.grad) return set_error(FL_ERR_STATE, "attention node %d: no gradient reached its output", self);
  if (qs.grad || !tape->finishes(self, n->in0) || qs.xform != XF_NONE)
    return set_error(FL_ERR_UNSUPPORTED, "attention node %d: its input must have no other consumer", self);
  Buf *nb = buf_new((size_t)M * 3 * D * e, st);
  if (!nb) return oom_error((size_t)M * 3 * D * e);
  Scratch delta;
  int rc = delta.get((size_t)L->B * H * L->T * sizeof(float), st);
  if (rc) {
    buf_unref(nb);
    return rc;
  }
  const double fl = 10.0 * D * L->T * (double)M, by = 8.0 * M * D * e + 8.0 * L->B * H * L->T;
  const DropSpec drop = make_drop_spec(L->rec_p_attn, L->rec_seed, 1);
  auto run = [&](int parts, hipStream_t s) {
    return launch_attention_bwd(L->dt, qs.value, os.value, os.grad, static_cast<const float *>(n->s0), L->lengths,
                                L->cfg.causal, drop, L->B, L->T, H, dh, nb->ptr, delta.f32(), s, parts);
  };
  // Worth a second stream only where dQ and dK/dV are independent kernels (the general path, whose
  // grids leave much of the chip idle); next to the parameter-gradient stream the matrix-core kernels
  // measured no gain from it.
  hipStream_t s2 = L->side && attention_bwd_parts_independent(L->dt, dh) ? side_stream2() : nullptr;
  hipError_t he;
  if (!s2) {
    he = timed(FL_K_ATTN_BWD, fl, by, st, [&] { return run(ATTN_BWD_ALL, st); });
  } else {
    // dQ and dK/dV only share their inputs (and delta): dK/dV go to the second side stream, and the
    // layer's stream waits for them before this function returns, so no buffer outlives its readers.
    he = timed(FL_K_ATTN_BWD, 0, 0, st, [&] { return run(ATTN_BWD_DELTA, st); });
    hipEvent_t forked = nullptr;
    if (he == hipSuccess && side_mark(L, &forked)) he = hipErrorUnknown;
    if (he == hipSuccess) he = timed(FL_K_ATTN_BWD, 0.4 * fl, 0.5 * by, st, [&] { return run(ATTN_BWD_DQ, st); });
    if (he == hipSuccess) he = hipStreamWaitEvent(s2, forked, 0);
    if (he == hipSuccess) he = timed(FL_K_ATTN_BWD, 0.6 * fl, 0.5 * by, s2, [&] { return run(ATTN_BWD_DKV, s2); });
    if (he == hipSuccess && !L->attn_join_event) he = hipEventCreateWithFlags(&L->attn_join_event, kEventFlags);
    if (he == hipSuccess) he = hipEventRecord(L->attn_join_event, s2);
    if (he == hipSuccess) he = hipStreamWaitEvent(st, L->attn_join_event, 0);
    if (he != hipSuccess) hipStreamSynchronize(s2);  // nothing of this function may still run when its buffers go
  }
  if (he != hipSuccess) {
    buf_unref(nb);
    FL_HIP(he);
  }
  set_grad(qs, nb->ptr, nb);
  set_grad(os, nullptr, nullptr);
  buf_unref(os.value_buf);
  Buf *t = n->saved[0];
  buf_unref(t);
  const_cast<Node *>(n)->saved[0] = nullptr;
  return 0;
}

int layernorm_backward(void *ctx, Tape *tape, const Node *n) {
  fl_layer *L = static_cast<fl_layer *>(ctx);
  const int self = tape->index_of(n);
  OpTag tag(FL_OP_LAYERNORM_BWD, self);
  hipStream_t st = L->stream;
  Slot &ys = tape->slots[n->out], &xs = tape->slots[n->in0];
  const int D = L->cfg.d_model, M = L->M, dt = L->dt;
  const size_t e = esize(L);
  if (!ys.grad) return set_error(FL_ERR_STATE, "layernorm node %d: no gradient reached its output", self);
  const bool fin = tape->finishes(self, n->in0);
  if (fin && xs.xform != XF_NONE)
    return set_error(FL_ERR_UNSUPPORTED, "layernorm node %d: cannot apply an activation derivative", self);
  const int gi = n->param == 0 ? P_LN1G : P_LN2G, bi = n->param == 0 ? P_LN1B : P_LN2B;
  const int parts = ln_bwd_parts(M, D);
  Scratch ws;
  FL_TRY(ws.get((size_t)parts * 3 * D * sizeof(float), st));
  Buf *nb = nullptr;
  void *dst;
  if (fin && xs.grad_dst) {
    dst = xs.grad_dst;
  } else {
    nb = buf_new((size_t)M * D * e, st);
    if (!nb) return oom_error((size_t)M * D * e);
    dst = nb->ptr;
  }
  const float *mean = static_cast<const float *>(n->s0);
  const double by = (double)M * D * e * (xs.grad ? 4 : 3) + 8.0 * M;
  hipError_t he = timed(FL_K_LN_BWD, 0, by, st, [&] {
    return launch_layernorm_bwd(dt, ys.grad, xs.value, mean, mean + M, L->params[gi], xs.grad, M, D, dst, ws.f32(), st);
  });
  if (he != hipSuccess) {
    buf_unref(nb);
    FL_HIP(he);
  }
  set_grad(xs, dst, nb);
  const bool want_bias = fin && xs.colsum_param >= 0;
  // second stage of the parameter-gradient sums: batched with the others on the parameter-gradient lane (no
  // fork of its own: the next linear operator's fork, or the one before the last batch, covers these sums)
  hipStream_t ps = L->side ? L->side : st;
  side_hold(L, ws.b);
  FL_TRY(reduce_later(L, ps, true, ws.b, parts, (size_t)3 * D, (size_t)D, want_bias ? 3 : 2, L->grads[gi], L->grads[bi],
                      want_bias ? L->grads[xs.colsum_param] : nullptr));
  if (want_bias) xs.colsum_done = true;
  set_grad(ys, nullptr, nullptr);
  buf_unref(ys.value_buf);
  Buf *t = n->saved[0];
  buf_unref(t);
  const_cast<Node *>(n)->saved[0] = nullptr;
  return 0;
}

// ---- forward operators (each enqueues its kernel and records its node) ------------------

// y = x W^T + b, optional activation (records the request for its derivative on y), optional dropout
// (site: 0 none, else the hidden-state site whose keep mask multiplies the result before the residual
// is added) and residual.
int op_linear(fl_layer *L, int lin, int xslot, int rslot, int act, int K, int N, void *y_ext, int *yslot, int site) {
  Tape &tp = L->tape;
  OpTag tag(FL_OP_LINEAR_FWD, (int)tp.nodes.size());
  hipStream_t st = L->stream;
  const int M = L->M, dt = L->dt;
  const size_t e = esize(L);
  Buf *yb = nullptr, *ub = nullptr;
  void *y = y_ext;
  if (!y) {
    yb = buf_new((size_t)M * N * e, st);
    if (!yb) return oom_error((size_t)M * N * e);
    y = yb->ptr;
  }
  GemmArgs a;
  a.A = tp.slots[xslot].value; a.lda = K; a.a_kc = true;
  a.B = L->params[kLinear[lin].w]; a.ldb = K; a.b_kc = true;
  a.M = M; a.N = N; a.K = K; a.C = y; a.ldc = N;
  a.alone = true;   // the forward pass runs one kernel at a time
  a.bias = L->params[kLinear[lin].b];
  a.act = act;
  if (rslot >= 0) a.residual = tp.slots[rslot].value;
  const bool dropped = site != 0 && L->rec_p_hidden > 0.f;
  if (dropped) {
    a.drop_where = 1;
    a.drop = make_drop_spec(L->rec_p_hidden, L->rec_seed, (uint32_t)site);
  }
  if (act == XF_GELU && !L->inference) {  // the derivative needs the pre-activation
    ub = buf_new((size_t)M * N * e, st);
    if (!ub) {
      buf_unref(yb);
      return oom_error((size_t)M * N * e);
    }
    a.preact = ub->ptr;
  }
  hipError_t he = timed(FL_K_GEMM_NT, 2.0 * M * N * K, ((double)M * N + (double)M * K + (double)N * K) * e, st,
                        [&] { return launch_gemm(dt, a, st); });
  if (he != hipSuccess) {
    buf_unref(yb);
    buf_unref(ub);
    FL_HIP(he);
  }
  const int ys = tp.new_slot();
  Slot &s = tp.slots[ys];
  s.value = y;
  s.value_buf = yb;
  // the bias gradient is the column sum of the gradient that enters the linear layer: with a dropped-out
  // output in front of a residual add that is NOT the gradient of this slot (linear_backward masks it first)
  s.colsum_param = dropped && act == XF_NONE ? -1 : kLinear[lin].b;
  if (act != XF_NONE) {
    s.xform = act;
    s.xform_aux = act == XF_GELU && ub ? ub->ptr : y;  // ReLU: the output's sign is the pre-activation's
    if (dropped) s.xform_drop_site = site;       // and the kept outputs were scaled: same mask on the way back
  }
  Node n;
  n.backward = linear_backward;
  n.op = OP_LINEAR;
  n.in0 = xslot; n.in1 = rslot; n.out = ys; n.param = lin;
  n.flags = dropped && act == XF_NONE ? site : 0;
  n.s0 = tp.slots[xslot].value;
  n.saved[0] = ub;
  n.rows = M; n.n_in = K; n.n_out = N;
  tp.record(n);
  *yslot = ys;
  return 0;
}

int op_attention(fl_layer *L, int qslot, int *oslot) {
  Tape &tp = L->tape;
  OpTag tag(FL_OP_ATTENTION_FWD, (int)tp.nodes.size());
  hipStream_t st = L->stream;
  const int D = L->cfg.d_model, H = L->cfg.n_heads, dh = D / H, M = L->M;
  const size_t e = esize(L);
  Buf *ob = buf_new((size_t)M * D * e, st);
  Buf *lb = buf_new((size_t)L->B * H * L->T * sizeof(float), st);
  if (!ob || !lb) {
    buf_unref(ob);
    buf_unref(lb);
    return oom_error((size_t)M * D * e);
  }
  const double fl = 4.0 * D * L->T * (double)M, by = 4.0 * M * D * e + 4.0 * L->B * H * L->T;
  hipError_t he = timed(FL_K_ATTN_FWD, fl, by, st, [&] {
    return launch_attention_fwd(L->dt, tp.slots[qslot].value, L->lengths, L->cfg.causal,
                                make_drop_spec(L->rec_p_attn, L->rec_seed, 1), L->B, L->T, H, dh, ob->ptr,
                                static_cast<float *>(lb->ptr), st);
  });
  if (he != hipSuccess) {
    buf_unref(ob);
    buf_unref(lb);
    FL_HIP(he);
  }
  const int os = tp.new_slot();
  tp.slots[os].value = ob->ptr;
  tp.slots[os].value_buf = ob;
  Node n;
  n.backward = attention_backward;
  n.op = OP_ATTN;
  n.in0 = qslot; n.out = os;
  n.s0 = lb->ptr;
  n.saved[0] = lb;
  n.rows = M;
  tp.record(n);
  *oslot = os;
  return 0;
}

int op_layernorm(fl_layer *L, int which, int xslot, void *y_ext, int *yslot) {
  Tape &tp = L->tape;
  OpTag tag(FL_OP_LAYERNORM_FWD, (int)tp.nodes.size());
  hipStream_t st = L->stream;
  const int D = L->cfg.d_model, M = L->M;
  const size_t e = esize(L);
  Buf *yb = nullptr;
  void *y = y_ext;
  if (!y) {
    yb = buf_new((size_t)M * D * e, st);
    if (!yb) return oom_error((size_t)M * D * e);
    y = yb->ptr;
  }
  Buf *sb = buf_new((size_t)2 * M * sizeof(float), st);
  if (!sb) {
    buf_unref(yb);
    return oom_error((size_t)2 * M * sizeof(float));
  }
  float *mean = static_cast<float *>(sb->ptr);
  const int gi = which == 0 ? P_LN1G : P_LN2G, bi = which == 0 ? P_LN1B : P_LN2B;
  hipError_t he = timed(FL_K_LN_FWD, 0, 2.0 * M * D * e + 8.0 * M, st, [&] {
    return launch_layernorm_fwd(L->dt, tp.slots[xslot].value, L->params[gi], L->params[bi], L->eps, M, D, y, mean,
                                mean + M, st);
  });
  if (he != hipSuccess) {
    buf_unref(yb);
    buf_unref(sb);
    FL_HIP(he);
  }
  const int ys = tp.new_slot();
  tp.slots[ys].value = y;
  tp.slots[ys].value_buf = yb;
  Node n;
  n.backward = layernorm_backward;
  n.op = OP_LN;
  n.in0 = xslot; n.out = ys; n.param = which;
  n.s0 = mean;
  n.saved[0] = sb;
  n.rows = M;
  tp.record(n);
  *yslot = ys;
  return 0;
}

void load_params(fl_layer *L, const fl_layer_params_t *p) {
  const void *v[P_COUNT] = {p->Wqkv, p->bqkv, p->Wo, p->bo, p->W1, p->b1, p->W2, p->b2,
                            p->ln1_g, p->ln1_b, p->ln2_g, p->ln2_b};
  memcpy(L->params, v, sizeof(v));
}

int check_ptrs(const void *const *v, int n, const char *what) {
  for (int i = 0; i < n; ++i) {
    if (!v[i]) return set_error(FL_ERR_INVALID_ARG, "%s: pointer %d is null", what, i);
    if (reinterpret_cast<uintptr_t>(v[i]) & 15)
      return set_error(FL_ERR_UNSUPPORTED, "%s: pointer %d is not 16-byte aligned", what, i);
  }
  return 0;
}

int forward_impl(fl_layer *L, const fl_layer_params_t *params, const void *X, const int32_t *lengths, int B, int T,
                 void *Y, hipStream_t st) {
  const fl_layer_config_t &c = L->cfg;
  if (B < 1 || T < 1 || B > c.max_B || T > c.max_T)
    return set_error(FL_ERR_INVALID_ARG, "B=%d T=%d outside 1..max_B=%d, 1..max_T=%d", B, T, c.max_B, c.max_T);
  if ((long)B * T > (1l << 24)) return set_error(FL_ERR_UNSUPPORTED, "B*T too large");
  load_params(L, params);
  FL_TRY(check_ptrs(L->params, P_COUNT, "params"));
  const void *io[2] = {X, Y};
  FL_TRY(check_ptrs(io, 2, "X/Y"));
  g_debug = debug_from_env();
  if (g_debug && lengths) {
    std::vector<int32_t> h((size_t)B);
    FL_HIP(hipMemcpyAsync(h.data(), lengths, (size_t)B * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    FL_HIP(hipStreamSynchronize(st));
    for (int b = 0; b < B; ++b)
      if (h[b] < 1 || h[b] > T)
        return set_error(FL_ERR_INVALID_ARG, "lengths[%d] = %d is outside 1..T = %d", b, h[b], T);
  }
  FL_TRY(finish_pending_join(L, st, false));
  release_tape(L);
  L->B = B; L->T = T; L->M = B * T; L->stream = st; L->lengths = lengths;
  L->rec_p_attn = L->p_attn; L->rec_p_hidden = L->p_hidden; L->rec_seed = L->seed;
  FL_TRY(wt_make(L));
  Tape &tp = L->tape;
  const int D = c.d_model, F = c.d_ffn;
  const int act = c.act == FL_ACT_RELU ? XF_RELU : XF_GELU;
  const int sx = tp.new_slot();
  tp.slots[sx].value = X;
  L->slot_x = sx;
  int s_qkv, s_o, s_r1, s_y1, s_g, s_out, s_n1;
  if (c.norm == FL_NORM_POST) {
    FL_TRY(op_linear(L, 0, sx, -1, XF_NONE, D, 3 * D, nullptr, &s_qkv, 0));
    FL_TRY(op_attention(L, s_qkv, &s_o));
    FL_TRY(op_linear(L, 1, s_o, sx, XF_NONE, D, D, nullptr, &s_r1, 2));   // R1 = X + drop(O Wo^T + bo)
    FL_TRY(op_layernorm(L, 0, s_r1, nullptr, &s_y1));                      // Y1 = LN1(R1)
    FL_TRY(op_linear(L, 2, s_y1, -1, act, D, F, nullptr, &s_g, 3));        // G = drop(act(Y1 W1^T + b1))
    int s_r2;
    FL_TRY(op_linear(L, 3, s_g, s_y1, XF_NONE, F, D, nullptr, &s_r2, 4));  // R2 = Y1 + drop(G W2^T + b2)
    FL_TRY(op_layernorm(L, 1, s_r2, Y, &s_out));                           // Y = LN2(R2)
  } else {
    FL_TRY(op_layernorm(L, 0, sx, nullptr, &s_n1));                        // N1 = LN1(X)
    FL_TRY(op_linear(L, 0, s_n1, -1, XF_NONE, D, 3 * D, nullptr, &s_qkv, 0));
    FL_TRY(op_attention(L, s_qkv, &s_o));
    FL_TRY(op_linear(L, 1, s_o, sx, XF_NONE, D, D, nullptr, &s_r1, 2));   // R1 = X + drop(O Wo^T + bo)
    FL_TRY(op_layernorm(L, 1, s_r1, nullptr, &s_y1));                      // N2 = LN2(R1)
    FL_TRY(op_linear(L, 2, s_y1, -1, act, D, F, nullptr, &s_g, 3));
    FL_TRY(op_linear(L, 3, s_g, s_r1, XF_NONE, F, D, Y, &s_out, 4));       // Y = R1 + drop(G W2^T + b2)
  }
  L->slot_y = s_out;
  tp.recorded = true;
  return 0;
}

// The allocation-free forward (fl_layer_forward_static): the same operators and kernels as forward_impl in
// evaluation mode, with every intermediate carved out of the static scratch array and given back as soon as
// its last reader is enqueued; nothing is kept for a backward pass and nothing is recorded.
int forward_static_impl(fl_layer *L, const fl_layer_params_t *params, const void *X, const int32_t *lengths, int B,
                        int T, void *Y, hipStream_t st) {
  const fl_layer_config_t &c = L->cfg;
  if (B < 1 || T < 1 || B > c.max_B || T > c.max_T)
    return set_error(FL_ERR_INVALID_ARG, "B=%d T=%d outside 1..max_B=%d, 1..max_T=%d", B, T, c.max_B, c.max_T);
  if ((long)B * T > (1l << 24)) return set_error(FL_ERR_UNSUPPORTED, "B*T too large");
  if (L->tape.recorded || L->join_pending)
    return set_error(FL_ERR_STATE, "the handle holds a recorded forward: run its backward (and join) first");
  load_params(L, params);
  FL_TRY(check_ptrs(L->params, P_COUNT, "params"));
  const void *io[2] = {X, Y};
  FL_TRY(check_ptrs(io, 2, "X/Y"));
  const int D = c.d_model, F = c.d_ffn;
  const size_t e = esize(L), M = (size_t)B * T;
  // the largest set of intermediates alive at once: the feed-forward block (its input, the hidden
  // activation and the residual sum around it)
  // or the attention block (the fused projections, the attention output and its row statistics)
  const size_t ffn = M * D * e * 2 + M * F * e, attn = M * D * e * 4 + M * c.n_heads * 4;
  const size_t need = (ffn > attn ? ffn : attn) + M * 8 + 4096;
  if (need > kStaticScratchBytes)
    return set_error(FL_ERR_UNSUPPORTED,
                     "B*T = %zu tokens need %zu bytes of intermediates, the static scratch holds %zu: use "
                     "fl_layer_forward, or fewer tokens per call", M, need, (size_t)kStaticScratchBytes);
  void *base = nullptr;
  FL_HIP(static_scratch_base(&base));
  Arena arena(base, kStaticScratchBytes);
  struct Mode {  // evaluation mode on this thread for the length of the call
    fl_layer *L;
    Mode(fl_layer *l, Arena *a) : L(l) { g_arena = a; g_no_alloc = true; L->inference = true; }
    ~Mode() {
      release_tape(L);  // while the arena still exists
      g_arena = nullptr; g_no_alloc = false; L->inference = false;
    }
  } mode(L, &arena);
  L->B = B; L->T = T; L->M = B * T; L->stream = st; L->lengths = lengths;
  L->rec_p_attn = 0.f; L->rec_p_hidden = 0.f; L->rec_seed = 0;  // evaluation mode: no dropout
  Tape &tp = L->tape;
  auto drop_value = [&](int slot) { buf_unref(tp.slots[slot].value_buf); };
  auto drop_saved = [&]() {  // what the node recorded last keeps for its backward
    for (Buf *&b : tp.nodes.back().saved) buf_unref(b);
  };
  const int act = c.act == FL_ACT_RELU ? XF_RELU : XF_GELU;
  const int sx = tp.new_slot();
  tp.slots[sx].value = X;
  int s_qkv, s_o, s_r1, s_y1, s_g, s_out, s_n1;
  if (c.norm == FL_NORM_POST) {
    FL_TRY(op_linear(L, 0, sx, -1, XF_NONE, D, 3 * D, nullptr, &s_qkv, 0));
    FL_TRY(op_attention(L, s_qkv, &s_o));
    drop_saved();        // the log-sum-exp
    drop_value(s_qkv);
    FL_TRY(op_linear(L, 1, s_o, sx, XF_NONE, D, D, nullptr, &s_r1, 0));
    drop_value(s_o);
    FL_TRY(op_layernorm(L, 0, s_r1, nullptr, &s_y1));
    drop_saved();        // mean / rstd
    drop_value(s_r1);
    FL_TRY(op_linear(L, 2, s_y1, -1, act, D, F, nullptr, &s_g, 0));
    int s_r2;
    FL_TRY(op_linear(L, 3, s_g, s_y1, XF_NONE, F, D, nullptr, &s_r2, 0));
    drop_value(s_g);
    drop_value(s_y1);
    FL_TRY(op_layernorm(L, 1, s_r2, Y, &s_out));
    drop_saved();
    drop_value(s_r2);
  } else {
    FL_TRY(op_layernorm(L, 0, sx, nullptr, &s_n1));
    drop_saved();
    FL_TRY(op_linear(L, 0, s_n1, -1, XF_NONE, D, 3 * D, nullptr, &s_qkv, 0));
    drop_value(s_n1);
    FL_TRY(op_attention(L, s_qkv, &s_o));
    drop_saved();
    drop_value(s_qkv);
    FL_TRY(op_linear(L, 1, s_o, sx, XF_NONE, D, D, nullptr, &s_r1, 0));
    drop_value(s_o);
    FL_TRY(op_layernorm(L, 1, s_r1, nullptr, &s_y1));
    drop_saved();
    FL_TRY(op_linear(L, 2, s_y1, -1, act, D, F, nullptr, &s_g, 0));
    drop_value(s_y1);
    FL_TRY(op_linear(L, 3, s_g, s_r1, XF_NONE, F, D, Y, &s_out, 0));
    drop_value(s_g);
    drop_value(s_r1);
  }
  return 0;  // ~Mode drops the recording: tape.recorded was never set
}

int backward_impl(fl_layer *L, const fl_layer_params_t *params, const void *dY, void *dX, fl_layer_grads_t *grads,
                  bool accumulate, hipStream_t st) {
  L->accumulate = accumulate;
  if (!L->tape.recorded) return set_error(FL_ERR_STATE, "backward without a recorded forward");
  if (st != L->stream) return set_error(FL_ERR_STATE, "backward on a different stream than forward");
  load_params(L, params);
  FL_TRY(check_ptrs(L->params, P_COUNT, "params"));
  void *g[P_COUNT] = {grads->Wqkv, grads->bqkv, grads->Wo, grads->bo, grads->W1, grads->b1, grads->W2, grads->b2,
                      grads->ln1_g, grads->ln1_b, grads->ln2_g, grads->ln2_b};
  memcpy(L->grads, g, sizeof(g));
  FL_TRY(check_ptrs(L->grads, P_COUNT, "grads"));
  const void *io[2] = {dY, dX};
  FL_TRY(check_ptrs(io, 2, "dY/dX"));
  Tape &tp = L->tape;
  tp.slots[L->slot_y].grad = const_cast<void *>(dY);
  tp.slots[L->slot_x].grad_dst = dX;
  // the events of a fork cost the host more than tiny kernels take: small problems stay on one stream
  L->side = g_overlap && (long)L->M * L->cfg.d_model >= (1l << 18) ? side_stream() : nullptr;
  L->forks = 0;
  L->tail_node = -1;
  L->tail_split = false;
  // (not with a deferred join: the layer's stream then goes straight on with the next layer's backward
  // pass, and work moved onto it delays that chain -- measured +1.2 % on the 12-layer stack)
  if (L->side && !L->defer_join)
    for (size_t i = 0; i < tp.nodes.size(); ++i)
      if (tp.nodes[i].backward == linear_backward) {   // first recorded = last replayed
        L->tail_node = (int)i;
        break;
      }
  int rc = tp.replay_reverse(L);
  if (!rc && !L->pending_side.empty()) {  // no later operator forked: fork now
    hipEvent_t ev;
    hipStream_t ps;
    rc = side_mark(L, &ev);
    if (!rc) rc = side_begin(L, ev, &ps);
    if (!rc) rc = run_pending_side(L, ps);
  }
  if (rc) {   // drop what the failed pass has collected
    L->pending_side.clear();
    L->reduce_jobs.clear();
    for (Buf *&b : L->reduce_bufs) buf_unref(b);
    L->reduce_bufs.clear();
    L->reduce_job_main.clear();
    L->reduce_from_main = false;
    L->reduce_has_side = false;
    L->tail_split = false;
  } else {
    rc = L->tail_split && L->side ? reduce_flush_split(L) : reduce_flush(L);
  }
  const bool landed = rc == 0 && tp.slots[L->slot_x].grad == dX;
  const int jrc = side_join(L, rc != 0, L->defer_join);
  release_tape(L);
  if (rc) return rc;
  if (jrc) return jrc;
  if (!landed) return set_error(FL_ERR_STATE, "input gradient did not reach its destination");
  return 0;
}

}  // namespace

// ------------------------------------------------------------------ C ABI
#define FL_GUARD_BEGIN try {
#define FL_GUARD_END                                                         \
  }                                                                          \
  catch (const std::bad_alloc &) {                                           \
    return (fl_status_t)set_error(FL_ERR_OOM, "host allocation failed");     \
  }                                                                          \
  catch (...) {                                                              \
    return (fl_status_t)set_error(FL_ERR_DEVICE, "unexpected internal error"); \
  }

extern "C" {

fl_status_t fl_layer_create(const fl_layer_config_t *cfg, fl_layer_t **out) {
  FL_GUARD_BEGIN
  if (!cfg || !out) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  *out = nullptr;
  if (cfg->max_B < 1 || cfg->max_T < 1 || cfg->d_model < 1 || cfg->n_heads < 1 || cfg->d_ffn < 1)
    return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "sizes must be positive");
  if (cfg->d_model % cfg->n_heads)
    return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "d_model=%d is not a multiple of n_heads=%d", cfg->d_model,
                                  cfg->n_heads);
  if ((unsigned)cfg->act > FL_ACT_GELU || (unsigned)cfg->norm > FL_NORM_PRE || (unsigned)cfg->dtype > FL_BF16)
    return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "unknown activation, norm placement or dtype");
  const int dh = cfg->d_model / cfg->n_heads;
  if (cfg->d_model % 8 || cfg->d_ffn % 8 || dh % 16 || dh > 256 || cfg->d_model > 4096)
    return (fl_status_t)set_error(FL_ERR_UNSUPPORTED,
                                  "need d_model %% 8 == 0, d_ffn %% 8 == 0, head size %% 16 == 0 and <= 256, "
                                  "d_model <= 4096 (got d_model=%d d_ffn=%d head size=%d)",
                                  cfg->d_model, cfg->d_ffn, dh);
  fl_layer *L = new fl_layer();
  L->cfg = *cfg;
  L->eps = cfg->ln_eps > 0.f ? cfg->ln_eps : 1e-5f;
  L->dt = cfg->dtype == FL_F32 ? DT_F32 : DT_BF16;
  *out = L;
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_layer_forward(fl_layer_t *layer, const fl_layer_params_t *params, const void *X,
                             const int32_t *lengths, int32_t B, int32_t T, void *Y, void *hip_stream) {
  FL_GUARD_BEGIN
  if (!layer || !params || !X || !Y) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  int rc = forward_impl(layer, params, X, lengths, B, T, Y, static_cast<hipStream_t>(hip_stream));
  if (rc) release_tape(layer);
  return (fl_status_t)rc;
  FL_GUARD_END
}

fl_status_t fl_layer_forward_static(fl_layer_t *layer, const fl_layer_params_t *params, const void *X,
                                    const int32_t *lengths, int32_t B, int32_t T, void *Y, void *hip_stream) {
  FL_GUARD_BEGIN
  if (!layer || !params || !X || !Y) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  return (fl_status_t)forward_static_impl(layer, params, X, lengths, B, T, Y, static_cast<hipStream_t>(hip_stream));
  FL_GUARD_END
}

fl_status_t fl_layer_set_dropout(fl_layer_t *layer, float p_attn, float p_hidden, uint64_t seed) {
  FL_GUARD_BEGIN
  if (!layer) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  if (!(p_attn >= 0.f && p_attn < 1.f) || !(p_hidden >= 0.f && p_hidden < 1.f))
    return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "dropout rates must be in [0, 1) (got %g, %g)", (double)p_attn,
                                  (double)p_hidden);
  layer->p_attn = p_attn;
  layer->p_hidden = p_hidden;
  layer->seed = seed;
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_layer_backward(fl_layer_t *layer, const fl_layer_params_t *params, const void *dY, void *dX,
                              fl_layer_grads_t *grads, void *hip_stream) {
  return fl_layer_backward_accumulate(layer, params, dY, dX, grads, 0, hip_stream);
}

fl_status_t fl_layer_backward_accumulate(fl_layer_t *layer, const fl_layer_params_t *params, const void *dY, void *dX,
                                         fl_layer_grads_t *grads, int32_t accumulate, void *hip_stream) {
  FL_GUARD_BEGIN
  if (!layer || !params || !dY || !dX || !grads) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  return (fl_status_t)backward_impl(layer, params, dY, dX, grads, accumulate != 0, static_cast<hipStream_t>(hip_stream));
  FL_GUARD_END
}

fl_status_t fl_layer_set_deferred_join(fl_layer_t *layer, int32_t enabled) {
  FL_GUARD_BEGIN
  if (!layer) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  layer->defer_join = enabled != 0;
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_layer_join(fl_layer_t *layer, void *hip_stream) {
  FL_GUARD_BEGIN
  if (!layer) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  return (fl_status_t)finish_pending_join(layer, static_cast<hipStream_t>(hip_stream), false);
  FL_GUARD_END
}

fl_status_t fl_opt_step(const fl_opt_config_t *cfg, fl_dtype_t dtype, int32_t n, void *const *params,
                        const void *const *grads, float *const *state_m, float *const *state_v, const int64_t *numel,
                        void *hip_stream) {
  return fl_opt_step_master(cfg, dtype, n, params, nullptr, grads, state_m, state_v, numel, hip_stream);
}

fl_status_t fl_opt_step_master(const fl_opt_config_t *cfg, fl_dtype_t dtype, int32_t n, void *const *params,
                               float *const *master, const void *const *grads, float *const *state_m,
                               float *const *state_v, const int64_t *numel, void *hip_stream) {
  FL_GUARD_BEGIN
  if (!cfg || !params || !grads || !numel) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  if (n < 1 || n > OPT_MAX_TENSORS)
    return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "n=%d outside 1..%d", n, OPT_MAX_TENSORS);
  if ((unsigned)cfg->kind > FL_OPT_ADAM || (unsigned)dtype > FL_BF16)
    return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "unknown optimizer kind or dtype");
  if (cfg->kind == FL_OPT_ADAM && (cfg->step < 1 || !(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) ||
                                   !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f)))
    return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "Adam needs step >= 1 and betas in [0, 1)");
  OptHyper h{cfg->lr, cfg->momentum, cfg->weight_decay, cfg->beta1, cfg->beta2, cfg->eps, 1.f, 1.f};
  if (cfg->kind == FL_OPT_ADAM) {
    h.inv_bias1 = (float)(1.0 / (1.0 - std::pow((double)cfg->beta1, (double)cfg->step)));
    h.inv_bias2 = (float)(1.0 / (1.0 - std::pow((double)cfg->beta2, (double)cfg->step)));
  }
  long long ne[OPT_MAX_TENSORS];
  for (int i = 0; i < n; ++i) ne[i] = (long long)numel[i];
  hipError_t e = launch_opt_step(dtype == FL_F32 ? DT_F32 : DT_BF16, cfg->kind == FL_OPT_SGD ? 0 : 1, h, n, params,
                                 grads, state_m, state_v, ne, static_cast<hipStream_t>(hip_stream), master);
  if (e != hipSuccess)
    return (fl_status_t)set_error(e == hipErrorInvalidValue ? FL_ERR_UNSUPPORTED : FL_ERR_DEVICE,
                                  "optimizer step: %s (needs numel %% 8 == 0, 16-byte aligned pointers, state "
                                  "buffers for momentum / Adam)", hipGetErrorString(e));
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_zero_grad(fl_dtype_t dtype, int32_t n, void *const *grads, const int64_t *numel, void *hip_stream) {
  FL_GUARD_BEGIN
  if (!grads || !numel) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  if (n < 1 || n > OPT_MAX_TENSORS || (unsigned)dtype > FL_BF16)
    return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "n=%d outside 1..%d, or unknown dtype", n, OPT_MAX_TENSORS);
  long long bytes[OPT_MAX_TENSORS];
  for (int i = 0; i < n; ++i) bytes[i] = (long long)numel[i] * (dtype == FL_F32 ? 4 : 2);
  hipError_t e = launch_zero_tensors(n, grads, bytes, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess)
    return (fl_status_t)set_error(e == hipErrorInvalidValue ? FL_ERR_UNSUPPORTED : FL_ERR_DEVICE, "zero_grad: %s",
                                  hipGetErrorString(e));
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_layer_destroy(fl_layer_t *layer) {
  FL_GUARD_BEGIN
  if (!layer) return FL_OK;
  finish_pending_join(layer, nullptr, true);
  release_tape(layer, true);  // the caller's stream may be gone by now
  if (layer->wt_fork_event) hipEventDestroy(layer->wt_fork_event);
  if (layer->wt_event) hipEventDestroy(layer->wt_event);
  for (hipEvent_t e : layer->fork_events) hipEventDestroy(e);  // work already enqueued against them still completes
  if (layer->join_event) hipEventDestroy(layer->join_event);
  if (layer->attn_join_event) hipEventDestroy(layer->attn_join_event);
  if (layer->caller_read_event) hipEventDestroy(layer->caller_read_event);
  if (layer->tail_event) hipEventDestroy(layer->tail_event);
  delete layer;
  return FL_OK;
  FL_GUARD_END
}

const char *fl_last_error(void) { return g_err; }

fl_status_t fl_set_grad_overlap(int32_t enabled) {
  g_overlap = enabled != 0;
  return FL_OK;
}

fl_status_t fl_alloc_get_stats(fl_alloc_stats_t *out) {
  FL_GUARD_BEGIN
  if (!out) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  AllocStats s = device_allocator().stats();
  out->backing_mallocs = s.backing_mallocs; out->backing_bytes = s.backing_bytes;
  out->cache_hits = s.cache_hits; out->cache_misses = s.cache_misses;
  out->live_bytes = s.live_bytes; out->peak_bytes = s.peak_bytes;
  out->cached_bytes = s.cached_bytes; out->split_count = s.split_count;
  out->requested_bytes = s.requested_bytes; out->largest_free_block = s.largest_free_block;
  out->free_blocks = s.free_blocks;
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_alloc_trace_enable(int32_t capacity) {
  FL_GUARD_BEGIN
  if (capacity < 0 || capacity > (1 << 20))
    return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "trace capacity %d outside [0, 2^20]", capacity);
  device_allocator().trace_enable((size_t)capacity);
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_alloc_trace_read(fl_alloc_event_t *out, int32_t cap, int32_t *n) {
  FL_GUARD_BEGIN
  if (!out || !n || cap < 0) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument or negative capacity");
  static_assert(sizeof(fl_alloc_event_t) == sizeof(AllocEvent), "the two event records must have one layout");
  *n = (int32_t)device_allocator().trace_read(reinterpret_cast<AllocEvent *>(out), (size_t)cap);
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_alloc_trim(void) {
  FL_GUARD_BEGIN
  hipError_t e = hipDeviceSynchronize();
  if (e != hipSuccess) return (fl_status_t)set_error(FL_ERR_DEVICE, "hipDeviceSynchronize: %s", hipGetErrorString(e));
  device_allocator().trim();
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_alloc_set_split_limit(uint64_t bytes) {
  FL_GUARD_BEGIN
  device_allocator().set_split_limit((size_t)bytes);
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_prof_enable(uint32_t class_mask) {
  FL_GUARD_BEGIN
  Prof &P = prof();
  std::lock_guard<std::mutex> g(P.mu);
  P.mask = class_mask & ((1u << FL_K_CLASS_COUNT) - 1);
  if (!P.mask) {
    for (ProfEvent &ev : P.pending) {
      P.pool.push_back(ev.a);
      P.pool.push_back(ev.b);
    }
    P.pending.clear();
  }
  return FL_OK;
  FL_GUARD_END
}

fl_status_t fl_prof_collect(fl_prof_entry_t *out, int32_t cap, int32_t *n) {
  FL_GUARD_BEGIN
  if (!out || !n || cap < 1) return (fl_status_t)set_error(FL_ERR_INVALID_ARG, "null argument");
  Prof &P = prof();
  std::lock_guard<std::mutex> g(P.mu);
  fl_prof_entry_t acc[FL_K_CLASS_COUNT];
  for (int i = 0; i < FL_K_CLASS_COUNT; ++i) acc[i] = fl_prof_entry_t{i, 0, 0.0, 0.0, 0.0, 0.0};
  const bool any = !P.pending.empty();
  for (ProfEvent &ev : P.pending) {
    hipError_t e = hipEventSynchronize(ev.b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
    if (e != hipSuccess) return (fl_status_t)set_error(FL_ERR_DEVICE, "event timing: %s", hipGetErrorString(e));
    acc[ev.cls].launches++;
    acc[ev.cls].total_ms += ms;
    acc[ev.cls].flops += ev.flops;
    acc[ev.cls].bytes += ev.bytes;
    P.pool.push_back(ev.a);
    P.pool.push_back(ev.b);
  }
  P.pending.clear();
  // What a pair of events reads with nothing between them on the same stream: the part of every
  // bracket that is not the kernel.  Smallest of 16 back-to-back pairs.
  double empty_ms = 0.0;
  if (any) {
    hipEvent_t ea = P.get(), eb = P.get();
    if (!ea || !eb) return (fl_status_t)set_error(FL_ERR_DEVICE, "event creation failed");
    float best = -1.f;
    for (int i = 0; i < 16; ++i) {
      float ms = 0.f;
      hipError_t e = hipEventRecord(ea, P.last_stream);
      if (e == hipSuccess) e = hipEventRecord(eb, P.last_stream);
      if (e == hipSuccess) e = hipEventSynchronize(eb);
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, ea, eb);
      if (e != hipSuccess) return (fl_status_t)set_error(FL_ERR_DEVICE, "event timing: %s", hipGetErrorString(e));
      if (best < 0.f || ms < best) best = ms;
    }
    P.pool.push_back(ea);
    P.pool.push_back(eb);
    empty_ms = best;
  }
  int k = 0;
  for (int i = 0; i < FL_K_CLASS_COUNT && k < cap; ++i)
    if (acc[i].launches) {
      acc[i].empty_bracket_ms = empty_ms;
      out[k++] = acc[i];
    }
  *n = k;
  return FL_OK;
  FL_GUARD_END
}

#ifdef FL_TEST_EXPORTS
// Test build only (declared in include/fl_test.h).
int32_t fl_test_layer_peek_linear(fl_layer_t *layer, int32_t lin, void *dst, uint64_t cap_bytes, uint64_t *bytes,
                                  void *hip_stream) {
  FL_GUARD_BEGIN
  if (!layer || !dst || !bytes) return set_error(FL_ERR_INVALID_ARG, "null argument");
  if (!layer->tape.recorded) return set_error(FL_ERR_STATE, "no recorded forward to look into");
  for (const Node &n : layer->tape.nodes) {
    if (n.op != OP_LINEAR || n.param != lin) continue;
    const size_t nb = (size_t)n.rows * n.n_out * esize(layer);
    *bytes = nb;
    if (nb > cap_bytes) return set_error(FL_ERR_INVALID_ARG, "destination holds %llu bytes, the value has %zu",
                                         (unsigned long long)cap_bytes, nb);
    FL_HIP(hipMemcpyAsync(dst, layer->tape.slots[n.out].value, nb, hipMemcpyDeviceToDevice,
                          static_cast<hipStream_t>(hip_stream)));
    return FL_OK;
  }
  return set_error(FL_ERR_INVALID_ARG, "the recorded forward has no linear operator %d", lin);
  FL_GUARD_END
}
#endif

}  // extern "C"
