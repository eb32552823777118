// Minimal reverse-mode tape (host code, header only).
//
// The paper's autograd wraps a tensor in a Variable, records every operator on a
// dynamic tape together with a gradient function, and backward() walks the tape
// in reverse, each gradient function adding into its inputs' gradients
// (Section 4.2 "Automatic Differentiation" and the cosine-operator listing).
// Section 5.2.1 lists three customisations made for very large graphs:
// pre-fused gradient computation for common operator sequences, explicit node
// lifetime instead of reference counting, and pruning.  This tape keeps the first
// two: nodes are plain structs in a vector owned by the tape (no per-node
// reference counts), and a value slot can carry *requests* that let the operator
// producing its gradient fuse the next gradient step into its own kernel
// (an activation derivative, a bias-gradient column sum).
//
// The tape knows nothing about kernels: a node's backward is a function pointer.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

namespace fl {

// A device buffer from the caching allocator, shared by the slots that alias it.
struct Buf {
  void *ptr = nullptr;
  size_t bytes = 0;
  int refs = 0;
  bool from_arena = false;  // carved out of the static scratch array instead (allocation-free forward)
};

enum GradXform : int32_t { XF_NONE = 0, XF_RELU = 1, XF_GELU = 2 };

// One value of the forward computation and, during backward, its gradient.
struct Slot {
  // forward
  const void *value = nullptr;  // device pointer of the value (may be caller-owned)
  Buf *value_buf = nullptr;     // set if the library owns the value
  int first_consumer = -1;      // index of the first node recorded with this slot as input:
                                // in reverse replay it is the LAST one to add to the gradient
  // requests to whoever finishes this slot's gradient (set by the node that produced the value)
  int32_t xform = XF_NONE;         // multiply the finished gradient by act'(aux)
  const void *xform_aux = nullptr;  // pre-activation (GELU) or activation output (ReLU)
  int32_t colsum_param = -1;        // also emit the gradient's column sums as this bias's gradient
  int32_t xform_drop_site = 0;      // also multiply it by the dropout keep mask of this site (0 = none)
  // backward
  void *grad = nullptr;      // gradient accumulated so far (nullptr = none yet)
  Buf *grad_buf = nullptr;   // set if the library owns it
  void *grad_dst = nullptr;  // caller-owned destination the finished gradient must land in
  bool xform_done = false, colsum_done = false;
};

struct Tape;
struct Node {
  typedef int (*BackwardFn)(void *ctx, Tape *tape, const Node *self);  // 0 = ok
  BackwardFn backward = nullptr;
  int32_t op = 0;          // operator id, for diagnostics
  int32_t in0 = -1, in1 = -1;  // input slots (in1: residual / second input, or -1)
  int32_t out = -1;        // output slot
  int32_t param = -1;      // which weight/bias pair or LayerNorm pair this node owns
  int32_t flags = 0;
  // saved tensors (device pointers; owned ones are listed in `saved`)
  const void *s0 = nullptr, *s1 = nullptr, *s2 = nullptr;
  Buf *saved[3] = {nullptr, nullptr, nullptr};
  int32_t rows = 0, n_in = 0, n_out = 0;
};

struct Tape {
  std::vector<Slot> slots;
  std::vector<Node> nodes;
  bool recorded = false;

  int new_slot() {
    slots.emplace_back();
    return static_cast<int>(slots.size()) - 1;
  }
  // Appends a node; notes, for each input slot, the first node that consumes it.
  int record(const Node &n) {
    int id = static_cast<int>(nodes.size());
    nodes.push_back(n);
    for (int s : {n.in0, n.in1})
      if (s >= 0 && slots[s].first_consumer < 0) slots[s].first_consumer = id;
    return id;
  }
  // True if `node` is the one whose backward finishes the gradient of `slot`.
  bool finishes(int node, int slot) const { return slots[slot].first_consumer == node; }
  int index_of(const Node *n) const { return static_cast<int>(n - nodes.data()); }

  // Replays the nodes last-to-first.  Stops at the first failure and returns its code.
  int replay_reverse(void *ctx) {
    for (int i = static_cast<int>(nodes.size()) - 1; i >= 0; --i) {
      int rc = nodes[i].backward ? nodes[i].backward(ctx, this, &nodes[i]) : 0;
      if (rc) return rc;
    }
    return 0;
  }
  void clear() {
    slots.clear();
    nodes.clear();
    recorded = false;
  }
};

}  // namespace fl
