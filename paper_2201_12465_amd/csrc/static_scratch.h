// Static device scratch of the allocation-free entry point (static_scratch.hip).
#pragma once
#include <hip/hip_runtime_api.h>
#include <cstddef>

namespace fl {
// Size of the array each GPU holds: enough for the intermediates of one inference forward pass of every
// benchmark shape (the largest, 12608 tokens x d_model 768 x d_ffn 3072 in bf16, needs 116 MB at its peak).
constexpr size_t kStaticScratchBytes = 128u << 20;
// Device address of the current device's array (looked up on the first call per device, then cached).
// Allocates nothing.
hipError_t static_scratch_base(void **base);
}  // namespace fl
