// Process-wide pieces shared by the C-ABI translation units.
#pragma once
#include "allocator.h"

namespace fl {
// Stores a printf-style message for fl_last_error() on this thread and returns `code`.
int set_error(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
// The caching allocator over hipMalloc/hipFree that every layer handle shares.
CachingAllocator &device_allocator();
}  // namespace fl
