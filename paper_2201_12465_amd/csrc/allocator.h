// Caching device allocator (host code, no HIP dependency: the backing store is a
// pair of function pointers so that unit tests can run it over a fake store).
//
// Follows the paper's memory-manager interface (Section 4.1.2 and the
// CachingMemoryManager listing: alloc(...) hands out a buffer, unlock(ptr) gives
// it back without returning it to the device) and the behaviour Section 5.2.2
// describes: freed blocks are cached by rounded size and reused, large cached
// blocks may be split to serve smaller requests, and a tunable limit stops
// blocks above a given size from being split.
//
// Buffers are reused in stream order: a block released while kernels that use it
// are still queued is only handed out again for work on the same stream, so the
// queued kernels finish first (Section 4.1.2: buffers are used asynchronously
// and are not freed until computation is complete).
#pragma once
#include <cstddef>
#include <cstdint>
#include <map>
#include <mutex>
#include <unordered_map>
#include <utility>
#include <vector>

namespace fl {

struct AllocStats {
  uint64_t backing_mallocs = 0, backing_bytes = 0, cache_hits = 0, cache_misses = 0;
  uint64_t live_bytes = 0, peak_bytes = 0, cached_bytes = 0, split_count = 0;
  uint64_t requested_bytes = 0;     // sum of the sizes asked for by the live blocks (<= live_bytes)
  uint64_t largest_free_block = 0;  // largest cached block: cached_bytes - this cannot serve one request
  uint64_t free_blocks = 0;         // number of cached blocks
};

// One entry of the allocation trace: ties an allocation to the operator that asked for it
// (Section 5.2.2: telemetry that tied individual tensor operations to specific allocations).
struct AllocEvent {
  uint64_t seq;        // running number of the event
  uint64_t ptr;        // address handed out / given back
  uint64_t requested;  // bytes asked for (0 for a release)
  uint64_t granted;    // size of the block
  int32_t tag;         // operator tag passed to alloc() (release: the tag the block was allocated with)
  int32_t kind;        // 0 = served from the cache, 1 = needed a backing allocation, 2 = release
};

// Returns 0 on success and stores the pointer; non-zero = out of memory.
typedef int (*backing_malloc_fn)(void **ptr, size_t bytes);
typedef int (*backing_free_fn)(void *ptr);

class CachingAllocator {
 public:
  static constexpr size_t kAlign = 512;          // every block size is a multiple of this
  static constexpr size_t kSmall = 1u << 20;      // requests up to 1 MiB come from 2 MiB slabs
  static constexpr size_t kSlabRound = 2u << 20;  // backing allocations are multiples of 2 MiB

  CachingAllocator(backing_malloc_fn m, backing_free_fn f) : bmalloc_(m), bfree_(f) {}
  ~CachingAllocator();
  CachingAllocator(const CachingAllocator &) = delete;
  CachingAllocator &operator=(const CachingAllocator &) = delete;

  // nullptr when the backing store is exhausted (after one attempt to free cached slabs).
  void *alloc(size_t bytes, const void *stream, int tag = 0);
  // Gives a block back to the cache.  Returns false if ptr is not a live block.
  bool release(void *ptr);
  // Frees every slab that is entirely unused.  Caller synchronises the device first.
  void trim();
  void set_split_limit(size_t bytes) {
    std::lock_guard<std::mutex> g(mu_);
    split_limit_ = bytes;
  }
  AllocStats stats() const;
  // Trace: a ring of the most recent `capacity` events (0 switches it off and drops what it holds).
  void trace_enable(size_t capacity);
  // Moves up to cap of the oldest recorded events to out and returns how many.
  size_t trace_read(AllocEvent *out, size_t cap);
  void set_backing(backing_malloc_fn m, backing_free_fn f) {
    std::lock_guard<std::mutex> g(mu_);
    bmalloc_ = m;
    bfree_ = f;
  }

 private:
  struct Block {
    char *ptr;
    size_t size;
    bool free;
    const void *stream;
    Block *prev, *next;  // address-ordered neighbours inside the slab
    void *slab;
    size_t requested = 0;
    int tag = 0;
  };
  typedef std::pair<const void *, size_t> Key;  // (stream, size)
  typedef std::multimap<Key, Block *> FreeMap;

  void free_insert(Block *b);
  void free_erase(Block *b);
  void trim_locked();

  mutable std::mutex mu_;
  backing_malloc_fn bmalloc_;
  backing_free_fn bfree_;
  FreeMap free_map_;
  std::unordered_map<Block *, FreeMap::iterator> free_pos_;
  std::unordered_map<void *, Block *> live_;
  std::unordered_map<void *, size_t> slabs_;  // slab base -> size
  size_t split_limit_ = 0;
  AllocStats st_;
  void trace_push(const AllocEvent &e);
  std::vector<AllocEvent> trace_;  // ring buffer
  size_t trace_cap_ = 0, trace_head_ = 0, trace_count_ = 0;
  uint64_t seq_ = 0;
};

}  // namespace fl
