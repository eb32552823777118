// Caching device allocator: see allocator.h for the behaviour it follows
// (paper Section 4.1.2, CachingMemoryManager listing, Section 5.2.2).
#include "allocator.h"

namespace fl {

static inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

CachingAllocator::~CachingAllocator() {
  // Device memory is reclaimed by the driver at process exit; calling into the
  // HIP runtime from a static destructor is not safe, so slabs are left alone.
  for (auto &kv : live_) delete kv.second;
  for (auto &kv : free_pos_) delete kv.first;
}

void CachingAllocator::free_insert(Block *b) {
  b->free = true;
  free_pos_[b] = free_map_.emplace(Key(b->stream, b->size), b);
  st_.cached_bytes += b->size;
}

void CachingAllocator::free_erase(Block *b) {
  auto it = free_pos_.find(b);
  free_map_.erase(it->second);
  free_pos_.erase(it);
  st_.cached_bytes -= b->size;
  b->free = false;
}

void *CachingAllocator::alloc(size_t bytes, const void *stream, int tag) {
  std::lock_guard<std::mutex> g(mu_);
  size_t need = round_up(bytes ? bytes : 1, kAlign);
  Block *b = nullptr;
  bool from_backing = false;
  // best fit among this stream's cached blocks
  auto it = free_map_.lower_bound(Key(stream, need));
  if (it != free_map_.end() && it->first.first == stream) {
    Block *c = it->second;
    // a block that may not be split is only taken if it wastes less than half of itself
    bool splittable = split_limit_ == 0 || c->size <= split_limit_;
    if (splittable || c->size - need < c->size / 2) {
      b = c;
      free_erase(b);
      st_.cache_hits++;
    }
  }
  if (!b) {
    st_.cache_misses++;
    size_t slab = need <= kSmall ? kSlabRound : round_up(need, kSlabRound);
    void *p = nullptr;
    if (bmalloc_(&p, slab) != 0 || !p) {
      trim_locked();  // give cached slabs back and retry once
      p = nullptr;
      if (bmalloc_(&p, slab) != 0 || !p) return nullptr;
    }
    st_.backing_mallocs++;
    from_backing = true;
    st_.backing_bytes += slab;
    slabs_[p] = slab;
    b = new Block{static_cast<char *>(p), slab, false, stream, nullptr, nullptr, p};
  }
  // split off the tail if it is worth keeping and the block may be split
  bool may_split = split_limit_ == 0 || b->size <= split_limit_;
  if (may_split && b->size - need >= kAlign) {
    Block *rest = new Block{b->ptr + need, b->size - need, false, stream, b, b->next, b->slab};
    if (b->next) b->next->prev = rest;
    b->next = rest;
    b->size = need;
    free_insert(rest);
    st_.split_count++;
  }
  b->stream = stream;
  b->requested = bytes;
  b->tag = tag;
  live_[b->ptr] = b;
  st_.live_bytes += b->size;
  st_.requested_bytes += bytes;
  if (trace_cap_)
    trace_push(AllocEvent{0, reinterpret_cast<uint64_t>(b->ptr), bytes, b->size, tag, from_backing ? 1 : 0});
  if (st_.live_bytes > st_.peak_bytes) st_.peak_bytes = st_.live_bytes;
  return b->ptr;
}

bool CachingAllocator::release(void *ptr) {
  std::lock_guard<std::mutex> g(mu_);
  auto it = live_.find(ptr);
  if (it == live_.end()) return false;
  Block *b = it->second;
  live_.erase(it);
  st_.live_bytes -= b->size;
  st_.requested_bytes -= b->requested;
  if (trace_cap_) trace_push(AllocEvent{0, reinterpret_cast<uint64_t>(b->ptr), 0, b->size, b->tag, 2});
  // merge with free neighbours that belong to the same stream
  if (b->next && b->next->free && b->next->stream == b->stream) {
    Block *n = b->next;
    free_erase(n);
    b->size += n->size;
    b->next = n->next;
    if (n->next) n->next->prev = b;
    delete n;
  }
  if (b->prev && b->prev->free && b->prev->stream == b->stream) {
    Block *p = b->prev;
    free_erase(p);
    p->size += b->size;
    p->next = b->next;
    if (b->next) b->next->prev = p;
    delete b;
    b = p;
  }
  free_insert(b);
  return true;
}

void CachingAllocator::trim_locked() {
  std::vector<Block *> whole;
  for (auto &kv : free_pos_) {
    Block *b = kv.first;
    if (!b->prev && !b->next) whole.push_back(b);  // the block spans its slab
  }
  for (Block *b : whole) {
    free_erase(b);
    bfree_(b->slab);
    st_.backing_bytes -= slabs_[b->slab];
    slabs_.erase(b->slab);
    delete b;
  }
}

AllocStats CachingAllocator::stats() const {
  std::lock_guard<std::mutex> g(mu_);
  AllocStats s = st_;
  s.free_blocks = free_map_.size();
  s.largest_free_block = 0;
  for (const auto &kv : free_map_)
    if (kv.first.second > s.largest_free_block) s.largest_free_block = kv.first.second;
  return s;
}

void CachingAllocator::trace_push(const AllocEvent &e) {
  AllocEvent ev = e;
  ev.seq = seq_++;
  const size_t pos = (trace_head_ + trace_count_) % trace_cap_;
  trace_[pos] = ev;
  if (trace_count_ < trace_cap_) trace_count_++;
  else trace_head_ = (trace_head_ + 1) % trace_cap_;  // the oldest entry is overwritten
}

void CachingAllocator::trace_enable(size_t capacity) {
  std::lock_guard<std::mutex> g(mu_);
  trace_.assign(capacity, AllocEvent{});
  trace_cap_ = capacity;
  trace_head_ = trace_count_ = 0;
}

size_t CachingAllocator::trace_read(AllocEvent *out, size_t cap) {
  std::lock_guard<std::mutex> g(mu_);
  size_t n = 0;
  while (n < cap && trace_count_ > 0) {
    out[n++] = trace_[trace_head_];
    trace_head_ = (trace_head_ + 1) % trace_cap_;
    trace_count_--;
  }
  return n;
}

void CachingAllocator::trim() {
  std::lock_guard<std::mutex> g(mu_);
  trim_locked();
}

}  // namespace fl
