// Offset allocator over one caller-provided block (device arena or pinned host pool): best-fit free
// list keyed by offset with coalescing.  Host-only integer arithmetic; sizes are multiples of 256.
#pragma once
#include <stdint.h>

#include <map>

class BlockArena {
 public:
  void reset(uint64_t capacity) {
    free_.clear();
    cap_ = capacity;
    high_ = 0;
    if (capacity) free_[0] = capacity;
  }
  // returns UINT64_MAX when no free range fits
  uint64_t alloc(uint64_t bytes) {
    auto best = free_.end();
    for (auto it = free_.begin(); it != free_.end(); ++it)
      if (it->second >= bytes && (best == free_.end() || it->second < best->second)) best = it;
    if (best == free_.end()) return UINT64_MAX;
    uint64_t off = best->first, sz = best->second;
    free_.erase(best);
    if (sz > bytes) free_[off + bytes] = sz - bytes;
    if (off + bytes > high_) high_ = off + bytes;
    return off;
  }
  void release(uint64_t off, uint64_t bytes) {
    auto nxt = free_.lower_bound(off);
    if (nxt != free_.end() && off + bytes == nxt->first) {
      bytes += nxt->second;
      nxt = free_.erase(nxt);
    }
    if (nxt != free_.begin()) {
      auto prv = std::prev(nxt);
      if (prv->first + prv->second == off) {
        prv->second += bytes;
        return;
      }
    }
    free_[off] = bytes;
  }
  uint64_t high_water() const { return high_; }
  uint64_t capacity() const { return cap_; }
  uint64_t largest_free() const {
    uint64_t m = 0;
    for (auto& kv : free_) if (kv.second > m) m = kv.second;
    return m;
  }

 private:
  std::map<uint64_t, uint64_t> free_;
  uint64_t cap_ = 0, high_ = 0;
};
