// Host-side first-fit allocator over a caller-supplied device workspace.
// It hands out offsets only (the device memory itself is never touched by the
// host), is fully deterministic - the same call sequence yields the same
// offsets - and is cheap to copy, so a call can be rehearsed on a copy before
// anything is launched.
#pragma once
#include <stddef.h>

#include <map>

namespace lynx {

class Arena {
 public:
  static constexpr size_t kAlign = 256;

  explicit Arena(size_t capacity = 0) : capacity_(capacity) {
    if (capacity_ > 0) free_[0] = capacity_;
  }

  // Lowest-address block that fits; false when none does.
  bool alloc(size_t bytes, size_t* offset) {
    const size_t need = round_up(bytes == 0 ? 1 : bytes);
    for (auto it = free_.begin(); it != free_.end(); ++it) {
      if (it->second >= need) {
        const size_t off = it->first, rest = it->second - need;
        free_.erase(it);
        if (rest > 0) free_[off + need] = rest;
        used_[off] = need;
        in_use_ += need;
        if (off + need > extent_peak_) extent_peak_ = off + need;
        *offset = off;
        return true;
      }
    }
    return false;
  }

  void release(size_t offset) {
    auto u = used_.find(offset);
    if (u == used_.end()) return;
    size_t off = offset, len = u->second;
    in_use_ -= len;
    used_.erase(u);
    auto next = free_.lower_bound(off);
    if (next != free_.end() && off + len == next->first) {
      len += next->second;
      next = free_.erase(next);
    }
    if (next != free_.begin()) {
      auto prev = next;
      --prev;
      if (prev->first + prev->second == off) {
        off = prev->first;
        len += prev->second;
        free_.erase(prev);
      }
    }
    free_[off] = len;
  }

  size_t in_use() const { return in_use_; }
  size_t extent_peak() const { return extent_peak_; }  // highest byte ever handed out
  size_t capacity() const { return capacity_; }
  static size_t round_up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

 private:
  size_t capacity_ = 0, in_use_ = 0, extent_peak_ = 0;
  std::map<size_t, size_t> free_;  // offset -> length
  std::map<size_t, size_t> used_;  // offset -> length
};

}  // namespace lynx
