// Host-side page bookkeeping: a lowest-index-first page allocator over free intervals and the
// planner that merges page copies into long runs (PipeMax Sec. 3.4.2: with the block-first
// layout a prefetch is sliced along the block dimension only, so consecutive pages of a
// sequence form one contiguous transfer).
#pragma once

#include <algorithm>
#include <iterator>
#include <map>
#include <vector>
#include <stdint.h>

namespace pmx {

class PagePool {
 public:
  explicit PagePool(int n_pages) : total_(n_pages), free_(n_pages) {
    if (n_pages > 0) iv_[0] = n_pages;
  }
  int total() const { return total_; }
  int free_count() const { return free_; }

  // Takes the n lowest free page indices (all or nothing).
  bool alloc(int n, int32_t* out) {
    if (n < 0 || n > free_) return false;
    int got = 0;
    while (got < n) {
      auto it = iv_.begin();
      int start = it->first, len = it->second;
      int take = (n - got < len) ? (n - got) : len;
      for (int i = 0; i < take; ++i) out[got + i] = start + i;
      got += take;
      iv_.erase(it);
      if (take < len) iv_[start + take] = len - take;
    }
    free_ -= n;
    return true;
  }

  // Returns pages to the pool.  Returns false (pool unchanged) if any page is out of range or
  // already free, or if the list holds a duplicate.
  bool release(const int32_t* pages, int n) {
    for (int i = 0; i < n; ++i)
      if (pages[i] < 0 || pages[i] >= total_ || is_free(pages[i])) return false;
    std::vector<int32_t> s(pages, pages + n);
    std::sort(s.begin(), s.end());
    for (int i = 1; i < n; ++i)
      if (s[i] == s[i - 1]) return false;
    int i = 0;
    while (i < n) {
      int j = i;
      while (j + 1 < n && s[j + 1] == s[j] + 1) ++j;
      insert_interval(s[i], j - i + 1);
      i = j + 1;
    }
    free_ += n;
    return true;
  }

  bool is_free(int page) const {
    auto it = iv_.upper_bound(page);
    if (it == iv_.begin()) return false;
    --it;
    return page < it->first + it->second;
  }

 private:
  void insert_interval(int start, int len) {
    auto nxt = iv_.lower_bound(start);
    if (nxt != iv_.begin()) {
      auto prv = std::prev(nxt);
      if (prv->first + prv->second == start) {
        start = prv->first;
        len += prv->second;
        iv_.erase(prv);
      }
    }
    if (nxt != iv_.end() && nxt->first == start + len) {
      len += nxt->second;
      iv_.erase(nxt);
    }
    iv_[start] = len;
  }

  int total_, free_;
  std::map<int, int> iv_;   // start -> length of each free interval
};

struct CopyRun {
  int32_t src, dst, count;
};

// Merges (src, dst) page pairs, in the order given, into runs of consecutive pages.
inline void plan_copy_runs(const int32_t* src, const int32_t* dst, int n, int max_run,
                           std::vector<CopyRun>& out) {
  out.clear();
  for (int i = 0; i < n; ++i) {
    if (!out.empty()) {
      CopyRun& r = out.back();
      if (r.count < max_run && src[i] == r.src + r.count && dst[i] == r.dst + r.count) {
        ++r.count;
        continue;
      }
    }
    out.push_back(CopyRun{src[i], dst[i], 1});
  }
}

}  // namespace pmx
