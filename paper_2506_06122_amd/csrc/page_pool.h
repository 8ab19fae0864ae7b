// Host-side paged KV allocator: a free list of page ids with reference counts and a
// reservation counter.  Pages of a prompt's prefix are shared by its samples through the
// reference count; a sample reserves its worst-case private pages at admission so that a
// decode step can never run out (requests are added according to resource availability:
// paper section 4.1, "Rollout Scheduler").
#pragma once
#include <cstdint>
#include <vector>

struct rollout_pool {
  std::vector<int32_t> free_list;   // stack; lowest ids on top at start
  std::vector<int32_t> refcount;
  int32_t reserved = 0;             // free pages promised to admitted samples
  int32_t peak_in_use = 0;

  explicit rollout_pool(int32_t n_pages) : refcount(n_pages > 0 ? n_pages : 0, 0) {
    free_list.reserve(refcount.size());
    for (int32_t i = (int32_t)refcount.size() - 1; i >= 0; --i) free_list.push_back(i);
  }
  int32_t total() const { return (int32_t)refcount.size(); }
  int32_t free_pages() const { return (int32_t)free_list.size(); }
  int32_t in_use() const { return total() - free_pages(); }
  int32_t unreserved() const { return free_pages() - reserved; }
  bool reserve(int32_t n) {
    if (n < 0 || n > unreserved()) return false;
    reserved += n;
    return true;
  }
  void unreserve(int32_t n) { reserved = n > reserved ? 0 : reserved - n; }
  // from_reservation: the page was promised earlier (always succeeds if promises were kept);
  // otherwise it must come out of the unreserved part.
  int32_t alloc(bool from_reservation) {
    if (from_reservation) {
      if (reserved <= 0 || free_list.empty()) return -1;
      --reserved;
    } else if (unreserved() <= 0) {
      return -1;
    }
    int32_t p = free_list.back();
    free_list.pop_back();
    refcount[p] = 1;
    if (in_use() > peak_in_use) peak_in_use = in_use();
    return p;
  }
  int32_t retain(int32_t p) {
    if (p < 0 || p >= total() || refcount[p] <= 0) return -1;
    return ++refcount[p];
  }
  int32_t release(int32_t p) {
    if (p < 0 || p >= total() || refcount[p] <= 0) return -1;
    if (--refcount[p] == 0) free_list.push_back(p);
    return refcount[p];
  }
};

// Page plan of one prompt with its samples; see rollout_plan_pages in rollout.h.
inline int64_t plan_pages(int32_t prompt_len, int32_t page_tokens, int32_t n_samples,
                          const int32_t* max_new, int32_t* shared, int32_t* tail,
                          int32_t* private_pages) {
  int32_t full = prompt_len / page_tokens;
  int32_t has_tail = (prompt_len % page_tokens) ? 1 : 0;
  int64_t total = full + has_tail;
  for (int32_t j = 0; j < n_samples; ++j) {
    // a sample that emits m tokens feeds m - 1 of them back: prompt_len + m - 1 cached positions
    int64_t cached = (int64_t)prompt_len + max_new[j] - 1;
    int32_t priv = max_new[j] <= 1 ? 0 : (int32_t)((cached + page_tokens - 1) / page_tokens - full);
    if (private_pages) private_pages[j] = priv;
    total += priv;
  }
  if (shared) *shared = full;
  if (tail) *tail = has_tail;
  return total;
}
