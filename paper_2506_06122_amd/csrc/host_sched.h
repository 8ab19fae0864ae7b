// Host-side state and bookkeeping of the rollout scheduler - the sample table, live-sample slots,
// page tables, the prompt queue and every decision that adds, grows or releases a request
// (paper section 4.1, "Rollout Scheduler": requests are added according to resource
// availability; section 4.3: add request / abort request at sample level).  Nothing here touches
// the GPU or includes a HIP header: rollout_ctx derives from HostState and api.hip drives the
// launches around these functions, and a CPU-only driver (tests/host/sched_driver.cpp) runs the
// same code under the address and undefined-behaviour sanitizers.
#pragma once
#include <algorithm>
#include <cstdint>
#include <deque>
#include <map>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/rollout.h"
#include "page_pool.h"

struct ApiError {
  int code;
  std::string msg;
};

inline int ceil_div_i(long long a, long long b) { return (int)((a + b - 1) / b); }

struct Sample {
  int64_t id;
  int slot;
  int prompt_len, n_emitted, max_new, eos_id;  // prompt_len: every cached token that is not a response token
  int last_token = -1;                         // the response token emitted last (not cached yet)
  int64_t group = -1;                          // the prompt's counter: samples of one prompt share its full pages
  int shared_len = 0;                          // positions held in those shared pages (a multiple of page_tokens)
  std::vector<int32_t> pages;  // one reference held on each
};

// Prompts waiting for admission and the bookkeeping of the queue-fed rollout.
struct QueuedPrompt {
  int64_t prompt_id;     // the prompt's counter (what its samples' `group` will be)
  int64_t first_sample;  // id of its sample 0; sample j carries first_sample + j
  std::vector<int32_t> tokens, max_new;  // max_new: one per sample
  int eos_id;
  float temperature, top_p;
};
// The shared pages of one admitted prompt while its prefill runs (the caller releases these
// references when the samples hold their own).
struct PromptPages {
  std::vector<int32_t> shared;
  int32_t tail = -1;
};
// A prompt whose prefill is spread over several queue steps (chunked prefill).  Everything it will
// hold is taken when it is admitted - the prompt's pages, its samples' slots and pages - so that a
// prompt once begun can always finish; its samples go live when its last chunk is cached.
struct PendingPrompt {
  QueuedPrompt prompt;
  int table_row = -1;          // the page-table row its prefill writes through
  int done = 0;                // prompt positions cached so far
  PromptPages pages;
  std::vector<Sample> samples;
  std::vector<int> copy_pairs;     // (source, destination) pages: private copies of the partial last page
  std::vector<int32_t> page_refs;  // every page reference taken at admission
  std::vector<int> slots;          // every live-sample slot taken at admission
};
struct PromptQueue {
  std::deque<QueuedPrompt> waiting;
  int chunk_rows = 0;               // > 0: chunked prefill, at most this many prompt rows per step
  std::deque<PendingPrompt> pending;  // admitted, prefill not complete (push order)
  std::vector<int> free_rows;       // page-table rows for pending prompts
  int n_samples = 0;      // fixed by the first push
  int admit_min = 1;      // admit only when this many waiting prompts fit (or nothing is live)
  int target = 0;         // close the queue once this many prompts are complete; 0 = never
  bool closed = false;
  std::unordered_map<int64_t, int> open;            // admitted prompt -> samples not ended yet
  std::unordered_map<int64_t, QueuedPrompt> admitted;  // admitted prompts kept while they can be preempted (growing pages)
  uint64_t pushed = 0, admitted_count = 0, completed = 0, aborted = 0, preempted = 0;
};

struct HostState {
  int page_tokens = 32, max_pages = 0, max_context = 0;
  bool grow_pages = false;       // pages are taken as contexts grow instead of all at admission
  rollout_pool* pool = nullptr;
  std::vector<int> h_page_table;  // [slot][max_pages]
  std::vector<int> free_slots;
  std::map<int64_t, Sample> live;
  int64_t prompt_counter = 0;   // prompts ever admitted or queued
  int64_t next_sample_id = 0;   // ids are handed out consecutively, n per prompt, at prefill or push time
  PromptQueue queue;
  bool live_dirty = true;       // the live set changed since the device copy of it was made
};

// Pages and live-sample slots taken by a call that has not completed yet: given back if the
// call leaves by an exception, so that a failing call changes no state.
struct Rollback {
  HostState& c;
  std::vector<int32_t> page_refs;  // one entry per reference taken (alloc or retain)
  std::vector<int> slots;
  bool armed = true;
  explicit Rollback(HostState& ctx) : c(ctx) {}
  int32_t alloc() {
    const int32_t pg = c.pool->alloc(false);
    if (pg < 0) throw ApiError{ROLLOUT_E_NOMEM, "internal: the KV pool ran out after admission was checked"};
    page_refs.push_back(pg);
    return pg;
  }
  void retain(int32_t pg) {
    c.pool->retain(pg);
    page_refs.push_back(pg);
  }
  int take_slot() {
    const int sl = c.free_slots.back();
    c.free_slots.pop_back();
    slots.push_back(sl);
    return sl;
  }
  void commit() { armed = false; }
  ~Rollback() {
    if (!armed) return;
    for (int32_t pg : page_refs) c.pool->release(pg);
    for (auto it = slots.rbegin(); it != slots.rend(); ++it) c.free_slots.push_back(*it);
  }
};

inline void release_sample(HostState& c, Sample& s) {
  for (int32_t p : s.pages) c.pool->release(p);
  s.pages.clear();
  if (s.slot >= 0) c.free_slots.push_back(s.slot);
  s.slot = -1;
}

// Pages a sample holds once it has `cached` positions in its cache.
inline int pages_for(const HostState& c, long long cached) { return ceil_div_i(cached, c.page_tokens); }

// Pages one prompt with its samples takes at admission: everything it can ever need (default), or,
// with growing pages, the prompt's pages plus for every running sample the page its first fed
// token goes to.
inline long long admission_pages(const HostState& c, int prompt_len, int n, const int32_t* max_new) {
  if (!c.grow_pages) return plan_pages(prompt_len, c.page_tokens, n, max_new, nullptr, nullptr, nullptr);
  const int full = prompt_len / c.page_tokens, has_tail = (prompt_len % c.page_tokens) != 0;
  long long total = full + has_tail;
  for (int j = 0; j < n; ++j)
    if (max_new[j] > 1) total += pages_for(c, (long long)prompt_len + 1) - full;
  return total;
}
inline int admission_slots(int n, const int32_t* max_new) {
  int s = 0;
  for (int j = 0; j < n; ++j) s += max_new[j] > 1;
  return s;
}

// Takes the pages and slots of prompt p (length len, counter `group`, first sample id `first`) and
// fills fresh[0..n): the prompt's full pages once, shared by reference; a private copy target for
// the partial last page of every running sample (copy_pairs: source, destination); the sample's
// own pages up to its initial cache size.  prompt_row: the page-table row the prefill itself uses.
inline void take_prompt_pages(HostState& c, Rollback& undo, int len, int n, const int32_t* max_new, int eos_id,
                              int64_t group, int64_t first, int prompt_row, PromptPages& pp, Sample* fresh,
                              std::vector<int>& copy_pairs) {
  const int T = c.page_tokens;
  const int full = len / T, has_tail = (len % T) != 0;
  int* prow = &c.h_page_table[(size_t)prompt_row * c.max_pages];
  for (int i = 0; i < full; ++i) {
    const int32_t pg = undo.alloc();
    pp.shared.push_back(pg);
    prow[i] = pg;
  }
  if (has_tail) {
    pp.tail = undo.alloc();
    prow[full] = pp.tail;
  }
  for (int j = 0; j < n; ++j) {
    Sample& s = fresh[j];
    s.group = group;
    s.id = first + j;
    s.shared_len = full * T;
    s.slot = -1;
    s.prompt_len = len;
    s.n_emitted = 0;
    s.max_new = max_new[j];
    s.eos_id = eos_id;
    s.pages.clear();
    if (s.max_new <= 1) continue;
    s.slot = undo.take_slot();
    int* srow = &c.h_page_table[(size_t)s.slot * c.max_pages];
    for (int i = 0; i < full; ++i) {
      undo.retain(pp.shared[i]);
      s.pages.push_back(pp.shared[i]);
      srow[i] = pp.shared[i];
    }
    const int total = c.grow_pages ? pages_for(c, (long long)len + 1) : pages_for(c, (long long)len + s.max_new - 1);
    for (int i = full; i < total; ++i) {
      const int32_t pg = undo.alloc();
      s.pages.push_back(pg);
      srow[i] = pg;
    }
    if (has_tail) {
      copy_pairs.push_back(pp.tail);
      copy_pairs.push_back(srow[full]);
    }
  }
}

// One page-table entry that changed on the host and has to reach the device copy.
struct PagePatch {
  int slot, index, page;
};

// Growing pages: the pages the next decode step writes to.  Sample s feeds its last token at
// position prompt_len + n_emitted - 1; when that position starts a page the sample does not hold
// yet, one is needed.  Returns the number of pages missing in all.
inline int pages_missing_for_step(const HostState& c) {
  int need = 0;
  for (const auto& kv : c.live) {
    const Sample& s = kv.second;
    need += pages_for(c, (long long)s.prompt_len + s.n_emitted) > (int)s.pages.size();
  }
  return need;
}
// Takes them (the caller has checked that the pool holds enough) and lists the table entries to patch.
inline void grow_pages_for_step(HostState& c, std::vector<PagePatch>& patches) {
  for (auto& kv : c.live) {
    Sample& s = kv.second;
    while (pages_for(c, (long long)s.prompt_len + s.n_emitted) > (int)s.pages.size()) {
      const int32_t pg = c.pool->alloc(false);
      if (pg < 0) throw ApiError{ROLLOUT_E_NOMEM, "internal: the KV pool ran out after the step was checked"};
      c.h_page_table[(size_t)s.slot * c.max_pages + s.pages.size()] = pg;
      patches.push_back(PagePatch{s.slot, (int)s.pages.size(), pg});
      s.pages.push_back(pg);
    }
  }
}

// ---- prompt queue -------------------------------------------------------------------------------
// a sample of prompt `group` has ended (finished, or aborted by the caller): the prompt is
// complete when its last one ends
inline void queue_note_finished(PromptQueue& q, int64_t group) {
  auto it = q.open.find(group);
  if (it == q.open.end()) return;  // admitted through rollout_prefill, not through the queue
  if (--it->second == 0) {
    q.open.erase(it);
    q.admitted.erase(group);
    q.completed += 1;
  }
}

struct AdmissionLimits {
  int max_prompts;        // prompts one prefill call takes
  long long max_samples;  // rows of the sampling workspace
};

// The longest run of waiting prompts, in push order, that one prefill call can take now: same
// sampling parameters, and slots and pages for all of them.  With growing pages a run is also cut
// where the pool would be left without one spare page per live sample (the next steps' growth).
// Returns the number of prompts; 0 when the policy says to wait (fewer than admit_min fit while
// samples are live).
inline int queue_select_run(const HostState& c, const AdmissionLimits& lim) {
  const PromptQueue& q = c.queue;
  const int n = q.n_samples;
  int k = 0, slots = 0;
  long long pages = 0;
  while (k < (int)q.waiting.size()) {
    const QueuedPrompt& e = q.waiting[k];
    const QueuedPrompt& head = q.waiting[0];
    if (e.eos_id != head.eos_id || e.temperature != head.temperature || e.top_p != head.top_p) break;
    const int s1 = admission_slots(n, e.max_new.data());
    const long long p1 = admission_pages(c, (int)e.tokens.size(), n, e.max_new.data());
    if (slots + s1 > (int)c.free_slots.size()) break;
    const long long spare = c.grow_pages ? (long long)c.live.size() + slots + s1 : 0;
    if (pages + p1 + spare > c.pool->unreserved()) break;
    if (k + 1 > lim.max_prompts || (long long)(k + 1) * n > lim.max_samples) break;
    slots += s1;
    pages += p1;
    ++k;
  }
  if (k < std::min<int>(q.admit_min, (int)q.waiting.size()) && !c.live.empty()) k = 0;
  return k;
}

// Growing pages, the pool is exhausted: the most recently admitted queued prompt that still has
// live samples gives way.  Its live samples are dropped (pages and slots return) and the prompt
// goes back to the head of the queue; it restarts from its prompt later, with the same sample ids
// and therefore the same tokens.  Returns the number of samples dropped, 0 when no queued prompt
// is live (then the caller has to abort something itself).
inline int queue_preempt_youngest(HostState& c, std::vector<int64_t>* dropped_ids) {
  PromptQueue& q = c.queue;
  int64_t victim = -1;
  for (const auto& kv : c.live)
    if (q.admitted.count(kv.second.group)) victim = std::max(victim, kv.second.group);
  if (victim < 0) return 0;
  int dropped = 0;
  for (auto it = c.live.begin(); it != c.live.end();) {
    if (it->second.group == victim) {
      if (dropped_ids) dropped_ids->push_back(it->first);
      release_sample(c, it->second);
      it = c.live.erase(it);
      ++dropped;
    } else {
      ++it;
    }
  }
  auto node = q.admitted.find(victim);
  q.waiting.push_front(std::move(node->second));
  q.admitted.erase(node);
  q.open.erase(victim);
  q.admitted_count -= 1;
  q.preempted += 1;
  c.live_dirty = true;
  return dropped;
}

// ---- chunked prefill ------------------------------------------------------------------------------
inline long long pending_rows_left(const PromptQueue& q) {
  long long rows = 0;
  for (const PendingPrompt& p : q.pending) rows += (long long)p.prompt.tokens.size() - p.done;
  return rows;
}

// The head of the queue becomes a pending prompt: its pages and its samples' slots and pages are
// taken now (the caller has checked with queue_select_run that they are there).  Leaves the queue
// untouched when it throws.
inline void queue_admit_pending(HostState& c) {
  PromptQueue& q = c.queue;
  if (q.waiting.empty() || q.free_rows.empty()) throw ApiError{ROLLOUT_E_STATE, "internal: nothing to admit"};
  const QueuedPrompt& e = q.waiting.front();
  const int n = q.n_samples;
  PendingPrompt pp;
  pp.table_row = q.free_rows.back();
  pp.samples.resize((size_t)n);
  {
    Rollback undo(c);
    take_prompt_pages(c, undo, (int)e.tokens.size(), n, e.max_new.data(), e.eos_id, e.prompt_id, e.first_sample,
                      pp.table_row, pp.pages, pp.samples.data(), pp.copy_pairs);
    pp.page_refs = std::move(undo.page_refs);
    pp.slots = std::move(undo.slots);
    undo.commit();
  }
  pp.prompt = std::move(q.waiting.front());
  q.waiting.pop_front();
  q.free_rows.pop_back();
  q.pending.push_back(std::move(pp));
  q.admitted_count += 1;
}

// Gives back everything a pending prompt holds (it never went live).
inline void release_pending(HostState& c, PendingPrompt& pp) {
  for (int32_t pg : pp.page_refs) c.pool->release(pg);
  for (auto it = pp.slots.rbegin(); it != pp.slots.rend(); ++it) c.free_slots.push_back(*it);
  pp.page_refs.clear();
  pp.slots.clear();
  for (Sample& s : pp.samples) {
    s.pages.clear();
    s.slot = -1;
  }
  c.queue.free_rows.push_back(pp.table_row);
  pp.table_row = -1;
}

// Growing pages, the pool is exhausted: the youngest pending prompt returns to the head of the
// queue and starts over later.  False when nothing is pending.
inline bool queue_preempt_pending(HostState& c) {
  PromptQueue& q = c.queue;
  if (q.pending.empty()) return false;
  PendingPrompt& pp = q.pending.back();
  release_pending(c, pp);
  q.waiting.push_front(std::move(pp.prompt));
  q.pending.pop_back();
  q.admitted_count -= 1;
  q.preempted += 1;
  return true;
}

// The prompt rows of one step: pending prompts in order, `budget` rows in all, the last one cut
// where the budget ends.  At most max_finishing prompts may reach their end in this step (each
// needs a logits row); one more is cut one row short.
struct ChunkSeq {
  int pending_index, begin, len;
  bool last;  // the chunk ends the prompt
};
inline int plan_chunk(const PromptQueue& q, long long budget, int max_finishing, std::vector<ChunkSeq>& out) {
  int rows = 0, finishing = 0;
  for (int i = 0; i < (int)q.pending.size() && budget > 0; ++i) {
    const PendingPrompt& p = q.pending[i];
    const int left = (int)p.prompt.tokens.size() - p.done;
    int take = (int)std::min<long long>(left, budget);
    if (take == left && finishing == max_finishing) --take;
    if (take <= 0) break;
    const bool last = take == left;
    finishing += last;
    out.push_back(ChunkSeq{i, p.done, take, last});
    rows += take;
    budget -= take;
    if (!last) break;  // prompts are cached in order: nothing starts behind an unfinished one
  }
  return rows;
}
