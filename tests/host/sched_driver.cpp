// CPU-only driver of the scheduler's host logic (csrc/host_sched.h, csrc/page_pool.h): a random
// walk of pushes, admissions, decode steps, early ends, caller aborts, failing admissions and -
// with growing pages - pool exhaustion and preemption, with the books checked after every step.
// With chunk_rows > 0 prompts are admitted as pending prompts and cached a chunk per step
// (chunked prefill), the half-cached ones giving way first when the pool runs out.
// Built and run by tests/test_host_sanitized.py under -fsanitize=address,undefined; no GPU, no HIP.
//
//   sched_driver <seed> <grow_pages 0|1> <pool pages> <slots> <prompts> [chunk_rows]
#include <cstdio>
#include <cstdlib>
#include <random>
#include <set>

#include "../../paper_2506_06122_amd/csrc/host_sched.h"

#define REQUIRE(cond)                                                       \
  do {                                                                      \
    if (!(cond)) {                                                          \
      std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
      std::exit(1);                                                         \
    }                                                                       \
  } while (0)

static const int kTempSlots = 8;

static void check_books(const HostState& c, int n_slots) {
  std::vector<int> refs(c.pool->total(), 0);
  std::set<int> slots;
  for (const auto& kv : c.live) {
    const Sample& s = kv.second;
    REQUIRE(s.slot >= 0 && s.slot < n_slots && slots.insert(s.slot).second);
    const long long cached = (long long)s.prompt_len + s.n_emitted - 1;
    REQUIRE((int)s.pages.size() >= pages_for(c, cached));
    if (!c.grow_pages) REQUIRE((int)s.pages.size() == pages_for(c, (long long)s.prompt_len + s.max_new - 1));
    REQUIRE((int)s.pages.size() <= c.max_pages);
    for (size_t i = 0; i < s.pages.size(); ++i) {
      REQUIRE(s.pages[i] >= 0 && s.pages[i] < c.pool->total());
      REQUIRE(c.h_page_table[(size_t)s.slot * c.max_pages + i] == s.pages[i]);
      refs[s.pages[i]] += 1;
    }
  }
  for (const PendingPrompt& pp : c.queue.pending) {  // admitted, not live yet: holds what its samples will hold
    REQUIRE(pp.table_row >= n_slots && pp.done >= 0 && pp.done < (int)pp.prompt.tokens.size());
    for (int32_t pg : pp.page_refs) {
      REQUIRE(pg >= 0 && pg < c.pool->total());
      refs[pg] += 1;
    }
    for (int sl : pp.slots) REQUIRE(sl >= 0 && sl < n_slots && slots.insert(sl).second);
  }
  int in_use = 0;
  for (int p = 0; p < c.pool->total(); ++p) {
    REQUIRE(c.pool->refcount[p] == refs[p]);
    in_use += refs[p] > 0;
  }
  REQUIRE(in_use == c.pool->in_use());
  for (int sl : c.free_slots) REQUIRE(slots.insert(sl).second);
  REQUIRE((int)slots.size() == n_slots);
}

int main(int argc, char** argv) {
  const unsigned seed = argc > 1 ? (unsigned)std::atoi(argv[1]) : 1;
  const bool grow = argc > 2 && std::atoi(argv[2]) != 0;
  const int n_pages = argc > 3 ? std::atoi(argv[3]) : 40;
  const int n_slots = argc > 4 ? std::atoi(argv[4]) : 12;
  const int n_prompts = argc > 5 ? std::atoi(argv[5]) : 60;
  const int chunk_rows = argc > 6 ? std::atoi(argv[6]) : 0;
  std::mt19937 rng(seed);
  auto uni = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };

  HostState c;
  c.page_tokens = 32;
  c.max_context = 384;
  c.max_pages = ceil_div_i(c.max_context, c.page_tokens);
  c.grow_pages = grow;
  c.pool = new rollout_pool(n_pages);
  c.h_page_table.assign((size_t)(n_slots + kTempSlots) * c.max_pages, -1);
  for (int s = n_slots - 1; s >= 0; --s) c.free_slots.push_back(s);
  PromptQueue& q = c.queue;
  const int n = uni(1, 3);
  const int early_end = (seed & 1) ? 60 : 2000;  // odd seeds: samples mostly end early; even seeds: they run to their limits
  q.n_samples = n;
  q.admit_min = uni(1, 2);
  q.chunk_rows = chunk_rows;
  for (int i = kTempSlots - 1; i >= 0; --i) q.free_rows.push_back(n_slots + i);

  // ---- pushes: what rollout_queue_push does on the host
  int pushed = 0, refused = 0;
  for (int p = 0; p < n_prompts; ++p) {
    QueuedPrompt e;
    const int len = uni(1, 150);
    e.tokens.assign(len, 7);
    for (int j = 0; j < n; ++j) e.max_new.push_back(uni(1, std::min(200, c.max_context - len + 1)));
    e.eos_id = 3;
    e.temperature = 1.f;
    e.top_p = 1.f;
    if (admission_slots(n, e.max_new.data()) > n_slots ||
        plan_pages(len, c.page_tokens, n, e.max_new.data(), nullptr, nullptr, nullptr) > c.pool->total()) {
      ++refused;  // could never run: refused at push
      continue;
    }
    e.prompt_id = c.prompt_counter++;
    e.first_sample = c.next_sample_id;
    c.next_sample_id += n;
    q.waiting.push_back(std::move(e));
    ++pushed;
  }
  q.pushed = pushed;

  long long steps = 0, emitted = 0, injected = 0, caller_aborts = 0;
  long long chunk_rows_done = 0, pending_preempted = 0;
  while (!q.waiting.empty() || !q.pending.empty() || !c.live.empty()) {
    REQUIRE(++steps < 200000);
    // (0) growing pages: make room
    bool dropped_any = false;
    if (c.grow_pages) {
      while (pages_missing_for_step(c) > c.pool->unreserved()) {
        if (queue_preempt_pending(c)) {  // the half-cached prompts give way first
          dropped_any = true;
          ++pending_preempted;
          check_books(c, n_slots);
          continue;
        }
        std::vector<int64_t> ids;
        const int dropped = queue_preempt_youngest(c, &ids);
        REQUIRE(dropped > 0 && (int)ids.size() == dropped);
        dropped_any = true;
        check_books(c, n_slots);
      }
    }
    // (1) admission
    if (chunk_rows > 0 && c.grow_pages && !q.pending.empty() && uni(0, 20) == 0) {
      // rarely the pool runs out while a prompt is half cached (admission keeps spare pages): send
      // one back now and then all the same, as step (0) would
      REQUIRE(queue_preempt_pending(c));
      dropped_any = true;
      ++pending_preempted;
      check_books(c, n_slots);
    }
    if (chunk_rows > 0) {
      // chunked prefill: what queue_step_chunked does on the host
      if (!dropped_any && !q.waiting.empty() && pending_rows_left(q) < q.chunk_rows) {
        int k = queue_select_run(c, AdmissionLimits{(int)q.free_rows.size(), 64});
        if (k > 0 && uni(0, 9) == 0) {  // a failing admission leaves the queue and the pool as they were
          const int before_use = c.pool->in_use(), before_slots = (int)c.free_slots.size(), before_res = c.pool->reserved;
          const size_t before_wait = q.waiting.size(), before_pend = q.pending.size(), before_rows = q.free_rows.size();
          c.pool->reserved = std::max(0, c.pool->free_pages() - uni(0, 2));
          bool threw = false;
          try {
            queue_admit_pending(c);
          } catch (const ApiError& err) {
            threw = true;
            REQUIRE(err.code == ROLLOUT_E_NOMEM);
          }
          c.pool->reserved = before_res;
          if (threw) {
            REQUIRE(c.pool->in_use() == before_use && (int)c.free_slots.size() == before_slots);
            REQUIRE(q.waiting.size() == before_wait && q.pending.size() == before_pend && q.free_rows.size() == before_rows);
          } else {
            --k;
          }
          injected += threw;
          check_books(c, n_slots);
        }
        while (k-- > 0 && pending_rows_left(q) < q.chunk_rows) queue_admit_pending(c);
      }
      check_books(c, n_slots);
      std::vector<ChunkSeq> seqs;
      const int B = (int)c.live.size();
      const int max_fin = uni(0, 3);
      const int rows = plan_chunk(q, std::min(chunk_rows, 64 - std::min(B, 63)), max_fin, seqs);
      int fin = 0, sum = 0;
      for (size_t i = 0; i < seqs.size(); ++i) {
        const ChunkSeq& cs = seqs[i];
        const PendingPrompt& pp = q.pending[cs.pending_index];
        REQUIRE(cs.pending_index == (int)i && cs.begin == pp.done && cs.len > 0);
        REQUIRE(cs.last == (cs.begin + cs.len == (int)pp.prompt.tokens.size()));
        REQUIRE(cs.last || i + 1 == seqs.size());  // only the last sequence may stop short
        fin += cs.last;
        sum += cs.len;
      }
      REQUIRE(sum == rows && rows <= chunk_rows && fin <= max_fin);
      chunk_rows_done += rows;
      for (const ChunkSeq& cs : seqs) q.pending[cs.pending_index].done += cs.len;
      for (int f = 0; f < fin; ++f) {  // the prompts that end hand over to their samples
        PendingPrompt& pp = q.pending.front();
        q.open[pp.prompt.prompt_id] = n;
        for (int j = 0; j < n; ++j) {
          Sample& s = pp.samples[j];
          s.n_emitted = 1;
          ++emitted;
          const bool done = s.max_new <= 1 || uni(0, 40) == 0;
          if (done) {
            release_sample(c, s);
            queue_note_finished(q, pp.prompt.prompt_id);
          } else {
            REQUIRE(c.live.emplace(s.id, std::move(s)).second);
          }
        }
        for (int32_t pg : pp.pages.shared) c.pool->release(pg);
        if (pp.pages.tail >= 0) c.pool->release(pp.pages.tail);
        q.free_rows.push_back(pp.table_row);
        if (c.grow_pages && q.open.count(pp.prompt.prompt_id)) q.admitted.emplace(pp.prompt.prompt_id, std::move(pp.prompt));
        q.pending.pop_front();
        c.live_dirty = true;
      }
      check_books(c, n_slots);
    }
    int k = dropped_any || chunk_rows > 0 ? 0 : queue_select_run(c, AdmissionLimits{kTempSlots, 64});
    if (k > 0 && uni(0, 9) == 0) {
      // a failing admission: the pool refuses after a few pages; nothing may stay taken
      const int before_use = c.pool->in_use(), before_slots = (int)c.free_slots.size(), before_res = c.pool->reserved;
      c.pool->reserved = std::max(0, c.pool->free_pages() - uni(0, 2));
      bool threw = false;
      try {
        Rollback undo(c);
        std::vector<Sample> fresh(n);
        std::vector<int> copies;
        PromptPages pp;
        const QueuedPrompt& e = q.waiting[0];
        take_prompt_pages(c, undo, (int)e.tokens.size(), n, e.max_new.data(), e.eos_id, e.prompt_id, e.first_sample,
                          n_slots, pp, fresh.data(), copies);
        // it fitted after all: give it back the ordinary way (undo is still armed)
      } catch (const ApiError& err) {
        threw = true;
        REQUIRE(err.code == ROLLOUT_E_NOMEM);
      }
      c.pool->reserved = before_res;
      REQUIRE(c.pool->in_use() == before_use && (int)c.free_slots.size() == before_slots);
      injected += threw;
      check_books(c, n_slots);
    }
    for (int i = 0; i < k; ++i) {
      const QueuedPrompt& e = q.waiting[i];
      Rollback undo(c);
      std::vector<Sample> fresh(n);
      std::vector<int> copies;
      PromptPages pp;
      take_prompt_pages(c, undo, (int)e.tokens.size(), n, e.max_new.data(), e.eos_id, e.prompt_id, e.first_sample,
                        n_slots + i, pp, fresh.data(), copies);
      REQUIRE(copies.size() % 2 == 0);
      undo.commit();
      q.open[e.prompt_id] = n;
      if (c.grow_pages) q.admitted.emplace(e.prompt_id, e);
      for (int j = 0; j < n; ++j) {
        Sample& s = fresh[j];
        s.n_emitted = 1;
        ++emitted;
        const bool done = s.max_new <= 1 || uni(0, 40) == 0;  // ends at the first token
        if (done) {
          release_sample(c, s);
          queue_note_finished(q, e.prompt_id);
        } else {
          REQUIRE(c.live.emplace(s.id, std::move(s)).second);
        }
      }
      for (int32_t pg : pp.shared) c.pool->release(pg);
      if (pp.tail >= 0) c.pool->release(pp.tail);
    }
    if (k > 0) {
      q.waiting.erase(q.waiting.begin(), q.waiting.begin() + k);
      q.admitted_count += k;
      c.live_dirty = true;
    }
    check_books(c, n_slots);
    // (2) decode step
    if (c.grow_pages) {
      REQUIRE(pages_missing_for_step(c) <= c.pool->unreserved());
      std::vector<PagePatch> patches;
      grow_pages_for_step(c, patches);
      for (const PagePatch& pt : patches) REQUIRE(c.h_page_table[(size_t)pt.slot * c.max_pages + pt.index] == pt.page);
    }
    for (auto it = c.live.begin(); it != c.live.end();) {
      Sample& s = it->second;
      s.n_emitted += 1;
      ++emitted;
      const bool done = s.n_emitted >= s.max_new || uni(0, early_end) == 0;  // the limit, or an early end
      if (done) {
        const int64_t group = s.group;
        release_sample(c, s);
        it = c.live.erase(it);
        queue_note_finished(q, group);
      } else {
        ++it;
      }
    }
    // (3) now and then the caller aborts a sample
    if (!c.live.empty() && uni(0, 25) == 0) {
      auto it = c.live.begin();
      std::advance(it, uni(0, (int)c.live.size() - 1));
      queue_note_finished(q, it->second.group);
      release_sample(c, it->second);
      c.live.erase(it);
      ++caller_aborts;
    }
    check_books(c, n_slots);
  }
  REQUIRE(c.pool->in_use() == 0 && c.pool->free_pages() == n_pages && c.pool->reserved == 0);
  REQUIRE((int)c.free_slots.size() == n_slots);
  REQUIRE(q.open.empty() && q.admitted.empty());
  REQUIRE((long long)q.completed == pushed);
  REQUIRE((long long)q.admitted_count == pushed);   // every preemption took its admission back
  REQUIRE((int)q.free_rows.size() == kTempSlots);
  std::printf("seed %u grow %d: %d prompts x %d samples pushed (%d refused), %lld steps, %lld tokens, %llu preemptions, "
              "%lld failing admissions rolled back, %lld caller aborts, peak pages %d of %d; chunked: %lld prompt rows, "
              "%lld half-cached prompts sent back\n",
              seed, (int)grow, pushed, n, refused, steps, emitted, (unsigned long long)q.preempted, injected,
              caller_aborts, c.pool->peak_in_use, n_pages, chunk_rows_done, pending_preempted);
  delete c.pool;
  return 0;
}
