// extern "C" boundary of librollout.so: argument checks, the sample table and page
// accounting on the host, and the launch sequences of prefill, decode step, teacher-forced
// log-probs and abort.  See include/rollout.h for the contract of each entry point.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "engine.h"

static thread_local std::string g_init_error;

static void fail(int code, const std::string& msg) { throw ApiError{code, msg}; }

template <typename F>
static int guarded(rollout_ctx* ctx, F&& body) {
  std::string* err = ctx ? &ctx->err : &g_init_error;
  try {
    body();
    return ROLLOUT_OK;
  } catch (const ApiError& e) {
    *err = e.msg;
    return e.code;
  } catch (const HipError& e) {
    *err = std::string("HIP error ") + hipGetErrorString(e.code) + " in " + e.expr + " (" + e.file + ":" +
           std::to_string(e.line) + ")";
    return ROLLOUT_E_HIP;
  } catch (const std::bad_alloc&) {
    *err = "host allocation failed";
    return ROLLOUT_E_NOMEM;
  } catch (...) {
    *err = "unexpected internal error";
    return ROLLOUT_E_STATE;
  }
}

static void h2d(void* dst, const void* src, size_t bytes, hipStream_t s) {
  if (bytes) HIP_TRY(hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, s));
}
static void d2h(void* dst, const void* src, size_t bytes, hipStream_t s) {
  if (bytes) HIP_TRY(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, s));
}

__global__ void init_slots_kernel(SlotState st, const int* __restrict__ slots, const int* __restrict__ sample_row,
                                  const int* __restrict__ pos, const int* __restrict__ tokens,
                                  const long long* __restrict__ ids, const float* __restrict__ inv_temp,
                                  const float* __restrict__ top_p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int sl = slots[i], row = sample_row[i];
  st.last_token[sl] = tokens[row];
  st.pos[sl] = pos[i];
  st.step[sl] = 1;
  st.sample_id[sl] = ids[row];
  st.inv_temp[sl] = inv_temp[row];
  st.top_p[sl] = top_p[row];
}

// A decode step ends with a few hundred bytes coming back; polling an event answers within
// microseconds where a blocking wait costs a scheduler round trip per step.
// The poll is bounded by wall clock (step_timeout_s): kernels that never finish must not hang the
// caller for good.  After a time-out the device state is unknown, so the context refuses every
// further call (E_STATE) and rollout_destroy is what is left to do.
static void wait_step_done(rollout_ctx& c) {
  if (!c.step_done) HIP_TRY(hipEventCreateWithFlags(&c.step_done, hipEventDisableTiming));
  HIP_TRY(hipEventRecord(c.step_done, c.stream));
  const auto t0 = std::chrono::steady_clock::now();
  for (unsigned polls = 0;; ++polls) {
    hipError_t e = hipEventQuery(c.step_done);
    if (e == hipSuccess) return;
    if (e != hipErrorNotReady) throw HipError(e, "hipEventQuery", __FILE__, __LINE__);
    if (((polls & 1023u) == 1023u || c.step_timeout_s <= 0) &&
        std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > c.step_timeout_s) {
      c.broken = true;
      throw ApiError{ROLLOUT_E_HIP, "the decode step's kernels did not finish within " +
                                        std::to_string(c.step_timeout_s) + " s; the context is unusable now"};
    }
  }
}

// Host wall clock of a phase (the wait for the device included), added to the statistics when the
// phase ends, by an exception too.
struct PhaseClock {
  double& total_ms;
  std::chrono::steady_clock::time_point t0 = std::chrono::steady_clock::now();
  explicit PhaseClock(double& slot) : total_ms(slot) {}
  ~PhaseClock() { total_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count(); }
};

static void check_usable(const rollout_ctx& c) {
  if (c.broken) throw ApiError{ROLLOUT_E_STATE, "an earlier call timed out on the device; destroy this context"};
}

static void refresh_stats(rollout_ctx& c) {
  c.stats.live_samples = (int32_t)c.live.size();
  c.stats.pages_total = c.pool->total();
  c.stats.pages_in_use = c.pool->in_use();
  c.stats.pages_reserved = c.pool->reserved;
  c.stats.pages_peak = c.pool->peak_in_use;
  c.stats.matrix_core_path = c.simple ? 0 : 1;
}

// Admission of P prompts with n samples each (all or none), their prefill and response
// position 0.  prompt_ids / first_ids: the prompts' counters and the ids of their first samples
// as handed out at push time (sample j of prompt p carries first_ids[p] + j), or both NULL to
// take the next P counters and the next P * n ids.
static void prefill_impl(rollout_ctx& c, int32_t n_prompts, const int32_t* tokens, const int32_t* offsets,
                         int32_t n_samples, const int32_t* max_new_tokens, int32_t eos_id, float temperature,
                         float top_p, const int32_t* forced_first, const uint32_t* uniform_override,
                         const int64_t* prompt_ids, const int64_t* first_ids, int64_t* sample_ids,
                         int32_t* first_tokens, float* first_logprobs, uint8_t* finished) {
  const rollout_model_desc& m = c.md;
  const int P = n_prompts, n = n_samples, R = c.r_max;
  PhaseClock clock(c.stats.prefill_ms);
  // ---- validation (no state changes before all of it passed) ----
  if (P < 1 || n < 1 || !tokens || !offsets || !max_new_tokens) fail(ROLLOUT_E_INVAL, "bad prompt arguments");
  if (!(temperature > 0.f) || !std::isfinite(temperature)) fail(ROLLOUT_E_INVAL, "temperature must be > 0");
  if (!(top_p >= 0.f)) fail(ROLLOUT_E_INVAL, "top_p must be >= 0");
  if (eos_id < -1 || eos_id >= m.vocab) fail(ROLLOUT_E_INVAL, "eos_id out of range");
  if (offsets[0] != 0) fail(ROLLOUT_E_INVAL, "offsets[0] must be 0");
  if ((long long)P * n > R) fail(ROLLOUT_E_NOMEM, "n_prompts * n_samples exceeds the workspace rows");
  if (P > rollout_ctx::kTempSlots || P > c.logit_rows) fail(ROLLOUT_E_NOMEM, "too many prompts in one call");
  int need_slots = 0;
  long long need_pages = 0;
  for (int p = 0; p < P; ++p) {
    int len = offsets[p + 1] - offsets[p];
    if (len < 1) fail(ROLLOUT_E_INVAL, "empty prompt");
    if (len > c.rd.max_batch_tokens) fail(ROLLOUT_E_NOMEM, "prompt longer than max_batch_tokens");
    for (int j = 0; j < n; ++j) {
      int mn = max_new_tokens[p * n + j];
      if (mn < 1) fail(ROLLOUT_E_INVAL, "max_new_tokens must be >= 1");
      if ((long long)len + mn - 1 > c.rd.max_context) fail(ROLLOUT_E_NOMEM, "prompt + response exceeds max_context");
      if (mn > 1) ++need_slots;
      if (forced_first && (forced_first[p * n + j] < 0 || forced_first[p * n + j] >= m.vocab))
        fail(ROLLOUT_E_INVAL, "forced token out of range");
    }
    for (int i = offsets[p]; i < offsets[p + 1]; ++i)
      if (tokens[i] < 0 || tokens[i] >= m.vocab) fail(ROLLOUT_E_INVAL, "prompt token out of range");
    need_pages += admission_pages(c, len, n, max_new_tokens + p * n);
  }
  if (need_slots > (int)c.free_slots.size()) fail(ROLLOUT_E_NOMEM, "not enough free live-sample slots");
  if (need_pages > c.pool->unreserved()) fail(ROLLOUT_E_NOMEM, "not enough free KV pages");
  if ((prompt_ids == nullptr) != (first_ids == nullptr)) fail(ROLLOUT_E_STATE, "internal: ids given in part");
  for (int p = 0; p < P; ++p)
    for (int j = 0; j < n; ++j)
      if (c.live.count((first_ids ? first_ids[p] : c.next_sample_id + (int64_t)p * n) + j))
        fail(ROLLOUT_E_STATE, "internal: a sample id is live already");

  // ---- pages and page tables (given back by `undo` if anything below throws) ----
  Rollback undo(c);
  const float inv_t = 1.0f / temperature;
  std::vector<PromptPages> pp(P);
  std::vector<Sample> fresh((size_t)P * n);
  std::vector<int> copy_pairs;
  for (int p = 0; p < P; ++p)
    take_prompt_pages(c, undo, offsets[p + 1] - offsets[p], n, max_new_tokens + p * n, eos_id,
                      prompt_ids ? prompt_ids[p] : c.prompt_counter + p,
                      first_ids ? first_ids[p] : c.next_sample_id + (int64_t)p * n, c.temp_slot0 + p, pp[p],
                      &fresh[(size_t)p * n], copy_pairs);
  engine_upload_page_table(c);

  // ---- forward over the prompts, in chunks of whole prompts ----
  int p0 = 0;
  while (p0 < P) {
    int p1 = p0, rows = 0;
    while (p1 < P && rows + (offsets[p1 + 1] - offsets[p1]) <= c.rd.max_batch_tokens) {
      rows += offsets[p1 + 1] - offsets[p1];
      ++p1;
    }
    int* ht = c.h_int.p;
    int r = 0, max_len = 0;
    for (int p = p0; p < p1; ++p) {
      for (int i = offsets[p]; i < offsets[p + 1]; ++i, ++r) {
        ht[r] = tokens[i];
        ht[R + r] = i - offsets[p];
        ht[2 * R + r] = c.temp_slot0 + p;
      }
      ht[3 * R + (p - p0)] = r - 1;  // last row of the prompt
      ht[4 * R + (p - p0)] = r - (offsets[p + 1] - offsets[p]);
      ht[5 * R + (p - p0)] = offsets[p + 1] - offsets[p];
      ht[6 * R + (p - p0)] = c.temp_slot0 + p;
      max_len = std::max(max_len, offsets[p + 1] - offsets[p]);
    }
    SeqBatch sb{c.seq_row0.p, c.seq_len.p, c.seq_slot.p, p1 - p0, max_len};
    if (!c.simple) {
      h2d(c.seq_row0.p, ht + 4 * R, (p1 - p0) * sizeof(int), c.stream);
      h2d(c.seq_len.p, ht + 5 * R, (p1 - p0) * sizeof(int), c.stream);
      h2d(c.seq_slot.p, ht + 6 * R, (p1 - p0) * sizeof(int), c.stream);
    }
    h2d(c.row_token.p, ht, rows * sizeof(int), c.stream);
    h2d(c.row_pos.p, ht + R, rows * sizeof(int), c.stream);
    h2d(c.row_slot.p, ht + 2 * R, rows * sizeof(int), c.stream);
    h2d(c.row_aux.p, ht + 3 * R, (p1 - p0) * sizeof(int), c.stream);
    c.timer.start_call();
    c.kv_tokens_this_call = rows;
    c.attn_flops_this_call = 0;
    for (int p = p0; p < p1; ++p) {
      double len = offsets[p + 1] - offsets[p];
      c.attn_flops_this_call += 2.0 * len * (len + 1) * c.q_dim;
    }
    engine_forward_rows(c, rows, &sb);
    engine_logits(c, c.row_aux.p, 0, p1 - p0, c.logits.p + (size_t)p0 * m.vocab);
    HIP_TRY(hipStreamSynchronize(c.stream));  // staging buffers are reused by the next chunk
    c.timer.collect();
    c.stats.prompt_tokens += rows;
    p0 = p1;
  }
  c.last_logit_rows = P;

  // ---- private copies of each prompt's partial last page ----
  if (!copy_pairs.empty()) {
    if (copy_pairs.size() > c.row_aux.n) fail(ROLLOUT_E_STATE, "internal: page copy list too long");
    std::memcpy(c.h_int.p, copy_pairs.data(), copy_pairs.size() * sizeof(int));
    h2d(c.row_aux.p, c.h_int.p, copy_pairs.size() * sizeof(int), c.stream);
    launch_copy_pages(c.kv_pool.p, c.row_aux.p, (int)copy_pairs.size() / 2, m.n_layers,
                      c.geom.layer_stride * c.elem, c.geom.page_stride * c.elem, c.stream);
    HIP_TRY(hipStreamSynchronize(c.stream));
  }

  // ---- response position 0 of every sample ----
  const int Rs = P * n;
  int* hi = c.h_int.p;
  float* hf = c.h_float.p;
  int n_new = 0;
  for (int i = 0; i < Rs; ++i) {
    hi[i] = i / n;                                       // logits row = prompt
    hi[R + i] = forced_first ? forced_first[i] : -1;
    hi[2 * R + i] = 0;                                   // response position
    hi[3 * R + i] = uniform_override ? (int)uniform_override[i] : 0;
    hf[i] = inv_t;
    hf[R + i] = top_p;
    c.h_ll.p[i] = fresh[i].id;
    if (fresh[i].slot >= 0) {
      hi[4 * R + n_new] = fresh[i].slot;
      hi[5 * R + n_new] = i;
      hi[6 * R + n_new] = fresh[i].prompt_len;
      ++n_new;
    }
  }
  h2d(c.row_aux.p, hi, Rs * sizeof(int), c.stream);
  h2d(c.row_forced.p, hi + R, Rs * sizeof(int), c.stream);
  h2d(c.row_step.p, hi + 2 * R, Rs * sizeof(int), c.stream);
  h2d(c.row_uniform.p, hi + 3 * R, Rs * sizeof(int), c.stream);
  h2d(c.row_inv_temp.p, hf, Rs * sizeof(float), c.stream);
  h2d(c.row_top_p.p, hf + R, Rs * sizeof(float), c.stream);
  h2d(c.row_sample_id.p, c.h_ll.p, Rs * sizeof(long long), c.stream);
  SampleRows sr{};
  sr.logits = c.logits.p;
  sr.logits_row = c.row_aux.p;
  sr.inv_temp = c.row_inv_temp.p;
  sr.top_p = c.row_top_p.p;
  sr.uniforms = uniform_override ? c.row_uniform.p : nullptr;
  sr.sample_id = c.row_sample_id.p;
  sr.step = c.row_step.p;
  sr.forced = c.row_forced.p;
  sr.seed = c.rd.seed;
  sr.tokens = c.out_tokens.p;
  sr.logprobs = c.out_logprobs.p;
  sr.weight_sums = nullptr;
  if (Rs <= c.samp_rows) {
    sr.part_max = c.samp_part_max.p;
    sr.seg_sums = c.samp_seg_sums.p;
  }
  launch_sample(sr, Rs, m.vocab, c.stream);
  if (n_new) {
    h2d(c.row_token.p, hi + 4 * R, n_new * sizeof(int), c.stream);  // slots
    h2d(c.row_pos.p, hi + 5 * R, n_new * sizeof(int), c.stream);    // sample rows
    h2d(c.row_slot.p, hi + 6 * R, n_new * sizeof(int), c.stream);   // positions
    init_slots_kernel<<<ceil_div(n_new, 256), 256, 0, c.stream>>>(c.st, c.row_token.p, c.row_pos.p, c.row_slot.p,
                                                                  c.out_tokens.p, c.row_sample_id.p,
                                                                  c.row_inv_temp.p, c.row_top_p.p, n_new);
  }
  d2h(hi + 7 * R, c.out_tokens.p, Rs * sizeof(int), c.stream);
  d2h(hf + 2 * R, c.out_logprobs.p, Rs * sizeof(float), c.stream);
  HIP_TRY(hipStreamSynchronize(c.stream));

  // ---- host bookkeeping (nothing below throws: the pages and slots now belong to the samples) ----
  undo.commit();
  for (int i = 0; i < Rs; ++i) {
    Sample& s = fresh[i];
    int tok = hi[7 * R + i];
    s.n_emitted = 1;
    s.last_token = tok;
    bool done = s.max_new <= 1 || (eos_id >= 0 && tok == eos_id);
    if (sample_ids) sample_ids[i] = s.id;
    if (first_tokens) first_tokens[i] = tok;
    if (first_logprobs) first_logprobs[i] = hf[2 * R + i];
    if (finished) finished[i] = done ? 1 : 0;
    c.stats.tokens_emitted += 1;
    c.stats.samples_admitted += 1;
    if (done) {
      release_sample(c, s);
      c.stats.samples_finished += 1;
    } else {
      const int64_t id = s.id;
      Sample moved = std::move(s);
      auto res = c.live.emplace(id, std::move(moved));
      if (!res.second) {  // cannot happen (ids were checked above); never drop pages and a slot silently
        release_sample(c, moved);
        c.stats.samples_aborted += 1;
      }
    }
  }
  for (int p = 0; p < P; ++p) {
    for (int32_t pg : pp[p].shared) c.pool->release(pg);
    if (pp[p].tail >= 0) c.pool->release(pp[p].tail);
  }
  if (!prompt_ids) {
    c.prompt_counter += P;
    c.next_sample_id += (int64_t)P * n;
  }
  c.stats.prompts_prefilled += P;
  c.live_dirty = true;
  refresh_stats(c);
}

// Prompt rows that ride along with a decode step (chunked prefill): the rows of `seqs`, cut from
// the queue's pending prompts, go through the same forward pass behind the decode rows.  The
// prompts that end in the step sample response position 0 of their samples; `first_*` receive
// those results, n samples per finishing prompt in the order of `seqs`.
struct StepChunk {
  std::vector<ChunkSeq> seqs;
  int rows = 0;
  std::vector<int64_t> first_ids, first_groups;
  std::vector<int32_t> first_tokens;
  std::vector<float> first_logprobs;
  std::vector<uint8_t> first_finished;
};

// The forward pass of a step that carries prompt rows: uploads the chunk's rows behind the B decode
// rows (tokens, positions, page-table rows; one packed sequence per prompt, continuing at its
// first uncached position), runs the forward, and computes the logits of the decode rows and of
// the last row of every prompt that ends here (logits rows B, B + 1, ...).  Returns the number of
// prompts that end.
static int forward_with_chunk(rollout_ctx& c, int B, const StepChunk& chunk) {
  const PromptQueue& q = c.queue;
  const int R = c.r_max, Rq = chunk.rows, n = q.n_samples;
  const int ns = (int)chunk.seqs.size();
  // pageable staging: each of these uploads is complete when its call returns
  std::vector<int> tok(Rq), pos(Rq), slot(Rq), row0(ns), len(ns), srow(ns), pos0(ns), want(B);
  for (int i = 0; i < B; ++i) want[i] = i;
  int r = 0, max_len = 0, n_fin = 0;
  c.chunk_kv_tokens = 0;
  for (int k = 0; k < ns; ++k) {
    const ChunkSeq& cs = chunk.seqs[k];
    const PendingPrompt& pp = q.pending[cs.pending_index];
    row0[k] = B + r;
    len[k] = cs.len;
    srow[k] = pp.table_row;
    pos0[k] = cs.begin;
    for (int i = 0; i < cs.len; ++i, ++r) {
      tok[r] = pp.prompt.tokens[cs.begin + i];
      pos[r] = cs.begin + i;
      slot[r] = pp.table_row;
    }
    if (cs.last) {
      want.push_back(B + r - 1);
      ++n_fin;
    }
    max_len = std::max(max_len, cs.len);
    c.chunk_kv_tokens += (double)cs.len * cs.begin + 0.5 * cs.len * (cs.len + 1.0);
  }
  if (ns > rollout_ctx::kTempSlots || B + n_fin > c.logit_rows || (long long)B + (long long)n_fin * n > R)
    fail(ROLLOUT_E_STATE, "internal: the chunk plan exceeds the workspaces");
  c.chunk_attn_flops = 4.0 * c.chunk_kv_tokens * c.q_dim;
  h2d(c.row_token.p + B, tok.data(), Rq * sizeof(int), c.stream);
  h2d(c.row_pos.p + B, pos.data(), Rq * sizeof(int), c.stream);
  h2d(c.row_slot.p + B, slot.data(), Rq * sizeof(int), c.stream);
  h2d(c.seq_row0.p, row0.data(), ns * sizeof(int), c.stream);
  h2d(c.seq_len.p, len.data(), ns * sizeof(int), c.stream);
  h2d(c.seq_slot.p, srow.data(), ns * sizeof(int), c.stream);
  h2d(c.seq_pos0.p, pos0.data(), ns * sizeof(int), c.stream);
  h2d(c.chunk_ints.p, want.data(), want.size() * sizeof(int), c.stream);
  SeqBatch sb{c.seq_row0.p, c.seq_len.p, c.seq_slot.p, ns, max_len};
  sb.pos0 = c.seq_pos0.p;
  sb.decode_rows = B;
  engine_forward_rows(c, B + Rq, &sb);
  engine_logits(c, c.chunk_ints.p, 0, B + n_fin, c.logits.p);
  c.last_logit_rows = B + n_fin;
  c.stats.prompt_tokens += Rq;
  return n_fin;
}

// The prompts `fin` end in this step (their last rows' logits are rows B, B + 1, ... of c.logits):
// private copies of each prompt's partial last page, response position 0 of its n samples drawn
// through rows B .. of the per-row sampling arrays, the slot state of the samples that go on, and
// the results on their way to pinned host memory (tokens at h_int + 7 r_max, log-probs at
// h_float + r_max); the caller waits for the stream.
static void sample_first_tokens(rollout_ctx& c, int B, const std::vector<PendingPrompt*>& fin) {
  const rollout_model_desc& m = c.md;
  const int R = c.r_max, n = c.queue.n_samples, n_fin = (int)fin.size(), Rs = n_fin * n;
  std::vector<int> pairs, lrow(Rs), step0(Rs, 0), forced(Rs, -1), slots, srows, spos;
  std::vector<float> inv_t(Rs), top_p(Rs);
  std::vector<long long> ids(Rs);
  for (int k = 0; k < n_fin; ++k) {
    const PendingPrompt& pp = *fin[k];
    pairs.insert(pairs.end(), pp.copy_pairs.begin(), pp.copy_pairs.end());
    for (int j = 0; j < n; ++j) {
      const int i = k * n + j;
      lrow[i] = B + k;
      inv_t[i] = 1.0f / pp.prompt.temperature;
      top_p[i] = pp.prompt.top_p;
      ids[i] = pp.samples[j].id;
      if (pp.samples[j].slot >= 0) {
        slots.push_back(pp.samples[j].slot);
        srows.push_back(i);
        spos.push_back(pp.samples[j].prompt_len);
      }
    }
  }
  const int n_new = (int)slots.size();
  if (pairs.size() + 3 * (size_t)n_new > 2 * (size_t)R) fail(ROLLOUT_E_STATE, "internal: page copy and slot lists too long");
  if (!pairs.empty()) {
    h2d(c.chunk_ints.p + R, pairs.data(), pairs.size() * sizeof(int), c.stream);
    launch_copy_pages(c.kv_pool.p, c.chunk_ints.p + R, (int)pairs.size() / 2, m.n_layers,
                      c.geom.layer_stride * c.elem, c.geom.page_stride * c.elem, c.stream);
  }
  h2d(c.row_aux.p + B, lrow.data(), Rs * sizeof(int), c.stream);
  h2d(c.row_forced.p + B, forced.data(), Rs * sizeof(int), c.stream);
  h2d(c.row_step.p + B, step0.data(), Rs * sizeof(int), c.stream);
  h2d(c.row_inv_temp.p + B, inv_t.data(), Rs * sizeof(float), c.stream);
  h2d(c.row_top_p.p + B, top_p.data(), Rs * sizeof(float), c.stream);
  h2d(c.row_sample_id.p + B, ids.data(), Rs * sizeof(long long), c.stream);
  SampleRows fr{};
  fr.logits = c.logits.p;
  fr.logits_row = c.row_aux.p + B;
  fr.inv_temp = c.row_inv_temp.p + B;
  fr.top_p = c.row_top_p.p + B;
  fr.uniforms = nullptr;
  fr.sample_id = c.row_sample_id.p + B;
  fr.step = c.row_step.p + B;
  fr.forced = c.row_forced.p + B;
  fr.seed = c.rd.seed;
  fr.tokens = c.out_tokens.p + B;
  fr.logprobs = c.out_logprobs.p + B;
  fr.weight_sums = nullptr;
  if (Rs <= c.samp_rows) {
    fr.part_max = c.samp_part_max.p;
    fr.seg_sums = c.samp_seg_sums.p;
  }
  launch_sample(fr, Rs, m.vocab, c.stream);
  if (n_new) {  // the lists sit behind the page pairs
    int* lists = c.chunk_ints.p + R + pairs.size();
    h2d(lists, slots.data(), n_new * sizeof(int), c.stream);
    h2d(lists + n_new, srows.data(), n_new * sizeof(int), c.stream);
    h2d(lists + 2 * n_new, spos.data(), n_new * sizeof(int), c.stream);
    init_slots_kernel<<<ceil_div(n_new, 256), 256, 0, c.stream>>>(c.st, lists, lists + n_new, lists + 2 * n_new,
                                                                  c.out_tokens.p + B, c.row_sample_id.p + B,
                                                                  c.row_inv_temp.p + B, c.row_top_p.p + B, n_new);
  }
  d2h(c.h_int.p + 7 * R, c.out_tokens.p + B, Rs * sizeof(int), c.stream);
  d2h(c.h_float.p + R, c.out_logprobs.p + B, Rs * sizeof(float), c.stream);
}

// Host bookkeeping after a step with prompt rows: the pending prompts' progress; the prompts that
// ended (`fin`, the first ones of the pending list) hand over to their samples, which go live or
// are finished at position 0, and leave the list.  Their results go to chunk.first_*.
static void commit_chunk(rollout_ctx& c, StepChunk& chunk, const std::vector<PendingPrompt*>& fin) {
  PromptQueue& q = c.queue;
  const int R = c.r_max, n = q.n_samples, n_fin = (int)fin.size(), Rs = n_fin * n;
  const int* first_tok = c.h_int.p + 7 * R;
  const float* first_lp = c.h_float.p + R;
  for (const ChunkSeq& cs : chunk.seqs) q.pending[cs.pending_index].done += cs.len;
  chunk.first_ids.resize(Rs);
  chunk.first_groups.resize(Rs);
  chunk.first_tokens.resize(Rs);
  chunk.first_logprobs.resize(Rs);
  chunk.first_finished.resize(Rs);
  for (int k = 0; k < n_fin; ++k) {
    PendingPrompt& pp = *fin[k];
    q.open[pp.prompt.prompt_id] = n;
    for (int j = 0; j < n; ++j) {
      const int i = k * n + j;
      Sample& s = pp.samples[j];
      const int tok = first_tok[i];
      s.n_emitted = 1;
      s.last_token = tok;
      const bool done = s.max_new <= 1 || (s.eos_id >= 0 && tok == s.eos_id);
      chunk.first_ids[i] = s.id;
      chunk.first_groups[i] = s.group;
      chunk.first_tokens[i] = tok;
      chunk.first_logprobs[i] = first_lp[i];
      chunk.first_finished[i] = done ? 1 : 0;
      c.stats.tokens_emitted += 1;
      c.stats.samples_admitted += 1;
      if (done) {
        release_sample(c, s);
        c.stats.samples_finished += 1;
      } else {
        const int64_t id = s.id;
        Sample moved = std::move(s);
        auto res = c.live.emplace(id, std::move(moved));
        if (!res.second) {  // cannot happen: ids are handed out once
          release_sample(c, moved);
          c.stats.samples_aborted += 1;
        }
      }
    }
    // the prefill's own references; the samples hold theirs
    for (int32_t pg : pp.pages.shared) c.pool->release(pg);
    if (pp.pages.tail >= 0) c.pool->release(pp.pages.tail);
    q.free_rows.push_back(pp.table_row);
    if (c.grow_pages) q.admitted.emplace(pp.prompt.prompt_id, std::move(pp.prompt));  // kept: it may have to start over
    c.stats.prompts_prefilled += 1;
    c.live_dirty = true;
  }
  // finished prompts sit at the front of the pending list (prompts are cached in order)
  for (int k = 0; k < n_fin; ++k) q.pending.pop_front();
}

// groups (optional): the prompt counter of every stepped sample, for the queue's bookkeeping
static void decode_impl(rollout_ctx& c, const int32_t* forced_tokens, const uint32_t* uniform_override,
                        int32_t* n_live, int64_t* sample_ids, int32_t* tokens, float* logprobs,
                        uint8_t* finished, int64_t* groups = nullptr, StepChunk* chunk = nullptr) {
  const rollout_model_desc& m = c.md;
  if (!n_live) fail(ROLLOUT_E_INVAL, "n_live is null");
  const int B = (int)c.live.size(), R = c.r_max;
  const int Rq = chunk ? chunk->rows : 0;
  PhaseClock clock(c.stats.decode_ms);
  if (B == 0 && Rq == 0) {
    *n_live = 0;
    return;
  }
  if (*n_live < B) fail(ROLLOUT_E_INVAL, "output capacity smaller than the live-sample count");
  if (Rq && (c.simple || B + Rq > R)) fail(ROLLOUT_E_STATE, "internal: the step cannot carry these prompt rows");
  if (forced_tokens)
    for (int i = 0; i < B; ++i)
      if (forced_tokens[i] < 0 || forced_tokens[i] >= m.vocab) fail(ROLLOUT_E_INVAL, "forced token out of range");
  int* hi = c.h_int.p;
  if (c.grow_pages) {  // the pages this step writes to (checked first: a failing call changes nothing)
    if (pages_missing_for_step(c) > c.pool->unreserved())
      fail(ROLLOUT_E_NOMEM, "the KV pool is exhausted: abort samples and call again");
    std::vector<PagePatch> patches;
    grow_pages_for_step(c, patches);
    if (!patches.empty()) {
      static_assert(sizeof(PagePatch) == 3 * sizeof(int), "patches travel as int triples");
      std::memcpy(hi + 4 * R, patches.data(), patches.size() * sizeof(PagePatch));
      h2d(c.d_page_patch.p, hi + 4 * R, patches.size() * sizeof(PagePatch), c.stream);
      launch_patch_page_table(c.d_page_table.p, c.max_pages, c.d_page_patch.p, (int)patches.size(), c.stream);
    }
  }
  if (c.live_dirty) {
    int i = 0;
    for (auto& kv : c.live) hi[i++] = kv.second.slot;
    h2d(c.d_live.p, hi, B * sizeof(int), c.stream);
    // Groups for the decode attention: live samples of one prompt (consecutive in id order), at
    // least two of them and at least 64 shared positions, in chunks of GROUP_MEMBERS.
    std::vector<int> grows, glen, gslot;  // pageable: their uploads complete before the call returns
    c.h_row_t0.assign(B, 0);
    c.n_groups = 0;
    c.max_shared = 0;
    c.shared_saved = 0;
    c.shared_dup = 0;
    {
      const Sample* first = nullptr;
      for (auto& kv : c.live) {
        if (first && kv.second.group == first->group) c.shared_dup += first->shared_len;
        else first = &kv.second;
      }
    }
    if (!c.simple) {
      std::vector<const Sample*> rows;
      rows.reserve(B);
      for (auto& kv : c.live) rows.push_back(&kv.second);
      for (int r0 = 0; r0 < B;) {
        int r1 = r0 + 1;
        while (r1 < B && rows[r1]->group == rows[r0]->group && r1 - r0 < GROUP_MEMBERS) ++r1;
        const int members = r1 - r0, len = rows[r0]->shared_len;
        if (members >= 2 && len >= 64) {
          for (int j = 0; j < GROUP_MEMBERS; ++j) grows.push_back(j < members ? r0 + j : -1);
          glen.push_back(len);
          gslot.push_back(rows[r0]->slot);
          for (int r = r0; r < r1; ++r) c.h_row_t0[r] = len;
          c.max_shared = std::max(c.max_shared, len);
          c.shared_saved += (long long)(members - 1) * len;
          ++c.n_groups;
        }
        r0 = r1;
      }
      if (c.n_groups) {
        h2d(c.grp_rows.p, grows.data(), grows.size() * sizeof(int), c.stream);
        h2d(c.grp_len.p, glen.data(), glen.size() * sizeof(int), c.stream);
        h2d(c.grp_slot.p, gslot.data(), gslot.size() * sizeof(int), c.stream);
        h2d(c.row_t0.p, c.h_row_t0.data(), B * sizeof(int), c.stream);
      }
    }
    c.live_dirty = false;
  }
  launch_gather_decode_rows(c.st, c.d_live.p, B, c.row_token.p, c.row_pos.p, c.row_slot.p, c.row_inv_temp.p,
                            c.row_top_p.p, c.row_sample_id.p, c.row_step.p, c.stream);
  c.decode_max_ctx = 1;
  c.decode_max_own = 1;
  c.kv_tokens_this_call = 0;
  {
    int r = 0;
    for (auto& kv : c.live) {
      const int ctx = kv.second.prompt_len + kv.second.n_emitted;
      c.decode_max_ctx = std::max(c.decode_max_ctx, ctx);
      c.decode_max_own = std::max(c.decode_max_own, ctx - (r < (int)c.h_row_t0.size() ? c.h_row_t0[r] : 0));
      c.kv_tokens_this_call += ctx;
      ++r;
    }
  }
  // one read of a shared prompt per group instead of one per member (opt-in), when it saves at
  // least a fifth of the positions
  c.use_groups = c.n_groups > 0 && B > 32 && c.md.n_q_heads / c.md.n_kv_heads <= 8 &&
                 (c.rd.flags & ROLLOUT_RT_PROMPT_GROUPS) &&
                 (double)c.shared_saved >= 0.2 * c.kv_tokens_this_call;
  c.kv_unique_tokens_this_call = c.kv_tokens_this_call - (double)c.shared_dup;
  c.attn_flops_this_call = 4.0 * c.kv_tokens_this_call * c.q_dim;
  int n_fin = 0;  // prompts that end in this step: their last rows' logits follow the decode rows'
  c.timer.start_call();
  if (!Rq) {
    engine_forward_rows(c, B, nullptr);
    c.timer.empty_bracket(c.stream);
    engine_logits(c, nullptr, 0, B, c.logits.p);
    c.last_logit_rows = B;
  } else {
    n_fin = forward_with_chunk(c, B, *chunk);
  }
  if (forced_tokens) {
    std::memcpy(hi + R, forced_tokens, B * sizeof(int));
    h2d(c.row_forced.p, hi + R, B * sizeof(int), c.stream);
  }
  if (uniform_override) {
    std::memcpy(hi + 2 * R, uniform_override, B * sizeof(int));
    h2d(c.row_uniform.p, hi + 2 * R, B * sizeof(int), c.stream);
  }
  SampleRows sr{};
  sr.logits = c.logits.p;
  sr.logits_row = nullptr;
  sr.inv_temp = c.row_inv_temp.p;
  sr.top_p = c.row_top_p.p;
  sr.uniforms = uniform_override ? c.row_uniform.p : nullptr;
  sr.sample_id = c.row_sample_id.p;
  sr.step = c.row_step.p;
  sr.forced = forced_tokens ? c.row_forced.p : nullptr;
  sr.seed = c.rd.seed;
  sr.tokens = c.out_tokens.p;
  sr.logprobs = c.out_logprobs.p;
  c.timer.begin("sample_kernel", 4.0 * B * m.vocab, 0, c.stream);
  if (B <= c.samp_rows) {
    sr.part_max = c.samp_part_max.p;
    sr.seg_sums = c.samp_seg_sums.p;
  }
  launch_sample(sr, B, m.vocab, c.stream);
  c.timer.end(c.stream);
  // pinned host memory is mapped for the device: the kernel stores the step's results there
  launch_scatter_tokens(c.st, c.row_slot.p, c.out_tokens.p, c.out_logprobs.p, B, 1, hi + 3 * R, c.h_float.p, c.stream);

  // prompts that end in this step: response position 0 of their samples
  std::vector<PendingPrompt*> fin;
  if (n_fin) {
    for (const ChunkSeq& cs : chunk->seqs)
      if (cs.last) fin.push_back(&c.queue.pending[cs.pending_index]);
    sample_first_tokens(c, B, fin);
  }
  wait_step_done(c);
  c.timer.collect();

  int i = 0;
  for (auto it = c.live.begin(); it != c.live.end(); ++i) {
    Sample& s = it->second;
    int tok = hi[3 * R + i];
    s.n_emitted += 1;
    s.last_token = tok;
    bool done = s.n_emitted >= s.max_new || (s.eos_id >= 0 && tok == s.eos_id);
    if (sample_ids) sample_ids[i] = s.id;
    if (groups) groups[i] = s.group;
    if (tokens) tokens[i] = tok;
    if (logprobs) logprobs[i] = c.h_float.p[i];
    if (finished) finished[i] = done ? 1 : 0;
    if (done) {
      release_sample(c, s);
      it = c.live.erase(it);
      c.stats.samples_finished += 1;
      c.live_dirty = true;
    } else {
      ++it;
    }
  }
  *n_live = B;
  if (B) c.stats.decode_steps += 1;
  c.stats.tokens_emitted += B;

  if (chunk) commit_chunk(c, *chunk, fin);
  refresh_stats(c);
}

__global__ void extend_slots_kernel(SlotState st, const int* __restrict__ slots, const int* __restrict__ new_pos,
                                    const int* __restrict__ tokens, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int sl = slots[i];
  st.last_token[sl] = tokens[i];
  st.pos[sl] = new_pos[i];
  st.step[sl] += 1;
}

// Appends tokens that the model did not generate to live samples' contexts and emits each
// sample's next response token: the sample's last response token and the appended tokens run
// through the model as one packed sequence that attends to the sample's cache (the same
// kernels as prefill, with a first position per sequence), and the next token is drawn from the
// logits of the last appended token.
static void extend_impl(rollout_ctx& c, int32_t n, const int64_t* sample_ids, const int32_t* tokens,
                        const int32_t* offsets, const int32_t* forced_next, const uint32_t* uniform_override,
                        int32_t* next_tokens, float* next_logprobs, uint8_t* finished) {
  const rollout_model_desc& m = c.md;
  const int T = c.page_tokens, R = c.r_max;
  PhaseClock clock(c.stats.extend_ms);
  if (n < 1 || !sample_ids || !tokens || !offsets) fail(ROLLOUT_E_INVAL, "bad arguments");
  if (offsets[0] != 0) fail(ROLLOUT_E_INVAL, "offsets[0] must be 0");
  if (n > rollout_ctx::kTempSlots || n > c.logit_rows) fail(ROLLOUT_E_NOMEM, "too many samples in one call");
  // ---- validation (no state changes before all of it passed) ----
  std::vector<Sample*> ss(n);
  std::vector<int> extra(n);
  long long rows = 0, extra_pages = 0;
  for (int i = 0; i < n; ++i) {
    auto it = c.live.find(sample_ids[i]);
    if (it == c.live.end()) fail(ROLLOUT_E_INVAL, "sample " + std::to_string(sample_ids[i]) + " is not live");
    for (int j = 0; j < i; ++j)
      if (sample_ids[j] == sample_ids[i]) fail(ROLLOUT_E_INVAL, "sample listed twice");
    Sample& s = it->second;
    ss[i] = &s;
    const int len = offsets[i + 1] - offsets[i];
    if (len < 1) fail(ROLLOUT_E_INVAL, "nothing to append");
    for (int k = offsets[i]; k < offsets[i + 1]; ++k)
      if (tokens[k] < 0 || tokens[k] >= m.vocab) fail(ROLLOUT_E_INVAL, "token out of range");
    if (forced_next && (forced_next[i] < 0 || forced_next[i] >= m.vocab)) fail(ROLLOUT_E_INVAL, "forced token out of range");
    const long long cached = (long long)s.prompt_len + len + s.max_new - 1;
    if (cached > c.rd.max_context) fail(ROLLOUT_E_NOMEM, "context + response exceeds max_context");
    extra[i] = std::max(0, ceil_div(cached, T) - (int)s.pages.size());
    extra_pages += extra[i];
    rows += len + 1;
  }
  if (rows > c.rd.max_batch_tokens || rows > R) fail(ROLLOUT_E_NOMEM, "appended tokens exceed max_batch_tokens");
  if (extra_pages > c.pool->unreserved()) fail(ROLLOUT_E_NOMEM, "not enough free KV pages");

  // ---- pages for the longer contexts ----
  for (int i = 0; i < n; ++i) {
    Sample& s = *ss[i];
    int* srow = &c.h_page_table[(size_t)s.slot * c.max_pages];
    for (int k = 0; k < extra[i]; ++k) {
      int32_t pg = c.pool->alloc(false);
      srow[s.pages.size()] = pg;
      s.pages.push_back(pg);
    }
  }
  if (extra_pages) engine_upload_page_table(c);

  // ---- rows: [last response token, appended tokens] per sample, positions after its cache ----
  int* hi = c.h_int.p;
  int r = 0, max_len = 0;
  double kv_tokens = 0, flops = 0;
  for (int i = 0; i < n; ++i) {
    Sample& s = *ss[i];
    const int len = offsets[i + 1] - offsets[i] + 1, p0 = s.prompt_len + s.n_emitted - 1;
    hi[4 * R + i] = r;
    hi[5 * R + i] = len;
    hi[6 * R + i] = s.slot;
    hi[7 * R + i] = p0;
    for (int k = 0; k < len; ++k, ++r) {
      hi[r] = k == 0 ? s.last_token : tokens[offsets[i] + k - 1];
      hi[R + r] = p0 + k;
      hi[2 * R + r] = s.slot;
    }
    hi[3 * R + i] = r - 1;  // last row: its logits give the next token
    max_len = std::max(max_len, len);
    kv_tokens += (double)len * p0 + 0.5 * len * (len + 1);
    flops += 4.0 * ((double)len * p0 + 0.5 * len * (len + 1)) * c.q_dim;
  }
  h2d(c.d_live.p, hi + 6 * R, n * sizeof(int), c.stream);
  c.live_dirty = true;  // d_live no longer holds the live list
  launch_gather_decode_rows(c.st, c.d_live.p, n, c.row_token.p, c.row_pos.p, c.row_slot.p, c.row_inv_temp.p,
                            c.row_top_p.p, c.row_sample_id.p, c.row_step.p, c.stream);
  h2d(c.row_token.p, hi, rows * sizeof(int), c.stream);
  h2d(c.row_pos.p, hi + R, rows * sizeof(int), c.stream);
  h2d(c.row_slot.p, hi + 2 * R, rows * sizeof(int), c.stream);
  h2d(c.row_aux.p, hi + 3 * R, n * sizeof(int), c.stream);
  SeqBatch sb{c.seq_row0.p, c.seq_len.p, c.seq_slot.p, n, max_len};
  if (!c.simple) {
    h2d(c.seq_row0.p, hi + 4 * R, n * sizeof(int), c.stream);
    h2d(c.seq_len.p, hi + 5 * R, n * sizeof(int), c.stream);
    h2d(c.seq_slot.p, hi + 6 * R, n * sizeof(int), c.stream);
    h2d(c.seq_pos0.p, hi + 7 * R, n * sizeof(int), c.stream);
    sb.pos0 = c.seq_pos0.p;
  }
  c.timer.start_call();
  c.kv_tokens_this_call = kv_tokens;
  c.attn_flops_this_call = flops;
  engine_forward_rows(c, (int)rows, &sb);
  engine_logits(c, c.row_aux.p, 0, n, c.logits.p);
  c.last_logit_rows = n;
  HIP_TRY(hipStreamSynchronize(c.stream));  // the staging buffers are reused below
  c.timer.collect();

  // ---- the next response token of every sample ----
  for (int i = 0; i < n; ++i) {
    Sample& s = *ss[i];
    hi[i] = s.prompt_len + (offsets[i + 1] - offsets[i]) + s.n_emitted;  // position of the token drawn now
    hi[R + i] = forced_next ? forced_next[i] : -1;
    hi[2 * R + i] = uniform_override ? (int)uniform_override[i] : 0;
  }
  h2d(c.row_aux.p + R, hi, n * sizeof(int), c.stream);
  h2d(c.row_forced.p, hi + R, n * sizeof(int), c.stream);
  h2d(c.row_uniform.p, hi + 2 * R, n * sizeof(int), c.stream);
  SampleRows sr{};
  sr.logits = c.logits.p;
  sr.logits_row = nullptr;
  sr.inv_temp = c.row_inv_temp.p;
  sr.top_p = c.row_top_p.p;
  sr.uniforms = uniform_override ? c.row_uniform.p : nullptr;
  sr.sample_id = c.row_sample_id.p;
  sr.step = c.row_step.p;
  sr.forced = forced_next ? c.row_forced.p : nullptr;
  sr.seed = c.rd.seed;
  sr.tokens = c.out_tokens.p;
  sr.logprobs = c.out_logprobs.p;
  if (n <= c.samp_rows) {
    sr.part_max = c.samp_part_max.p;
    sr.seg_sums = c.samp_seg_sums.p;
  }
  launch_sample(sr, n, m.vocab, c.stream);
  extend_slots_kernel<<<ceil_div(n, 256), 256, 0, c.stream>>>(c.st, c.d_live.p, c.row_aux.p + R, c.out_tokens.p, n);
  d2h(hi + 3 * R, c.out_tokens.p, n * sizeof(int), c.stream);
  d2h(c.h_float.p, c.out_logprobs.p, n * sizeof(float), c.stream);
  HIP_TRY(hipStreamSynchronize(c.stream));

  // ---- host bookkeeping ----
  for (int i = 0; i < n; ++i) {
    Sample& s = *ss[i];
    const int tok = hi[3 * R + i];
    s.prompt_len += offsets[i + 1] - offsets[i];
    s.n_emitted += 1;
    s.last_token = tok;
    const bool done = s.n_emitted >= s.max_new || (s.eos_id >= 0 && tok == s.eos_id);
    if (next_tokens) next_tokens[i] = tok;
    if (next_logprobs) next_logprobs[i] = c.h_float.p[i];
    if (finished) finished[i] = done ? 1 : 0;
    c.stats.prompt_tokens += offsets[i + 1] - offsets[i];
    c.stats.tokens_emitted += 1;
    if (done) {
      release_sample(c, s);
      c.live.erase(sample_ids[i]);
      c.stats.samples_finished += 1;
    }
  }
  refresh_stats(c);
}

// The target is reached: abort what still runs, drop what still waits or is half cached.
static void close_queue(rollout_ctx& c) {
  PromptQueue& q = c.queue;
  const int running = (int)c.live.size();
  for (auto& kv : c.live) release_sample(c, kv.second);
  c.live.clear();
  c.live_dirty = true;
  c.stats.samples_aborted += running;
  q.aborted += running;
  for (PendingPrompt& pp : q.pending) release_pending(c, pp);
  q.pending.clear();
  q.waiting.clear();
  q.open.clear();
  q.admitted.clear();
  q.closed = true;
  refresh_stats(c);
}

// One step of the queue-fed rollout with chunked prefill (paper section 4.3, "add request" while
// the other samples keep decoding): a single forward pass carries one decode row per live sample
// and up to chunk_rows rows of the pending prompts.  A prompt's samples emit response position 0
// in the step that caches its last rows and take part in the decode rows from the next step on.
static void queue_step_chunked(rollout_ctx& c, int cap, int32_t* n_out, int32_t* n_admitted, int64_t* sample_ids,
                               int32_t* tokens, float* logprobs, uint8_t* finished) {
  PromptQueue& q = c.queue;
  const int n = q.n_samples;
  // (0) growing pages: make room for the pages this step writes - first the prompts that are only
  // half cached (nothing of theirs is lost but the work), then the youngest running prompt
  int n_preempted = 0;
  if (c.grow_pages) {
    while (pages_missing_for_step(c) > c.pool->unreserved()) {
      if (queue_preempt_pending(c)) {
        ++n_preempted;
        continue;
      }
      const int dropped = queue_preempt_youngest(c, nullptr);
      if (!dropped) fail(ROLLOUT_E_NOMEM, "the KV pool is exhausted and no queued prompt can give way: abort samples");
      c.stats.samples_aborted += dropped;
      n_preempted += dropped;
    }
  }
  // (1) admission: keep about one step's worth of prompt rows pending
  bool admitted_any = false;
  if (!n_preempted && !q.waiting.empty() && pending_rows_left(q) < q.chunk_rows) {
    int k = queue_select_run(c, AdmissionLimits{(int)q.free_rows.size(), (long long)c.r_max});
    while (k-- > 0 && pending_rows_left(q) < q.chunk_rows) {
      queue_admit_pending(c);
      admitted_any = true;
    }
  }
  if (admitted_any) engine_upload_page_table(c);
  // (2) the step's rows
  const int B = (int)c.live.size();
  StepChunk chunk;
  const long long budget = std::min<long long>({(long long)q.chunk_rows, (long long)c.r_max - B, (long long)rollout_ctx::kTempSlots});
  const int max_fin = (int)std::min<long long>(c.logit_rows - B, ((long long)c.r_max - B) / std::max(n, 1));
  chunk.rows = plan_chunk(q, budget, std::max(max_fin, 0), chunk.seqs);
  int n_adm = 0;
  for (const ChunkSeq& cs : chunk.seqs) n_adm += cs.last ? n : 0;
  if (cap < B + n_adm) fail(ROLLOUT_E_INVAL, "output capacity smaller than live samples + samples of the prompts that end");
  // (3) one forward pass for both
  int n_dec = cap - n_adm;
  std::vector<int64_t> ids_dec(B), grp_dec(B);
  std::vector<uint8_t> fin_dec(B);
  decode_impl(c, nullptr, nullptr, &n_dec, ids_dec.data(), tokens ? tokens + n_adm : nullptr,
              logprobs ? logprobs + n_adm : nullptr, fin_dec.data(), grp_dec.data(), &chunk);
  for (int i = 0; i < n_adm; ++i) {
    if (sample_ids) sample_ids[i] = chunk.first_ids[i];
    if (tokens) tokens[i] = chunk.first_tokens[i];
    if (logprobs) logprobs[i] = chunk.first_logprobs[i];
    if (finished) finished[i] = chunk.first_finished[i];
    if (chunk.first_finished[i]) queue_note_finished(q, chunk.first_groups[i]);
  }
  for (int i = 0; i < n_dec; ++i) {
    if (sample_ids) sample_ids[n_adm + i] = ids_dec[i];
    if (finished) finished[n_adm + i] = fin_dec[i];
    if (fin_dec[i]) queue_note_finished(q, grp_dec[i]);
  }
  *n_admitted = n_adm;
  *n_out = n_adm + n_dec;
  // (4) enough prompts complete
  if (q.target > 0 && q.completed >= (uint64_t)q.target) close_queue(c);
}

extern "C" {

int rollout_abi_version(void) { return ROLLOUT_ABI_VERSION; }

const char* rollout_last_error(rollout_ctx* ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

int rollout_init(rollout_ctx** out, const rollout_model_desc* model, const rollout_weights* weights,
                 const rollout_runtime_desc* runtime) {
  if (out) *out = nullptr;
  rollout_ctx* c = nullptr;
  int rc = guarded(nullptr, [&] {
    if (!out || !model || !weights || !runtime) fail(ROLLOUT_E_INVAL, "null argument");
    c = new rollout_ctx();
    c->md = *model;
    c->rd = *runtime;
    engine_init(*c, *weights);
    (void)rollout_sample_static_prepare();  // address of the static sampler scratch on this device
    if (const char* t = std::getenv("ROLLOUT_STEP_TIMEOUT_MS")) c->step_timeout_s = std::atof(t) * 1e-3;
    refresh_stats(*c);
  });
  if (rc != ROLLOUT_OK) {
    delete c;
    return rc;
  }
  *out = c;
  return ROLLOUT_OK;
}

void rollout_destroy(rollout_ctx* ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);
  delete ctx;
}

int rollout_get_stats(rollout_ctx* ctx, rollout_stats* out) {
  if (!ctx || !out) return ROLLOUT_E_INVAL;
  refresh_stats(*ctx);
  *out = ctx->stats;
  return ROLLOUT_OK;
}

int rollout_kernel_stats(rollout_ctx* ctx, int32_t* n, rollout_kernel_stat* out) {
  if (!ctx || !n || (*n > 0 && !out)) return ROLLOUT_E_INVAL;
  int k = 0;
  for (auto& kv : ctx->timer.acc) {
    if (k >= *n) break;
    std::memset(&out[k], 0, sizeof(out[k]));
    std::strncpy(out[k].name, kv.first.c_str(), sizeof(out[k].name) - 1);
    out[k].launches = kv.second.launches;
    out[k].ms = kv.second.ms;
    out[k].bytes = kv.second.bytes;
    out[k].flops = kv.second.flops;
    ++k;
  }
  *n = k;
  return ROLLOUT_OK;
}

int rollout_live_samples(rollout_ctx* ctx, int32_t capacity, int64_t* ids) {
  if (!ctx) return ROLLOUT_E_INVAL;
  if (ids) {
    int32_t i = 0;
    for (auto& kv : ctx->live) {
      if (i >= capacity) break;
      ids[i++] = kv.first;
    }
  }
  return (int)ctx->live.size();
}

int rollout_prefill(rollout_ctx* ctx, int32_t n_prompts, const int32_t* tokens, const int32_t* offsets,
                    int32_t n_samples, const int32_t* max_new_tokens, int32_t eos_id, float temperature,
                    float top_p, const int32_t* forced_first, const uint32_t* uniform_override,
                    int64_t* sample_ids, int32_t* first_tokens, float* first_logprobs, uint8_t* finished) {
  if (!ctx) return ROLLOUT_E_INVAL;
  return guarded(ctx, [&] {
    check_usable(*ctx);
    prefill_impl(*ctx, n_prompts, tokens, offsets, n_samples, max_new_tokens, eos_id, temperature, top_p,
                 forced_first, uniform_override, nullptr, nullptr, sample_ids, first_tokens, first_logprobs,
                 finished);
  });
}

int rollout_decode_step(rollout_ctx* ctx, const int32_t* forced_tokens, const uint32_t* uniform_override,
                        int32_t* n_live, int64_t* sample_ids, int32_t* tokens, float* logprobs,
                        uint8_t* finished) {
  if (!ctx) return ROLLOUT_E_INVAL;
  return guarded(ctx, [&] {
    check_usable(*ctx);
    decode_impl(*ctx, forced_tokens, uniform_override, n_live, sample_ids, tokens, logprobs, finished);
  });
}

// ---- queue-fed continuous rollout -------------------------------------------------------
int rollout_queue_push(rollout_ctx* ctx, int32_t n_prompts, const int32_t* tokens, const int32_t* offsets,
                       int32_t n_samples, const int32_t* max_new_tokens, int32_t eos_id, float temperature,
                       float top_p, int64_t* first_sample_ids) {
  if (!ctx) return ROLLOUT_E_INVAL;
  return guarded(ctx, [&] {
    rollout_ctx& c = *ctx;
    check_usable(c);
    PromptQueue& q = c.queue;
    const int P = n_prompts, n = n_samples;
    if (P < 1 || n < 1 || !tokens || !offsets || !max_new_tokens) fail(ROLLOUT_E_INVAL, "bad prompt arguments");
    if (q.closed) fail(ROLLOUT_E_INVAL, "the queue is closed");
    if (q.n_samples && q.n_samples != n) fail(ROLLOUT_E_INVAL, "n_samples differs from earlier pushes");
    if (!(temperature > 0.f) || !std::isfinite(temperature)) fail(ROLLOUT_E_INVAL, "temperature must be > 0");
    if (!(top_p >= 0.f)) fail(ROLLOUT_E_INVAL, "top_p must be >= 0");
    if (eos_id < -1 || eos_id >= c.md.vocab) fail(ROLLOUT_E_INVAL, "eos_id out of range");
    if (offsets[0] != 0) fail(ROLLOUT_E_INVAL, "offsets[0] must be 0");
    if (n > c.r_max) fail(ROLLOUT_E_NOMEM, "n_samples exceeds the workspace rows");
    std::vector<QueuedPrompt> fresh(P);
    for (int p = 0; p < P; ++p) {
      const int len = offsets[p + 1] - offsets[p];
      if (len < 1) fail(ROLLOUT_E_INVAL, "empty prompt");
      if (len > c.rd.max_batch_tokens) fail(ROLLOUT_E_NOMEM, "prompt longer than max_batch_tokens");
      QueuedPrompt& e = fresh[p];
      e.tokens.assign(tokens + offsets[p], tokens + offsets[p + 1]);
      e.max_new.assign(max_new_tokens + (size_t)p * n, max_new_tokens + (size_t)(p + 1) * n);
      e.eos_id = eos_id;
      e.temperature = temperature;
      e.top_p = top_p;
      for (int t : e.tokens)
        if (t < 0 || t >= c.md.vocab) fail(ROLLOUT_E_INVAL, "prompt token out of range");
      for (int mn : e.max_new) {
        if (mn < 1) fail(ROLLOUT_E_INVAL, "max_new_tokens must be >= 1");
        if ((long long)len + mn - 1 > c.rd.max_context) fail(ROLLOUT_E_NOMEM, "prompt + response exceeds max_context");
      }
      // alone in an idle context the prompt must fit whatever its samples do, so that it always makes progress
      if (admission_slots(n, e.max_new.data()) > c.rd.max_live_samples)
        fail(ROLLOUT_E_NOMEM, "more samples than live-sample slots");
      if (plan_pages(len, c.page_tokens, n, e.max_new.data(), nullptr, nullptr, nullptr) > c.pool->total())
        fail(ROLLOUT_E_NOMEM, "more pages than the pool holds");
    }
    q.n_samples = n;
    for (int p = 0; p < P; ++p) {
      fresh[p].prompt_id = c.prompt_counter++;
      fresh[p].first_sample = c.next_sample_id;
      c.next_sample_id += n;
      if (first_sample_ids) first_sample_ids[p] = fresh[p].first_sample;
      q.waiting.push_back(std::move(fresh[p]));
    }
    q.pushed += P;
  });
}

int rollout_queue_policy(rollout_ctx* ctx, int32_t admit_min_prompts, int32_t target_prompts) {
  if (!ctx || admit_min_prompts < 1 || target_prompts < 0) return ROLLOUT_E_INVAL;
  ctx->queue.admit_min = admit_min_prompts;
  ctx->queue.target = target_prompts;
  return ROLLOUT_OK;
}

int rollout_queue_chunking(rollout_ctx* ctx, int32_t chunk_rows) {
  if (!ctx || chunk_rows < 0) return ROLLOUT_E_INVAL;
  return guarded(ctx, [&] {
    if (chunk_rows > 0 && ctx->simple) fail(ROLLOUT_E_STATE, "chunked prefill runs on the matrix-core path only");
    if (!ctx->queue.pending.empty()) fail(ROLLOUT_E_STATE, "a prompt's prefill is under way");
    ctx->queue.chunk_rows = chunk_rows;
  });
}

int rollout_queue_get_stats(rollout_ctx* ctx, rollout_queue_stats* out) {
  if (!ctx || !out) return ROLLOUT_E_INVAL;
  const PromptQueue& q = ctx->queue;
  out->prompts_pushed = q.pushed;
  out->prompts_admitted = q.admitted_count;
  out->prompts_completed = q.completed;
  out->samples_aborted = q.aborted;
  out->prompts_preempted = q.preempted;
  out->prompts_waiting = (int32_t)q.waiting.size();
  out->prompts_pending = (int32_t)q.pending.size();
  out->closed = q.closed ? 1 : 0;
  return ROLLOUT_OK;
}

int rollout_queue_step(rollout_ctx* ctx, int32_t* n_out, int32_t* n_admitted, int64_t* sample_ids,
                       int32_t* tokens, float* logprobs, uint8_t* finished) {
  if (!ctx) return ROLLOUT_E_INVAL;
  return guarded(ctx, [&] {
    rollout_ctx& c = *ctx;
    PromptQueue& q = c.queue;
    check_usable(c);
    if (!n_out || !n_admitted) fail(ROLLOUT_E_INVAL, "n_out / n_admitted is null");
    const int cap = *n_out, n = q.n_samples;
    *n_out = 0;
    *n_admitted = 0;
    if (q.closed) return;
    if (q.chunk_rows > 0) {
      queue_step_chunked(c, cap, n_out, n_admitted, sample_ids, tokens, logprobs, finished);
      return;
    }

    // (0) growing pages: make room for this step's new pages - the youngest queued prompt gives way
    int n_preempted = 0;
    if (c.grow_pages) {
      while (pages_missing_for_step(c) > c.pool->unreserved()) {
        const int dropped = queue_preempt_youngest(c, nullptr);
        if (!dropped) fail(ROLLOUT_E_NOMEM, "the KV pool is exhausted and no queued prompt can give way: abort samples");
        c.stats.samples_aborted += dropped;
        n_preempted += dropped;
      }
    }
    // (1) the longest run of waiting prompts, in push order, that one prefill call can take
    int k = n_preempted ? 0 : queue_select_run(c, AdmissionLimits{std::min(rollout_ctx::kTempSlots, c.logit_rows), (long long)c.r_max});
    long long rows = 0;
    for (int i = 0; i < k; ++i) rows += (long long)q.waiting[i].tokens.size();
    const int live_before = (int)c.live.size();
    if (cap < live_before + 2 * k * n) fail(ROLLOUT_E_INVAL, "output capacity smaller than live samples + 2 x admitted samples");
    std::vector<uint8_t> fin_local;
    int n_adm = 0;
    if (k > 0) {
      std::vector<int32_t> toks, offs(1, 0), max_new;
      std::vector<int64_t> pids, firsts;
      toks.reserve((size_t)rows);
      for (int i = 0; i < k; ++i) {
        const QueuedPrompt& e = q.waiting[i];
        toks.insert(toks.end(), e.tokens.begin(), e.tokens.end());
        offs.push_back((int32_t)toks.size());
        max_new.insert(max_new.end(), e.max_new.begin(), e.max_new.end());
        pids.push_back(e.prompt_id);
        firsts.push_back(e.first_sample);
      }
      n_adm = k * n;
      std::vector<int64_t> ids_local(n_adm);
      fin_local.assign(n_adm, 0);
      const int eos_id = q.waiting[0].eos_id;
      const float temperature = q.waiting[0].temperature, top_p = q.waiting[0].top_p;
      prefill_impl(c, k, toks.data(), offs.data(), n, max_new.data(), eos_id, temperature, top_p,
                   nullptr, nullptr, pids.data(), firsts.data(), ids_local.data(), tokens, logprobs,
                   fin_local.data());
      for (int i = 0; i < k; ++i) {
        q.open[pids[i]] = n;
        if (c.grow_pages) q.admitted.emplace(pids[i], q.waiting[i]);  // kept: it may have to start over
      }
      for (int i = 0; i < n_adm; ++i) {
        if (sample_ids) sample_ids[i] = ids_local[i];
        if (finished) finished[i] = fin_local[i];
        if (fin_local[i]) queue_note_finished(q, pids[i / n]);
      }
      q.waiting.erase(q.waiting.begin(), q.waiting.begin() + k);
      q.admitted_count += k;
    }

    // (2) one decode step over everything that is live now
    int n_dec = cap - n_adm;
    std::vector<int64_t> ids_dec(c.live.size()), grp_dec(c.live.size());
    std::vector<uint8_t> fin_dec(c.live.size());
    decode_impl(c, nullptr, nullptr, &n_dec, ids_dec.data(), tokens ? tokens + n_adm : nullptr,
                logprobs ? logprobs + n_adm : nullptr, fin_dec.data(), grp_dec.data());
    for (int i = 0; i < n_dec; ++i) {
      if (sample_ids) sample_ids[n_adm + i] = ids_dec[i];
      if (finished) finished[n_adm + i] = fin_dec[i];
      if (fin_dec[i]) queue_note_finished(q, grp_dec[i]);
    }
    *n_admitted = n_adm;
    *n_out = n_adm + n_dec;

    // (3) enough prompts complete: abort what still runs, drop what still waits
    if (q.target > 0 && q.completed >= (uint64_t)q.target) close_queue(c);
  });
}

int rollout_extend(rollout_ctx* ctx, int32_t n, const int64_t* sample_ids, const int32_t* tokens,
                   const int32_t* offsets, const int32_t* forced_next, const uint32_t* uniform_override,
                   int32_t* next_tokens, float* next_logprobs, uint8_t* finished) {
  if (!ctx) return ROLLOUT_E_INVAL;
  return guarded(ctx, [&] {
    check_usable(*ctx);
    extend_impl(*ctx, n, sample_ids, tokens, offsets, forced_next, uniform_override, next_tokens, next_logprobs,
                finished);
  });
}

int rollout_update_weights(rollout_ctx* ctx, int32_t n, const rollout_tensor_update* updates) {
  if (!ctx) return ROLLOUT_E_INVAL;
  return guarded(ctx, [&] {
    rollout_ctx& c = *ctx;
    check_usable(c);
    if (n < 0 || (n > 0 && !updates)) fail(ROLLOUT_E_INVAL, "bad arguments");
    if (!c.live.empty() || !c.queue.waiting.empty() || !c.queue.pending.empty())
      fail(ROLLOUT_E_STATE, "weights cannot change while samples are live or prompts wait");
    for (int i = 0; i < n; ++i) {  // the whole bucket is checked before any of it is applied
      const rollout_tensor_update& u = updates[i];
      if (!u.data) fail(ROLLOUT_E_INVAL, "null weight pointer");
      engine_check_tensor(c, u.layer, u.tensor);
    }
    for (int i = 0; i < n; ++i) engine_load_tensor(c, updates[i].layer, updates[i].tensor, updates[i].data);
    HIP_TRY(hipStreamSynchronize(c.stream));
    c.h_is_final = false;
  });
}

int rollout_abort(rollout_ctx* ctx, int32_t n, const int64_t* sample_ids) {
  if (!ctx || n < 0 || (n > 0 && !sample_ids)) return ROLLOUT_E_INVAL;
  int aborted = 0;
  for (int i = 0; i < n; ++i) {
    auto it = ctx->live.find(sample_ids[i]);
    if (it == ctx->live.end()) continue;
    queue_note_finished(ctx->queue, it->second.group);  // it no longer holds its prompt open
    release_sample(*ctx, it->second);
    ctx->live.erase(it);
    ++aborted;
  }
  if (aborted) ctx->live_dirty = true;
  ctx->stats.samples_aborted += aborted;
  refresh_stats(*ctx);
  return aborted;
}

int rollout_debug_logits(rollout_ctx* ctx, int32_t* rows, float* out) {
  if (!ctx) return ROLLOUT_E_INVAL;
  return guarded(ctx, [&] {
    rollout_ctx& c = *ctx;
    if (!rows || !out) fail(ROLLOUT_E_INVAL, "null argument");
    if (c.last_logit_rows < 1) fail(ROLLOUT_E_STATE, "no logits computed yet");
    if (*rows < c.last_logit_rows) fail(ROLLOUT_E_INVAL, "capacity smaller than the number of rows");
    HIP_TRY(hipMemcpyAsync(out, c.logits.p, (size_t)c.last_logit_rows * c.md.vocab * sizeof(float),
                           hipMemcpyDeviceToHost, c.stream));
    HIP_TRY(hipStreamSynchronize(c.stream));
    *rows = c.last_logit_rows;
  });
}

int rollout_debug_routing(rollout_ctx* ctx, int32_t* rows, int32_t* out) {
  if (!ctx) return ROLLOUT_E_INVAL;
  return guarded(ctx, [&] {
    rollout_ctx& c = *ctx;
    if (!rows || !out) fail(ROLLOUT_E_INVAL, "null argument");
    if (!c.route_log.p || c.last_route_rows < 1) fail(ROLLOUT_E_STATE, "routing is not being recorded");
    if (*rows < c.last_route_rows) fail(ROLLOUT_E_INVAL, "capacity smaller than the number of rows");
    const int k = c.md.top_k, n = c.last_route_rows;
    HIP_TRY(hipMemcpy2DAsync(out, (size_t)n * k * sizeof(int), c.route_log.p, (size_t)c.r_max * k * sizeof(int),
                             (size_t)n * k * sizeof(int), c.md.n_layers, hipMemcpyDeviceToHost, c.stream));
    HIP_TRY(hipStreamSynchronize(c.stream));
    *rows = n;
  });
}

int rollout_logprobs(rollout_ctx* ctx, int32_t n_seqs, const int32_t* tokens, const int32_t* cu_seqlens,
                     float temperature, float* logprobs) {
  if (!ctx) return ROLLOUT_E_INVAL;
  return guarded(ctx, [&] {
    rollout_ctx& c = *ctx;
    check_usable(c);
    const rollout_model_desc& m = c.md;
    const int T = c.page_tokens, R = c.r_max;
    PhaseClock clock(c.stats.logprobs_ms);
    if (n_seqs < 0 || !cu_seqlens || (n_seqs > 0 && (!tokens || !logprobs))) fail(ROLLOUT_E_INVAL, "null argument");
    if (!(temperature > 0.f) || !std::isfinite(temperature)) fail(ROLLOUT_E_INVAL, "temperature must be > 0");
    if (n_seqs && cu_seqlens[0] != 0) fail(ROLLOUT_E_INVAL, "cu_seqlens[0] must be 0");
    const int max_seq = std::min(c.rd.max_batch_tokens, c.rd.max_context);
    for (int s = 0; s < n_seqs; ++s) {
      int len = cu_seqlens[s + 1] - cu_seqlens[s];
      if (len < 1) fail(ROLLOUT_E_INVAL, "empty sequence");
      if (len > max_seq) fail(ROLLOUT_E_NOMEM, "sequence longer than max_batch_tokens or max_context");
      if (ceil_div(len, T) > c.pool->unreserved()) fail(ROLLOUT_E_NOMEM, "not enough free KV pages for one sequence");
      for (int i = cu_seqlens[s]; i < cu_seqlens[s + 1]; ++i)
        if (tokens[i] < 0 || tokens[i] >= m.vocab) fail(ROLLOUT_E_INVAL, "token out of range");
    }
    const float inv_t = 1.0f / temperature;
    int s0 = 0;
    while (s0 < n_seqs) {
      // chunk of whole sequences bounded by rows, temporary slots and free pages
      int s1 = s0, rows = 0, pages = 0;
      while (s1 < n_seqs && s1 - s0 < rollout_ctx::kTempSlots) {
        int len = cu_seqlens[s1 + 1] - cu_seqlens[s1];
        if (rows + len > c.rd.max_batch_tokens || pages + ceil_div(len, T) > c.pool->unreserved()) break;
        rows += len;
        pages += ceil_div(len, T);
        ++s1;
      }
      Rollback held(c);  // the chunk's scratch pages: back to the pool however the chunk ends
      int* ht = c.h_int.p;
      int r = 0, max_len = 0;
      for (int s = s0; s < s1; ++s) {
        int len = cu_seqlens[s + 1] - cu_seqlens[s];
        ht[4 * R + (s - s0)] = r;
        ht[5 * R + (s - s0)] = len;
        ht[6 * R + (s - s0)] = c.temp_slot0 + (s - s0);
        max_len = std::max(max_len, len);
        int* prow = &c.h_page_table[(size_t)(c.temp_slot0 + (s - s0)) * c.max_pages];
        for (int i = 0; i < ceil_div(len, T); ++i) prow[i] = held.alloc();
        for (int i = 0; i < len; ++i, ++r) {
          int g = cu_seqlens[s] + i;
          ht[r] = tokens[g];
          ht[R + r] = i;
          ht[2 * R + r] = c.temp_slot0 + (s - s0);
          ht[3 * R + r] = i + 1 < len ? tokens[g + 1] : -1;  // target of this row
        }
      }
      engine_upload_page_table(c);
      h2d(c.row_token.p, ht, rows * sizeof(int), c.stream);
      h2d(c.row_pos.p, ht + R, rows * sizeof(int), c.stream);
      h2d(c.row_slot.p, ht + 2 * R, rows * sizeof(int), c.stream);
      h2d(c.row_aux.p, ht + 3 * R, rows * sizeof(int), c.stream);
      SeqBatch sb{c.seq_row0.p, c.seq_len.p, c.seq_slot.p, s1 - s0, max_len};
      if (!c.simple) {
        h2d(c.seq_row0.p, ht + 4 * R, (s1 - s0) * sizeof(int), c.stream);
        h2d(c.seq_len.p, ht + 5 * R, (s1 - s0) * sizeof(int), c.stream);
        h2d(c.seq_slot.p, ht + 6 * R, (s1 - s0) * sizeof(int), c.stream);
      }
      c.timer.start_call();
      c.kv_tokens_this_call = rows;
      c.attn_flops_this_call = 0;
      for (int s = s0; s < s1; ++s) {
        double len = cu_seqlens[s + 1] - cu_seqlens[s];
        c.attn_flops_this_call += 2.0 * len * (len + 1) * c.q_dim;
      }
      engine_forward_rows(c, rows, &sb);
      engine_target_logprobs(c, rows, c.row_aux.p, inv_t, c.out_logprobs.p);
      d2h(c.h_float.p, c.out_logprobs.p, rows * sizeof(float), c.stream);
      HIP_TRY(hipStreamSynchronize(c.stream));
      c.timer.collect();
      // row i of a sequence holds log p(token i+1); shift by one and zero the first entry
      r = 0;
      for (int s = s0; s < s1; ++s) {
        int a = cu_seqlens[s], len = cu_seqlens[s + 1] - a;
        logprobs[a] = 0.f;
        for (int i = 0; i + 1 < len; ++i) logprobs[a + i + 1] = c.h_float.p[r + i];
        r += len;
      }
      c.last_logit_rows = 0;
      s0 = s1;
    }
    refresh_stats(c);
  });
}

}  // extern "C"

// Device scratch of the two context-free entry points below: one grow-only buffer per device,
// kept until the process ends, so that a call allocates only when it needs more than any call
// before it.  The mutex is held for the whole call (both calls return after their stream has
// drained), so calls on one device take turns.
namespace {
struct CallScratch {
  std::mutex mu;
  char* p = nullptr;
  size_t bytes = 0;
  size_t used = 0;
  void begin() { used = 0; }
  void reserve(size_t need) {
    if (need <= bytes) return;
    if (p) (void)hipFree(p);
    p = nullptr;
    bytes = 0;
    HIP_TRY(hipMalloc((void**)&p, need));
    bytes = need;
  }
  template <typename T>
  T* take(size_t count) {  // after reserve(): 256-byte aligned pieces of the buffer
    T* out = (T*)(p + used);
    used += (count * sizeof(T) + 255) / 256 * 256;
    return out;
  }
  static size_t piece(size_t bytes_) { return (bytes_ + 255) / 256 * 256; }
};
CallScratch& call_scratch() {
  static CallScratch per_device[64];
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) throw ApiError{ROLLOUT_E_HIP, "device index out of range"};
  return per_device[dev];
}
}  // namespace

extern "C" {

int rollout_sample(const float* logits, int32_t rows, int32_t vocab, float temperature, float top_p,
                   const uint32_t* uniforms, const int32_t* forced, void* hip_stream, int32_t* tokens,
                   float* logprobs, uint64_t* weight_sums) {
  return guarded(nullptr, [&] {
    if (!logits || rows < 0 || vocab < 1 || vocab > 262144 || !uniforms || !tokens || !logprobs)
      fail(ROLLOUT_E_INVAL, "bad argument");
    if (!(temperature > 0.f) || !std::isfinite(temperature) || !(top_p >= 0.f)) fail(ROLLOUT_E_INVAL, "bad sampling parameters");
    if (forced)
      for (int i = 0; i < rows; ++i)
        if (forced[i] >= vocab) fail(ROLLOUT_E_INVAL, "forced token out of range");
    if (rows == 0) return;
    hipStream_t s = (hipStream_t)hip_stream;
    CallScratch& cs = call_scratch();
    std::lock_guard<std::mutex> lock(cs.mu);
    const size_t R = rows;
    cs.reserve(4 * CallScratch::piece(R * 4) + 2 * CallScratch::piece(R * 4) + CallScratch::piece(R * 8) +
               CallScratch::piece(R * kSampleParts * 4) + CallScratch::piece(R * kSampleSegments * 8));
    cs.begin();
    float *invt = cs.take<float>(R), *tp = cs.take<float>(R), *lp = cs.take<float>(R);
    unsigned* un = cs.take<unsigned>(R);
    int *fo = cs.take<int>(R), *tok = cs.take<int>(R);
    unsigned long long* ws = cs.take<unsigned long long>(R);
    std::vector<float> hv(rows, 1.0f / temperature), hp(rows, top_p);
    HIP_TRY(hipMemcpyAsync(invt, hv.data(), rows * sizeof(float), hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(tp, hp.data(), rows * sizeof(float), hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(un, uniforms, rows * sizeof(unsigned), hipMemcpyHostToDevice, s));
    if (forced) HIP_TRY(hipMemcpyAsync(fo, forced, rows * sizeof(int), hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));  // host staging vectors are pageable
    SampleRows sr{};
    sr.logits = logits;
    sr.inv_temp = invt;
    sr.top_p = tp;
    sr.uniforms = un;
    sr.forced = forced ? fo : nullptr;
    sr.tokens = tok;
    sr.logprobs = lp;
    sr.weight_sums = ws;
    sr.part_max = cs.take<float>(R * kSampleParts);
    sr.seg_sums = cs.take<unsigned long long>(R * kSampleSegments);
    launch_sample(sr, rows, vocab, s);
    HIP_TRY(hipMemcpyAsync(tokens, tok, rows * sizeof(int), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(logprobs, lp, rows * sizeof(float), hipMemcpyDeviceToHost, s));
    if (weight_sums)
      HIP_TRY(hipMemcpyAsync(weight_sums, ws, rows * sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
  });
}

int rollout_policy_loss(int32_t n_seqs, const int32_t* cu_seqlens, const float* logp_new, const float* logp_old,
                        const float* logp_ref, const uint8_t* mask, const float* rewards,
                        const rollout_loss_params* params, void* hip_stream, float* loss, float* grad,
                        float* advantages) {
  return guarded(nullptr, [&] {
    if (n_seqs < 0 || !cu_seqlens || !params || !loss) fail(ROLLOUT_E_INVAL, "bad argument");
    if (cu_seqlens[0] != 0) fail(ROLLOUT_E_INVAL, "cu_seqlens[0] must be 0");
    for (int i = 0; i < n_seqs; ++i)
      if (cu_seqlens[i + 1] < cu_seqlens[i]) fail(ROLLOUT_E_INVAL, "cu_seqlens must not decrease");
    const long long total = cu_seqlens[n_seqs];
    if (total > 0 && (!logp_new || !logp_old || !mask || !grad || !rewards)) fail(ROLLOUT_E_INVAL, "null array");
    const rollout_loss_params& q = *params;
    if (!(q.gamma >= 0.f) || !(q.reward_clip >= 0.f) || !(q.adv_clip >= 0.f) || !(q.eps_low >= 0.f) ||
        !(q.eps_high >= 0.f) || !std::isfinite(q.kl_coef))
      fail(ROLLOUT_E_INVAL, "bad loss parameters");
    hipStream_t s = (hipStream_t)hip_stream;
    CallScratch& cs = call_scratch();
    std::lock_guard<std::mutex> lock(cs.mu);
    const size_t S1 = (size_t)std::max(n_seqs, 1);
    cs.reserve(CallScratch::piece((S1 + 1) * 4) + CallScratch::piece(S1 * 4) + CallScratch::piece(2 * S1 * 4) +
               CallScratch::piece(2 * 4));
    cs.begin();
    struct { int* p; } cu{cs.take<int>(S1 + 1)};
    struct { float* p; } rw{cs.take<float>(S1)}, part{cs.take<float>(2 * S1)}, result{cs.take<float>(2)};
    HIP_TRY(hipMemcpyAsync(cu.p, cu_seqlens, (n_seqs + 1) * sizeof(int), hipMemcpyHostToDevice, s));
    if (n_seqs) HIP_TRY(hipMemcpyAsync(rw.p, rewards, n_seqs * sizeof(float), hipMemcpyHostToDevice, s));
    PolicyLossArgs p{};
    p.n_seqs = n_seqs;
    p.total = total;
    p.cu_seqlens = cu.p;
    p.logp_new = logp_new;
    p.logp_old = logp_old;
    p.logp_ref = logp_ref;
    p.mask = mask;
    p.rewards = rw.p;
    p.gamma = q.gamma;
    p.kl_coef = q.kl_coef;
    p.reward_clip = q.reward_clip;
    p.adv_clip = q.adv_clip;
    p.eps_low = q.eps_low;
    p.eps_high = q.eps_high;
    p.grad = grad;
    p.advantages = advantages;
    p.part_sum = part.p;
    p.part_cnt = part.p + std::max(n_seqs, 1);
    p.result = result.p;
    launch_policy_loss(p, s);
    float out[2];
    HIP_TRY(hipMemcpyAsync(out, result.p, sizeof(out), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    *loss = out[0];
  });
}

int rollout_philox_words(uint64_t seed, int32_t n, const int64_t* sample_ids, const uint32_t* steps,
                         uint32_t* words) {
  return guarded(nullptr, [&] {
    if (n < 0 || (n > 0 && (!sample_ids || !steps || !words))) fail(ROLLOUT_E_INVAL, "bad argument");
    if (n == 0) return;
    DevBuf<long long> ids;
    DevBuf<unsigned> st, out;
    ids.alloc(n); st.alloc(n); out.alloc(n);
    HIP_TRY(hipMemcpy(ids.p, sample_ids, n * sizeof(long long), hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(st.p, steps, n * sizeof(unsigned), hipMemcpyHostToDevice));
    launch_philox_words(seed, ids.p, st.p, out.p, n, nullptr);
    HIP_TRY(hipMemcpy(words, out.p, n * sizeof(unsigned), hipMemcpyDeviceToHost));
  });
}

// ---- host-side page pool ------------------------------------------------------------------
rollout_pool* rollout_pool_create(int32_t n_pages) { return n_pages > 0 ? new (std::nothrow) rollout_pool(n_pages) : nullptr; }
void rollout_pool_destroy(rollout_pool* p) { delete p; }
int32_t rollout_pool_free_pages(const rollout_pool* p) { return p ? p->free_pages() : ROLLOUT_E_INVAL; }
int32_t rollout_pool_unreserved(const rollout_pool* p) { return p ? p->unreserved() : ROLLOUT_E_INVAL; }
int rollout_pool_reserve(rollout_pool* p, int32_t n) {
  if (!p || n < 0) return ROLLOUT_E_INVAL;
  return p->reserve(n) ? ROLLOUT_OK : ROLLOUT_E_NOMEM;
}
void rollout_pool_unreserve(rollout_pool* p, int32_t n) {
  if (p && n > 0) p->unreserve(n);
}
int32_t rollout_pool_alloc(rollout_pool* p, int from_reservation) {
  if (!p) return ROLLOUT_E_INVAL;
  int32_t pg = p->alloc(from_reservation != 0);
  return pg < 0 ? ROLLOUT_E_NOMEM : pg;
}
int rollout_pool_retain(rollout_pool* p, int32_t page) {
  if (!p) return ROLLOUT_E_INVAL;
  int32_t r = p->retain(page);
  return r < 0 ? ROLLOUT_E_INVAL : r;
}
int rollout_pool_release(rollout_pool* p, int32_t page) {
  if (!p) return ROLLOUT_E_INVAL;
  int32_t r = p->release(page);
  return r < 0 ? ROLLOUT_E_INVAL : r;
}
int32_t rollout_pool_refcount(const rollout_pool* p, int32_t page) {
  if (!p || page < 0 || page >= p->total()) return ROLLOUT_E_INVAL;
  return p->refcount[page];
}
int64_t rollout_plan_pages(int32_t prompt_len, int32_t page_tokens, int32_t n_samples, const int32_t* max_new_tokens,
                           int32_t* shared, int32_t* tail, int32_t* private_pages) {
  if (prompt_len < 1 || page_tokens < 1 || n_samples < 0 || (n_samples > 0 && !max_new_tokens)) return ROLLOUT_E_INVAL;
  return plan_pages(prompt_len, page_tokens, n_samples, max_new_tokens, shared, tail, private_pages);
}

}  // extern "C"
