/*
 * rollout.h - C ABI of the MI355X rollout-generation library (librollout.so).
 *
 * The library runs the generation stage of an RL-for-LLM iteration on one GPU: for a
 * batch of prompts it computes the key-value cache (prefill phase), then generates n
 * sampled responses per prompt token by token (decoding phase) until each sample meets
 * its termination criterion, and it evaluates the inference stage's single forward pass
 * that yields per-token log-probs of given sequences (paper section 2.1, "Optimization
 * Workflow").  Requests live and die sample by sample: prompts can be added while others
 * decode and any sample can be aborted (paper section 4.1, "Rollout Scheduler"; section
 * 4.3, "Sample-level Rollout Lifecycle Control").
 *
 * Conventions
 *   - Every function returns ROLLOUT_OK (0) or a negative ROLLOUT_E_* code unless stated
 *     otherwise; rollout_last_error() gives the text.  A failing call changes no state.
 *     No C++ exception crosses this boundary.
 *   - "host" pointers are ordinary CPU memory owned by the caller; "device" pointers are
 *     HIP device memory on the current device.  Output buffers are caller-allocated and
 *     valid when the call returns (the library synchronises its stream once per call).
 *   - A context is bound to the device that was current in rollout_init and is not
 *     thread-safe; calls on one context must not overlap.
 *   - Sample ids are handed out consecutively, in call order: a call that adds P prompts with
 *     n samples each takes the next P * n ids, sample j of its prompt p getting first + p * n + j
 *     (so with one n throughout, id = prompt counter * n + j; calls may use different n).  A
 *     sample's tokens depend only on the weights, its prompt, the seed and its id, never on what
 *     else is in flight.
 *   - Response position t = 0 is emitted by rollout_prefill, position t >= 1 by the t-th
 *     rollout_decode_step after it.  A sample finishes when it emits eos_id (the token is
 *     reported) or its max_new_tokens-th token.
 */
#ifndef ROLLOUT_H
#define ROLLOUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ROLLOUT_ABI_VERSION 3

#define ROLLOUT_OK 0
#define ROLLOUT_E_INVAL (-1) /* bad argument or unsupported shape */
#define ROLLOUT_E_NOMEM (-2) /* KV pool, live-sample table or workspace too small; nothing admitted */
#define ROLLOUT_E_HIP (-3)   /* a HIP call failed, no usable GPU, or a decode step's kernels did not finish in time */
#define ROLLOUT_E_STATE (-4) /* call not valid in the context's current state (also: every call after a time-out) */

#define ROLLOUT_DTYPE_F32 0
#define ROLLOUT_DTYPE_BF16 1

/* runtime flags */
#define ROLLOUT_RT_SIMPLE_KERNELS 1u /* run every operator with the plain one-op-per-kernel path */
#define ROLLOUT_RT_RECORD_ROUTING 2u /* MoE: keep each forward's expert choices for rollout_debug_routing */
#define ROLLOUT_RT_KERNEL_TIMING 4u  /* bracket kernels with HIP events on sampled calls, see rollout_kernel_stats */
#define ROLLOUT_RT_PROMPT_GROUPS 8u   /* decode steps with more than 32 live samples: up to 4 samples of a prompt attend to its
                                         shared pages together, each key and value fragment read once for all of them (fewer
                                         bytes, one more launch; off by default: slower at the sizes measured so far) */

#define ROLLOUT_RT_GROW_PAGES 16u     /* KV pages are taken as contexts grow instead of all at admission: a sample is admitted
                                         with the pages of its prompt plus the one its first fed token goes to, and every
                                         decode step takes the pages it is about to write.  For workloads that end by EOS
                                         long before max_new_tokens, where reserving the worst case would leave most of the
                                         pool idle.  The pool can then run out: rollout_decode_step returns E_NOMEM (nothing
                                         changed; abort samples and call again), rollout_queue_step makes room itself, see there */

typedef struct rollout_ctx rollout_ctx; /* opaque; created by rollout_init, freed by rollout_destroy */

/* model flags: what tells the named model families apart in their public definitions (the
 * paper trains Qwen2.5 dense and Qwen3 mixture-of-experts models, section 5.1) */
#define ROLLOUT_MODEL_QKV_BIAS 1u     /* the q, k and v projections add a bias (Qwen2.5) */
#define ROLLOUT_MODEL_QK_NORM 2u      /* RMSNorm over head_dim on every q and k head before the rotary
                                         embedding, gains q_norm / k_norm, eps = rms_eps (Qwen3) */
#define ROLLOUT_MODEL_TIED_LM_HEAD 4u /* logits = h . embed^T; weights.lm_head is ignored */

/* Decoder-only transformer shape.  Operators: RMSNorm, projections without bias (but see the
 * flags), half-split rotary embedding, grouped-query causal attention, SwiGLU feed-forward or
 * (n_experts > 0) a mixture of SwiGLU experts with top_k softmax routing, lm_head.
 * flags: ROLLOUT_MODEL_*. */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
  int32_t n_experts, top_k, expert_ffn_dim; /* 0, 0, 0 = dense */
  float rms_eps, rope_theta;
  int32_t dtype; /* ROLLOUT_DTYPE_*: storage type of the weights.  The KV cache is fp32 for F32
                    models and 16-bit IEEE half for BF16 models (same bytes per token as bf16,
                    three more mantissa bits); activations are fp32 or bf16 hi+lo pairs. */
  uint32_t flags;
} rollout_model_desc;

/* One layer's tensors: DEVICE pointers, model dtype, row-major [out_features][in_features]
 * (y = W x).  Dense: w_gate, w_up [ffn][hidden], w_down [hidden][ffn], router NULL.
 * MoE: router [n_experts][hidden]; w_gate, w_up [n_experts][expert_ffn][hidden];
 * w_down [n_experts][hidden][expert_ffn]. */
typedef struct {
  const void *norm1, *wq, *wk, *wv, *wo, *norm2;
  const void *w_gate, *w_up, *w_down;
  const void *router;
  const void *bq, *bk, *bv;     /* ROLLOUT_MODEL_QKV_BIAS: [Hq dh], [Hkv dh], [Hkv dh]; else ignored */
  const void *q_norm, *k_norm;  /* ROLLOUT_MODEL_QK_NORM: [head_dim] gains; else ignored */
} rollout_layer_weights;

/* embed [vocab][hidden], final_norm [hidden], lm_head [vocab][hidden]: DEVICE pointers.
 * layers: HOST array of n_layers entries.  rollout_init copies every tensor into the
 * library's own layout; the caller may free its copies as soon as rollout_init returns. */
typedef struct {
  const void *embed, *final_norm, *lm_head;
  const rollout_layer_weights *layers;
} rollout_weights;

typedef struct {
  size_t kv_pool_bytes;     /* device bytes for KV pages; the library allocates them */
  int32_t page_tokens;      /* tokens per page: a multiple of 32 */
  int32_t max_live_samples; /* capacity of the live-sample table */
  int32_t max_context;      /* longest prompt + response per sample, in tokens */
  int32_t max_batch_tokens; /* rows per prefill / log-prob chunk (workspace); >= longest sequence */
  void *hip_stream;         /* hipStream_t the library launches on; NULL = the null stream */
  uint64_t seed;            /* key of the Philox4x32-10 stream that drives sampling */
  uint32_t flags;           /* ROLLOUT_RT_* */
  uint32_t timing_stride;   /* with ROLLOUT_RT_KERNEL_TIMING: time every timing_stride-th call (0 or 1 = all) */
} rollout_runtime_desc;

typedef struct {
  uint64_t decode_steps, tokens_emitted, prompts_prefilled, prompt_tokens, samples_admitted,
      samples_finished, samples_aborted;
  int32_t live_samples, pages_total, pages_in_use, pages_reserved, pages_peak;
  int32_t matrix_core_path; /* 1 when the bf16 matrix-core kernels run, 0 for the plain path */
  /* host wall clock spent inside the calls of each phase, the wait for the device included (ms):
   * rollout_prefill (and the whole-prompt prefills of the queue), decode steps (chunked queue steps
   * as a whole), rollout_extend, rollout_logprobs */
  double prefill_ms, decode_ms, extend_ms, logprobs_ms;
} rollout_stats;

/* Accumulated HIP-event timings of one kernel on the context's stream (sampled calls only):
 * name = the kernel as a profiler shows it; bytes / flops = the algorithmic traffic and
 * arithmetic of the timed launches (operands read once, results written once). */
typedef struct {
  char name[64];
  uint64_t launches;
  double ms, bytes, flops;
} rollout_kernel_stat;

/* Creates a context on the current device: copies the weights, allocates the KV pool and
 * workspaces.  Paper section 2.1: the actor model that generates responses.
 * Errors: E_INVAL (bad shape / descriptor), E_HIP (no device, allocation failed). */
int rollout_init(rollout_ctx **out, const rollout_model_desc *model, const rollout_weights *weights,
                 const rollout_runtime_desc *runtime);

/* Prefill phase + first token ("add request", paper sections 2.1 and 4.3).  Admits
 * n_prompts prompts with n_samples samples each, all or none: computes each prompt's KV
 * cache once into pages shared by its samples, then draws response position 0 for every
 * sample from the prompt's last-position logits.  May be called while other samples are
 * live.
 *   tokens            host int32, the prompts concatenated; offsets host int32 [n_prompts+1]
 *   max_new_tokens    host int32 [n_prompts*n_samples], each >= 1
 *   eos_id            token id that ends a sample, or -1
 *   temperature, top_p  sampling parameters stored per sample (temperature > 0)
 *   forced_first      NULL, or host int32 [n_prompts*n_samples]: tokens to emit instead of
 *                     drawn ones (teacher forcing); their log-probs are reported
 *   uniform_override  NULL, or host uint32 [n_prompts*n_samples]: words to use instead of
 *                     the Philox stream for this draw
 * Outputs (host, [n_prompts*n_samples], any may be NULL): sample_ids, first_tokens,
 * first_logprobs, finished (1 when the sample already ended).
 * Errors: E_INVAL; E_NOMEM when pages (worst case reserved up front: every sample's
 * max_new_tokens), live slots or max_batch_tokens do not suffice - nothing is admitted. */
int rollout_prefill(rollout_ctx *ctx, int32_t n_prompts, const int32_t *tokens, const int32_t *offsets,
                    int32_t n_samples, const int32_t *max_new_tokens, int32_t eos_id, float temperature,
                    float top_p, const int32_t *forced_first, const uint32_t *uniform_override,
                    int64_t *sample_ids, int32_t *first_tokens, float *first_logprobs, uint8_t *finished);

/* Number of live samples; when ids != NULL writes up to capacity ids in ascending order,
 * the order every per-sample array of rollout_decode_step uses.  Returns the count. */
int rollout_live_samples(rollout_ctx *ctx, int32_t capacity, int64_t *ids);

/* One decoding-phase step (paper section 2.1): feeds every live sample's last token,
 * extends its KV cache by one position and emits its next token and that token's log-prob
 * (log-softmax of the temperature-scaled logits over the full vocabulary).  Finished
 * samples leave the live set and their pages return to the pool.
 *   forced_tokens     NULL, or host int32 [live]: tokens to emit instead of drawn ones
 *   uniform_override  NULL, or host uint32 [live]
 *   n_live            in: capacity of the output arrays; out: samples stepped
 * Outputs (host, ascending sample id, any may be NULL): sample_ids, tokens, logprobs,
 * finished.  Errors: E_INVAL (capacity too small); E_HIP when the step's kernels do not finish
 * within five minutes of wall clock (the context then refuses every further call with E_STATE:
 * destroy it).  With no live sample: *n_live = 0, OK. */
int rollout_decode_step(rollout_ctx *ctx, const int32_t *forced_tokens, const uint32_t *uniform_override,
                        int32_t *n_live, int64_t *sample_ids, int32_t *tokens, float *logprobs,
                        uint8_t *finished);

/* Inference-stage forward (paper section 2.1: one forward pass over generated sequences,
 * prefill only): log p(token_t | tokens_<t) at `temperature` for packed sequences, with the
 * same kernels as prefill.  tokens host int32 [cu_seqlens[n_seqs]]; cu_seqlens host int32
 * [n_seqs+1]; logprobs host float [total], 0 at each sequence's first token.  Uses free KV
 * pages as scratch.  Errors: E_INVAL; E_NOMEM if one sequence exceeds max_batch_tokens,
 * max_context or the free pages. */
int rollout_logprobs(rollout_ctx *ctx, int32_t n_seqs, const int32_t *tokens, const int32_t *cu_seqlens,
                     float temperature, float *logprobs);

/* Multi-turn continuation (the agentic pipeline's generate - environment - generate loop,
 * paper section 2.1 "generation" with environment interaction and section 5.2): appends
 * tokens the model did not generate - an environment's observation, a tool result - to the
 * contexts of live samples and emits each sample's next response token.  For sample i the
 * tokens tokens[offsets[i] .. offsets[i+1]) follow its last emitted token; the next token is
 * drawn (or forced) from the distribution after the last appended token and counts towards
 * max_new_tokens; appended tokens do not.  The appended tokens run through the model as one
 * packed sequence per sample that attends to the sample's cache, so the cost is one forward
 * pass whatever their number.
 *   sample_ids   host int64 [n], live and distinct; outputs follow this order
 *   tokens       host int32, the appended tokens concatenated; offsets host int32 [n+1], each
 *                sample gets at least one
 *   forced_next, uniform_override   NULL or host [n], as in rollout_decode_step
 * Outputs (host [n], any may be NULL): next_tokens, next_logprobs, finished.
 * rollout_debug_logits then returns the n logits rows the tokens were drawn from.
 * All or nothing.  Errors: E_INVAL (a sample is not live or listed twice, nothing to append,
 * token out of range); E_NOMEM (context + remaining response beyond max_context, all rows
 * beyond max_batch_tokens, not enough free pages for the longer contexts). */
int rollout_extend(rollout_ctx *ctx, int32_t n, const int64_t *sample_ids, const int32_t *tokens,
                   const int32_t *offsets, const int32_t *forced_next, const uint32_t *uniform_override,
                   int32_t *next_tokens, float *next_logprobs, uint8_t *finished);

/* "Abort request" (paper section 4.3): drops the listed live samples and frees their
 * pages.  Ids that are not live are ignored.  Returns the number aborted.  For the queue-fed
 * rollout an aborted sample counts as ended: its prompt is complete once its other samples
 * have ended too. */
int rollout_abort(rollout_ctx *ctx, int32_t n, const int64_t *sample_ids);

/* ---- Queue-fed continuous rollout ---------------------------------------------------------
 * The sample-level lifecycle of paper sections 4.1 and 4.3 driven by the library: prompts wait
 * in a host-side queue, are admitted ("add request") as live-sample slots and KV pages free
 * up while the other samples keep decoding, and once a target number of prompts has all its
 * samples finished the still-running samples are aborted ("abort request") and the waiting
 * prompts dropped - the mechanism that dynamic sampling uses to cut the long tail.  A sample's
 * tokens still depend only on (weights, prompt, seed, sample id): the queue decides when a
 * sample runs, never what it emits. */
typedef struct {
  uint64_t prompts_pushed, prompts_admitted, prompts_completed; /* completed = every sample finished or aborted by the caller */
  uint64_t samples_aborted;                                     /* by the target policy */
  uint64_t prompts_preempted;                                   /* ROLLOUT_RT_GROW_PAGES: sent back to the queue to make room */
  int32_t prompts_waiting;
  int32_t closed;                                               /* 1 once the target was reached */
  int32_t prompts_pending;                                      /* chunked prefill: admitted, prompt not fully cached yet */
} rollout_queue_stats;

/* Appends n_prompts prompts (n_samples samples each) to the queue; host arrays as for
 * rollout_prefill, copied.  Nothing runs on the GPU.  first_sample_ids (host int64 [n_prompts],
 * may be NULL) receives the id of each prompt's sample 0; its sample j will carry that id + j.
 * Ids are taken here, in push order, from the same sequence rollout_prefill uses.
 * Errors (nothing is queued): E_INVAL (bad arguments; n_samples differs from earlier pushes;
 * queue closed); E_NOMEM when a prompt could never be admitted, even into an idle context
 * (longer than max_batch_tokens, prompt + response beyond max_context, more samples than
 * live-sample slots, more pages than the pool holds). */
int rollout_queue_push(rollout_ctx *ctx, int32_t n_prompts, const int32_t *tokens, const int32_t *offsets,
                       int32_t n_samples, const int32_t *max_new_tokens, int32_t eos_id, float temperature,
                       float top_p, int64_t *first_sample_ids);

/* admit_min_prompts >= 1: a step admits waiting prompts only when at least that many of them
 * (or all that wait) fit, or when no sample is live - fewer, larger prefill calls.
 * target_prompts: 0 = run everything; otherwise the queue closes when that many admitted
 * prompts are complete. */
int rollout_queue_policy(rollout_ctx *ctx, int32_t admit_min_prompts, int32_t target_prompts);

/* One scheduling step: (1) admits the longest run of waiting prompts, in push order, that
 * fits the free slots, the unreserved pages and one prefill call, subject to the policy -
 * their prefill runs and response position 0 of their samples is emitted; (2) one decode step
 * over every live sample, the newly admitted ones included; (3) when the target is reached,
 * aborts every live sample, drops the waiting prompts and closes the queue.
 *   n_out       in: capacity of the output arrays; out: entries written
 *   n_admitted  out: the first *n_admitted entries are position-0 tokens of newly admitted
 *               samples (ascending id); the rest is the decode step's output (ascending id)
 * Outputs as for rollout_decode_step.  With nothing waiting and nothing live, or after the
 * queue closed: *n_out = 0.  Errors: E_INVAL (capacity below live samples + 2 x samples that
 * would be admitted: nothing happens).
 * With ROLLOUT_RT_GROW_PAGES a step first makes sure the pool holds the pages it is about to
 * write: while it does not, the most recently admitted prompt that still runs gives way - its
 * live samples are dropped and the prompt returns to the head of the queue (a step that drops
 * samples admits nothing).  The prompt starts over when it is admitted again: all its samples
 * appear once more among the newly admitted entries, from response position 0, and - their ids
 * being the same - emit the same tokens as before; a caller that sees a known id there discards
 * what it had collected for it.  Prompts are admitted only while the pool keeps one spare page
 * per live sample.  E_NOMEM when the pool is exhausted by samples that did not come through the
 * queue (abort some). */
int rollout_queue_step(rollout_ctx *ctx, int32_t *n_out, int32_t *n_admitted, int64_t *sample_ids,
                       int32_t *tokens, float *logprobs, uint8_t *finished);

/* Chunked prefill for the queue-fed rollout (paper section 4.3: requests are added while the
 * other samples keep decoding).  chunk_rows = 0 (default): rollout_queue_step runs the whole
 * prefill of the prompts it admits before its decode step, as described above.  chunk_rows > 0:
 * a step is ONE forward pass that carries a decode row for every live sample and at most
 * chunk_rows rows of admitted prompts, in push order, a prompt being cut where the budget ends
 * and continued in the next step (its rows attend to what earlier steps cached).  A prompt
 * takes its pages and its samples' slots and pages when it is admitted; its samples emit
 * response position 0 in the step that caches its last rows - they are that step's first
 * *n_admitted entries - and decode from the next step on, so a sample appears at most once per
 * step and the capacity needed is live samples + samples of the prompts that end.  A step can
 * return *n_out = 0 while prompts are still being cached: the queue is drained when
 * rollout_queue_get_stats shows nothing waiting and nothing pending and no sample is live.
 * With ROLLOUT_RT_GROW_PAGES the prompts that are only partly cached give way first when the pool
 * runs out (they return to the head of the queue and count as preempted).  A sample's tokens do
 * not depend on the setting beyond rounding: the chunks change which rows share a matrix tile.
 * Matrix-core path only.  Errors: E_INVAL (chunk_rows < 0), E_STATE (plain path; a prompt is
 * partly cached right now). */
int rollout_queue_chunking(rollout_ctx *ctx, int32_t chunk_rows);

int rollout_queue_get_stats(rollout_ctx *ctx, rollout_queue_stats *out);

/* ---- Weight refresh ------------------------------------------------------------------------
 * The receiving half of the parameter synchronisation between the training and the generation
 * stage of an iteration (paper section 2.1: the updated actor generates the next iteration's
 * responses; section 4.3: the model update is sent to the inference workers in buckets).  Each
 * call takes one bucket: tensors as rollout_init takes them (DEVICE pointers, model dtype,
 * row-major [out_features][in_features]) and re-orders them into the library's layout in
 * place.  Returns when the copies are done, so the caller may reuse the bucket's memory.
 * The KV pool and every other allocation stay as they are.
 * Errors: E_INVAL (unknown tensor, layer out of range - model-level tensors take layer -1 -,
 * null pointer; nothing of the bucket is applied); E_STATE while samples are live or prompts
 * wait in the queue (their cached keys and values belong to the old weights). */
enum {
  ROLLOUT_W_EMBED = 0, ROLLOUT_W_FINAL_NORM = 1, ROLLOUT_W_LM_HEAD = 2,                   /* layer -1 */
  ROLLOUT_W_NORM1 = 3, ROLLOUT_W_WQ = 4, ROLLOUT_W_WK = 5, ROLLOUT_W_WV = 6, ROLLOUT_W_WO = 7,
  ROLLOUT_W_NORM2 = 8, ROLLOUT_W_GATE = 9, ROLLOUT_W_UP = 10, ROLLOUT_W_DOWN = 11, ROLLOUT_W_ROUTER = 12,
  ROLLOUT_W_BQ = 13, ROLLOUT_W_BK = 14, ROLLOUT_W_BV = 15, ROLLOUT_W_Q_NORM = 16, ROLLOUT_W_K_NORM = 17
};
typedef struct {
  int32_t layer;    /* 0 .. n_layers-1, or -1 for embed / final_norm / lm_head */
  int32_t tensor;   /* ROLLOUT_W_* */
  const void *data; /* DEVICE pointer, shape as in rollout_layer_weights / rollout_weights */
} rollout_tensor_update;
int rollout_update_weights(rollout_ctx *ctx, int32_t n, const rollout_tensor_update *updates);

/* ---- Policy-gradient objective ------------------------------------------------------------
 * What the training stage does with the log-probs (paper sections 5.1 and 5.2: PPO loss whose
 * advantage is the REINFORCE return instead of a GAE estimate, rewards clipped at 20 and
 * advantages at 10; section 2.1: the reference model contributes a KL penalty).  Token by token,
 * over the tokens with mask = 1 ("counted", t_1 < ... < t_L inside each sequence):
 *   rho_j = -kl_coef (logp_old - logp_ref) at t_j (0 without logp_ref); the sequence's reward,
 *           clipped to +-reward_clip, is added to rho_L
 *   G_L = rho_L, G_j = rho_j + gamma G_{j+1};  A_j = clip(G_j, +-adv_clip)
 *   r_j = exp(logp_new - logp_old);  s_j = min(r_j A_j, clip(r_j, 1 - eps_low, 1 + eps_high) A_j)
 *   loss = -(sum of s over all counted tokens) / N, N = their number (0 when N = 0)
 *   grad = d loss / d logp_new = -(r_j A_j) / N where the unclipped term is the minimum, else 0
 * Tokens that are not counted get advantage 0 and gradient 0.  The paper fixes neither the
 * discount nor the KL coefficient nor the ratio bounds: they are parameters.
 *   cu_seqlens  HOST int32 [n_seqs+1], packed sequences;  rewards HOST float [n_seqs]
 *   logp_new, logp_old, logp_ref (or NULL), mask (uint8)   DEVICE arrays [cu_seqlens[n_seqs]]
 *   grad DEVICE [total];  advantages DEVICE [total] or NULL;  loss HOST float
 * Runs on hip_stream (NULL = the null stream) and returns when the loss has arrived.  Sums are
 * taken in a fixed order: the result does not depend on scheduling.  Errors: E_INVAL, E_HIP. */
typedef struct {
  float gamma, kl_coef, reward_clip, adv_clip, eps_low, eps_high;
} rollout_loss_params;
int rollout_policy_loss(int32_t n_seqs, const int32_t *cu_seqlens, const float *logp_new, const float *logp_old,
                        const float *logp_ref, const uint8_t *mask, const float *rewards,
                        const rollout_loss_params *params, void *hip_stream, float *loss, float *grad,
                        float *advantages);

/* Parity hook: copies the fp32 logits rows of the last prefill (one per prompt, prompt
 * order) or decode step (one per stepped sample, ascending id) to host `out`
 * [rows][vocab].  rows: in capacity, out count.  Errors: E_INVAL, E_STATE (none yet). */
int rollout_debug_logits(rollout_ctx *ctx, int32_t *rows, float *out);

/* Parity hook (MoE models, ROLLOUT_RT_RECORD_ROUTING): the experts chosen for every row of
 * the last forward pass (the last prefill chunk's prompt tokens in packed order, or the last
 * decode step's samples in ascending id), host int32 `out` [n_layers][rows][top_k].
 * rows: in capacity, out count.  Errors: E_INVAL, E_STATE (not recording / nothing yet). */
int rollout_debug_routing(rollout_ctx *ctx, int32_t *rows, int32_t *out);

int rollout_get_stats(rollout_ctx *ctx, rollout_stats *out);
/* Per-kernel timings gathered under ROLLOUT_RT_KERNEL_TIMING.  n: in capacity of `out`, out
 * number of entries written (kernels with at least one timed launch).  The entry named
 * "(empty bracket)" is a pair of event records around nothing, taken once in every timed
 * decode step: the cost of the measurement itself, which every other entry's ms includes
 * once per launch. */
int rollout_kernel_stats(rollout_ctx *ctx, int32_t *n, rollout_kernel_stat *out);
const char *rollout_last_error(rollout_ctx *ctx); /* ctx may be NULL: error of the last failed rollout_init */
void rollout_destroy(rollout_ctx *ctx);
int rollout_abi_version(void);

/* Stand-alone sampling over given logits (the decode step's last stage): for each row,
 * temperature scaling, top-p nucleus on integer weights, inverse-CDF draw with the row's
 * 32-bit word, and the log-prob of the chosen token.
 *   logits DEVICE float [rows][vocab] (row stride = vocab); uniforms host uint32 [rows];
 *   forced NULL or host int32 [rows] (then tokens = forced, log-probs of those);
 *   tokens host int32 [rows]; logprobs host float [rows]; weight_sums NULL or host uint64
 *   [rows] (sum of the integer weights, for parity).  hip_stream as in the runtime desc.
 * Errors: E_INVAL, E_HIP. */
int rollout_sample(const float *logits, int32_t rows, int32_t vocab, float temperature, float top_p,
                   const uint32_t *uniforms, const int32_t *forced, void *hip_stream, int32_t *tokens,
                   float *logprobs, uint64_t *weight_sums);

/* rollout_sample for callers that cannot allocate device memory or wait: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and results as
 * rollout_sample, but every array is DEVICE memory - logits [rows][vocab], uniforms uint32 [rows],
 * forced int32 [rows] or NULL (ids outside [0, vocab) are drawn), tokens int32 [rows], logprobs
 * float [rows], weight_sums uint64 [rows] or NULL - and the call only enqueues kernels on
 * hip_stream: no allocation, no host-device copy, no synchronisation; outputs are valid once the
 * stream has reached that point.  The kernels' scratch (per-row parameters and the partial maxima
 * and segment sums of the two sweeps, about 8.3 KB per row) is a fixed device array inside the
 * library, one copy per GPU, kept until the process ends: rows <= ROLLOUT_SAMPLE_STATIC_MAX_ROWS,
 * else E_INVAL.  Every call on a GPU uses that one array, which keeps the last call's contents
 * (nothing in it has to start at zero: each call writes what it reads): calls that overlap on one
 * GPU - two streams, two threads - race; serialise them.  The array's address is looked up on
 * the first call on a device (rollout_init does it too); make that first call, or
 * rollout_sample_static_prepare(), outside graph capture.  Errors: E_INVAL, E_HIP;
 * rollout_sample_static_error() gives the calling thread's last error text. */
#define ROLLOUT_SAMPLE_STATIC_MAX_ROWS 256
int rollout_sample_static(const float *logits, int32_t rows, int32_t vocab, float temperature, float top_p,
                          const uint32_t *uniforms, const int32_t *forced, void *hip_stream, int32_t *tokens,
                          float *logprobs, uint64_t *weight_sums);
int rollout_sample_static_prepare(void); /* looks the array up for the current device; allocates nothing */
const char *rollout_sample_static_error(void);

/* Writes words[i] = Philox4x32-10 output word 0 for key (seed lo, seed hi) and counter
 * (sample_ids[i] lo, sample_ids[i] hi, steps[i], 0), computed on the device; all arrays
 * host, length n.  Parity hook for the generator. */
int rollout_philox_words(uint64_t seed, int32_t n, const int64_t *sample_ids, const uint32_t *steps,
                         uint32_t *words);

/* ---- paged KV allocator, host side (paper section 4.1: requests are added "based on
 * current resource availability").  Pure CPU bookkeeping, usable without a GPU. ---- */
typedef struct rollout_pool rollout_pool;
rollout_pool *rollout_pool_create(int32_t n_pages);
void rollout_pool_destroy(rollout_pool *p);
int32_t rollout_pool_free_pages(const rollout_pool *p);     /* pages on the free list */
int32_t rollout_pool_unreserved(const rollout_pool *p);     /* free pages not promised to anyone */
int rollout_pool_reserve(rollout_pool *p, int32_t n);       /* promise n pages; E_NOMEM if unavailable */
void rollout_pool_unreserve(rollout_pool *p, int32_t n);    /* give back unused promises */
int32_t rollout_pool_alloc(rollout_pool *p, int from_reservation); /* page id (refcount 1) or E_NOMEM */
int rollout_pool_retain(rollout_pool *p, int32_t page);     /* refcount + 1; returns new count or E_INVAL */
int rollout_pool_release(rollout_pool *p, int32_t page);    /* refcount - 1, frees at 0; new count or E_INVAL */
int32_t rollout_pool_refcount(const rollout_pool *p, int32_t page);

/* Pages one prompt and its samples need: *shared = full prompt pages (one copy, shared by
 * all samples), *tail = 1 when the prompt ends inside a page (staged once, copied per
 * sample), private_pages[j] = pages sample j will own when it runs to max_new_tokens[j]
 * (0 when it emits a single token).  Returns the peak total, shared + tail + sum private. */
int64_t rollout_plan_pages(int32_t prompt_len, int32_t page_tokens, int32_t n_samples,
                           const int32_t *max_new_tokens, int32_t *shared, int32_t *tail,
                           int32_t *private_pages);

#ifdef __cplusplus
}
#endif
#endif /* ROLLOUT_H */
