// Rollout engine: library-owned weights, paged KV pool, per-slot decode state, the
// sample table and the forward pass over a batch of rows.  One context = one GPU.
#pragma once
#include <deque>
#include <map>
#include <unordered_map>
#include <string>
#include <vector>

#include "../../include/rollout.h"
#include "common.h"
#include "host_sched.h"
#include "kernels.h"
#include "kernels_fast.h"

template <typename T>
struct DevBuf {
  T* p = nullptr;
  size_t n = 0;
  void alloc(size_t count) {
    release();
    n = count;
    if (count) HIP_TRY(hipMalloc((void**)&p, count * sizeof(T)));
  }
  void release() {
    if (p) (void)hipFree(p);
    p = nullptr;
    n = 0;
  }
  ~DevBuf() { release(); }
  DevBuf() = default;
  DevBuf(const DevBuf&) = delete;
  DevBuf& operator=(const DevBuf&) = delete;
  DevBuf(DevBuf&& o) noexcept : p(o.p), n(o.n) {
    o.p = nullptr;
    o.n = 0;
  }
};

template <typename T>
struct PinnedBuf {
  T* p = nullptr;
  size_t n = 0;
  void alloc(size_t count) {
    release();
    n = count;
    if (count) HIP_TRY(hipHostMalloc((void**)&p, count * sizeof(T), hipHostMallocDefault));
  }
  void release() {
    if (p) (void)hipHostFree(p);
    p = nullptr;
    n = 0;
  }
  ~PinnedBuf() { release(); }
  PinnedBuf() = default;
  PinnedBuf(const PinnedBuf&) = delete;
  PinnedBuf& operator=(const PinnedBuf&) = delete;
};

struct LayerWeights {
  DevBuf<float> norm1, norm2;
  DevBuf<float> qkv_bias;        // [q | k | v] biases (ROLLOUT_MODEL_QKV_BIAS)
  DevBuf<float> q_gain, k_gain;  // [head_dim] gains of the per-head q / k RMSNorm (ROLLOUT_MODEL_QK_NORM)
  DevBuf<char> wqkv;       // [(Hq + 2 Hkv) dh][hidden]
  DevBuf<char> wo;         // [hidden][Hq dh]
  DevBuf<char> w_gate_up;  // dense [2F][hidden] (gate rows, then up rows); MoE [E][2Fe][hidden]
  DevBuf<char> w_down;     // dense [hidden][F]; MoE [E][hidden][Fe]
  DevBuf<char> router;     // MoE [E][hidden]
  // matrix-core path: fragment-ordered copies (kernels_gemm.hip)
  DevBuf<char> wqkv_p, wo_p, w_gate_up_p, w_down_p;  // gate/up: n-tiles alternate gate, up
  DevBuf<char> router_p;   // MoE: w_gate_up_p, w_down_p hold the experts one after another
};

// Packed sequences of a prefill / log-prob forward (device arrays); NULL = one row per sample.
struct SeqBatch {
  const int *row0, *len, *slot;
  int n_seqs, max_len;
  const int* pos0 = nullptr;  // first position of each sequence (NULL = 0)
  int decode_rows = 0;        // rows [0, decode_rows) before the sequences: one decode row per live sample
};

// HIP-event brackets around kernel launches on sampled calls (ROLLOUT_RT_KERNEL_TIMING),
// accumulated per kernel name.
struct KernelTimer {
  bool enabled = false, active = false;
  unsigned stride = 1, calls = 0;
  struct Rec {
    const char* name;
    double bytes, flops;
    hipEvent_t a, b;
  };
  struct Acc {
    uint64_t launches = 0;
    double ms = 0, bytes = 0, flops = 0;
  };
  std::vector<hipEvent_t> pool;
  size_t used = 0;
  std::vector<Rec> pending;
  std::map<std::string, Acc> acc;

  void start_call() { active = enabled && (calls++ % (stride ? stride : 1)) == 0; }
  // A bracket with nothing inside, recorded under the name "(empty bracket)" in mid-stream of a
  // timed call: what two event records cost by themselves, for the reader of the figures
  // to subtract.
  void empty_bracket(hipStream_t s) {
    begin("(empty bracket)", 0, 0, s);
    end(s);
  }
  hipEvent_t get() {
    if (used == pool.size()) {
      hipEvent_t e;
      HIP_TRY(hipEventCreate(&e));
      pool.push_back(e);
    }
    return pool[used++];
  }
  void begin(const char* name, double bytes, double flops, hipStream_t s) {
    if (!active) return;
    Rec r{name, bytes, flops, get(), get()};
    HIP_TRY(hipEventRecord(r.a, s));
    pending.push_back(r);
  }
  void end(hipStream_t s) {
    if (active) HIP_TRY(hipEventRecord(pending.back().b, s));
  }
  void collect() {  // after the stream has been synchronised
    for (Rec& r : pending) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
        Acc& a = acc[r.name];
        a.launches += 1;
        a.ms += ms;
        a.bytes += r.bytes;
        a.flops += r.flops;
      }
    }
    pending.clear();
    used = 0;
    active = false;
  }
  ~KernelTimer() {
    for (hipEvent_t e : pool) (void)hipEventDestroy(e);
  }
};

// The host-side scheduler state (sample table, slots, page tables, prompt queue) is HostState.
struct rollout_ctx : HostState {
  rollout_model_desc md{};
  rollout_runtime_desc rd{};
  hipStream_t stream = nullptr;
  int device = 0;
  bool simple = true;
  std::string err;

  // derived sizes
  int q_dim = 0, kv_dim = 0, qkv_dim = 0, elem = 4;
  int n_slots = 0, temp_slot0 = 0, r_max = 0, logit_rows = 0;
  static constexpr int kTempSlots = 1024;
  static constexpr int kPendingRows = 64;  // page-table rows behind the temporary ones: prompts whose prefill is under way

  // weights
  DevBuf<char> embed, lm_head, lm_head_p;
  DevBuf<float> final_norm;
  std::vector<LayerWeights> layers;
  DevBuf<float> cos_sin;

  // KV cache
  DevBuf<char> kv_pool;
  KvGeom geom{};
  DevBuf<int> d_page_table;
  DevBuf<int> d_page_patch;     // growing pages: (slot, index, page) triples of a step's new pages

  // per-slot decode state
  DevBuf<int> st_last_token, st_pos, st_step;
  DevBuf<long long> st_sample_id;
  DevBuf<float> st_inv_temp, st_top_p;
  SlotState st{};

  bool broken = false;          // a step timed out: the device state is unknown, every call is refused
  double step_timeout_s = 300;  // wall-clock bound of the wait that ends a decode step
  DevBuf<int> d_live;

  // workspaces
  DevBuf<float> x, h, qkv, attn, gate_up, act, hn, logits, router_logits, moe_wt;
  DevBuf<int> moe_idx, route_log;  // route_log [n_layers][r_max][top_k] when recording
  // matrix-core MoE block: expert-sorted slots and the row blocks of the grouped projections
  DevBuf<int> moe_pos, moe_count, moe_row_map, moe_slot_of, moe_group_of_block, moe_block_begin, moe_block_end;
  DevBuf<float> moe_y;             // [r_max * top_k][hidden] expert results per slot
  int moe_max_blocks = 0;
  int last_route_rows = 0;
  // matrix-core path workspaces
  DevBuf<uint16_t> h_bf16, q_bf16, attn_bf16, act_bf16, hn_bf16;
  DevBuf<float> partial, attn_part_o, attn_part_ml;
  DevBuf<float> lse_max, lse_sum, lse_tgt;  // log-sum-exp parts of the teacher-forced pass, [parts][r_max]
  long long partial_rows = 0;   // capacity of `partial` in rows of partial_ld floats
  int partial_ld = 0;
  int attn_max_parts = 0;       // capacity of attn_part_* in (row, kv head, split) triples
  int decode_max_ctx = 0;       // longest context among the rows of the current decode step
  // decode attention with shared prompts: groups of up to 8 live samples of one prompt
  DevBuf<int> grp_rows, grp_len, grp_slot, row_t0;
  std::vector<int> h_row_t0;    // per live row (ascending id): start of its own range, 0 = not grouped
  int n_groups = 0, max_shared = 0;
  long long shared_saved = 0;   // positions that grouping reads once instead of once per member
  long long shared_dup = 0;     // positions cached once but attended by several live samples, counted per extra sample
  bool use_groups = false;      // this decode step attends shared prompts by group
  int decode_max_own = 0;       // longest own range (context - row_t0) among the rows
  double kv_unique_tokens_this_call = 0;  // cached positions counted once per group where pages are shared
  double kv_tokens_this_call = 0;   // cached positions attended by the current forward (for timing records)
  double attn_flops_this_call = 0;
  DevBuf<int> seq_row0, seq_len, seq_slot, seq_pos0;
  // a decode step that carries a chunk of prompt rows (chunked prefill)
  DevBuf<int> chunk_ints;        // [3 r_max]: rows whose logits are wanted, then (source, destination) page pairs
  double chunk_kv_tokens = 0, chunk_attn_flops = 0;  // the chunk's share of the attention, for the timing records
  DevBuf<float> ssq;            // [partials][256] partial sums of squares of the residual rows (decode path)
  int ssq_partials = 0;
  bool h_is_final = false;      // the last forward left x * final gain in h_bf16 (decode path)
  DevBuf<int> row_token, row_pos, row_slot, row_step, row_aux, row_forced, out_tokens;
  DevBuf<long long> row_sample_id;
  DevBuf<float> row_inv_temp, row_top_p, out_logprobs;
  DevBuf<unsigned> row_uniform;
  DevBuf<float> samp_part_max;               // sampler scratch, see SampleRows
  DevBuf<unsigned long long> samp_seg_sums;
  int samp_rows = 0;                         // rows the sampler scratch holds
  PinnedBuf<int> h_int;      // staging, 8 * r_max ints
  PinnedBuf<float> h_float;  // staging, 4 * r_max floats
  PinnedBuf<long long> h_ll; // staging, r_max
  int last_logit_rows = 0;

  rollout_stats stats{};
  KernelTimer timer;
  hipEvent_t step_done = nullptr;

  ~rollout_ctx() {
    delete pool;
    if (step_done) (void)hipEventDestroy(step_done);
  }
};

// engine.hip
void engine_init(rollout_ctx& c, const rollout_weights& w);
// uses c.row_token / row_pos / row_slot; result in c.x.  seqs describes packed sequences
// (prefill, log-probs) or is NULL when every row is one sample's next position (decode).
void engine_forward_rows(rollout_ctx& c, int rows, const SeqBatch* seqs);
// logits of `n` rows of c.x selected by rows_index (device, or NULL for rows first..first+n) into out
void engine_logits(rollout_ctx& c, const int* rows_index, int first, int n, float* out);
// out[r] = log-softmax(logits of row r of c.x * inv_t)[target[r]] for rows 0..n-1 (0 where
// target[r] < 0); target and out are device arrays
void engine_target_logprobs(rollout_ctx& c, int n, const int* target, float inv_t, float* out);
void engine_upload_page_table(rollout_ctx& c);
// one tensor (ROLLOUT_W_*, device pointer, caller's layout) into the library's layout, on c.stream
void engine_load_tensor(rollout_ctx& c, int layer, int which, const void* src);
// throws E_INVAL unless this model has tensor `which` (ROLLOUT_W_*) at `layer`
void engine_check_tensor(const rollout_ctx& c, int layer, int which);
