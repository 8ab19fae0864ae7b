// Host-callable launchers of every device kernel in the library.  All launches are
// asynchronous on the given stream; pointers are device memory unless noted.
#pragma once
#include "common.h"

// ---- plain one-op-per-kernel path (any storage type; used for fp32 models and as the
// ---- cross-check path for bf16) -------------------------------------------------------
template <typename T>
void launch_embed(const T* table, const int* tokens, float* x, int rows, int hidden, hipStream_t s);

// out[r] = x[r] * gain * rsqrt(mean(x[r]^2) + eps); rows_index (optional) selects source rows
void launch_rmsnorm_f32(const float* x, const float* gain, float* out, const int* rows_index, int rows,
                        int hidden, float eps, hipStream_t s);

// out[m][n] = sum_k a[m][k] w[n][k] (+ residual[m][n]); a fp32 [M][K], w T [N][K]
template <typename T>
void launch_linear_simple(const float* a, int lda, const T* w, float* out, int ldo, const float* residual,
                          int ldr, int M, int N, int K, hipStream_t s);

// rotary embedding of q (in place) and k, then k and v of every row go to the row's page
// plain path: bias and per-head RMSNorm of the fused [q | k | v] rows, in place (NULL parts are skipped)
void launch_qkv_bias_norm(float* qkv, const float* bias, const float* q_gain, const float* k_gain, float eps,
                          int rows, int n_q_heads, int n_kv_heads, int dh, hipStream_t s);
template <typename KT>
void launch_rope_kvwrite(float* qkv, const float* cos_sin, const int* row_pos, const int* row_slot,
                         const int* page_table, int max_pages, KT* kv_pool, KvGeom geom, int layer, int rows,
                         int n_q_heads, hipStream_t s);

// causal grouped-query attention of each row over cached positions 0..pos of its slot
template <typename KT>
void launch_attention_simple(const float* qkv, float* out, const int* row_pos, const int* row_slot,
                             const int* page_table, int max_pages, const KT* kv_pool, KvGeom geom, int layer,
                             int rows, int n_q_heads, hipStream_t s);

// act[r][f] = silu(gate_up[r][f]) * gate_up[r][F + f]
void launch_swiglu_f32(const float* gate_up, float* act, int rows, int ffn, hipStream_t s);

// top-k routing: idx/wt [rows][top_k]; ties to the lower expert index; wt = softmax of the selected logits
void launch_moe_route(const float* router_logits, int* idx, float* wt, int rows, int n_experts, int top_k,
                      hipStream_t s);
// act[(r,j)][f] = silu(Wg_e h_r)[f] * (Wu_e h_r)[f], e = idx[r][j]; w_gate_up is [E][2*Fe][hidden]
template <typename T>
void launch_moe_gate_up_simple(const float* h, const T* w_gate_up, const int* idx, float* act, int rows,
                               int top_k, int hidden, int expert_ffn, hipStream_t s);
// x[r][n] += sum_j wt[r][j] * (Wd_e act_(r,j))[n]; w_down is [E][hidden][Fe]
template <typename T>
void launch_moe_down_simple(const float* act, const T* w_down, const int* idx, const float* wt, float* x,
                            int rows, int top_k, int hidden, int expert_ffn, hipStream_t s);

// copies whole pages (all layers, all heads, K and V): pairs = (src_page, dst_page) x n
void launch_copy_pages(void* kv_pool, const int* pairs, int n_pairs, int n_layers, long long layer_stride_bytes,
                       long long page_stride_bytes, hipStream_t s);

// page_table[slot * max_pages + index] = page for n (slot, index, page) triples: the entries that
// changed on the host since the table was uploaded
void launch_patch_page_table(int* page_table, int max_pages, const int* triples, int n, hipStream_t s);

void launch_convert_to_f32(const void* src, int dtype, float* dst, long long n, hipStream_t s);

// ---- sampling ---------------------------------------------------------------------------
struct SampleRows {
  const float* logits;      // [*][vocab]
  const int* logits_row;    // [rows] row of `logits` each draw reads, or NULL (identity)
  const float* inv_temp;    // [rows]
  const float* top_p;       // [rows]
  const unsigned* uniforms; // [rows] or NULL -> Philox(seed, sample_id, step)
  const long long* sample_id;  // [rows] (Philox only)
  const int* step;             // [rows] (Philox only)
  const int* forced;        // [rows] or NULL; entries outside [0, vocab) mean "draw"
  unsigned long long seed;
  int* tokens;              // out [rows]
  float* logprobs;          // out [rows]
  unsigned long long* weight_sums;  // out [rows] or NULL
  // Scratch that lets a row's two sweeps over the vocabulary run on several workgroups (the
  // sums are integers, so the split changes nothing): both or neither.
  float* part_max = nullptr;               // [rows][kSampleParts]
  unsigned long long* seg_sums = nullptr;  // [rows][kSampleSegments]
};
constexpr int kSampleParts = 64, kSampleSegments = 1024;
void launch_sample(const SampleRows& r, int rows, int vocab, hipStream_t s);
void launch_philox_words(unsigned long long seed, const long long* ids, const unsigned* steps, unsigned* out,
                         int n, hipStream_t s);
// out[r] = log softmax(logits[r] * inv_temp)[target[r]]; target < 0 writes 0
void launch_logprob_gather(const float* logits, const int* target, float inv_temp, float* out, int rows,
                           int vocab, hipStream_t s);

// ---- per-slot decode state -------------------------------------------------------------
struct SlotState {
  int* last_token;       // [slots]
  int* pos;              // [slots] cached positions so far = position of the next fed token
  int* step;             // [slots] response position of the next token to emit
  long long* sample_id;  // [slots]
  float* inv_temp;       // [slots]
  float* top_p;          // [slots]
};
// row r <- slot live[r]: token, position, slot, sampling parameters
void launch_gather_decode_rows(SlotState st, const int* live, int rows, int* row_token, int* row_pos,
                               int* row_slot, float* row_inv_temp, float* row_top_p, long long* row_sample_id,
                               int* row_step, hipStream_t s);
// after a draw: slot's last token, position (+1 when advance_pos) and step (+1); the rows' tokens and
// log-probs are also stored to host_tokens / host_logprobs (pinned host memory, mapped for the device)
void launch_scatter_tokens(SlotState st, const int* row_slot, const int* tokens, const float* logprobs, int rows,
                           int advance_pos, int* host_tokens, float* host_logprobs, hipStream_t s);
