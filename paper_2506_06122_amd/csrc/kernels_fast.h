// Launchers of the matrix-core (bf16) path: packed-weight projections, fused row kernels
// and paged attention.  Pointers are device memory; launches are asynchronous.
#pragma once
#include <algorithm>

#include "common.h"

// Epilogues of the projection kernels:
//   EPI_F32          out[m][n] fp32 (split-K planes allowed)
//   EPI_SWIGLU_BF16  column tiles alternate gate, up: act[m][f] = silu(gate) * up as bf16 hi/lo
//   EPI_RESID        stream kernel only: x[m][n] += result (fp32, in place); h = x * gain as
//                    bf16 hi/lo planes (the next projection's operand, not yet normalised);
//                    ssq_out[workgroup column][m] = sum of x^2 over the workgroup's columns
// Any stream-kernel epilogue first scales row m by rsqrt(sum_p rinv_ssq[p][m] / K + eps) when
// rinv_ssq is given: the second half of the RMSNorm of the projection's input.
//   EPI_LSE          tile kernel only, the teacher-forced log-prob pass: the result z = out *
//                    lse_scale never reaches memory; per (workgroup column, row) the kernel
//                    stores max z and sum exp(z - max) over the workgroup's columns, and the
//                    workgroup that owns column lse_target[m] stores that z (launch_lse_finish
//                    turns these into log-probs)
enum { EPI_F32 = 0, EPI_SWIGLU_BF16 = 1, EPI_RESID = 2, EPI_LSE = 3 };

// Fragment order of an activation plane [rows][K] (decode steps with at most 32 rows): the
// 16-row x 32-deep operand fragment of the 16x16x32 matrix instruction is stored as one
// contiguous 1 KiB block [lane][8] with lane = (k % 32 / 8) * 16 + row % 16, fragments ordered
// [row / 16][k / 32].  A wavefront then reads an operand fragment as whole cache lines, as it
// reads a weight fragment.  Rows are padded to a multiple of 16 (the pad is never written and
// what is read from it only reaches output rows that are not stored).
__host__ __device__ inline long long frag_offset(int m, int k, int k_tiles) {
  return (((long long)(m >> 4) * k_tiles + (k >> 5)) << 9) + ((((k >> 3) & 3) * 16 + (m & 15)) << 3) + (k & 7);
}

// A read-only range that spare workgroups of a launch walk, one dword per 128-byte line, while
// the launch's own workgroups wait on memory latency: the projection that streams these weights
// next then finds them in the memory-side cache (256 MiB) instead of HBM.
struct TouchRange {
  const void* p = nullptr;
  long long lines = 0;  // 128-byte lines
  int wgs = 0;          // workgroups that share the walk (0 = none)
};
#ifdef __HIPCC__
// Workgroup `wg` of t.wgs reads one dword of every 128-byte line of its share of the range,
// up to 8 loads in flight per lane; the values go nowhere.
__device__ inline void touch_range(const TouchRange& t, int wg) {
  const long long stride = (long long)t.wgs * blockDim.x;
  const char* p = (const char*)t.p;
  unsigned acc = 0;
  long long i = (long long)wg * blockDim.x + threadIdx.x;
  for (; i + 7 * stride < t.lines; i += 8 * stride) {
    unsigned v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = *(const unsigned*)(p + (i + u * stride) * 128);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  for (; i < t.lines; i += stride) acc ^= *(const unsigned*)(p + i * 128);
  asm volatile("" ::"v"(acc));  // keeps the loads
}
#endif

struct GemmArgs {
  const void* a;     // bf16 [rows][K], row stride lda: hi parts of the activations
  const void* a_lo;  // same shape: lo parts (value = hi + lo)
  bool frag = false; // stream kernel: `a`, `h` and the EPI_SWIGLU_BF16 result are in fragment order
  const void* w;     // packed bf16 weight, N/16 x K/32 fragments of 1 KiB
  void* out;         // EPI_F32: float [splits][M][ldo]; EPI_SWIGLU_BF16: bf16 [M][ldo] (ldo = N/2)
  int M, N, K, lda, ldo;
  long long out_lo_offset = 0;  // EPI_SWIGLU_BF16: elements from the hi plane of `out` to its lo plane
  long long split_stride;  // floats between split planes (EPI_F32)
  int k_tiles_per_split;   // filled by the launcher
  int grid_nx = 0, grid_ny = 0, grid_nz = 0;  // tile kernels: column blocks, row blocks, K splits (launcher)
  // input normalisation (stream kernel)
  const float* rinv_ssq = nullptr;  // [rinv_partials][ssq_stride] partial sums of squares of the input rows
  int rinv_partials = 0;
  int ssq_stride = 0;
  float eps = 0.f;
  TouchRange touch;   // stream kernel: walked by the workgroups with blockIdx.x >= touch_x0
  int touch_x0 = 0;   // filled by the launcher
  // EPI_RESID
  float* x = nullptr;            // [M][N] residual stream, updated in place
  const float* gain = nullptr;   // [N] gain of the RMSNorm that follows
  uint16_t* h = nullptr;         // bf16 [M][N], hi plane
  long long h_lo_offset = 0;     // elements from the hi plane of h to its lo plane
  float* ssq_out = nullptr;      // [grid columns][ssq_stride]
  // grouped launch (mixture of experts, tile kernel): row block y works on rows
  // [block_row_begin[y], block_row_end[y]) of the expert-sorted order with the weights of
  // group_of_block[y]; row_map maps a sorted row to its source row in `a`.
  const int* group_of_block = nullptr;
  const int* block_row_begin = nullptr;
  const int* block_row_end = nullptr;
  const int* row_map = nullptr;
  long long group_stride16 = 0;  // 16-byte units between consecutive groups' packed weights
  int n_row_blocks = 0;
  // EPI_LSE
  const int* lse_target = nullptr;  // [M] target column of row m, or -1
  float lse_scale = 1.f;            // 1 / temperature
  float* lse_max = nullptr;         // [grid columns][lse_stride]
  float* lse_sum = nullptr;         // [grid columns][lse_stride]
  float* lse_tgt = nullptr;         // [M]
  int lse_stride = 0;
};

// How one projection is launched: kind 0 = gemm_stream_kernel (rows <= 256), 1 = gemm_tile_kernel.
struct GemmPlan {
  int kind, mt, nt, nw, splits, kc;
  const char* name;  // kernel name as a profiler shows it (without the argument list)
};
GemmPlan gemm_plan(int M, int N, int K, int epi, int max_splits);
GemmPlan gemm_plan_tiled(int M, int N, int K, int epi, int max_splits);  // the tile kernel for any M
// column parts per row that an EPI_LSE launch with this plan writes
inline int lse_parts(const GemmPlan& pl, int N) { return ceil_div(N >> 4, 4 * pl.nt); }
// out[m] = lse_tgt[m] - log sum_n exp(z[m][n]) from the parts of an EPI_LSE launch; 0 where target < 0
void launch_lse_finish(const float* lse_max, const float* lse_sum, const float* lse_tgt, const int* target,
                       int parts, int stride, int rows, float* out, hipStream_t s);
// returns the number of split planes written (EPI_F32; <= plan.splits)
int launch_gemm_bf16(GemmArgs a, int epi, const GemmPlan& plan, hipStream_t s);
void launch_pack_weight(const void* src, void* dst, int N, int K, int tile_offset, int tile_stride, hipStream_t s);

// x[r] (+= sum of `splits` partial planes) ; h[r] = bf16(x[r] * gain * rsqrt(mean(x[r]^2) + eps)).
//   tokens != NULL : x[r] is first loaded from the bf16 embedding row tokens[r]
//   rows_index != NULL : source row of x is rows_index[r], x is not written back (final norm)
struct RowNormArgs {
  float* x;
  const float* partial;     // [splits][rows][hidden] or NULL
  long long split_stride;
  int splits;
  const float* gain;
  uint16_t* h;              // bf16 [rows][hidden], hi plane
  long long h_lo_offset;    // elements from the hi plane to the lo plane
  float* ssq_out;           // when set: h = x * gain without the rsqrt factor, ssq_out[r] = sum x[r]^2
  bool h_frag = false;      // h in fragment order
  const int* tokens;
  const uint16_t* embed;
  const int* rows_index;
  int rows, hidden;
  float eps;
  // mixture of experts: x[r] += sum_j moe_wt[r][j] * moe_y[moe_slot[r][j]] (picks in order)
  const float* moe_y = nullptr;    // [slots][hidden]
  const int* moe_slot = nullptr;   // [rows][moe_k]
  const float* moe_wt = nullptr;   // [rows][moe_k]
  int moe_k = 0;
};
void launch_row_norm(const RowNormArgs& a, hipStream_t s);

// What some model families do to q, k, v between the projection and the rotary embedding
// (head_dim 128 here: one wavefront holds one head as 64 rotary pairs).
struct QkvExtras {
  const float* bias = nullptr;    // [q | k | v] added to the projection, or NULL
  const float* q_gain = nullptr;  // [128] gains of an RMSNorm over each q head, or NULL
  const float* k_gain = nullptr;  // [128] the same for each k head
  float eps = 0.f;
};
// x0, x1 = elements i and i + 64 of one head, all 64 lanes of the wavefront taking part:
// adds the bias (element offset `off` of the fused row) and normalises the head.
__device__ inline void qkv_extras(const QkvExtras& e, int off, int i, const float* gain, float& x0, float& x1) {
  if (e.bias) {
    x0 += e.bias[off + i];
    x1 += e.bias[off + i + 64];
  }
  if (gain) {
    const float rinv = 1.0f / sqrtf(wave_sum(x0 * x0 + x1 * x1) / 128.0f + e.eps);
    x0 *= rinv * gain[i];
    x1 *= rinv * gain[i + 64];
  }
}

// Sums the split planes of the fused QKV projection, applies the rotary embedding to q and
// k, writes q as bf16 [rows][q_dim] (and optionally as fp32 into q_f32 [rows][q_f32_ld]) and
// stores k, v into the row's KV page (bf16, the pool's element order).
struct QkvPostArgs {
  const float* partial;
  long long split_stride;
  int splits;
  const float* cos_sin;
  const int *row_pos, *row_slot, *page_table;
  int max_pages;
  uint16_t* q_bf16;         // hi plane [rows][q_dim]
  long long q_lo_offset;    // elements to the lo plane
  float* q_f32;
  int q_f32_ld;
  uint16_t* kv_pool;
  KvGeom geom;
  int layer, rows, n_q_heads;
  QkvExtras extra;
};
void launch_qkv_post(const QkvPostArgs& a, hipStream_t s);

void launch_f32_to_bf16(const float* src, uint16_t* dst, long long n, hipStream_t s);

constexpr int GROUP_MEMBERS = 4;  // samples of one prompt that attend to its shared pages together

// Paged grouped-query attention on the matrix cores (KV_MATRIX pool, head_dim 128).
struct AttnArgs {
  const uint16_t* q;        // prefill: half-precision hi plane [rows][n_q_heads][128], rotary applied
  long long q_lo_offset;    // elements to its lo plane
  uint16_t* out;            // bf16 hi plane [rows][n_q_heads][128]
  long long out_lo_offset;  // elements to its lo plane
  bool out_frag = false;    // decode: out in fragment order, K = n_q_heads * 128
  const uint16_t* kv_pool;
  KvGeom geom;
  const int* page_table;
  int max_pages, layer, n_q_heads;
  // decode: one row per sample
  const int *row_pos, *row_slot;
  int rows;
  int n_splits, split_tokens;      // KV range per workgroup (multiple of 128)
  float* part_o;                   // [rows][n_kv_heads][n_slots][16][128]
  float* part_ml;                  // [rows][n_kv_heads][n_slots][2][16]
  int n_slots = 0;                 // partial results per (row, KV head); the launcher sets n_splits when 0
  // decode with shared prompts (launch_attention_decode_grouped): the samples of one prompt
  // attend to the prompt's shared pages together - each key and value fragment is read once
  // for all of them - and every row attends alone only to what follows its row_t0.
  const int* row_t0 = nullptr;     // [rows] first position of the row's own range (0 = no shared part)
  int slot0 = 0;                   // partial slots [0, slot0) hold the shared part, [slot0, slot0 + n_splits) the own
  const int* grp_rows = nullptr;   // [n_groups][GROUP_MEMBERS] rows of a group's members, -1 = none
  const int* grp_len = nullptr;    // [n_groups] shared positions (a multiple of 32)
  const int* grp_slot = nullptr;   // [n_groups] page-table row of one member
  int n_groups = 0, n_splits_a = 0, split_tokens_a = 0;  // shared part: splits of split_tokens_a (multiple of 128)
  // decode (rotary + KV write + attention in one launch, split merge in a second)
  const float* qkv_raw;            // fp32 [planes][rows][(n_q_heads + 2 n_kv_heads) * 128], projections before
                                   // rotary, as split-K planes that the kernel sums in ascending order
  int qkv_planes;                  // >= 1
  long long qkv_plane_stride;      // floats between planes
  const float* cos_sin;
  QkvExtras extra;                 // decode: bias / per-head norm of the new q, k, v
  uint16_t* kv_pool_w;
  // prefill: packed sequences
  const int *seq_row0, *seq_len, *seq_slot;
  const int* seq_pos0 = nullptr;   // position of each sequence's first row (NULL = 0): rows that
                                   // continue a cached context attend to it as well
  int n_seqs, max_seq_len;
};
void launch_attention_prefill(const AttnArgs& a, hipStream_t s);
// Decode attention: partial results per (row, KV head, slot) when a.n_splits > 1 or the launch is
// the grouped one - launch_attention_merge then joins the slots; with one split the result is final.
void launch_attention_decode_fused(const AttnArgs& a, hipStream_t s);
// the same with shared prompts; needs n_q_heads / n_kv_heads <= 8 (4 members x heads <= 32 columns)
void launch_attention_decode_grouped(const AttnArgs& a, hipStream_t s);
void launch_attention_merge(const AttnArgs& a, hipStream_t s);

// ---- policy-gradient objective over packed rollouts (kernels_loss.hip) ----------------------
struct PolicyLossArgs {
  int n_seqs;
  long long total;            // tokens = cu_seqlens[n_seqs]
  const int* cu_seqlens;      // [n_seqs + 1]
  const float *logp_new, *logp_old, *logp_ref;  // [total]; logp_ref may be NULL
  const unsigned char* mask;  // [total] 1 = the token counts
  const float* rewards;       // [n_seqs]
  float gamma, kl_coef, reward_clip, adv_clip, eps_low, eps_high;
  float* grad;                // [total] d loss / d logp_new
  float* advantages;          // [total] or NULL
  float *part_sum, *part_cnt; // [n_seqs] scratch
  float* result;              // [2]: loss, 1 / N
};
void launch_policy_loss(const PolicyLossArgs& p, hipStream_t s);

// ---- mixture-of-experts block on the matrix-core path ---------------------------------------
// Routing: sums the split planes of the router projection, picks the top_k experts of every
// row by (logit descending, expert index ascending), mixes with the softmax over the picked
// logits, and takes each pick's position inside its expert's list from an integer counter.
struct MoeRouteArgs {
  const float* partial;     // [splits][rows][n_experts] router logits (split planes)
  long long split_stride;
  int splits;
  int rows, n_experts, top_k;
  int* idx;                 // [rows][top_k] expert of pick j
  float* wt;                // [rows][top_k] mixing weight of pick j
  int* pos;                 // [rows][top_k] position of the pick inside its expert's list
  int* count;               // [n_experts], zero on entry: picks per expert
  int* route_log;           // optional copy of idx (parity hook)
};
void launch_moe_route_topk(const MoeRouteArgs& a, hipStream_t s);

// Plan of the grouped projections: expert-sorted slots, cut into row blocks of 64.
struct MoePlanArgs {
  const int* count;         // [n_experts]
  const int* idx;           // [rows * top_k]
  const int* pos;           // [rows * top_k]
  int rows, n_experts, top_k, max_blocks;
  int* row_map;             // [rows * top_k] slot -> source row
  int* slot_of;             // [rows * top_k] (row, pick) -> slot
  int* group_of_block;      // [max_blocks]
  int* block_row_begin;     // [max_blocks]
  int* block_row_end;       // [max_blocks]; unused blocks get begin = end = 0
};
void launch_moe_plan(const MoePlanArgs& a, hipStream_t s);
constexpr int kMoeBlockRows = 64;
