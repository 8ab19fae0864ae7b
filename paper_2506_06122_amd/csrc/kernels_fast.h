// Launchers of the matrix-core (bf16) path: packed-weight projections, fused row kernels
// and paged attention.  Pointers are device memory; launches are asynchronous.
#pragma once
#include <algorithm>

#include "common.h"

enum { EPI_F32 = 0, EPI_SWIGLU_BF16 = 1 };

struct GemmArgs {
  const void* a;     // bf16 [rows][K], row stride lda
  const void* w;     // packed bf16 weight, N/16 x K/32 fragments of 1 KiB
  void* out;         // EPI_F32: float [splits][M][ldo]; EPI_SWIGLU_BF16: bf16 [M][ldo] (ldo = N/2)
  int M, N, K, lda, ldo;
  long long split_stride;  // floats between split planes (EPI_F32)
  int k_tiles_per_split;   // filled by the launcher
  // grouped launch (mixture of experts): row block y works on rows
  // [block_row_begin[y], block_row_end[y]) of the expert-sorted order with the weights of
  // group_of_block[y]; row_map maps a sorted row to its source row in `a`.
  const int* group_of_block = nullptr;
  const int* block_row_begin = nullptr;
  const int* block_row_end = nullptr;
  const int* row_map = nullptr;
  long long group_stride16 = 0;  // 16-byte units between consecutive groups' packed weights
  int n_row_blocks = 0;
  int rows_per_block = 0;        // 0 = pick from M
};

int gemm_rows_per_block(int M);
int gemm_pick_splits(int M, int N, int K, int max_splits);
// returns the number of split planes actually written (<= splits)
int launch_gemm_bf16(GemmArgs a, int epi, int splits, hipStream_t s);
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
  uint16_t* h;              // bf16 [rows][hidden]
  const int* tokens;
  const uint16_t* embed;
  const int* rows_index;
  int rows, hidden;
  float eps;
};
void launch_row_norm(const RowNormArgs& a, hipStream_t s);

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
  uint16_t* q_bf16;
  float* q_f32;
  int q_f32_ld;
  uint16_t* kv_pool;
  KvGeom geom;
  int layer, rows, n_q_heads;
};
void launch_qkv_post(const QkvPostArgs& a, hipStream_t s);

void launch_f32_to_bf16(const float* src, uint16_t* dst, long long n, hipStream_t s);

// Paged grouped-query attention on the matrix cores (KV_MATRIX pool, head_dim 128).
struct AttnArgs {
  const uint16_t* q;        // bf16 [rows][n_q_heads][128], rotary applied
  uint16_t* out;            // bf16 [rows][n_q_heads][128]
  const uint16_t* kv_pool;
  KvGeom geom;
  const int* page_table;
  int max_pages, layer, n_q_heads;
  // decode: one row per sample
  const int *row_pos, *row_slot;
  int rows;
  int n_splits, split_tokens;      // KV range per workgroup (multiple of 128)
  float* part_o;                   // [rows][n_kv_heads][n_splits][16][128]
  float* part_ml;                  // [rows][n_kv_heads][n_splits][2][16]
  // prefill: packed sequences
  const int *seq_row0, *seq_len, *seq_slot;
  int n_seqs, max_seq_len;
};
void launch_attention_decode(const AttnArgs& a, hipStream_t s);
void launch_attention_prefill(const AttnArgs& a, hipStream_t s);
