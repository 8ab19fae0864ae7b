// Paged grouped-query attention on the matrix cores, head_dim 128, half-precision KV pages in
// the KV_MATRIX element order (common.h).  Queries and probabilities enter the matrix
// instructions as hi + lo half-precision pairs, so keys and values are the only rounded
// operands; the result leaves as hi + lo bf16 planes for the output projection.
//
// Decoding is memory-bound (paper section 2.1) and its attention streams every cached key
// and value once per step, so the kernels are built around that stream: each wavefront
// takes 32 cached positions at a time as sixteen contiguous 1 KiB loads (8 key fragments,
// 8 value fragments), computes transposed scores S^T = K q^T with 16x16x32 f16 matrix
// instructions (columns = the query rows that share the KV head), runs the online softmax
// on the fragment (per-column max and sum are a register reduction plus two cross-lane
// steps), and feeds the probabilities straight back as the B operand of O^T += V^T P^T.
// The value pages are stored in exactly the k-order in which a score fragment holds its
// probabilities, so P never moves between lanes.
//
//   decode  : one workgroup per (KV split, KV head, sample); columns = the G query heads;
//             the rotary embedding of the new query and key and the KV-page write ride in
//             the prologue; its 4 wavefronts interleave over the split's 32-position groups
//             and merge through LDS; several splits per sample merge in a second small kernel.
//   decode, shared prompts (optional): in the same launch, workgroups of (split, KV head, up
//             to 4 samples of one prompt) take the prompt's shared pages with the members'
//             query heads as columns, and the per-sample workgroups start after those pages.
//   prefill : one wavefront per (16 query positions, query head); columns = positions;
//             causal limit per column; a sequence may continue a cached context (its rows
//             then attend to that context too).
#include "kernels_fast.h"

typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
union Frag {
  uint4 u;
  f16x8 v;
  uint16_t h[8];
};
#define MFMA16(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0)

#define DH 128
#define GROUP_U4 512  // uint4 per 32-position group of one K (or V) block: 32 * 128 * 2 / 16
// Probabilities are scaled by 2^10 before they become half-precision operands, so that the
// small probabilities of a long, flat attention row stay in the normal range; the output
// accumulators carry the same factor until the final normalisation.
#define P_SCALE 1024.0f

// One 32-position group (fragments already in registers) against this lane's query column.
// limit = last visible position of the column.  m, l in log2 units; o = unnormalised
// output^T fragments.
__device__ inline void attend_frags(const Frag (&k)[2][4], const Frag (&v)[8], const Frag (&q)[8], int tok0,
                                    int limit, float scale_log2, float& m, float& l, f32x4 (&o)[8], int lane) {
  const int g = lane >> 4;
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {  // q[4..7] = lo parts of the query, q[0..3] = hi parts
    s0 = MFMA16(k[0][ks].v, q[4 + ks].v, s0);
    s1 = MFMA16(k[1][ks].v, q[4 + ks].v, s1);
  }
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    s0 = MFMA16(k[0][ks].v, q[ks].v, s0);
    s1 = MFMA16(k[1][ks].v, q[ks].v, s1);
  }
  float sc[8];
  const int tbase = tok0 + 4 * g;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    sc[i] = (tbase + i <= limit) ? s0[i] * scale_log2 : -INFINITY;
    sc[4 + i] = (tbase + 16 + i <= limit) ? s1[i] * scale_log2 : -INFINITY;
  }
  float mx = sc[0];
#pragma unroll
  for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sc[e]);
  mx = fmaxf(mx, __shfl_xor(mx, 16, WAVE));
  mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
  const float m_new = fmaxf(m, mx);
  const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
  float ps = 0.f;
  Frag pb, pl;  // probabilities as hi + lo half-precision parts
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float p = exp2f(sc[e] - m_use);
    ps += p;
    split_f16(p * P_SCALE, pb.h[e], pl.h[e]);
  }
  ps += __shfl_xor(ps, 16, WAVE);
  ps += __shfl_xor(ps, 32, WAVE);
  const float alpha = exp2f(m - m_use);
  l = l * alpha + ps;
  m = m_new;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    o[j][0] *= alpha;
    o[j][1] *= alpha;
    o[j][2] *= alpha;
    o[j][3] *= alpha;
    o[j] = MFMA16(v[j].v, pl.v, o[j]);
    o[j] = MFMA16(v[j].v, pb.v, o[j]);
  }
}

// key and value fragments of one 32-position group from its KV page
__device__ __forceinline__ void load_group(const uint4* __restrict__ kblk, const uint4* __restrict__ vblk,
                                           Frag (&k)[2][4], Frag (&v)[8], int lane) {
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) k[t][ks].u = kblk[(t * 4 + ks) * 64 + lane];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j].u = vblk[j * 64 + lane];
}

// The same, with the group's key and value fragments streamed from a KV page.
__device__ inline void attend_group(const uint4* __restrict__ kblk, const uint4* __restrict__ vblk,
                                    const Frag (&q)[8], int tok0, int limit, float scale_log2, float& m,
                                    float& l, f32x4 (&o)[8], int lane) {
  Frag k[2][4], v[8];
  load_group(kblk, vblk, k, v, lane);
  attend_frags(k, v, q, tok0, limit, scale_log2, m, l, o, lane);
}

// the 32-position group that starts at position tok0, inside page `page`
__device__ inline const uint4* page_block(const AttnArgs& a, int page, int kv_head, int tok0, int is_v) {
  const int gip = (tok0 % a.geom.page_tokens) >> 5;
  return (const uint4*)(a.kv_pool + kv_block_base(a.geom, a.layer, page, kv_head, is_v)) + gip * GROUP_U4;
}
__device__ inline const uint4* group_block(const AttnArgs& a, int slot, int kv_head, int tok0, int is_v) {
  return page_block(a, a.page_table[(long long)slot * a.max_pages + tok0 / a.geom.page_tokens], kv_head, tok0, is_v);
}

// four consecutive values as hi + lo bf16 parts into the two planes of an activation buffer
__device__ inline void store4_split(uint16_t* dst, long long lo_offset, float a, float b, float c, float d) {
  uint16_t hi[4], lo[4];
  split_bf16(a, hi[0], lo[0]);
  split_bf16(b, hi[1], lo[1]);
  split_bf16(c, hi[2], lo[2]);
  split_bf16(d, hi[3], lo[3]);
  *(uint2*)dst = make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
  *(uint2*)(dst + lo_offset) = make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
}
__device__ inline void store1_split(uint16_t* dst, long long lo_offset, float a) {
  uint16_t hi, lo;
  split_bf16(a, hi, lo);
  dst[0] = hi;
  dst[lo_offset] = lo;
}

// element (row b, column k) of the decode result
__device__ inline long long out_offset(const AttnArgs& a, int b, int k) {
  const int q_dim = a.n_q_heads * DH;
  return a.out_frag ? frag_offset(b, k, q_dim >> 5) : (long long)b * q_dim + k;
}

// ------------------------------------------------------------------------------ fused decode
// One launch per layer for a decode step: sums nothing and stores nothing in between.
// Prologue: rotary embedding of this sample's G query rows (kept in LDS as hi + lo half-precision parts) and, in the
// workgroup whose split holds the new position, of the new key; that key and the new value
// are written to the sample's page and also kept in LDS.  Main loop: the cached positions
// t0..pos-1 from the pages (t0 = 0 unless the sample's prompt is attended by its group, below).
// The new position itself is attended from LDS as a one-token group, so nothing written in
// this launch is read back from memory.  With several partial results per (sample, KV head)
// they go to attn_merge_fused_kernel.
// EXTRA: the model adds a bias to q, k, v and / or normalises q and k heads (a.extra).
struct DecodeSmem {
  uint16_t* q;   // [2][q_cols][DH] hi parts, lo parts
  int q_cols;
  uint16_t* kv;  // [2][DH]
  float* m;      // [4][ml_cols]
  float* l;      // [4][ml_cols]
  int ml_cols;
  float* o;      // [4][16 * DH]
};

// elements p[0] and p[64] summed over the split-K planes in ascending order, eight planes'
// loads in flight together
__device__ __forceinline__ void sum_planes(const AttnArgs& a, const float* p, float& x0, float& x1) {
  x0 = 0.f;
  x1 = 0.f;
  constexpr int ZR = 8;
  for (int z = 0; z < a.qkv_planes; z += ZR) {
    const long long st = a.qkv_plane_stride;
    const float* q = p + (long long)z * st;
    const int left = a.qkv_planes - z;
    float u[ZR], w[ZR];
#pragma unroll
    for (int i = 0; i < ZR; ++i) {
      u[i] = i < left ? q[i * st] : 0.f;
      w[i] = i < left ? q[i * st + 64] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < ZR; ++i) {
      x0 += u[i];
      x1 += w[i];
    }
  }
}

// Sum over the split-K planes of this thread's N query elements (x0 = element i, x1 = element
// i + 64 of each column's head), planes in ascending order.  The loads of up to eight planes (four
// with more than four columns) of all columns are in flight together: under load a round trip to memory costs more than
// anything else this kernel does before its main loop.
template <int N>
__device__ __forceinline__ void sum_query_planes(const AttnArgs& a, const float* const (&src)[N], float (&x0)[N],
                                                 float (&x1)[N]) {
  if (a.qkv_planes == 1) {
#pragma unroll
    for (int n = 0; n < N; ++n) {
      x0[n] = 0.f + src[n][0];
      x1[n] = 0.f + src[n][64];
    }
    return;
  }
#pragma unroll
  for (int n = 0; n < N; ++n) x0[n] = x1[n] = 0.f;
  constexpr int ZR = N <= 4 ? 8 : 4;  // planes per round: 64 values in flight per thread
  for (int z = 0; z < a.qkv_planes; z += ZR) {
    float u0[ZR][N], u1[ZR][N];
#pragma unroll
    for (int q = 0; q < ZR; ++q) {
      const bool on = z + q < a.qkv_planes;
      const long long o = (long long)(on ? z + q : z) * a.qkv_plane_stride;
#pragma unroll
      for (int n = 0; n < N; ++n) {
        u0[q][n] = on ? src[n][o] : 0.f;
        u1[q][n] = on ? src[n][o + 64] : 0.f;
      }
    }
#pragma unroll
    for (int q = 0; q < ZR; ++q)
#pragma unroll
      for (int n = 0; n < N; ++n) {
        x0[n] += u0[q][n];
        x1[n] += u1[q][n];
      }
  }
}

// Query staging.  Thread t of the workgroup owns the rotary pairs idx = t + 256 n, n < N:
// column idx / 64 (the same in all 64 lanes), pair idx % 64.  rows[n] / heads[n] name the
// sample row and the query head inside its KV group that column holds (row < 0: the column
// is empty).  x0 / x1: the projection's elements, planes summed; cs: cos, sin of the row's position.
// Bias / head norm, the rotary embedding, and the hi + lo half-precision parts into sm.q.
template <bool EXTRA, int N>
__device__ __forceinline__ void rotate_and_stage(const AttnArgs& a, const DecodeSmem& sm, int kvh, int G,
                                                 const int (&rows)[N], const int (&heads)[N], float (&x0)[N],
                                                 float (&x1)[N], const float2 (&cs)[N]) {
  const int tid = threadIdx.x, i = tid & 63;
#pragma unroll
  for (int n = 0; n < N; ++n) {
    const int col = (tid + 256 * n) >> 6;
    float u = 0.f, w = 0.f;
    if (rows[n] >= 0) {  // uniform over the wavefront
      if (EXTRA) qkv_extras(a.extra, (kvh * G + heads[n]) * DH, i, a.extra.q_gain, x0[n], x1[n]);
      const float cc = cs[n].x, sn = cs[n].y;
      u = x0[n] * cc - x1[n] * sn;
      w = x1[n] * cc + x0[n] * sn;
    }
    uint16_t* hi = sm.q + (long long)col * DH;
    uint16_t* lo = hi + (long long)sm.q_cols * DH;
    split_f16(u, hi[i], lo[i]);
    split_f16(w, hi[i + 64], lo[i + 64]);
  }
}
// the two together, positions read from row_pos (columns of several rows)
template <bool EXTRA, int N>
__device__ __forceinline__ void stage_queries(const AttnArgs& a, const DecodeSmem& sm, int kvh, int G,
                                              const int (&rows)[N], const int (&heads)[N]) {
  const int i = threadIdx.x & 63;
  const int q_dim = a.n_q_heads * DH, kv_dim = a.geom.n_kv_heads * DH;
  const float* src[N];
  float x0[N], x1[N];
  float2 cs[N];  // requested with the planes
#pragma unroll
  for (int n = 0; n < N; ++n) {
    const int b = max(rows[n], 0);  // empty columns read row 0 and are zeroed below
    src[n] = a.qkv_raw + (long long)b * (q_dim + 2 * kv_dim) + (kvh * G + heads[n]) * DH + i;
    cs[n] = *(const float2*)(a.cos_sin + (long long)a.row_pos[b] * DH + 2 * i);
  }
  sum_query_planes<N>(a, src, x0, x1);
  rotate_and_stage<EXTRA, N>(a, sm, kvh, G, rows, heads, x0, x1, cs);
}

// the 4 wavefronts' results of 16 columns -> one (max, sum, unnormalised output) per column in
// sm.o[0..3], sm.m, sm.l (columns ml0 ..); every thread of the workgroup calls it
__device__ __forceinline__ float merged_max(const DecodeSmem& sm, int col) {
  return fmaxf(fmaxf(sm.m[col], sm.m[sm.ml_cols + col]), fmaxf(sm.m[2 * sm.ml_cols + col], sm.m[3 * sm.ml_cols + col]));
}
__device__ __forceinline__ float merged_sum(const DecodeSmem& sm, int col) {
  return sm.l[col] + sm.l[sm.ml_cols + col] + sm.l[2 * sm.ml_cols + col] + sm.l[3 * sm.ml_cols + col];
}
__device__ __forceinline__ void merge_wavefronts(const DecodeSmem& sm, int ml0, float m, float l, const f32x4 (&o)[8],
                                                 int wave, int c, int g) {
  if (g == 0) sm.m[wave * sm.ml_cols + ml0 + c] = m;
  __syncthreads();
  const float M = merged_max(sm, ml0 + c);
  const float M_use = (M == -INFINITY) ? 0.f : M;
  const float w = exp2f(m - M_use);
  if (g == 0) sm.l[wave * sm.ml_cols + ml0 + c] = l * w;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) sm.o[wave * (16 * DH) + c * DH + 16 * j + 4 * g + i] = o[j][i] * w;
  __syncthreads();
}
// element e of the merged, unnormalised output: the wavefronts' parts in ascending order
__device__ __forceinline__ float merged_out(const DecodeSmem& sm, int e) {
  return sm.o[e] + sm.o[16 * DH + e] + sm.o[2 * 16 * DH + e] + sm.o[3 * 16 * DH + e];
}

// one workgroup = (own-range split, KV head, sample); wavefront w takes the groups w, w + 4, ...
// of the split.  What the workgroup needs before its main loop comes in three sets of loads:
// (1) the row's position and page-table row, and - they depend on neither - every split-K plane
// of its query columns and of the new key and value; (2) what depends on the position: cos and
// sin, the page of the new position and the page of the wavefront's first group; (3) that
// group's keys and values, in flight while the queries are rotated and staged.
template <bool EXTRA>
__device__ __forceinline__ void decode_own_range(const AttnArgs& a, const DecodeSmem& sm, int split, int kvh, int b) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, g = lane >> 4, i = lane;
  const int n_kv = a.geom.n_kv_heads;
  const int G = a.n_q_heads / n_kv;
  const int T = a.geom.page_tokens;
  const int pos = a.row_pos[b];
  const int t0 = a.row_t0 ? a.row_t0[b] : 0;
  const int slot = a.row_slot[b];
  const int q_dim = a.n_q_heads * DH, kv_dim = n_kv * DH;
  const float* row = a.qkv_raw + (long long)b * (q_dim + 2 * kv_dim);
  // ---- first set of loads (does not wait for the position)
  int rows[4], heads[4];
  const float* src[4];
  float x0[4], x1[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) {
    heads[n] = wave + 4 * n;  // column = head inside the KV group
    rows[n] = heads[n] < G ? b : -1;
    heads[n] = min(heads[n], G - 1);
    src[n] = row + (kvh * G + heads[n]) * DH + i;
  }
  // the new key (even wavefronts) or value (odd ones); wavefronts 0 and 1 of the split that owns
  // the new position use theirs
  const bool is_v = wave & 1;
  float n0, n1;
  sum_planes(a, row + q_dim + (is_v ? kv_dim : 0) + kvh * DH + i, n0, n1);
  sum_query_planes<4>(a, src, x0, x1);
  const int used = (pos - t0) / a.split_tokens + 1;  // splits that hold at least the new position
  if (split >= used) return;
  const bool owner = split == used - 1;
  const bool direct = used == 1 && t0 == 0;          // the only partial result of this (sample, KV head)
  const bool writer = owner && wave < 2;
  const int t_begin = t0 + split * a.split_tokens;
  const int t_end = min(pos, t_begin + a.split_tokens);  // cached positions only
  int tok0 = t_begin + wave * 32;
  // ---- second set: what depends on the position
  const int* pt = a.page_table + (long long)slot * a.max_pages;
  const float2 rot = *(const float2*)(a.cos_sin + (long long)pos * DH + 2 * i);
  const int new_page = writer ? pt[pos / T] : 0;
  const int first_page = tok0 < t_end ? pt[tok0 / T] : 0;
  // ---- third set: the first group's keys and values
  Frag k[2][4], v[8];
  if (tok0 < t_end)
    load_group(page_block(a, first_page, kvh, tok0, 0), page_block(a, first_page, kvh, tok0, 1), k, v, lane);
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
  const float2 cs[4] = {rot, rot, rot, rot};
  rotate_and_stage<EXTRA, 4>(a, sm, kvh, G, rows, heads, x0, x1, cs);
  if (writer) {
    const int tok = pos % T;
    if (!is_v) {
      if (EXTRA) qkv_extras(a.extra, q_dim + kvh * DH, i, a.extra.k_gain, n0, n1);  // wavefront 0
      const uint16_t k0 = f32_to_f16(n0 * rot.x - n1 * rot.y).bits, k1 = f32_to_f16(n1 * rot.x + n0 * rot.y).bits;
      sm.kv[i] = k0;
      sm.kv[i + 64] = k1;
      uint16_t* dst = a.kv_pool_w + kv_block_base(a.geom, a.layer, new_page, kvh, 0);
      dst[kv_k_offset(a.geom, tok, i)] = k0;
      dst[kv_k_offset(a.geom, tok, i + 64)] = k1;
    } else {
      if (EXTRA) qkv_extras(a.extra, q_dim + kv_dim + kvh * DH, i, nullptr, n0, n1);  // wavefront 1: bias only
      const uint16_t v0 = f32_to_f16(n0).bits, v1 = f32_to_f16(n1).bits;
      sm.kv[DH + i] = v0;
      sm.kv[DH + i + 64] = v1;
      uint16_t* dst = a.kv_pool_w + kv_block_base(a.geom, a.layer, new_page, kvh, 1);
      dst[kv_v_offset(a.geom, tok, i)] = v0;
      dst[kv_v_offset(a.geom, tok, i + 64)] = v1;
    }
  }
  __syncthreads();

  Frag q[8];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    q[ks].u = *(const uint4*)&sm.q[c * DH + ks * 32 + g * 8];
    q[4 + ks].u = *(const uint4*)&sm.q[(sm.q_cols + c) * DH + ks * 32 + g * 8];
  }
  float m = -INFINITY, l = 0.f;
  f32x4 o[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (tok0 < t_end) {  // the group that is in registers already
    attend_frags(k, v, q, tok0, pos - 1, scale_log2, m, l, o, lane);
    tok0 += 128;
  }
  for (; tok0 < t_end; tok0 += 128)
    attend_group(group_block(a, slot, kvh, tok0, 0), group_block(a, slot, kvh, tok0, 1), q, tok0, pos - 1,
                 scale_log2, m, l, o, lane);
  if (owner && wave == 3) {  // the new position, from LDS: token 0 of a group that starts at pos
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      k[0][ks].u = make_uint4(0, 0, 0, 0);
      k[1][ks].u = make_uint4(0, 0, 0, 0);
      if (c == 0) k[0][ks].u = *(const uint4*)&sm.kv[ks * 32 + g * 8];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      v[j].u = make_uint4(0, 0, 0, 0);
      if (g == 0) v[j].h[0] = sm.kv[DH + 16 * j + c];
    }
    attend_frags(k, v, q, pos, pos, scale_log2, m, l, o, lane);
  }

  merge_wavefronts(sm, 0, m, l, o, wave, c, g);
  const int n_slots = a.n_slots ? a.n_slots : a.n_splits;
  const long long part = ((long long)b * n_kv + kvh) * n_slots + a.slot0 + split;
  for (int e = tid; e < G * DH; e += 256) {
    const int col = e >> 7;
    const float acc = merged_out(sm, e);
    if (direct) store1_split(a.out + out_offset(a, b, kvh * G * DH + e), a.out_lo_offset, acc / (merged_sum(sm, col) * P_SCALE));
    else a.part_o[part * (16 * DH) + e] = acc;
  }
  if (!direct && tid < 16) {
    a.part_ml[part * 32 + tid] = merged_max(sm, tid);
    a.part_ml[part * 32 + 16 + tid] = merged_sum(sm, tid);
  }
}

template <bool EXTRA>
__global__ __launch_bounds__(256, 3) void attn_decode_fused_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t q_s[2 * 16 * DH];
  __shared__ __attribute__((aligned(16))) uint16_t kv_s[2 * DH];
  __shared__ float m_s[4 * 16], l_s[4 * 16];
  __shared__ float o_s[4 * 16 * DH];
  decode_own_range<EXTRA>(a, DecodeSmem{q_s, 16, kv_s, m_s, l_s, 16, o_s}, blockIdx.x, blockIdx.y, blockIdx.z);
}

// ------------------------------------------------------------------------------ shared prompts
// The n samples of a prompt share the prompt's full pages.  A group workgroup = (split of the
// shared positions, KV head, up to 4 samples of one prompt): the members' query heads are the
// columns - 4 G of them in NCT tiles of 16 - so one pass over the shared keys and values serves
// all members, and each member's partial result lands in its own partial slot [0, slot0).
// The same launch holds the own-range workgroups of every sample (decode_own_range from
// row_t0 on); attn_merge_fused_kernel joins the slots.  Every shared position is visible to
// every member (it precedes their prompts' ends), so no causal limit applies here.
template <int NCT, bool EXTRA>
__device__ __forceinline__ void decode_shared_range(const AttnArgs& a, const DecodeSmem& sm, int split, int kvh,
                                                    int grp) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int n_kv = a.geom.n_kv_heads;
  const int G = a.n_q_heads / n_kv;
  const int len = a.grp_len[grp];
  const int t_begin = split * a.split_tokens_a;
  if (t_begin >= len) return;
  const int t_end = min(len, t_begin + a.split_tokens_a);
  const int slot = a.grp_slot[grp];
  const int* members = a.grp_rows + grp * GROUP_MEMBERS;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);

  {
    int rows[4 * NCT], heads[4 * NCT];
#pragma unroll
    for (int n = 0; n < 4 * NCT; ++n) {
      const int col = (tid >> 6) + 4 * n, j = col / G;
      rows[n] = j < GROUP_MEMBERS ? members[j] : -1;
      heads[n] = col % G;
    }
    stage_queries<EXTRA, 4 * NCT>(a, sm, kvh, G, rows, heads);
  }
  __syncthreads();

  // one pass over the range per column tile: the second pass finds the fragments in L2, and the
  // registers stay those of a single tile (three workgroups per CU)
  const int n_slots = a.n_slots ? a.n_slots : a.n_splits;
#pragma unroll 1
  for (int ct = 0; ct < NCT; ++ct) {
    Frag q[8];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      q[ks].u = *(const uint4*)&sm.q[(ct * 16 + c) * DH + ks * 32 + g * 8];
      q[4 + ks].u = *(const uint4*)&sm.q[(sm.q_cols + ct * 16 + c) * DH + ks * 32 + g * 8];
    }
    float m = -INFINITY, l = 0.f;
    f32x4 o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int tok0 = t_begin + wave * 32; tok0 < t_end; tok0 += 128)
      attend_group(group_block(a, slot, kvh, tok0, 0), group_block(a, slot, kvh, tok0, 1), q, tok0, 0x7fffffff,
                   scale_log2, m, l, o, lane);
    merge_wavefronts(sm, ct * 16, m, l, o, wave, c, g);
    for (int e = tid; e < 16 * DH; e += 256) {
      const int col = ct * 16 + (e >> 7);
      const int j = col / G, hc = col % G;
      const int b = j < GROUP_MEMBERS ? members[j] : -1;
      if (b < 0) continue;
      const long long part = ((long long)b * n_kv + kvh) * n_slots + split;
      a.part_o[part * (16 * DH) + hc * DH + (e & 127)] =
          sm.o[e] + sm.o[16 * DH + e] + sm.o[2 * 16 * DH + e] + sm.o[3 * 16 * DH + e];
    }
    if (tid < 16) {
      const int col = ct * 16 + tid;
      const int j = col / G, hc = col % G;
      const int b = j < GROUP_MEMBERS ? members[j] : -1;
      if (b >= 0) {
        const long long part = ((long long)b * n_kv + kvh) * n_slots + split;
        a.part_ml[part * 32 + hc] = merged_max(sm, col);
        a.part_ml[part * 32 + 16 + hc] = merged_sum(sm, col);
      }
    }
    __syncthreads();  // sm.o is reused by the next tile
  }
}

// workgroups [0, n_groups * n_kv * n_splits_a) take the shared ranges, the rest the own ranges
template <int NCT, bool EXTRA>
__global__ __launch_bounds__(256, 3) void attn_decode_grouped_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t q_s[2 * NCT * 16 * DH];
  __shared__ __attribute__((aligned(16))) uint16_t kv_s[2 * DH];
  __shared__ float m_s[4 * NCT * 16], l_s[4 * NCT * 16];
  __shared__ float o_s[4 * 16 * DH];
  const DecodeSmem sm{q_s, NCT * 16, kv_s, m_s, l_s, NCT * 16, o_s};
  const int n_kv = a.geom.n_kv_heads;
  const int n_shared = a.n_groups * n_kv * a.n_splits_a;
  int w = blockIdx.x;
  if (w < n_shared) {
    decode_shared_range<NCT, EXTRA>(a, sm, w % a.n_splits_a, (w / a.n_splits_a) % n_kv, w / (a.n_splits_a * n_kv));
  } else {
    w -= n_shared;
    decode_own_range<EXTRA>(a, sm, w % a.n_splits, (w / a.n_splits) % n_kv, w / (a.n_splits * n_kv));
  }
}

// Merge of the partial results of one (sample, KV head), at most 16 slots: a launch of its
// own, because a launch boundary is the cheapest way to publish results between workgroups here.
__global__ __launch_bounds__(256) void attn_merge_fused_kernel(AttnArgs a) {
  __shared__ float w_s[16][16];  // [slot][column] weight 2^(m_s - M) / (L 2^10)
  const int tid = threadIdx.x, kvh = blockIdx.x, b = blockIdx.y;
  const int n_kv = a.geom.n_kv_heads;
  const int G = a.n_q_heads / n_kv;
  const int n_slots = a.n_slots ? a.n_slots : a.n_splits;
  const long long part0 = ((long long)b * n_kv + kvh) * n_slots;
  // Every load is requested at once - the row's position, which tells the slots in use, and all
  // 16 slots' maxima, sums and outputs (up to 4 x 16 values per thread for 8 query heads; slots
  // past the last one read the last one) - and what an unused slot held is dropped afterwards:
  // one round trip to memory instead of three.
  const int t0 = a.row_t0 ? a.row_t0[b] : 0;
  const int pos = a.row_pos[b];
  const int ms = min(tid >> 4, n_slots - 1), mcol = tid & 15;
  const float m_ld = a.part_ml[(part0 + ms) * 32 + mcol];
  const float l_ld = a.part_ml[(part0 + ms) * 32 + 16 + mcol];
  constexpr int E_MAX = 4;  // the first 1024 of the G * DH outputs; more than 8 query heads: the rest below
  float v[E_MAX][16];
#pragma unroll
  for (int i = 0; i < E_MAX; ++i) {
    const int e = tid + 256 * i;
#pragma unroll
    for (int s = 0; s < 16; ++s)
      v[i][s] = e < G * DH ? a.part_o[(part0 + min(s, n_slots - 1)) * (16 * DH) + e] : 0.f;
  }
  const int used_shared = t0 ? (t0 + a.split_tokens_a - 1) / a.split_tokens_a : 0;
  const int used_own = (pos - t0) / a.split_tokens + 1;
  if (used_shared == 0 && used_own == 1) return;  // the attention kernel wrote the result itself
  const unsigned valid = ((1u << used_shared) - 1u) | (((1u << used_own) - 1u) << a.slot0);
#pragma unroll
  for (int i = 0; i < E_MAX; ++i)
#pragma unroll
    for (int s = 0; s < 16; ++s)
      if (!((valid >> s) & 1u)) v[i][s] = 0.f;
  {
    const int s = tid >> 4, col = tid & 15;  // 256 threads = 16 slots x 16 columns
    const bool on = (valid >> s) & 1u;
    const float m = on ? m_ld : -INFINITY;
    const float l = on ? l_ld : 0.f;
    w_s[s][col] = m;
    __syncthreads();
    float M = -INFINITY;
#pragma unroll
    for (int q = 0; q < 16; ++q) M = fmaxf(M, w_s[q][col]);
    const float w = exp2f(m - M);  // 0 for unused slots
    __syncthreads();
    w_s[s][col] = w;
    // total weight of the column, same order in every thread
    __shared__ float lw_s[16][16];
    lw_s[s][col] = l * w;
    __syncthreads();
    float L = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) L += lw_s[q][col];
    __syncthreads();
    w_s[s][col] = w / (L * P_SCALE);
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < E_MAX; ++i) {
    const int e = tid + 256 * i;
    if (e >= G * DH) break;
    const int col = e >> 7;
    float acc = 0.f;
#pragma unroll
    for (int s = 0; s < 16; ++s) acc += v[i][s] * w_s[s][col];
    store1_split(a.out + out_offset(a, b, kvh * G * DH + e), a.out_lo_offset, acc);
  }
  for (int e = tid + 256 * E_MAX; e < G * DH; e += 256) {
    const int col = e >> 7;
    float u[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) u[s] = ((valid >> s) & 1u) ? a.part_o[(part0 + s) * (16 * DH) + e] : 0.f;
    float acc = 0.f;
#pragma unroll
    for (int s = 0; s < 16; ++s) acc += u[s] * w_s[s][col];
    store1_split(a.out + out_offset(a, b, kvh * G * DH + e), a.out_lo_offset, acc);
  }
}

void launch_attention_decode_fused(const AttnArgs& a, hipStream_t s) {
  if (!a.rows) return;
  const dim3 grid(a.n_splits, a.geom.n_kv_heads, a.rows);
  if (a.extra.bias || a.extra.q_gain) attn_decode_fused_kernel<true><<<grid, 256, 0, s>>>(a);
  else attn_decode_fused_kernel<false><<<grid, 256, 0, s>>>(a);
}
void launch_attention_merge(const AttnArgs& a, hipStream_t s) {
  if (a.rows) attn_merge_fused_kernel<<<dim3(a.geom.n_kv_heads, a.rows), 256, 0, s>>>(a);
}

template <int NCT>
static void launch_grouped(const AttnArgs& a, unsigned grid, hipStream_t s) {
  if (a.extra.bias || a.extra.q_gain) attn_decode_grouped_kernel<NCT, true><<<grid, 256, 0, s>>>(a);
  else attn_decode_grouped_kernel<NCT, false><<<grid, 256, 0, s>>>(a);
}
void launch_attention_decode_grouped(const AttnArgs& a, hipStream_t s) {
  if (!a.rows) return;
  const int n_kv = a.geom.n_kv_heads, G = a.n_q_heads / n_kv;
  const unsigned grid = (unsigned)(a.n_groups * n_kv * a.n_splits_a + a.rows * n_kv * a.n_splits);
  if (GROUP_MEMBERS * G <= 16) launch_grouped<1>(a, grid, s);
  else launch_grouped<2>(a, grid, s);
}

// ------------------------------------------------------------------------------ prefill
__global__ __launch_bounds__(256) void attn_prefill_kernel(AttnArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int seq = blockIdx.z, head = blockIdx.y;
  const int len = a.seq_len[seq];
  const int q0 = blockIdx.x * 64 + wave * 16;
  if (q0 >= len) return;  // wavefronts are independent: no barrier below
  const int row0 = a.seq_row0[seq], slot = a.seq_slot[seq];
  const int p0 = a.seq_pos0 ? a.seq_pos0[seq] : 0;  // cached positions before the sequence's first row
  const int kvh = head / (a.n_q_heads / a.geom.n_kv_heads);
  const int qi = q0 + c;                             // row of this column inside the sequence
  const int pos = p0 + qi;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
  Frag q[8];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    q[ks].u = make_uint4(0, 0, 0, 0);
    q[4 + ks].u = make_uint4(0, 0, 0, 0);
    if (qi < len) {
      const uint16_t* src = a.q + ((long long)(row0 + qi) * a.n_q_heads + head) * DH + ks * 32 + g * 8;
      q[ks].u = *(const uint4*)src;
      q[4 + ks].u = *(const uint4*)(src + a.q_lo_offset);
    }
  }
  float m = -INFINITY, l = 0.f;
  f32x4 o[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int last = p0 + min(q0 + 15, len - 1);
  for (int tok0 = 0; tok0 <= last; tok0 += 32)
    attend_group(group_block(a, slot, kvh, tok0, 0), group_block(a, slot, kvh, tok0, 1), q, tok0, pos, scale_log2,
                 m, l, o, lane);
  if (qi < len) {
    uint16_t* dst = a.out + ((long long)(row0 + qi) * a.n_q_heads + head) * DH + 4 * g;
    const float inv = 1.0f / (l * P_SCALE);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      store4_split(dst + 16 * j, a.out_lo_offset, o[j][0] * inv, o[j][1] * inv, o[j][2] * inv, o[j][3] * inv);
  }
}

void launch_attention_prefill(const AttnArgs& a, hipStream_t s) {
  if (!a.n_seqs) return;
  attn_prefill_kernel<<<dim3(ceil_div(a.max_seq_len, 64), a.n_q_heads, a.n_seqs), 256, 0, s>>>(a);
}
