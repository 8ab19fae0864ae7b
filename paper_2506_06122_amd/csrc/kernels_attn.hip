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
//   prefill : one wavefront per (16 query positions, query head); columns = positions;
//             causal limit per column.
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

// The same, with the group's key and value fragments streamed from a KV page.
__device__ inline void attend_group(const uint4* __restrict__ kblk, const uint4* __restrict__ vblk,
                                    const Frag (&q)[8], int tok0, int limit, float scale_log2, float& m,
                                    float& l, f32x4 (&o)[8], int lane) {
  Frag k[2][4], v[8];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) k[t][ks].u = kblk[(t * 4 + ks) * 64 + lane];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j].u = vblk[j * 64 + lane];
  attend_frags(k, v, q, tok0, limit, scale_log2, m, l, o, lane);
}

__device__ inline const uint4* group_block(const AttnArgs& a, int slot, int kv_head, int tok0, int is_v) {
  const int page = a.page_table[(long long)slot * a.max_pages + tok0 / a.geom.page_tokens];
  const int gip = (tok0 % a.geom.page_tokens) >> 5;
  return (const uint4*)(a.kv_pool + kv_block_base(a.geom, a.layer, page, kv_head, is_v)) + gip * GROUP_U4;
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
// 0..pos-1 from the pages.  The new position itself is attended from LDS as a one-token
// group, so nothing written in this launch is read back from memory.  With several KV
// splits per (sample, KV head) the partial results go to attn_merge_fused_kernel.
// EXTRA: the model adds a bias to q, k, v and / or normalises q and k heads (a.extra).
template <bool EXTRA>
__global__ __launch_bounds__(256, 3) void attn_decode_fused_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t q_s[2][16][DH];  // hi parts, lo parts
  __shared__ __attribute__((aligned(16))) uint16_t kv_s[2][DH];
  __shared__ float m_s[4][16];
  __shared__ float l_s[4][16];
  __shared__ float o_s[4][16 * DH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int n_kv = a.geom.n_kv_heads;
  const int G = a.n_q_heads / n_kv;
  const int pos = a.row_pos[b];
  const int used = pos / a.split_tokens + 1;  // splits that hold at least the new position
  if (split >= used) return;
  const bool owner = split == used - 1;
  const int slot = a.row_slot[b];
  const int q_dim = a.n_q_heads * DH, kv_dim = n_kv * DH;
  const float* row = a.qkv_raw + (long long)b * (q_dim + 2 * kv_dim);
  const float* cs = a.cos_sin + (long long)pos * DH;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);

  for (int idx = tid; idx < 16 * (DH / 2); idx += 256) {
    const int hc = idx >> 6, i = idx & 63;
    float u = 0.f, w = 0.f;
    if (hc < G) {
      const float* src = row + (kvh * G + hc) * DH;
      const float cc = cs[2 * i], sn = cs[2 * i + 1];
      float x0 = src[i], x1 = src[i + 64];
      for (int z = 1; z < a.qkv_planes; ++z) {
        x0 += src[z * a.qkv_plane_stride + i];
        x1 += src[z * a.qkv_plane_stride + i + 64];
      }
      if (EXTRA) qkv_extras(a.extra, (kvh * G + hc) * DH, i, a.extra.q_gain, x0, x1);  // hc: same in all 64 lanes
      u = x0 * cc - x1 * sn;
      w = x1 * cc + x0 * sn;
    }
    split_f16(u, q_s[0][hc][i], q_s[1][hc][i]);
    split_f16(w, q_s[0][hc][i + 64], q_s[1][hc][i + 64]);
  }
  if (owner && tid < 128) {
    const int page = a.page_table[(long long)slot * a.max_pages + pos / a.geom.page_tokens];
    const int tok = pos % a.geom.page_tokens;
    const int i = tid & 63;
    if (tid < 64) {
      const float* src = row + q_dim + kvh * DH;
      const float cc = cs[2 * i], sn = cs[2 * i + 1];
      float x0 = src[i], x1 = src[i + 64];
      for (int z = 1; z < a.qkv_planes; ++z) {
        x0 += src[z * a.qkv_plane_stride + i];
        x1 += src[z * a.qkv_plane_stride + i + 64];
      }
      if (EXTRA) qkv_extras(a.extra, q_dim + kvh * DH, i, a.extra.k_gain, x0, x1);  // wavefront 0
      const uint16_t k0 = f32_to_f16(x0 * cc - x1 * sn).bits, k1 = f32_to_f16(x1 * cc + x0 * sn).bits;
      kv_s[0][i] = k0;
      kv_s[0][i + 64] = k1;
      uint16_t* dst = a.kv_pool_w + kv_block_base(a.geom, a.layer, page, kvh, 0);
      dst[kv_k_offset(a.geom, tok, i)] = k0;
      dst[kv_k_offset(a.geom, tok, i + 64)] = k1;
    } else {
      const float* src = row + q_dim + kv_dim + kvh * DH;
      float y0 = src[i], y1 = src[i + 64];
      for (int z = 1; z < a.qkv_planes; ++z) {
        y0 += src[z * a.qkv_plane_stride + i];
        y1 += src[z * a.qkv_plane_stride + i + 64];
      }
      if (EXTRA) qkv_extras(a.extra, q_dim + kv_dim + kvh * DH, i, nullptr, y0, y1);  // wavefront 1: bias only
      const uint16_t v0 = f32_to_f16(y0).bits, v1 = f32_to_f16(y1).bits;
      kv_s[1][i] = v0;
      kv_s[1][i + 64] = v1;
      uint16_t* dst = a.kv_pool_w + kv_block_base(a.geom, a.layer, page, kvh, 1);
      dst[kv_v_offset(a.geom, tok, i)] = v0;
      dst[kv_v_offset(a.geom, tok, i + 64)] = v1;
    }
  }
  __syncthreads();

  Frag q[8];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    q[ks].u = *(const uint4*)&q_s[0][c][ks * 32 + g * 8];
    q[4 + ks].u = *(const uint4*)&q_s[1][c][ks * 32 + g * 8];
  }
  float m = -INFINITY, l = 0.f;
  f32x4 o[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int t_begin = split * a.split_tokens;
  const int t_end = min(pos, t_begin + a.split_tokens);  // cached positions only
  for (int tok0 = t_begin + wave * 32; tok0 < t_end; tok0 += 128)
    attend_group(group_block(a, slot, kvh, tok0, 0), group_block(a, slot, kvh, tok0, 1), q, tok0, pos - 1,
                 scale_log2, m, l, o, lane);
  if (owner && wave == 3) {  // the new position, from LDS: token 0 of a group that starts at pos
    Frag k[2][4], v[8];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      k[0][ks].u = make_uint4(0, 0, 0, 0);
      k[1][ks].u = make_uint4(0, 0, 0, 0);
      if (c == 0) k[0][ks].u = *(const uint4*)&kv_s[0][ks * 32 + g * 8];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      v[j].u = make_uint4(0, 0, 0, 0);
      if (g == 0) v[j].h[0] = kv_s[1][16 * j + c];
    }
    attend_frags(k, v, q, pos, pos, scale_log2, m, l, o, lane);
  }

  // merge the 4 wavefronts: common max, rescale, sum
  if (g == 0) m_s[wave][c] = m;
  __syncthreads();
  const float M = fmaxf(fmaxf(m_s[0][c], m_s[1][c]), fmaxf(m_s[2][c], m_s[3][c]));
  const float M_use = (M == -INFINITY) ? 0.f : M;
  const float w = exp2f(m - M_use);
  if (g == 0) l_s[wave][c] = l * w;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) o_s[wave][c * DH + 16 * j + 4 * g + i] = o[j][i] * w;
  __syncthreads();
  const long long pair = (long long)b * n_kv + kvh;
  const long long part = pair * a.n_splits + split;
  for (int e = tid; e < G * DH; e += 256) {
    const int col = e >> 7;
    const float acc = o_s[0][e] + o_s[1][e] + o_s[2][e] + o_s[3][e];
    if (used == 1) {
      const float L = l_s[0][col] + l_s[1][col] + l_s[2][col] + l_s[3][col];
      store1_split(a.out + out_offset(a, b, kvh * G * DH + e), a.out_lo_offset, acc / (L * P_SCALE));
    } else {
      a.part_o[part * (16 * DH) + e] = acc;
    }
  }
  if (used > 1 && tid < 16) {
    a.part_ml[part * 32 + tid] = fmaxf(fmaxf(m_s[0][tid], m_s[1][tid]), fmaxf(m_s[2][tid], m_s[3][tid]));
    a.part_ml[part * 32 + 16 + tid] = l_s[0][tid] + l_s[1][tid] + l_s[2][tid] + l_s[3][tid];
  }
}

// Merge of the KV splits of one (sample, KV head), at most 16 of them: a launch of its own,
// because a launch boundary is the cheapest way to publish results between workgroups here.
__global__ __launch_bounds__(256) void attn_merge_fused_kernel(AttnArgs a) {
  __shared__ float w_s[16][16];  // [split][column] weight 2^(m_s - M) / (L 2^10)
  const int tid = threadIdx.x, kvh = blockIdx.x, b = blockIdx.y;
  const int n_kv = a.geom.n_kv_heads;
  const int G = a.n_q_heads / n_kv;
  const int used = a.row_pos[b] / a.split_tokens + 1;
  if (used == 1) return;  // the attention kernel wrote the result itself
  const long long part0 = ((long long)b * n_kv + kvh) * a.n_splits;
  {
    const int s = tid >> 4, col = tid & 15;  // 256 threads = 16 splits x 16 columns
    const float m = s < used ? a.part_ml[(part0 + s) * 32 + col] : -INFINITY;
    const float l = s < used ? a.part_ml[(part0 + s) * 32 + 16 + col] : 0.f;
    w_s[s][col] = m;
    __syncthreads();
    float M = -INFINITY;
#pragma unroll
    for (int q = 0; q < 16; ++q) M = fmaxf(M, w_s[q][col]);
    const float w = exp2f(m - M);  // 0 for unused splits
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
  for (int e = tid; e < G * DH; e += 256) {
    const int col = e >> 7;
    float v[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) v[s] = s < used ? a.part_o[(part0 + s) * (16 * DH) + e] : 0.f;
    float acc = 0.f;
#pragma unroll
    for (int s = 0; s < 16; ++s) acc += v[s] * w_s[s][col];
    store1_split(a.out + out_offset(a, b, kvh * G * DH + e), a.out_lo_offset, acc);
  }
}

void launch_attention_decode_fused(const AttnArgs& a, hipStream_t s) {
  if (!a.rows) return;
  const dim3 grid(a.n_splits, a.geom.n_kv_heads, a.rows);
  if (a.extra.bias || a.extra.q_gain) attn_decode_fused_kernel<true><<<grid, 256, 0, s>>>(a);
  else attn_decode_fused_kernel<false><<<grid, 256, 0, s>>>(a);
  if (a.n_splits > 1) attn_merge_fused_kernel<<<dim3(a.geom.n_kv_heads, a.rows), 256, 0, s>>>(a);
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
