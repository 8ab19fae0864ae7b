// Paged grouped-query attention on the matrix cores, head_dim 128, bf16 KV pages in the
// KV_MATRIX element order (common.h).
//
// Decoding is memory-bound (paper section 2.1) and its attention streams every cached key
// and value once per step, so the kernels are built around that stream: each wavefront
// takes 32 cached positions at a time as sixteen contiguous 1 KiB loads (8 key fragments,
// 8 value fragments), computes transposed scores S^T = K q^T with 16x16x32 bf16 matrix
// instructions (columns = the query rows that share the KV head), runs the online softmax
// on the fragment (per-column max and sum are a register reduction plus two cross-lane
// steps), and feeds the probabilities straight back as the B operand of O^T += V^T P^T.
// The value pages are stored in exactly the k-order in which a score fragment holds its
// probabilities, so P never moves between lanes.
//
//   decode  : one workgroup per (KV split, KV head, sample); columns = the G query heads;
//             its 4 wavefronts interleave over the split's 32-position groups and merge
//             through LDS; several splits per sample merge in a second small kernel.
//   prefill : one wavefront per (16 query positions, query head); columns = positions;
//             causal limit per column.
#include "kernels_fast.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
union Frag {
  uint4 u;
  bf16x8 v;
  uint16_t h[8];
};

#define DH 128
#define GROUP_U4 512  // uint4 per 32-position group of one K (or V) block: 32 * 128 * 2 / 16

// One 32-position group against this lane's query column.  limit = last visible position
// of the column.  m, l in log2 units; o = unnormalised output^T fragments.
__device__ inline void attend_group(const uint4* __restrict__ kblk, const uint4* __restrict__ vblk,
                                    const Frag (&q)[4], int tok0, int limit, float scale_log2, float& m,
                                    float& l, f32x4 (&o)[8], int lane) {
  const int g = lane >> 4;
  Frag k[2][4], v[8];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) k[t][ks].u = kblk[(t * 4 + ks) * 64 + lane];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j].u = vblk[j * 64 + lane];
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[0][ks].v, q[ks].v, s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[1][ks].v, q[ks].v, s1, 0, 0, 0);
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
  Frag pb;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float p = exp2f(sc[e] - m_use);
    ps += p;
    pb.h[e] = f32_to_bf16(p).bits;
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
    o[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v[j].v, pb.v, o[j], 0, 0, 0);
  }
}

__device__ inline const uint4* group_block(const AttnArgs& a, int slot, int kv_head, int tok0, int is_v) {
  const int page = a.page_table[(long long)slot * a.max_pages + tok0 / a.geom.page_tokens];
  const int gip = (tok0 % a.geom.page_tokens) >> 5;
  return (const uint4*)(a.kv_pool + kv_block_base(a.geom, a.layer, page, kv_head, is_v)) + gip * GROUP_U4;
}

__device__ inline uint2 pack4_bf16(float a, float b, float c, float d) {
  return make_uint2((uint32_t)f32_to_bf16(a).bits | ((uint32_t)f32_to_bf16(b).bits << 16),
                    (uint32_t)f32_to_bf16(c).bits | ((uint32_t)f32_to_bf16(d).bits << 16));
}

// ------------------------------------------------------------------------------ decode
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnArgs a) {
  __shared__ float m_s[4][16];
  __shared__ float l_s[4][16];
  __shared__ float o_s[4][16 * DH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int G = a.n_q_heads / a.geom.n_kv_heads;
  const int ctx = a.row_pos[b] + 1;
  const int slot = a.row_slot[b];
  const int t_begin = split * a.split_tokens;
  const int t_end = min(ctx, t_begin + a.split_tokens);
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);

  Frag q[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    q[ks].u = make_uint4(0, 0, 0, 0);
    if (c < G) q[ks].u = *(const uint4*)(a.q + ((long long)b * a.n_q_heads + kvh * G + c) * DH + ks * 32 + g * 8);
  }
  float m = -INFINITY, l = 0.f;
  f32x4 o[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int tok0 = t_begin + wave * 32; tok0 < t_end; tok0 += 128)
    attend_group(group_block(a, slot, kvh, tok0, 0), group_block(a, slot, kvh, tok0, 1), q, tok0, ctx - 1,
                 scale_log2, m, l, o, lane);

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
  const long long part = ((long long)b * a.geom.n_kv_heads + kvh) * a.n_splits + split;
  for (int e = threadIdx.x; e < 16 * DH; e += 256) {
    const int col = e >> 7, dim = e & 127;
    if (col >= G) continue;
    const float acc = o_s[0][e] + o_s[1][e] + o_s[2][e] + o_s[3][e];
    if (a.n_splits == 1) {
      const float L = l_s[0][col] + l_s[1][col] + l_s[2][col] + l_s[3][col];
      a.out[((long long)b * a.n_q_heads + kvh * G + col) * DH + dim] = f32_to_bf16(acc / L).bits;
    } else {
      a.part_o[part * (16 * DH) + e] = acc;
    }
  }
  if (a.n_splits > 1 && threadIdx.x < 16) {
    const int col = threadIdx.x;
    a.part_ml[part * 32 + col] = fmaxf(fmaxf(m_s[0][col], m_s[1][col]), fmaxf(m_s[2][col], m_s[3][col]));
    a.part_ml[part * 32 + 16 + col] = l_s[0][col] + l_s[1][col] + l_s[2][col] + l_s[3][col];
  }
}

__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a) {
  const int kvh = blockIdx.x, b = blockIdx.y;
  const int G = a.n_q_heads / a.geom.n_kv_heads;
  const long long part0 = ((long long)b * a.geom.n_kv_heads + kvh) * a.n_splits;
  const int ctx = a.row_pos[b] + 1;
  const int used = min(a.n_splits, (ctx + a.split_tokens - 1) / a.split_tokens);
  for (int e = threadIdx.x; e < G * DH; e += 256) {
    const int col = e >> 7;
    float M = -INFINITY;
    for (int s = 0; s < used; ++s) M = fmaxf(M, a.part_ml[(part0 + s) * 32 + col]);
    float L = 0.f, acc = 0.f;
    for (int s = 0; s < used; ++s) {
      const float w = exp2f(a.part_ml[(part0 + s) * 32 + col] - M);
      L += a.part_ml[(part0 + s) * 32 + 16 + col] * w;
      acc += a.part_o[(part0 + s) * (16 * DH) + e] * w;
    }
    a.out[((long long)b * a.n_q_heads + kvh * G) * DH + e] = f32_to_bf16(acc / L).bits;
  }
}

void launch_attention_decode(const AttnArgs& a, hipStream_t s) {
  if (!a.rows) return;
  attn_decode_kernel<<<dim3(a.n_splits, a.geom.n_kv_heads, a.rows), 256, 0, s>>>(a);
  if (a.n_splits > 1) attn_merge_kernel<<<dim3(a.geom.n_kv_heads, a.rows), 256, 0, s>>>(a);
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
  const int kvh = head / (a.n_q_heads / a.geom.n_kv_heads);
  const int pos = q0 + c;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
  Frag q[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    q[ks].u = make_uint4(0, 0, 0, 0);
    if (pos < len) q[ks].u = *(const uint4*)(a.q + ((long long)(row0 + pos) * a.n_q_heads + head) * DH + ks * 32 + g * 8);
  }
  float m = -INFINITY, l = 0.f;
  f32x4 o[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int last = min(q0 + 15, len - 1);
  for (int tok0 = 0; tok0 <= last; tok0 += 32)
    attend_group(group_block(a, slot, kvh, tok0, 0), group_block(a, slot, kvh, tok0, 1), q, tok0, pos, scale_log2,
                 m, l, o, lane);
  if (pos < len) {
    uint16_t* dst = a.out + ((long long)(row0 + pos) * a.n_q_heads + head) * DH + 4 * g;
    const float inv = 1.0f / l;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      *(uint2*)(dst + 16 * j) = pack4_bf16(o[j][0] * inv, o[j][1] * inv, o[j][2] * inv, o[j][3] * inv);
  }
}

void launch_attention_prefill(const AttnArgs& a, hipStream_t s) {
  if (!a.n_seqs) return;
  attn_prefill_kernel<<<dim3(ceil_div(a.max_seq_len, 64), a.n_q_heads, a.n_seqs), 256, 0, s>>>(a);
}
