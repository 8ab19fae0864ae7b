// Fused per-row kernels of the matrix-core path: residual add + RMSNorm + bf16 cast (with
// optional embedding gather), and split-K reduction + rotary embedding + KV-page write.
// The residual stream stays fp32; only projection inputs and the KV cache are bf16.
#include "kernels_fast.h"

#define ROW_T 256

// One workgroup per row; the row is staged in LDS between the two passes (hidden <= 8192).
__global__ __launch_bounds__(ROW_T) void row_norm_kernel(RowNormArgs a) {
  __shared__ float row_s[8192];
  __shared__ float partial[ROW_T / WAVE];
  const int r = blockIdx.x, t = threadIdx.x;
  const long long src_row = a.rows_index ? a.rows_index[r] : r;
  const long long tok = a.tokens ? a.tokens[r] : 0;
  float ss = 0.f;
  for (int i = t; i < a.hidden; i += ROW_T) {
    float x;
    if (a.tokens) {
      bf16_t e;
      e.bits = a.embed[tok * a.hidden + i];
      x = bf16_to_f32(e);
    } else {
      x = a.x[src_row * a.hidden + i];
    }
    const float* pp = a.partial + (long long)r * a.hidden + i;
    for (int z = 0; z < a.splits; z += 4) {  // four planes at a time, loads issued together
      float p0 = pp[(long long)z * a.split_stride], p1 = 0.f, p2 = 0.f, p3 = 0.f;
      if (z + 1 < a.splits) p1 = pp[(long long)(z + 1) * a.split_stride];
      if (z + 2 < a.splits) p2 = pp[(long long)(z + 2) * a.split_stride];
      if (z + 3 < a.splits) p3 = pp[(long long)(z + 3) * a.split_stride];
      x = (((x + p0) + p1) + p2) + p3;
    }
    for (int j = 0; j < a.moe_k; ++j)
      x += a.moe_wt[(long long)r * a.moe_k + j] *
           a.moe_y[(long long)a.moe_slot[(long long)r * a.moe_k + j] * a.hidden + i];
    row_s[i] = x;
    ss += x * x;
  }
  ss = wave_sum(ss);
  if ((t & 63) == 0) partial[t >> 6] = ss;
  __syncthreads();
  float total = 0.f;
#pragma unroll
  for (int w = 0; w < ROW_T / WAVE; ++w) total += partial[w];
  const float rinv = a.ssq_out ? 1.0f : 1.0f / sqrtf(total / (float)a.hidden + a.eps);
  if (a.ssq_out && t == 0) a.ssq_out[r] = total;
  const bool write_x = !a.rows_index && (a.splits || a.tokens || a.moe_k);
  for (int i = t; i < a.hidden; i += ROW_T) {
    const float x = row_s[i];
    if (write_x) a.x[(long long)r * a.hidden + i] = x;
    uint16_t hi, lo;
    split_bf16(x * a.gain[i] * rinv, hi, lo);
    a.h[(long long)r * a.hidden + i] = hi;
    a.h[a.h_lo_offset + (long long)r * a.hidden + i] = lo;
  }
}
void launch_row_norm(const RowNormArgs& a, hipStream_t s) {
  if (a.rows) row_norm_kernel<<<a.rows, ROW_T, 0, s>>>(a);
}

// One thread per rotary pair (head, i): grid (rows, heads / 4), 4 heads of 64 pairs per block.
__global__ __launch_bounds__(256) void qkv_post_kernel(QkvPostArgs a) {
  const int r = blockIdx.x;
  const KvGeom& g = a.geom;
  const int dh = g.head_dim, half = dh >> 1;
  const int n_heads = a.n_q_heads + 2 * g.n_kv_heads;
  const int per_block = 256 / half;  // heads per block
  const int head = blockIdx.y * per_block + threadIdx.x / half, i = threadIdx.x % half;
  if (head >= n_heads) return;
  const int pos = a.row_pos[r];
  const long long row_off = (long long)r * n_heads * dh + head * dh;
  const float* p = a.partial + row_off;
  float u = 0.f, w = 0.f;
  for (int z = 0; z < a.splits; z += 4) {  // four planes at a time, loads issued together
    const float* q = p + (long long)z * a.split_stride;
    float u0 = q[i], w0 = q[i + half], u1 = 0.f, u2 = 0.f, u3 = 0.f, w1 = 0.f, w2 = 0.f, w3 = 0.f;
    if (z + 1 < a.splits) { u1 = q[a.split_stride + i]; w1 = q[a.split_stride + i + half]; }
    if (z + 2 < a.splits) { u2 = q[2 * a.split_stride + i]; w2 = q[2 * a.split_stride + i + half]; }
    if (z + 3 < a.splits) { u3 = q[3 * a.split_stride + i]; w3 = q[3 * a.split_stride + i + half]; }
    u = (((u + u0) + u1) + u2) + u3;
    w = (((w + w0) + w1) + w2) + w3;
  }
  if (head < a.n_q_heads + g.n_kv_heads) {
    const float* cs = a.cos_sin + (long long)pos * dh;
    float c = cs[2 * i], sn = cs[2 * i + 1];
    float ru = u * c - w * sn, rw = w * c + u * sn;
    u = ru;
    w = rw;
  }
  if (head < a.n_q_heads) {
    long long o = ((long long)r * a.n_q_heads + head) * dh;
    uint16_t hi, lo;  // the attention kernels multiply q with half-precision keys
    split_f16(u, hi, lo);
    a.q_bf16[o + i] = hi;
    a.q_bf16[a.q_lo_offset + o + i] = lo;
    split_f16(w, hi, lo);
    a.q_bf16[o + i + half] = hi;
    a.q_bf16[a.q_lo_offset + o + i + half] = lo;
    if (a.q_f32) {
      a.q_f32[(long long)r * a.q_f32_ld + head * dh + i] = u;
      a.q_f32[(long long)r * a.q_f32_ld + head * dh + i + half] = w;
    }
  } else {
    const int page = a.page_table[(long long)a.row_slot[r] * a.max_pages + pos / g.page_tokens];
    const int tok = pos % g.page_tokens;
    int is_v = head >= a.n_q_heads + g.n_kv_heads;
    int kvh = head - a.n_q_heads - (is_v ? g.n_kv_heads : 0);
    uint16_t* dst = a.kv_pool + kv_block_base(g, a.layer, page, kvh, is_v);
    if (is_v) {
      dst[kv_v_offset(g, tok, i)] = f32_to_f16(u).bits;
      dst[kv_v_offset(g, tok, i + half)] = f32_to_f16(w).bits;
    } else {
      dst[kv_k_offset(g, tok, i)] = f32_to_f16(u).bits;
      dst[kv_k_offset(g, tok, i + half)] = f32_to_f16(w).bits;
    }
  }
}
void launch_qkv_post(const QkvPostArgs& a, hipStream_t s) {
  if (!a.rows) return;
  const int per_block = 256 / (a.geom.head_dim / 2);
  const int n_heads = a.n_q_heads + 2 * a.geom.n_kv_heads;
  qkv_post_kernel<<<dim3(a.rows, ceil_div(n_heads, per_block)), 256, 0, s>>>(a);
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, uint16_t* __restrict__ dst, long long n) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = f32_to_bf16(src[i]).bits;
}
void launch_f32_to_bf16(const float* src, uint16_t* dst, long long n, hipStream_t s) {
  if (n) f32_to_bf16_kernel<<<ceil_div(n, 256), 256, 0, s>>>(src, dst, n);
}
