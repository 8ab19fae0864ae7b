// Fused per-row kernels of the matrix-core path: residual add + RMSNorm + bf16 cast (with
// optional embedding gather), and split-K reduction + rotary embedding + KV-page write.
// The residual stream stays fp32; only projection inputs and the KV cache are bf16.
#include "kernels_fast.h"

#define ROW_T 256
#define ROW_MAX_PER_THREAD 32  // hidden <= 8192

__global__ __launch_bounds__(ROW_T) void row_norm_kernel(RowNormArgs a) {
  __shared__ float partial[ROW_T / WAVE];
  const int r = blockIdx.x, t = threadIdx.x;
  const long long src_row = a.rows_index ? a.rows_index[r] : r;
  float v[ROW_MAX_PER_THREAD];
  float ss = 0.f;
  const int n_per = (a.hidden + ROW_T - 1) / ROW_T;
#pragma unroll
  for (int j = 0; j < ROW_MAX_PER_THREAD; ++j) {
    if (j >= n_per) break;
    int i = t + j * ROW_T;
    float x = 0.f;
    if (i < a.hidden) {
      if (a.tokens) {
        bf16_t e;
        e.bits = a.embed[(long long)a.tokens[r] * a.hidden + i];
        x = bf16_to_f32(e);
      } else {
        x = a.x[src_row * a.hidden + i];
      }
      for (int z = 0; z < a.splits; ++z) x += a.partial[z * a.split_stride + (long long)r * a.hidden + i];
    }
    v[j] = x;
    ss += x * x;
  }
  ss = wave_sum(ss);
  if ((t & 63) == 0) partial[t >> 6] = ss;
  __syncthreads();
  float total = 0.f;
#pragma unroll
  for (int w = 0; w < ROW_T / WAVE; ++w) total += partial[w];
  const float rinv = 1.0f / sqrtf(total / (float)a.hidden + a.eps);
#pragma unroll
  for (int j = 0; j < ROW_MAX_PER_THREAD; ++j) {
    if (j >= n_per) break;
    int i = t + j * ROW_T;
    if (i < a.hidden) {
      if (!a.rows_index && (a.splits || a.tokens)) a.x[(long long)r * a.hidden + i] = v[j];
      a.h[(long long)r * a.hidden + i] = f32_to_bf16(v[j] * a.gain[i] * rinv).bits;
    }
  }
}
void launch_row_norm(const RowNormArgs& a, hipStream_t s) {
  if (a.rows) row_norm_kernel<<<a.rows, ROW_T, 0, s>>>(a);
}

__global__ void qkv_post_kernel(QkvPostArgs a) {
  const int r = blockIdx.x;
  const KvGeom& g = a.geom;
  const int dh = g.head_dim, half = dh >> 1;
  const int n_heads = a.n_q_heads + 2 * g.n_kv_heads;
  const int pos = a.row_pos[r];
  const int page = a.page_table[(long long)a.row_slot[r] * a.max_pages + pos / g.page_tokens];
  const int tok = pos % g.page_tokens;
  const float* cs = a.cos_sin + (long long)pos * dh;
  const long long row_off = (long long)r * n_heads * dh;
  for (int idx = threadIdx.x; idx < n_heads * half; idx += blockDim.x) {
    int head = idx / half, i = idx % half;
    float u = 0.f, w = 0.f;
    for (int z = 0; z < a.splits; ++z) {
      const float* p = a.partial + z * a.split_stride + row_off + head * dh;
      u += p[i];
      w += p[i + half];
    }
    if (head < a.n_q_heads + g.n_kv_heads) {
      float c = cs[2 * i], sn = cs[2 * i + 1];
      float ru = u * c - w * sn, rw = w * c + u * sn;
      u = ru;
      w = rw;
    }
    if (head < a.n_q_heads) {
      long long o = ((long long)r * a.n_q_heads + head) * dh;
      a.q_bf16[o + i] = f32_to_bf16(u).bits;
      a.q_bf16[o + i + half] = f32_to_bf16(w).bits;
      if (a.q_f32) {
        a.q_f32[(long long)r * a.q_f32_ld + head * dh + i] = u;
        a.q_f32[(long long)r * a.q_f32_ld + head * dh + i + half] = w;
      }
    } else {
      int is_v = head >= a.n_q_heads + g.n_kv_heads;
      int kvh = head - a.n_q_heads - (is_v ? g.n_kv_heads : 0);
      uint16_t* dst = a.kv_pool + kv_block_base(g, a.layer, page, kvh, is_v);
      if (is_v) {
        dst[kv_v_offset(g, tok, i)] = f32_to_bf16(u).bits;
        dst[kv_v_offset(g, tok, i + half)] = f32_to_bf16(w).bits;
      } else {
        dst[kv_k_offset(g, tok, i)] = f32_to_bf16(u).bits;
        dst[kv_k_offset(g, tok, i + half)] = f32_to_bf16(w).bits;
      }
    }
  }
}
void launch_qkv_post(const QkvPostArgs& a, hipStream_t s) {
  if (a.rows) qkv_post_kernel<<<a.rows, 256, 0, s>>>(a);
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, uint16_t* __restrict__ dst, long long n) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = f32_to_bf16(src[i]).bits;
}
void launch_f32_to_bf16(const float* src, uint16_t* dst, long long n, hipStream_t s) {
  if (n) f32_to_bf16_kernel<<<ceil_div(n, 256), 256, 0, s>>>(src, dst, n);
}
