// Fused per-row kernels of the matrix-core path: residual add + RMSNorm + bf16 cast (with
// optional embedding gather), and split-K reduction + rotary embedding + KV-page write.
// The residual stream stays fp32; only projection inputs and the KV cache are bf16.
#include "kernels_fast.h"

#define ROW_T 256

// One workgroup per row; thread t holds the row's float4 chunks t, t + 256, ... (V of them) in
// registers, so every load of the row is in flight before the first use (hidden <= 1024 V).
template <int V>
__global__ __launch_bounds__(ROW_T) void row_norm_kernel(RowNormArgs a) {
  __shared__ float partial[ROW_T / WAVE];
  const int r = blockIdx.x, t = threadIdx.x;
  const int n4 = a.hidden >> 2;
  const long long src_row = a.rows_index ? a.rows_index[r] : r;
  float4 x[V];
  if (a.tokens) {
    const uint2* e = (const uint2*)(a.embed + (long long)a.tokens[r] * a.hidden);
#pragma unroll
    for (int v = 0; v < V; ++v) {
      const int c = t + ROW_T * v;
      uint2 u = make_uint2(0, 0);
      if (c < n4) u = e[c];
      x[v] = make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                         __uint_as_float(u.y & 0xffff0000u));
    }
  } else {
    const float4* xs = (const float4*)(a.x + src_row * a.hidden);
#pragma unroll
    for (int v = 0; v < V; ++v) {
      const int c = t + ROW_T * v;
      x[v] = c < n4 ? xs[c] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  // the gain is not needed before the end: requested now, it arrives with the row
  float4 gn[V];
#pragma unroll
  for (int v = 0; v < V; ++v) {
    const int c = t + ROW_T * v;
    gn[v] = c < n4 ? ((const float4*)a.gain)[c] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  // split planes, added in ascending order; the loads of four planes are issued together (a
  // projection with a deep K leaves up to 16 planes: two at a time were eight round trips)
  for (int z = 0; z < a.splits; z += 4) {
    float4 u[4][V];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4* pz = (const float4*)(a.partial + (long long)(z + q) * a.split_stride + (long long)r * a.hidden);
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const int c = t + ROW_T * v;
        u[q][v] = (z + q < a.splits && c < n4) ? pz[c] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int v = 0; v < V; ++v) {
        x[v].x += u[q][v].x;
        x[v].y += u[q][v].y;
        x[v].z += u[q][v].z;
        x[v].w += u[q][v].w;
      }
  }
  for (int j = 0; j < a.moe_k; ++j) {  // the row's expert picks, in pick order
    const float wt = a.moe_wt[(long long)r * a.moe_k + j];
    const float4* y = (const float4*)(a.moe_y + (long long)a.moe_slot[(long long)r * a.moe_k + j] * a.hidden);
#pragma unroll
    for (int v = 0; v < V; ++v) {
      const int c = t + ROW_T * v;
      if (c < n4) {
        const float4 yv = y[c];
        x[v].x += wt * yv.x;
        x[v].y += wt * yv.y;
        x[v].z += wt * yv.z;
        x[v].w += wt * yv.w;
      }
    }
  }
  float ss = 0.f;
#pragma unroll
  for (int v = 0; v < V; ++v) ss += x[v].x * x[v].x + x[v].y * x[v].y + x[v].z * x[v].z + x[v].w * x[v].w;
  ss = wave_sum(ss);
  if ((t & 63) == 0) partial[t >> 6] = ss;
  __syncthreads();
  float total = 0.f;
#pragma unroll
  for (int w = 0; w < ROW_T / WAVE; ++w) total += partial[w];
  const float rinv = a.ssq_out ? 1.0f : 1.0f / sqrtf(total / (float)a.hidden + a.eps);
  if (a.ssq_out && t == 0) a.ssq_out[r] = total;
  const bool write_x = !a.rows_index && (a.splits || a.tokens || a.moe_k);
#pragma unroll
  for (int v = 0; v < V; ++v) {
    const int c = t + ROW_T * v;
    if (c >= n4) continue;
    if (write_x) ((float4*)(a.x + (long long)r * a.hidden))[c] = x[v];
    uint16_t hi[4], lo[4];
    split_bf16(x[v].x * gn[v].x * rinv, hi[0], lo[0]);
    split_bf16(x[v].y * gn[v].y * rinv, hi[1], lo[1]);
    split_bf16(x[v].z * gn[v].z * rinv, hi[2], lo[2]);
    split_bf16(x[v].w * gn[v].w * rinv, hi[3], lo[3]);
    uint16_t* hp = a.h + (a.h_frag ? frag_offset(r, 4 * c, a.hidden >> 5) : (long long)r * a.hidden + 4 * c);
    *(uint2*)hp = make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
    *(uint2*)(hp + a.h_lo_offset) =
        make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
  }
}
void launch_row_norm(const RowNormArgs& a, hipStream_t s) {
  if (!a.rows) return;
  const int chunks = ceil_div(a.hidden >> 2, ROW_T);  // hidden is a multiple of 32 and at most 8192
  if (chunks <= 1) row_norm_kernel<1><<<a.rows, ROW_T, 0, s>>>(a);
  else if (chunks <= 2) row_norm_kernel<2><<<a.rows, ROW_T, 0, s>>>(a);
  else if (chunks <= 4) row_norm_kernel<4><<<a.rows, ROW_T, 0, s>>>(a);
  else row_norm_kernel<8><<<a.rows, ROW_T, 0, s>>>(a);
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
  // bias and per-head norm: this launch runs with head_dim 128, a wavefront per head
  if (a.extra.bias || a.extra.q_gain)
    qkv_extras(a.extra, head * dh, i,
               head < a.n_q_heads ? a.extra.q_gain : head < a.n_q_heads + g.n_kv_heads ? a.extra.k_gain : nullptr, u, w);
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
