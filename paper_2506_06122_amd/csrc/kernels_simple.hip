// Plain one-operator-per-kernel path: fp32 activations, weights and KV cache in any
// storage type.  It serves fp32 models and cross-checks the matrix-core path; clarity
// over speed.  Operators: paper section 2.1 names the phases (prefill, decoding); the
// operator definitions are the standard ones of the model families in section 5.1.
#include "kernels.h"

// ---------------------------------------------------------------- embedding
template <typename T>
__global__ void embed_kernel(const T* __restrict__ table, const int* __restrict__ tokens,
                             float* __restrict__ x, int hidden) {
  int r = blockIdx.x;
  const T* src = table + (long long)tokens[r] * hidden;
  for (int i = threadIdx.x; i < hidden; i += blockDim.x) x[(long long)r * hidden + i] = to_f32(src[i]);
}
template <typename T>
void launch_embed(const T* table, const int* tokens, float* x, int rows, int hidden, hipStream_t s) {
  if (rows) embed_kernel<T><<<rows, 256, 0, s>>>(table, tokens, x, hidden);
}
template void launch_embed<float>(const float*, const int*, float*, int, int, hipStream_t);
template void launch_embed<bf16_t>(const bf16_t*, const int*, float*, int, int, hipStream_t);

// ---------------------------------------------------------------- RMSNorm
__global__ void rmsnorm_f32_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                   float* __restrict__ out, const int* __restrict__ rows_index, int hidden,
                                   float eps) {
  __shared__ float partial[4];
  int r = blockIdx.x;
  const float* src = x + (long long)(rows_index ? rows_index[r] : r) * hidden;
  float ss = 0.f;
  for (int i = threadIdx.x; i < hidden; i += blockDim.x) ss += src[i] * src[i];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) partial[threadIdx.x >> 6] = ss;
  __syncthreads();
  float total = partial[0] + partial[1] + partial[2] + partial[3];
  float rinv = 1.0f / sqrtf(total / (float)hidden + eps);
  for (int i = threadIdx.x; i < hidden; i += blockDim.x)
    out[(long long)r * hidden + i] = src[i] * gain[i] * rinv;
}
void launch_rmsnorm_f32(const float* x, const float* gain, float* out, const int* rows_index, int rows,
                        int hidden, float eps, hipStream_t s) {
  if (rows) rmsnorm_f32_kernel<<<rows, 256, 0, s>>>(x, gain, out, rows_index, hidden, eps);
}

// ---------------------------------------------------------------- linear
// One wavefront per output column and tile of LIN_ROWS rows: lanes stride over k.
#define LIN_ROWS 8
template <typename T>
__global__ void linear_simple_kernel(const float* __restrict__ a, int lda, const T* __restrict__ w,
                                     float* out, int ldo, const float* residual, int ldr, int M, int N,
                                     int K) {  // out may alias residual (in-place residual add)
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int n = blockIdx.x * 4 + wave;
  int m0 = blockIdx.y * LIN_ROWS;
  if (n >= N) return;
  float acc[LIN_ROWS];
#pragma unroll
  for (int i = 0; i < LIN_ROWS; ++i) acc[i] = 0.f;
  const T* wr = w + (long long)n * K;
  for (int k = lane; k < K; k += WAVE) {
    float wv = to_f32(wr[k]);
#pragma unroll
    for (int i = 0; i < LIN_ROWS; ++i)
      if (m0 + i < M) acc[i] += a[(long long)(m0 + i) * lda + k] * wv;
  }
#pragma unroll
  for (int i = 0; i < LIN_ROWS; ++i) {
    float v = wave_sum(acc[i]);
    if (lane == 0 && m0 + i < M) {
      if (residual) v += residual[(long long)(m0 + i) * ldr + n];
      out[(long long)(m0 + i) * ldo + n] = v;
    }
  }
}
template <typename T>
void launch_linear_simple(const float* a, int lda, const T* w, float* out, int ldo, const float* residual,
                          int ldr, int M, int N, int K, hipStream_t s) {
  if (!M || !N) return;
  dim3 grid(ceil_div(N, 4), ceil_div(M, LIN_ROWS));
  linear_simple_kernel<T><<<grid, 256, 0, s>>>(a, lda, w, out, ldo, residual, ldr, M, N, K);
}
template void launch_linear_simple<float>(const float*, int, const float*, float*, int, const float*, int, int,
                                          int, int, hipStream_t);
template void launch_linear_simple<bf16_t>(const float*, int, const bf16_t*, float*, int, const float*, int,
                                           int, int, int, hipStream_t);

// ---------------------------------------------------------------- q/k/v bias and per-head norm
// One wavefront per (row, head) of the fused [q | k | v] rows, in place: adds the bias, then
// normalises q and k heads over head_dim with their gains (either part may be absent).
__global__ void qkv_bias_norm_kernel(float* __restrict__ qkv, const float* __restrict__ bias,
                                     const float* __restrict__ q_gain, const float* __restrict__ k_gain, float eps,
                                     int n_q_heads, int n_kv_heads, int dh) {
  const int r = blockIdx.x, head = blockIdx.y * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int n_heads = n_q_heads + 2 * n_kv_heads;
  if (head >= n_heads) return;
  float* x = qkv + ((long long)r * n_heads + head) * dh;
  float ss = 0.f;
  for (int i = lane; i < dh; i += 64) {
    const float v = x[i] + (bias ? bias[head * dh + i] : 0.f);
    x[i] = v;
    ss += v * v;
  }
  const float* gain = head < n_q_heads ? q_gain : head < n_q_heads + n_kv_heads ? k_gain : nullptr;
  if (!gain) return;
  const float rinv = 1.0f / sqrtf(wave_sum(ss) / (float)dh + eps);
  for (int i = lane; i < dh; i += 64) x[i] *= rinv * gain[i];
}
void launch_qkv_bias_norm(float* qkv, const float* bias, const float* q_gain, const float* k_gain, float eps,
                          int rows, int n_q_heads, int n_kv_heads, int dh, hipStream_t s) {
  if (rows && (bias || q_gain))
    qkv_bias_norm_kernel<<<dim3(rows, ceil_div(n_q_heads + 2 * n_kv_heads, 4)), 256, 0, s>>>(
        qkv, bias, q_gain, k_gain, eps, n_q_heads, n_kv_heads, dh);
}

// ---------------------------------------------------------------- RoPE + KV write
// qkv row = [q heads | k heads | v heads] x head_dim.  Half-split pairing: (u_i, u_{i+dh/2})
// rotates by pos * theta^(-2i/dh); cos_sin[pos][i] = (cos, sin) interleaved.
template <typename KT>
__global__ void rope_kvwrite_kernel(float* __restrict__ qkv, const float* __restrict__ cos_sin,
                                    const int* __restrict__ row_pos, const int* __restrict__ row_slot,
                                    const int* __restrict__ page_table, int max_pages, KT* __restrict__ kv_pool,
                                    KvGeom g, int layer, int n_q_heads) {
  int r = blockIdx.x;
  int dh = g.head_dim, half = dh >> 1;
  int pos = row_pos[r];
  int n_heads = n_q_heads + 2 * g.n_kv_heads;
  float* row = qkv + (long long)r * n_heads * dh;
  int page = page_table[(long long)row_slot[r] * max_pages + pos / g.page_tokens];
  int tok = pos % g.page_tokens;
  const float* cs = cos_sin + (long long)pos * dh;  // half pairs of (cos, sin)
  for (int idx = threadIdx.x; idx < n_heads * half; idx += blockDim.x) {
    int head = idx / half, i = idx % half;
    float a = row[head * dh + i], b = row[head * dh + i + half];
    if (head < n_q_heads + g.n_kv_heads) {
      float c = cs[2 * i], sn = cs[2 * i + 1];
      float ra = a * c - b * sn, rb = b * c + a * sn;
      a = ra;
      b = rb;
    }
    if (head < n_q_heads) {
      row[head * dh + i] = a;
      row[head * dh + i + half] = b;
    } else if (head < n_q_heads + g.n_kv_heads) {
      int kvh = head - n_q_heads;
      KT* dst = kv_pool + kv_block_base(g, layer, page, kvh, 0);
      dst[kv_k_offset(g, tok, i)] = from_f32<KT>(a);
      dst[kv_k_offset(g, tok, i + half)] = from_f32<KT>(b);
    } else {
      int kvh = head - n_q_heads - g.n_kv_heads;
      KT* dst = kv_pool + kv_block_base(g, layer, page, kvh, 1);
      dst[kv_v_offset(g, tok, i)] = from_f32<KT>(a);
      dst[kv_v_offset(g, tok, i + half)] = from_f32<KT>(b);
    }
  }
}
template <typename KT>
void launch_rope_kvwrite(float* qkv, const float* cos_sin, const int* row_pos, const int* row_slot,
                         const int* page_table, int max_pages, KT* kv_pool, KvGeom geom, int layer, int rows,
                         int n_q_heads, hipStream_t s) {
  if (rows)
    rope_kvwrite_kernel<KT><<<rows, 256, 0, s>>>(qkv, cos_sin, row_pos, row_slot, page_table, max_pages,
                                                   kv_pool, geom, layer, n_q_heads);
}
template void launch_rope_kvwrite<float>(float*, const float*, const int*, const int*, const int*, int, float*,
                                         KvGeom, int, int, int, hipStream_t);
template void launch_rope_kvwrite<f16_t>(float*, const float*, const int*, const int*, const int*, int, f16_t*,
                                         KvGeom, int, int, int, hipStream_t);

// ---------------------------------------------------------------- attention
// One block of ATT_T threads per (row, query head).  Cached positions are taken ATT_T at a
// time: thread t scores position base + t, the block updates the running max and sum
// (online softmax), then thread i accumulates output dimension i.
#define ATT_T 128
template <typename KT>
__global__ void attention_simple_kernel(const float* __restrict__ qkv, float* __restrict__ out,
                                        const int* __restrict__ row_pos, const int* __restrict__ row_slot,
                                        const int* __restrict__ page_table, int max_pages,
                                        const KT* __restrict__ kv_pool, KvGeom g, int layer, int n_q_heads) {
  __shared__ float q_s[256];
  __shared__ float p_s[ATT_T];
  __shared__ float red[2];
  int r = blockIdx.x, head = blockIdx.y, t = threadIdx.x;
  int dh = g.head_dim;
  int kvh = head / (n_q_heads / g.n_kv_heads);
  int n_heads = n_q_heads + 2 * g.n_kv_heads;
  int ctx = row_pos[r] + 1;
  const int* pages = page_table + (long long)row_slot[r] * max_pages;
  float scale = 1.0f / sqrtf((float)dh);
  for (int i = t; i < dh; i += ATT_T) q_s[i] = qkv[((long long)r * n_heads + head) * dh + i];
  __syncthreads();
  float m = -INFINITY, l = 0.f, acc0 = 0.f, acc1 = 0.f;  // thread t owns dims t and t + ATT_T
  for (int base = 0; base < ctx; base += ATT_T) {
    int u = base + t;
    float sc = -INFINITY;
    if (u < ctx) {
      const KT* kb = kv_pool + kv_block_base(g, layer, pages[u / g.page_tokens], kvh, 0);
      int tok = u % g.page_tokens;
      float dot = 0.f;
      for (int i = 0; i < dh; ++i) dot += q_s[i] * to_f32(kb[kv_k_offset(g, tok, i)]);
      sc = dot * scale;
    }
    float cm = wave_max(sc);
    if ((t & 63) == 0) red[t >> 6] = cm;
    __syncthreads();
    float m_new = fmaxf(m, fmaxf(red[0], red[1]));
    __syncthreads();
    float p = (u < ctx) ? expf(sc - m_new) : 0.f;
    p_s[t] = p;
    float ps = wave_sum(p);
    if ((t & 63) == 0) red[t >> 6] = ps;
    __syncthreads();
    float alpha = expf(m - m_new);  // m = -inf on the first chunk gives 0
    l = l * alpha + red[0] + red[1];
    acc0 *= alpha;
    acc1 *= alpha;
    int n_here = min(ATT_T, ctx - base);
    for (int j = 0; j < n_here; ++j) {
      int uu = base + j;
      const KT* vb = kv_pool + kv_block_base(g, layer, pages[uu / g.page_tokens], kvh, 1);
      int tok = uu % g.page_tokens;
      float pj = p_s[j];
      if (t < dh) acc0 += pj * to_f32(vb[kv_v_offset(g, tok, t)]);
      if (t + ATT_T < dh) acc1 += pj * to_f32(vb[kv_v_offset(g, tok, t + ATT_T)]);
    }
    m = m_new;
    __syncthreads();
  }
  float* o = out + ((long long)r * n_q_heads + head) * dh;
  if (t < dh) o[t] = acc0 / l;
  if (t + ATT_T < dh) o[t + ATT_T] = acc1 / l;
}
template <typename KT>
void launch_attention_simple(const float* qkv, float* out, const int* row_pos, const int* row_slot,
                             const int* page_table, int max_pages, const KT* kv_pool, KvGeom geom, int layer,
                             int rows, int n_q_heads, hipStream_t s) {
  if (rows)
    attention_simple_kernel<KT><<<dim3(rows, n_q_heads), ATT_T, 0, s>>>(
        qkv, out, row_pos, row_slot, page_table, max_pages, kv_pool, geom, layer, n_q_heads);
}
template void launch_attention_simple<float>(const float*, float*, const int*, const int*, const int*, int,
                                             const float*, KvGeom, int, int, int, hipStream_t);
template void launch_attention_simple<f16_t>(const float*, float*, const int*, const int*, const int*, int,
                                             const f16_t*, KvGeom, int, int, int, hipStream_t);

// ---------------------------------------------------------------- SwiGLU
__global__ void swiglu_f32_kernel(const float* __restrict__ gate_up, float* __restrict__ act, int ffn) {
  int r = blockIdx.y;
  int f = blockIdx.x * blockDim.x + threadIdx.x;
  if (f >= ffn) return;
  float gt = gate_up[(long long)r * 2 * ffn + f], up = gate_up[(long long)r * 2 * ffn + ffn + f];
  act[(long long)r * ffn + f] = gt / (1.0f + expf(-gt)) * up;
}
void launch_swiglu_f32(const float* gate_up, float* act, int rows, int ffn, hipStream_t s) {
  if (rows) swiglu_f32_kernel<<<dim3(ceil_div(ffn, 256), rows), 256, 0, s>>>(gate_up, act, ffn);
}

// ---------------------------------------------------------------- mixture of experts
// One wavefront per row: k rounds of arg-max over the experts (ties to the lower index),
// then a softmax over the k selected logits.
__global__ void moe_route_kernel(const float* __restrict__ logits, int* __restrict__ idx,
                                 float* __restrict__ wt, int n_experts, int top_k) {
  int r = blockIdx.x, lane = threadIdx.x;
  const float* row = logits + (long long)r * n_experts;
  unsigned taken = 0;  // bit c: this lane's expert lane + 64 c is already selected
  float first = 0.f, denom = 0.f, my_w = 0.f;
  int my_e = 0;
  for (int j = 0; j < top_k; ++j) {
    float best = -INFINITY;
    int best_e = 0x7fffffff;
    for (int e = lane, c = 0; e < n_experts; e += WAVE, ++c) {
      float v = row[e];
      if (!((taken >> c) & 1u) && (v > best || (v == best && e < best_e))) {
        best = v;
        best_e = e;
      }
    }
    for (int o = 32; o > 0; o >>= 1) {
      float ov = __shfl_xor(best, o, WAVE);
      int oe = __shfl_xor(best_e, o, WAVE);
      if (ov > best || (ov == best && oe < best_e)) {
        best = ov;
        best_e = oe;
      }
    }
    if ((best_e & 63) == lane) taken |= 1u << (best_e >> 6);
    if (j == 0) first = best;  // the largest selected logit
    float e_w = expf(best - first);
    denom += e_w;
    if (lane == j) {
      my_e = best_e;
      my_w = e_w;
    }
  }
  if (lane < top_k) {
    idx[(long long)r * top_k + lane] = my_e;
    wt[(long long)r * top_k + lane] = my_w / denom;
  }
}
void launch_moe_route(const float* router_logits, int* idx, float* wt, int rows, int n_experts, int top_k,
                      hipStream_t s) {
  if (rows) moe_route_kernel<<<rows, WAVE, 0, s>>>(router_logits, idx, wt, n_experts, top_k);
}

template <typename T>
__global__ void moe_gate_up_simple_kernel(const float* __restrict__ h, const T* __restrict__ w_gate_up,
                                          const int* __restrict__ idx, float* __restrict__ act, int hidden,
                                          int fe, int top_k) {
  int slot = blockIdx.y;  // (row, j)
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int f = blockIdx.x * 4 + wave;
  if (f >= fe) return;
  int e = idx[slot];
  const float* hv = h + (long long)(slot / top_k) * hidden;
  const T* wg = w_gate_up + ((long long)e * 2 * fe + f) * hidden;
  const T* wu = wg + (long long)fe * hidden;
  float ag = 0.f, au = 0.f;
  for (int k = lane; k < hidden; k += WAVE) {
    float x = hv[k];
    ag += x * to_f32(wg[k]);
    au += x * to_f32(wu[k]);
  }
  ag = wave_sum(ag);
  au = wave_sum(au);
  if (lane == 0) act[(long long)slot * fe + f] = ag / (1.0f + expf(-ag)) * au;
}
template <typename T>
void launch_moe_gate_up_simple(const float* h, const T* w_gate_up, const int* idx, float* act, int rows,
                               int top_k, int hidden, int expert_ffn, hipStream_t s) {
  if (rows)
    moe_gate_up_simple_kernel<T><<<dim3(ceil_div(expert_ffn, 4), rows * top_k), 256, 0, s>>>(
        h, w_gate_up, idx, act, hidden, expert_ffn, top_k);
}
template void launch_moe_gate_up_simple<float>(const float*, const float*, const int*, float*, int, int, int,
                                               int, hipStream_t);
template void launch_moe_gate_up_simple<bf16_t>(const float*, const bf16_t*, const int*, float*, int, int, int,
                                                int, hipStream_t);

template <typename T>
__global__ void moe_down_simple_kernel(const float* __restrict__ act, const T* __restrict__ w_down,
                                       const int* __restrict__ idx, const float* __restrict__ wt,
                                       float* __restrict__ x, int hidden, int fe, int top_k) {
  int r = blockIdx.y;
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int n = blockIdx.x * 4 + wave;
  if (n >= hidden) return;
  float total = 0.f;
  for (int j = 0; j < top_k; ++j) {
    int e = idx[(long long)r * top_k + j];
    const T* wd = w_down + ((long long)e * hidden + n) * fe;
    const float* a = act + ((long long)r * top_k + j) * fe;
    float acc = 0.f;
    for (int k = lane; k < fe; k += WAVE) acc += a[k] * to_f32(wd[k]);
    total += wt[(long long)r * top_k + j] * wave_sum(acc);
  }
  if (lane == 0) x[(long long)r * hidden + n] += total;
}
template <typename T>
void launch_moe_down_simple(const float* act, const T* w_down, const int* idx, const float* wt, float* x,
                            int rows, int top_k, int hidden, int expert_ffn, hipStream_t s) {
  if (rows)
    moe_down_simple_kernel<T><<<dim3(ceil_div(hidden, 4), rows), 256, 0, s>>>(act, w_down, idx, wt, x, hidden,
                                                                                expert_ffn, top_k);
}
template void launch_moe_down_simple<float>(const float*, const float*, const int*, const float*, float*, int,
                                            int, int, int, hipStream_t);
template void launch_moe_down_simple<bf16_t>(const float*, const bf16_t*, const int*, const float*, float*, int,
                                             int, int, int, hipStream_t);

// ---------------------------------------------------------------- page copy, conversions
__global__ void copy_pages_kernel(char* __restrict__ pool, const int* __restrict__ pairs,
                                  long long layer_stride, long long page_stride) {
  int pair = blockIdx.x, layer = blockIdx.y;
  const uint4* src = (const uint4*)(pool + layer * layer_stride + (long long)pairs[2 * pair] * page_stride);
  uint4* dst = (uint4*)(pool + layer * layer_stride + (long long)pairs[2 * pair + 1] * page_stride);
  for (long long i = threadIdx.x; i < page_stride / 16; i += blockDim.x) dst[i] = src[i];
}
void launch_copy_pages(void* kv_pool, const int* pairs, int n_pairs, int n_layers, long long layer_stride_bytes,
                       long long page_stride_bytes, hipStream_t s) {
  if (n_pairs)
    copy_pages_kernel<<<dim3(n_pairs, n_layers), 256, 0, s>>>((char*)kv_pool, pairs, layer_stride_bytes,
                                                               page_stride_bytes);
}

__global__ void convert_to_f32_kernel(const void* __restrict__ src, int is_bf16, float* __restrict__ dst,
                                      long long n) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = is_bf16 ? bf16_to_f32(((const bf16_t*)src)[i]) : ((const float*)src)[i];
}
void launch_convert_to_f32(const void* src, int dtype, float* dst, long long n, hipStream_t s) {
  if (n) convert_to_f32_kernel<<<ceil_div(n, 256), 256, 0, s>>>(src, dtype == 1, dst, n);
}

// ---------------------------------------------------------------- decode row plumbing
__global__ void gather_decode_rows_kernel(SlotState st, const int* __restrict__ live, int rows, int* row_token,
                                          int* row_pos, int* row_slot, float* row_inv_temp, float* row_top_p,
                                          long long* row_sample_id, int* row_step) {
  int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  int sl = live[r];
  row_token[r] = st.last_token[sl];
  row_pos[r] = st.pos[sl];
  row_slot[r] = sl;
  row_inv_temp[r] = st.inv_temp[sl];
  row_top_p[r] = st.top_p[sl];
  row_sample_id[r] = st.sample_id[sl];
  row_step[r] = st.step[sl];
}
void launch_gather_decode_rows(SlotState st, const int* live, int rows, int* row_token, int* row_pos,
                               int* row_slot, float* row_inv_temp, float* row_top_p, long long* row_sample_id,
                               int* row_step, hipStream_t s) {
  if (rows)
    gather_decode_rows_kernel<<<ceil_div(rows, 256), 256, 0, s>>>(st, live, rows, row_token, row_pos, row_slot,
                                                                   row_inv_temp, row_top_p, row_sample_id,
                                                                   row_step);
}

// A decode step's last kernel: the drawn tokens go back into the slots and, with the log-probs,
// straight into pinned host memory, where the host reads them once the step's event has fired
// (no copy launches).
__global__ void scatter_tokens_kernel(SlotState st, const int* __restrict__ row_slot,
                                      const int* __restrict__ tokens, const float* __restrict__ logprobs, int rows,
                                      int advance_pos, int* __restrict__ host_tokens,
                                      float* __restrict__ host_logprobs) {
  int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  int sl = row_slot[r];
  const int tok = tokens[r];
  st.last_token[sl] = tok;
  if (advance_pos) st.pos[sl] += 1;
  st.step[sl] += 1;
  host_tokens[r] = tok;
  host_logprobs[r] = logprobs[r];
}
void launch_scatter_tokens(SlotState st, const int* row_slot, const int* tokens, const float* logprobs, int rows,
                           int advance_pos, int* host_tokens, float* host_logprobs, hipStream_t s) {
  if (rows)
    scatter_tokens_kernel<<<ceil_div(rows, 256), 256, 0, s>>>(st, row_slot, tokens, logprobs, rows, advance_pos,
                                                              host_tokens, host_logprobs);
}

// ---------------------------------------------------------------- page-table patches
__global__ void patch_page_table_kernel(int* __restrict__ page_table, int max_pages, const int* __restrict__ triples,
                                        int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) page_table[(long long)triples[3 * i] * max_pages + triples[3 * i + 1]] = triples[3 * i + 2];
}
void launch_patch_page_table(int* page_table, int max_pages, const int* triples, int n, hipStream_t s) {
  if (n) patch_page_table_kernel<<<ceil_div(n, 256), 256, 0, s>>>(page_table, max_pages, triples, n);
}
