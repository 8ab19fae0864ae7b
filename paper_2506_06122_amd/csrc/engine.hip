// Engine set-up and the forward pass over a batch of rows (prompt tokens during prefill,
// one row per live sample during decoding, all tokens of packed sequences in the
// teacher-forced pass): paper section 2.1, "Optimization Workflow".
#include "engine.h"

#include <cmath>
#include <cstring>

static void fail(int code, const std::string& msg) { throw ApiError{code, msg}; }

static void copy_d2d(void* dst, const void* src, size_t bytes, hipStream_t s) {
  if (bytes) HIP_TRY(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, s));
}

static void load_gain(rollout_ctx& c, DevBuf<float>& dst, const void* src) {
  launch_convert_to_f32(src, c.md.dtype, dst.p, c.md.hidden, c.stream);
}

static void load_matrix(rollout_ctx& c, DevBuf<char>& dst, size_t dst_off_elems, const void* src, size_t elems) {
  copy_d2d(dst.p + dst_off_elems * c.elem, src, elems * c.elem, c.stream);
}

// Buffers of every weight in the library's own layout (sizes depend on the shape only).
static void alloc_weights(rollout_ctx& c) {
  const rollout_model_desc& m = c.md;
  const bool moe = m.n_experts > 0;
  const size_t d = m.hidden;
  c.embed.alloc((size_t)m.vocab * d * c.elem);
  if (c.simple) c.lm_head.alloc((size_t)m.vocab * d * c.elem);
  else c.lm_head_p.alloc((size_t)m.vocab * d * 2);
  c.final_norm.alloc(d);
  c.layers.resize(m.n_layers);
  for (LayerWeights& L : c.layers) {
    L.norm1.alloc(d);
    L.norm2.alloc(d);
    if (m.flags & ROLLOUT_MODEL_QKV_BIAS) L.qkv_bias.alloc(c.qkv_dim);
    if (m.flags & ROLLOUT_MODEL_QK_NORM) {
      L.q_gain.alloc(m.head_dim);
      L.k_gain.alloc(m.head_dim);
    }
    if (!c.simple) {
      // MoE: the experts' matrices are stacked, [E * Fe][hidden] and [E * hidden][Fe]; Fe is a
      // multiple of 16, so the stacked gate/up column tiles still alternate inside every expert
      const size_t f = moe ? (size_t)m.n_experts * m.expert_ffn_dim : (size_t)m.ffn_dim;
      if (moe) L.router_p.alloc((size_t)m.n_experts * d * 2);
      L.wqkv_p.alloc((size_t)c.qkv_dim * d * 2);
      L.wo_p.alloc(d * c.q_dim * 2);
      L.w_gate_up_p.alloc(2 * f * d * 2);
      L.w_down_p.alloc(f * d * 2);
      continue;
    }
    L.wqkv.alloc((size_t)c.qkv_dim * d * c.elem);
    L.wo.alloc(d * c.q_dim * c.elem);
    const size_t f = moe ? (size_t)m.n_experts * m.expert_ffn_dim : (size_t)m.ffn_dim;
    if (moe) L.router.alloc((size_t)m.n_experts * d * c.elem);
    L.w_gate_up.alloc(2 * f * d * c.elem);
    L.w_down.alloc(d * f * c.elem);
  }
}

// Does this model have tensor `which` at `layer`?
void engine_check_tensor(const rollout_ctx& c, int layer, int which) {
  const rollout_model_desc& m = c.md;
  const bool model_level = which == ROLLOUT_W_EMBED || which == ROLLOUT_W_FINAL_NORM || which == ROLLOUT_W_LM_HEAD;
  if (which < ROLLOUT_W_EMBED || which > ROLLOUT_W_K_NORM) fail(ROLLOUT_E_INVAL, "unknown tensor");
  if (model_level ? layer != -1 : (layer < 0 || layer >= m.n_layers))
    fail(ROLLOUT_E_INVAL, "layer out of range (model-level tensors take layer -1)");
  if (which == ROLLOUT_W_ROUTER && !m.n_experts) fail(ROLLOUT_E_INVAL, "a dense model has no router");
  if (which == ROLLOUT_W_LM_HEAD && (m.flags & ROLLOUT_MODEL_TIED_LM_HEAD))
    fail(ROLLOUT_E_INVAL, "the lm_head of this model is its embedding matrix");
  if (which >= ROLLOUT_W_BQ && which <= ROLLOUT_W_BV && !(m.flags & ROLLOUT_MODEL_QKV_BIAS))
    fail(ROLLOUT_E_INVAL, "this model has no q/k/v bias");
  if (which >= ROLLOUT_W_Q_NORM && which <= ROLLOUT_W_K_NORM && !(m.flags & ROLLOUT_MODEL_QK_NORM))
    fail(ROLLOUT_E_INVAL, "this model has no q/k norm");
}

// One tensor, given as at rollout_init (device pointer, model dtype, row-major), into the
// library's layout: asynchronous on the context's stream.
void engine_load_tensor(rollout_ctx& c, int layer, int which, const void* src) {
  const rollout_model_desc& m = c.md;
  const bool moe = m.n_experts > 0;
  const size_t d = m.hidden;
  if (!src) fail(ROLLOUT_E_INVAL, "null weight pointer");
  const bool model_level = which == ROLLOUT_W_EMBED || which == ROLLOUT_W_FINAL_NORM || which == ROLLOUT_W_LM_HEAD;
  engine_check_tensor(c, layer, which);
  const bool tied = (m.flags & ROLLOUT_MODEL_TIED_LM_HEAD) != 0;
  if (which == ROLLOUT_W_EMBED) {
    load_matrix(c, c.embed, 0, src, (size_t)m.vocab * d);
    if (!tied) return;
    which = ROLLOUT_W_LM_HEAD;  // the embedding matrix is the logits projection as well
  }
  if (which == ROLLOUT_W_FINAL_NORM) return load_gain(c, c.final_norm, src);
  if (which == ROLLOUT_W_LM_HEAD) {
    if (c.simple) return load_matrix(c, c.lm_head, 0, src, (size_t)m.vocab * d);
    return launch_pack_weight(src, c.lm_head_p.p, m.vocab, (int)d, 0, 1, c.stream);
  }
  (void)model_level;
  LayerWeights& L = c.layers[layer];
  if (which == ROLLOUT_W_NORM1) return load_gain(c, L.norm1, src);
  if (which == ROLLOUT_W_NORM2) return load_gain(c, L.norm2, src);
  if (which == ROLLOUT_W_BQ) return launch_convert_to_f32(src, m.dtype, L.qkv_bias.p, c.q_dim, c.stream);
  if (which == ROLLOUT_W_BK) return launch_convert_to_f32(src, m.dtype, L.qkv_bias.p + c.q_dim, c.kv_dim, c.stream);
  if (which == ROLLOUT_W_BV)
    return launch_convert_to_f32(src, m.dtype, L.qkv_bias.p + c.q_dim + c.kv_dim, c.kv_dim, c.stream);
  if (which == ROLLOUT_W_Q_NORM) return launch_convert_to_f32(src, m.dtype, L.q_gain.p, m.head_dim, c.stream);
  if (which == ROLLOUT_W_K_NORM) return launch_convert_to_f32(src, m.dtype, L.k_gain.p, m.head_dim, c.stream);
  const size_t fe = m.expert_ffn_dim, E = m.n_experts;
  if (!c.simple) {
    const int f = moe ? m.n_experts * m.expert_ffn_dim : m.ffn_dim;
    const int down_rows = moe ? m.n_experts * (int)d : (int)d;
    const int down_k = moe ? m.expert_ffn_dim : m.ffn_dim;
    switch (which) {
      case ROLLOUT_W_WQ: return launch_pack_weight(src, L.wqkv_p.p, c.q_dim, (int)d, 0, 1, c.stream);
      case ROLLOUT_W_WK: return launch_pack_weight(src, L.wqkv_p.p, c.kv_dim, (int)d, c.q_dim / 16, 1, c.stream);
      case ROLLOUT_W_WV:
        return launch_pack_weight(src, L.wqkv_p.p, c.kv_dim, (int)d, (c.q_dim + c.kv_dim) / 16, 1, c.stream);
      case ROLLOUT_W_WO: return launch_pack_weight(src, L.wo_p.p, (int)d, c.q_dim, 0, 1, c.stream);
      case ROLLOUT_W_GATE: return launch_pack_weight(src, L.w_gate_up_p.p, f, (int)d, 0, 2, c.stream);
      case ROLLOUT_W_UP: return launch_pack_weight(src, L.w_gate_up_p.p, f, (int)d, 1, 2, c.stream);
      case ROLLOUT_W_DOWN: return launch_pack_weight(src, L.w_down_p.p, down_rows, down_k, 0, 1, c.stream);
      default: return launch_pack_weight(src, L.router_p.p, m.n_experts, (int)d, 0, 1, c.stream);
    }
  }
  switch (which) {
    case ROLLOUT_W_WQ: return load_matrix(c, L.wqkv, 0, src, (size_t)c.q_dim * d);
    case ROLLOUT_W_WK: return load_matrix(c, L.wqkv, (size_t)c.q_dim * d, src, (size_t)c.kv_dim * d);
    case ROLLOUT_W_WV: return load_matrix(c, L.wqkv, (size_t)(c.q_dim + c.kv_dim) * d, src, (size_t)c.kv_dim * d);
    case ROLLOUT_W_WO: return load_matrix(c, L.wo, 0, src, d * c.q_dim);
    case ROLLOUT_W_ROUTER: return load_matrix(c, L.router, 0, src, E * d);
    case ROLLOUT_W_DOWN: return load_matrix(c, L.w_down, 0, src, moe ? E * d * fe : d * (size_t)m.ffn_dim);
    default: break;
  }
  // gate / up of the plain path: [gate rows; up rows], per expert for MoE
  const size_t half = which == ROLLOUT_W_UP ? 1 : 0;
  if (moe) {
    HIP_TRY(hipMemcpy2DAsync(L.w_gate_up.p + half * fe * d * c.elem, 2 * fe * d * c.elem, src, fe * d * c.elem,
                             fe * d * c.elem, E, hipMemcpyDeviceToDevice, c.stream));
  } else {
    const size_t f = m.ffn_dim;
    load_matrix(c, L.w_gate_up, half * f * d, src, f * d);
  }
}

void engine_init(rollout_ctx& c, const rollout_weights& w) {
  const rollout_model_desc& m = c.md;
  const rollout_runtime_desc& r = c.rd;
  if (m.n_layers < 1 || m.hidden < 1 || m.n_q_heads < 1 || m.n_kv_heads < 1 || m.vocab < 2)
    fail(ROLLOUT_E_INVAL, "model shape fields must be positive");
  if (m.vocab > 262144) fail(ROLLOUT_E_INVAL, "vocab must be at most 262144");
  if (m.n_q_heads % m.n_kv_heads) fail(ROLLOUT_E_INVAL, "n_q_heads must be a multiple of n_kv_heads");
  if (m.head_dim < 32 || m.head_dim > 256 || m.head_dim % 32)
    fail(ROLLOUT_E_INVAL, "head_dim must be a multiple of 32 in [32, 256]");
  if (m.dtype != ROLLOUT_DTYPE_F32 && m.dtype != ROLLOUT_DTYPE_BF16) fail(ROLLOUT_E_INVAL, "unknown dtype");
  if (m.flags & ~(ROLLOUT_MODEL_QKV_BIAS | ROLLOUT_MODEL_QK_NORM | ROLLOUT_MODEL_TIED_LM_HEAD))
    fail(ROLLOUT_E_INVAL, "unknown model flag");
  const bool moe = m.n_experts > 0;
  if (moe) {
    if (m.top_k < 1 || m.top_k > m.n_experts || m.top_k > 64 || m.n_experts > 256 || m.expert_ffn_dim < 1)
      fail(ROLLOUT_E_INVAL, "MoE needs 1 <= top_k <= min(n_experts, 64), n_experts <= 256, expert_ffn_dim >= 1");
  } else if (m.ffn_dim < 1) {
    fail(ROLLOUT_E_INVAL, "ffn_dim must be positive for a dense model");
  }
  if (!(m.rms_eps >= 0.f) || !(m.rope_theta > 0.f)) fail(ROLLOUT_E_INVAL, "rms_eps >= 0 and rope_theta > 0 required");
  if (r.page_tokens < 32 || r.page_tokens % 32) fail(ROLLOUT_E_INVAL, "page_tokens must be a positive multiple of 32");
  if (r.max_live_samples < 1 || r.max_context < 2 || r.max_batch_tokens < 1)
    fail(ROLLOUT_E_INVAL, "max_live_samples, max_context, max_batch_tokens must be positive");
  if (r.flags & ~(ROLLOUT_RT_SIMPLE_KERNELS | ROLLOUT_RT_RECORD_ROUTING | ROLLOUT_RT_KERNEL_TIMING |
                  ROLLOUT_RT_PROMPT_GROUPS | ROLLOUT_RT_GROW_PAGES))
    fail(ROLLOUT_E_INVAL, "unknown runtime flag");
  const bool tied = (m.flags & ROLLOUT_MODEL_TIED_LM_HEAD) != 0;
  if (!w.embed || !w.final_norm || (!tied && !w.lm_head) || !w.layers) fail(ROLLOUT_E_INVAL, "null weight pointer");

  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev < 1) fail(ROLLOUT_E_HIP, "no HIP device");
  HIP_TRY(hipGetDevice(&c.device));
  c.stream = (hipStream_t)r.hip_stream;
  // The matrix-core path needs bf16 storage, head_dim 128, at most 16 query heads per KV head
  // (the columns of one attention tile) and fragment-aligned dimensions; anything else runs
  // the plain path.
  c.simple = (r.flags & ROLLOUT_RT_SIMPLE_KERNELS) || m.dtype != ROLLOUT_DTYPE_BF16 || m.head_dim != 128 ||
             m.n_q_heads / m.n_kv_heads > 16 || m.hidden % 32 || m.hidden > 8192 || m.vocab % 16 ||
             (moe ? (m.n_experts % 16 || m.expert_ffn_dim % 32) : m.ffn_dim % 32);
  c.elem = m.dtype == ROLLOUT_DTYPE_BF16 ? 2 : 4;
  c.timer.enabled = (r.flags & ROLLOUT_RT_KERNEL_TIMING) != 0;
  c.timer.stride = r.timing_stride;
  c.q_dim = m.n_q_heads * m.head_dim;
  c.kv_dim = m.n_kv_heads * m.head_dim;
  c.qkv_dim = c.q_dim + 2 * c.kv_dim;
  c.page_tokens = r.page_tokens;
  c.max_context = r.max_context;
  c.grow_pages = (r.flags & ROLLOUT_RT_GROW_PAGES) != 0;
  c.max_pages = ceil_div(r.max_context, r.page_tokens);
  c.temp_slot0 = r.max_live_samples;
  c.n_slots = r.max_live_samples + rollout_ctx::kTempSlots + rollout_ctx::kPendingRows;
  c.queue.free_rows.clear();
  for (int i = rollout_ctx::kPendingRows - 1; i >= 0; --i) c.queue.free_rows.push_back(c.temp_slot0 + rollout_ctx::kTempSlots + i);
  c.r_max = std::max(r.max_batch_tokens, r.max_live_samples);
  c.logit_rows = std::max(r.max_live_samples, std::min(c.r_max, 1024));

  // ---- weights ----
  const size_t d = m.hidden;
  alloc_weights(c);
  engine_load_tensor(c, -1, ROLLOUT_W_EMBED, w.embed);
  if (!tied) engine_load_tensor(c, -1, ROLLOUT_W_LM_HEAD, w.lm_head);
  engine_load_tensor(c, -1, ROLLOUT_W_FINAL_NORM, w.final_norm);
  for (int l = 0; l < m.n_layers; ++l) {
    const rollout_layer_weights& s = w.layers[l];
    const void* src[] = {s.norm1, s.wq, s.wk, s.wv, s.wo, s.norm2, s.w_gate, s.w_up, s.w_down};
    for (int t = 0; t < 9; ++t) engine_load_tensor(c, l, ROLLOUT_W_NORM1 + t, src[t]);
    if (moe) engine_load_tensor(c, l, ROLLOUT_W_ROUTER, s.router);
    if (m.flags & ROLLOUT_MODEL_QKV_BIAS) {
      engine_load_tensor(c, l, ROLLOUT_W_BQ, s.bq);
      engine_load_tensor(c, l, ROLLOUT_W_BK, s.bk);
      engine_load_tensor(c, l, ROLLOUT_W_BV, s.bv);
    }
    if (m.flags & ROLLOUT_MODEL_QK_NORM) {
      engine_load_tensor(c, l, ROLLOUT_W_Q_NORM, s.q_norm);
      engine_load_tensor(c, l, ROLLOUT_W_K_NORM, s.k_norm);
    }
  }

  // ---- rotary table: cos/sin of pos * theta^(-2i/dh), computed in double ----
  {
    const int half = m.head_dim / 2;
    std::vector<float> tab((size_t)r.max_context * m.head_dim);
    for (int i = 0; i < half; ++i) {
      double inv_freq = std::pow((double)m.rope_theta, -2.0 * i / m.head_dim);
      for (int p = 0; p < r.max_context; ++p) {
        double phi = (double)p * inv_freq;
        tab[(size_t)p * m.head_dim + 2 * i] = (float)std::cos(phi);
        tab[(size_t)p * m.head_dim + 2 * i + 1] = (float)std::sin(phi);
      }
    }
    c.cos_sin.alloc(tab.size());
    HIP_TRY(hipMemcpyAsync(c.cos_sin.p, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice, c.stream));
    HIP_TRY(hipStreamSynchronize(c.stream));
  }

  // ---- KV pool ----
  c.geom.n_kv_heads = m.n_kv_heads;
  c.geom.head_dim = m.head_dim;
  c.geom.page_tokens = r.page_tokens;
  c.geom.layout = c.simple ? KV_LINEAR : KV_MATRIX;
  c.geom.page_stride = (long long)m.n_kv_heads * 2 * r.page_tokens * m.head_dim;
  const size_t page_bytes_all_layers = (size_t)c.geom.page_stride * c.elem * m.n_layers;
  long long n_pages = (long long)(r.kv_pool_bytes / page_bytes_all_layers);
  if (n_pages < 1) fail(ROLLOUT_E_INVAL, "kv_pool_bytes holds less than one page");
  if (n_pages > 0x7fffffff) n_pages = 0x7fffffff;
  c.geom.layer_stride = n_pages * c.geom.page_stride;
  c.kv_pool.alloc((size_t)n_pages * page_bytes_all_layers);
  // attention multiplies masked positions' values by zero: they must be finite
  HIP_TRY(hipMemsetAsync(c.kv_pool.p, 0, (size_t)n_pages * page_bytes_all_layers, c.stream));
  c.pool = new rollout_pool((int32_t)n_pages);
  c.h_page_table.assign((size_t)c.n_slots * c.max_pages, 0);
  c.d_page_table.alloc(c.h_page_table.size());
  HIP_TRY(hipMemsetAsync(c.d_page_table.p, 0, c.h_page_table.size() * sizeof(int), c.stream));

  // ---- slot state ----
  c.st_last_token.alloc(c.n_slots);
  c.st_pos.alloc(c.n_slots);
  c.st_step.alloc(c.n_slots);
  c.st_sample_id.alloc(c.n_slots);
  c.st_inv_temp.alloc(c.n_slots);
  c.st_top_p.alloc(c.n_slots);
  c.st = SlotState{c.st_last_token.p, c.st_pos.p, c.st_step.p, c.st_sample_id.p, c.st_inv_temp.p, c.st_top_p.p};
  c.d_live.alloc(r.max_live_samples);
  if (c.grow_pages) c.d_page_patch.alloc(3 * (size_t)r.max_live_samples);
  for (int s = r.max_live_samples - 1; s >= 0; --s) c.free_slots.push_back(s);

  // ---- workspaces ----
  const size_t R = c.r_max;
  c.x.alloc(R * d);
  if (!c.simple) {
    // activation buffers hold two planes each: hi parts, then lo parts; rows padded to whole
    // 16-row fragments for the small decode steps, which keep them in fragment order
    const size_t Rp = (R + 31) / 32 * 32;
    c.h_bf16.alloc(2 * Rp * d);
    c.q_bf16.alloc(2 * R * c.q_dim);
    c.attn_bf16.alloc(2 * Rp * c.q_dim);
    c.act_bf16.alloc(2 * Rp * (moe ? (size_t)m.top_k * m.expert_ffn_dim : (size_t)m.ffn_dim));
    if (moe) {
      const size_t picks = R * m.top_k;
      c.moe_max_blocks = (int)(std::min<size_t>(m.n_experts, picks) + picks / kMoeBlockRows + 1);
      c.moe_idx.alloc(picks);
      c.moe_wt.alloc(picks);
      c.moe_pos.alloc(picks);
      c.moe_row_map.alloc(picks);
      c.moe_slot_of.alloc(picks);
      c.moe_count.alloc((size_t)m.n_layers * m.n_experts);
      c.moe_group_of_block.alloc(c.moe_max_blocks);
      c.moe_block_begin.alloc(c.moe_max_blocks);
      c.moe_block_end.alloc(c.moe_max_blocks);
      c.moe_y.alloc(picks * d);
      if (r.flags & ROLLOUT_RT_RECORD_ROUTING) c.route_log.alloc((size_t)m.n_layers * R * m.top_k);
    }
    c.hn_bf16.alloc(2 * (size_t)c.logit_rows * d);
    c.partial_ld = std::max({c.qkv_dim, (int)d, moe ? m.n_experts : 0});
    c.partial_rows = std::max<long long>(R, 2048);
    c.partial.alloc((size_t)c.partial_rows * c.partial_ld);
    c.attn_max_parts = std::max(8 * r.max_live_samples * m.n_kv_heads, 1024);
    c.grp_rows.alloc(8 * (size_t)r.max_live_samples);
    c.grp_len.alloc(r.max_live_samples);
    c.grp_slot.alloc(r.max_live_samples);
    c.row_t0.alloc(r.max_live_samples);
    c.attn_part_o.alloc((size_t)c.attn_max_parts * 16 * 128);
    c.attn_part_ml.alloc((size_t)c.attn_max_parts * 32);
    c.ssq.alloc((size_t)(d / 16 + 1) * 256);
    {
      const size_t parts = ceil_div(m.vocab / 16, 8);  // the narrowest tile configuration
      c.lse_max.alloc(parts * R);
      c.lse_sum.alloc(parts * R);
      c.lse_tgt.alloc(R);
    }
    c.seq_row0.alloc(rollout_ctx::kTempSlots);
    c.seq_len.alloc(rollout_ctx::kTempSlots);
    c.seq_slot.alloc(rollout_ctx::kTempSlots);
    c.seq_pos0.alloc(rollout_ctx::kTempSlots);
    c.chunk_ints.alloc(3 * R);
  } else {
    c.h.alloc(R * d);
    c.qkv.alloc(R * c.qkv_dim);
    c.attn.alloc(R * c.q_dim);
    c.hn.alloc((size_t)c.logit_rows * d);
  }
  if (c.simple && moe) {
    c.router_logits.alloc(R * m.n_experts);
    c.moe_idx.alloc(R * m.top_k);
    c.moe_wt.alloc(R * m.top_k);
    c.act.alloc(R * m.top_k * m.expert_ffn_dim);
    if (r.flags & ROLLOUT_RT_RECORD_ROUTING) c.route_log.alloc((size_t)m.n_layers * R * m.top_k);
  } else if (c.simple) {
    c.gate_up.alloc(R * 2 * m.ffn_dim);
    c.act.alloc(R * m.ffn_dim);
  }
  c.logits.alloc((size_t)c.logit_rows * m.vocab);
  c.row_token.alloc(R);
  c.row_pos.alloc(R);
  c.row_slot.alloc(R);
  c.row_step.alloc(R);
  c.row_aux.alloc(2 * R);
  c.row_forced.alloc(R);
  c.out_tokens.alloc(R);
  c.row_sample_id.alloc(R);
  c.row_inv_temp.alloc(R);
  c.row_top_p.alloc(R);
  c.out_logprobs.alloc(R);
  c.row_uniform.alloc(R);
  c.samp_rows = (int)std::min<size_t>(R, 4096);
  c.samp_part_max.alloc((size_t)c.samp_rows * kSampleParts);
  c.samp_seg_sums.alloc((size_t)c.samp_rows * kSampleSegments);
  c.h_int.alloc(8 * R);
  c.h_float.alloc(4 * R);
  c.h_ll.alloc(R);
  HIP_TRY(hipStreamSynchronize(c.stream));
}

void engine_upload_page_table(rollout_ctx& c) {
  HIP_TRY(hipMemcpyAsync(c.d_page_table.p, c.h_page_table.data(), c.h_page_table.size() * sizeof(int),
                         hipMemcpyHostToDevice, c.stream));
}

// ------------------------------------------------------------------------------------------
// T = storage type of the weights; KT = storage type of the KV cache (fp32 models: fp32,
// bf16 models: IEEE half, see common.h)
template <typename T, typename KT>
static void forward_rows_simple(rollout_ctx& c, int R) {
  const rollout_model_desc& m = c.md;
  hipStream_t s = c.stream;
  const int d = m.hidden;
  launch_embed<T>((const T*)c.embed.p, c.row_token.p, c.x.p, R, d, s);
  for (int l = 0; l < m.n_layers; ++l) {
    LayerWeights& L = c.layers[l];
    launch_rmsnorm_f32(c.x.p, L.norm1.p, c.h.p, nullptr, R, d, m.rms_eps, s);
    launch_linear_simple<T>(c.h.p, d, (const T*)L.wqkv.p, c.qkv.p, c.qkv_dim, nullptr, 0, R, c.qkv_dim, d, s);
    launch_qkv_bias_norm(c.qkv.p, L.qkv_bias.p, L.q_gain.p, L.k_gain.p, m.rms_eps, R, m.n_q_heads, m.n_kv_heads,
                         m.head_dim, s);
    launch_rope_kvwrite<KT>(c.qkv.p, c.cos_sin.p, c.row_pos.p, c.row_slot.p, c.d_page_table.p, c.max_pages,
                            (KT*)c.kv_pool.p, c.geom, l, R, m.n_q_heads, s);
    launch_attention_simple<KT>(c.qkv.p, c.attn.p, c.row_pos.p, c.row_slot.p, c.d_page_table.p, c.max_pages,
                                (const KT*)c.kv_pool.p, c.geom, l, R, m.n_q_heads, s);
    launch_linear_simple<T>(c.attn.p, c.q_dim, (const T*)L.wo.p, c.x.p, d, c.x.p, d, R, d, c.q_dim, s);
    launch_rmsnorm_f32(c.x.p, L.norm2.p, c.h.p, nullptr, R, d, m.rms_eps, s);
    if (m.n_experts > 0) {
      launch_linear_simple<T>(c.h.p, d, (const T*)L.router.p, c.router_logits.p, m.n_experts, nullptr, 0, R,
                              m.n_experts, d, s);
      launch_moe_route(c.router_logits.p, c.moe_idx.p, c.moe_wt.p, R, m.n_experts, m.top_k, s);
      if (c.route_log.p)
        HIP_TRY(hipMemcpyAsync(c.route_log.p + (size_t)l * c.r_max * m.top_k, c.moe_idx.p,
                               (size_t)R * m.top_k * sizeof(int), hipMemcpyDeviceToDevice, s));
      launch_moe_gate_up_simple<T>(c.h.p, (const T*)L.w_gate_up.p, c.moe_idx.p, c.act.p, R, m.top_k, d,
                                   m.expert_ffn_dim, s);
      launch_moe_down_simple<T>(c.act.p, (const T*)L.w_down.p, c.moe_idx.p, c.moe_wt.p, c.x.p, R, m.top_k, d,
                                m.expert_ffn_dim, s);
    } else {
      launch_linear_simple<T>(c.h.p, d, (const T*)L.w_gate_up.p, c.gate_up.p, 2 * m.ffn_dim, nullptr, 0, R,
                              2 * m.ffn_dim, d, s);
      launch_swiglu_f32(c.gate_up.p, c.act.p, R, m.ffn_dim, s);
      launch_linear_simple<T>(c.act.p, m.ffn_dim, (const T*)L.w_down.p, c.x.p, d, c.x.p, d, R, d, m.ffn_dim, s);
    }
  }
}

// ------------------------------------------------------------------------------------------
// Matrix-core path, many rows (prefill, teacher-forced pass, decode steps with more than 32
// live samples).  Per layer: QKV projection -> sum + rotary + KV-page write -> paged
// attention -> O projection -> residual + norm -> gate/up projection with SwiGLU in the
// epilogue -> down projection -> residual + next norm.
static double gemm_bytes(int M, int N, int K, int out_elem) {  // operands once, result once
  return 2.0 * N * K + 2.0 * M * K + (double)out_elem * M * N;
}

static int project(rollout_ctx& c, const uint16_t* a, long long a_lo_off, int lda, const void* w, int M, int N,
                   int K) {
  GemmArgs g{};
  g.a = a;
  g.a_lo = a + a_lo_off;
  g.w = w;
  g.out = c.partial.p;
  g.M = M;
  g.N = N;
  g.K = K;
  g.lda = lda;
  g.ldo = N;
  g.split_stride = (long long)M * N;
  const int cap = (int)std::min<long long>(16, (c.partial_rows * c.partial_ld) / ((long long)M * N));
  const GemmPlan pl = gemm_plan(M, N, K, EPI_F32, std::max(1, cap));
  c.timer.begin(pl.name, gemm_bytes(M, N, K, 4), 2.0 * M * N * K, c.stream);
  const int z = launch_gemm_bf16(g, EPI_F32, pl, c.stream);
  c.timer.end(c.stream);
  return z;
}

static void gate_up(rollout_ctx& c, LayerWeights& L, int R) {
  const int d = c.md.hidden, f = c.md.ffn_dim;
  GemmArgs gu{};
  gu.a = c.h_bf16.p;
  gu.a_lo = c.h_bf16.p + c.h_bf16.n / 2;
  gu.w = L.w_gate_up_p.p;
  gu.out = c.act_bf16.p;
  gu.out_lo_offset = (long long)(c.act_bf16.n / 2);
  gu.M = R;
  gu.N = 2 * f;
  gu.K = d;
  gu.lda = d;
  gu.ldo = f;
  const GemmPlan pl = gemm_plan(R, 2 * f, d, EPI_SWIGLU_BF16, 1);
  c.timer.begin(pl.name, 2.0 * 2 * f * d + 2.0 * R * d + 2.0 * R * f, 2.0 * R * 2 * f * d, c.stream);
  launch_gemm_bf16(gu, EPI_SWIGLU_BF16, pl, c.stream);
  c.timer.end(c.stream);
}

static void embed_and_norm(rollout_ctx& c, int R) {
  RowNormArgs rn{};
  rn.x = c.x.p;
  rn.h = c.h_bf16.p;
  rn.h_lo_offset = (long long)(c.h_bf16.n / 2);
  rn.rows = R;
  rn.hidden = c.md.hidden;
  rn.eps = c.md.rms_eps;
  rn.tokens = c.row_token.p;
  rn.embed = (const uint16_t*)c.embed.p;
  rn.gain = c.layers[0].norm1.p;
  c.timer.begin("row_norm_kernel", (double)R * c.md.hidden * (2 + 4 + 2), 0, c.stream);
  launch_row_norm(rn, c.stream);
  c.timer.end(c.stream);
}

// KV splits per (sample, KV head) of a decode step: one workgroup per CU, at least 256 cached
// positions each, at most the 16 the merge kernels take.  (Measured: more, shorter splits lose
// to the per-workgroup prologue and the longer merge.)
// The second launch of a decode attention whose rows have several partial results: joins the
// slots of every (row, KV head).  Timed under its own name; bytes = the slots read (output
// fragments, maxima and sums) and the rows written as two bf16 planes.
static void merge_attention_slots(rollout_ctx& c, const AttnArgs& at, int rows) {
  const int slots = at.n_slots ? at.n_slots : at.n_splits;
  c.timer.begin("attn_merge_fused_kernel",
                (double)rows * c.md.n_kv_heads * slots * (16 * 128 + 32) * 4.0 + 4.0 * rows * c.q_dim, 0, c.stream);
  launch_attention_merge(at, c.stream);
  c.timer.end(c.stream);
}

static int decode_attention_splits(const rollout_ctx& c, int base) {
  return std::max(1, std::min({ceil_div(256, base), ceil_div(c.decode_max_ctx, 256), c.attn_max_parts / base, 16}));
}

// Mixture-of-experts feed-forward block: router projection -> top-k routing -> plan of the
// expert-sorted row blocks -> grouped gate/up projection with SwiGLU -> grouped down
// projection -> weighted sum of each row's picks + residual + next norm.
static void moe_block(rollout_ctx& c, LayerWeights& L, int layer, int R, RowNormArgs rn, const float* next_gain) {
  const rollout_model_desc& m = c.md;
  hipStream_t s = c.stream;
  const int d = m.hidden, fe = m.expert_ffn_dim, E = m.n_experts, k = m.top_k;
  const int picks = R * k;
  const int z = project(c, c.h_bf16.p, (long long)(c.h_bf16.n / 2), d, L.router_p.p, R, E, d);

  MoeRouteArgs ra{};
  ra.partial = c.partial.p;
  ra.split_stride = (long long)R * E;
  ra.splits = z;
  ra.rows = R;
  ra.n_experts = E;
  ra.top_k = k;
  ra.idx = c.moe_idx.p;
  ra.wt = c.moe_wt.p;
  ra.pos = c.moe_pos.p;
  ra.count = c.moe_count.p + (size_t)layer * E;
  ra.route_log = c.route_log.p ? c.route_log.p + (size_t)layer * c.r_max * k : nullptr;
  c.timer.begin("moe_route_topk_kernel", (double)R * E * 4 * z, 0, s);
  launch_moe_route_topk(ra, s);
  c.timer.end(s);

  MoePlanArgs pa{};
  pa.count = ra.count;
  pa.idx = c.moe_idx.p;
  pa.pos = c.moe_pos.p;
  pa.rows = R;
  pa.n_experts = E;
  pa.top_k = k;
  pa.max_blocks = std::min(c.moe_max_blocks, std::min(E, picks) + picks / kMoeBlockRows + 1);
  pa.row_map = c.moe_row_map.p;
  pa.slot_of = c.moe_slot_of.p;
  pa.group_of_block = c.moe_group_of_block.p;
  pa.block_row_begin = c.moe_block_begin.p;
  pa.block_row_end = c.moe_block_end.p;
  c.timer.begin("moe_plan_kernel", (double)picks * 16, 0, s);
  launch_moe_plan(pa, s);
  c.timer.end(s);

  // Expected number of experts with at least one pick under uniform routing: the weight bytes
  // of the timing records (the true count stays on the device).
  const double touched = E * (1.0 - std::pow(1.0 - 1.0 / E, (double)picks));
  GemmPlan pl{};
  pl.kind = 1;
  pl.mt = kMoeBlockRows / 16;
  pl.nt = 2;
  pl.nw = 4;
  pl.splits = 1;
  pl.kc = 2;

  GemmArgs gu{};
  gu.a = c.h_bf16.p;
  gu.a_lo = c.h_bf16.p + c.h_bf16.n / 2;
  gu.w = L.w_gate_up_p.p;
  gu.out = c.act_bf16.p;
  gu.out_lo_offset = (long long)(c.act_bf16.n / 2);
  gu.M = picks;
  gu.N = 2 * fe;
  gu.K = d;
  gu.lda = d;
  gu.ldo = fe;
  gu.group_of_block = pa.group_of_block;
  gu.block_row_begin = pa.block_row_begin;
  gu.block_row_end = pa.block_row_end;
  gu.row_map = pa.row_map;
  gu.group_stride16 = (long long)2 * fe * d * 2 / 16;
  gu.n_row_blocks = pa.max_blocks;
  pl.name = "gemm_tile_ring_kernel<4,2,2,1,1>";
  c.timer.begin(pl.name, touched * 2.0 * 2 * fe * d + 4.0 * picks * d + 4.0 * picks * fe, 2.0 * picks * 2 * fe * d, s);
  launch_gemm_bf16(gu, EPI_SWIGLU_BF16, pl, s);
  c.timer.end(s);

  GemmArgs dn{};
  dn.a = c.act_bf16.p;
  dn.a_lo = c.act_bf16.p + c.act_bf16.n / 2;
  dn.w = L.w_down_p.p;
  dn.out = c.moe_y.p;
  dn.M = picks;
  dn.N = d;
  dn.K = fe;
  dn.lda = fe;
  dn.ldo = d;
  dn.split_stride = 0;
  dn.group_of_block = pa.group_of_block;
  dn.block_row_begin = pa.block_row_begin;
  dn.block_row_end = pa.block_row_end;
  dn.group_stride16 = (long long)d * fe * 2 / 16;
  dn.n_row_blocks = pa.max_blocks;
  pl.name = "gemm_tile_ring_kernel<4,2,2,1,0>";
  c.timer.begin(pl.name, touched * 2.0 * d * fe + 4.0 * picks * fe + 4.0 * picks * d, 2.0 * picks * d * fe, s);
  launch_gemm_bf16(dn, EPI_F32, pl, s);
  c.timer.end(s);

  rn.splits = 0;
  rn.gain = next_gain;
  rn.moe_y = c.moe_y.p;
  rn.moe_slot = c.moe_slot_of.p;
  rn.moe_wt = c.moe_wt.p;
  rn.moe_k = k;
  c.timer.begin("row_norm_kernel", (double)R * d * (4 + 4 + 2 + 2 + 4.0 * k), 0, s);
  launch_row_norm(rn, s);
  c.timer.end(s);
}

static void forward_rows_tiled(rollout_ctx& c, int R, const SeqBatch* seqs) {
  const rollout_model_desc& m = c.md;
  hipStream_t s = c.stream;
  const int d = m.hidden, f = m.ffn_dim;
  if (m.n_experts > 0)  // the per-layer pick counters of the routing kernels start at zero
    HIP_TRY(hipMemsetAsync(c.moe_count.p, 0, c.moe_count.n * sizeof(int), s));
  embed_and_norm(c, R);
  RowNormArgs rn{};
  rn.x = c.x.p;
  rn.h = c.h_bf16.p;
  rn.h_lo_offset = (long long)(c.h_bf16.n / 2);
  rn.rows = R;
  rn.hidden = d;
  rn.eps = m.rms_eps;
  rn.partial = c.partial.p;
  rn.split_stride = (long long)R * d;
  const double rn_bytes = (double)R * d * (4 + 4 + 2);
  for (int l = 0; l < m.n_layers; ++l) {
    LayerWeights& L = c.layers[l];
    int z = project(c, c.h_bf16.p, (long long)(c.h_bf16.n / 2), d, L.wqkv_p.p, R, c.qkv_dim, d);
    AttnArgs at{};
    at.out = c.attn_bf16.p;
    at.out_lo_offset = (long long)(c.attn_bf16.n / 2);
    at.kv_pool = (const uint16_t*)c.kv_pool.p;
    at.geom = c.geom;
    at.page_table = c.d_page_table.p;
    at.max_pages = c.max_pages;
    at.layer = l;
    at.n_q_heads = m.n_q_heads;
    // algorithmic bytes: every cached position once, a prompt's shared pages once for all its samples
    // Rows [0, Bd) are decode rows (one per live sample), rows [Bd, R) packed sequences; a step of
    // the queue-fed rollout with a chunk of prompt rows has both.
    const int Bd = seqs ? seqs->decode_rows : R, Rq = R - Bd;
    const double kv_unit = (double)m.n_kv_heads * 128 * 2 * 2;
    if (Rq > 0) {
      // packed sequences: sum the planes, rotate, write the KV pages, then causal attention
      const double kv_bytes = (Bd ? c.chunk_kv_tokens : c.kv_tokens_this_call) * kv_unit;
      QkvPostArgs qp{};
      qp.partial = c.partial.p + (size_t)Bd * c.qkv_dim;
      qp.split_stride = (long long)R * c.qkv_dim;
      qp.splits = z;
      qp.cos_sin = c.cos_sin.p;
      qp.row_pos = c.row_pos.p + Bd;
      qp.row_slot = c.row_slot.p + Bd;
      qp.page_table = c.d_page_table.p;
      qp.max_pages = c.max_pages;
      qp.q_bf16 = c.q_bf16.p + (size_t)Bd * c.q_dim;
      qp.q_lo_offset = (long long)(c.q_bf16.n / 2);
      qp.kv_pool = (uint16_t*)c.kv_pool.p;
      qp.geom = c.geom;
      qp.layer = l;
      qp.rows = Rq;
      qp.n_q_heads = m.n_q_heads;
      qp.extra = QkvExtras{L.qkv_bias.p, L.q_gain.p, L.k_gain.p, m.rms_eps};
      c.timer.begin("qkv_post_kernel", (double)Rq * c.qkv_dim * (4 + 2), 0, s);
      launch_qkv_post(qp, s);
      c.timer.end(s);
      at.q = c.q_bf16.p;
      at.q_lo_offset = (long long)(c.q_bf16.n / 2);
      at.seq_row0 = seqs->row0;
      at.seq_len = seqs->len;
      at.seq_slot = seqs->slot;
      at.seq_pos0 = seqs->pos0;
      at.n_seqs = seqs->n_seqs;
      at.max_seq_len = seqs->max_len;
      c.timer.begin("attn_prefill_kernel", kv_bytes + 4.0 * Rq * c.q_dim, Bd ? c.chunk_attn_flops : c.attn_flops_this_call, s);
      launch_attention_prefill(at, s);
      c.timer.end(s);
    }
    if (Bd > 0) {
      // one row per sample: the fused decode attention sums the projection's planes itself
      const double kv_bytes = c.kv_unique_tokens_this_call * kv_unit;
      at.kv_pool_w = (uint16_t*)c.kv_pool.p;
      at.row_pos = c.row_pos.p;
      at.row_slot = c.row_slot.p;
      at.rows = Bd;
      at.qkv_raw = c.partial.p;
      at.qkv_planes = z;
      at.qkv_plane_stride = (long long)R * c.qkv_dim;
      at.cos_sin = c.cos_sin.p;
      at.extra = QkvExtras{L.qkv_bias.p, L.q_gain.p, L.k_gain.p, m.rms_eps};
      const int base = Bd * m.n_kv_heads;
      at.part_o = c.attn_part_o.p;
      at.part_ml = c.attn_part_ml.p;
      const double qo_bytes = (double)Bd * (4.0 * z * c.qkv_dim + 4.0 * c.q_dim);
      if (c.use_groups) {
        // shared prompts by group, in splits of at least 128 positions that give every CU a
        // workgroup; own ranges in splits of 1024 or more (few, long-lived workgroups: one round on the chip)
        at.row_t0 = c.row_t0.p;
        at.grp_rows = c.grp_rows.p;
        at.grp_len = c.grp_len.p;
        at.grp_slot = c.grp_slot.p;
        at.n_groups = c.n_groups;
        const int want_a = std::max(1, std::min(4, ceil_div(128, c.n_groups * m.n_kv_heads)));
        at.split_tokens_a = ceil_div(ceil_div(c.max_shared, want_a), 128) * 128;
        at.n_splits_a = ceil_div(c.max_shared, at.split_tokens_a);
        at.slot0 = at.n_splits_a;
        const int max_own = std::min(16 - at.slot0, std::max(1, c.attn_max_parts / base - at.slot0));
        at.split_tokens = std::max(1024, ceil_div(ceil_div(c.decode_max_own, max_own), 128) * 128);
        at.n_splits = ceil_div(c.decode_max_own, at.split_tokens);
        at.n_slots = at.slot0 + at.n_splits;
        const int G = m.n_q_heads / m.n_kv_heads;
        static const char* const names[2][2] = {
            {"attn_decode_grouped_kernel<1,false>", "attn_decode_grouped_kernel<1,true>"},
            {"attn_decode_grouped_kernel<2,false>", "attn_decode_grouped_kernel<2,true>"}};
        c.timer.begin(names[GROUP_MEMBERS * G <= 16 ? 0 : 1][at.extra.bias || at.extra.q_gain ? 1 : 0],
                      kv_bytes + qo_bytes, c.attn_flops_this_call, s);
        launch_attention_decode_grouped(at, s);
        c.timer.end(s);
        merge_attention_slots(c, at, Bd);
      } else {
        const int n_splits = decode_attention_splits(c, base);
        at.split_tokens = ceil_div(ceil_div(c.decode_max_ctx, n_splits), 128) * 128;
        at.n_splits = ceil_div(c.decode_max_ctx, at.split_tokens);
        c.timer.begin(at.extra.bias || at.extra.q_gain ? "attn_decode_fused_kernel<true>" : "attn_decode_fused_kernel<false>",
                      kv_bytes + qo_bytes, c.attn_flops_this_call, s);
        launch_attention_decode_fused(at, s);
        c.timer.end(s);
        if (at.n_splits > 1) merge_attention_slots(c, at, Bd);
      }
    }

    z = project(c, c.attn_bf16.p, (long long)(c.attn_bf16.n / 2), c.q_dim, L.wo_p.p, R, d, c.q_dim);
    rn.splits = z;
    rn.gain = L.norm2.p;
    c.timer.begin("row_norm_kernel", rn_bytes + 4.0 * z * R * d, 0, s);
    launch_row_norm(rn, s);
    c.timer.end(s);

    const float* next_gain = l + 1 < m.n_layers ? c.layers[l + 1].norm1.p : c.final_norm.p;
    if (m.n_experts > 0) {
      moe_block(c, L, l, R, rn, next_gain);
      continue;
    }
    gate_up(c, L, R);

    z = project(c, c.act_bf16.p, (long long)(c.act_bf16.n / 2), f, L.w_down_p.p, R, d, f);
    rn.splits = z;
    rn.gain = next_gain;
    c.timer.begin("row_norm_kernel", rn_bytes + 4.0 * z * R * d, 0, s);
    launch_row_norm(rn, s);
    c.timer.end(s);
  }
  c.h_is_final = false;
}

// ------------------------------------------------------------------------------------------
// Matrix-core path, one decode step with at most 32 live samples: five launches per layer
// (six when attention is split over the cached positions).
//   QKV projection -> fused attention (rotary, KV-page write, paged attention) -> O projection
//   with the residual add -> gate/up projection with SwiGLU -> down projection with the
//   residual add.
// RMSNorm is split around the launches: a residual-producing epilogue stores x * gain and
// partial sums of squares, the consuming projection scales its output rows by
// rsqrt(mean + eps).  The last down projection uses the final norm's gain, so the logits
// projection reads its operand directly.
static void stream_project(rollout_ctx& c, const DevBuf<uint16_t>& a, int lda, const void* w, int M, int N, int K,
                           int epi, bool normalise_input, void* out, int ldo, long long out_lo_offset,
                           const float* resid_gain, const TouchRange& touch = TouchRange{}) {
  GemmArgs g{};
  g.touch = touch;
  g.a = a.p;
  g.a_lo = a.p + a.n / 2;
  g.w = w;
  g.out = out;
  g.out_lo_offset = out_lo_offset;
  g.M = M;
  g.N = N;
  g.K = K;
  g.lda = lda;
  g.ldo = ldo;
  g.frag = true;  // every operand plane of this path is in fragment order
  g.eps = c.md.rms_eps;
  g.ssq_stride = 256;
  if (normalise_input) {
    g.rinv_ssq = c.ssq.p;
    g.rinv_partials = c.ssq_partials;
  }
  const GemmPlan pl = gemm_plan(M, N, K, epi, 1);
  double bytes = 2.0 * N * K + 2.0 * 2 * M * K;  // weights once, both activation planes once
  if (epi == EPI_RESID) {
    g.x = c.x.p;
    g.gain = resid_gain;
    g.h = c.h_bf16.p;
    g.h_lo_offset = (long long)(c.h_bf16.n / 2);
    g.ssq_out = c.ssq.p;
    bytes += (double)M * N * (4 + 4 + 2 + 2);  // x read and written, two operand planes written
  } else if (epi == EPI_SWIGLU_BF16) {
    bytes += (double)M * (N / 2) * (2 + 2);
  } else {
    bytes += 4.0 * M * N;
  }
  c.timer.begin(pl.name, bytes, 2.0 * M * N * K, c.stream);
  launch_gemm_bf16(g, epi, pl, c.stream);
  c.timer.end(c.stream);
  if (epi == EPI_RESID) c.ssq_partials = ceil_div(N >> 4, pl.nt);
}

static void forward_rows_decode(rollout_ctx& c, int R) {
  const rollout_model_desc& m = c.md;
  hipStream_t s = c.stream;
  const int d = m.hidden, f = m.ffn_dim;
  {
    RowNormArgs rn{};
    rn.x = c.x.p;
    rn.h = c.h_bf16.p;
    rn.h_lo_offset = (long long)(c.h_bf16.n / 2);
    rn.rows = R;
    rn.hidden = d;
    rn.eps = m.rms_eps;
    rn.tokens = c.row_token.p;
    rn.embed = (const uint16_t*)c.embed.p;
    rn.gain = c.layers[0].norm1.p;
    rn.ssq_out = c.ssq.p;
    rn.h_frag = true;
    c.timer.begin("row_norm_kernel", (double)R * d * (2 + 4 + 2 + 2), 0, s);
    launch_row_norm(rn, s);
    c.timer.end(s);
    c.ssq_partials = 1;
  }
  for (int l = 0; l < m.n_layers; ++l) {
    LayerWeights& L = c.layers[l];
    // The down projection has only hidden/16 workgroups, each streaming a deep slice: it is the
    // one projection here that gains more from finding its weights in the memory-side cache
    // (11 -> 7 us at config 2's shape) than walking them costs the launch that hosts the walk
    // (the QKV projection, which leaves half the CUs idle: +1.6 us).  Hosted by the attention
    // or O-projection launch, or done for the gate/up weights, the walk cost what it gained.
    TouchRange down_touch;
    if (L.w_down_p.n <= ((size_t)64 << 20)) {
      down_touch.p = L.w_down_p.p;
      down_touch.lines = (long long)(L.w_down_p.n / 128);
      down_touch.wgs = 128;
    }
    stream_project(c, c.h_bf16, d, L.wqkv_p.p, R, c.qkv_dim, d, EPI_F32, true, c.partial.p, c.qkv_dim, 0, nullptr,
                   down_touch);

    AttnArgs at{};
    at.out = c.attn_bf16.p;
    at.out_lo_offset = (long long)(c.attn_bf16.n / 2);
    at.out_frag = true;
    at.kv_pool = (const uint16_t*)c.kv_pool.p;
    at.kv_pool_w = (uint16_t*)c.kv_pool.p;
    at.geom = c.geom;
    at.page_table = c.d_page_table.p;
    at.max_pages = c.max_pages;
    at.layer = l;
    at.n_q_heads = m.n_q_heads;
    at.row_pos = c.row_pos.p;
    at.row_slot = c.row_slot.p;
    at.rows = R;
    at.qkv_raw = c.partial.p;
    at.qkv_planes = 1;
    at.cos_sin = c.cos_sin.p;
    at.extra = QkvExtras{L.qkv_bias.p, L.q_gain.p, L.k_gain.p, m.rms_eps};
    const int base = R * m.n_kv_heads;
    const int n_splits = decode_attention_splits(c, base);
    at.split_tokens = ceil_div(ceil_div(c.decode_max_ctx, n_splits), 128) * 128;
    at.n_splits = ceil_div(c.decode_max_ctx, at.split_tokens);
    at.part_o = c.attn_part_o.p;
    at.part_ml = c.attn_part_ml.p;
    // every cached key and value once (a shared prompt once for all its samples), q in, out
    c.timer.begin(at.extra.bias || at.extra.q_gain ? "attn_decode_fused_kernel<true>" : "attn_decode_fused_kernel<false>",
                  c.kv_unique_tokens_this_call * (double)m.n_kv_heads * 128 * 2 * 2 + (double)R * (4.0 * c.qkv_dim + 4.0 * c.q_dim),
                  c.attn_flops_this_call, s);
    launch_attention_decode_fused(at, s);
    c.timer.end(s);
    if (at.n_splits > 1) merge_attention_slots(c, at, R);

    stream_project(c, c.attn_bf16, c.q_dim, L.wo_p.p, R, d, c.q_dim, EPI_RESID, false, nullptr, d, 0, L.norm2.p);
    stream_project(c, c.h_bf16, d, L.w_gate_up_p.p, R, 2 * f, d, EPI_SWIGLU_BF16, true, c.act_bf16.p, f,
                   (long long)(c.act_bf16.n / 2), nullptr);
    stream_project(c, c.act_bf16, f, L.w_down_p.p, R, d, f, EPI_RESID, false, nullptr, d, 0,
                   l + 1 < m.n_layers ? c.layers[l + 1].norm1.p : c.final_norm.p);
  }
  c.h_is_final = true;
}

void engine_forward_rows(rollout_ctx& c, int rows, const SeqBatch* seqs) {
  if (rows < 1) return;
  c.last_route_rows = rows;
  if (!c.simple) {
    if (!seqs && rows <= 32 && !c.md.n_experts)
      forward_rows_decode(c, rows);
    else
      forward_rows_tiled(c, rows, seqs);
  } else if (c.md.dtype == ROLLOUT_DTYPE_F32) {
    forward_rows_simple<float, float>(c, rows);
  } else {
    forward_rows_simple<bf16_t, f16_t>(c, rows);
  }
}

void engine_logits(rollout_ctx& c, const int* rows_index, int first, int n, float* out) {
  if (n < 1) return;
  const int d = c.md.hidden;
  if (!c.simple) {
    const uint16_t* hn = c.hn_bf16.p;
    long long hn_lo = (long long)(c.hn_bf16.n / 2);
    const bool from_h = c.h_is_final && !rows_index && first == 0;
    if (from_h) {
      hn = c.h_bf16.p;  // the fused decode path already applied the final norm's gain
      hn_lo = (long long)(c.h_bf16.n / 2);
    } else {
      RowNormArgs rn{};
      rn.x = c.x.p + (size_t)first * d;
      rn.h = c.hn_bf16.p;
      rn.h_lo_offset = hn_lo;
      rn.gain = c.final_norm.p;
      rn.rows_index = rows_index;
      rn.rows = n;
      rn.hidden = d;
      rn.eps = c.md.rms_eps;
      c.timer.begin("row_norm_kernel", (double)n * d * (4 + 2), 0, c.stream);
      launch_row_norm(rn, c.stream);
      c.timer.end(c.stream);
    }
    GemmArgs g{};
    g.a = hn;
    g.a_lo = hn + hn_lo;
    if (from_h) {  // h holds x * gain in fragment order; the rsqrt factor rides in the epilogue
      g.frag = true;
      g.rinv_ssq = c.ssq.p;
      g.rinv_partials = c.ssq_partials;
      g.ssq_stride = 256;
      g.eps = c.md.rms_eps;
    }
    g.w = c.lm_head_p.p;
    g.out = out;
    g.M = n;
    g.N = c.md.vocab;
    g.K = d;
    g.lda = d;
    g.ldo = c.md.vocab;
    const GemmPlan pl = gemm_plan(n, g.N, d, EPI_F32, 1);
    c.timer.begin(pl.name, gemm_bytes(n, g.N, d, 4), 2.0 * n * g.N * d, c.stream);
    launch_gemm_bf16(g, EPI_F32, pl, c.stream);
    c.timer.end(c.stream);
    return;
  }
  launch_rmsnorm_f32(c.x.p + (size_t)first * d, c.final_norm.p, c.hn.p, rows_index, n, d, c.md.rms_eps, c.stream);
  if (c.md.dtype == ROLLOUT_DTYPE_F32)
    launch_linear_simple<float>(c.hn.p, d, (const float*)c.lm_head.p, out, c.md.vocab, nullptr, 0, n, c.md.vocab,
                                d, c.stream);
  else
    launch_linear_simple<bf16_t>(c.hn.p, d, (const bf16_t*)c.lm_head.p, out, c.md.vocab, nullptr, 0, n,
                                 c.md.vocab, d, c.stream);
}

// Teacher-forced log-probs without materialising logits (matrix-core path): final norm into
// the operand planes, then the logits projection with the log-sum-exp epilogue, then one
// small pass over the per-workgroup parts.  The plain path stores logits chunk by chunk.
void engine_target_logprobs(rollout_ctx& c, int n, const int* target, float inv_t, float* out) {
  if (n < 1) return;
  const int d = c.md.hidden, V = c.md.vocab;
  if (c.simple) {
    for (int off = 0; off < n; off += c.logit_rows) {
      const int nr = std::min(c.logit_rows, n - off);
      engine_logits(c, nullptr, off, nr, c.logits.p);
      launch_logprob_gather(c.logits.p, target + off, inv_t, out + off, nr, V, c.stream);
    }
    return;
  }
  RowNormArgs rn{};
  rn.x = c.x.p;
  rn.h = c.h_bf16.p;  // the layers' operand buffer is free after the forward pass
  rn.h_lo_offset = (long long)(c.h_bf16.n / 2);
  rn.gain = c.final_norm.p;
  rn.rows = n;
  rn.hidden = d;
  rn.eps = c.md.rms_eps;
  c.timer.begin("row_norm_kernel", (double)n * d * (4 + 2 + 2), 0, c.stream);
  launch_row_norm(rn, c.stream);
  c.timer.end(c.stream);
  c.h_is_final = false;

  GemmArgs g{};
  g.a = c.h_bf16.p;
  g.a_lo = c.h_bf16.p + c.h_bf16.n / 2;
  g.w = c.lm_head_p.p;
  g.M = n;
  g.N = V;
  g.K = d;
  g.lda = d;
  g.lse_target = target;
  g.lse_scale = inv_t;
  g.lse_max = c.lse_max.p;
  g.lse_sum = c.lse_sum.p;
  g.lse_tgt = c.lse_tgt.p;
  g.lse_stride = c.r_max;
  const GemmPlan pl = gemm_plan(n, V, d, EPI_LSE, 1);
  const int parts = lse_parts(pl, V);
  // weights and operand planes once; the parts written and read back are the only result traffic
  c.timer.begin(pl.name, 2.0 * V * d + 4.0 * n * d + 16.0 * parts * n, 2.0 * n * V * d, c.stream);
  launch_gemm_bf16(g, EPI_LSE, pl, c.stream);
  c.timer.end(c.stream);
  c.timer.begin("lse_finish_kernel", 8.0 * parts * n, 0, c.stream);
  launch_lse_finish(c.lse_max.p, c.lse_sum.p, c.lse_tgt.p, target, parts, c.r_max, n, out, c.stream);
  c.timer.end(c.stream);
}
