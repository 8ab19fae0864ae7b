// Temperature / top-p sampling over the full vocabulary on integer weights, the
// Philox4x32-10 generator that drives it, and the log-prob gather of the teacher-forced
// pass.  The paper leaves the sampler to its serving engines (section 2.1: the actor
// generates tokens until the termination criteria are met); the integer procedure below
// exists so that a drawn token id is one exact function of (logits row, temperature,
// top-p, 32-bit word) whatever the reduction order:
//   z = logit * inv_T; d = z - max z; w = floor(P(frac(t)) * 2^(40 + floor(t))), t = d*log2(e),
//   w = 0 for t < -40; S = sum w; nucleus = shortest prefix in (w desc, id asc) order whose
//   weight reaches theta = max(1, floor(S * floor(top_p 2^24) / 2^24)); R = floor(S_N x / 2^32);
//   token = first id of the nucleus, ascending, whose running weight exceeds R.
// Every floating-point step is a single rounded fp32 operation: no contraction allowed.
#include <algorithm>

#include "kernels.h"

#pragma clang fp contract(off)

#define SAMP_T 1024

__device__ inline unsigned long long fixexp_weight(float d) {
#pragma clang fp contract(off)
  const float log2e = 0x1.715476p+0f;
  float t = d * log2e;
  if (!(t >= -40.0f)) return 0ull;
  float n = floorf(t);
  float f = t - n;
  float y = 0x1.5bd2aep-16f;
  y = y * f;
  y = y + 0x1.3262dep-13f;
  y = y * f;
  y = y + 0x1.5efc6ap-10f;
  y = y * f;
  y = y + 0x1.3b1a32p-7f;
  y = y * f;
  y = y + 0x1.c6b140p-5f;
  y = y * f;
  y = y + 0x1.ebfbdep-3f;
  y = y * f;
  y = y + 0x1.62e430p-1f;
  y = y * f;
  y = y + 0x1.000000p+0f;
  // floor(y * 2^(40 + n)) from the bits of y: y = mant * 2^(e - 23)
  unsigned bits = __float_as_uint(y);
  int e = (int)((bits >> 23) & 0xffu) - 127;
  unsigned long long mant = (unsigned long long)((bits & 0x7fffffu) | 0x800000u);
  int shift = e - 23 + 40 + (int)n;
  return shift >= 0 ? (mant << shift) : (shift > -64 ? (mant >> (-shift)) : 0ull);
}

__device__ inline float scaled_logit(float logit, float inv_t) {
#pragma clang fp contract(off)
  return logit * inv_t;
}
__device__ inline float shifted(float z, float m) {
#pragma clang fp contract(off)
  return z - m;
}

__device__ inline unsigned long long shfl_up_u64(unsigned long long v, int o) {
  unsigned lo = __shfl_up((unsigned)(v & 0xffffffffull), o, WAVE);
  unsigned hi = __shfl_up((unsigned)(v >> 32), o, WAVE);
  return ((unsigned long long)hi << 32) | lo;
}

struct SampShared {
  unsigned long long vals[SAMP_T];
  unsigned long long wave_part[SAMP_T / WAVE];
  unsigned long long bcast[2];
  float fwave[SAMP_T / WAVE];
};

__device__ inline float block_max(float v, SampShared& sh) {
  v = wave_max(v);
  if ((threadIdx.x & 63) == 0) sh.fwave[threadIdx.x >> 6] = v;
  __syncthreads();
  float m = sh.fwave[0];
  for (int i = 1; i < SAMP_T / WAVE; ++i) m = fmaxf(m, sh.fwave[i]);
  __syncthreads();
  return m;
}

__device__ inline unsigned long long block_sum_u64(unsigned long long v, SampShared& sh) {
  v = wave_sum_u64(v);
  if ((threadIdx.x & 63) == 0) sh.wave_part[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long s = 0;
  for (int i = 0; i < SAMP_T / WAVE; ++i) s += sh.wave_part[i];
  __syncthreads();
  return s;
}

// Smallest thread index whose inclusive prefix of `local` exceeds `target`, and the
// exclusive prefix before that thread.  Requires sum(local) > target.
__device__ inline void block_find(unsigned long long local, unsigned long long target, SampShared& sh,
                                  int& t_star, unsigned long long& before) {
  int tid = threadIdx.x;
  sh.vals[tid] = local;
  if (tid == 0) {
    sh.bcast[0] = 0;
    sh.bcast[1] = 0;
  }
  __syncthreads();
  if (tid < WAVE) {
    const int per = SAMP_T / WAVE;
    unsigned long long mine = 0;
    for (int j = 0; j < per; ++j) mine += sh.vals[tid * per + j];
    unsigned long long inc = mine;
    for (int o = 1; o < WAVE; o <<= 1) {
      unsigned long long up = shfl_up_u64(inc, o);
      if (tid >= o) inc += up;
    }
    unsigned long long exc = inc - mine;
    if (exc <= target && target < inc) {
      unsigned long long acc = exc;
      int j = 0;
      for (; j < per - 1; ++j) {
        unsigned long long v = sh.vals[tid * per + j];
        if (acc + v > target) break;
        acc += v;
      }
      sh.bcast[0] = (unsigned long long)(tid * per + j);
      sh.bcast[1] = acc;
    }
  }
  __syncthreads();
  t_star = (int)sh.bcast[0];
  before = sh.bcast[1];
  __syncthreads();
}

__device__ inline void philox_round(unsigned& c0, unsigned& c1, unsigned& c2, unsigned& c3, unsigned k0,
                                    unsigned k1) {
  const unsigned MA = 0xD2511F53u, MB = 0xCD9E8D57u;
  unsigned hi0 = __umulhi(MA, c0), lo0 = MA * c0;
  unsigned hi1 = __umulhi(MB, c2), lo1 = MB * c2;
  unsigned n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
  c0 = n0;
  c1 = lo1;
  c2 = n2;
  c3 = lo0;
}
// Philox4x32-10 (Salmon et al., SC'11), output word 0.
__device__ inline unsigned philox_word0(unsigned long long seed, unsigned long long sample_id, unsigned step) {
  unsigned k0 = (unsigned)seed, k1 = (unsigned)(seed >> 32);
  unsigned c0 = (unsigned)sample_id, c1 = (unsigned)(sample_id >> 32), c2 = step, c3 = 0u;
  for (int r = 0; r < 10; ++r) {
    philox_round(c0, c1, c2, c3, k0, k1);
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}

__global__ void philox_words_kernel(unsigned long long seed, const long long* __restrict__ ids,
                                    const unsigned* __restrict__ steps, unsigned* __restrict__ out, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = philox_word0(seed, (unsigned long long)ids[i], steps[i]);
}
void launch_philox_words(unsigned long long seed, const long long* ids, const unsigned* steps, unsigned* out,
                         int n, hipStream_t s) {
  if (n) philox_words_kernel<<<ceil_div(n, 256), 256, 0, s>>>(seed, ids, steps, out, n);
}

// The vocabulary is walked in segments of 256 consecutive ids: one wavefront, 4 ids per lane,
// 16 segments per 4096-id tile of the block.  Every pass is a coalesced sweep that leaves one
// value per segment in LDS; a prefix search over at most 1024 segment values then names the
// segment that holds the id in question, and one wavefront resolves it inside the segment.
struct Seg4 {
  unsigned long long w[4];
};

__device__ inline Seg4 load_weights4(const float* __restrict__ row, int i0, int vocab, bool vec_ok, float inv_t,
                                     float m) {
  float v[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  if (vec_ok && i0 + 3 < vocab) {
    const float4 t = *(const float4*)(row + i0);
    v[0] = t.x;
    v[1] = t.y;
    v[2] = t.z;
    v[3] = t.w;
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (i0 + e < vocab) v[e] = row[i0 + e];
  }
  Seg4 out;
#pragma unroll
  for (int e = 0; e < 4; ++e) out.w[e] = i0 + e < vocab ? fixexp_weight(shifted(scaled_logit(v[e], inv_t), m)) : 0ull;
  return out;
}

// Smallest segment whose inclusive prefix of sh.vals[0..n_seg) exceeds target, and the
// exclusive prefix before it.  Requires the total to exceed target.
__device__ inline void find_segment(SampShared& sh, int n_seg, unsigned long long target, int& seg,
                                    unsigned long long& before) {
  const int tid = threadIdx.x;
  if (tid == 0) {
    sh.bcast[0] = 0;
    sh.bcast[1] = 0;
  }
  __syncthreads();
  if (tid < WAVE) {
    const int per = SAMP_T / WAVE;
    unsigned long long mine = 0;
    for (int j = 0; j < per; ++j) mine += tid * per + j < n_seg ? sh.vals[tid * per + j] : 0ull;
    unsigned long long inc = mine;
    for (int o = 1; o < WAVE; o <<= 1) {
      unsigned long long up = shfl_up_u64(inc, o);
      if (tid >= o) inc += up;
    }
    unsigned long long exc = inc - mine;
    if (exc <= target && target < inc) {
      unsigned long long acc = exc;
      int j = 0;
      for (; j < per - 1; ++j) {
        unsigned long long v = tid * per + j < n_seg ? sh.vals[tid * per + j] : 0ull;
        if (acc + v > target) break;
        acc += v;
      }
      sh.bcast[0] = (unsigned long long)(tid * per + j);
      sh.bcast[1] = acc;
    }
  }
  __syncthreads();
  seg = (int)sh.bcast[0];
  before = sh.bcast[1];
  __syncthreads();
}

// One wavefront: index of the element of its 4-per-lane values whose running sum first exceeds
// target (values in ascending id order: lane-major, element-minor).
__device__ inline int resolve_in_segment(const unsigned long long (&v)[4], unsigned long long target, int lane) {
  const unsigned long long mine = v[0] + v[1] + v[2] + v[3];
  unsigned long long inc = mine;
  for (int o = 1; o < WAVE; o <<= 1) {
    unsigned long long up = shfl_up_u64(inc, o);
    if (lane >= o) inc += up;
  }
  const unsigned long long exc = inc - mine;
  int found = -1;
  if (exc <= target && target < inc) {
    unsigned long long acc = exc;
    found = lane * 4 + 3;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc += v[e];
      if (acc > target && found == lane * 4 + 3) found = lane * 4 + e;
    }
  }
  // exactly one lane found it
  for (int o = WAVE / 2; o > 0; o >>= 1) found = max(found, __shfl_xor(found, o, WAVE));
  return found;
}

// First sweep on `parts` workgroups per row: maximum of the scaled logits over tiles
// blockIdx.x, blockIdx.x + parts, ...
__global__ __launch_bounds__(SAMP_T) void sample_max_kernel(SampleRows a, int vocab, int parts) {
  __shared__ SampShared sh;
  const int tid = threadIdx.x, r = blockIdx.y;
  const float* row = a.logits + (long long)(a.logits_row ? a.logits_row[r] : r) * vocab;
  const float inv_t = a.inv_temp[r];
  const bool vec_ok = (vocab & 3) == 0 && (((unsigned long long)row) & 15ull) == 0;
  const int n_tiles = (vocab + 4095) >> 12;
  float m = -INFINITY;
  for (int t = blockIdx.x; t < n_tiles; t += parts) {
    const int i0 = t * 4096 + tid * 4;
    if (vec_ok && i0 + 3 < vocab) {
      const float4 v = *(const float4*)(row + i0);
      m = fmaxf(fmaxf(m, fmaxf(scaled_logit(v.x, inv_t), scaled_logit(v.y, inv_t))),
                fmaxf(scaled_logit(v.z, inv_t), scaled_logit(v.w, inv_t)));
    } else {
      for (int e = 0; e < 4; ++e)
        if (i0 + e < vocab) m = fmaxf(m, scaled_logit(row[i0 + e], inv_t));
    }
  }
  m = block_max(m, sh);
  if (tid == 0) a.part_max[(long long)r * kSampleParts + blockIdx.x] = m;
}

// Second sweep on `parts` workgroups per row: the weights of the same tiles, one sum per
// 256-id segment.
__global__ __launch_bounds__(SAMP_T) void sample_segments_kernel(SampleRows a, int vocab, int parts) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = blockIdx.y;
  const float* row = a.logits + (long long)(a.logits_row ? a.logits_row[r] : r) * vocab;
  const float inv_t = a.inv_temp[r];
  const bool vec_ok = (vocab & 3) == 0 && (((unsigned long long)row) & 15ull) == 0;
  const int n_seg = (vocab + 255) >> 8;
  const int n_tiles = (vocab + 4095) >> 12;
  float m = -INFINITY;
  for (int q = 0; q < parts; ++q) m = fmaxf(m, a.part_max[(long long)r * kSampleParts + q]);
  for (int t = blockIdx.x; t < n_tiles; t += parts) {
    const Seg4 q = load_weights4(row, t * 4096 + tid * 4, vocab, vec_ok, inv_t, m);
    const unsigned long long ws = wave_sum_u64(q.w[0] + q.w[1] + q.w[2] + q.w[3]);
    if (lane == 0 && t * 16 + wave < n_seg) a.seg_sums[(long long)r * kSampleSegments + t * 16 + wave] = ws;
  }
}

// parts = 0: this kernel sweeps the row itself; else it starts from what the two kernels above left
__global__ __launch_bounds__(SAMP_T) void sample_kernel(SampleRows a, int vocab, int parts) {
  __shared__ SampShared sh;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = blockIdx.x;
  const float* row = a.logits + (long long)(a.logits_row ? a.logits_row[r] : r) * vocab;
  const float inv_t = a.inv_temp[r];
  const bool vec_ok = (vocab & 3) == 0 && (((unsigned long long)row) & 15ull) == 0;
  const int n_seg = (vocab + 255) >> 8;
  const int n_tiles = (vocab + 4095) >> 12;

  float m = -INFINITY;
  unsigned long long local = 0;
  if (parts) {
    for (int q = 0; q < parts; ++q) m = fmaxf(m, a.part_max[(long long)r * kSampleParts + q]);
    if (tid < n_seg) {
      local = a.seg_sums[(long long)r * kSampleSegments + tid];
      sh.vals[tid] = local;
    }
  } else {
    for (int t = 0; t < n_tiles; ++t) {
      const int i0 = t * 4096 + tid * 4;
      if (vec_ok && i0 + 3 < vocab) {
        const float4 v = *(const float4*)(row + i0);
        m = fmaxf(fmaxf(m, fmaxf(scaled_logit(v.x, inv_t), scaled_logit(v.y, inv_t))),
                  fmaxf(scaled_logit(v.z, inv_t), scaled_logit(v.w, inv_t)));
      } else {
        for (int e = 0; e < 4; ++e)
          if (i0 + e < vocab) m = fmaxf(m, scaled_logit(row[i0 + e], inv_t));
      }
    }
    m = block_max(m, sh);

    // pass: all weights, one sum per segment
    for (int t = 0; t < n_tiles; ++t) {
      const Seg4 q = load_weights4(row, t * 4096 + tid * 4, vocab, vec_ok, inv_t, m);
      const unsigned long long mine = q.w[0] + q.w[1] + q.w[2] + q.w[3];
      local += mine;
      const unsigned long long ws = wave_sum_u64(mine);
      if (lane == 0 && t * 16 + wave < n_seg) sh.vals[t * 16 + wave] = ws;
    }
  }
  const unsigned long long S = block_sum_u64(local, sh);  // also orders the writes to sh.vals

  int token = a.forced ? a.forced[r] : -1;
  if ((unsigned)token >= (unsigned)vocab) {  // nothing forced (an id outside the vocabulary forces nothing)
    const float top_p = a.top_p[r];
    // nucleus membership: w > tau, or w == tau and id <= tie_cut
    unsigned long long tau = 0, s_n = S;
    int tie_cut = vocab;
    if (top_p < 1.0f) {
      unsigned long long p24 = (unsigned long long)floorf(fmaxf(top_p, 0.f) * 16777216.0f);
      unsigned long long theta = (S >> 24) * p24 + (((S & 0xffffffull) * p24) >> 24);
      if (theta < 1) theta = 1;
      // largest tau with sum_{w >= tau} w >= theta, bit by bit (w <= 2^40)
      for (int b = 40; b >= 0; --b) {
        const unsigned long long cand = tau | (1ull << b);
        unsigned long long part = 0;
        for (int t = 0; t < n_tiles; ++t) {
          const Seg4 q = load_weights4(row, t * 4096 + tid * 4, vocab, vec_ok, inv_t, m);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (q.w[e] >= cand) part += q.w[e];
        }
        if (block_sum_u64(part, sh) >= theta) tau = cand;
      }
      // weight above tau, and ties at tau counted per segment
      unsigned long long above = 0;
      for (int t = 0; t < n_tiles; ++t) {
        const Seg4 q = load_weights4(row, t * 4096 + tid * 4, vocab, vec_ok, inv_t, m);
        unsigned long long ties = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (q.w[e] > tau) above += q.w[e];
          if (q.w[e] == tau) ties += 1;
        }
        const unsigned long long ws = wave_sum_u64(ties);
        if (lane == 0 && t * 16 + wave < n_seg) sh.vals[t * 16 + wave] = ws;
      }
      const unsigned long long sum_above = block_sum_u64(above, sh);
      const unsigned long long need = theta - sum_above;         // > 0 by maximality of tau
      const unsigned long long k_ties = (need + tau - 1) / tau;  // ties admitted, ascending id
      int seg;
      unsigned long long before;
      find_segment(sh, n_seg, k_ties - 1, seg, before);
      if (wave == 0) {
        const Seg4 q = load_weights4(row, seg * 256 + lane * 4, vocab, vec_ok, inv_t, m);
        const unsigned long long is_tie[4] = {q.w[0] == tau, q.w[1] == tau, q.w[2] == tau, q.w[3] == tau};
        const int idx = resolve_in_segment(is_tie, k_ties - 1 - before, lane);
        if (lane == 0) sh.bcast[0] = (unsigned long long)(seg * 256 + idx);
      }
      __syncthreads();
      tie_cut = (int)sh.bcast[0];
      __syncthreads();
      s_n = sum_above + k_ties * tau;
      // nucleus weight per segment
      for (int t = 0; t < n_tiles; ++t) {
        const int i0 = t * 4096 + tid * 4;
        const Seg4 q = load_weights4(row, i0, vocab, vec_ok, inv_t, m);
        unsigned long long mine = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (q.w[e] > tau || (q.w[e] == tau && i0 + e <= tie_cut)) mine += q.w[e];
        const unsigned long long ws = wave_sum_u64(mine);
        if (lane == 0 && t * 16 + wave < n_seg) sh.vals[t * 16 + wave] = ws;
      }
      __syncthreads();
    }
    // inverse CDF in ascending id order over the nucleus
    const unsigned x = a.uniforms ? a.uniforms[r]
                                  : philox_word0(a.seed, (unsigned long long)a.sample_id[r], (unsigned)a.step[r]);
    const unsigned long long R = (s_n >> 32) * x + (((s_n & 0xffffffffull) * x) >> 32);
    int seg;
    unsigned long long before;
    find_segment(sh, n_seg, R, seg, before);
    if (wave == 0) {
      const int i0 = seg * 256 + lane * 4;
      const Seg4 q = load_weights4(row, i0, vocab, vec_ok, inv_t, m);
      unsigned long long v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (q.w[e] > tau || (q.w[e] == tau && i0 + e <= tie_cut)) ? q.w[e] : 0ull;
      const int idx = resolve_in_segment(v, R - before, lane);
      if (lane == 0) sh.bcast[0] = (unsigned long long)(seg * 256 + idx);
    }
    __syncthreads();
    token = (int)sh.bcast[0];
  }
  if (tid == 0) {
    float d = shifted(scaled_logit(row[token], inv_t), m);
    a.tokens[r] = token;
    a.logprobs[r] = d - (float)(log((double)S) - 40.0 * 0.693147180559945309417);
    if (a.weight_sums) a.weight_sums[r] = S;
  }
}

void launch_sample(const SampleRows& r, int rows, int vocab, hipStream_t s) {
  if (!rows) return;
  // Large vocabularies with scratch at hand: the two sweeps of a row on several workgroups
  // (about 512 in all), then the selection; else everything in one workgroup per row.
  const int n_tiles = (vocab + 4095) >> 12;
  int parts = 0;
  if (r.part_max && r.seg_sums && n_tiles >= 8 && vocab <= 256 * kSampleSegments)
    parts = std::max(2, std::min({n_tiles, kSampleParts, 512 / rows}));
  if (parts >= 2) {
    sample_max_kernel<<<dim3(parts, rows), SAMP_T, 0, s>>>(r, vocab, parts);
    sample_segments_kernel<<<dim3(parts, rows), SAMP_T, 0, s>>>(r, vocab, parts);
    sample_kernel<<<rows, SAMP_T, 0, s>>>(r, vocab, parts);
  } else {
    sample_kernel<<<rows, SAMP_T, 0, s>>>(r, vocab, 0);
  }
}

// ---------------------------------------------------------------- teacher-forced gather
__global__ __launch_bounds__(SAMP_T) void logprob_gather_kernel(const float* __restrict__ logits,
                                                                const int* __restrict__ target, float inv_t,
                                                                float* __restrict__ out, int vocab) {
  __shared__ SampShared sh;
  const int tid = threadIdx.x, r = blockIdx.x;
  const int tgt = target[r];
  if (tgt < 0) {
    if (tid == 0) out[r] = 0.f;
    return;
  }
  const float* row = logits + (long long)r * vocab;
  float m = -INFINITY;
  for (int i = tid; i < vocab; i += SAMP_T) m = fmaxf(m, row[i] * inv_t);
  m = block_max(m, sh);
  float part = 0.f;
  for (int i = tid; i < vocab; i += SAMP_T) part += expf(row[i] * inv_t - m);
  part = wave_sum(part);
  if ((tid & 63) == 0) sh.fwave[tid >> 6] = part;
  __syncthreads();
  if (tid == 0) {
    float total = 0.f;
    for (int i = 0; i < SAMP_T / WAVE; ++i) total += sh.fwave[i];
    out[r] = row[tgt] * inv_t - m - logf(total);
  }
}
void launch_logprob_gather(const float* logits, const int* target, float inv_temp, float* out, int rows,
                           int vocab, hipStream_t s) {
  if (rows) logprob_gather_kernel<<<rows, SAMP_T, 0, s>>>(logits, target, inv_temp, out, vocab);
}
