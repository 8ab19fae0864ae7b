// Shared device/host helpers of the rollout library: storage types, wavefront
// reductions, KV-page addressing.  gfx950 only (64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#define WAVE 64

// ---- storage types -------------------------------------------------------------------
struct bf16_t {
  uint16_t bits;
};

__host__ __device__ inline float bf16_to_f32(bf16_t v) {
  union {
    uint32_t u;
    float f;
  } c;
  c.u = (uint32_t)v.bits << 16;
  return c.f;
}

// round to nearest, ties to even; NaN stays NaN
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union {
    uint32_t u;
    float f;
  } c;
  c.f = f;
  bf16_t out;
  if ((c.u & 0x7fffffffu) > 0x7f800000u) {
    out.bits = (uint16_t)((c.u >> 16) | 0x40u);
    return out;
  }
  uint32_t lsb = (c.u >> 16) & 1u;
  out.bits = (uint16_t)((c.u + 0x7fffu + lsb) >> 16);
  return out;
}

// v = hi + lo with both parts bf16: carries about 16 significant bits through bf16 arithmetic
__host__ __device__ inline void split_bf16(float v, uint16_t& hi, uint16_t& lo) {
  const bf16_t h = f32_to_bf16(v);
  hi = h.bits;
  lo = f32_to_bf16(v - bf16_to_f32(h)).bits;
}

// IEEE half: the 16-bit format of the KV cache of bf16 models.  Keys and values are of order
// one, so the three extra mantissa bits over bf16 are what keeps 28-layer logits within
// tolerance of the unrounded reference at the same bytes per cached token.  Values saturate
// at the largest finite half.
struct f16_t {
  uint16_t bits;
};
__host__ __device__ inline float f16_to_f32(f16_t v) { return (float)__builtin_bit_cast(_Float16, v.bits); }
__host__ __device__ inline f16_t f32_to_f16(float f) {
  f = f > 65504.f ? 65504.f : (f < -65504.f ? -65504.f : f);
  f16_t out;
  out.bits = __builtin_bit_cast(uint16_t, (_Float16)f);
  return out;
}
// v = hi + lo with both parts half precision (about 22 significant bits)
__host__ __device__ inline void split_f16(float v, uint16_t& hi, uint16_t& lo) {
  const _Float16 h = (_Float16)v;
  hi = __builtin_bit_cast(uint16_t, h);
  lo = __builtin_bit_cast(uint16_t, (_Float16)(v - (float)h));
}

__host__ __device__ inline float to_f32(float v) { return v; }
__host__ __device__ inline float to_f32(bf16_t v) { return bf16_to_f32(v); }
__host__ __device__ inline float to_f32(f16_t v) { return f16_to_f32(v); }
template <typename T>
__host__ __device__ inline T from_f32(float v);
template <>
__host__ __device__ inline float from_f32<float>(float v) {
  return v;
}
template <>
__host__ __device__ inline bf16_t from_f32<bf16_t>(float v) {
  return f32_to_bf16(v);
}
template <>
__host__ __device__ inline f16_t from_f32<f16_t>(float v) {
  return f32_to_f16(v);
}

// ---- wavefront reductions (every lane gets the result) ---------------------------------
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}
__device__ inline unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) {
    unsigned lo = __shfl_xor((unsigned)(v & 0xffffffffull), o, WAVE);
    unsigned hi = __shfl_xor((unsigned)(v >> 32), o, WAVE);
    v += ((unsigned long long)hi << 32) | lo;
  }
  return v;
}

// ---- KV pages ---------------------------------------------------------------------------
// The pool is [layer][page][kv_head][K|V][page_tokens * head_dim] elements.  Inside one
// (page, kv_head, K|V) block two element orders exist:
//   KV_LINEAR   [token][dim]
//   KV_MATRIX   the order the matrix-core attention kernels load with one contiguous
//               16-byte read per lane (see kv_k_offset / kv_v_offset).
enum KvLayout { KV_LINEAR = 0, KV_MATRIX = 1 };

struct KvGeom {
  int n_kv_heads, head_dim, page_tokens, layout;
  long long layer_stride;  // elements per layer = n_pages * page_stride
  long long page_stride;   // elements per page  = n_kv_heads * 2 * page_tokens * head_dim
};

// element offset of K[token][dim] inside a (page, head) K block
__host__ __device__ inline int kv_k_offset(const KvGeom& g, int tok, int dim) {
  if (g.layout == KV_LINEAR) return tok * g.head_dim + dim;
  // 16-token tiles; per tile head_dim/32 k-steps; per k-step 64 lanes x 8 elements, lane =
  // (dim % 32 / 8) * 16 + token % 16: the A/B fragment of a 16x16x32 matrix instruction.
  int tile = tok >> 4, r = tok & 15;
  int kstep = dim >> 5, grp = (dim & 31) >> 3, e = dim & 7;
  return ((tile * (g.head_dim >> 5) + kstep) * 64 + grp * 16 + r) * 8 + e;
}

// element offset of V[token][dim] inside a (page, head) V block
__host__ __device__ inline int kv_v_offset(const KvGeom& g, int tok, int dim) {
  if (g.layout == KV_LINEAR) return tok * g.head_dim + dim;
  // 32-token groups; per group head_dim/16 dim-tiles; per tile 64 lanes x 8 elements, lane =
  // grp * 16 + dim % 16, where the lane's 8 elements are tokens 4*grp..4*grp+3 of the first
  // 16-token tile and of the second: the order in which a transposed-score fragment holds
  // its probabilities, so that P needs no cross-lane movement before P.V.
  int group = tok >> 5, t = tok & 31;
  int half = t >> 4, tt = t & 15;
  int grp = tt >> 2, e = (tt & 3) + 4 * half;
  int tile = dim >> 4, r = dim & 15;
  return ((group * (g.head_dim >> 4) + tile) * 64 + grp * 16 + r) * 8 + e;
}

__host__ __device__ inline long long kv_block_base(const KvGeom& g, int layer, int page, int head, int is_v) {
  return (long long)layer * g.layer_stride + (long long)page * g.page_stride +
         (long long)(head * 2 + is_v) * g.page_tokens * g.head_dim;
}

// ---- host error plumbing ---------------------------------------------------------------
#define HIP_TRY(expr)                                                                       \
  do {                                                                                      \
    hipError_t _e = (expr);                                                                 \
    if (_e != hipSuccess) throw HipError(_e, #expr, __FILE__, __LINE__);                    \
  } while (0)

struct HipError {
  hipError_t code;
  const char* expr;
  const char* file;
  int line;
  HipError(hipError_t c, const char* e, const char* f, int l) : code(c), expr(e), file(f), line(l) {}
};

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }
