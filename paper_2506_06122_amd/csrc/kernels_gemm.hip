// bf16 projections on the matrix cores: out[m][n] = sum_k a[m][k] w[n][k], fp32 accumulate.
//
// The decoding phase is memory-bound (paper section 2.1): with few live rows every
// projection is a stream over the weight matrix.  Weights are therefore re-ordered once,
// at load time, into the fragment order of the 16x16x32 bf16 matrix instruction
//     packed[n_tile][k_tile][lane][8],  lane = (k % 32 / 8) * 16 + n % 16
// so that a wavefront reads each 16-column x 32-deep weight fragment as one contiguous
// 1 KiB load straight into registers, and a whole row of fragments [n_tile][*] is one
// contiguous stream.  The instruction computes D = W_frag . A_frag^T, i.e. a tile of
// out^T, so each lane ends up with four consecutive output columns of one row.
//
// Activations keep near-fp32 precision through the bf16 instruction: every activation value v
// travels as two bf16 numbers, hi = bf16(v) and lo = bf16(v - hi), in two planes of the same
// shape, and each weight fragment is multiplied with both (the weights themselves are bf16
// exactly, so nothing else is rounded).  That doubles the matrix instructions, which the
// memory-bound decode step does not notice.
//
// Three kernels:
//   gemm_stream_kernel  (rows <= 32, decoding): the NW wavefronts of a workgroup share NT
//       column tiles and interleave over the K range in chunks of KU fragments, so one
//       workgroup walks one contiguous weight stream with NW x KU x NT KiB in flight; the
//       partial accumulators meet in LDS.  Activations come straight from L2, stored in
//       fragment order by their producers (frag_offset, kernels_fast.h) so that an operand
//       fragment, like a weight fragment, is whole cache lines.  Narrow outputs (few column
//       tiles) use wide workgroups (16 wavefronts) rather than split-K planes, so every output
//       element is complete inside one workgroup and the epilogue can carry the neighbouring
//       element-wise work:
//         - RMSNorm is split in two.  The producer of the residual stream (EPI_RESID) adds
//           its result to x, stores x * gain as the next projection's operand and one
//           partial sum of squares per (workgroup, row); the consumer sums those partials
//           in a fixed order (all its wavefronts share the loads) and scales its output rows
//           by rsqrt(mean + eps) - a row scale commutes with the projection.  No workgroup
//           ever waits for another.
//         - SwiGLU on interleaved gate/up column tiles (EPI_SWIGLU_BF16).
//       Workgroups past the last column block, if the launcher adds any, walk a later
//       projection's weights into the memory-side cache (TouchRange, kernels_fast.h).
//   gemm_tile_ring_kernel (33 to 512 rows, every projection of a decode step, the logits
//       included): 64 x 128 output tile per workgroup (32 x 128 where that fills the chip
//       better), activations (row-major) staged through LDS in fragment order as whole cache
//       lines, weights read directly; split-K planes when the tiles alone do not fill the chip.
//   gemm_tile_kernel    (more than 512 rows: prefill, teacher-forced pass): 64 x 256 tile, the
//       same staging, software-pipelined over a ring of register slots.
#include <cstdio>

#include "kernels_fast.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

union Frag {
  uint4 u;
  bf16x8 v;
};

__device__ inline float silu_f(float a) { return a / (1.0f + __expf(-a)); }

__device__ inline uint2 pack4(const uint16_t (&h)[4]) {
  return make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
}

// D[n][m] tile(s) -> memory.  lane (r, g) holds rows n = 4g..4g+3 of a tile at column m = r.
template <int EPI>
__device__ inline void store_unit(const GemmArgs& p, int m, int nt, const f32x4& t0, const f32x4& t1, int g,
                                  int z, bool two) {
  if (EPI == EPI_F32) {
    float* out = (float*)p.out + (long long)z * p.split_stride + (long long)m * p.ldo;
    *(float4*)(out + nt * 16 + g * 4) = make_float4(t0[0], t0[1], t0[2], t0[3]);
    if (two) *(float4*)(out + (nt + 1) * 16 + g * 4) = make_float4(t1[0], t1[1], t1[2], t1[3]);
  } else {  // EPI_SWIGLU_BF16: tile nt = gate, nt + 1 = up; act[m][f] = silu(gate) * up
    const int f = (nt >> 1) * 16 + g * 4;
    uint16_t* out = (uint16_t*)p.out + (p.frag ? frag_offset(m, f, p.ldo >> 5) : (long long)m * p.ldo + f);
    uint16_t h[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) split_bf16(silu_f(t0[e]) * t1[e], h[e], lo[e]);
    *(uint2*)out = pack4(h);
    *(uint2*)(out + p.out_lo_offset) = pack4(lo);
  }
}

template <int MT, int NT, int KU, int NW, int EPI>
__global__ __launch_bounds__(NW * 64) void gemm_stream_kernel(GemmArgs p) {
  static_assert(EPI != EPI_RESID || NT <= 2, "one unit must cover a workgroup's columns");
  __shared__ float4 red[NW * MT * NT * 64];
  __shared__ float rs_part[NW * MT * 64];
  if (p.touch.wgs > 0 && (int)blockIdx.x >= p.touch_x0) {  // uniform over the workgroup
    if (blockIdx.y == 0) touch_range(p.touch, blockIdx.x - p.touch_x0);  // one walk, whatever the row blocks
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int n_tiles = p.N >> 4, k_tiles = p.K >> 5;
  const int nt0 = blockIdx.x * NT;
  const int m0 = blockIdx.y * (MT * 16);
  const int kt_begin = blockIdx.z * p.k_tiles_per_split;
  const int kt_end = min(k_tiles, kt_begin + p.k_tiles_per_split);
  const uint4* wp = (const uint4*)p.w;
  const uint16_t* a_base = (const uint16_t*)p.a;

  f32x4 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // activation pointers of this lane (row m0 + 16 i + r, k = 8 g .. 8 g + 7 of k-tile 0), or null
  // past the last row; a k-tile further on is a_kstep elements away
  const uint16_t* a_row[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int m = m0 + i * 16 + r;
    a_row[i] = m >= p.M ? nullptr
               : p.frag ? a_base + (((long long)(m >> 4) * k_tiles) << 9) + lane * 8
                        : a_base + (long long)m * p.lda + g * 8;
  }
  const int a_kstep = p.frag ? 512 : 32;
  const long long lo_off = (const uint16_t*)p.a_lo - a_base;

  // Epilogue unit (one row tile, up to two column tiles) of this wavefront, if it has one.  Its
  // operands - the input rows' partial sums of squares, the residual values and the gain - are
  // requested now, so that they arrive while the weights stream.
  constexpr int NU = NT >= 2 ? NT / 2 : 1;  // units per row tile
  constexpr int TW = NT >= 2 ? 2 : 1;       // column tiles per unit
  static_assert(MT * NU <= NW, "at most one epilogue unit per wavefront");
  const bool has_unit = wave < MT * NU;
  const int ui = wave / NU, uj = (wave % NU) * TW;
  const int um = m0 + ui * 16 + r;
  const bool valid = has_unit && um < p.M && nt0 + uj + TW - 1 < n_tiles;
  float4 xv[TW], gn[TW];
  // The input rows' sums of squares come as one partial per workgroup of the producing launch
  // (hidden/16 of them): every wavefront takes the partials w, w + NW, ... - a lane those of its
  // group g, for row r of each row tile - so that no wavefront has more than a few loads to wait
  // for; the shares meet in LDS with the accumulators.
  float rs_share[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    rs_share[i] = 0.f;
    const int m = m0 + i * 16 + r;
    if (p.rinv_ssq && m < p.M)
      for (int pp = wave * 4 + g; pp < p.rinv_partials; pp += NW * 4)
        rs_share[i] += p.rinv_ssq[(long long)pp * p.ssq_stride + m];
  }
  if (EPI == EPI_RESID && valid) {
#pragma unroll
    for (int q = 0; q < TW; ++q) {
      const int n = (nt0 + uj + q) * 16 + g * 4;
      xv[q] = *(const float4*)(p.x + (long long)um * p.N + n);
      gn[q] = *(const float4*)(p.gain + n);
    }
  }

  for (int kt = kt_begin + wave * KU; kt < kt_end; kt += NW * KU) {
    Frag b[KU][NT], a[KU][MT], al[KU][MT];
#pragma unroll
    for (int kk = 0; kk < KU; ++kk) {
      const bool live = kt + kk < kt_end;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        b[kk][j].u = make_uint4(0, 0, 0, 0);
        if (live && nt0 + j < n_tiles) b[kk][j].u = wp[((long long)(nt0 + j) * k_tiles + kt + kk) * 64 + lane];
      }
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        a[kk][i].u = make_uint4(0, 0, 0, 0);
        al[kk][i].u = make_uint4(0, 0, 0, 0);
        if (live && a_row[i]) {
          a[kk][i].u = *(const uint4*)(a_row[i] + (kt + kk) * a_kstep);
          al[kk][i].u = *(const uint4*)(a_row[i] + lo_off + (kt + kk) * a_kstep);
        }
      }
    }
#pragma unroll
    for (int kk = 0; kk < KU; ++kk)
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[kk][j].v, al[kk][i].v, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[kk][j].v, a[kk][i].v, acc[i][j], 0, 0, 0);
        }
  }

  // the wavefronts' partial tiles meet in LDS; units of (one row tile, two column tiles)
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
      red[(wave * MT * NT + i * NT + j) * 64 + lane] = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
  if (p.rinv_ssq) {
#pragma unroll
    for (int i = 0; i < MT; ++i) rs_part[(wave * MT + i) * 64 + lane] = rs_share[i];
  }
  __syncthreads();
  if (!has_unit) return;
  f32x4 t[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
  for (int q = 0; q < TW; ++q)
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float4 v = red[(w * MT * NT + ui * NT + uj + q) * 64 + lane];
      t[q][0] += v.x;
      t[q][1] += v.y;
      t[q][2] += v.z;
      t[q][3] += v.w;
    }
  if (p.rinv_ssq) {
    // second half of the RMSNorm of this projection's input: scale row m by
    // rsqrt(mean(x^2) + eps); the 4 lanes of a row share the partial sums
    float rs = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) rs += rs_part[(w * MT + ui) * 64 + lane];
    rs += __shfl_xor(rs, 16, WAVE);
    rs += __shfl_xor(rs, 32, WAVE);
    const float rinv = 1.0f / sqrtf(rs / (float)p.K + p.eps);
#pragma unroll
    for (int q = 0; q < TW; ++q) {
      t[q][0] *= rinv;
      t[q][1] *= rinv;
      t[q][2] *= rinv;
      t[q][3] *= rinv;
    }
  }
  if (EPI == EPI_RESID) {
    float ss = 0.f;
    if (valid) {
#pragma unroll
      for (int q = 0; q < TW; ++q) {
        const int n = (nt0 + uj + q) * 16 + g * 4;
        float4 x4 = xv[q];
        x4.x += t[q][0];
        x4.y += t[q][1];
        x4.z += t[q][2];
        x4.w += t[q][3];
        *(float4*)(p.x + (long long)um * p.N + n) = x4;
        ss += x4.x * x4.x + x4.y * x4.y + x4.z * x4.z + x4.w * x4.w;
        uint16_t hi[4], lo[4];
        split_bf16(x4.x * gn[q].x, hi[0], lo[0]);
        split_bf16(x4.y * gn[q].y, hi[1], lo[1]);
        split_bf16(x4.z * gn[q].z, hi[2], lo[2]);
        split_bf16(x4.w * gn[q].w, hi[3], lo[3]);
        uint16_t* hp = p.h + (p.frag ? frag_offset(um, n, n_tiles >> 1) : (long long)um * p.N + n);
        *(uint2*)hp = pack4(hi);
        *(uint2*)(hp + p.h_lo_offset) = pack4(lo);
      }
    }
    ss += __shfl_xor(ss, 16, WAVE);
    ss += __shfl_xor(ss, 32, WAVE);
    if (g == 0 && um < p.M) p.ssq_out[(long long)blockIdx.x * p.ssq_stride + um] = ss;
  } else if (valid) {
    store_unit<EPI>(p, um, nt0 + uj, t[0], t[1], g, blockIdx.z, TW == 2);
  }
}

// Workgroup -> (column block, row block, K split) of the tile kernels.  The launch is
// one-dimensional and workgroups go to the 8 XCDs (each with its own L2) round-robin by index,
// so index % 8 is the XCD and index / 8 the order inside it.  The unit of work handed to an XCD
// is a group of up to 16 consecutive row blocks of one (column block, split) pair, which run back
// to back: the pair's weight slab is fetched from HBM once per group, into that XCD's L2,
// instead of once per row block and XCD.  Units go round the XCDs with the pair (and inside it
// the split) varying fastest, so the XCDs stay balanced and, with 8 or 16 splits, each keeps to
// a slice of the K range, i.e. of the activations.
__device__ inline bool tile_block(const GemmArgs& p, int& bx, int& by, int& bz) {
  const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
  const int gm = min(p.grid_ny, 16);
  const int pairs = p.grid_nx * p.grid_nz;
  const int unit = (idx / gm) * 8 + xcd;
  const int pair = unit % pairs;
  by = (unit / pairs) * gm + idx % gm;
  bx = pair / p.grid_nz;
  bz = pair % p.grid_nz;
  return by < p.grid_ny;  // units past the last one land past the last row block
}

// ------------------------------------------------------------------------------------------
// Tiled kernel: a workgroup of 4 wavefronts computes MT*16 rows x 4*NT*16 columns; each
// wavefront owns NT column tiles and reads its weight fragments straight from memory, the
// activation fragments (hi and lo planes) of KC k-tiles (one stage) are staged in LDS for all
// four.  Software-pipelined over a ring of R register slots: while stage s is multiplied (its
// weights read in place from slot s % R, its activations from one LDS buffer), the loads of
// stage s+R-1 are issued into the slot stage s-1 has just left, and stage s+1's activations
// move from their slot to the other LDS buffer - all in one basic block, so the matrix
// instructions overlap the memory instructions.  One barrier per stage: a wavefront reaches
// the barrier that ends stage s only after its reads of stage s's buffer, which the write of
// stage s+2 is the next to touch.
// Loads are never predicated: rows, column tiles and k-tiles past the end read the last valid
// one instead (results of such rows and columns are not stored; the weights of a k-tile past
// the end are zeroed).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int MT, int NT, int KC, int R, int EPI>
__global__ __launch_bounds__(256) void gemm_tile_kernel(GemmArgs p) {
  constexpr int FR = 2 * MT * KC;      // activation fragments per stage: [kk][plane][mt]
  static_assert(FR % 4 == 0 && (2 * MT) % 4 == 0, "the fragments divide evenly over the wavefronts");
  constexpr int PER = FR / 4;          // fragments each wavefront stages: f = 4 s + wave
  __shared__ u32x4 a_lds[2][FR * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int n_tiles = p.N >> 4, k_tiles = p.K >> 5;
  int bx, by, bz;
  if (!tile_block(p, bx, by, bz)) return;  // padding of the XCD-aware launch (uniform)
  const int nt0 = (bx * 4 + wave) * NT;
  int m0 = by * (MT * 16);
  const int kt_begin = bz * p.k_tiles_per_split;
  const int kt_end = min(k_tiles, kt_begin + p.k_tiles_per_split);

  // grouped (per-expert) launches: this row block belongs to one group with its own weights
  const u32x4* wp = (const u32x4*)p.w;
  const int* row_map = nullptr;
  int m_limit = p.M;
  if (p.group_of_block) {
    int grp = p.group_of_block[by];
    wp += (long long)grp * p.group_stride16;
    m0 = p.block_row_begin[by];
    m_limit = p.block_row_end[by];
    row_map = p.row_map;
    if (m0 >= m_limit) return;  // unused block of the plan (uniform over the workgroup)
  }
  const uint16_t* a_base = (const uint16_t*)p.a;
  const long long lo_off = (const uint16_t*)p.a_lo - a_base;

  // Staging of the activations: one load instruction brings 8 rows x 128 bytes - both k-tiles
  // of the stage, one plane - as full cache lines (a 16-row x 64-byte fragment load costs the
  // L2 path twice as much per byte).  Unit u = 4 s + wave -> (plane, group of 8 rows); a lane
  // holds chunk c = lane % 8 of row lane / 8, i.e. k-tile c / 4, fragment column group c % 4.
  // In LDS a fragment's sixteen 16-byte slots of one column group are permuted by
  // row ^ (2 * group + k-tile), which spreads a row's 8 chunks over all banks.
  static_assert(KC == 2 && FR == 4 * MT, "a stage is two k-tiles");
  const int st_kk = (lane & 7) >> 2, st_g = lane & 3;
  const uint16_t* st_src[PER];
  int st_dst[PER];
#pragma unroll
  for (int s = 0; s < PER; ++s) {
    const int u = 4 * s + wave;
    const int plane = u / (2 * MT), rg = u % (2 * MT);
    const int mt = rg >> 1, rr = (rg & 1) * 8 + (lane >> 3);
    const int m = min(m0 + mt * 16 + rr, m_limit - 1);
    const long long row = row_map ? row_map[m] : m;
    st_src[s] = a_base + row * p.lda + st_g * 8 + (plane ? lo_off : 0);
    st_dst[s] = ((st_kk * 2 + plane) * MT + mt) * 64 + st_g * 16 + (rr ^ ((2 * st_g + st_kk) & 7));
  }
  const int rd_off[2] = {g * 16 + (r ^ ((2 * g) & 7)), g * 16 + (r ^ ((2 * g + 1) & 7))};
  const u32x4* w_src[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) w_src[j] = wp + (long long)min(nt0 + j, n_tiles - 1) * k_tiles * 64 + lane;

  f32x4 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  u32x4 rst[R][PER];
  u32x4 rb[R][KC][NT];
#define GEMM_LOAD_STAGE(KT, SLOT)                                                                 \
  {                                                                                               \
    _Pragma("unroll") for (int s = 0; s < PER; ++s) {                                             \
      const int k = min((KT) + st_kk, kt_end - 1);                                                \
      rst[SLOT][s] = *(const u32x4*)(st_src[s] + (long long)k * 32);                              \
    }                                                                                             \
    _Pragma("unroll") for (int kk = 0; kk < KC; ++kk)                                             \
        _Pragma("unroll") for (int j = 0; j < NT; ++j) {                                          \
      rb[SLOT][kk][j] = w_src[j][(long long)min((KT) + kk, kt_end - 1) * 64];                     \
      if (kk > 0 && (KT) + kk >= kt_end) rb[SLOT][kk][j] = u32x4{0u, 0u, 0u, 0u};                 \
    }                                                                                             \
  }
#pragma unroll
  for (int d = 0; d < R - 1; ++d) GEMM_LOAD_STAGE(kt_begin + d * KC, d)
#pragma unroll
  for (int s = 0; s < PER; ++s) a_lds[0][st_dst[s]] = rst[0][s];
  __syncthreads();
  int buf = 0;
  for (int kt = kt_begin; kt < kt_end; kt += R * KC) {
#pragma unroll
    for (int d = 0; d < R; ++d) {
      const int k0 = kt + d * KC;
      if (k0 < kt_end) {  // uniform over the workgroup
        u32x4 a[KC][2][MT];
#pragma unroll
        for (int kk = 0; kk < KC; ++kk)
#pragma unroll
          for (int plane = 1; plane >= 0; --plane)
#pragma unroll
            for (int i = 0; i < MT; ++i) a[kk][plane][i] = a_lds[buf][((kk * 2 + plane) * MT + i) * 64 + rd_off[kk]];
        GEMM_LOAD_STAGE(k0 + (R - 1) * KC, (d + R - 1) % R)
#pragma unroll
        for (int kk = 0; kk < KC; ++kk)
#pragma unroll
          for (int plane = 1; plane >= 0; --plane)  // lo parts first, then hi
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
              for (int j = 0; j < NT; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, rb[d][kk][j]),
                                                                    __builtin_bit_cast(bf16x8, a[kk][plane][i]),
                                                                    acc[i][j], 0, 0, 0);
        if (k0 + KC < kt_end) {
#pragma unroll
          for (int s = 0; s < PER; ++s) a_lds[buf ^ 1][st_dst[s]] = rst[(d + 1) % R][s];
        }
        __syncthreads();
        buf ^= 1;
      }
    }
  }
#undef GEMM_LOAD_STAGE
  if constexpr (EPI == EPI_LSE) {
    // log-sum-exp parts of this workgroup's columns: per wavefront over its NT tiles (the 4
    // lanes of a row meet by shuffles), then over the 4 wavefronts through LDS
    __shared__ float part_m[4][MT * 16], part_s[4][MT * 16];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int m = m0 + i * 16 + r;
      const int tgt = m < m_limit ? p.lse_target[m] : -1;
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < NT; ++j)
        if (nt0 + j < n_tiles) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[i][j][e] *= p.lse_scale;
            mx = fmaxf(mx, acc[i][j][e]);
            if ((nt0 + j) * 16 + g * 4 + e == tgt) p.lse_tgt[m] = acc[i][j][e];
          }
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, WAVE));
      mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
      float sm = 0.f;
#pragma unroll
      for (int j = 0; j < NT; ++j)
        if (nt0 + j < n_tiles) {
#pragma unroll
          for (int e = 0; e < 4; ++e) sm += expf(acc[i][j][e] - mx);
        }
      sm += __shfl_xor(sm, 16, WAVE);
      sm += __shfl_xor(sm, 32, WAVE);
      if (g == 0) {
        part_m[wave][i * 16 + r] = mx;
        part_s[wave][i * 16 + r] = sm;
      }
    }
    __syncthreads();
    if (threadIdx.x < MT * 16 && m0 + (int)threadIdx.x < m_limit) {
      float mx = -INFINITY;
#pragma unroll
      for (int w = 0; w < 4; ++w) mx = fmaxf(mx, part_m[w][threadIdx.x]);
      float sm = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w)
        if (part_m[w][threadIdx.x] > -INFINITY) sm += part_s[w][threadIdx.x] * expf(part_m[w][threadIdx.x] - mx);
      p.lse_max[(long long)bx * p.lse_stride + m0 + threadIdx.x] = mx;
      p.lse_sum[(long long)bx * p.lse_stride + m0 + threadIdx.x] = sm;
    }
    return;
  }
  if (nt0 >= n_tiles) return;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int m = m0 + i * 16 + r;
    if (m >= m_limit) continue;
#pragma unroll
    for (int j = 0; j < NT; j += 2)
      if (nt0 + j < n_tiles)  // an odd last column tile (fp32 results only) is stored alone
        store_unit<EPI == EPI_LSE ? EPI_F32 : EPI>(p, m, nt0 + j, acc[i][j], acc[i][j + 1], g, bz,
                                                  nt0 + j + 1 < n_tiles);
  }
}

// ------------------------------------------------------------------------------------------
// The same tile with predicated loads and a ring of D prefetched stages whose activations go
// to LDS and whose weights go to the multiply operands at the top of each stage: the leaner
// variant (fewer registers, rows past the end are not loaded) that the decode-sized
// projections run best with.
template <int MT, int NT, int KC, int D, int EPI>
__global__ __launch_bounds__(256) void gemm_tile_ring_kernel(GemmArgs p) {
  constexpr int FR = 2 * MT * KC;      // activation fragments per stage: [kk][plane][mt]
  constexpr int PER = (FR + 3) / 4;    // fragments each wavefront stages
  __shared__ uint4 a_lds[2][FR * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int n_tiles = p.N >> 4, k_tiles = p.K >> 5;
  int bx, by, bz;
  if (!tile_block(p, bx, by, bz)) return;  // padding of the XCD-aware launch (uniform)
  const int nt0 = (bx * 4 + wave) * NT;
  int m0 = by * (MT * 16);
  const int kt_begin = bz * p.k_tiles_per_split;
  const int kt_end = min(k_tiles, kt_begin + p.k_tiles_per_split);

  // grouped (per-expert) launches: this row block belongs to one group with its own weights
  const uint4* wp = (const uint4*)p.w;
  const int* row_map = nullptr;
  int m_limit = p.M;
  if (p.group_of_block) {
    int grp = p.group_of_block[by];
    wp += (long long)grp * p.group_stride16;
    m0 = p.block_row_begin[by];
    m_limit = p.block_row_end[by];
    row_map = p.row_map;
    if (m0 >= m_limit) return;  // unused block of the plan (uniform over the workgroup)
  }
  const uint16_t* a_base = (const uint16_t*)p.a;
  const long long lo_off = (const uint16_t*)p.a_lo - a_base;

  // Staging of the activations: one load instruction brings 8 rows x 128 bytes - both k-tiles
  // of the stage, one plane - as full cache lines (a 16-row x 64-byte fragment load costs the
  // L2 path twice as much per byte).  Unit u = wave + 4 s -> (plane, group of 8 rows); a lane
  // holds chunk c = lane % 8 of row lane / 8, i.e. k-tile c / 4, fragment column group c % 4.
  // In LDS a fragment's sixteen 16-byte slots of one column group are permuted by
  // row ^ (2 * group + k-tile), which spreads a row's 8 chunks over all banks.
  static_assert(KC == 2 && FR == 4 * MT, "a stage is two k-tiles");
  const int st_kk = (lane & 7) >> 2, st_g = lane & 3;
  const uint16_t* st_src[PER];
  int st_dst[PER];
#pragma unroll
  for (int s = 0; s < PER; ++s) {
    const int u = wave + 4 * s;
    const int plane = u / (2 * MT), rg = u % (2 * MT);
    const int mt = rg >> 1, rr = (rg & 1) * 8 + (lane >> 3);
    const int m = m0 + mt * 16 + rr;
    st_src[s] = nullptr;
    if (m < m_limit) {
      const long long row = row_map ? row_map[m] : m;
      st_src[s] = a_base + row * p.lda + (lane & 7) * 8 + (plane ? lo_off : 0);
    }
    st_dst[s] = ((st_kk * 2 + plane) * MT + mt) * 64 + st_g * 16 + (rr ^ ((2 * st_g + st_kk) & 7));
  }
  const int rd_off[2] = {g * 16 + (r ^ ((2 * g) & 7)), g * 16 + (r ^ ((2 * g + 1) & 7))};

  f32x4 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  struct Stage {
    uint4 st[PER];
    Frag b[KC][NT];
  };
  Stage ring[D];
  Frag cur[KC][NT];
  auto load_stage = [&](int kt, Stage& sg) {
#pragma unroll
    for (int s = 0; s < PER; ++s) {
      sg.st[s] = make_uint4(0, 0, 0, 0);
      if (st_src[s] && kt + st_kk < kt_end) sg.st[s] = *(const uint4*)(st_src[s] + (long long)kt * 32);
    }
#pragma unroll
    for (int kk = 0; kk < KC; ++kk)
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        sg.b[kk][j].u = make_uint4(0, 0, 0, 0);
        if (kt + kk < kt_end && nt0 + j < n_tiles)
          sg.b[kk][j].u = wp[((long long)(nt0 + j) * k_tiles + kt + kk) * 64 + lane];
      }
  };

#pragma unroll
  for (int d = 0; d < D; ++d) load_stage(kt_begin + d * KC, ring[d]);
  int buf = 0;
  for (int kt = kt_begin; kt < kt_end; kt += D * KC) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const int k0 = kt + d * KC;
      if (k0 >= kt_end) break;  // uniform over the workgroup
#pragma unroll
      for (int s = 0; s < PER; ++s) a_lds[buf][st_dst[s]] = ring[d].st[s];
#pragma unroll
      for (int kk = 0; kk < KC; ++kk)
#pragma unroll
        for (int j = 0; j < NT; ++j) cur[kk][j] = ring[d].b[kk][j];
      load_stage(k0 + D * KC, ring[d]);
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < KC; ++kk)
#pragma unroll
        for (int plane = 1; plane >= 0; --plane) {  // lo parts first, then hi
          Frag a[MT];
#pragma unroll
          for (int i = 0; i < MT; ++i) a[i].u = a_lds[buf][((kk * 2 + plane) * MT + i) * 64 + rd_off[kk]];
#pragma unroll
          for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur[kk][j].v, a[i].v, acc[i][j], 0, 0, 0);
        }
      buf ^= 1;
    }
  }
  if constexpr (EPI == EPI_LSE) {
    // log-sum-exp parts of this workgroup's columns: per wavefront over its NT tiles (the 4
    // lanes of a row meet by shuffles), then over the 4 wavefronts through LDS
    __shared__ float part_m[4][MT * 16], part_s[4][MT * 16];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int m = m0 + i * 16 + r;
      const int tgt = m < m_limit ? p.lse_target[m] : -1;
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < NT; ++j)
        if (nt0 + j < n_tiles) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[i][j][e] *= p.lse_scale;
            mx = fmaxf(mx, acc[i][j][e]);
            if ((nt0 + j) * 16 + g * 4 + e == tgt) p.lse_tgt[m] = acc[i][j][e];
          }
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, WAVE));
      mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
      float sm = 0.f;
#pragma unroll
      for (int j = 0; j < NT; ++j)
        if (nt0 + j < n_tiles) {
#pragma unroll
          for (int e = 0; e < 4; ++e) sm += expf(acc[i][j][e] - mx);
        }
      sm += __shfl_xor(sm, 16, WAVE);
      sm += __shfl_xor(sm, 32, WAVE);
      if (g == 0) {
        part_m[wave][i * 16 + r] = mx;
        part_s[wave][i * 16 + r] = sm;
      }
    }
    __syncthreads();
    if (threadIdx.x < MT * 16 && m0 + (int)threadIdx.x < m_limit) {
      float mx = -INFINITY;
#pragma unroll
      for (int w = 0; w < 4; ++w) mx = fmaxf(mx, part_m[w][threadIdx.x]);
      float sm = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w)
        if (part_m[w][threadIdx.x] > -INFINITY) sm += part_s[w][threadIdx.x] * expf(part_m[w][threadIdx.x] - mx);
      p.lse_max[(long long)bx * p.lse_stride + m0 + threadIdx.x] = mx;
      p.lse_sum[(long long)bx * p.lse_stride + m0 + threadIdx.x] = sm;
    }
    return;
  }
  if (nt0 >= n_tiles) return;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int m = m0 + i * 16 + r;
    if (m >= m_limit) continue;
#pragma unroll
    for (int j = 0; j < NT; j += 2)
      if (nt0 + j < n_tiles)  // an odd last column tile (fp32 results only) is stored alone
        store_unit<EPI == EPI_LSE ? EPI_F32 : EPI>(p, m, nt0 + j, acc[i][j], acc[i][j + 1], g, bz,
                                                  nt0 + j + 1 < n_tiles);
  }
}

// ------------------------------------------------------------------------------------------
template <int MT, int NT, int KU, int NW>
static void launch_stream(const GemmArgs& a, int epi, dim3 grid, hipStream_t s) {
  if (epi == EPI_F32)
    gemm_stream_kernel<MT, NT, KU, NW, EPI_F32><<<grid, NW * 64, 0, s>>>(a);
  else if (epi == EPI_SWIGLU_BF16)
    gemm_stream_kernel<MT, NT, KU, NW, EPI_SWIGLU_BF16><<<grid, NW * 64, 0, s>>>(a);
  else
    gemm_stream_kernel<MT, NT, KU, NW, EPI_RESID><<<grid, NW * 64, 0, s>>>(a);
}

static const char* stream_name(int mt, int nt, int nw, int epi) {
  static char names[3][2][2][3][40];
  static bool init = false;
  if (!init) {
    const int mts[3] = {1, 2, 4}, nws[2] = {4, 16};
    for (int a = 0; a < 3; ++a)
      for (int b = 0; b < 2; ++b)
        for (int c = 0; c < 2; ++c)
          for (int e = 0; e < 3; ++e)
            snprintf(names[a][b][c][e], 40, "gemm_stream_kernel<%d,%d,%d,%d,%d>", mts[a], b + 1, mts[a] == 4 ? 2 : 4,
                     nws[c], e);
    init = true;
  }
  return names[mt == 1 ? 0 : mt == 2 ? 1 : 2][nt - 1][nw == 4 ? 0 : 1][epi];
}

// tiled kernel: the largest tile that still gives every CU a workgroup, then split-K planes
GemmPlan gemm_plan_tiled(int M, int N, int K, int epi, int max_splits) {
  GemmPlan pl{};
  const int n_tiles = N >> 4, k_tiles = K >> 5;
  pl.kind = 1;
  pl.nw = 4;
  static const int cfg[2][2] = {{4, 4}, {4, 2}};
  static const char* const names[2][3] = {
      {"gemm_tile_kernel<4,4,2,2,0>", "gemm_tile_kernel<4,4,2,2,1>", "gemm_tile_kernel<4,4,2,2,3>"},
      {"gemm_tile_ring_kernel<4,2,2,1,0>", "gemm_tile_ring_kernel<4,2,2,1,1>", "gemm_tile_ring_kernel<4,2,2,1,3>"}};
  // 64 x 256 tiles for prefill-sized row counts when they still give every CU two workgroups;
  // 64 x 128 otherwise and for every decode-sized launch (at most 512 rows: measured 8-25 %
  // faster there at all widths, the logits projection included)
  int pick = 1;
  long long blocks = 0;
  for (int c = 0; c < 2; ++c) {
    blocks = (long long)ceil_div(M, 16 * cfg[c][0]) * ceil_div(n_tiles, 4 * cfg[c][1]);
    if ((blocks >= 576 && M > 512) || c == 1) {
      pick = c;
      break;
    }
  }
  pl.mt = cfg[pick][0];
  pl.nt = cfg[pick][1];
  pl.kc = 2;
  pl.splits = 1;
  if (pick == 1 && epi == EPI_F32 && M <= 128 && blocks < 512) {
    pl.mt = 2;
    blocks = (long long)ceil_div(M, 32) * ceil_div(n_tiles, 8);
  }
  if (epi == EPI_F32 && blocks < 256) {
    int z = (int)((768 + blocks - 1) / blocks);
    z = std::min(z, std::max(1, k_tiles / 8));
    pl.splits = std::max(1, std::min(z, max_splits));
  }
  pl.name = names[pick][epi == EPI_F32 ? 0 : epi == EPI_SWIGLU_BF16 ? 1 : 2];
  // SwiGLU projection (no split-K possible) of at most 128 rows, when 64-row blocks give fewer
  // than two workgroups per CU: 32-row blocks give the chip twice the workgroups - one or two
  // 64-row blocks leave CUs idle or with one long workgroup
  if (pick == 1 && epi == EPI_SWIGLU_BF16 && M <= 128 && blocks < 512) {
    pl.mt = 2;
    pl.name = "gemm_tile_ring_kernel<2,2,2,1,1>";
  }
  if (pick == 1 && epi == EPI_F32 && pl.mt == 2) pl.name = "gemm_tile_ring_kernel<2,2,2,1,0>";
  return pl;
}

GemmPlan gemm_plan(int M, int N, int K, int epi, int max_splits) {
  if (M > 32 || epi == EPI_LSE) return gemm_plan_tiled(M, N, K, epi, max_splits);
  GemmPlan pl{};
  const int n_tiles = N >> 4, k_tiles = K >> 5;
  pl.kind = 0;
  pl.mt = M <= 16 ? 1 : M <= 32 ? 2 : 4;
  const int m_blocks = ceil_div(M, 16 * pl.mt);
  // wide outputs: two column tiles and 4 wavefronts per workgroup; narrow outputs: one column
  // tile and 16 wavefronts, so that the K range, not the column count, fills the CUs
  const bool wide = (long long)(n_tiles / 2) * m_blocks >= 512;
  pl.nt = (wide || epi == EPI_SWIGLU_BF16) ? 2 : 1;
  pl.nw = wide ? 4 : 16;
  // narrow but not tiny (the fused QKV projection of 7B-class models): two column tiles per
  // wide workgroup halve the activation re-reads and still leave more than a hundred
  // workgroups.  (Measured: the residual epilogue's projections run better with one.)
  if (!wide && epi == EPI_F32 && n_tiles >= 192 && n_tiles % 2 == 0) pl.nt = 2;
  if (epi == EPI_SWIGLU_BF16 && !wide) pl.nw = 4;
  // 17-32 rows, narrow output with at most 160 workgroup columns (QKV, and at the 1.5B shape O
  // and down): two row blocks of the one-row-tile kernel instead of one two-row-tile block -
  // twice the workgroups on a chip they do not fill, the second block's weights from L2
  // (measured at 32 rows: down 25 -> 17 us at the 1.5B shape, QKV 22 -> 17 us at 7B; with 224
  // columns, the 7B O and down projections, the two-row-tile block stays ahead)
  if (pl.mt == 2 && !wide && epi != EPI_SWIGLU_BF16 && n_tiles / pl.nt <= 160) pl.mt = 1;
  pl.splits = 1;
  if (epi == EPI_F32 && !wide && max_splits > 1) {
    const long long blocks = (long long)n_tiles * m_blocks;
    int z = (int)((256 + blocks - 1) / blocks);
    z = std::min(z, std::max(1, k_tiles / 64));
    pl.splits = std::max(1, std::min({z, max_splits, 4}));
  }
  pl.name = stream_name(pl.mt, pl.nt, pl.nw, epi);
  return pl;
}

template <int MT, int NT, int KC, int R>
static void launch_tile(const GemmArgs& a, int epi, dim3 grid, hipStream_t s) {
  if (epi == EPI_F32) gemm_tile_kernel<MT, NT, KC, R, EPI_F32><<<grid, 256, 0, s>>>(a);
  else if (epi == EPI_SWIGLU_BF16) gemm_tile_kernel<MT, NT, KC, R, EPI_SWIGLU_BF16><<<grid, 256, 0, s>>>(a);
  else gemm_tile_kernel<MT, NT, KC, R, EPI_LSE><<<grid, 256, 0, s>>>(a);
}

template <int MT, int NT, int KC, int D>
static void launch_tile_ring(const GemmArgs& a, int epi, dim3 grid, hipStream_t s) {
  if (epi == EPI_F32) gemm_tile_ring_kernel<MT, NT, KC, D, EPI_F32><<<grid, 256, 0, s>>>(a);
  else if (epi == EPI_SWIGLU_BF16) gemm_tile_ring_kernel<MT, NT, KC, D, EPI_SWIGLU_BF16><<<grid, 256, 0, s>>>(a);
  else gemm_tile_ring_kernel<MT, NT, KC, D, EPI_LSE><<<grid, 256, 0, s>>>(a);
}

template <int MT, int KU>
static void launch_stream_mt(const GemmArgs& a, int epi, const GemmPlan& pl, dim3 grid, hipStream_t s) {
  if (pl.nt == 1 && pl.nw == 4) launch_stream<MT, 1, KU, 4>(a, epi, grid, s);
  else if (pl.nt == 1) launch_stream<MT, 1, KU, 16>(a, epi, grid, s);
  else if (pl.nw == 4) launch_stream<MT, 2, KU, 4>(a, epi, grid, s);
  else launch_stream<MT, 2, KU, 16>(a, epi, grid, s);
}

int launch_gemm_bf16(GemmArgs a, int epi, const GemmPlan& pl, hipStream_t s) {
  if (a.M < 1 || a.N < 16) return 0;
  const int n_tiles = a.N >> 4, k_tiles = a.K >> 5;
  if (pl.kind == 1) {
    int per = ceil_div(ceil_div(k_tiles, epi == EPI_F32 ? pl.splits : 1), 2) * 2;
    const int splits = ceil_div(k_tiles, per);
    a.k_tiles_per_split = per;
    const int m_blocks = a.group_of_block ? a.n_row_blocks : ceil_div(a.M, 16 * pl.mt);
    a.grid_nx = ceil_div(n_tiles, 4 * pl.nt);
    a.grid_ny = m_blocks;
    a.grid_nz = splits;
    const int gm = std::min(a.grid_ny, 16);
    const long long units = (long long)a.grid_nx * a.grid_nz * ceil_div(a.grid_ny, gm);
    dim3 grid((unsigned)(ceil_div(units, 8) * 8 * gm));
    if (pl.nt == 4) launch_tile<4, 4, 2, 2>(a, epi, grid, s);
    else if (pl.mt == 2 && epi == EPI_SWIGLU_BF16) gemm_tile_ring_kernel<2, 2, 2, 1, EPI_SWIGLU_BF16><<<grid, 256, 0, s>>>(a);
    else if (pl.mt == 2 && epi == EPI_F32) gemm_tile_ring_kernel<2, 2, 2, 1, EPI_F32><<<grid, 256, 0, s>>>(a);
    else launch_tile_ring<4, 2, 2, 1>(a, epi, grid, s);
    return splits;
  }
  int per = ceil_div(k_tiles, epi == EPI_F32 ? pl.splits : 1);
  const int splits = ceil_div(k_tiles, per);
  a.k_tiles_per_split = per;
  dim3 grid(ceil_div(n_tiles, pl.nt), ceil_div(a.M, 16 * pl.mt), splits);
  if (a.touch.wgs > 0 && grid.z == 1) {
    a.touch_x0 = (int)grid.x;
    grid.x += (unsigned)a.touch.wgs;
  } else {
    a.touch.wgs = 0;
  }
  if (pl.mt == 1) launch_stream_mt<1, 4>(a, epi, pl, grid, s);
  else if (pl.mt == 2) launch_stream_mt<2, 4>(a, epi, pl, grid, s);
  else launch_stream_mt<4, 2>(a, epi, pl, grid, s);
  return splits;
}

// ---------------------------------------------------------------- log-prob from the parts
// one thread per row; parts are [part][row], so a wavefront reads 64 consecutive rows
__global__ __launch_bounds__(256) void lse_finish_kernel(const float* __restrict__ lse_max,
                                                         const float* __restrict__ lse_sum,
                                                         const float* __restrict__ lse_tgt,
                                                         const int* __restrict__ target, int parts, int stride,
                                                         int rows, float* __restrict__ out) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= rows) return;
  if (target[r] < 0) {
    out[r] = 0.f;
    return;
  }
  float mx = -INFINITY, sm = 0.f;
  for (int q = 0; q < parts; ++q) {
    const float pm = lse_max[(long long)q * stride + r], ps = lse_sum[(long long)q * stride + r];
    if (pm > mx) {
      sm = sm * expf(mx - pm) + ps;  // exp(-inf) = 0 on the first part
      mx = pm;
    } else if (pm > -INFINITY) {
      sm += ps * expf(pm - mx);
    }
  }
  out[r] = lse_tgt[r] - mx - logf(sm);
}
void launch_lse_finish(const float* lse_max, const float* lse_sum, const float* lse_tgt, const int* target,
                       int parts, int stride, int rows, float* out, hipStream_t s) {
  if (rows) lse_finish_kernel<<<ceil_div(rows, 256), 256, 0, s>>>(lse_max, lse_sum, lse_tgt, target, parts, stride, rows, out);
}

// ---------------------------------------------------------------- weight re-ordering
// dst tile (tile_offset + nt * tile_stride) <- rows nt*16.. of src [N][K] (row-major bf16).
// A wavefront moves 8 rows x 128 bytes - two k-tiles of half a row tile - so that both its
// reads and its writes are whole cache lines (lane = row * 8 + chunk; chunk = k-tile * 4 +
// column group; the 8 rows of one chunk land in 8 consecutive 16-byte slots of a fragment).
// An odd last k-tile is moved as 16 rows x 64 bytes by the first 64 lanes' worth of pieces.
__global__ void pack_weight_kernel(const uint16_t* __restrict__ src, uint4* __restrict__ dst, int N, int K,
                                   int tile_offset, int tile_stride) {
  const int k_tiles = K >> 5, k_pairs = k_tiles >> 1;
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;  // one 16-byte piece each
  const long long paired = (long long)(N >> 4) * k_pairs * 128;
  if (idx < paired) {
    const int lane = (int)(idx & 63);
    long long t = idx >> 6;
    const int half = (int)(t & 1);
    t >>= 1;
    const int kp = (int)(t % k_pairs), nt = (int)(t / k_pairs);
    const int r = half * 8 + (lane >> 3), chunk = lane & 7;
    const int kt = 2 * kp + (chunk >> 2), g = chunk & 3;
    const uint4 v = *(const uint4*)(src + (long long)(nt * 16 + r) * K + kt * 32 + g * 8);
    dst[((long long)(tile_offset + nt * tile_stride) * k_tiles + kt) * 64 + g * 16 + r] = v;
    return;
  }
  if (!(k_tiles & 1)) return;
  const long long rest = idx - paired;  // the odd last k-tile of every row tile
  if (rest >= (long long)(N >> 4) * 64) return;
  const int lane = (int)(rest & 63), nt = (int)(rest >> 6), kt = k_tiles - 1;
  const int r = lane & 15, g = lane >> 4;
  const uint4 v = *(const uint4*)(src + (long long)(nt * 16 + r) * K + kt * 32 + g * 8);
  dst[((long long)(tile_offset + nt * tile_stride) * k_tiles + kt) * 64 + lane] = v;
}
void launch_pack_weight(const void* src, void* dst, int N, int K, int tile_offset, int tile_stride, hipStream_t s) {
  long long total = (long long)(N >> 4) * (K >> 5) * 64;
  if (total) pack_weight_kernel<<<ceil_div(total, 256), 256, 0, s>>>((const uint16_t*)src, (uint4*)dst, N, K,
                                                                      tile_offset, tile_stride);
}
