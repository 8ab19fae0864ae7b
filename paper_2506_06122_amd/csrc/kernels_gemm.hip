// bf16 projections on the matrix cores: out[m][n] = sum_k a[m][k] w[n][k], fp32 accumulate.
//
// The decoding phase is memory-bound (paper section 2.1): with few live rows every
// projection is a stream over the weight matrix.  Weights are therefore re-ordered once,
// at load time, into the fragment order of the 16x16x32 bf16 matrix instruction
//     packed[n_tile][k_tile][lane][8],  lane = (k % 32 / 8) * 16 + n % 16
// so that a wavefront reads each 16-column x 32-deep weight fragment as one contiguous
// 1 KiB load straight into registers (no LDS round trip for the operand that is read once).
// Activations (small, re-read by every workgroup, L2-resident) are staged through LDS in
// the same fragment order.  The instruction computes D = W_frag . A_frag^T, i.e. a tile of
// out^T, so each lane ends up with four consecutive output columns of one row.
//
// A workgroup of 4 wavefronts covers MT*16 rows x 4*NT*16 columns over one K split;
// split-K partials go to separate fp32 planes that the consumer kernel sums in a fixed
// order (deterministic).
#include "kernels_fast.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

union Frag {
  uint4 u;
  bf16x8 v;
};

__device__ inline float silu_f(float a) { return a / (1.0f + __expf(-a)); }

template <int MT, int NT, int KC, bool A_LDS, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs p) {
  __shared__ uint4 a_lds[A_LDS ? KC * MT * 64 : 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int n_tiles = p.N >> 4, k_tiles = p.K >> 5;
  const int nt0 = (blockIdx.x * 4 + wave) * NT;
  int m0 = blockIdx.y * (MT * 16);
  const int kt_begin = blockIdx.z * p.k_tiles_per_split;
  const int kt_end = min(k_tiles, kt_begin + p.k_tiles_per_split);
  const bool wave_active = nt0 < n_tiles;

  // grouped (per-expert) launches: this row block belongs to one group with its own weights
  const uint4* wp = (const uint4*)p.w;
  const int* row_map = nullptr;
  int m_limit = p.M;
  if (p.group_of_block) {
    int grp = p.group_of_block[blockIdx.y];
    wp += (long long)grp * p.group_stride16;
    m0 = p.block_row_begin[blockIdx.y];
    m_limit = p.block_row_end[blockIdx.y];
    row_map = p.row_map;
  }

  f32x4 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const uint16_t* a_base = (const uint16_t*)p.a;
  for (int kt = kt_begin; kt < kt_end; kt += KC) {
    const int kc = min(KC, kt_end - kt);
    // weight fragments of this chunk: contiguous 1 KiB per (n_tile, k_tile)
    Frag b[KC][NT];
    if (wave_active) {
#pragma unroll
      for (int kk = 0; kk < KC; ++kk)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          if (kk < kc && nt0 + j < n_tiles) b[kk][j].u = wp[((long long)(nt0 + j) * k_tiles + kt + kk) * 64 + lane];
    }
    if (A_LDS) {
      __syncthreads();  // previous chunk fully consumed
      for (int f = wave; f < kc * MT; f += 4) {
        int kk = f / MT, mt = f % MT;
        int m = m0 + mt * 16 + r;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (m < m_limit) {
          long long row = row_map ? row_map[m] : m;
          v = *(const uint4*)(a_base + row * p.lda + (long long)(kt + kk) * 32 + g * 8);
        }
        a_lds[(kk * MT + mt) * 64 + lane] = v;
      }
      __syncthreads();
    }
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
      if (kk < kc) {
        Frag a[MT];
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          if (A_LDS) {
            a[i].u = a_lds[(kk * MT + i) * 64 + lane];
          } else {
            int m = m0 + i * 16 + r;
            a[i].u = make_uint4(0, 0, 0, 0);
            if (m < m_limit) {
              long long row = row_map ? row_map[m] : m;
              a[i].u = *(const uint4*)(a_base + row * p.lda + (long long)(kt + kk) * 32 + g * 8);
            }
          }
        }
        if (wave_active) {
#pragma unroll
          for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[kk][j].v, a[i].v, acc[i][j], 0, 0, 0);
        }
      }
    }
  }
  if (!wave_active) return;

  // D[n][m]: lane (r, g) holds rows n = 4g..4g+3 of the tile at column m = r
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int m = m0 + i * 16 + r;
    if (m >= m_limit) continue;
    if (EPI == EPI_F32) {
      float* out = (float*)p.out + (long long)blockIdx.z * p.split_stride + (long long)m * p.ldo;
#pragma unroll
      for (int j = 0; j < NT; ++j)
        if (nt0 + j < n_tiles)
          *(float4*)(out + (nt0 + j) * 16 + g * 4) = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
    } else {  // EPI_SWIGLU_BF16: n-tiles alternate gate, up; act[m][f] = silu(gate) * up
      uint16_t* out = (uint16_t*)p.out + (long long)m * p.ldo;
#pragma unroll
      for (int j = 0; j < NT; j += 2) {
        if (nt0 + j + 1 >= n_tiles) break;
        uint16_t h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = f32_to_bf16(silu_f(acc[i][j][e]) * acc[i][j + 1][e]).bits;
        uint2 packed = make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
        *(uint2*)(out + ((nt0 + j) >> 1) * 16 + g * 4) = packed;
      }
    }
  }
}

template <int MT, int NT, int KC, bool A_LDS>
static void launch_cfg(const GemmArgs& a, int epi, dim3 grid, hipStream_t s) {
  if (epi == EPI_F32)
    gemm_bf16_kernel<MT, NT, KC, A_LDS, EPI_F32><<<grid, 256, 0, s>>>(a);
  else
    gemm_bf16_kernel<MT, NT, KC, A_LDS, EPI_SWIGLU_BF16><<<grid, 256, 0, s>>>(a);
}

int gemm_rows_per_block(int M) { return M <= 16 ? 16 : M <= 32 ? 32 : M <= 64 ? 64 : 128; }

int gemm_pick_splits(int M, int N, int K, int max_splits) {
  const int bm = gemm_rows_per_block(M);
  const int nt = bm == 128 ? 4 : 2;
  const long long blocks = (long long)ceil_div(N >> 4, 4 * nt) * ceil_div(M, bm);
  const int k_tiles = K >> 5;
  int z = (int)((768 + blocks - 1) / blocks);       // aim for about three workgroups per CU
  z = std::min(z, std::max(1, k_tiles / 8));        // at least 8 k-tiles (256 deep) per split
  return std::max(1, std::min(z, max_splits));
}

int launch_gemm_bf16(GemmArgs a, int epi, int splits, hipStream_t s) {
  if (a.M < 1 || a.N < 16) return 0;
  const int k_tiles = a.K >> 5;
  const int bm = a.rows_per_block ? a.rows_per_block : gemm_rows_per_block(a.M);
  const int nt = bm == 128 ? 4 : 2;
  const int kc = bm == 128 ? 2 : 4;
  splits = std::max(1, std::min(splits, k_tiles));
  int per = ceil_div(k_tiles, splits);
  per = ceil_div(per, kc) * kc;
  splits = ceil_div(k_tiles, per);
  a.k_tiles_per_split = per;
  const int m_blocks = a.group_of_block ? a.n_row_blocks : ceil_div(a.M, bm);
  dim3 grid(ceil_div(a.N >> 4, 4 * nt), m_blocks, splits);
  switch (bm) {
    case 16: launch_cfg<1, 2, 4, false>(a, epi, grid, s); break;
    case 32: launch_cfg<2, 2, 4, true>(a, epi, grid, s); break;
    case 64: launch_cfg<4, 2, 4, true>(a, epi, grid, s); break;
    default: launch_cfg<8, 4, 2, true>(a, epi, grid, s); break;
  }
  return splits;
}

// ---------------------------------------------------------------- weight re-ordering
// dst tile (tile_offset + nt * tile_stride) <- rows nt*16.. of src [N][K] (row-major bf16)
__global__ void pack_weight_kernel(const uint16_t* __restrict__ src, uint4* __restrict__ dst, int N, int K,
                                   int tile_offset, int tile_stride) {
  const int k_tiles = K >> 5;
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;  // one 16-byte piece each
  long long total = (long long)(N >> 4) * k_tiles * 64;
  if (idx >= total) return;
  int lane = (int)(idx & 63);
  long long t = idx >> 6;
  int kt = (int)(t % k_tiles);
  int nt = (int)(t / k_tiles);
  int r = lane & 15, g = lane >> 4;
  const uint4 v = *(const uint4*)(src + (long long)(nt * 16 + r) * K + kt * 32 + g * 8);
  dst[((long long)(tile_offset + nt * tile_stride) * k_tiles + kt) * 64 + lane] = v;
}
void launch_pack_weight(const void* src, void* dst, int N, int K, int tile_offset, int tile_stride, hipStream_t s) {
  long long total = (long long)(N >> 4) * (K >> 5) * 64;
  if (total) pack_weight_kernel<<<ceil_div(total, 256), 256, 0, s>>>((const uint16_t*)src, (uint4*)dst, N, K,
                                                                      tile_offset, tile_stride);
}
