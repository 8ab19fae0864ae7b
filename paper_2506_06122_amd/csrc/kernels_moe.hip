// Mixture-of-experts block of the matrix-core path: routing and the plan of the grouped
// expert projections.  The projections themselves are gemm_tile_kernel launches whose row
// blocks each belong to one expert (kernels_gemm.hip); the weighted sum of the experts'
// results rides in row_norm_kernel (kernels_rows.hip).
//
// Routing follows the usual top-k definition: the k largest router logits of a row, ties to
// the lower expert index; mixing weights are the softmax over those k logits.  Each pick gets
// a position inside its expert's list from an integer atomic counter: which pick gets which
// position depends on timing, but no result depends on the position - a slot's projection
// rows are computed independently and a row's picks are summed in pick order.
#include "kernels_fast.h"

#define MOE_MAX_PER_LANE 4  // n_experts <= 256
#define NO_EXPERT 0x7fffffff

// one wavefront per row
__global__ __launch_bounds__(256) void moe_route_topk_kernel(MoeRouteArgs a) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= a.rows) return;
  float v[MOE_MAX_PER_LANE];
  bool taken[MOE_MAX_PER_LANE];
#pragma unroll
  for (int q = 0; q < MOE_MAX_PER_LANE; ++q) {
    const int e = lane + 64 * q;
    float s = -INFINITY;
    if (e < a.n_experts) {
      s = 0.f;
      const float* p = a.partial + (long long)r * a.n_experts + e;
      for (int z = 0; z < a.splits; ++z) s += p[(long long)z * a.split_stride];
    }
    v[q] = s;
    taken[q] = e >= a.n_experts;
  }
  float top = 0.f, denom = 0.f, my_w = 0.f;
  int my_e = 0;
  for (int j = 0; j < a.top_k; ++j) {
    // this lane's best remaining candidate, then the wavefront's: larger logit, then lower index
    float bv = -INFINITY;
    int be = NO_EXPERT;
#pragma unroll
    for (int q = 0; q < MOE_MAX_PER_LANE; ++q)
      if (!taken[q] && (be == NO_EXPERT || v[q] > bv)) {
        bv = v[q];
        be = lane + 64 * q;
      }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o, WAVE);
      const int oe = __shfl_xor(be, o, WAVE);
      if (oe != NO_EXPERT && (be == NO_EXPERT || ov > bv || (ov == bv && oe < be))) {
        bv = ov;
        be = oe;
      }
    }
    if (j == 0) top = bv;
    const float w = expf(bv - top);
    denom += w;
#pragma unroll
    for (int q = 0; q < MOE_MAX_PER_LANE; ++q)
      if (be == lane + 64 * q) taken[q] = true;
    if (lane == j) {  // lane j keeps pick j (top_k <= 64)
      my_e = be;
      my_w = w;
    }
  }
  if (lane < a.top_k) {
    const long long o = (long long)r * a.top_k + lane;
    a.idx[o] = my_e;
    a.wt[o] = my_w / denom;
    a.pos[o] = atomicAdd(a.count + my_e, 1);
    if (a.route_log) a.route_log[o] = my_e;
  }
}
void launch_moe_route_topk(const MoeRouteArgs& a, hipStream_t s) {
  if (a.rows) moe_route_topk_kernel<<<ceil_div(a.rows, 4), 256, 0, s>>>(a);
}

// One workgroup: exclusive prefix of the expert counts, the row blocks of every expert, then
// the slot of every pick.
__global__ __launch_bounds__(1024) void moe_plan_kernel(MoePlanArgs a) {
  __shared__ int cnt[256], start[257], block0[257];
  const int t = threadIdx.x;
  if (t < 256) cnt[t] = t < a.n_experts ? a.count[t] : 0;
  __syncthreads();
  if (t <= a.n_experts) {
    int s = 0, b = 0;
    for (int e = 0; e < t; ++e) {
      s += cnt[e];
      b += (cnt[e] + kMoeBlockRows - 1) / kMoeBlockRows;
    }
    start[t] = s;
    block0[t] = b;
  }
  __syncthreads();
  if (t < a.n_experts) {
    const int n = cnt[t];
    for (int b = block0[t], r0 = 0; r0 < n; ++b, r0 += kMoeBlockRows) {
      a.group_of_block[b] = t;
      a.block_row_begin[b] = start[t] + r0;
      a.block_row_end[b] = start[t] + min(n, r0 + kMoeBlockRows);
    }
  }
  for (int b = block0[a.n_experts] + t; b < a.max_blocks; b += 1024) {
    a.group_of_block[b] = 0;
    a.block_row_begin[b] = 0;
    a.block_row_end[b] = 0;
  }
  const int picks = a.rows * a.top_k;
  for (int i = t; i < picks; i += 1024) {
    const int slot = start[a.idx[i]] + a.pos[i];
    a.row_map[slot] = i / a.top_k;
    a.slot_of[i] = slot;
  }
}
void launch_moe_plan(const MoePlanArgs& a, hipStream_t s) {
  if (a.rows) moe_plan_kernel<<<1, 1024, 0, s>>>(a);
}
