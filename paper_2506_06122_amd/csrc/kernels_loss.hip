// Policy-gradient objective over packed rollouts: the training stage's consumer of the
// log-probs (paper sections 5.1 and 5.2: PPO loss on REINFORCE returns, rewards clipped at 20,
// advantages at 10; section 2.1: KL penalty from the reference model).  Definitions, token by
// token, in include/rollout.h.
//
// One workgroup per sequence.  The return G_j = rho_j + gamma G_{j+1} over the counted tokens
// is a first-order linear recurrence, so a chunk of 256 tokens, taken from the sequence's end,
// is a scan of affine maps y -> a y + b (a = gamma, b = rho for a counted token; the identity
// for any other): Hillis-Steele inside a wavefront, the four wavefront totals composed through
// LDS, the chunk's last value carried to the next chunk.  Sums for the loss leave as one
// partial per sequence and are added in sequence order by a second launch, so the result does
// not depend on scheduling.
#include "kernels_fast.h"

struct Affine {
  float a, b;  // y -> a y + b
};
// apply `first`, then `second`
__device__ inline Affine then(const Affine& first, const Affine& second) {
  return Affine{second.a * first.a, second.a * first.b + second.b};
}

__global__ __launch_bounds__(256) void policy_advantage_kernel(PolicyLossArgs p) {
  __shared__ int last_s[4];
  __shared__ Affine total_s[4];
  __shared__ float carry_s;
  __shared__ float sum_s[4], cnt_s[4];
  const int seq = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = p.cu_seqlens[seq], hi = p.cu_seqlens[seq + 1];
  // the sequence's last counted token takes the clipped sequence reward
  int last = -1;
  for (int t = lo + tid; t < hi; t += 256)
    if (p.mask[t]) last = max(last, t);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) last = max(last, __shfl_xor(last, o, WAVE));
  if (lane == 0) last_s[wave] = last;
  if (tid == 0) carry_s = 0.f;
  __syncthreads();
  last = max(max(last_s[0], last_s[1]), max(last_s[2], last_s[3]));
  const float reward = fminf(fmaxf(p.rewards[seq], -p.reward_clip), p.reward_clip);
  float s_sum = 0.f, s_cnt = 0.f;
  for (int top = hi; top > lo; top -= 256) {  // chunks from the end; thread 0 takes the latest token
    const int t = top - 1 - tid;
    const bool in = t >= lo;
    const bool counted = in && p.mask[t];
    float lp_new = 0.f, lp_old = 0.f;
    Affine f{1.f, 0.f};
    if (counted) {
      lp_new = p.logp_new[t];
      lp_old = p.logp_old[t];
      f.a = p.gamma;
      f.b = (p.logp_ref ? -p.kl_coef * (lp_old - p.logp_ref[t]) : 0.f) + (t == last ? reward : 0.f);
    }
    // inclusive scan over the threads: f becomes "everything from thread 0 up to this thread"
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
      Affine prev{__shfl_up(f.a, o, WAVE), __shfl_up(f.b, o, WAVE)};
      if (lane >= o) f = then(prev, f);
    }
    if (lane == WAVE - 1) total_s[wave] = f;
    __syncthreads();
    float y = carry_s;  // value entering this wavefront
    for (int w = 0; w < wave; ++w) y = total_s[w].a * y + total_s[w].b;
    const float g = f.a * y + f.b;
    __syncthreads();
    if (tid == 255) carry_s = g;
    if (in) {
      float adv = 0.f, grad = 0.f;
      if (counted) {
        adv = fminf(fmaxf(g, -p.adv_clip), p.adv_clip);
        const float r = expf(lp_new - lp_old);
        const float plain = r * adv, clipped = fminf(fmaxf(r, 1.f - p.eps_low), 1.f + p.eps_high) * adv;
        s_sum += fminf(plain, clipped);
        s_cnt += 1.f;
        if (plain <= clipped) grad = -plain;  // scaled by 1 / N in policy_scale_kernel
      }
      if (p.advantages) p.advantages[t] = adv;
      p.grad[t] = grad;
    }
    __syncthreads();
  }
  s_sum = wave_sum(s_sum);
  s_cnt = wave_sum(s_cnt);
  if (lane == 0) {
    sum_s[wave] = s_sum;
    cnt_s[wave] = s_cnt;
  }
  __syncthreads();
  if (tid == 0) {
    p.part_sum[seq] = (sum_s[0] + sum_s[1]) + (sum_s[2] + sum_s[3]);
    p.part_cnt[seq] = (cnt_s[0] + cnt_s[1]) + (cnt_s[2] + cnt_s[3]);
  }
}

// one workgroup: the per-sequence partials in sequence order, as doubles
__global__ __launch_bounds__(256) void policy_finish_kernel(PolicyLossArgs p) {
  __shared__ double s_s[256], c_s[256];
  const int tid = threadIdx.x;
  double s = 0.0, c = 0.0;
  for (int i = tid; i < p.n_seqs; i += 256) {
    s += p.part_sum[i];
    c += p.part_cnt[i];
  }
  s_s[tid] = s;
  c_s[tid] = c;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) {
      s_s[tid] += s_s[tid + o];
      c_s[tid] += c_s[tid + o];
    }
    __syncthreads();
  }
  if (tid == 0) {
    const double n = c_s[0];
    p.result[0] = n > 0 ? (float)(-s_s[0] / n) : 0.f;
    p.result[1] = n > 0 ? (float)(1.0 / n) : 0.f;
  }
}

__global__ __launch_bounds__(256) void policy_scale_kernel(float* __restrict__ grad, const float* __restrict__ result,
                                                           long long total) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t < total) grad[t] *= result[1];
}

void launch_policy_loss(const PolicyLossArgs& p, hipStream_t s) {
  if (p.n_seqs > 0) policy_advantage_kernel<<<p.n_seqs, 256, 0, s>>>(p);
  policy_finish_kernel<<<1, 256, 0, s>>>(p);
  if (p.total > 0) policy_scale_kernel<<<(unsigned)ceil_div(p.total, 256), 256, 0, s>>>(p.grad, p.result, p.total);
}
