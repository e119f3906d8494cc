// Exact scores of the candidates (k_score) and the likelihood / prior they are built from.
#pragma once
#include "sweep.h"

namespace rtk {

// --------------------------------------------------------------- k_score ----
// Likelihood factor of an entry that was sent in the previous round.
__device__ __forceinline__ float likelihood_sent(float a_now, float a_before, float g_before,
                                                 float w, float mu, int kind) {
  const float num = __fsub_rn(g_before, __fmul_rn(w, a_before));
  const float den = __fmul_rn(w, a_now);
  if (den == 0.0f) return 1.0f;
  const float D = __fdiv_rn(num, den);
  const float r = fabsf(__fadd_rn(1.0f, D));
  const float x = __fdiv_rn(r, mu);
  if (x != x) return 1.0f;
  if (kind == 1) return x < 1.0f ? x : 1.0f;     // cumulative function of a uniform innovation
  if (kind == 2) return erf_f32_cr(x);           // of a Gaussian innovation (constants dropped as for tanh)
  return tanh_f32_cr(x);
}

// What the score variants need: the number of square roots of the prior and
// the kind of likelihood (0 tanh, 1 clipped linear, 2 erf).
struct ScoreKind { int roots, likelihood; };

// Score bits of one candidate: index word `raw` with the sent flag, value a,
// and a_before = the value the worker sent for this entry in the previous
// round (read only when the flag is set).
__device__ __forceinline__ uint32_t score_entry(uint32_t raw, float a, float a_before, int use_reg,
                                                const float* __restrict__ gprev, float w, float mu,
                                                ScoreKind sk) {
  float f = 1.0f;
  if (use_reg && (raw & kSentFlag)) f = likelihood_sent(a, a_before, gprev[raw & ~kSentFlag], w, mu, sk.likelihood);
  return __float_as_uint(__fmul_rn(prior_of(a, sk.roots), f));
}

// grid (ceil(cap_r/2048), regions, N): a block covers 2048 consecutive slots of
// one region of the speculative candidate list, eight per thread.
constexpr int kScoreSlots = 2048;

// VARIANTS = false: the score of Algorithm 2 (plain prior, tanh) only -- the
// code of the other priors and likelihoods (double-precision power and erf)
// would otherwise cost this kernel registers, and with them resident waves, in
// every round.
template <bool VARIANTS>
__global__ void __launch_bounds__(kBlock)
k_score(WorkerCtl* __restrict__ ctl, const int32_t* __restrict__ cand_idx,
        const float* __restrict__ cand_val, const float* __restrict__ cand_prev,
        uint32_t* __restrict__ cand_key, uint32_t* __restrict__ bnd_key,
        const float* __restrict__ gprev, int64_t d, uint32_t cap_r,
        uint32_t cap_total, uint32_t bnd_cap, const float* __restrict__ omega, float mu, int use_reg,
        ScoreKind sk_in) {
  const ScoreKind sk = VARIANTS ? sk_in : ScoreKind{0, 0};
  __shared__ uint32_t s_stage[kScoreSlots];
  __shared__ uint32_t s_cnt[3];       // boundary entries, valid, above window
  __shared__ uint32_t s_base;
  const uint32_t n = blockIdx.z, r = blockIdx.y, tid = threadIdx.x;
  WorkerCtl& c = ctl[n];
  if (c.overflow) return;                     // list is incomplete; the dense selection rebuilds it
  const uint32_t lim = region_limit(c, r, cap_r);
  const uint32_t p0 = blockIdx.x * kScoreSlots;
  if (p0 >= lim) return;
  const uint32_t tau_lo = c.tau_lo, win_lo = c.win_lo, win_hi = c.win_hi;
  const bool windowed = win_lo != kNoBound;
  if (tid < 3) s_cnt[tid] = 0;
  __syncthreads();
  const size_t cbase = (size_t)n * cap_total + (size_t)r * cap_r;
  const float w = omega[n];
  uint32_t n_val = 0, n_hi = 0;
  // all loads of the thread's slots are issued before anything is computed, so
  // the block pays the memory latency once per stage, not once per slot
  constexpr int kPer = kScoreSlots / kBlock;
  uint32_t raw[kPer];
  float av[kPer], ab[kPer], gp[kPer];
#pragma unroll
  for (int q = 0; q < kPer; ++q) {
    const uint32_t p = p0 + q * kBlock + tid;
    const bool in = p < lim;
    raw[q] = in ? (uint32_t)cand_idx[cbase + p] : 0xFFFFFFFFu;
    av[q] = in ? cand_val[cbase + p] : 0.0f;
    ab[q] = (in && use_reg) ? cand_prev[cbase + p] : 0.0f;
  }
#pragma unroll
  for (int q = 0; q < kPer; ++q) {
    const uint32_t j = raw[q] & ~kSentFlag;
    if ((int64_t)j >= d) raw[q] = 0xFFFFFFFFu;               // empty slot
    gp[q] = (use_reg && raw[q] != 0xFFFFFFFFu && (raw[q] & kSentFlag)) ? gprev[j] : 0.0f;
  }
#pragma unroll
  for (int q = 0; q < kPer; ++q) {
    if (raw[q] == 0xFFFFFFFFu) continue;
    const uint32_t p = p0 + q * kBlock + tid;
    float f = 1.0f;
    if (use_reg && (raw[q] & kSentFlag)) f = likelihood_sent(av[q], ab[q], gp[q], w, mu, sk.likelihood);
    const uint32_t key = __float_as_uint(__fmul_rn(prior_of(av[q], sk.roots), f));
    cand_key[cbase + p] = key;
    n_val += key >= tau_lo;
    if (windowed) {
      if (key >= win_hi) ++n_hi;
      else if (key >= win_lo) s_stage[atomicAdd(&s_cnt[0], 1u)] = key;
    }
  }
  for (int o = 32; o > 0; o >>= 1) { n_val += __shfl_down(n_val, o); n_hi += __shfl_down(n_hi, o); }
  if ((tid & 63) == 0) {
    if (n_val) atomicAdd(&s_cnt[1], n_val);
    if (n_hi) atomicAdd(&s_cnt[2], n_hi);
  }
  __syncthreads();
  const uint32_t nb = s_cnt[0];
  if (tid == 0) {
    if (s_cnt[1]) atomicAdd(&c.n_valid, s_cnt[1]);
    if (s_cnt[2]) atomicAdd(&c.n_hi, s_cnt[2]);
    uint32_t b = 0;
    if (nb) b = atomicAdd(&c.n_bnd, nb);       // n_bnd > bnd_cap marks an overflow of the list
    s_base = b;
  }
  __syncthreads();
  if (nb == 0) return;
  const uint32_t b = s_base;
  if (b + nb > bnd_cap) return;
  uint32_t* out = bnd_key + (size_t)n * bnd_cap + b;
  for (uint32_t i = tid; i < nb; i += kBlock) out[i] = s_stage[i];
}

}  // namespace rtk
