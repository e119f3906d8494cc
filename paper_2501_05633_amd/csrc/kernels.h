// HIP kernels of the RegTop-k round for gfx950 (wave64).
//
// Data flow of one round (all N workers batched; rows of length d):
//
//   k_begin         reset counters, load this round's speculative bound and window
//   k_accum_emit    a = eps + g written over eps (the one dense read/write sweep);
//                   eps is taken as 0 where the previous round's mask bit is set
//                   (the sent entries are never zeroed in memory: one bit per
//                   entry is read here instead of k scattered writes per worker);
//                   entries with |a| >= tau_lo are appended, in index order per
//                   4096-entry chunk, to the worker's candidate list
//   k_score         exact score of every candidate (regulariser for entries sent in
//                   the previous round; the value sent then travels with the
//                   candidate: the sweep finds it in the state it overwrites);
//                   scores inside a narrow window around the expected
//                   k-th score are also copied to a short boundary list, those
//                   above it are counted
//   k_select        one block per worker: checks the speculation (no overflow and
//                   >= k candidates scored >= tau_lo), then finds the k-th largest
//                   score exactly - from the boundary list held in LDS when the
//                   window contains it, otherwise by a three-level radix select
//                   over all candidates - and derives next round's bound/window
//   k_dense_all     for workers whose speculation failed (and in round 0): exact
//                   radix select of the 2k largest |a| (a superset of the true
//                   top-k, see below), count, scan and an ordered emission of
//                   exactly those entries as the candidate list, then their
//                   scores and the exact k-th score; one kernel with grid
//                   barriers between its phases, which returns at once when no
//                   worker is flagged
//   k_chunk_count / k_chunk_scan / k_compact
//                   ordered compaction of the selected (index, value) pairs,
//                   lowest-index ties first; writes the round's mask (1 bit per
//                   entry)
//   k_aggregate     per 4096-entry tile: LDS accumulation of w*value in ascending
//                   worker order, tile written once (zero fill included)
//
// Why 2k largest |a| suffice when the speculation fails: the score never
// exceeds |a| and differs from it only on the k entries sent in the previous
// round; among the 2k entries with the largest (|a|, lower index first) at
// least k are therefore scored at their full |a|, and each of them beats every
// entry outside that set.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tanh_cr.h"

namespace rtk {

constexpr int kChunk = 4096;        // entries per chunk (one block iteration, one aggregation tile)
constexpr int kChunkLog = 12;
constexpr int kBlock = 256;
constexpr int kMaxRegions = 64;
constexpr uint32_t kNoBound = 0xFFFFFFFFu;
constexpr int kChunkWords = kChunk / 32;   // mask words per chunk
constexpr uint32_t kSentFlag = 0x80000000u; // in a candidate's index: the entry was sent in the previous round

// score bits (sign bit is always 0): level 1 = bits 30..19, level 2 = 18..8, level 3 = 7..0
constexpr int kL1Shift = 19, kL1Bins = 4096;
constexpr int kL2Shift = 8, kL2Bins = 2048;
constexpr int kL3Bins = 256;

// half width of the window around the predicted k-th score, in bit patterns
constexpr uint32_t kWinMaxHalf = 1u << 22, kWinMinHalf = 1u << 10, kWinDefaultHalf = 1u << 16;

struct WorkerCtl {
  uint32_t tau_lo;        // speculative lower bound on the k-th score (bit pattern) or kNoBound
  uint32_t next_tau_lo;   // bound for the next round
  uint32_t win_lo;        // window [win_lo, win_hi) around the expected k-th score, or kNoBound
  uint32_t win_hi;
  uint32_t next_win_lo;
  uint32_t next_win_hi;
  uint32_t overflow;      // a candidate region overflowed in k_accum_emit
  uint32_t need_dense;    // dense selection runs for this worker
  uint32_t n_cand;        // candidates handed to the exact selection
  uint32_t n_valid;       // candidates with score >= tau_lo
  uint32_t n_hi;          // candidates with score >= win_hi
  uint32_t n_bnd;         // candidates with score inside the window (boundary list length)
  uint32_t dense_total;   // candidates written by the dense emission (compact from slot 0)
  uint32_t used_window;   // 1 if the k-th score was found from the boundary list
  uint32_t tau;           // k-th largest score (bits)
  uint32_t n_gt;          // candidates with score > tau
  uint32_t budget;        // ties to take, lowest indices first
  uint32_t ties_total;
  uint32_t f_prefix;      // radix-select state of the dense selection over |a| bits
  uint32_t f_krem;
  uint32_t f_tau;
  uint32_t f_budget;
  uint32_t err;           // bit 0: selected count != k, bit 1: bad set_state input
  uint32_t tau_prev;      // k-th score of the previous round or kNoBound
  uint32_t centre;        // predicted k-th score of this round (window centre) or kNoBound
  uint32_t err_prev;      // |prediction error| of the previous round
  float margin_scale;     // widens the bound's safety margin after a failed speculation
  uint32_t extrapolated;  // this round's prediction used the drift of two earlier rounds
  uint32_t tau_lo_mag;    // smallest |a| bit pattern whose prior reaches tau_lo (= tau_lo for the plain prior)
  uint32_t pad[3];
  uint32_t cursor[kMaxRegions];
};

__device__ __forceinline__ uint32_t lanes_below(uint64_t ballot) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

__device__ __forceinline__ uint32_t key_of(float a) { return __float_as_uint(a) & 0x7FFFFFFFu; }

// Prior |a|^y for y = 2^-roots, roots = 0..3 (appendix remark on sub-linear
// scaling): `roots` correctly rounded binary32 square roots of |a|.
__device__ __forceinline__ float prior_of(float a, int roots) {
  float p = fabsf(a);
  for (int i = 0; i < roots; ++i) p = sqrtf(p);      // correctly rounded (the __fsqrt_rn intrinsic is the approximate one here)
  return p;
}
__device__ __forceinline__ uint32_t prior_key(float a, int roots) { return __float_as_uint(prior_of(a, roots)); }

// Smallest |a| bit pattern whose prior reaches the score bound tau (bit
// pattern): the sweep compares magnitudes, the bound lives in score space, and
// the prior is monotone but not one-to-one.  kNoBound stays kNoBound; a bound
// no finite magnitude reaches gives the pattern of +inf.
__device__ __forceinline__ uint32_t magnitude_bound(uint32_t tau, int roots) {
  if (roots == 0 || tau == 0xFFFFFFFFu) return tau;
  uint32_t lo = 0, hi = 0x7F800000u;              // prior(hi) = +inf >= any finite tau
  while (lo < hi) {
    const uint32_t mid = lo + (hi - lo) / 2;
    if (prior_key(__uint_as_float(mid), roots) >= tau) hi = mid; else lo = mid + 1;
  }
  return lo;
}

// Number of valid candidate slots in region r of a worker's list.  The
// speculative sweep fills every region from its own cursor; the dense emission
// writes one compact run from slot 0 across the region boundaries.
__device__ __forceinline__ uint32_t region_limit(const WorkerCtl& c, uint32_t r, uint32_t cap_r) {
  if (c.need_dense) {
    const uint32_t lo = r * cap_r;
    if (c.dense_total <= lo) return 0;
    const uint32_t left = c.dense_total - lo;
    return left < cap_r ? left : cap_r;
  }
  const uint32_t cur = c.cursor[r];
  return cur < cap_r ? cur : cap_r;
}

// Exclusive prefix sum over the NT threads of a block; *total gets the sum.
constexpr int kScanBlock = 1024;

template <int NT>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* s_w /*[16]*/, uint32_t* total) {
  const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  uint32_t x = v;
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(x, o);
    if (lane >= (uint32_t)o) x += y;
  }
  if (lane == 63) s_w[wv] = x;
  __syncthreads();
  uint32_t wb = 0, tot = 0;
  for (uint32_t i = 0; i < NT / 64; ++i) { const uint32_t t = s_w[i]; if (i < wv) wb += t; tot += t; }
  __syncthreads();
  *total = tot;
  return wb + x - v;
}

// State shared by all workers of a context.
struct GlobalCtl {
  uint32_t any_dense;     // some worker needs the dense selection this round
  uint32_t bar_count;     // grid barrier of the dense selection: arrivals
  uint32_t bar_gen;       //   and generation
  uint32_t bar_err;       // a barrier wait ran into its spin limit (reported as an error)
  uint32_t pad[60];
};

// Barrier across the (co-resident) blocks of the dense-selection kernel.  Every
// wait is bounded: after kBarrierSpinLimit polls a block gives up, records the
// fact and carries on, so the grid always drains.
constexpr uint32_t kBarrierSpinLimit = 1u << 22;

__device__ __forceinline__ void grid_barrier(GlobalCtl* g, uint32_t nblocks) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __threadfence();
    const uint32_t gen = __hip_atomic_load(&g->bar_gen, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t arrived = atomicAdd(&g->bar_count, 1u) + 1u;
    if (arrived == nblocks) {
      __hip_atomic_store(&g->bar_count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __threadfence();
      atomicAdd(&g->bar_gen, 1u);
    } else {
      uint32_t spins = 0;
      // relaxed polls with a pause: an acquiring load per poll makes the hundreds of waiting blocks
      // slow down the few that work in the one-block-per-worker phases (the fence below orders the exit)
      while (__hip_atomic_load(&g->bar_gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gen) {
        __builtin_amdgcn_s_sleep(32);
        if (++spins > kBarrierSpinLimit) { atomicOr(&g->bar_err, 1u); break; }
      }
    }
  }
  __syncthreads();
  __threadfence();
}

// ---------------------------------------------------------------- k_begin ----
__global__ void __launch_bounds__(kBlock)
k_begin(WorkerCtl* ctl, GlobalCtl* gctl, int force_dense, int roots) {
  const uint32_t n = blockIdx.x, tid = threadIdx.x;
  if (n == 0 && tid == 0) gctl->any_dense = 0;
  WorkerCtl& c = ctl[n];
  if (tid < kMaxRegions) c.cursor[tid] = 0;
  if (tid == 0) {
    c.tau_lo = force_dense ? kNoBound : c.next_tau_lo;
    c.tau_lo_mag = magnitude_bound(c.tau_lo, roots);
    c.win_lo = force_dense ? kNoBound : c.next_win_lo;
    c.win_hi = c.next_win_hi;
    c.overflow = 0; c.need_dense = 0; c.n_cand = 0; c.n_valid = 0; c.n_hi = 0; c.n_bnd = 0;
    c.dense_total = 0; c.used_window = 0;
    c.tau = 0; c.n_gt = 0; c.budget = 0; c.ties_total = 0;
    c.f_prefix = 0; c.f_krem = 0; c.f_tau = 0; c.f_budget = 0;
  }
}

// ----------------------------------------------------- chunk in registers ----
// A block of 256 threads holds one chunk of 4096 entries: wave v covers entries
// [v*1024, v*1024+1024) of the chunk, iteration i the 256 entries after i*256,
// lane l the four entries at l*4.  flags bit (i*4+c) marks entry (i, l, c).
// ordered_positions gives every flagged entry its rank in ascending index order
// within the block and returns the block's total.
struct ChunkPos {
  uint32_t lane_base[4];   // rank of the lane's first flagged entry of iteration i within the wave
  uint32_t wave_base;      // flagged entries in lower waves
  uint32_t total;          // flagged entries in the block
};

__device__ __forceinline__ ChunkPos ordered_positions(uint32_t flags, uint32_t* s_wtot /*[4]*/) {
  const uint32_t tid = threadIdx.x, wv = tid >> 6;
  ChunkPos cp;
  uint32_t run = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t below = 0, tot = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint64_t b = __ballot((flags >> (i * 4 + c)) & 1u);
      below += lanes_below(b);
      tot += (uint32_t)__popcll(b);
    }
    cp.lane_base[i] = run + below;
    run += tot;
  }
  if ((tid & 63) == 0) s_wtot[wv] = run;
  __syncthreads();
  uint32_t wb = 0, total = 0;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const uint32_t x = s_wtot[v];
    if (v < (int)wv) wb += x;
    total += x;
  }
  cp.wave_base = wb;
  cp.total = total;
  return cp;
}

// ---------------------------------------------------------- k_accum_emit ----
// grid (nc, N).  VEC: d % 4 == 0 and 16-byte aligned rows.  The sweep touches
// every byte exactly once, so it loads and stores with the non-temporal hint.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Local gradients arrive as binary32 or as bfloat16 (the upper half of a
// binary32 pattern: widening is exact, the arithmetic stays binary32).
struct bf16_t { uint16_t bits; };
__device__ __forceinline__ float grad_at(const float* g, size_t i) { return g[i]; }
__device__ __forceinline__ float grad_at(const bf16_t* g, size_t i) {
  return __uint_as_float((uint32_t)g[i].bits << 16);
}
// four consecutive gradients from an address aligned to the four of them
__device__ __forceinline__ f32x4 grad4_at(const float* g, size_t i) {
  return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g + i));
}
__device__ __forceinline__ f32x4 grad4_at(const bf16_t* g, size_t i) {
  const u32x2 w = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(g + i));
  f32x4 r;
  r.x = __uint_as_float(w.x << 16);
  r.y = __uint_as_float(w.x & 0xFFFF0000u);
  r.z = __uint_as_float(w.y << 16);
  r.w = __uint_as_float(w.y & 0xFFFF0000u);
  return r;
}

template <bool VEC, typename G>
__global__ void __launch_bounds__(kBlock)
k_accum_emit(float* __restrict__ e, const G* __restrict__ g, const uint32_t* __restrict__ mask,
             const uint32_t* __restrict__ prev_sel_off, int64_t d, WorkerCtl* __restrict__ ctl,
             int32_t* __restrict__ cand_idx,
             float* __restrict__ cand_val, float* __restrict__ cand_prev, uint32_t* __restrict__ ch_off,
             uint32_t* __restrict__ ch_cnt, uint32_t nc, uint32_t cap_r, uint32_t cap_total,
             uint32_t regions) {
  __shared__ uint32_t s_wtot[4];
  __shared__ uint32_t s_base;
  const uint32_t c = blockIdx.x, n = blockIdx.y;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const size_t row = (size_t)n * (size_t)d;
  const uint32_t tau_lo = ctl[n].tau_lo_mag;        // bound on |a|: the sweep never evaluates the prior
  const int64_t base = (int64_t)c * kChunk + (int64_t)wv * 1024 + lane * 4;
  float a[4][4];
  float eo[4][4];       // what the state held: a^{t-1} where the entry was sent, the error elsewhere
  uint32_t flags = 0;
  // previous round's mask: the 4 bits of entries j0..j0+3 lie in one word
  // (chunks from which nothing was sent have no mask bits: their words are not read)
  const uint32_t* mrow = mask + (size_t)n * nc * kChunkWords;
  const bool sent_any = prev_sel_off[(size_t)n * (nc + 1) + c + 1] != prev_sel_off[(size_t)n * (nc + 1) + c];
  uint32_t mb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t j0 = base + i * 256;
    mb[i] = (sent_any && j0 < d) ? (mrow[j0 >> 5] >> (j0 & 31)) & 15u : 0u;
  }
  if (VEC) {
    f32x4 ev[4], gv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t j0 = base + i * 256;
      if (j0 < d) {
        ev[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(e + row + j0));
        gv[i] = grad4_at(g, row + j0);
      } else {
        ev[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        gv[i] = ev[i];
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t j0 = base + i * 256;
      eo[i][0] = ev[i].x; eo[i][1] = ev[i].y; eo[i][2] = ev[i].z; eo[i][3] = ev[i].w;
      f32x4 z4 = ev[i];
      if (mb[i]) {                          // sent last round: the error restarts from zero
        if (mb[i] & 1u) z4.x = 0.f;
        if (mb[i] & 2u) z4.y = 0.f;
        if (mb[i] & 4u) z4.z = 0.f;
        if (mb[i] & 8u) z4.w = 0.f;
      }
      const f32x4 s4 = z4 + gv[i];
      a[i][0] = s4.x; a[i][1] = s4.y; a[i][2] = s4.z; a[i][3] = s4.w;
      if (j0 < d) {
        __builtin_nontemporal_store(s4, reinterpret_cast<f32x4*>(e + row + j0));
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (key_of(a[i][q]) >= tau_lo) flags |= 1u << (i * 4 + q);
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int64_t j = base + i * 256 + q;
        a[i][q] = 0.f;
        eo[i][q] = 0.f;
        if (j < d) {
          eo[i][q] = e[row + j];
          const float eps = ((mb[i] >> q) & 1u) ? 0.f : eo[i][q];
          a[i][q] = eps + grad_at(g, row + j);
          e[row + j] = a[i][q];
          if (key_of(a[i][q]) >= tau_lo) flags |= 1u << (i * 4 + q);
        }
      }
    }
  }
  const ChunkPos cp = ordered_positions(flags, s_wtot);
  const size_t tix = (size_t)n * nc + c;
  if (cp.total == 0) {
    if (tid == 0) { ch_off[tix] = 0; ch_cnt[tix] = 0; }
    return;
  }
  if (tid == 0) {
    const uint32_t r = c % regions;
    const uint32_t off = atomicAdd(&ctl[n].cursor[r], cp.total);
    uint32_t b = kNoBound;
    if (off + cp.total <= cap_r) b = r * cap_r + off;
    else ctl[n].overflow = 1;
    s_base = b;
    ch_off[tix] = (b == kNoBound) ? 0 : b;
    ch_cnt[tix] = (b == kNoBound) ? 0 : cp.total;
  }
  __syncthreads();
  const uint32_t b = s_base;
  if (b == kNoBound || flags == 0) return;
  const size_t out = (size_t)n * cap_total + b + cp.wave_base;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t p = cp.lane_base[i];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if ((flags >> (i * 4 + q)) & 1u) {
        cand_idx[out + p] = (int32_t)((uint32_t)(base + i * 256 + q) | (((mb[i] >> q) & 1u) ? kSentFlag : 0u));
        cand_val[out + p] = a[i][q];
        cand_prev[out + p] = eo[i][q];
        ++p;
      }
    }
  }
}

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
  return tanh_f32_cr(x);
}

// What the score variants need: the number of square roots of the prior and
// the kind of likelihood (0 tanh, 1 clipped linear).
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

__global__ void __launch_bounds__(kBlock)
k_score(WorkerCtl* __restrict__ ctl, const int32_t* __restrict__ cand_idx,
        const float* __restrict__ cand_val, const float* __restrict__ cand_prev,
        uint32_t* __restrict__ cand_key, uint32_t* __restrict__ bnd_key,
        const float* __restrict__ gprev, int64_t d, uint32_t cap_r,
        uint32_t cap_total, uint32_t bnd_cap, const float* __restrict__ omega, float mu, int use_reg,
        ScoreKind sk) {
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

// -------------------------------------------------------------- k_select ----
// One block of 1024 threads per worker.
struct RankHit { uint32_t bin, above; };   // bin == kNoBound: rank not reached

// Descending search in an LDS histogram: the bin b with
//   count(bins > b) < want <= count(bins >= b);  above = count(bins > b).
// nbins in {16, 512, 4096}.  All NT threads of the block call it.
template <int NT>
__device__ __forceinline__ RankHit find_rank_desc(const uint32_t* hist, uint32_t nbins, uint32_t want,
                                                  uint32_t* s_w, uint32_t* s_out) {
  const uint32_t tid = threadIdx.x;
  const uint32_t per = nbins >= (uint32_t)NT ? nbins / NT : 1u;
  constexpr uint32_t kMaxPer = 4096 / NT;
  uint32_t loc[kMaxPer];
  uint32_t s = 0;
#pragma unroll
  for (uint32_t q = 0; q < kMaxPer; ++q) {
    const uint32_t i = tid * per + q;
    loc[q] = (q < per && i < nbins) ? hist[nbins - 1 - i] : 0u;
    s += loc[q];
  }
  if (tid == 0) { s_out[0] = kNoBound; s_out[1] = 0; }
  uint32_t total;
  const uint32_t above = block_excl_scan<NT>(s, s_w, &total);
  if (above < want && want <= above + s) {
    uint32_t run = above;
#pragma unroll
    for (uint32_t q = 0; q < kMaxPer; ++q) {
      if (run < want && want <= run + loc[q]) { s_out[0] = nbins - 1 - (tid * per + q); s_out[1] = run; }
      run += loc[q];
    }
  }
  __syncthreads();
  RankHit h{s_out[0], s_out[1]};
  __syncthreads();
  return h;
}

// Where the keys of a selection come from: the short boundary list (in LDS
// when it fits, else in memory) or all candidate regions of the worker.
struct KeySource {
  const uint32_t* lds;      // non-null: count keys in LDS
  const uint32_t* flat;     // non-null: count keys, contiguous in memory
  const uint32_t* regions;  // else: candidate regions of cap_r slots each
  uint32_t count, cap_r, n_regions;
  const WorkerCtl* ctl;
};

// Calls f(key) for every key of the source; memory is read 128 bits at a time,
// two loads in flight per thread.
template <int NT, typename F>
__device__ __forceinline__ void for_each_key(const KeySource& src, F f) {
  const uint32_t tid = threadIdx.x;
  if (src.lds) {
    for (uint32_t i = tid; i < src.count; i += NT) f(src.lds[i]);
    return;
  }
  const uint32_t nseg = src.flat ? 1u : src.n_regions;
  for (uint32_t r = 0; r < nseg; ++r) {
    const uint32_t lim = src.flat ? src.count : region_limit(*src.ctl, r, src.cap_r);
    const uint32_t* base = src.flat ? src.flat : src.regions + (size_t)r * src.cap_r;
    const uint4* b4 = reinterpret_cast<const uint4*>(base);
    const uint32_t n4 = lim / 4;
    uint32_t i = tid;
    for (; i + NT < n4; i += 2 * NT) {
      const uint4 x = b4[i], y = b4[i + NT];
      f(x.x); f(x.y); f(x.z); f(x.w); f(y.x); f(y.y); f(y.z); f(y.w);
    }
    if (i < n4) { const uint4 x = b4[i]; f(x.x); f(x.y); f(x.z); f(x.w); }
    if (tid < lim - n4 * 4) f(base[n4 * 4 + tid]);
  }
}

// Exact `rank`-th largest key among the keys >= base of the source; at least
// `rank` such keys must exist.  Three histogram levels over rel = key - base:
// bits 24..13 (keys with rel >= 2^25 are counted apart; if the rank lies among
// them the base moves up by 2^25 and the level is repeated), bits 12..4, bits
// 3..0.  The fine first level spreads neighbouring scores over many bins, so
// the LDS atomics rarely collide.  Returns tau; *budget = how many keys equal
// to tau belong to the top `rank`; *ties = keys equal to tau.
template <int NT>
__device__ __forceinline__ uint32_t rel_select(KeySource src, uint32_t base, uint32_t rank,
                                               uint32_t* s_hist, uint32_t* s_w, uint32_t* s_out,
                                               uint32_t* s_stash, uint32_t stash_cap,
                                               uint32_t* budget, uint32_t* ties) {
  const uint32_t tid = threadIdx.x;
  uint32_t want = rank;
  RankHit ha{0u, 0u};
  for (int guard = 0; guard < 64; ++guard) {
    for (uint32_t i = tid; i < kL1Bins; i += NT) s_hist[i] = 0;
    __syncthreads();
    uint32_t over = 0;
    for_each_key<NT>(src, [&](uint32_t key) {
      if (key < base) return;
      const uint32_t rel = key - base;
      if (rel >> 25) ++over;
      else atomicAdd(&s_hist[rel >> 13], 1u);
    });
    uint32_t n_over;
    (void)block_excl_scan<NT>(over, s_w, &n_over);     // also orders the LDS atomics
    if (want > n_over) {
      want -= n_over;
      ha = find_rank_desc<NT>(s_hist, kL1Bins, want, s_w, s_out);
      break;
    }
    base += 1u << 25;                                   // the rank lies higher up
    __syncthreads();
  }
  want -= ha.above;
  const uint32_t pa = ha.bin;
  // the keys of that bin are usually few: gather them in LDS once, so that the
  // two finer levels need no further pass over memory
  const uint32_t in_bin = s_hist[pa];
  __syncthreads();
  if (!src.lds && s_stash != nullptr && in_bin <= stash_cap) {
    if (tid == 0) s_out[0] = 0;
    __syncthreads();
    for_each_key<NT>(src, [&](uint32_t key) {
      if (key < base) return;
      if (((key - base) >> 13) == pa) s_stash[atomicAdd(&s_out[0], 1u)] = key;
    });
    __syncthreads();
    src.lds = s_stash;
    src.count = in_bin;
    __syncthreads();
  }
  for (uint32_t i = tid; i < 512; i += NT) s_hist[i] = 0;
  __syncthreads();
  for_each_key<NT>(src, [&](uint32_t key) {
    if (key < base) return;
    const uint32_t rel = key - base;
    if ((rel >> 13) == pa) atomicAdd(&s_hist[(rel >> 4) & 511u], 1u);
  });
  __syncthreads();
  const RankHit hb = find_rank_desc<NT>(s_hist, 512, want, s_w, s_out);
  want -= hb.above;
  const uint32_t pb = (pa << 9) | hb.bin;
  if (tid < 16) s_hist[tid] = 0;
  __syncthreads();
  for_each_key<NT>(src, [&](uint32_t key) {
    if (key < base) return;
    const uint32_t rel = key - base;
    if ((rel >> 4) == pb) atomicAdd(&s_hist[rel & 15u], 1u);
  });
  __syncthreads();
  const RankHit hc = find_rank_desc<NT>(s_hist, 16, want, s_w, s_out);
  *budget = want - hc.above;
  *ties = s_hist[hc.bin];
  return base + ((pb << 4) | hc.bin);
}

constexpr uint32_t kLdsKeys = 11264;    // boundary keys held in LDS (longer lists are read from memory)

// SECOND = false: first invocation, all workers (validates the speculation).
// SECOND = true : after the dense selection, flagged workers only.
template <bool SECOND, int NT>
__device__ __forceinline__ void select_worker(uint32_t n, WorkerCtl* ctl, GlobalCtl* gctl,
                                              const uint32_t* cand_key,
                                              const uint32_t* bnd_key, int64_t k,
                                              uint32_t cap_r, uint32_t cap_total, uint32_t regions,
                                              uint32_t bnd_cap, float cand_target, int force_dense,
                                              uint32_t* s_hist, uint32_t* s_keys, uint32_t* s_w,
                                              uint32_t* s_out) {
  const uint32_t tid = threadIdx.x;
  WorkerCtl& c = ctl[n];
  if (SECOND && !c.need_dense) return;
  const uint32_t K = (uint32_t)k;
  uint32_t n_tot = 0;
  if (!SECOND) {
    for (uint32_t r = 0; r < regions; ++r) n_tot += region_limit(c, r, cap_r);
    const bool need = force_dense || c.overflow || c.tau_lo == kNoBound || c.n_valid < K;
    if (tid == 0) {
      c.n_cand = n_tot;
      c.need_dense = need ? 1u : 0u;
      if (need) atomicOr(&gctl->any_dense, 1u);
    }
    if (need) return;
  } else {
    n_tot = c.dense_total;
    if (tid == 0) c.n_cand = n_tot;
  }
  const uint32_t win_lo = c.win_lo, win_hi = c.win_hi;
  const uint32_t n_hi = c.n_hi, n_bnd = c.n_bnd;
  const bool window = !SECOND && win_lo != kNoBound && n_bnd <= bnd_cap && n_hi < K && K <= n_hi + n_bnd;

  KeySource src;
  src.ctl = &c; src.cap_r = cap_r; src.n_regions = regions;
  src.lds = nullptr; src.flat = nullptr; src.regions = cand_key + (size_t)n * cap_total; src.count = n_tot;
  uint32_t base, rank;
  if (window) {
    // the k-th score lies inside the window: select among the boundary list only
    const uint32_t* list = bnd_key + (size_t)n * bnd_cap;
    src.count = n_bnd;
    if (s_keys != nullptr && n_bnd <= kLdsKeys) {
      for (uint32_t i = tid; i < n_bnd; i += NT) s_keys[i] = list[i];
      src.lds = s_keys;
    } else {
      src.flat = list;
    }
    base = win_lo;
    rank = K - n_hi;
  } else {
    // all candidates; only scores >= the bound can hold the k-th (at least k do)
    // (dense list: the 2k-th largest |a| when the list has 2k entries; a shorter
    // list is the whole row, whose scores may all be damped)
    base = SECOND ? (c.dense_total >= 2 * K ? c.f_tau : 0u) : c.tau_lo;
    rank = K;
  }
  __syncthreads();
  uint32_t budget, ties;
  // (the key buffer in LDS is free for the gathering unless it holds the boundary list)
  uint32_t* stash = (s_keys != nullptr && src.lds == nullptr) ? s_keys : nullptr;
  const uint32_t tau = rel_select<NT>(src, base, rank, s_hist, s_w, s_out, stash, kLdsKeys, &budget, &ties);

  if (tid == 0) {
    c.tau = tau;
    c.budget = budget;
    c.n_gt = K - budget;
    c.ties_total = ties;
    c.used_window = window ? 1u : 0u;
    // ---- bound and window of the next round
    // density of scores per bit pattern just below / around tau
    double dens;
    if (window) dens = (double)n_bnd / (double)(win_hi - win_lo);
    else dens = tau > base ? (double)(n_tot - K + 1) / (double)(tau - base) : 1.0;
    if (dens < 1e-7) dens = 1e-7;
    // After a failed speculation the history may say nothing about the next
    // round.  The bound was too high (fewer than k valid candidates): the k-th
    // score fell, which a drift never does - restart from this round's value.
    // The bound was too low (overflow): a shock if the k-th score is more than
    // twice what was expected; anything less can be the growth of the first
    // rounds (the accumulated gradient of an unsent entry doubles from round 0
    // to round 1, then grows by 3/2, 4/3, ...), an upward drift that was
    // underestimated and that the extrapolation below keeps following.
    bool shock = false;
    if (SECOND && c.tau_lo != kNoBound) {
      const uint32_t ref = c.centre != kNoBound ? c.centre : c.tau_prev;
      if (!c.overflow) shock = true;
      else if (ref != kNoBound && tau > ref && tau - ref > (1u << 23)) shock = true;
    }
    // the k-th score drifts from round to round: extrapolate linearly
    int64_t drift = 0;
    if (!shock && c.tau_prev != kNoBound) drift = (int64_t)tau - (int64_t)c.tau_prev;
    if (drift > (1 << 22)) drift = 1 << 22;
    if (drift < -(1 << 22)) drift = -(1 << 22);
    int64_t centre = (int64_t)tau + drift;
    if (centre < 0) centre = 0;
    if (centre > 0x7F000000) centre = 0x7F000000;
    // expected error of that prediction: how far this round's prediction was off
    // if it was an extrapolation (two earlier rounds known), else half the drift
    const uint32_t adrift = (uint32_t)(drift < 0 ? -drift : drift);
    uint32_t err;
    if (shock) err = kWinDefaultHalf;
    else if (c.centre != kNoBound && c.extrapolated) err = tau > c.centre ? tau - c.centre : c.centre - tau;
    else if (c.tau_prev != kNoBound) err = adrift / 2;
    else err = kWinDefaultHalf;
    if (!shock && (double)err < 0.7 * (double)c.err_prev) err = (uint32_t)(0.7 * (double)c.err_prev);
    double half = 3.0 * (double)err + 1024.0;
    const double by_count = 10000.0 / dens;                // at least about 20000 boundary entries
    if (half < by_count) half = by_count;
    const double cap_half = (double)bnd_cap / (4.0 * dens);
    if (half > cap_half) half = cap_half;
    if (half < (double)kWinMinHalf) half = (double)kWinMinHalf;
    if (half > (double)kWinMaxHalf) half = (double)kWinMaxHalf;
    const uint32_t h = (uint32_t)half;
    // bound: below the (cautiously) predicted k-th score by a margin that aims at
    // cand_target*k candidates and covers the prediction error.  An upward drift
    // is only followed half way (it usually slows down; too low a bound merely
    // costs candidates, too high a bound costs a dense selection).  After a
    // failed speculation the margin grows if the bound was too high (fewer than
    // k valid candidates) and shrinks if it was too low (overflow); it relaxes
    // back afterwards.
    float ms = c.margin_scale;
    if (!(ms > 0.0f)) ms = 1.0f;
    if (SECOND) {
      if (c.overflow) ms = ms * 0.5f < 0.125f ? 0.125f : ms * 0.5f;
      else if (c.tau_lo != kNoBound) ms = ms * 2.0f > 16.0f ? 16.0f : ms * 2.0f;
    } else {
      ms = ms > 1.0f ? 1.0f + (ms - 1.0f) * 0.7f : (ms * 1.3f > 1.0f ? 1.0f : ms * 1.3f);
    }
    c.margin_scale = ms;
    double margin = ((double)cand_target - 1.0) * (double)K / dens;
    if (margin < (double)err + 1024.0) margin = (double)err + 1024.0;
    margin *= (double)ms;
    if (margin > 16777216.0) margin = 16777216.0;
    const int64_t anchor = drift > 0 ? (int64_t)tau + drift / 2 : centre;
    int64_t lo = anchor - (int64_t)margin;
    if (shock && c.dense_total >= 2 * K) {
      // The dense selection's list is exactly the 2k entries of largest prior,
      // ending at f_tau.  Whether the new level persists (the k-th score stays
      // near tau) or the residuals of this round dominate the next one - after a
      // single spike, or when the gradients have collapsed - so that its k-th
      // score is this round's 2k-th, about f_tau: a bound half a list's spacing
      // below f_tau holds about 2.5k candidates, inside the buffer, and at
      // least k valid ones.
      const double below = 0.5 * (double)(tau > c.f_tau ? tau - c.f_tau : 0u) * (double)(ms > 1.0f ? ms : 1.0f);
      const int64_t lo2 = (int64_t)c.f_tau - (int64_t)(below < 16777216.0 ? below : 16777216.0) - 1024;
      if (lo2 < lo) lo = lo2;
    }
    const bool speculate = (int64_t)n_tot >= (int64_t)((double)cand_target * (double)K) || !SECOND;
    c.next_tau_lo = speculate ? (uint32_t)(lo > 0 ? lo : 0) : kNoBound;
    c.next_win_lo = speculate ? (uint32_t)(centre > (int64_t)h ? centre - (int64_t)h : 0) : kNoBound;
    c.next_win_hi = (uint32_t)centre + h;
    c.tau_prev = tau;
    c.centre = speculate ? (uint32_t)centre : kNoBound;
    c.err_prev = err;
    c.extrapolated = (speculate && drift != 0) ? 1u : 0u;
  }
}

// grid (N), 1024 threads: the first selection of a round, for all workers.
__global__ void __launch_bounds__(kScanBlock)
k_select(WorkerCtl* ctl, GlobalCtl* gctl, const uint32_t* __restrict__ cand_key,
         const uint32_t* __restrict__ bnd_key, int64_t k, uint32_t cap_r, uint32_t cap_total,
         uint32_t regions, uint32_t bnd_cap, float cand_target, int force_dense) {
  __shared__ uint32_t s_hist[kL1Bins];
  __shared__ uint32_t s_keys[kLdsKeys];
  __shared__ uint32_t s_w[16];
  __shared__ uint32_t s_out[2];
  select_worker<false, kScanBlock>(blockIdx.x, ctl, gctl, cand_key, bnd_key, k, cap_r, cap_total, regions,
                                   bnd_cap, cand_target, force_dense, s_hist, s_keys, s_w, s_out);
}

// -------------------------------------------------------------- sampling ----
// A round that starts without a bound from the previous one (round 0, after a
// reset or set_state) gets one from a strided sample of a = eps + g: the level-1
// histogram of the sample, from which k_sample_bound takes the bin edge above
// which about 1.6k entries of the whole row are expected.  The bound is only a
// guess - the selection verifies it like any other and falls back to the dense
// selection if it was wrong.
constexpr uint32_t kSampleMax = 1u << 18;     // sampled entries per worker (whole row if shorter)

// grid (blocks, N).  Sample i is the group of 4 entries at 4*i*stride4.
template <typename G>
__global__ void __launch_bounds__(kBlock)
k_sample_hist(const float* __restrict__ e, const G* __restrict__ g, const uint32_t* __restrict__ mask,
              int64_t d, uint32_t nc, uint32_t* __restrict__ shist, uint32_t n_groups, uint32_t stride4,
              int roots) {
  __shared__ uint32_t s_hist[kL1Bins];
  const uint32_t n = blockIdx.y, tid = threadIdx.x;
  for (uint32_t i = tid; i < kL1Bins; i += kBlock) s_hist[i] = 0;
  __syncthreads();
  const size_t row = (size_t)n * (size_t)d;
  const uint32_t* mrow = mask + (size_t)n * nc * kChunkWords;
  const bool vec = (d % 4 == 0) && (reinterpret_cast<uintptr_t>(g) % (4 * sizeof(G)) == 0);
  for (uint32_t i = blockIdx.x * kBlock + tid; i < n_groups; i += gridDim.x * kBlock) {
    const int64_t j0 = (int64_t)i * stride4 * 4;
    if (vec && j0 + 4 <= d) {                           // one 128-bit load of the state, one of the gradients
      const uint32_t mb = (mrow[j0 >> 5] >> (j0 & 31)) & 15u;
      f32x4 ev = *reinterpret_cast<const f32x4*>(e + row + j0);
      const f32x4 gv = grad4_at(g, row + j0);
      if (mb & 1u) ev.x = 0.f;
      if (mb & 2u) ev.y = 0.f;
      if (mb & 4u) ev.z = 0.f;
      if (mb & 8u) ev.w = 0.f;
      const f32x4 a4 = ev + gv;
      atomicAdd(&s_hist[prior_key(a4.x, roots) >> kL1Shift], 1u);
      atomicAdd(&s_hist[prior_key(a4.y, roots) >> kL1Shift], 1u);
      atomicAdd(&s_hist[prior_key(a4.z, roots) >> kL1Shift], 1u);
      atomicAdd(&s_hist[prior_key(a4.w, roots) >> kL1Shift], 1u);
      continue;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t j = j0 + q;
      if (j < d) {
        const uint32_t sent = (mrow[j >> 5] >> (j & 31)) & 1u;
        const float a = (sent ? 0.0f : e[row + j]) + grad_at(g, row + j);
        atomicAdd(&s_hist[prior_key(a, roots) >> kL1Shift], 1u);
      }
    }
  }
  __syncthreads();
  uint32_t* gh = shist + (size_t)n * 3 * kL1Bins;
  for (uint32_t i = tid; i < kL1Bins; i += kBlock) {
    const uint32_t v = s_hist[i];
    if (v) atomicAdd(&gh[i], v);
  }
}

// grid (N), 1024 threads.  Sets this round's bound from the sample histogram.
__global__ void __launch_bounds__(kScanBlock)
k_sample_bound(WorkerCtl* ctl, const uint32_t* __restrict__ shist, int64_t d, int64_t k,
               uint32_t n_sampled, int roots) {
  __shared__ uint32_t s_hist[kL1Bins];
  __shared__ uint32_t s_w[16];
  __shared__ uint32_t s_out[2];
  const uint32_t n = blockIdx.x, tid = threadIdx.x;
  const uint32_t* gh = shist + (size_t)n * 3 * kL1Bins;
  for (uint32_t i = tid; i < kL1Bins; i += kScanBlock) s_hist[i] = gh[i];
  __syncthreads();
  // sample rank that corresponds to about 1.6k entries of the row, plus four
  // standard deviations of the sampling noise
  const double frac = (double)n_sampled / (double)d;
  double want = 1.6 * (double)k * frac;
  want += 4.0 * sqrt(want) + 1.0;
  const RankHit h = want < (double)n_sampled ? find_rank_desc<kScanBlock>(s_hist, kL1Bins, (uint32_t)want, s_w, s_out)
                                            : RankHit{kNoBound, 0u};
  if (tid == 0 && h.bin != kNoBound && h.bin > 0) {
    ctl[n].tau_lo = h.bin << kL1Shift;
    ctl[n].tau_lo_mag = magnitude_bound(h.bin << kL1Shift, roots);
    ctl[n].win_lo = kNoBound;
  }
}

// ---------------------------------------------------------- k_chunk_scan ----
// One block of NT threads per worker.  Exclusive scans over the chunks of one worker:
//   tie_off[c] = ties before chunk c;
//   sel[c]     = gt[c] + clamp(budget - tie_off[c], 0, tie[c])   (lowest-index ties first);
//   sel_off[c] = selected entries before chunk c  (nc+1 values).
// DENSE: budget = f_budget, sel_off/sel go to ch_off/ch_cnt (placement of the
// dense emission) and dense_total.  Otherwise budget = ctl.budget, sel_off goes
// to the round's sel_off table and the total is checked against k.  tie_off is
// written in both cases.
// (No __restrict__ here and in select_worker: inside k_dense_all these arrays
// are written by other blocks in the phase before.)
template <bool DENSE, int NT>
__device__ __forceinline__ void chunk_scan_worker(uint32_t n, WorkerCtl* ctl, const uint32_t* ch_gt,
                                                  const uint32_t* ch_tie, uint32_t* out_off,
                                                  uint32_t* out_cnt, uint32_t* out_tieoff, uint32_t nc,
                                                  int64_t k, uint32_t* s_w /*[>= 2 * NT / 64]*/) {
  constexpr uint32_t W = NT / 64;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  WorkerCtl& c = ctl[n];
  const uint32_t budget = DENSE ? c.f_budget : c.budget;
  const uint32_t* gt = ch_gt + (size_t)n * nc;
  const uint32_t* tie = ch_tie + (size_t)n * nc;
  uint32_t* off = out_off + (size_t)n * (DENSE ? nc : nc + 1);
  uint32_t* cnt = DENSE ? out_cnt + (size_t)n * nc : nullptr;
  uint32_t* tof = out_tieoff + (size_t)n * nc;
  // The ties taken before chunk c number min(budget, ties before c), so the two
  // running sums of gt and tie give everything.  Every wave owns a contiguous
  // run of 64-chunk tiles (coalesced loads): first its totals, then, after the
  // waves' totals are placed, the running sums and the outputs.
  const uint32_t tiles = (nc + 63) / 64;
  const uint32_t per = (tiles + W - 1) / W;
  const uint32_t t0 = wv * per < tiles ? wv * per : tiles;
  const uint32_t t1 = t0 + per < tiles ? t0 + per : tiles;
  uint32_t gsum = 0, tsum = 0;
#pragma unroll 8
  for (uint32_t t = t0; t < t1; ++t) {
    const uint32_t ci = t * 64 + lane;
    if (ci < nc) { gsum += gt[ci]; tsum += tie[ci]; }
  }
  for (int o = 32; o > 0; o >>= 1) { gsum += __shfl_down(gsum, o); tsum += __shfl_down(tsum, o); }
  if (lane == 0) { s_w[wv] = gsum; s_w[W + wv] = tsum; }
  __syncthreads();
  uint32_t grun = 0, trun = 0, gtot = 0, ttot = 0;
  for (uint32_t i = 0; i < W; ++i) {
    const uint32_t g = s_w[i], t = s_w[W + i];
    if (i < wv) { grun += g; trun += t; }
    gtot += g; ttot += t;
  }
  __syncthreads();
#pragma unroll 4
  for (uint32_t t = t0; t < t1; ++t) {
    const uint32_t ci = t * 64 + lane;
    const uint32_t g = ci < nc ? gt[ci] : 0u, ti = ci < nc ? tie[ci] : 0u;
    uint32_t gx = g, tx = ti;                            // inclusive running sums inside the tile
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t gy = __shfl_up(gx, o), ty = __shfl_up(tx, o);
      if (lane >= (uint32_t)o) { gx += gy; tx += ty; }
    }
    const uint32_t g_before = grun + gx - g, t_before = trun + tx - ti;
    if (ci < nc) {
      const uint32_t taken_before = t_before < budget ? t_before : budget;
      uint32_t take = 0;
      if (t_before < budget) { take = budget - t_before; if (take > ti) take = ti; }
      off[ci] = g_before + taken_before;
      tof[ci] = t_before;
      if (DENSE) cnt[ci] = g + take;
    }
    grun += __shfl(gx, 63);
    trun += __shfl(tx, 63);
  }
  if (tid == 0) {
    const uint32_t sel_run = gtot + (ttot < budget ? ttot : budget);
    if (DENSE) c.dense_total = sel_run;
    else {
      off[nc] = sel_run;
      if ((int64_t)sel_run != k) c.err |= 1u;
    }
  }
}


// grid (N), 1024 threads: the scan of the final compaction.
__global__ void __launch_bounds__(kScanBlock)
k_chunk_scan(WorkerCtl* ctl, const uint32_t* __restrict__ ch_gt, const uint32_t* __restrict__ ch_tie,
             uint32_t* __restrict__ sel_off, uint32_t* __restrict__ tie_off, uint32_t nc, int64_t k) {
  __shared__ uint32_t s_w[2 * kScanBlock / 64];
  chunk_scan_worker<false, kScanBlock>(blockIdx.x, ctl, ch_gt, ch_tie, sel_off, nullptr, tie_off, nc, k, s_w);
}

// ------------------------------------------------------------ dense path ----
// The dense selection of the workers whose speculation failed (and of every
// worker in round 0) runs as ONE kernel, k_dense_all, whose phases are
// separated by grid barriers: when no worker is flagged - the usual case - the
// whole path costs a single launch that returns at once.  The grid is sized by
// the host so that all blocks are resident together.
//
// Phases, for flagged workers only:
//   clear histograms | 3 x (histogram of |a| bits, pick the bin of rank
//   min(2k,d)) | per-chunk counts | chunk scan | ordered emission of the 2k
//   largest |a| as the candidate list | scores | exact k-th score.

// Histogram level LEVEL of worker n's row; block b of G covers a strided share.
template <int LEVEL, bool VEC>
__device__ __forceinline__ void dense_hist_worker(uint32_t n, uint32_t b, uint32_t G, const float* a,
                                                  int64_t d, const WorkerCtl* ctl, uint32_t* fhist,
                                                  uint32_t* s_hist, int roots) {
  const uint32_t tid = threadIdx.x;
  constexpr uint32_t bins = LEVEL == 1 ? kL1Bins : (LEVEL == 2 ? kL2Bins : kL3Bins);
  for (uint32_t i = tid; i < bins; i += kBlock) s_hist[i] = 0;
  __syncthreads();
  const uint32_t prefix = ctl[n].f_prefix;
  const float* row = a + (size_t)n * (size_t)d;
  auto put = [&](float v) {
    const uint32_t key = prior_key(v, roots);
    if (LEVEL == 1) atomicAdd(&s_hist[key >> kL1Shift], 1u);
    else if (LEVEL == 2) { if ((key >> kL1Shift) == prefix) atomicAdd(&s_hist[(key >> kL2Shift) & (kL2Bins - 1)], 1u); }
    else { if ((key >> kL2Shift) == prefix) atomicAdd(&s_hist[key & (kL3Bins - 1)], 1u); }
  };
  if (VEC) {
    const float4* row4 = reinterpret_cast<const float4*>(row);
    const int64_t d4 = d / 4;
    // four loads in flight per thread: the few resident blocks must cover the memory latency themselves
    const int64_t step = (int64_t)G * kBlock;
    int64_t j = (int64_t)b * kBlock + tid;
    for (; j + 3 * step < d4; j += 4 * step) {
      const float4 v0 = row4[j], v1 = row4[j + step], v2 = row4[j + 2 * step], v3 = row4[j + 3 * step];
      put(v0.x); put(v0.y); put(v0.z); put(v0.w);
      put(v1.x); put(v1.y); put(v1.z); put(v1.w);
      put(v2.x); put(v2.y); put(v2.z); put(v2.w);
      put(v3.x); put(v3.y); put(v3.z); put(v3.w);
    }
    for (; j < d4; j += step) {
      const float4 v = row4[j];
      put(v.x); put(v.y); put(v.z); put(v.w);
    }
  } else {
    for (int64_t j = (int64_t)b * kBlock + tid; j < d; j += (int64_t)G * kBlock) put(row[j]);
  }
  __syncthreads();
  uint32_t* gh = fhist + ((size_t)n * 3 + (LEVEL - 1)) * kL1Bins;
  for (uint32_t i = tid; i < bins; i += kBlock) {
    const uint32_t v = s_hist[i];
    if (v) atomicAdd(&gh[i], v);
  }
  __syncthreads();
}

// Level LEVEL of the radix select of rank min(2k, d) over the |a| bits of worker
// n: finds, from the top bin downwards, the bin in which the cumulative count
// reaches the wanted rank.  One block.
template <int LEVEL>
__device__ __forceinline__ void dense_scan_worker(uint32_t n, WorkerCtl* ctl, const uint32_t* hist_all,
                                                  int64_t k, int64_t d, uint32_t* s_sum,
                                                  uint32_t* s_scan) {
  constexpr uint32_t bins = LEVEL == 1 ? kL1Bins : (LEVEL == 2 ? kL2Bins : kL3Bins);
  constexpr uint32_t per = bins / kBlock;            // bins per thread (16, 8, 1)
  const uint32_t tid = threadIdx.x;
  WorkerCtl& c = ctl[n];
  const uint32_t* h = hist_all + ((size_t)n * 3 + (LEVEL - 1)) * kL1Bins;
  uint32_t want;
  if (LEVEL == 1) want = (uint32_t)(2 * k < d ? 2 * k : d);
  else want = c.f_krem;
  // thread t owns bins [bins-1-t*per .. bins-(t+1)*per], i.e. descending order
  uint32_t loc[per];
  uint32_t s = 0;
#pragma unroll
  for (uint32_t q = 0; q < per; ++q) { loc[q] = h[bins - 1 - (tid * per + q)]; s += loc[q]; }
  s_sum[tid] = s;
  __syncthreads();
  if (tid == 0) {
    uint32_t run = 0;
    for (uint32_t i = 0; i < kBlock; ++i) { s_scan[i] = run; run += s_sum[i]; }
  }
  __syncthreads();
  const uint32_t above = s_scan[tid];               // count in bins above this thread's
  if (above < want && want <= above + s) {
    uint32_t run = above;
#pragma unroll
    for (uint32_t q = 0; q < per; ++q) {
      if (run < want && want <= run + loc[q]) {
        const uint32_t bin = bins - 1 - (tid * per + q);
        const uint32_t krem = want - run;            // rank wanted inside this bin
        if (LEVEL == 1) { c.f_prefix = bin; c.f_krem = krem; }
        else if (LEVEL == 2) { c.f_prefix = (c.f_prefix << 11) | bin; c.f_krem = krem; }
        else { c.f_tau = (c.f_prefix << 8) | bin; c.f_budget = krem; }
      }
      run += loc[q];
    }
  }
  __syncthreads();
}

// Chunk c of worker n: entries with |a| bits > f_tau and == f_tau.
template <bool VEC>
__device__ __forceinline__ void dense_count_chunk(uint32_t n, uint32_t c, const float* a, int64_t d,
                                                  const WorkerCtl* ctl, uint32_t* ch_gt,
                                                  uint32_t* ch_tie, uint32_t nc, uint32_t* s_gt,
                                                  uint32_t* s_tie, int roots) {
  const uint32_t tid = threadIdx.x;
  const uint32_t tau = ctl[n].f_tau;
  const float* row = a + (size_t)n * (size_t)d;
  uint32_t gt = 0, tie = 0;
  if (VEC) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t j = (int64_t)c * kChunk + (i * kBlock + tid) * 4;
      if (j < d) {
        const float4 v = *reinterpret_cast<const float4*>(row + j);
        const uint32_t k0 = prior_key(v.x, roots), k1 = prior_key(v.y, roots), k2 = prior_key(v.z, roots),
                       k3 = prior_key(v.w, roots);
        gt += (k0 > tau) + (k1 > tau) + (k2 > tau) + (k3 > tau);
        tie += (k0 == tau) + (k1 == tau) + (k2 == tau) + (k3 == tau);
      }
    }
  } else {
    for (int i = 0; i < 16; ++i) {
      const int64_t j = (int64_t)c * kChunk + i * kBlock + tid;
      if (j < d) {
        const uint32_t key = prior_key(row[j], roots);
        gt += key > tau;
        tie += key == tau;
      }
    }
  }
  for (int o = 32; o > 0; o >>= 1) { gt += __shfl_down(gt, o); tie += __shfl_down(tie, o); }
  if ((tid & 63) == 0) { s_gt[tid >> 6] = gt; s_tie[tid >> 6] = tie; }
  __syncthreads();
  if (tid == 0) {
    ch_gt[(size_t)n * nc + c] = s_gt[0] + s_gt[1] + s_gt[2] + s_gt[3];
    ch_tie[(size_t)n * nc + c] = s_tie[0] + s_tie[1] + s_tie[2] + s_tie[3];
  }
  __syncthreads();
}

// Chunk c of worker n: writes its share of the 2k largest |a| (ties: lowest
// indices) to the candidate list, in index order, at the offsets of the scan.
// The sweep has overwritten the state by now, so the value sent in the previous
// round is fetched from that round's list: its position there is the number of
// mask bits before the entry (prev_sel_off[c] of them in lower chunks; s_mw /
// s_rk, 128 words each, hold the chunk's mask words and their running counts).
template <bool VEC>
__device__ __forceinline__ void dense_emit_chunk(uint32_t n, uint32_t c, const float* a_rows,
                                                 const uint32_t* mask, int64_t d, const WorkerCtl* ctl,
                                                 int32_t* cand_idx, float* cand_val, float* cand_prev,
                                                 const uint32_t* ch_off, const uint32_t* ch_cnt,
                                                 const uint32_t* tie_off, const uint32_t* prev_sel_off,
                                                 const float* prev_val, int64_t k, uint32_t nc,
                                                 uint32_t cap_total, uint32_t* s_wtot, uint32_t* s_ttot,
                                                 uint32_t* s_mw, uint32_t* s_rk, int roots) {
  const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const uint32_t* mrow = mask + (size_t)n * nc * kChunkWords;
  const size_t tix = (size_t)n * nc + c;
  if (ch_cnt[tix] == 0) return;
  if (tid < kChunkWords) s_mw[tid] = mrow[(size_t)c * kChunkWords + tid];
  __syncthreads();
  if (tid < 64) {                                    // wave 0: running count of mask bits, two words per lane
    const uint32_t c0 = (uint32_t)__popc(s_mw[2 * tid]), c1 = (uint32_t)__popc(s_mw[2 * tid + 1]);
    uint32_t x = c0 + c1;
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t y = __shfl_up(x, o);
      if (tid >= (uint32_t)o) x += y;
    }
    const uint32_t before = prev_sel_off[(size_t)n * (nc + 1) + c] + x - (c0 + c1);
    s_rk[2 * tid] = before;
    s_rk[2 * tid + 1] = before + c0;
  }
  __syncthreads();
  const float* pv = prev_val + (size_t)n * k;
  const uint32_t tau = ctl[n].f_tau, budget = ctl[n].f_budget;
  const size_t row = (size_t)n * (size_t)d;
  const int64_t base = (int64_t)c * kChunk + (int64_t)wv * 1024 + lane * 4;
  float a[4][4];
  uint32_t gtf = 0, tief = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t j0 = base + i * 256;
    if (VEC) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j0 < d) v = *reinterpret_cast<const float4*>(a_rows + row + j0);
      a[i][0] = v.x; a[i][1] = v.y; a[i][2] = v.z; a[i][3] = v.w;
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) a[i][q] = (j0 + q < d) ? a_rows[row + j0 + q] : 0.f;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (j0 + q < d) {
        const uint32_t key = prior_key(a[i][q], roots);
        if (key > tau) gtf |= 1u << (i * 4 + q);
        else if (key == tau) tief |= 1u << (i * 4 + q);
      }
    }
  }
  // rank of every tie within the chunk (index order) decides which ties are taken
  const uint32_t tie_before = tie_off[tix];          // ties in lower chunks
  ChunkPos tp = ordered_positions(tief, s_ttot);
  uint32_t flags = gtf;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t p = tie_before + tp.wave_base + tp.lane_base[i];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if ((tief >> (i * 4 + q)) & 1u) {
        if (p < budget) flags |= 1u << (i * 4 + q);
        ++p;
      }
    }
  }
  __syncthreads();
  const ChunkPos cp = ordered_positions(flags, s_wtot);
  const size_t out = (size_t)n * cap_total + ch_off[tix] + cp.wave_base;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t p = cp.lane_base[i];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if ((flags >> (i * 4 + q)) & 1u) {
        const int64_t j = base + i * 256 + q;
        const uint32_t wl = (uint32_t)(j >> 5) & (kChunkWords - 1), bit = (uint32_t)j & 31u;
        const uint32_t sent = (s_mw[wl] >> bit) & 1u;
        float ab = 0.0f;
        if (sent) {
          const uint32_t rank = s_rk[wl] + (uint32_t)__popc(s_mw[wl] & ((1u << bit) - 1u));
          if ((int64_t)rank < k) ab = pv[rank];
        }
        cand_idx[out + p] = (int32_t)((uint32_t)j | (sent ? kSentFlag : 0u));
        cand_val[out + p] = a[i][q];
        cand_prev[out + p] = ab;
        ++p;
      }
    }
  }
  __syncthreads();
}

// The r-th flagged worker (ascending), found by the whole block: thread t
// counts the flags of a contiguous range of workers, a block scan places the
// ranges, the thread whose range holds rank r walks it.  Returns N if r is past
// the last flagged worker; *n_flagged gets their number.  s_w [16], s_out [2].
__device__ __forceinline__ uint32_t flagged_worker(const WorkerCtl* ctl, int32_t N, uint32_t r,
                                                   uint32_t* n_flagged, uint32_t* s_w, uint32_t* s_out) {
  const uint32_t tid = threadIdx.x;
  const uint32_t per = ((uint32_t)N + kBlock - 1) / kBlock;
  const uint32_t n0 = tid * per < (uint32_t)N ? tid * per : (uint32_t)N;
  const uint32_t n1 = n0 + per < (uint32_t)N ? n0 + per : (uint32_t)N;
  uint32_t mine = 0;
  for (uint32_t n = n0; n < n1; ++n) mine += ctl[n].need_dense != 0;
  if (tid == 0) s_out[0] = (uint32_t)N;
  uint32_t total;
  const uint32_t before = block_excl_scan<kBlock>(mine, s_w, &total);
  if (r >= before && r < before + mine) {
    uint32_t seen = before;
    for (uint32_t n = n0; n < n1; ++n) {
      if (ctl[n].need_dense != 0) {
        if (seen == r) { s_out[0] = n; break; }
        ++seen;
      }
    }
  }
  __syncthreads();
  const uint32_t hit = s_out[0];
  __syncthreads();
  *n_flagged = total;
  return hit;
}

// grid (G): G blocks resident together.  See the section header.
template <bool VEC>
__global__ void __launch_bounds__(kBlock)
k_dense_all(const float* a_rows, const uint32_t* mask, const uint32_t* prev_sel_off, int64_t d, WorkerCtl* ctl,
            GlobalCtl* gctl, uint32_t* fhist, uint32_t* ch_gt, uint32_t* ch_tie, uint32_t* ch_off,
            uint32_t* ch_cnt, uint32_t* tie_off, int32_t* cand_idx, float* cand_val, float* cand_prev,
            uint32_t* cand_key,
            const uint32_t* bnd_key, const float* prev_val, const float* gprev, int64_t k, uint32_t nc,
            int32_t N, uint32_t cap_r, uint32_t cap_total, uint32_t regions, uint32_t bnd_cap,
            const float* omega, float mu, int use_reg, float cand_target, ScoreKind sk) {
  if (gctl->any_dense == 0) return;
  const int roots = sk.roots;
  __shared__ uint32_t s_hist[kL1Bins];
  __shared__ uint32_t s_a[kBlock], s_b[kBlock];
  __shared__ uint32_t s_w[16], s_out[2], s_x[4], s_y[4];
  const uint32_t b = blockIdx.x, G = gridDim.x, tid = threadIdx.x;

  for (int32_t n = 0; n < N; ++n) {
    if (!ctl[n].need_dense) continue;
    uint32_t* fh = fhist + (size_t)n * 3 * kL1Bins;
    for (uint32_t i = b * kBlock + tid; i < 3 * kL1Bins; i += G * kBlock) fh[i] = 0;
  }
  grid_barrier(gctl, G);

  // The histogram passes give every flagged worker its own group of blocks (all
  // workers at once, each histogram fed by G / n_flagged blocks), so that the
  // blocks' final adds do not all queue on the same few words.
  uint32_t n_flagged;
  (void)flagged_worker(ctl, N, 0xFFFFFFFFu, &n_flagged, s_w, s_out);
  if (n_flagged == 0) return;                                   // every block sees the same flags
  const uint32_t groups = n_flagged < G ? n_flagged : G;
  const uint32_t grp = b % groups, sub = b / groups;
  const uint32_t sub_cnt = (G - grp + groups - 1) / groups;     // blocks of this group
  const uint32_t first_worker = flagged_worker(ctl, N, grp, &n_flagged, s_w, s_out);
  for (uint32_t r = grp; r < n_flagged; r += groups) {
    const uint32_t n = r == grp ? first_worker : flagged_worker(ctl, N, r, &n_flagged, s_w, s_out);
    if (n < (uint32_t)N) dense_hist_worker<1, VEC>(n, sub, sub_cnt, a_rows, d, ctl, fhist, s_hist, roots);
  }
  grid_barrier(gctl, G);
  for (int32_t n = b; n < N; n += G)
    if (ctl[n].need_dense) dense_scan_worker<1>(n, ctl, fhist, k, d, s_a, s_b);
  grid_barrier(gctl, G);
  for (uint32_t r = grp; r < n_flagged; r += groups) {
    const uint32_t n = r == grp ? first_worker : flagged_worker(ctl, N, r, &n_flagged, s_w, s_out);
    if (n < (uint32_t)N) dense_hist_worker<2, VEC>(n, sub, sub_cnt, a_rows, d, ctl, fhist, s_hist, roots);
  }
  grid_barrier(gctl, G);
  for (int32_t n = b; n < N; n += G)
    if (ctl[n].need_dense) dense_scan_worker<2>(n, ctl, fhist, k, d, s_a, s_b);
  grid_barrier(gctl, G);
  for (uint32_t r = grp; r < n_flagged; r += groups) {
    const uint32_t n = r == grp ? first_worker : flagged_worker(ctl, N, r, &n_flagged, s_w, s_out);
    if (n < (uint32_t)N) dense_hist_worker<3, VEC>(n, sub, sub_cnt, a_rows, d, ctl, fhist, s_hist, roots);
  }
  grid_barrier(gctl, G);
  for (int32_t n = b; n < N; n += G)
    if (ctl[n].need_dense) dense_scan_worker<3>(n, ctl, fhist, k, d, s_a, s_b);
  grid_barrier(gctl, G);

  for (int32_t n = 0; n < N; ++n) {
    if (!ctl[n].need_dense) continue;
    for (uint32_t c = b; c < nc; c += G) dense_count_chunk<VEC>(n, c, a_rows, d, ctl, ch_gt, ch_tie, nc, s_x, s_y, roots);
  }
  grid_barrier(gctl, G);
  for (int32_t n = b; n < N; n += G)
    if (ctl[n].need_dense) chunk_scan_worker<true, kBlock>(n, ctl, ch_gt, ch_tie, ch_off, ch_cnt, tie_off, nc, k, s_w);
  grid_barrier(gctl, G);
  for (int32_t n = 0; n < N; ++n) {
    if (!ctl[n].need_dense) continue;
    for (uint32_t c = b; c < nc; c += G)
      dense_emit_chunk<VEC>(n, c, a_rows, mask, d, ctl, cand_idx, cand_val, cand_prev, ch_off, ch_cnt, tie_off,
                            prev_sel_off, prev_val, k, nc, cap_total, s_x, s_y, s_a, s_b, roots);
  }
  grid_barrier(gctl, G);

  for (int32_t n = 0; n < N; ++n) {
    if (!ctl[n].need_dense) continue;
    const uint32_t total = ctl[n].dense_total;
    const size_t cb = (size_t)n * cap_total;
    const float w = omega[n];
    for (uint32_t p = b * kBlock + tid; p < total; p += G * kBlock)
      cand_key[cb + p] = score_entry((uint32_t)cand_idx[cb + p], cand_val[cb + p], cand_prev[cb + p], use_reg, gprev, w, mu, sk);
  }
  grid_barrier(gctl, G);
  for (int32_t n = b; n < N; n += G)
    if (ctl[n].need_dense)
      select_worker<true, kBlock>(n, ctl, gctl, cand_key, bnd_key, k, cap_r, cap_total, regions, bnd_cap,
                                  cand_target, 0, s_hist, nullptr, s_w, s_out);
}

// --------------------------------------------------------- k_chunk_count ----
// grid (ceil(nc/4), N): one wave per chunk.  Candidates of the chunk with
// score > tau and == tau.  Most chunks are empty and a few hold hundreds of
// candidates, so a lane takes eight at a time with all loads in flight together.
constexpr int kLaneBatch = 8;
__global__ void __launch_bounds__(kBlock)
k_chunk_count(const WorkerCtl* __restrict__ ctl, const uint32_t* __restrict__ cand_key,
              const uint32_t* __restrict__ ch_off, const uint32_t* __restrict__ ch_cnt,
              uint32_t* __restrict__ ch_gt, uint32_t* __restrict__ ch_tie, uint32_t nc,
              uint32_t cap_total) {
  const uint32_t n = blockIdx.y, lane = threadIdx.x & 63;
  const uint32_t c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= nc) return;
  const size_t tix = (size_t)n * nc + c;
  const uint32_t tau = ctl[n].tau;
  const uint32_t off = ch_off[tix], cnt = ch_cnt[tix];
  const uint32_t* key = cand_key + (size_t)n * cap_total + off;
  uint32_t gt = 0, tie = 0;
  for (uint32_t p0 = 0; p0 < cnt; p0 += 64 * kLaneBatch) {
    uint32_t kk[kLaneBatch];
#pragma unroll
    for (int q = 0; q < kLaneBatch; ++q) {
      const uint32_t p = p0 + q * 64 + lane;
      kk[q] = p < cnt ? key[p] : 0u;
    }
#pragma unroll
    for (int q = 0; q < kLaneBatch; ++q) {
      const bool in = p0 + q * 64 + lane < cnt;
      gt += in && kk[q] > tau;
      tie += in && kk[q] == tau;
    }
  }
  for (int o = 32; o > 0; o >>= 1) { gt += __shfl_down(gt, o); tie += __shfl_down(tie, o); }
  if (lane == 0) { ch_gt[tix] = gt; ch_tie[tix] = tie; }
}

// ------------------------------------------------------------- k_compact ----
// grid (ceil(nc/4), N): one wave per chunk.  Writes the selected pairs of the
// chunk in index order at sel_off[c], and the chunk's words of the round's mask
// (bit = entry selected).
__global__ void __launch_bounds__(kBlock)
k_compact(const WorkerCtl* __restrict__ ctl, const uint32_t* __restrict__ cand_key,
          const int32_t* __restrict__ cand_idx, const float* __restrict__ cand_val,
          const uint32_t* __restrict__ ch_off, const uint32_t* __restrict__ ch_cnt,
          const uint32_t* __restrict__ sel_off, const uint32_t* __restrict__ prev_sel_off,
          const uint32_t* __restrict__ tie_off, int32_t* __restrict__ out_idx,
          float* __restrict__ out_val, uint32_t* __restrict__ mask,
          int64_t k, uint32_t nc, uint32_t cap_total) {
  __shared__ uint32_t s_m[4][kChunkWords];
  const uint32_t n = blockIdx.y, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint32_t c = blockIdx.x * 4 + wv;
  const bool live = c < nc;
  s_m[wv][lane] = 0;
  s_m[wv][lane + 64] = 0;
  __syncthreads();
  uint32_t first = 0;
  bool was_empty = true, is_empty = true;
  if (live) {
    const size_t tix = (size_t)n * nc + c;
    const size_t so = (size_t)n * (nc + 1) + c;
    const uint32_t cnt = ch_cnt[tix];
    const uint32_t off = ch_off[tix];
    const uint32_t tau = ctl[n].tau, budget = ctl[n].budget;
    const size_t cb = (size_t)n * cap_total + off;
    first = sel_off[so];
    was_empty = prev_sel_off[so + 1] == prev_sel_off[so];
    is_empty = sel_off[so + 1] == first;
    uint32_t out = first;
    uint32_t tie_run = tie_off[tix];
    for (uint32_t p0 = 0; p0 < cnt; p0 += 64 * kLaneBatch) {
      // keys, indices and values of eight candidates per lane, all loads in flight together
      uint32_t kk[kLaneBatch], jj[kLaneBatch];
      float vv[kLaneBatch];
#pragma unroll
      for (int q = 0; q < kLaneBatch; ++q) {
        const uint32_t p = p0 + q * 64 + lane;
        const bool in = p < cnt;
        kk[q] = in ? cand_key[cb + p] : 0u;
        jj[q] = in ? (uint32_t)cand_idx[cb + p] & ~kSentFlag : 0u;
        vv[q] = in ? cand_val[cb + p] : 0.0f;
      }
#pragma unroll
      for (int q = 0; q < kLaneBatch; ++q) {
        if (p0 + q * 64 >= cnt) break;                       // uniform over the wave
        const bool in = p0 + q * 64 + lane < cnt;
        const bool is_tie = in && kk[q] == tau;
        const uint64_t tb = __ballot(is_tie);
        const bool take = in && (kk[q] > tau || (is_tie && tie_run + lanes_below(tb) < budget));
        const uint64_t sb = __ballot(take);
        if (take) {
          const uint32_t o = out + lanes_below(sb);
          if ((int64_t)o < k) {
            out_idx[(size_t)n * k + o] = (int32_t)jj[q];
            out_val[(size_t)n * k + o] = vv[q];
            const uint32_t jl = jj[q] & (kChunk - 1);
            atomicOr(&s_m[wv][jl >> 5], 1u << (jl & 31));
          }
        }
        tie_run += (uint32_t)__popcll(tb);
        out += (uint32_t)__popcll(sb);
      }
    }
  }
  __syncthreads();
  if (live) {
    // a chunk without selected entries in the previous round has all-zero mask
    // words already: nothing to write if it has none now either
    if (!(was_empty && is_empty)) {
      const size_t wbase = ((size_t)n * nc + c) * kChunkWords;
      reinterpret_cast<uint2*>(mask + wbase)[lane] = make_uint2(s_m[wv][2 * lane], s_m[wv][2 * lane + 1]);
    }
  }
}

// ----------------------------------------------------------- k_aggregate ----
// grid (nc).  agg tile of 4096 entries: +0, then + omega_n*val of every worker in
// ascending worker order (indices of one worker are distinct, so plain LDS
// read-modify-write), written once (tiles that are zero and already hold zeros
// are left alone).  Workers are taken 32 at a time: the
// chunk's selected entries of all 32 are first staged in LDS with independent
// loads (so memory latency is paid once per batch), then applied to the tile
// one worker after the other.
constexpr uint32_t kAggStage = 1024;

__global__ void __launch_bounds__(kBlock)
k_aggregate(const int32_t* __restrict__ out_idx, const float* __restrict__ out_val,
            const uint32_t* __restrict__ sel_off, float* __restrict__ agg,
            uint32_t* __restrict__ agg_hot, int64_t d, int64_t k, uint32_t nc, int32_t N,
            const float* __restrict__ omega) {
  __shared__ float s_tile[kChunk];
  __shared__ uint32_t s_j[kAggStage];
  __shared__ float s_v[kAggStage];
  __shared__ uint32_t s_s0[32], s_pre[33];
  __shared__ float s_w[32];
  const uint32_t c = blockIdx.x, tid = threadIdx.x;
  for (uint32_t i = tid; i < kChunk; i += kBlock) s_tile[i] = 0.0f;
  const int32_t jbase = (int32_t)(c << kChunkLog);
  uint32_t any_entries = 0;
  for (int32_t b0 = 0; b0 < N; b0 += 32) {
    const int32_t nb = N - b0 < 32 ? N - b0 : 32;
    __syncthreads();                                  // previous batch applied, s_* free
    if ((int32_t)tid < nb) {
      const size_t o = (size_t)(b0 + tid) * (nc + 1) + c;
      const uint32_t a0 = sel_off[o];
      s_s0[tid] = a0;
      s_w[tid] = omega[b0 + tid];
      s_pre[tid + 1] = sel_off[o + 1] - a0;            // length, turned into a prefix below
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t run = 0;
      s_pre[0] = 0;
      for (int32_t i = 0; i < nb; ++i) { run += s_pre[i + 1]; s_pre[i + 1] = run; }
    }
    __syncthreads();
    const uint32_t total = s_pre[nb];
    any_entries |= total;
    for (uint32_t q0 = 0; q0 < total; q0 += kAggStage) {   // usually one pass
      const uint32_t q1 = q0 + kAggStage < total ? q0 + kAggStage : total;
      for (uint32_t q = q0 + tid; q < q1; q += kBlock) {
        int32_t i = 0;
        while (s_pre[i + 1] <= q) ++i;                 // worker of flattened entry q
        const size_t src = (size_t)(b0 + i) * k + s_s0[i] + (q - s_pre[i]);
        s_j[q - q0] = (uint32_t)(out_idx[src] - jbase);
        s_v[q - q0] = out_val[src];
      }
      __syncthreads();
      for (int32_t i = 0; i < nb; ++i) {               // ascending worker order
        const uint32_t lo = s_pre[i] > q0 ? s_pre[i] : q0;
        const uint32_t hi = s_pre[i + 1] < q1 ? s_pre[i + 1] : q1;
        if (lo < hi) {                                 // uniform over the block
          const float w = s_w[i];
          for (uint32_t q = lo + tid; q < hi; q += kBlock) {
            const uint32_t j = s_j[q - q0];
            if (j < (uint32_t)kChunk) s_tile[j] = __fadd_rn(s_tile[j], __fmul_rn(w, s_v[q - q0]));
          }
          __syncthreads();
        }
      }
    }
  }
  __syncthreads();
  // agg_hot[c] tells whether this tile of the output buffer holds anything but
  // zeros: a tile no worker selected from is only written if it has to be cleared
  const uint32_t was_hot = agg_hot[c];
  if (!any_entries && !was_hot) return;
  if (tid == 0) agg_hot[c] = any_entries ? 1u : 0u;
  const int64_t j0 = (int64_t)c * kChunk;
  if (j0 + kChunk <= d && (d % 4) == 0) {
    for (uint32_t i = tid * 4; i < kChunk; i += kBlock * 4)
      *reinterpret_cast<float4*>(agg + j0 + i) = make_float4(s_tile[i], s_tile[i + 1], s_tile[i + 2], s_tile[i + 3]);
  } else {
    for (uint32_t i = tid; i < kChunk; i += kBlock)
      if (j0 + i < d) agg[j0 + i] = s_tile[i];
  }
}

// ---------------------------------------------------------- global Top-k ----
// The genie-aided baseline (subsection "Statistical Global Top-k"): all workers
// share the mask of the k largest entries of abar = sum_n omega_n a_n.
//
// k_global_accum, grid (nc): a block owns one 4096-entry chunk of all N rows.
// For n = 0..N-1 it forms a_n = eps_n + g_n (eps taken as 0 where the previous
// mask bit is set), stores it over the state and adds omega_n * a_n to the
// chunk of abar held in registers, in ascending worker order from +0 -- the
// order of the aggregation.
template <bool VEC>
__global__ void __launch_bounds__(kBlock)
k_global_accum(float* __restrict__ e, const float* __restrict__ g, const uint32_t* __restrict__ mask,
               const uint32_t* __restrict__ prev_sel_off, int64_t d, uint32_t nc, int32_t N,
               const float* __restrict__ omega, float* __restrict__ abar) {
  const uint32_t c = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int64_t base = (int64_t)c * kChunk + (int64_t)wv * 1024 + lane * 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[i][q] = 0.0f;
  for (int32_t n = 0; n < N; ++n) {
    const size_t row = (size_t)n * (size_t)d;
    const uint32_t* mrow = mask + (size_t)n * nc * kChunkWords;
    const size_t so = (size_t)n * (nc + 1) + c;
    const bool sent_any = prev_sel_off[so + 1] != prev_sel_off[so];
    const float w = omega[n];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t j0 = base + i * 256;
      if (j0 >= d) continue;
      const uint32_t mb = sent_any ? (mrow[j0 >> 5] >> (j0 & 31)) & 15u : 0u;
      if (VEC) {
        f32x4 ev = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(e + row + j0));
        const f32x4 gv = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g + row + j0));
        if (mb & 1u) ev.x = 0.f;
        if (mb & 2u) ev.y = 0.f;
        if (mb & 4u) ev.z = 0.f;
        if (mb & 8u) ev.w = 0.f;
        const f32x4 a4 = ev + gv;
        __builtin_nontemporal_store(a4, reinterpret_cast<f32x4*>(e + row + j0));
        acc[i][0] = __fadd_rn(acc[i][0], __fmul_rn(w, a4.x));
        acc[i][1] = __fadd_rn(acc[i][1], __fmul_rn(w, a4.y));
        acc[i][2] = __fadd_rn(acc[i][2], __fmul_rn(w, a4.z));
        acc[i][3] = __fadd_rn(acc[i][3], __fmul_rn(w, a4.w));
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int64_t j = j0 + q;
          if (j < d) {
            const float eps = ((mb >> q) & 1u) ? 0.f : e[row + j];
            const float a = eps + g[row + j];
            e[row + j] = a;
            acc[i][q] = __fadd_rn(acc[i][q], __fmul_rn(w, a));
          }
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t j0 = base + i * 256;
    if (j0 >= d) continue;
    if (VEC) {
      *reinterpret_cast<f32x4*>(abar + j0) = f32x4{acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (j0 + q < d) abar[j0 + q] = acc[i][q];
    }
  }
}

// k_global_apply, grid (ceil(nc/4), N): one wave per (worker, chunk).  Gives
// worker n the shared selection sidx [k] (ascending; chunk c holds positions
// ssel_off[c] .. ssel_off[c+1]) with shared mask words smask: index row, its own
// values a_n[j] gathered from the state, mask words and chunk offsets.
__global__ void __launch_bounds__(kBlock)
k_global_apply(const float* __restrict__ e, const int32_t* __restrict__ sidx,
               const uint32_t* __restrict__ ssel_off, const uint32_t* __restrict__ smask,
               const uint32_t* __restrict__ prev_sel_off, int32_t* __restrict__ out_idx,
               float* __restrict__ out_val, uint32_t* __restrict__ sel_off, uint32_t* __restrict__ mask,
               int64_t d, int64_t k, uint32_t nc) {
  const uint32_t n = blockIdx.y, lane = threadIdx.x & 63;
  const uint32_t c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= nc) return;
  const uint32_t p0 = ssel_off[c], p1 = ssel_off[c + 1];
  const size_t so = (size_t)n * (nc + 1) + c;
  const bool was_empty = prev_sel_off[so + 1] == prev_sel_off[so];
  if (lane == 0) {
    sel_off[so] = p0;
    if (c == nc - 1) sel_off[so + 1] = p1;
  }
  const size_t row = (size_t)n * (size_t)d;
  for (uint32_t p = p0 + lane; p < p1; p += 64) {
    const int32_t j = sidx[p];
    out_idx[(size_t)n * k + p] = j;
    out_val[(size_t)n * k + p] = e[row + (size_t)j];
  }
  if (!(was_empty && p0 == p1)) {
    const size_t wbase = ((size_t)n * nc + c) * kChunkWords;
    reinterpret_cast<uint2*>(mask + wbase)[lane] = reinterpret_cast<const uint2*>(smask + (size_t)c * kChunkWords)[lane];
  }
}

// -------------------------------------------------------- k_mask_overlap ----
// Number of entries that exactly c workers selected in the last round,
// c = 0..N.  A thread takes one mask word position (32 entries) and adds the N
// workers' words as bit-sliced counters: plane b holds bit b of the 32 column
// sums.  Entries that at most three workers selected (the bulk) are counted
// by population count, the others one by one.  grid-stride over the
// ceil(d/32) word positions.  Same-address global atomics cost about 12 ns each
// on this chip, so when N + 1 <= 1024 every block leaves its histogram in
// partial[block][0..N] and k_overlap_sum adds the blocks up; larger N add to
// counts directly (counts zeroed beforehand).
constexpr int kOverlapPlanes = 16;          // N <= 65535
constexpr uint32_t kOverlapBins = 1024;     // LDS histogram when N + 1 fits

__global__ void __launch_bounds__(kBlock)
k_mask_overlap(const uint32_t* __restrict__ mask, int64_t d, uint32_t nc, int32_t N, int planes,
               unsigned long long* __restrict__ counts, uint32_t* __restrict__ partial) {
  __shared__ uint32_t s_hist[kOverlapBins];
  const uint32_t tid = threadIdx.x;
  const bool lds = (uint32_t)N + 1u <= kOverlapBins;
  if (lds) for (uint32_t i = tid; i <= (uint32_t)N; i += kBlock) s_hist[i] = 0;
  __syncthreads();
  const size_t row_words = (size_t)nc * kChunkWords;
  const size_t nw = (size_t)((d + 31) / 32);
  uint32_t small[4] = {0, 0, 0, 0};                     // column sums 0..3, counted by population count
  for (size_t wd = (size_t)blockIdx.x * kBlock + tid; wd < nw; wd += (size_t)gridDim.x * kBlock) {
    uint32_t p[kOverlapPlanes];
#pragma unroll
    for (int b = 0; b < kOverlapPlanes; ++b) p[b] = 0;
    for (int32_t n0 = 0; n0 < N; n0 += 8) {           // eight independent loads in flight
      uint32_t m[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) m[q] = n0 + q < N ? mask[(size_t)(n0 + q) * row_words + wd] : 0u;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        uint32_t carry = m[q];
#pragma unroll
        for (int b = 0; b < kOverlapPlanes; ++b) {
          if (b < planes && carry) { const uint32_t t = p[b] & carry; p[b] ^= carry; carry = t; }
        }
      }
    }
    const int64_t left = d - (int64_t)wd * 32;
    const uint32_t valid = left >= 32 ? 0xFFFFFFFFu : ((1u << (uint32_t)left) - 1u);
    uint32_t high = 0;                                   // column sum >= 4
#pragma unroll
    for (int b = 2; b < kOverlapPlanes; ++b) high |= p[b];
    const uint32_t low = ~high & valid;
    small[0] += (uint32_t)__popc(~p[1] & ~p[0] & low);
    small[1] += (uint32_t)__popc(~p[1] & p[0] & low);
    small[2] += (uint32_t)__popc(p[1] & ~p[0] & low);
    small[3] += (uint32_t)__popc(p[1] & p[0] & low);
    uint32_t todo = high & valid;
    while (todo) {
      const uint32_t i = (uint32_t)__ffs(todo) - 1u;
      todo &= todo - 1u;
      uint32_t c = 0;
#pragma unroll
      for (int b = 0; b < kOverlapPlanes; ++b) c |= ((p[b] >> i) & 1u) << b;
      if (lds) atomicAdd(&s_hist[c], 1u);
      else atomicAdd(&counts[c], 1ull);
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    uint32_t v = small[q];
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    if ((tid & 63) == 0 && v && q <= N) {
      if (lds) atomicAdd(&s_hist[q], v);
      else atomicAdd(&counts[q], (unsigned long long)v);
    }
  }
  __syncthreads();
  if (lds)
    for (uint32_t i = tid; i <= (uint32_t)N; i += kBlock)
      partial[(size_t)blockIdx.x * ((uint32_t)N + 1u) + i] = s_hist[i];
}

// counts[c] = sum over the blocks of partial[block][c].  grid (N+1): one block per c.
__global__ void __launch_bounds__(kBlock)
k_overlap_sum(const uint32_t* __restrict__ partial, uint32_t blocks, int32_t N,
              unsigned long long* __restrict__ counts) {
  __shared__ unsigned long long s_part[kBlock / 64];
  const uint32_t c = blockIdx.x, tid = threadIdx.x;
  unsigned long long s = 0;
  for (uint32_t b = tid; b < blocks; b += kBlock) s += partial[(size_t)b * ((uint32_t)N + 1u) + c];
  for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o);
  if ((tid & 63) == 0) s_part[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) {
    unsigned long long t = 0;
    for (uint32_t i = 0; i < kBlock / 64; ++i) t += s_part[i];
    counts[c] = t;
  }
}

// ---------------------------------------------------------- k_sgd_update ----
// theta <- theta - eta * g, the product rounded before the subtraction.
template <bool VEC>
__global__ void __launch_bounds__(kBlock)
k_sgd_update(float* __restrict__ theta, const float* __restrict__ g, float eta, int64_t d) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  if (VEC) {
    const int64_t n4 = d / 4;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += stride) {
      const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(theta) + i);
      const f32x4 x = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g) + i);
      f32x4 o;
      o.x = __fsub_rn(t.x, __fmul_rn(eta, x.x));
      o.y = __fsub_rn(t.y, __fmul_rn(eta, x.y));
      o.z = __fsub_rn(t.z, __fmul_rn(eta, x.z));
      o.w = __fsub_rn(t.w, __fmul_rn(eta, x.w));
      __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(theta) + i);
    }
  } else {
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < d; i += stride)
      theta[i] = __fsub_rn(theta[i], __fmul_rn(eta, g[i]));
  }
}

// ------------------------------------------------------------- utilities ----
__global__ void k_fill_u32(uint32_t* p, size_t n, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

__global__ void k_copy_u32(uint32_t* dst, const uint32_t* src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

__global__ void k_init_ctl(WorkerCtl* ctl) {
  uint32_t* p = reinterpret_cast<uint32_t*>(&ctl[blockIdx.x]);
  for (uint32_t i = threadIdx.x; i < sizeof(WorkerCtl) / 4; i += blockDim.x) p[i] = 0;
  __syncthreads();
  if (threadIdx.x == 0) {
    WorkerCtl& c = ctl[blockIdx.x];
    c.tau_lo = kNoBound; c.tau_lo_mag = kNoBound; c.next_tau_lo = kNoBound; c.win_lo = kNoBound; c.next_win_lo = kNoBound;
    c.tau_prev = kNoBound; c.centre = kNoBound; c.margin_scale = 1.0f;
  }
}

// set_state: the state keeps, at the entries sent in the previous round, the
// value that was sent (the sweep reads it from there and restarts the error at
// zero): state[n][pidx[n][i]] = pval[n][i].  Indices outside [0,d) are skipped
// (k_check_ascending reports them).
__global__ void k_scatter_prev(float* __restrict__ e, const int32_t* __restrict__ pidx,
                               const float* __restrict__ pval, int64_t d, int64_t k, int32_t N) {
  const size_t total = (size_t)N * (size_t)k;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const size_t n = i / (size_t)k;
    const int64_t j = pidx[i];
    if (j >= 0 && j < d) e[n * (size_t)d + (size_t)j] = pval[i];
  }
}

// set_state: mask words and per-chunk offsets from an ascending index list.
// grid (ceil(nc/4), N): one wave per chunk.
__global__ void __launch_bounds__(kBlock)
k_build_mask(const int32_t* __restrict__ pidx, uint32_t* __restrict__ mask,
             uint32_t* __restrict__ sel_off, int64_t k, uint32_t nc) {
  __shared__ uint32_t s_m[4][kChunkWords];
  const uint32_t n = blockIdx.y, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint32_t c = blockIdx.x * 4 + wv;
  const bool live = c < nc;
  s_m[wv][lane] = 0;
  s_m[wv][lane + 64] = 0;
  __syncthreads();
  uint32_t first = 0;
  if (live) {
    const int32_t* pi = pidx + (size_t)n * k;
    const int64_t t0 = (int64_t)c * kChunk, t1 = t0 + kChunk;
    int64_t lo = 0, hi = k;
    while (lo < hi) { const int64_t mid = (lo + hi) >> 1; if ((int64_t)pi[mid] < t0) lo = mid + 1; else hi = mid; }
    first = (uint32_t)lo;
    if (lane == 0) {
      sel_off[(size_t)n * (nc + 1) + c] = first;
      if (c == nc - 1) sel_off[(size_t)n * (nc + 1) + nc] = (uint32_t)k;
    }
    for (int64_t p = lo + lane; p < k; p += 64) {
      const int64_t j = pi[p];
      if (j >= t1 || j < t0) break;
      const uint32_t jl = (uint32_t)(j - t0);
      atomicOr(&s_m[wv][jl >> 5], 1u << (jl & 31));
    }
  }
  __syncthreads();
  if (live) {
    const size_t wbase = ((size_t)n * nc + c) * kChunkWords;
    reinterpret_cast<uint2*>(mask + wbase)[lane] = make_uint2(s_m[wv][2 * lane], s_m[wv][2 * lane + 1]);
  }
}

// get_state: eps as the method defines it (0 on the last round's mask).
__global__ void k_export_eps(float* __restrict__ dst, const float* __restrict__ e,
                             const uint32_t* __restrict__ mask, int64_t d, uint32_t nc, int32_t N) {
  const size_t total = (size_t)N * (size_t)d;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const size_t n = i / (size_t)d, j = i - n * (size_t)d;
    const uint32_t bit = (mask[n * nc * kChunkWords + (j >> 5)] >> (j & 31)) & 1u;
    dst[i] = bit ? 0.0f : e[i];
  }
}

// grid (blocks, N)
__global__ void k_check_ascending(const int32_t* __restrict__ pidx, WorkerCtl* ctl, int64_t d, int64_t k) {
  const uint32_t n = blockIdx.y;
  const int32_t* pi = pidx + (size_t)n * k;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < k; i += (int64_t)gridDim.x * blockDim.x) {
    const int32_t v = pi[i];
    if (v < 0 || (int64_t)v >= d || (i > 0 && pi[i - 1] >= v)) atomicOr(&ctl[n].err, 2u);
  }
}

__global__ void k_tanh(const float* __restrict__ x, float* __restrict__ y, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    y[i] = tanh_f32_cr(x[i]);
}

}  // namespace rtk
