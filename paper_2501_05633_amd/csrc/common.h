// Constants, control blocks and small device helpers shared by all kernels of the RegTop-k round.
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
  uint32_t f_prefix;      // radix-select state of the dense selection over the prior's bits: bin chosen at
  uint32_t f_krem;        //   level 1 and the rank wanted inside it
  uint32_t f_prefix2;     //   the same after level 2 (the bins of levels 1 and 2 joined).  One pair per level:
  uint32_t f_krem2;       //   several blocks store a level's (identical) result, none updates a pair in place
  uint32_t f_tau;
  uint32_t f_budget;
  uint32_t err;           // bit 0: selected count != k, bit 1: bad set_state input, bit 2: the dense selection of this worker was abandoned
  uint32_t tau_prev;      // k-th score of the previous round or kNoBound
  uint32_t centre;        // predicted k-th score of this round (window centre) or kNoBound
  uint32_t err_prev;      // |prediction error| of the previous round
  float margin_scale;     // widens the bound's safety margin after a failed speculation
  uint32_t extrapolated;  // this round's prediction used the drift of two earlier rounds
  uint32_t tau_lo_mag;    // smallest |a| bit pattern whose prior reaches tau_lo (= tau_lo for the plain prior)
  // diagnostics of the last completed round, copied before the counters are cleared for the next one
  uint32_t snap_tau_lo, snap_n_cand, snap_used_dense, snap_overflow, snap_used_window, snap_n_bnd, snap_n_valid, snap_win_half;
  uint32_t f_want;        // entries the dense selection lists: k + k_prev (not clamped to d)
  uint32_t next_tau_lo_mag; // next_tau_lo as a bound on |a| (its pre-image under the prior), set with it
  uint32_t err_hi;        // largest |prediction error| of the recent rounds (decays by a fifth per round)
  uint32_t pred_x;        // what the linear extrapolation predicted for this round, or kNoBound
  float acc_x, acc_l;     // decayed sums of the errors of the extrapolation / of "same as last round"
  uint32_t pad[1];
  uint32_t cursor[kMaxRegions];
};

__device__ __forceinline__ uint32_t lanes_below(uint64_t ballot) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

__device__ __forceinline__ uint32_t key_of(float a) { return __float_as_uint(a) & 0x7FFFFFFFu; }

// Prior |a|^y (appendix remark on sub-linear scaling).  `roots` is the prior's
// code: 0..3 = that many correctly rounded binary32 square roots of |a|
// (y = 2^-roots); a negative value = minus the bit pattern of a binary32
// exponent 0 < y < 1, the prior then being the correctly rounded |a|^y.
__host__ __device__ __forceinline__ int prior_code_of_exponent(float y) {
  return -(int)__builtin_bit_cast(uint32_t, y);
}
__device__ __forceinline__ float prior_of(float a, int roots) {
  float p = fabsf(a);
  if (roots < 0) return pow_f32_cr(p, __uint_as_float((uint32_t)(-roots)));
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
// wait is bounded: after kBarrierSpinLimit polls a block gives up and records
// the fact in bar_err (and in *host_err, a word of pinned host memory that the
// next regtopk_step looks at); the blocks still waiting see bar_err and leave as
// well.  Returns false, to every thread of the block, when the barrier did not
// complete: the caller must return without touching memory again, so the grid
// always drains and nothing is computed from half-finished phases.
constexpr uint32_t kBarrierSpinLimit = 1u << 22;

__device__ __forceinline__ bool grid_barrier(GlobalCtl* g, uint32_t nblocks, uint32_t* host_err) {
  __shared__ uint32_t s_ok;
  __syncthreads();
  if (threadIdx.x == 0) {
    __threadfence();
    uint32_t ok = 1;
    if (__hip_atomic_load(&g->bar_err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
      ok = 0;
    } else {
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
          ++spins;
          if ((spins & 63u) == 0 && __hip_atomic_load(&g->bar_err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
            ok = 0;                                      // another block gave up
            break;
          }
          if (spins > kBarrierSpinLimit) {
            atomicOr(&g->bar_err, 1u);
            if (host_err) __hip_atomic_store(host_err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            ok = 0;
            break;
          }
        }
      }
    }
    // The acquiring fence (it drops what this compute unit's L1 and this XCD's L2 hold of other XCDs'
    // lines) is issued once, by this thread, before the block's own barrier hands its effect to the
    // other waves: the fences of a device's blocks queue up (about 0.1 us per block and barrier for a
    // fence per wave, 0.06 us for one per block; 768 blocks).
    __threadfence();
    s_ok = ok;
  }
  __syncthreads();
  return s_ok != 0;
}

}  // namespace rtk
