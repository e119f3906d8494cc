// HIP kernels of the RegTop-k round for gfx950 (wave64).
//
// Data flow of one round (all N workers batched; rows of length d):
//
//   k_begin         reset counters / histograms, load this round's speculative bound
//   k_accum_emit    a = eps + g written over eps (the one dense read/write sweep);
//                   entries with |a| >= tau_lo are appended, in index order per
//                   4096-entry chunk, to the worker's candidate list
//   k_score         exact score of every candidate (regulariser for entries sent in
//                   the previous round, found by binary search in that round's
//                   index list) + level-1 histogram of the score bits
//   k_validate      the speculation holds iff no overflow and >= k candidates have
//                   score >= tau_lo; otherwise the worker is flagged for
//   k_dense_*       the dense selection: exact radix select of the 2k largest |a|
//                   (a superset of the true top-k, see below), count, scan and an
//                   ordered emission of exactly those entries as the candidate list
//   k_cand_hist     levels 2 and 3 of the radix select over the candidate scores
//   k_select_scan   picks the histogram bin that holds the wanted rank
//   k_chunk_count / k_chunk_scan / k_compact
//                   ordered compaction of the selected (index, value) pairs,
//                   lowest-index ties first, and zeroing of eps on the mask
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

// score bits (sign bit is always 0): level 1 = bits 30..19, level 2 = 18..8, level 3 = 7..0
constexpr int kL1Shift = 19, kL1Bins = 4096;
constexpr int kL2Shift = 8, kL2Bins = 2048;
constexpr int kL3Bins = 256;

struct WorkerCtl {
  uint32_t tau_lo;        // speculative lower bound (bit pattern, multiple of 2^19) or kNoBound
  uint32_t next_tau_lo;   // bound for the next round
  uint32_t overflow;      // a candidate region overflowed in k_accum_emit
  uint32_t need_dense;    // dense selection runs for this worker
  uint32_t n_cand;        // candidates handed to the exact selection
  uint32_t dense_total;   // candidates written by the dense emission (compact from slot 0)
  uint32_t c_prefix;      // radix-select state over candidate scores
  uint32_t c_krem;
  uint32_t tau;           // k-th largest score (bits)
  uint32_t n_gt;          // candidates with score > tau
  uint32_t budget;        // ties to take, lowest indices first
  uint32_t ties_total;
  uint32_t f_prefix;      // radix-select state of the dense selection over |a| bits
  uint32_t f_krem;
  uint32_t f_tau;
  uint32_t f_budget;
  uint32_t err;           // bit 0: selected count != k, bit 1: bad set_state input
  uint32_t pad[15];
  uint32_t cursor[kMaxRegions];
};

__device__ __forceinline__ uint32_t lanes_below(uint64_t ballot) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

__device__ __forceinline__ uint32_t key_of(float a) { return __float_as_uint(a) & 0x7FFFFFFFu; }

__device__ __forceinline__ bool slot_valid(const WorkerCtl& c, uint32_t p, uint32_t cap_r) {
  if (c.need_dense) return p < c.dense_total;
  const uint32_t r = p / cap_r;
  const uint32_t cur = c.cursor[r] < cap_r ? c.cursor[r] : cap_r;
  return (p - r * cap_r) < cur;
}

// ---------------------------------------------------------------- k_begin ----
__global__ void __launch_bounds__(kBlock)
k_begin(WorkerCtl* ctl, uint32_t* chist, uint32_t* fhist, int force_dense) {
  const uint32_t n = blockIdx.x, tid = threadIdx.x;
  uint32_t* ch = chist + (size_t)n * 3 * kL1Bins;
  uint32_t* fh = fhist + (size_t)n * 3 * kL1Bins;
  for (uint32_t i = tid; i < 3 * kL1Bins; i += kBlock) { ch[i] = 0; fh[i] = 0; }
  WorkerCtl& c = ctl[n];
  if (tid < kMaxRegions) c.cursor[tid] = 0;
  if (tid == 0) {
    c.tau_lo = force_dense ? kNoBound : c.next_tau_lo;
    c.overflow = 0; c.need_dense = 0; c.n_cand = 0; c.dense_total = 0;
    c.c_prefix = 0; c.c_krem = 0; c.tau = 0; c.n_gt = 0; c.budget = 0; c.ties_total = 0;
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

template <bool VEC>
__global__ void __launch_bounds__(kBlock)
k_accum_emit(float* __restrict__ e, const float* __restrict__ g, int64_t d,
             WorkerCtl* __restrict__ ctl, int32_t* __restrict__ cand_idx,
             float* __restrict__ cand_val, uint32_t* __restrict__ ch_off,
             uint32_t* __restrict__ ch_cnt, uint32_t nc, uint32_t cap_r, uint32_t cap_total,
             uint32_t regions) {
  __shared__ uint32_t s_wtot[4];
  __shared__ uint32_t s_base;
  const uint32_t c = blockIdx.x, n = blockIdx.y;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const size_t row = (size_t)n * (size_t)d;
  const uint32_t tau_lo = ctl[n].tau_lo;
  const int64_t base = (int64_t)c * kChunk + (int64_t)wv * 1024 + lane * 4;
  float a[4][4];
  uint32_t flags = 0;
  if (VEC) {
    f32x4 ev[4], gv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t j0 = base + i * 256;
      if (j0 < d) {
        ev[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(e + row + j0));
        gv[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g + row + j0));
      } else {
        ev[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        gv[i] = ev[i];
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t j0 = base + i * 256;
      const f32x4 s4 = ev[i] + gv[i];
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
        if (j < d) {
          a[i][q] = e[row + j] + g[row + j];
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
        cand_idx[out + p] = (int32_t)(base + i * 256 + q);
        cand_val[out + p] = a[i][q];
        ++p;
      }
    }
  }
}

// --------------------------------------------------------------- k_score ----
// Likelihood factor of an entry that was sent in the previous round.
__device__ __forceinline__ float likelihood_sent(float a_now, float a_before, float g_before,
                                                 float w, float mu) {
  const float num = __fsub_rn(g_before, __fmul_rn(w, a_before));
  const float den = __fmul_rn(w, a_now);
  if (den == 0.0f) return 1.0f;
  const float D = __fdiv_rn(num, den);
  const float r = fabsf(__fadd_rn(1.0f, D));
  const float x = __fdiv_rn(r, mu);
  if (x != x) return 1.0f;
  return tanh_f32_cr(x);
}

// grid (blocks, N).  only_dense: second invocation, for the workers whose
// candidate list was rebuilt by the dense selection.
__global__ void __launch_bounds__(kBlock)
k_score(const WorkerCtl* __restrict__ ctl, const int32_t* __restrict__ cand_idx,
        const float* __restrict__ cand_val, uint32_t* __restrict__ cand_key,
        const int32_t* __restrict__ prev_idx, const float* __restrict__ prev_val,
        const uint32_t* __restrict__ prev_sel_off, const float* __restrict__ gprev,
        uint32_t* __restrict__ chist, int64_t d, int64_t k, uint32_t nc, uint32_t cap_r,
        uint32_t cap_total, float w, float mu, int use_reg, int only_dense) {
  __shared__ uint32_t s_hist[kL1Bins];
  const uint32_t n = blockIdx.y, tid = threadIdx.x;
  const WorkerCtl& c = ctl[n];
  if (only_dense && !c.need_dense) return;
  if (!only_dense && c.overflow) return;      // list is incomplete; the dense selection rebuilds it
  for (uint32_t i = tid; i < kL1Bins; i += kBlock) s_hist[i] = 0;
  __syncthreads();
  const size_t cbase = (size_t)n * cap_total;
  const int32_t* pi = prev_idx + (size_t)n * k;
  const float* pv = prev_val + (size_t)n * k;
  const uint32_t* so = prev_sel_off + (size_t)n * (nc + 1);
  for (uint32_t p = blockIdx.x * kBlock + tid; p < cap_total; p += gridDim.x * kBlock) {
    if (!slot_valid(c, p, cap_r)) continue;
    const int32_t j = cand_idx[cbase + p];
    if (j < 0 || (int64_t)j >= d) continue;
    const float a = cand_val[cbase + p];
    float f = 1.0f;
    if (use_reg) {
      const uint32_t cj = (uint32_t)j >> kChunkLog;
      uint32_t lo = so[cj], hi = so[cj + 1];
      while (lo < hi) {                       // lower bound of j in the chunk's slice
        const uint32_t mid = (lo + hi) >> 1;
        if (pi[mid] < j) lo = mid + 1; else hi = mid;
      }
      if (lo < so[cj + 1] && pi[lo] == j) f = likelihood_sent(a, pv[lo], gprev[j], w, mu);
    }
    const uint32_t key = __float_as_uint(__fmul_rn(fabsf(a), f));
    cand_key[cbase + p] = key;
    atomicAdd(&s_hist[key >> kL1Shift], 1u);
  }
  __syncthreads();
  uint32_t* gh = chist + (size_t)n * 3 * kL1Bins;
  for (uint32_t i = tid; i < kL1Bins; i += kBlock) {
    const uint32_t v = s_hist[i];
    if (v) atomicAdd(&gh[i], v);
  }
}

// ------------------------------------------------------------ k_validate ----
// grid (N).  Decides whether the speculative candidate list is a superset of
// the true top-k: no overflow and at least k candidates scored >= tau_lo.
__global__ void __launch_bounds__(kBlock)
k_validate(WorkerCtl* ctl, uint32_t* chist, int64_t k, uint32_t regions, int force_dense) {
  __shared__ uint32_t s_red[kBlock];
  __shared__ uint32_t s_need;
  const uint32_t n = blockIdx.x, tid = threadIdx.x;
  WorkerCtl& c = ctl[n];
  uint32_t* h = chist + (size_t)n * 3 * kL1Bins;
  const uint32_t tl = c.tau_lo;
  const uint32_t first = (tl == kNoBound) ? kL1Bins : (tl >> kL1Shift);
  uint32_t s = 0;
  for (uint32_t i = tid; i < kL1Bins; i += kBlock)
    if (i >= first) s += h[i];
  s_red[tid] = s;
  __syncthreads();
  for (uint32_t o = kBlock / 2; o > 0; o >>= 1) {
    if (tid < o) s_red[tid] += s_red[tid + o];
    __syncthreads();
  }
  if (tid == 0) {
    uint32_t tot = 0;
    for (uint32_t r = 0; r < regions; ++r) tot += c.cursor[r];
    const uint32_t need = (force_dense || c.overflow || (int64_t)s_red[0] < k) ? 1u : 0u;
    c.n_cand = tot;
    c.need_dense = need;
    s_need = need;
  }
  __syncthreads();
  if (s_need)
    for (uint32_t i = tid; i < kL1Bins; i += kBlock) h[i] = 0;
}

// ---------------------------------------------------------- k_dense_hist ----
// grid (blocks, N).  Histogram of the |a| bits of flagged workers' rows.
template <int LEVEL>
__global__ void __launch_bounds__(kBlock)
k_dense_hist(const float* __restrict__ a, int64_t d, const WorkerCtl* __restrict__ ctl,
             uint32_t* __restrict__ fhist) {
  __shared__ uint32_t s_hist[kL1Bins];
  const uint32_t n = blockIdx.y, tid = threadIdx.x;
  const WorkerCtl& c = ctl[n];
  if (!c.need_dense) return;
  constexpr uint32_t bins = LEVEL == 1 ? kL1Bins : (LEVEL == 2 ? kL2Bins : kL3Bins);
  for (uint32_t i = tid; i < bins; i += kBlock) s_hist[i] = 0;
  __syncthreads();
  const uint32_t prefix = c.f_prefix;
  const float* row = a + (size_t)n * (size_t)d;
  for (int64_t j = (int64_t)blockIdx.x * kBlock + tid; j < d; j += (int64_t)gridDim.x * kBlock) {
    const uint32_t key = key_of(row[j]);
    if (LEVEL == 1) atomicAdd(&s_hist[key >> kL1Shift], 1u);
    else if (LEVEL == 2) { if ((key >> kL1Shift) == prefix) atomicAdd(&s_hist[(key >> kL2Shift) & (kL2Bins - 1)], 1u); }
    else { if ((key >> kL2Shift) == prefix) atomicAdd(&s_hist[key & (kL3Bins - 1)], 1u); }
  }
  __syncthreads();
  uint32_t* gh = fhist + ((size_t)n * 3 + (LEVEL - 1)) * kL1Bins;
  for (uint32_t i = tid; i < bins; i += kBlock) {
    const uint32_t v = s_hist[i];
    if (v) atomicAdd(&gh[i], v);
  }
}

// ----------------------------------------------------------- k_cand_hist ----
// grid (blocks, N).  Levels 2 and 3 over the candidate score bits.
template <int LEVEL>
__global__ void __launch_bounds__(kBlock)
k_cand_hist(const WorkerCtl* __restrict__ ctl, const uint32_t* __restrict__ cand_key,
            uint32_t* __restrict__ chist, uint32_t cap_r, uint32_t cap_total) {
  __shared__ uint32_t s_hist[kL2Bins];
  const uint32_t n = blockIdx.y, tid = threadIdx.x;
  const WorkerCtl& c = ctl[n];
  constexpr uint32_t bins = LEVEL == 2 ? kL2Bins : kL3Bins;
  for (uint32_t i = tid; i < bins; i += kBlock) s_hist[i] = 0;
  __syncthreads();
  const uint32_t prefix = c.c_prefix;
  const size_t cbase = (size_t)n * cap_total;
  for (uint32_t p = blockIdx.x * kBlock + tid; p < cap_total; p += gridDim.x * kBlock) {
    if (!slot_valid(c, p, cap_r)) continue;
    const uint32_t key = cand_key[cbase + p];
    if (LEVEL == 2) { if ((key >> kL1Shift) == prefix) atomicAdd(&s_hist[(key >> kL2Shift) & (kL2Bins - 1)], 1u); }
    else { if ((key >> kL2Shift) == prefix) atomicAdd(&s_hist[key & (kL3Bins - 1)], 1u); }
  }
  __syncthreads();
  uint32_t* gh = chist + ((size_t)n * 3 + (LEVEL - 1)) * kL1Bins;
  for (uint32_t i = tid; i < bins; i += kBlock) {
    const uint32_t v = s_hist[i];
    if (v) atomicAdd(&gh[i], v);
  }
}

// --------------------------------------------------------- k_select_scan ----
// grid (N), one block per worker.  Finds, from the top bin downwards, the bin
// in which the cumulative count reaches the wanted rank.
//   DENSE = false: radix select of rank k over candidate scores (levels 1..3);
//                  level 1 also derives the next round's speculative bound.
//   DENSE = true : radix select of rank min(2k, d) over |a| bits, flagged workers.
template <bool DENSE, int LEVEL>
__global__ void __launch_bounds__(kBlock)
k_select_scan(WorkerCtl* ctl, const uint32_t* __restrict__ hist_all, int64_t k, int64_t d,
              float cand_target) {
  constexpr uint32_t bins = LEVEL == 1 ? kL1Bins : (LEVEL == 2 ? kL2Bins : kL3Bins);
  constexpr uint32_t per = bins / kBlock;            // bins per thread (16, 8, 1)
  __shared__ uint32_t s_sum[kBlock];
  __shared__ uint32_t s_scan[kBlock];
  const uint32_t n = blockIdx.x, tid = threadIdx.x;
  WorkerCtl& c = ctl[n];
  if (DENSE && !c.need_dense) return;
  const uint32_t* h = hist_all + ((size_t)n * 3 + (LEVEL - 1)) * kL1Bins;
  uint32_t want;
  if (LEVEL == 1) {
    int64_t r = DENSE ? (2 * k < d ? 2 * k : d) : k;
    want = (uint32_t)r;
  } else {
    want = DENSE ? c.f_krem : c.c_krem;
  }
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
        if (DENSE) {
          if (LEVEL == 1) { c.f_prefix = bin; c.f_krem = krem; }
          else if (LEVEL == 2) { c.f_prefix = (c.f_prefix << 11) | bin; c.f_krem = krem; }
          else { c.f_tau = (c.f_prefix << 8) | bin; c.f_budget = krem; }
        } else {
          if (LEVEL == 1) { c.c_prefix = bin; c.c_krem = krem; }
          else if (LEVEL == 2) { c.c_prefix = (c.c_prefix << 11) | bin; c.c_krem = krem; }
          else {
            c.tau = (c.c_prefix << 8) | bin; c.budget = krem;
            c.n_gt = (uint32_t)k - krem; c.ties_total = loc[q];
          }
        }
      }
      run += loc[q];
    }
  }
  if (!DENSE && LEVEL == 1) {
    // next round's bound: the bin edge at which about cand_target*k candidates
    // of this round lie above; if this round had fewer, two bins below its own.
    const uint32_t tgt = (uint32_t)((double)cand_target * (double)k);
    uint32_t total = 0;
    if (tid == kBlock - 1) total = above + s;
    if (above < tgt && tgt <= above + s) {
      uint32_t run = above;
#pragma unroll
      for (uint32_t q = 0; q < per; ++q) {
        if (run < tgt && tgt <= run + loc[q]) c.next_tau_lo = (bins - 1 - (tid * per + q)) << kL1Shift;
        run += loc[q];
      }
    }
    if (tid == kBlock - 1 && total < tgt) {
      uint32_t lowest = 0;                            // lowest non-empty bin = this thread's region or above
      const uint32_t tl = c.tau_lo;
      uint32_t b = (tl == kNoBound) ? 0u : (tl >> kL1Shift);
      lowest = b > 2 ? b - 2 : 0;
      c.next_tau_lo = (tl == kNoBound) ? kNoBound : (lowest << kL1Shift);
    }
  }
}

// --------------------------------------------------------- k_dense_count ----
// grid (nc, N).  Per chunk: entries with |a| bits > f_tau and == f_tau.
__global__ void __launch_bounds__(kBlock)
k_dense_count(const float* __restrict__ a, int64_t d, const WorkerCtl* __restrict__ ctl,
              uint32_t* __restrict__ ch_gt, uint32_t* __restrict__ ch_tie, uint32_t nc) {
  __shared__ uint32_t s_gt[4], s_tie[4];
  const uint32_t c = blockIdx.x, n = blockIdx.y, tid = threadIdx.x;
  const WorkerCtl& w = ctl[n];
  if (!w.need_dense) return;
  const uint32_t tau = w.f_tau;
  const float* row = a + (size_t)n * (size_t)d;
  uint32_t gt = 0, tie = 0;
  for (int i = 0; i < 16; ++i) {
    const int64_t j = (int64_t)c * kChunk + i * kBlock + tid;
    if (j < d) {
      const uint32_t key = key_of(row[j]);
      gt += key > tau;
      tie += key == tau;
    }
  }
  for (int o = 32; o > 0; o >>= 1) { gt += __shfl_down(gt, o); tie += __shfl_down(tie, o); }
  if ((tid & 63) == 0) { s_gt[tid >> 6] = gt; s_tie[tid >> 6] = tie; }
  __syncthreads();
  if (tid == 0) {
    ch_gt[(size_t)n * nc + c] = s_gt[0] + s_gt[1] + s_gt[2] + s_gt[3];
    ch_tie[(size_t)n * nc + c] = s_tie[0] + s_tie[1] + s_tie[2] + s_tie[3];
  }
}

// ---------------------------------------------------------- k_chunk_scan ----
// grid (N), 1024 threads.  Exclusive scans over the chunks of one worker:
//   tie_off[c] = ties before chunk c;
//   sel[c]     = gt[c] + clamp(budget - tie_off[c], 0, tie[c])   (lowest-index ties first);
//   sel_off[c] = selected entries before chunk c  (nc+1 values).
// DENSE: budget = f_budget, sel_off/sel go to ch_off/ch_cnt (placement of the
// dense emission) and dense_total.  Otherwise budget = ctl.budget, sel_off goes
// to the round's sel_off table and the total is checked against k.  tie_off is
// written in both cases.
constexpr int kScanBlock = 1024;

__device__ __forceinline__ uint32_t block_excl_scan_1024(uint32_t v, uint32_t* s_w /*[16]*/,
                                                         uint32_t* total) {
  const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  uint32_t x = v;
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(x, o);
    if (lane >= (uint32_t)o) x += y;
  }
  if (lane == 63) s_w[wv] = x;
  __syncthreads();
  uint32_t wb = 0, tot = 0;
  for (uint32_t i = 0; i < 16; ++i) { const uint32_t t = s_w[i]; if (i < wv) wb += t; tot += t; }
  __syncthreads();
  *total = tot;
  return wb + x - v;
}

template <bool DENSE>
__global__ void __launch_bounds__(kScanBlock)
k_chunk_scan(WorkerCtl* ctl, const uint32_t* __restrict__ ch_gt, const uint32_t* __restrict__ ch_tie,
             uint32_t* __restrict__ out_off, uint32_t* __restrict__ out_cnt,
             uint32_t* __restrict__ out_tieoff, uint32_t nc, int64_t k) {
  __shared__ uint32_t s_w[16];
  const uint32_t n = blockIdx.x, tid = threadIdx.x;
  WorkerCtl& c = ctl[n];
  if (DENSE && !c.need_dense) return;
  const uint32_t budget = DENSE ? c.f_budget : c.budget;
  const uint32_t* gt = ch_gt + (size_t)n * nc;
  const uint32_t* tie = ch_tie + (size_t)n * nc;
  uint32_t* off = out_off + (size_t)n * (DENSE ? nc : nc + 1);
  uint32_t* cnt = DENSE ? out_cnt + (size_t)n * nc : nullptr;
  uint32_t* tof = out_tieoff + (size_t)n * nc;
  uint32_t tie_run = 0, sel_run = 0;
  for (uint32_t base = 0; base < nc; base += kScanBlock) {
    const uint32_t ci = base + tid;
    const uint32_t t = ci < nc ? tie[ci] : 0;
    const uint32_t g = ci < nc ? gt[ci] : 0;
    uint32_t ttot, stot;
    const uint32_t toff = tie_run + block_excl_scan_1024(t, s_w, &ttot);
    uint32_t take = 0;
    if (toff < budget) { take = budget - toff; if (take > t) take = t; }
    const uint32_t sel = g + take;
    const uint32_t soff = sel_run + block_excl_scan_1024(sel, s_w, &stot);
    if (ci < nc) {
      off[ci] = soff;
      tof[ci] = toff;
      if (DENSE) cnt[ci] = sel;
    }
    tie_run += ttot;
    sel_run += stot;
  }
  if (tid == 0) {
    if (DENSE) c.dense_total = sel_run;
    else {
      off[nc] = sel_run;
      if ((int64_t)sel_run != k) c.err |= 1u;
    }
  }
}

// ---------------------------------------------------------- k_dense_emit ----
// grid (nc, N).  Writes the 2k largest |a| (ties: lowest indices) of a flagged
// worker as its candidate list, in index order, at the offsets of the scan.
template <bool VEC>
__global__ void __launch_bounds__(kBlock)
k_dense_emit(const float* __restrict__ a_rows, int64_t d, WorkerCtl* __restrict__ ctl,
             int32_t* __restrict__ cand_idx, float* __restrict__ cand_val,
             const uint32_t* __restrict__ ch_off, const uint32_t* __restrict__ ch_cnt,
             const uint32_t* __restrict__ tie_off, uint32_t nc, uint32_t cap_total) {
  __shared__ uint32_t s_wtot[4];
  __shared__ uint32_t s_ttot[4];
  const uint32_t c = blockIdx.x, n = blockIdx.y;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const WorkerCtl& w = ctl[n];
  if (!w.need_dense) return;
  const size_t tix = (size_t)n * nc + c;
  if (ch_cnt[tix] == 0) return;
  const uint32_t tau = w.f_tau, budget = w.f_budget;
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
        const uint32_t key = key_of(a[i][q]);
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
  if (flags == 0) return;
  const size_t out = (size_t)n * cap_total + ch_off[tix] + cp.wave_base;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t p = cp.lane_base[i];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if ((flags >> (i * 4 + q)) & 1u) {
        cand_idx[out + p] = (int32_t)(base + i * 256 + q);
        cand_val[out + p] = a[i][q];
        ++p;
      }
    }
  }
}

// --------------------------------------------------------- k_chunk_count ----
// grid (ceil(nc/4), N): one wave per chunk.  Candidates of the chunk with
// score > tau and == tau.
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
  for (uint32_t p = lane; p < cnt; p += 64) {
    const uint32_t kk = key[p];
    gt += kk > tau;
    tie += kk == tau;
  }
  for (int o = 32; o > 0; o >>= 1) { gt += __shfl_down(gt, o); tie += __shfl_down(tie, o); }
  if (lane == 0) { ch_gt[tix] = gt; ch_tie[tix] = tie; }
}

// ------------------------------------------------------------- k_compact ----
// grid (ceil(nc/4), N): one wave per chunk.  Writes the selected pairs of the
// chunk in index order at sel_off[c] and zeroes eps there.
__global__ void __launch_bounds__(kBlock)
k_compact(const WorkerCtl* __restrict__ ctl, const uint32_t* __restrict__ cand_key,
          const int32_t* __restrict__ cand_idx, const float* __restrict__ cand_val,
          const uint32_t* __restrict__ ch_off, const uint32_t* __restrict__ ch_cnt,
          const uint32_t* __restrict__ sel_off, const uint32_t* __restrict__ tie_off,
          int32_t* __restrict__ out_idx, float* __restrict__ out_val, float* __restrict__ e,
          int64_t d, int64_t k, uint32_t nc, uint32_t cap_total) {
  const uint32_t n = blockIdx.y, lane = threadIdx.x & 63;
  const uint32_t c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= nc) return;
  const size_t tix = (size_t)n * nc + c;
  const uint32_t cnt = ch_cnt[tix];
  if (cnt == 0) return;
  const uint32_t off = ch_off[tix];
  const uint32_t tau = ctl[n].tau, budget = ctl[n].budget;
  const size_t cb = (size_t)n * cap_total + off;
  uint32_t out = sel_off[(size_t)n * (nc + 1) + c];
  uint32_t tie_run = tie_off[tix];
  for (uint32_t p0 = 0; p0 < cnt; p0 += 64) {
    const uint32_t p = p0 + lane;
    uint32_t kk = 0;
    bool in = p < cnt;
    if (in) kk = cand_key[cb + p];
    const bool is_tie = in && kk == tau;
    const uint64_t tb = __ballot(is_tie);
    const bool take = in && (kk > tau || (is_tie && tie_run + lanes_below(tb) < budget));
    const uint64_t sb = __ballot(take);
    if (take) {
      const uint32_t o = out + lanes_below(sb);
      if ((int64_t)o < k) {
        const int32_t j = cand_idx[cb + p];
        out_idx[(size_t)n * k + o] = j;
        out_val[(size_t)n * k + o] = cand_val[cb + p];
        e[(size_t)n * (size_t)d + j] = 0.0f;
      }
    }
    tie_run += (uint32_t)__popcll(tb);
    out += (uint32_t)__popcll(sb);
  }
}

// ----------------------------------------------------------- k_aggregate ----
// grid (nc).  agg tile of 4096 entries: +0, then + w*val of every worker in
// ascending worker order (indices of one worker are distinct, so plain LDS
// read-modify-write), written once.
__global__ void __launch_bounds__(kBlock)
k_aggregate(const int32_t* __restrict__ out_idx, const float* __restrict__ out_val,
            const uint32_t* __restrict__ sel_off, float* __restrict__ agg, int64_t d, int64_t k,
            uint32_t nc, int32_t N, float w) {
  __shared__ float s_tile[kChunk];
  const uint32_t c = blockIdx.x, tid = threadIdx.x;
  for (uint32_t i = tid; i < kChunk; i += kBlock) s_tile[i] = 0.0f;
  __syncthreads();
  const int32_t jbase = (int32_t)(c << kChunkLog);
  for (int32_t n = 0; n < N; ++n) {
    const uint32_t s0 = sel_off[(size_t)n * (nc + 1) + c];
    const uint32_t s1 = sel_off[(size_t)n * (nc + 1) + c + 1];
    for (uint32_t p = s0 + tid; p < s1; p += kBlock) {
      const int32_t j = out_idx[(size_t)n * k + p] - jbase;
      if ((uint32_t)j < (uint32_t)kChunk)
        s_tile[j] = __fadd_rn(s_tile[j], __fmul_rn(w, out_val[(size_t)n * k + p]));
    }
    __syncthreads();
  }
  const int64_t j0 = (int64_t)c * kChunk;
  for (uint32_t i = tid; i < kChunk; i += kBlock)
    if (j0 + i < d) agg[j0 + i] = s_tile[i];
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
  if (threadIdx.x == 0) { ctl[blockIdx.x].tau_lo = kNoBound; ctl[blockIdx.x].next_tau_lo = kNoBound; }
}

// set_state: rebuild the per-chunk offsets of a previous index list and check it.
// grid (ceil((nc+1)/256), N)
__global__ void k_rebuild_sel_off(const int32_t* __restrict__ pidx, uint32_t* __restrict__ sel_off,
                                  WorkerCtl* ctl, int64_t d, int64_t k, uint32_t nc) {
  const uint32_t n = blockIdx.y;
  const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c > nc) return;
  const int32_t* pi = pidx + (size_t)n * k;
  const int64_t target = (int64_t)c * kChunk;
  int64_t lo = 0, hi = k;
  while (lo < hi) { const int64_t mid = (lo + hi) >> 1; if ((int64_t)pi[mid] < target) lo = mid + 1; else hi = mid; }
  sel_off[(size_t)n * (nc + 1) + c] = (uint32_t)lo;
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
