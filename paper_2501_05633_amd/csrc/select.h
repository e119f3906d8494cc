// Exact k-th score per worker: rank search in histograms, relative radix select, the controller of the next round's bound (k_select), the sampled bound of rounds without history, and the chunk scan.
#pragma once
#include "score.h"

namespace rtk {

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
// eight loads in flight per thread.
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
    constexpr uint32_t kFlight = 8;                    // 128-bit loads of a thread in flight together
    for (; i + (kFlight - 1) * NT < n4; i += kFlight * NT) {
      uint4 x[kFlight];
#pragma unroll
      for (uint32_t u = 0; u < kFlight; ++u) x[u] = b4[i + u * NT];
#pragma unroll
      for (uint32_t u = 0; u < kFlight; ++u) { f(x[u].x); f(x[u].y); f(x[u].z); f(x[u].w); }
    }
    {
      uint4 x[kFlight];
#pragma unroll
      for (uint32_t u = 0; u < kFlight; ++u) x[u] = i + u * NT < n4 ? b4[i + u * NT] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (uint32_t u = 0; u < kFlight; ++u)
        if (i + u * NT < n4) { f(x[u].x); f(x[u].y); f(x[u].z); f(x[u].w); }
    }
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
  // A short contiguous list (the boundary list, normally) is read from memory
  // once, all loads of a thread in flight together, and kept in registers for
  // every pass below.
  constexpr uint32_t kRegVec = 8;
  uint4 rk[kRegVec];
  uint32_t rtail = 0, n4 = 0, rem = 0;
  bool in_regs = src.flat != nullptr && src.lds == nullptr && src.count <= 4u * kRegVec * (uint32_t)NT;
  if (in_regs) {
    n4 = src.count / 4;
    rem = src.count - 4 * n4;
    const uint4* b4 = reinterpret_cast<const uint4*>(src.flat);
#pragma unroll
    for (uint32_t q = 0; q < kRegVec; ++q) {
      const uint32_t i = tid + q * NT;
      rk[q] = i < n4 ? b4[i] : make_uint4(0u, 0u, 0u, 0u);
    }
    if (tid < rem) rtail = src.flat[n4 * 4 + tid];
  }
  auto each_key = [&](auto f) {
    if (in_regs) {
#pragma unroll
      for (uint32_t q = 0; q < kRegVec; ++q)
        if (tid + q * NT < n4) { f(rk[q].x); f(rk[q].y); f(rk[q].z); f(rk[q].w); }
      if (tid < rem) f(rtail);
    } else {
      for_each_key<NT>(src, f);
    }
  };
  for (int guard = 0; guard < 64; ++guard) {
    for (uint32_t i = tid; i < kL1Bins; i += NT) s_hist[i] = 0;
    __syncthreads();
    uint32_t over = 0;
    each_key([&](uint32_t key) {
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
  // two finer levels need no further pass over the whole list
  const uint32_t in_bin = s_hist[pa];
  __syncthreads();
  if (!src.lds && s_stash != nullptr && in_bin <= stash_cap) {
    if (tid == 0) s_out[0] = 0;
    __syncthreads();
    each_key([&](uint32_t key) {
      if (key < base) return;
      if (((key - base) >> 13) == pa) s_stash[atomicAdd(&s_out[0], 1u)] = key;
    });
    __syncthreads();
    src.lds = s_stash;
    src.count = in_bin;
    in_regs = false;
    __syncthreads();
  }
  for (uint32_t i = tid; i < 512; i += NT) s_hist[i] = 0;
  __syncthreads();
  each_key([&](uint32_t key) {
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
  each_key([&](uint32_t key) {
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

constexpr uint32_t kLdsKeys = 11264;    // LDS room for the keys of the bin chosen at the first level

// SECOND = false: first invocation, all workers (validates the speculation).
// SECOND = true : after the dense selection, flagged workers only.
// Returns true (to every thread) if it flagged the worker for the dense selection.
template <bool SECOND, int NT>
__device__ __forceinline__ bool select_worker(uint32_t n, WorkerCtl* ctl, GlobalCtl* gctl,
                                              const uint32_t* cand_key,
                                              const uint32_t* bnd_key, int64_t k,
                                              uint32_t cap_r, uint32_t cap_total, uint32_t regions,
                                              uint32_t bnd_cap, float cand_target, int force_dense, int roots,
                                              uint32_t* s_hist, uint32_t* s_keys, uint32_t keys_cap,
                                              uint32_t* s_w, uint32_t* s_out) {
  const uint32_t tid = threadIdx.x;
  // The worker's control block is read once, by the block together, into LDS:
  // the many fields consulted below (most of them by thread 0 alone, one after
  // the other) then cost no memory round trip each.  Results are stored to the
  // block in memory (w).
  __shared__ WorkerCtl s_ctl;
  WorkerCtl& w = ctl[n];
  __syncthreads();            // (a caller's loop: thread 0 may still be reading the copy of the worker before)
  {
    const uint32_t* src = reinterpret_cast<const uint32_t*>(&w);
    uint32_t* dst = reinterpret_cast<uint32_t*>(&s_ctl);
    for (uint32_t i = tid; i < sizeof(WorkerCtl) / 4; i += NT) dst[i] = src[i];
  }
  __syncthreads();
  const WorkerCtl& c = s_ctl;
  if (SECOND && !c.need_dense) return false;
  const uint32_t K = (uint32_t)k;
  uint32_t n_tot = 0;
  if (!SECOND) {
    for (uint32_t r = 0; r < regions; ++r) n_tot += region_limit(c, r, cap_r);
    const bool need = force_dense || c.overflow || c.tau_lo == kNoBound || c.n_valid < K;
    if (need) {
      if (tid == 0) {
        w.n_cand = n_tot;
        w.need_dense = 1u;
        atomicOr(&gctl->any_dense, 1u);
      }
      return true;
    }
    // (n_cand and need_dense = 0 are stored with the other results at the end: a store ahead of
    // the barriers below would make the first of them wait for it)
  } else {
    n_tot = c.dense_total;
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
    // (read from memory: after the first level only the keys of one bin remain, and those are
    // gathered in LDS - copying the whole list there first is slower even when it fits)
    src.flat = list;
    base = win_lo;
    rank = K - n_hi;
  } else {
    // all candidates; only scores >= the bound can hold the k-th (at least k do)
    // (dense list: its smallest prior when the list has all the k + k_prev entries
    // asked for; a shorter list is the whole row, whose scores may all be damped)
    base = SECOND ? (c.dense_total >= c.f_want ? c.f_tau : 0u) : c.tau_lo;
    rank = K;
  }
  __syncthreads();
  uint32_t budget, ties;
  // (the key buffer in LDS is free for the gathering unless it holds the boundary list)
  uint32_t* stash = (s_keys != nullptr && src.lds == nullptr) ? s_keys : nullptr;
  const uint32_t tau = rel_select<NT>(src, base, rank, s_hist, s_w, s_out, stash, keys_cap, &budget, &ties);

  if (tid == 0) {
    w.n_cand = n_tot;
    if (!SECOND) w.need_dense = 0u;
    w.tau = tau;
    w.budget = budget;
    w.n_gt = K - budget;
    w.ties_total = ties;
    w.used_window = window ? 1u : 0u;
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
    // The k-th score drifts from round to round: extrapolate linearly -- unless
    // "same as last round" has been the better prediction lately (gradients whose
    // scale jitters from round to round: extrapolating doubles such noise).
    int64_t drift = 0;
    if (!shock && c.tau_prev != kNoBound) drift = (int64_t)tau - (int64_t)c.tau_prev;
    if (drift > (1 << 22)) drift = 1 << 22;
    if (drift < -(1 << 22)) drift = -(1 << 22);
    float acc_x = 0.0f, acc_l = 0.0f;
    if (!shock && c.tau_prev != kNoBound && c.pred_x != kNoBound) {
      const uint32_t ex = tau > c.pred_x ? tau - c.pred_x : c.pred_x - tau;
      const uint32_t el = tau > c.tau_prev ? tau - c.tau_prev : c.tau_prev - tau;
      acc_x = 0.7f * c.acc_x + (float)ex;
      acc_l = 0.7f * c.acc_l + (float)el;
    }
    w.acc_x = acc_x;
    w.acc_l = acc_l;
    const int64_t px = (int64_t)tau + drift;
    w.pred_x = (!shock && c.tau_prev != kNoBound) ? (uint32_t)(px < 0 ? 0 : (px > 0x7F000000 ? 0x7F000000 : px)) : kNoBound;
    const bool have_two = !shock && c.tau_prev != kNoBound;      // the prediction rests on two observed rounds
    const int64_t seen_drift = drift;
    if (acc_l < acc_x) drift = 0;
    int64_t centre = (int64_t)tau + drift;
    if (centre < 0) centre = 0;
    if (centre > 0x7F000000) centre = 0x7F000000;
    // expected error of that prediction: how far this round's prediction was off
    // if it rested on two earlier rounds, else half the drift
    const uint32_t adrift = (uint32_t)(seen_drift < 0 ? -seen_drift : seen_drift);
    uint32_t err;
    if (shock) err = kWinDefaultHalf;
    else if (c.centre != kNoBound && c.extrapolated) err = tau > c.centre ? tau - c.centre : c.centre - tau;
    else if (c.tau_prev != kNoBound) err = adrift / 2;
    else err = kWinDefaultHalf;
    if (!shock && (double)err < 0.5 * (double)c.err_prev) err = (uint32_t)(0.5 * (double)c.err_prev);
    // volatility: the largest error of the recent rounds.  The last error alone says little about
    // the next when the scale of the gradients jitters; the bound's margin below covers this one.
    uint32_t err_hi = shock ? err : (uint32_t)(0.8 * (double)c.err_hi);
    if (err_hi < err) err_hi = err;
    w.err_hi = err_hi;
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
    w.margin_scale = ms;
    const double by_target = ((double)cand_target - 1.0) * (double)K / dens;
    double margin = by_target;
    if (margin < 1.5 * (double)err_hi + 1024.0) margin = 1.5 * (double)err_hi + 1024.0;
    // ... but not so far down that the candidates would outgrow their buffer (room for 4k and some
    // slack): the number of entries above a bound grows like an exponential of the distance in bit
    // patterns (a power of the magnitude), whose rate two counts of this round give -- k entries
    // above tau and `above_ref` above `ref`, the bound (or the end of the dense selection's list).
    // The volatility term is cut off where that model expects 2.2k candidates (it underestimates:
    // the rate grows further down; a cut at 3k overflowed in the first rounds of the cnn workload).
    {
      const uint32_t ref = SECOND ? c.f_tau : c.tau_lo;
      const double above_ref = SECOND ? (double)c.dense_total : (double)c.n_valid;
      if (ref != kNoBound && tau > ref && above_ref > 1.02 * (double)K) {
        const double reach = (double)(tau - ref) * log(2.2) / log(above_ref / (double)K);
        const double most = reach > by_target ? reach : by_target;
        if (margin > most) margin = most;
      }
    }
    margin *= (double)ms;
    if (margin > 16777216.0) margin = 16777216.0;
    const int64_t anchor = drift > 0 ? (int64_t)tau + drift / 2 : centre;
    int64_t lo = anchor - (int64_t)margin;
    if (shock && c.dense_total >= c.f_want) {
      // The dense selection's list is exactly the k + k_prev (normally 2k) entries of
      // largest prior, ending at f_tau.  Whether the new level persists (the k-th score stays
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
    const uint32_t nlo = speculate ? (uint32_t)(lo > 0 ? lo : 0) : kNoBound;
    w.next_tau_lo = nlo;
    w.next_tau_lo_mag = magnitude_bound(nlo, roots);
    w.next_win_lo = speculate ? (uint32_t)(centre > (int64_t)h ? centre - (int64_t)h : 0) : kNoBound;
    w.next_win_hi = (uint32_t)centre + h;
    w.tau_prev = tau;
    w.centre = speculate ? (uint32_t)centre : kNoBound;
    w.err_prev = err;
    w.extrapolated = (speculate && have_two && seen_drift != 0) ? 1u : 0u;
  }
  return false;
}

// grid (N), 1024 threads: the first selection of a round, for all workers.
__global__ void __launch_bounds__(kScanBlock)
k_select(WorkerCtl* ctl, GlobalCtl* gctl, const uint32_t* __restrict__ cand_key,
         const uint32_t* __restrict__ bnd_key, const uint32_t* __restrict__ kn, uint32_t cap_r, uint32_t cap_total,
         uint32_t regions, uint32_t bnd_cap, float cand_target, int force_dense, int roots,
         uint32_t* __restrict__ fhist) {
  __shared__ uint32_t s_hist[kL1Bins];
  __shared__ uint32_t s_keys[kLdsKeys];
  __shared__ uint32_t s_w[16];
  __shared__ uint32_t s_out[2];
  const bool flagged = select_worker<false, kScanBlock>(blockIdx.x, ctl, gctl, cand_key, bnd_key, (int64_t)kn[blockIdx.x], cap_r,
                                                        cap_total, regions, bnd_cap, cand_target, force_dense, roots,
                                                        s_hist, s_keys, kLdsKeys, s_w, s_out);
  // a worker handed to the dense selection gets its three histograms cleared here, which saves that
  // kernel a phase and a grid barrier
  if (flagged) {
    uint32_t* fh = fhist + (size_t)blockIdx.x * 3 * kL1Bins;
    for (uint32_t i = threadIdx.x; i < 3 * kL1Bins; i += kScanBlock) fh[i] = 0;
  }
}

// -------------------------------------------------------------- sampling ----
// A round that starts without a bound from the previous one (round 0, after a
// reset or set_state) gets one from a strided sample of a = eps + g: the level-1
// histogram of the sample, from which k_sample_bound takes the bin edge above
// which about 1.6k entries of the whole row are expected.  The bound is only a
// guess - the selection verifies it like any other and falls back to the dense
// selection if it was wrong.
constexpr uint32_t kSampleMax = 1u << 18;     // sampled entries per worker (whole row if shorter)

// The sample is made of whole 32-entry lines (128 bytes of the state, of the
// gradients, and one mask word): memory hands out nothing smaller, and scattered
// groups of four cost eight times the traffic for the same number of entries
// (78 us against 16 us for the target workload's 16 x 2^18 entries).  Line l of
// the sample is line l * line_stride of the row; sample group i is the group
// i % 8 of sample line i / 8.
__device__ __forceinline__ int64_t sample_group_start(uint32_t i, uint32_t line_stride) {
  return (int64_t)(i >> 3) * line_stride * 32 + (int64_t)(i & 7u) * 4;
}

// grid (blocks, N).  PLAIN: the prior of Algorithm 2 (|a| itself) -- an instantiation without the
// code of the other priors, whose registers would halve the resident waves.
template <typename G, bool PLAIN>
__global__ void __launch_bounds__(kBlock)
k_sample_hist(const float* __restrict__ e, const G* __restrict__ g, const uint32_t* __restrict__ mask,
              int64_t d, uint32_t nc, uint32_t* __restrict__ shist, uint32_t n_groups, uint32_t line_stride,
              int roots_in) {
  const int roots = PLAIN ? 0 : roots_in;
  __shared__ uint32_t s_hist[kL1Bins];
  const uint32_t n = blockIdx.y, tid = threadIdx.x;
  for (uint32_t i = tid; i < kL1Bins; i += kBlock) s_hist[i] = 0;
  __syncthreads();
  const size_t row = (size_t)n * (size_t)d;
  const uint32_t* mrow = mask + (size_t)n * nc * kChunkWords;
  const bool vec = (d % 4 == 0) && (reinterpret_cast<uintptr_t>(g) % (4 * sizeof(G)) == 0);
  // a thread issues the loads of kSampleFlight sample groups before it uses the first
  constexpr int kSampleFlight = 4;
  const uint32_t step = gridDim.x * kBlock;
  for (uint32_t i0 = blockIdx.x * kBlock + tid; i0 < n_groups; i0 += step * kSampleFlight) {
    f32x4 ev[kSampleFlight], gv[kSampleFlight];
    uint32_t mb[kSampleFlight];
    bool fast[kSampleFlight];
#pragma unroll
    for (int u = 0; u < kSampleFlight; ++u) {
      const uint32_t i = i0 + (uint32_t)u * step;
      const int64_t j0 = sample_group_start(i, line_stride);
      fast[u] = vec && i < n_groups && j0 + 4 <= d;
      if (fast[u]) {                                    // one 128-bit load of the state, one of the gradients
        mb[u] = (mrow[j0 >> 5] >> (j0 & 31)) & 15u;
        ev[u] = *reinterpret_cast<const f32x4*>(e + row + j0);
        gv[u] = grad4_at(g, row + j0);
      }
    }
#pragma unroll
    for (int u = 0; u < kSampleFlight; ++u) {
      const uint32_t i = i0 + (uint32_t)u * step;
      if (i >= n_groups) break;
      const int64_t j0 = sample_group_start(i, line_stride);
      if (fast[u]) {
        f32x4 z = ev[u];
        if (mb[u] & 1u) z.x = 0.f;
        if (mb[u] & 2u) z.y = 0.f;
        if (mb[u] & 4u) z.z = 0.f;
        if (mb[u] & 8u) z.w = 0.f;
        const f32x4 a4 = z + gv[u];
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
  }
  __syncthreads();
  uint32_t* gh = shist + (size_t)n * 3 * kL1Bins;
  for (uint32_t i = tid; i < kL1Bins; i += kBlock) {
    const uint32_t v = s_hist[i];
    if (v) atomicAdd(&gh[i], v);
  }
}

// The same sample of a row whose state already holds the accumulated values.
__global__ void __launch_bounds__(kBlock)
k_sample_hist_state(const float* __restrict__ e, int64_t d, uint32_t* __restrict__ shist, uint32_t n_groups,
                    uint32_t line_stride, int roots) {
  __shared__ uint32_t s_hist[kL1Bins];
  const uint32_t n = blockIdx.y, tid = threadIdx.x;
  for (uint32_t i = tid; i < kL1Bins; i += kBlock) s_hist[i] = 0;
  __syncthreads();
  const size_t row = (size_t)n * (size_t)d;
  for (uint32_t i = blockIdx.x * kBlock + tid; i < n_groups; i += gridDim.x * kBlock) {
    const int64_t j0 = sample_group_start(i, line_stride);
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (j0 + q < d) atomicAdd(&s_hist[prior_key(e[row + j0 + q], roots) >> kL1Shift], 1u);
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
k_sample_bound(WorkerCtl* ctl, const uint32_t* __restrict__ shist, int64_t d, const uint32_t* __restrict__ kn,
               uint32_t n_sampled, int roots) {
  __shared__ uint32_t s_hist[kL1Bins];
  __shared__ uint32_t s_w[16];
  __shared__ uint32_t s_out[2];
  const uint32_t n = blockIdx.x, tid = threadIdx.x;
  const int64_t k = (int64_t)kn[n];
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

// ------------------------------------------------------------ chunk scan ----
// (Used by the dense selection to place its emission; the compaction of the
// round computes the same sums on the fly from two levels of partial sums.)
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


}  // namespace rtk
