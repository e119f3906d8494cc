// Ordered compaction of the selected pairs (k_chunk_count, k_compact) and the aggregation (k_aggregate).
#pragma once
#include "dense.h"

namespace rtk {

// --------------------------------------------------------- k_chunk_count ----
// Counting and compaction walk the candidate list chunk by chunk.  Most chunks
// are empty and a few hold hundreds of candidates, and what bounds these
// kernels is the number of waves that must each wait for two or three memory
// round trips: so a wave takes four chunks at once, sixteen lanes each
// (kChunksPerBlock chunks per block), and a lane takes eight candidates at a
// time with all its loads in flight together.
constexpr int kLaneBatch = 8;
constexpr uint32_t kLanesPerChunk = 16;
constexpr uint32_t kChunksPerWave = 64 / kLanesPerChunk;
constexpr uint32_t kChunksPerBlock = (kBlock / 64) * kChunksPerWave;

// grid (ceil(nc/kChunksPerBlock), N).  Candidates of the chunk with score > tau
// and == tau, per chunk and summed over the block's chunks (blk_gt, blk_tie:
// [N, gridDim.x]); the compaction builds its running sums from these two levels.
__global__ void __launch_bounds__(kBlock)
k_chunk_count(const WorkerCtl* __restrict__ ctl, const uint32_t* __restrict__ cand_key,
              const uint32_t* __restrict__ ch_off, const uint32_t* __restrict__ ch_cnt,
              uint32_t* __restrict__ ch_gt, uint32_t* __restrict__ ch_tie,
              uint32_t* __restrict__ blk_gt, uint32_t* __restrict__ blk_tie, uint32_t nc,
              uint32_t cap_total) {
  __shared__ uint32_t s_g[kBlock / 64], s_t[kBlock / 64];
  const uint32_t n = blockIdx.y, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint32_t grp = lane / kLanesPerChunk, gl = lane % kLanesPerChunk;
  const uint32_t c = (blockIdx.x * (kBlock / 64) + wv) * kChunksPerWave + grp;
  const bool live = c < nc;
  const size_t tix = (size_t)n * nc + (live ? c : 0);
  const uint32_t tau = ctl[n].tau;
  const bool abandoned = (ctl[n].err & 4u) != 0;     // dense selection given up: the lists are not to be read
  const uint32_t off = live ? ch_off[tix] : 0u, cnt = (live && !abandoned) ? ch_cnt[tix] : 0u;
  const uint32_t* key = cand_key + (size_t)n * cap_total + off;
  uint32_t gt = 0, tie = 0;
  for (uint32_t p0 = 0; p0 < cnt; p0 += kLanesPerChunk * kLaneBatch) {   // trip count uniform within a group of lanes
    uint32_t kk[kLaneBatch];
#pragma unroll
    for (int q = 0; q < kLaneBatch; ++q) {
      const uint32_t p = p0 + q * kLanesPerChunk + gl;
      kk[q] = p < cnt ? key[p] : 0u;
    }
#pragma unroll
    for (int q = 0; q < kLaneBatch; ++q) {
      const bool in = p0 + q * kLanesPerChunk + gl < cnt;
      gt += in && kk[q] > tau;
      tie += in && kk[q] == tau;
    }
  }
  for (uint32_t o = kLanesPerChunk / 2; o > 0; o >>= 1) { gt += __shfl_xor(gt, o); tie += __shfl_xor(tie, o); }
  if (live && gl == 0) { ch_gt[tix] = gt; ch_tie[tix] = tie; }
  // totals of the block: the groups' sums sit in their lane 0
  uint32_t wg = gl == 0 ? gt : 0u, wt = gl == 0 ? tie : 0u;
  for (int o = 32; o > 0; o >>= 1) { wg += __shfl_down(wg, o); wt += __shfl_down(wt, o); }
  if (lane == 0) { s_g[wv] = wg; s_t[wv] = wt; }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t bg = 0, bt = 0;
    for (uint32_t i = 0; i < kBlock / 64; ++i) { bg += s_g[i]; bt += s_t[i]; }
    blk_gt[(size_t)n * gridDim.x + blockIdx.x] = bg;
    blk_tie[(size_t)n * gridDim.x + blockIdx.x] = bt;
  }
}

// ------------------------------------------------------------- k_compact ----
// grid (ceil(nc/(4 * 64 / LPC)), N), LPC lanes per chunk.  Writes the selected
// pairs of the chunk in index order at sel_off[c], and the chunk's words of the
// round's mask (bit = entry selected).  The ordered placement is a chain of
// ballots over the chunk's candidates, so here the full chunks want more lanes
// than the counting does.  Where a chunk's pairs go follows from two running
// sums over the chunks before it, of the counts of scores > tau and == tau (the
// ties taken before a chunk number min(budget, ties before it)): the block adds
// up the counting blocks' totals before its own counting block, every group of
// lanes the chunks before its own inside that block.  It also writes sel_off
// (selected entries before each chunk; the last chunk adds the total).
constexpr uint32_t kCompactLanes = 32;

template <uint32_t LPC>
__global__ void __launch_bounds__(kBlock)
k_compact(WorkerCtl* ctl, GlobalCtl* gctl, const uint32_t* __restrict__ cand_key,
          const int32_t* __restrict__ cand_idx, const float* __restrict__ cand_val,
          const uint32_t* __restrict__ ch_off, const uint32_t* __restrict__ ch_cnt,
          const uint32_t* __restrict__ ch_gt, const uint32_t* __restrict__ ch_tie,
          const uint32_t* __restrict__ blk_gt, const uint32_t* __restrict__ blk_tie, uint32_t n_blk,
          uint32_t* __restrict__ sel_off, const uint32_t* __restrict__ prev_sel_off,
          int32_t* __restrict__ out_idx,
          float* __restrict__ out_val, uint32_t* __restrict__ mask,
          int64_t k, const uint32_t* __restrict__ kn, uint32_t nc, uint32_t cap_total, int next_force_dense) {
  constexpr uint32_t kCPW = 64 / LPC, kCPB = (kBlock / 64) * kCPW;
  static_assert(kChunksPerBlock % kCPB == 0, "a compaction block must lie inside one counting block");
  static_assert(kChunksPerBlock <= LPC, "one load per lane must cover the chunks of a counting block");
  __shared__ uint32_t s_m[kCPB][kChunkWords];
  __shared__ uint32_t s_g[kBlock / 64], s_t[kBlock / 64];
  constexpr uint32_t kWordsPerLane = kChunkWords / LPC;
  const uint32_t n = blockIdx.y, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint32_t grp = lane / LPC, gl = lane % LPC;
  const uint32_t slot = wv * kCPW + grp;                       // this group's chunk inside the block
  const uint32_t c = blockIdx.x * kCPB + slot;
  const bool live = c < nc;
#pragma unroll
  for (uint32_t i = 0; i < kWordsPerLane; ++i) s_m[slot][gl * kWordsPerLane + i] = 0;
  // running sums, level 1: the counting blocks before this block's own
  const uint32_t cblk = (blockIdx.x * kCPB) / kChunksPerBlock;           // the block's counting block
  uint32_t bg = 0, bt = 0;
  for (uint32_t i = threadIdx.x; i < cblk; i += kBlock) {
    bg += blk_gt[(size_t)n * n_blk + i];
    bt += blk_tie[(size_t)n * n_blk + i];
  }
  for (int o = 32; o > 0; o >>= 1) { bg += __shfl_down(bg, o); bt += __shfl_down(bt, o); }
  if (lane == 0) { s_g[wv] = bg; s_t[wv] = bt; }
  uint32_t cnt = 0, off = 0, my_gt = 0, my_tie = 0, in_g = 0, in_t = 0;
  bool was_empty = true;
  const size_t so = (size_t)n * (nc + 1) + (live ? c : 0);
  if (live) {
    const size_t tix = (size_t)n * nc + c;
    cnt = (ctl[n].err & 4u) ? 0u : ch_cnt[tix];       // nothing is read for a worker whose dense selection was given up
    off = ch_off[tix];
    my_gt = ch_gt[tix];
    my_tie = ch_tie[tix];
    was_empty = prev_sel_off[so + 1] == prev_sel_off[so];
    // level 2: the chunks before this one inside the counting block (fewer than kChunksPerBlock <= LPC)
    const uint32_t cfirst = cblk * kChunksPerBlock;
    if (cfirst + gl < c) { in_g = ch_gt[(size_t)n * nc + cfirst + gl]; in_t = ch_tie[(size_t)n * nc + cfirst + gl]; }
  }
  for (uint32_t o = LPC / 2; o > 0; o >>= 1) { in_g += __shfl_xor(in_g, o); in_t += __shfl_xor(in_t, o); }
  __syncthreads();                                                       // mask words zeroed, block sums placed
  uint32_t gt_before = in_g, tie_before = in_t;
  for (uint32_t i = 0; i < kBlock / 64; ++i) { gt_before += s_g[i]; tie_before += s_t[i]; }
  const uint32_t tau = ctl[n].tau, budget = ctl[n].budget;
  const uint32_t first = gt_before + (tie_before < budget ? tie_before : budget);
  uint32_t my_take = 0;
  if (tie_before < budget) { my_take = budget - tie_before; if (my_take > my_tie) my_take = my_tie; }
  const uint32_t my_sel = my_gt + my_take;
  const bool is_empty = my_sel == 0;
  uint32_t tie_run = tie_before;
  if (live && gl == 0) {
    sel_off[so] = first;
    if (c == nc - 1) {
      sel_off[so + 1] = first + my_sel;
      if (first + my_sel != kn[n]) atomicOr(&ctl[n].err, 1u);
    }
  }
  // a worker that keeps fewer than k entries: the rest of its row of the lists is (-1, 0)
  if (live && c == nc - 1)
    for (int64_t o = (int64_t)kn[n] + gl; o < k; o += LPC) { out_idx[(size_t)n * k + o] = -1; out_val[(size_t)n * k + o] = 0.0f; }
  const size_t cb = (size_t)n * cap_total + off;
  const uint64_t below_mask = (1ull << gl) - 1ull, group_bits = LPC == 64 ? ~0ull : (1ull << LPC) - 1ull;
  const uint32_t gshift = grp * LPC;
  uint32_t out = first;
  for (uint32_t p0 = 0; p0 < cnt; p0 += LPC * kLaneBatch) {   // trip count uniform within a group of lanes
    // keys, indices and values of eight candidates per lane, all loads in flight together
    uint32_t kk[kLaneBatch], jj[kLaneBatch];
    float vv[kLaneBatch];
#pragma unroll
    for (int q = 0; q < kLaneBatch; ++q) {
      const uint32_t p = p0 + q * LPC + gl;
      const bool in = p < cnt;
      kk[q] = in ? cand_key[cb + p] : 0u;
      jj[q] = in ? (uint32_t)cand_idx[cb + p] & ~kSentFlag : 0u;
      vv[q] = in ? cand_val[cb + p] : 0.0f;
    }
#pragma unroll
    for (int q = 0; q < kLaneBatch; ++q) {
      if (p0 + q * LPC >= cnt) break;                                    // uniform over the group
      const bool in = p0 + q * LPC + gl < cnt;
      const bool is_tie = in && kk[q] == tau;
      // ballots span the wave; a group reads its own bits (the lanes of
      // other groups that have left their loop contribute zeros)
      const uint64_t tb = (__ballot(is_tie) >> gshift) & group_bits;
      const bool take = in && (kk[q] > tau || (is_tie && tie_run + (uint32_t)__popcll(tb & below_mask) < budget));
      const uint64_t sb = (__ballot(take) >> gshift) & group_bits;
      if (take) {
        const uint32_t o = out + (uint32_t)__popcll(sb & below_mask);
        if ((int64_t)o < k) {
          out_idx[(size_t)n * k + o] = (int32_t)jj[q];
          out_val[(size_t)n * k + o] = vv[q];
          const uint32_t jl = jj[q] & (kChunk - 1);
          atomicOr(&s_m[slot][jl >> 5], 1u << (jl & 31));
        }
      }
      tie_run += (uint32_t)__popcll(tb);
      out += (uint32_t)__popcll(sb);
    }
  }
  __syncthreads();
  // The first block of a worker also prepares its control block for the next
  // round (what k_begin does after a start without history): a snapshot of the
  // round's diagnostics, cursors and counters cleared, the next bound and window
  // loaded.  No later kernel of the round and no other block of this one reads
  // what is cleared here (they read tau, budget and err).
  if (blockIdx.x == 0) {
    WorkerCtl& wc = ctl[n];
    if (threadIdx.x < kMaxRegions) wc.cursor[threadIdx.x] = 0;
    if (threadIdx.x == 0) {
      wc.snap_tau_lo = wc.tau_lo;
      wc.snap_n_cand = wc.need_dense ? wc.dense_total : wc.n_cand;
      wc.snap_used_dense = wc.need_dense;
      wc.snap_overflow = wc.overflow;
      wc.snap_used_window = wc.used_window;
      wc.snap_n_bnd = wc.n_bnd;
      wc.snap_n_valid = wc.n_valid;
      wc.snap_win_half = wc.win_lo == kNoBound ? 0u : (wc.win_hi - wc.win_lo) / 2;
      begin_round(wc, next_force_dense);
      if (n == 0) { gctl->any_dense = 0; gctl->bar_count = 0; }
    }
  }
  // a chunk without selected entries in the previous round has all-zero mask
  // words already: nothing to write if it has none now either
  if (live && !(was_empty && is_empty)) {
    const size_t wbase = ((size_t)n * nc + c) * kChunkWords + gl * kWordsPerLane;
    const uint32_t* m = &s_m[slot][gl * kWordsPerLane];
    if (kWordsPerLane == 2) {
      reinterpret_cast<uint2*>(mask + wbase)[0] = make_uint2(m[0], m[1]);
    } else {
#pragma unroll
      for (uint32_t i = 0; i < kWordsPerLane / 4; ++i)
        reinterpret_cast<uint4*>(mask + wbase)[i] = make_uint4(m[4 * i], m[4 * i + 1], m[4 * i + 2], m[4 * i + 3]);
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
  __shared__ uint32_t s_hot;
  const uint32_t c = blockIdx.x, tid = threadIdx.x;
  // agg_hot[c] tells whether this tile of the output buffer holds anything but
  // zeros.  Only thread 0 touches the word: it hands the old value to the block
  // through LDS here and stores the new one at the end.
  if (tid == 0) s_hot = agg_hot[c];
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
  // a tile no worker selected from is only written if it has to be cleared
  const uint32_t was_hot = s_hot;
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

}  // namespace rtk
