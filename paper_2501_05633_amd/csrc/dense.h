// The dense selection of workers whose speculation failed: one kernel with grid barriers (k_dense_all).
#pragma once
#include "select.h"

namespace rtk {

// ------------------------------------------------------------ dense path ----
// The dense selection of the workers whose speculation failed (or of every
// worker when the option forces it) runs as ONE kernel, k_dense_all, whose phases are
// separated by grid barriers: when no worker is flagged - the usual case - the
// whole path costs a single launch that returns at once.  The grid is sized by
// the host so that all blocks are resident together.
//
// Phases, for flagged workers only:
//   3 x (histogram of the prior's bits, every flagged
//   worker fed by its own group of blocks; pick the bin of rank
//   min(k + k_prev, d)) | per-chunk counts | chunk scan | ordered emission of
//   the k + k_prev largest priors as the candidate list | scores | exact k-th
//   score.  (k_prev: entries the worker sent in the previous round; 2k when
//   every round keeps k.)

// Histogram level LEVEL of worker n's row; block b of G covers a strided share.
template <int LEVEL, bool VEC>
__device__ __forceinline__ void dense_hist_worker(uint32_t n, uint32_t b, uint32_t G, const float* a,
                                                  int64_t d, const WorkerCtl* ctl, uint32_t* fhist,
                                                  uint32_t* s_hist, int roots) {
  const uint32_t tid = threadIdx.x;
  constexpr uint32_t bins = LEVEL == 1 ? kL1Bins : (LEVEL == 2 ? kL2Bins : kL3Bins);
  for (uint32_t i = tid; i < bins; i += kBlock) s_hist[i] = 0;
  __syncthreads();
  const uint32_t prefix = LEVEL == 2 ? ctl[n].f_prefix : (LEVEL == 3 ? ctl[n].f_prefix2 : 0u);
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

// Level LEVEL of the radix select of rank min(k + k_prev, d) over the prior's
// bits of worker n (k entries to keep now, k_prev entries sent in the previous
// round): finds, from the top bin downwards, the bin in which the cumulative
// count reaches the wanted rank.  One block; levels 1 and 2 are run by every
// block that is about to feed the worker's next histogram (they all find and
// store the same result), which saves a grid barrier per level.
template <int LEVEL>
__device__ __forceinline__ void dense_scan_worker(uint32_t n, WorkerCtl* ctl, const uint32_t* hist_all,
                                                  int64_t k, int64_t k_prev, int64_t d, uint32_t* s_sum,
                                                  uint32_t* s_scan) {
  constexpr uint32_t bins = LEVEL == 1 ? kL1Bins : (LEVEL == 2 ? kL2Bins : kL3Bins);
  constexpr uint32_t per = bins / kBlock;            // bins per thread (16, 8, 1)
  const uint32_t tid = threadIdx.x;
  WorkerCtl& c = ctl[n];
  const uint32_t* h = hist_all + ((size_t)n * 3 + (LEVEL - 1)) * kL1Bins;
  uint32_t want;
  if (LEVEL == 1) {
    want = (uint32_t)(k + k_prev < d ? k + k_prev : d);
    if (tid == 0) c.f_want = (uint32_t)(k + k_prev);
  } else {
    want = LEVEL == 2 ? c.f_krem : c.f_krem2;
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
        if (LEVEL == 1) { c.f_prefix = bin; c.f_krem = krem; }
        else if (LEVEL == 2) { c.f_prefix2 = (c.f_prefix << 11) | bin; c.f_krem2 = krem; }
        else { c.f_tau = (c.f_prefix2 << 8) | bin; c.f_budget = krem; }
      }
      run += loc[q];
    }
  }
  __syncthreads();
}

// The chunks c = first, first + stride, ... of worker n, one per WAVE (no block barrier): entries
// with prior bits > f_tau and == f_tau.  A lane keeps eight 128-bit loads in flight: the few
// resident waves of this kernel must cover the memory latency themselves.
template <bool VEC>
__device__ __forceinline__ void dense_count_chunks(uint32_t n, uint32_t first, uint32_t stride, const float* a,
                                                   int64_t d, const WorkerCtl* ctl, uint32_t* ch_gt,
                                                   uint32_t* ch_tie, uint32_t nc, int roots) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t tau = ctl[n].f_tau;
  const float* row = a + (size_t)n * (size_t)d;
  for (uint32_t c = first; c < nc; c += stride) {
    uint32_t gt = 0, tie = 0;
    const int64_t c0 = (int64_t)c * kChunk;
    if (VEC) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        float4 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int64_t j = c0 + ((h * 8 + i) * 64 + lane) * 4;
          v[i] = j < d ? *reinterpret_cast<const float4*>(row + j) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int64_t j = c0 + ((h * 8 + i) * 64 + lane) * 4;
          if (j < d) {
            const uint32_t k0 = prior_key(v[i].x, roots), k1 = prior_key(v[i].y, roots), k2 = prior_key(v[i].z, roots),
                           k3 = prior_key(v[i].w, roots);
            gt += (k0 > tau) + (k1 > tau) + (k2 > tau) + (k3 > tau);
            tie += (k0 == tau) + (k1 == tau) + (k2 == tau) + (k3 == tau);
          }
        }
      }
    } else {
      for (int i = 0; i < 64; ++i) {
        const int64_t j = c0 + i * 64 + lane;
        if (j < d) {
          const uint32_t key = prior_key(row[j], roots);
          gt += key > tau;
          tie += key == tau;
        }
      }
    }
    for (int o = 32; o > 0; o >>= 1) { gt += __shfl_down(gt, o); tie += __shfl_down(tie, o); }
    if (lane == 0) {
      ch_gt[(size_t)n * nc + c] = gt;
      ch_tie[(size_t)n * nc + c] = tie;
    }
  }
}

// Chunk c of worker n: writes its share of the k + k_prev largest |a| (ties: lowest
// indices) to the candidate list, in index order, at the offsets of the scan.
// The sweep has overwritten the state by now, so the value sent in the previous
// round is fetched from that round's list: its position there is the number of
// mask bits before the entry (prev_sel_off[c] of them in lower chunks; s_mw /
// s_rk, 128 words each, hold the chunk's mask words and their running counts).
// The caller has found the chunk's count non-zero.  Everything else the chunk
// needs from memory (offsets, mask words, the entries) is loaded at the top,
// before the first barrier, so that the few resident blocks of this kernel wait
// for memory twice per chunk (these loads, then the previous values), not once
// per step.
template <bool VEC>
__device__ __forceinline__ void dense_emit_chunk(uint32_t n, uint32_t c, const float* a_rows,
                                                 const uint32_t* mask, int64_t d, const WorkerCtl* ctl,
                                                 int32_t* cand_idx, float* cand_val, float* cand_prev,
                                                 const uint32_t* ch_off,
                                                 const uint32_t* tie_off, const uint32_t* prev_sel_off,
                                                 const float* prev_val, int64_t k, uint32_t nc,
                                                 uint32_t cap_total, uint32_t* s_wtot, uint32_t* s_ttot,
                                                 uint32_t* s_mw, uint32_t* s_rk, int roots) {
  const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const uint32_t* mrow = mask + (size_t)n * nc * kChunkWords;
  const size_t tix = (size_t)n * nc + c;
  const uint32_t mword = tid < kChunkWords ? mrow[(size_t)c * kChunkWords + tid] : 0u;
  const uint32_t sent_before = prev_sel_off[(size_t)n * (nc + 1) + c];
  const uint32_t tie_before = tie_off[tix];          // ties in lower chunks
  const uint32_t first_slot = ch_off[tix];
  const uint32_t tau = ctl[n].f_tau, budget = ctl[n].f_budget;
  const size_t row = (size_t)n * (size_t)d;
  const int64_t base = (int64_t)c * kChunk + (int64_t)wv * 1024 + lane * 4;
  float a[4][4];
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
  }
  if (tid < kChunkWords) s_mw[tid] = mword;
  __syncthreads();
  if (tid < 64) {                                    // wave 0: running count of mask bits, two words per lane
    const uint32_t c0 = (uint32_t)__popc(s_mw[2 * tid]), c1 = (uint32_t)__popc(s_mw[2 * tid + 1]);
    uint32_t x = c0 + c1;
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t y = __shfl_up(x, o);
      if (tid >= (uint32_t)o) x += y;
    }
    const uint32_t before = sent_before + x - (c0 + c1);
    s_rk[2 * tid] = before;
    s_rk[2 * tid + 1] = before + c0;
  }
  uint32_t gtf = 0, tief = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t j0 = base + i * 256;
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
  // (the barrier inside also publishes s_rk)
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
  const ChunkPos cp = ordered_positions(flags, s_wtot);
  const float* pv = prev_val + (size_t)n * k;
  const size_t out = (size_t)n * cap_total + first_slot + cp.wave_base;
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

// A grid barrier did not complete (its blocks were not resident together within
// the spin limit): the flagged workers' selection is abandoned.  Their error
// bit makes the counting and compaction kernels skip them and regtopk_get_stats
// fail; the host-visible word set by the barrier makes the next regtopk_step fail.
__device__ __forceinline__ void dense_abandon(WorkerCtl* ctl, int32_t N) {
  for (int32_t n = threadIdx.x; n < N; n += kBlock)
    if (ctl[n].need_dense) atomicOr(&ctl[n].err, 4u);
}

// grid (G): G blocks resident together.  See the section header.
// The kernel is compiled for four waves per SIMD (128 registers; the double-double
// code of the score variants spills a little): left to itself the compiler takes
// 173 registers, which halves the resident blocks -- and the grid is one block per
// compute unit less than fit, so one block per unit instead of three.  The passes
// over the rows are bound by how many loads the resident waves keep in flight
// (all 16 workers of the target workload: 5.5 ms at one block per unit, 3.9 ms at three).
template <bool VEC>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(4, 4)))
k_dense_all(const float* a_rows, const uint32_t* mask, const uint32_t* prev_sel_off, int64_t d, WorkerCtl* ctl,
            GlobalCtl* gctl, uint32_t* fhist, uint32_t* ch_gt, uint32_t* ch_tie, uint32_t* ch_off,
            uint32_t* ch_cnt, uint32_t* tie_off, int32_t* cand_idx, float* cand_val, float* cand_prev,
            uint32_t* cand_key,
            const uint32_t* bnd_key, const float* prev_val, const float* gprev, int64_t k, const uint32_t* kn, uint32_t nc,
            int32_t N, uint32_t cap_r, uint32_t cap_total, uint32_t regions, uint32_t bnd_cap,
            const float* omega, float mu, int use_reg, float cand_target, ScoreKind sk,
            uint32_t* host_err) {
  if (gctl->any_dense == 0) return;
  const int roots = sk.roots;
  __shared__ uint32_t s_hist[kL1Bins];
  __shared__ uint32_t s_a[kBlock], s_b[kBlock];
  __shared__ uint32_t s_w[16], s_out[2], s_x[4], s_y[4];
  const uint32_t b = blockIdx.x, G = gridDim.x, tid = threadIdx.x;

  // (k_select has cleared the histograms of the workers it flagged)
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
  if (!grid_barrier(gctl, G, host_err)) { dense_abandon(ctl, N); return; }
  for (uint32_t r = grp; r < n_flagged; r += groups) {
    const uint32_t n = r == grp ? first_worker : flagged_worker(ctl, N, r, &n_flagged, s_w, s_out);
    if (n < (uint32_t)N) {
      dense_scan_worker<1>(n, ctl, fhist, (int64_t)kn[n], (int64_t)prev_sel_off[(size_t)n * (nc + 1) + nc], d, s_a, s_b);
      dense_hist_worker<2, VEC>(n, sub, sub_cnt, a_rows, d, ctl, fhist, s_hist, roots);
    }
  }
  if (!grid_barrier(gctl, G, host_err)) { dense_abandon(ctl, N); return; }
  for (uint32_t r = grp; r < n_flagged; r += groups) {
    const uint32_t n = r == grp ? first_worker : flagged_worker(ctl, N, r, &n_flagged, s_w, s_out);
    if (n < (uint32_t)N) {
      dense_scan_worker<2>(n, ctl, fhist, (int64_t)kn[n], (int64_t)prev_sel_off[(size_t)n * (nc + 1) + nc], d, s_a, s_b);
      dense_hist_worker<3, VEC>(n, sub, sub_cnt, a_rows, d, ctl, fhist, s_hist, roots);
    }
  }
  if (!grid_barrier(gctl, G, host_err)) { dense_abandon(ctl, N); return; }
  for (int32_t n = b; n < N; n += G)
    if (ctl[n].need_dense) dense_scan_worker<3>(n, ctl, fhist, (int64_t)kn[n], (int64_t)prev_sel_off[(size_t)n * (nc + 1) + nc], d, s_a, s_b);
  if (!grid_barrier(gctl, G, host_err)) { dense_abandon(ctl, N); return; }

  for (int32_t n = 0; n < N; ++n) {
    if (!ctl[n].need_dense) continue;
    dense_count_chunks<VEC>(n, b * (kBlock / 64) + (tid >> 6), G * (kBlock / 64), a_rows, d, ctl, ch_gt, ch_tie, nc, roots);
  }
  if (!grid_barrier(gctl, G, host_err)) { dense_abandon(ctl, N); return; }
  for (int32_t n = b; n < N; n += G)
    if (ctl[n].need_dense) chunk_scan_worker<true, kBlock>(n, ctl, ch_gt, ch_tie, ch_off, ch_cnt, tie_off, nc, (int64_t)kn[n], s_w);
  if (!grid_barrier(gctl, G, host_err)) { dense_abandon(ctl, N); return; }
  for (int32_t n = 0; n < N; ++n) {
    if (!ctl[n].need_dense) continue;
    // (the count of the block's next chunk is fetched while the current one is emitted)
    uint32_t cnt = b < nc ? ch_cnt[(size_t)n * nc + b] : 0u;
    for (uint32_t c = b; c < nc; c += G) {
      const uint32_t cnt_next = c + G < nc ? ch_cnt[(size_t)n * nc + c + G] : 0u;
      if (cnt)
        dense_emit_chunk<VEC>(n, c, a_rows, mask, d, ctl, cand_idx, cand_val, cand_prev, ch_off, tie_off,
                              prev_sel_off, prev_val, k, nc, cap_total, s_x, s_y, s_a, s_b, roots);
      cnt = cnt_next;
    }
  }
  if (!grid_barrier(gctl, G, host_err)) { dense_abandon(ctl, N); return; }

  for (int32_t n = 0; n < N; ++n) {
    if (!ctl[n].need_dense) continue;
    const uint32_t total = ctl[n].dense_total;
    const size_t cb = (size_t)n * cap_total;
    const float w = omega[n];
    for (uint32_t p = b * kBlock + tid; p < total; p += G * kBlock)
      cand_key[cb + p] = score_entry((uint32_t)cand_idx[cb + p], cand_val[cb + p], cand_prev[cb + p], use_reg, gprev, w, mu, sk);
  }
  if (!grid_barrier(gctl, G, host_err)) { dense_abandon(ctl, N); return; }
  for (int32_t n = b; n < N; n += G)
    if (ctl[n].need_dense)
      // (the finer levels of the selection use the first 512 words of the histogram's LDS; the rest
      // of it takes the keys of the bin chosen at the first level, which saves two passes over the list)
      select_worker<true, kBlock>(n, ctl, gctl, cand_key, bnd_key, (int64_t)kn[n], cap_r, cap_total, regions, bnd_cap,
                                  cand_target, 0, roots, s_hist, s_hist + 512, kL1Bins - 512, s_w, s_out);
}

}  // namespace rtk
