// The dense sweep: per-round reset, ordered positions of flagged entries inside a chunk, and k_accum_emit.
#pragma once
#include "common.h"

namespace rtk {

// ---------------------------------------------------------------- k_begin ----
// Start of a round for one worker (one thread; the cursors are cleared by the
// caller): this round's bound and window from what the last selection left,
// counters cleared.  (The bound on |a| that goes with the score bound was computed
// by the selection that left it: for a root or power prior that is a binary search
// through the prior, too heavy for the kernels that call this.)
__device__ __forceinline__ void begin_round(WorkerCtl& c, int force_dense) {
  c.tau_lo = force_dense ? kNoBound : c.next_tau_lo;
  c.tau_lo_mag = force_dense ? kNoBound : c.next_tau_lo_mag;
  c.win_lo = force_dense ? kNoBound : c.next_win_lo;
  c.win_hi = c.next_win_hi;
  c.overflow = 0; c.need_dense = 0; c.n_cand = 0; c.n_valid = 0; c.n_hi = 0; c.n_bnd = 0;
  c.dense_total = 0; c.used_window = 0;
}

// Normally the last kernel of a round prepares the next one; this kernel does it
// after a start without history (create, reset, set_state) or a change of an
// option the preparation depends on.
__global__ void __launch_bounds__(kBlock)
k_begin(WorkerCtl* ctl, GlobalCtl* gctl, int force_dense) {
  const uint32_t n = blockIdx.x, tid = threadIdx.x;
  if (n == 0 && tid == 0) { gctl->any_dense = 0; gctl->bar_count = 0; }   // (arrivals of an abandoned barrier are dropped)
  WorkerCtl& c = ctl[n];
  if (tid < kMaxRegions) c.cursor[tid] = 0;
  if (tid == 0) {
    begin_round(c, force_dense);
    c.tau = 0; c.n_gt = 0; c.budget = 0; c.ties_total = 0;
    c.f_prefix = 0; c.f_krem = 0; c.f_prefix2 = 0; c.f_krem2 = 0; c.f_tau = 0; c.f_budget = 0;
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
// grid (nc, N).  The sweep for rows of any length and alignment, with scalar
// loads (k_accum_emit_vec takes the rows that can be read 128 bits at a time).
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

// Appends the flagged entries of the block's chunk (flags bit i*4+q = entry
// (i, lane, q), see ChunkPos) to worker n's candidate list, in index order: one
// atomic per block reserves room in region c % regions.  a = accumulated
// gradients, eo = what the state held, mb = previous-mask bits.  Called by all
// threads of the block.
__device__ __forceinline__ void emit_chunk(uint32_t flags, const float (&a)[4][4], const float (&eo)[4][4],
                                           const uint32_t (&mb)[4], int64_t base, uint32_t n, uint32_t c,
                                           WorkerCtl* __restrict__ ctl, int32_t* __restrict__ cand_idx,
                                           float* __restrict__ cand_val, float* __restrict__ cand_prev,
                                           uint32_t* __restrict__ ch_off, uint32_t* __restrict__ ch_cnt,
                                           uint32_t nc, uint32_t cap_r, uint32_t cap_total, uint32_t regions,
                                           uint32_t* s_wtot, uint32_t* s_base_p) {
  const uint32_t tid = threadIdx.x;
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
    *s_base_p = b;
  }
  __syncthreads();
  const uint32_t b = *s_base_p;
  if (tid == 0) {                        // (stored after the barrier, which would otherwise wait for these stores)
    ch_off[tix] = (b == kNoBound) ? 0 : b;
    ch_cnt[tix] = (b == kNoBound) ? 0 : cp.total;
  }
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

template <typename G>
__global__ void __launch_bounds__(kBlock)
k_accum_emit(float* __restrict__ e, const G* __restrict__ g, const uint32_t* __restrict__ mask,
             int64_t d, WorkerCtl* __restrict__ ctl,
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
  // previous round's mask: the 4 bits of entries j0..j0+3 lie in one word (chunks
  // from which nothing was sent hold zeros)
  const uint32_t* mrow = mask + (size_t)n * nc * kChunkWords;
  uint32_t mb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t j0 = base + i * 256;
    mb[i] = j0 < d ? (mrow[j0 >> 5] >> (j0 & 31)) & 15u : 0u;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t j = j0 + q;
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
  emit_chunk(flags, a, eo, mb, base, n, c, ctl, cand_idx, cand_val, cand_prev, ch_off, ch_cnt, nc, cap_r, cap_total, regions,
             s_wtot, &s_base);
}

// ----------------------------------------------------------- k_emit_only ----
// The sweep of a row whose state already holds the accumulated values (the
// selector of the global Top-k round: k_global_accum leaves abar there): nothing
// is added or stored, the entries with |a| >= the bound are emitted.  grid (nc, N).
template <bool VEC>
__global__ void __launch_bounds__(kBlock)
k_emit_only(const float* __restrict__ e, int64_t d, WorkerCtl* __restrict__ ctl, int32_t* __restrict__ cand_idx,
            float* __restrict__ cand_val, float* __restrict__ cand_prev, uint32_t* __restrict__ ch_off,
            uint32_t* __restrict__ ch_cnt, uint32_t nc, uint32_t cap_r, uint32_t cap_total, uint32_t regions) {
  __shared__ uint32_t s_wtot[4];
  __shared__ uint32_t s_base;
  const uint32_t c = blockIdx.x, n = blockIdx.y;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const size_t row = (size_t)n * (size_t)d;
  const uint32_t tau_lo = ctl[n].tau_lo_mag;
  const int64_t base = (int64_t)c * kChunk + (int64_t)wv * 1024 + lane * 4;
  float a[4][4], eo[4][4];
  uint32_t mb[4] = {0u, 0u, 0u, 0u};
  uint32_t flags = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t j0 = base + i * 256;
    f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
    if (VEC) {
      if (j0 < d) v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(e + row + j0));
    } else {
      if (j0 < d) v.x = e[row + j0];
      if (j0 + 1 < d) v.y = e[row + j0 + 1];
      if (j0 + 2 < d) v.z = e[row + j0 + 2];
      if (j0 + 3 < d) v.w = e[row + j0 + 3];
    }
    a[i][0] = v.x; a[i][1] = v.y; a[i][2] = v.z; a[i][3] = v.w;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      eo[i][q] = 0.f;
      if (j0 + q < d && key_of(a[i][q]) >= tau_lo) flags |= 1u << (i * 4 + q);
    }
  }
  emit_chunk(flags, a, eo, mb, base, n, c, ctl, cand_idx, cand_val, cand_prev, ch_off, ch_cnt, nc, cap_r, cap_total, regions,
             s_wtot, &s_base);
}


// ------------------------------------------------------ k_accum_emit_vec ----
// The sweep for rows that can be read 128 bits at a time (d % 4 == 0, aligned):
// grid (nc, N), 1024 / NI threads per block, NI groups of four entries per
// thread; wave v covers entries [v*256*NI, (v+1)*256*NI) of the chunk,
// iteration i the 256 entries after i*256, lane l the four entries at l*4.
// Measured on the target workload: NI = 4 (256 threads) 777 us, NI = 2 (512
// threads) 751 us, NI = 1 (1024 threads) 801 us; the host launches NI = 2.
// Same steps as k_accum_emit above.  The sweep touches every byte exactly once,
// so it loads and stores with the non-temporal hint; the mask words are read
// unconditionally, together with the state and the gradients, so that no load
// waits for another.
constexpr int kSweepNI = 2;

template <typename G, int NI>
__global__ void __launch_bounds__(1024 / NI)
k_accum_emit_vec(float* __restrict__ e, const G* __restrict__ g, const uint32_t* __restrict__ mask,
               int64_t d, WorkerCtl* __restrict__ ctl, int32_t* __restrict__ cand_idx,
               float* __restrict__ cand_val, float* __restrict__ cand_prev, uint32_t* __restrict__ ch_off,
               uint32_t* __restrict__ ch_cnt, uint32_t nc, uint32_t cap_r, uint32_t cap_total, uint32_t regions) {
  constexpr int W = 16 / NI;
  __shared__ uint32_t s_wtot[W];
  __shared__ uint32_t s_base;
  const uint32_t c = blockIdx.x, n = blockIdx.y;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const size_t row = (size_t)n * (size_t)d;
  const uint32_t tau_lo = ctl[n].tau_lo_mag;
  const int64_t base = (int64_t)c * kChunk + (int64_t)wv * (256 * NI) + lane * 4;
  const uint32_t* mrow = mask + (size_t)n * nc * kChunkWords;
  float a[NI][4], eo[NI][4];
  uint32_t mb[NI];
  uint32_t flags = 0;
  f32x4 ev[NI], gv[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int64_t j0 = base + i * 256;
    if (j0 < d) {
      mb[i] = (mrow[j0 >> 5] >> (j0 & 31)) & 15u;
      ev[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(e + row + j0));
      gv[i] = grad4_at(g, row + j0);
    } else {
      mb[i] = 0;
      ev[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      gv[i] = ev[i];
    }
  }
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int64_t j0 = base + i * 256;
    eo[i][0] = ev[i].x; eo[i][1] = ev[i].y; eo[i][2] = ev[i].z; eo[i][3] = ev[i].w;
    f32x4 z4 = ev[i];
    if (mb[i]) {
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
  uint32_t lane_base[NI];
  uint32_t run = 0;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    uint32_t below = 0, tot = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint64_t b = __ballot((flags >> (i * 4 + q)) & 1u);
      below += lanes_below(b);
      tot += (uint32_t)__popcll(b);
    }
    lane_base[i] = run + below;
    run += tot;
  }
  if (lane == 0) s_wtot[wv] = run;
  __syncthreads();
  uint32_t wb = 0, total = 0;
#pragma unroll
  for (int v = 0; v < W; ++v) {
    const uint32_t x = s_wtot[v];
    if (v < (int)wv) wb += x;
    total += x;
  }
  const size_t tix = (size_t)n * nc + c;
  if (total == 0) {
    if (tid == 0) { ch_off[tix] = 0; ch_cnt[tix] = 0; }
    return;
  }
  if (tid == 0) {
    const uint32_t r = c % regions;
    const uint32_t off = atomicAdd(&ctl[n].cursor[r], total);
    uint32_t b = kNoBound;
    if (off + total <= cap_r) b = r * cap_r + off;
    else ctl[n].overflow = 1;
    s_base = b;
  }
  __syncthreads();
  const uint32_t b = s_base;
  if (tid == 0) {
    ch_off[tix] = (b == kNoBound) ? 0 : b;
    ch_cnt[tix] = (b == kNoBound) ? 0 : total;
  }
  if (b == kNoBound || flags == 0) return;
  const size_t out = (size_t)n * cap_total + b + wb;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    uint32_t p = lane_base[i];
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

}  // namespace rtk
