// What sits around the round: the genie-aided global Top-k kernels, the mask-overlap count, the SGD update, and the fill / copy / state kernels.
#pragma once
#include "compact.h"

namespace rtk {

// ---------------------------------------------------------- global Top-k ----
// The genie-aided baseline (subsection "Statistical Global Top-k"): all workers
// share the mask of the k largest entries of abar = sum_n omega_n a_n.
//
// k_global_accum, grid (ceil(d/256)): a wave owns 256 entries (one group of four
// per lane) of all N rows.  For n = 0..N-1 it forms a_n = eps_n + g_n (eps taken
// as 0 where the previous mask bit is set), stores it over the state and adds
// omega_n * a_n to the entries of abar held in registers, in ascending worker
// order from +0 -- the order of the aggregation.  Sixteen rows are loaded at a
// time: the N row streams lie far apart in memory, and this kernel only nears
// the streaming rate of the chip with that many loads of a lane in flight
// (4 rows at a time: 895 us on the target workload, 8: 855 us, 16: 811 us).
constexpr int kGlobalRows = 16;
constexpr int kGlobalBlock = 64;

template <bool VEC, int kGlobalRows, int BT>
__global__ void __launch_bounds__(BT)
k_global_accum(float* __restrict__ e, const float* __restrict__ g, const uint32_t* __restrict__ mask,
               int64_t d, uint32_t nc, int32_t N, const float* __restrict__ omega, float* __restrict__ abar) {
  const int64_t j0 = (int64_t)blockIdx.x * (4 * BT) + (int64_t)threadIdx.x * 4;
  if (j0 >= d) return;
  const size_t row_words = (size_t)nc * kChunkWords;
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (VEC) {
    for (int32_t n0 = 0; n0 < N; n0 += kGlobalRows) {
      f32x4 ev[kGlobalRows], gv[kGlobalRows];
      uint32_t mb[kGlobalRows];
      float w[kGlobalRows];
#pragma unroll
      for (int u = 0; u < kGlobalRows; ++u) {
        const int32_t n = n0 + u;
        if (n < N) {
          const size_t row = (size_t)n * (size_t)d;
          mb[u] = (mask[(size_t)n * row_words + (size_t)(j0 >> 5)] >> (j0 & 31)) & 15u;
          ev[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(e + row + j0));
          gv[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g + row + j0));
          w[u] = omega[n];
        } else {
          mb[u] = 0; w[u] = 0.0f;
          ev[u] = f32x4{0.f, 0.f, 0.f, 0.f};
          gv[u] = ev[u];
        }
      }
#pragma unroll
      for (int u = 0; u < kGlobalRows; ++u) {
        const int32_t n = n0 + u;
        if (n < N) {
          f32x4 z = ev[u];
          if (mb[u] & 1u) z.x = 0.f;
          if (mb[u] & 2u) z.y = 0.f;
          if (mb[u] & 4u) z.z = 0.f;
          if (mb[u] & 8u) z.w = 0.f;
          const f32x4 a4 = z + gv[u];
          __builtin_nontemporal_store(a4, reinterpret_cast<f32x4*>(e + (size_t)n * (size_t)d + j0));
          acc[0] = __fadd_rn(acc[0], __fmul_rn(w[u], a4.x));
          acc[1] = __fadd_rn(acc[1], __fmul_rn(w[u], a4.y));
          acc[2] = __fadd_rn(acc[2], __fmul_rn(w[u], a4.z));
          acc[3] = __fadd_rn(acc[3], __fmul_rn(w[u], a4.w));
        }
      }
    }
    *reinterpret_cast<f32x4*>(abar + j0) = f32x4{acc[0], acc[1], acc[2], acc[3]};
  } else {
    for (int32_t n = 0; n < N; ++n) {
      const size_t row = (size_t)n * (size_t)d;
      const uint32_t mb = (mask[(size_t)n * row_words + (size_t)(j0 >> 5)] >> (j0 & 31)) & 15u;
      const float w = omega[n];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int64_t j = j0 + q;
        if (j < d) {
          const float eps = ((mb >> q) & 1u) ? 0.f : e[row + j];
          const float a = eps + g[row + j];
          e[row + j] = a;
          acc[q] = __fadd_rn(acc[q], __fmul_rn(w, a));
        }
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (j0 + q < d) abar[j0 + q] = acc[q];
  }
}

// k_global_apply gives every worker the shared selection sidx [k] (ascending;
// chunk c holds positions ssel_off[c] .. ssel_off[c+1]) with shared mask words
// smask.  grid (A + B, N) with A = ceil(k/256), B = ceil(nc/4):
//   blocks x < A : a thread per selected entry p -- the index row and the
//                  worker's own value a_n[sidx[p]] gathered from its state;
//   blocks x >= A: a wave per chunk -- chunk offsets and mask words (chunks
//                  that were and stay empty keep their zero words).
__global__ void __launch_bounds__(kBlock)
k_global_apply(const float* __restrict__ e, const int32_t* __restrict__ sidx,
               const uint32_t* __restrict__ ssel_off, const uint32_t* __restrict__ smask,
               const uint32_t* __restrict__ prev_sel_off, int32_t* __restrict__ out_idx,
               float* __restrict__ out_val, uint32_t* __restrict__ sel_off, uint32_t* __restrict__ mask,
               int64_t d, int64_t k, uint32_t nc, uint32_t entry_blocks) {
  const uint32_t n = blockIdx.y;
  if (blockIdx.x < entry_blocks) {
    const int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (p < k) {
      const int32_t j = sidx[p];
      out_idx[(size_t)n * k + p] = j;
      out_val[(size_t)n * k + p] = e[(size_t)n * (size_t)d + (size_t)j];
    }
    return;
  }
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t c = (blockIdx.x - entry_blocks) * 4 + (threadIdx.x >> 6);
  if (c >= nc) return;
  const uint32_t p0 = ssel_off[c], p1 = ssel_off[c + 1];
  const size_t so = (size_t)n * (nc + 1) + c;
  const bool was_empty = prev_sel_off[so + 1] == prev_sel_off[so];
  if (lane == 0) {
    sel_off[so] = p0;
    if (c == nc - 1) sel_off[so + 1] = p1;
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
    c.tau_lo = kNoBound; c.tau_lo_mag = kNoBound; c.next_tau_lo = kNoBound; c.next_tau_lo_mag = kNoBound; c.win_lo = kNoBound; c.next_win_lo = kNoBound;
    c.tau_prev = kNoBound; c.centre = kNoBound; c.pred_x = kNoBound; c.margin_scale = 1.0f;
  }
}

// set_state: the state keeps, at the entries sent in the previous round, the
// value that was sent (the sweep reads it from there and restarts the error at
// zero): state[n][pidx[n][i]] = pval[n][i].  Indices outside [0,d) are skipped
// (k_check_ascending reports them).
__global__ void k_scatter_prev(float* __restrict__ e, const int32_t* __restrict__ pidx,
                               const float* __restrict__ pval, int64_t d, int64_t k,
                               const uint32_t* __restrict__ kn, int32_t N) {
  const size_t total = (size_t)N * (size_t)k;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const size_t n = i / (size_t)k;
    if (i - n * (size_t)k >= kn[n]) continue;        // beyond the worker's own list length
    const int64_t j = pidx[i];
    if (j >= 0 && j < d) e[n * (size_t)d + (size_t)j] = pval[i];
  }
}

// set_state: mask words and per-chunk offsets from an ascending index list.
// grid (ceil(nc/4), N): one wave per chunk.
__global__ void __launch_bounds__(kBlock)
k_build_mask(const int32_t* __restrict__ pidx, uint32_t* __restrict__ mask,
             uint32_t* __restrict__ sel_off, int64_t k, const uint32_t* __restrict__ kn, uint32_t nc) {
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
    const int64_t len = (int64_t)kn[n];               // the worker's own list length
    int64_t lo = 0, hi = len;
    while (lo < hi) { const int64_t mid = (lo + hi) >> 1; if ((int64_t)pi[mid] < t0) lo = mid + 1; else hi = mid; }
    first = (uint32_t)lo;
    if (lane == 0) {
      sel_off[(size_t)n * (nc + 1) + c] = first;
      if (c == nc - 1) sel_off[(size_t)n * (nc + 1) + nc] = (uint32_t)len;
    }
    for (int64_t p = lo + lane; p < len; p += 64) {
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
__global__ void k_check_ascending(const int32_t* __restrict__ pidx, WorkerCtl* ctl, int64_t d, int64_t k,
                                  const uint32_t* __restrict__ kn) {
  const uint32_t n = blockIdx.y;
  const int32_t* pi = pidx + (size_t)n * k;
  const int64_t len = (int64_t)kn[n];
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < len; i += (int64_t)gridDim.x * blockDim.x) {
    const int32_t v = pi[i];
    if (v < 0 || (int64_t)v >= d || (i > 0 && pi[i - 1] >= v)) atomicOr(&ctl[n].err, 2u);
  }
}

__global__ void k_tanh(const float* __restrict__ x, float* __restrict__ y, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    y[i] = tanh_f32_cr(x[i]);
}

__global__ void k_pow(const float* __restrict__ x, float y, float* __restrict__ out, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    out[i] = pow_f32_cr(x[i], y);
}

__global__ void k_erf(const float* __restrict__ x, float* __restrict__ y, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    y[i] = erf_f32_cr(x[i]);
}

}  // namespace rtk
