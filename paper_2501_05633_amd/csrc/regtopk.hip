// C ABI of the RegTop-k round (see include/regtopk.h): context, arena layout
// and the kernel sequence of one round.  Host code only enqueues; the only
// host synchronisation is in regtopk_get_stats.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/regtopk.h"
#include "kernels.h"

using namespace rtk;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                   \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess)                                                               \
      return fail(REGTOPK_HIP_ERROR, "%s failed: %s", #expr, hipGetErrorString(e_));    \
  } while (0)

// Work of a context is enqueued on the device it was created on: the calling
// thread's current device must be that one (its memory is not another device's).
#define DEVICE_TRY(c)                                                                    \
  do {                                                                                  \
    int dev_ = -1;                                                                      \
    HIP_TRY(hipGetDevice(&dev_));                                                       \
    if (dev_ != (c)->device)                                                            \
      return fail(REGTOPK_INVALID_ARG, "the context lives on device %d, the current device is %d", (c)->device, dev_); \
  } while (0)

constexpr size_t kAlign = 256;
size_t up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// The dense-selection kernel synchronises its blocks with grid barriers, so all
// of them must be resident together.  Two such kernels that run at the same
// time on one device (two contexts driven on two streams) could each be partly
// resident and wait for each other, so the library keeps them apart: while more
// than one context lives on a device, every launch of that kernel first waits
// for the previous one of any other stream (an event per device, re-recorded
// after each launch).  A lone context pays nothing.
constexpr int kMaxDevices = 64;
struct DeviceGate {
  std::mutex m;
  int live = 0;                 // user contexts alive on the device
  hipEvent_t ev = nullptr;      // recorded after the last dense-selection launch
  hipStream_t last = nullptr;   // its stream
  bool recorded = false;
};
DeviceGate g_gate[kMaxDevices];

// Scratch of regtopk_mask_overlap_static: per-block histograms of the overlap
// count, kStaticOverlapBlocks rows of kOverlapBins words (4 MiB).  Every GPU
// holds its own copy of the array until the process ends.  In host code the
// name `g_overlap_scratch` is only a handle for hipGetSymbolAddress; the
// address the kernels get is looked up once per device and kept in
// g_overlap_ptr.
constexpr uint32_t kStaticOverlapBlocks = 1024;
static __device__ __align__(256) uint32_t g_overlap_scratch[kStaticOverlapBlocks * kOverlapBins];
std::mutex g_overlap_mutex;
uint32_t* g_overlap_ptr[kMaxDevices] = {};

struct Layout {
  uint32_t nc, regions, cap_r, cap_total, bnd_cap;
  size_t e, out_idx[2], out_val[2], agg[2], cand_idx, cand_val, cand_key;
  size_t ch_off, ch_cnt, ch_gt, ch_tie, tie_off, sel_off[2], agg_hot[2], mask, cand_prev, bnd_key, fhist, ctl, gctl, omega, kn, blk_gt, blk_tie, total;
};

bool valid_sizes(int32_t N, int64_t d, int64_t k) {
  return N >= 1 && N <= 65535 && d >= 1 && d < ((int64_t)1 << 31) && k >= 1 && k <= d;
}

// Lays the arena out.  Every capacity is computed in 64 bits and checked before
// it is narrowed; returns false (and leaves L.total at 0) when a piece would not
// fit the 32-bit slot numbers the kernels use.
bool make_layout(int32_t N, int64_t d, int64_t k, Layout* out) {
  Layout L{};
  *out = L;
  if (!valid_sizes(N, d, k)) return false;
  const uint64_t nc = (uint64_t)((d + kChunk - 1) / kChunk);
  uint64_t R = nc / 64;
  if (R < 1) R = 1;
  if (R > 32) R = 32;
  // Room for 4k candidates in total (the dense selection needs min(2k,d)),
  // with a quarter of slack per region for uneven chunk populations -- but never
  // more than the region's chunks hold entries (chunk c feeds region c % R),
  // which no sweep can exceed.
  uint64_t want = (uint64_t)4 * (uint64_t)k;
  if (want < 1024) want = 1024;
  uint64_t per = (want + R - 1) / R;
  if (R > 1) per += per / 4;
  per = (per + 63) / 64 * 64;
  const uint64_t region_max = (nc + R - 1) / R * (uint64_t)kChunk;
  if (per > region_max) per = region_max;
  const uint64_t cap_total = per * R;
  const uint64_t need_dense = (uint64_t)(2 * k < d ? 2 * k : d);
  if (cap_total > 0xFFFFFFFFull || cap_total < need_dense) return false;
  L.nc = (uint32_t)nc;
  L.regions = (uint32_t)R;
  L.cap_r = (uint32_t)per;
  L.cap_total = (uint32_t)cap_total;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += up(bytes); return at; };
  const size_t nd = (size_t)N * (size_t)d, nk = (size_t)N * (size_t)k;
  const size_t ncand = (size_t)N * L.cap_total, nch = (size_t)N * L.nc;
  L.e = take(nd * 4);
  for (int b = 0; b < 2; ++b) { L.out_idx[b] = take(nk * 4); L.out_val[b] = take(nk * 4); L.agg[b] = take((size_t)d * 4); }
  L.cand_idx = take(ncand * 4);
  L.cand_val = take(ncand * 4);
  L.cand_key = take(ncand * 4);
  L.cand_prev = take(ncand * 4);
  L.ch_off = take(nch * 4);
  L.ch_cnt = take(nch * 4);
  L.ch_gt = take(nch * 4);
  L.ch_tie = take(nch * 4);
  L.tie_off = take(nch * 4);
  for (int b = 0; b < 2; ++b) { L.sel_off[b] = take(((size_t)N * (L.nc + 1)) * 4); L.agg_hot[b] = take((size_t)L.nc * 4); }
  L.mask = take(nch * kChunkWords * 4);
  // the boundary list never holds more than the candidate list does
  L.bnd_cap = L.cap_total < 262144u ? L.cap_total : 262144u;
  L.bnd_key = take((size_t)N * L.bnd_cap * 4);
  L.fhist = take((size_t)N * 3 * kL1Bins * 4);
  L.ctl = take((size_t)N * sizeof(WorkerCtl));
  L.gctl = take(sizeof(GlobalCtl));
  L.omega = take((size_t)N * 4);
  L.kn = take((size_t)N * 4);
  const size_t nblk = (size_t)N * ((L.nc + kChunksPerBlock - 1) / kChunksPerBlock);
  L.blk_gt = take(nblk * 4);
  L.blk_tie = take(nblk * 4);
  L.total = o;
  *out = L;
  return true;
}

}  // namespace

constexpr int kProfRounds = 64;
constexpr int kFreshRounds = 3;      // rounds that sample their bound after a start without history

struct regtopk_ctx {
  int32_t N;
  int64_t d, k;
  float mu;
  int64_t t;
  bool have_prev;       // a previous mask exists (round >= 1 or set_state with t >= 1)
  int fresh;            // rounds still to take their bound from a sample: no (reliable) bound is carried over yet
  bool owns_arena;
  int device;
  int dense_blocks;     // grid of the dense-selection kernel: all blocks resident together
  int force_dense;
  int prior_roots;      // prior's code: 0..3 square roots, or negative for a general exponent (prior_of)
  int likelihood;       // 0 tanh, 1 clipped linear
  bool reinit_ctl;      // the score space changed: drop the bounds carried over from earlier rounds
  bool need_begin;      // the control blocks are not prepared for the next round (k_begin must run)
  float cand_target;
  int profile;                  // 0 off, 1 record the stage events in every step, 2 only those around the sweep
  int ev_level[kProfRounds];    // level at which a round of the ring was recorded
  hipEvent_t ev[kProfRounds][5];
  int64_t prof_rounds;          // steps recorded since profiling was switched on
  uint32_t* host_err;   // pinned host word the dense-selection kernel sets when it abandons a round
  bool uniform_k;       // every worker keeps k entries (no regtopk_set_worker_k with other values)
  bool internal;        // the selector of a global Top-k round: always driven on its owner's stream
  regtopk_ctx* gsel;    // global Top-k: a one-row context that selects over the unsparsified aggregate
  char* arena;
  Layout L;
  template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(arena + off); }
};

namespace {

int zero_state(regtopk_ctx* c, hipStream_t s) {
  const size_t ne = (size_t)c->N * (size_t)c->d;
  k_fill_u32<<<2048, 256, 0, s>>>(c->at<uint32_t>(c->L.e), ne, 0u);
  for (int b = 0; b < 2; ++b) {
    k_fill_u32<<<256, 256, 0, s>>>(c->at<uint32_t>(c->L.sel_off[b]), (size_t)c->N * (c->L.nc + 1), 0u);
    k_fill_u32<<<64, 256, 0, s>>>(c->at<uint32_t>(c->L.agg_hot[b]), (size_t)c->L.nc, 0u);
    k_fill_u32<<<1024, 256, 0, s>>>(c->at<uint32_t>(c->L.agg[b]), (size_t)c->d, 0u);     // agg_hot == 0 means zeros
  }
  k_fill_u32<<<1024, 256, 0, s>>>(c->at<uint32_t>(c->L.mask), (size_t)c->N * c->L.nc * kChunkWords, 0u);
  k_init_ctl<<<c->N, 256, 0, s>>>(c->at<WorkerCtl>(c->L.ctl));
  k_fill_u32<<<1, 64, 0, s>>>(c->at<uint32_t>(c->L.gctl), sizeof(GlobalCtl) / 4, 0u);
  k_fill_u32<<<1, 64, 0, s>>>(c->host_err, 1, 0u);      // (pinned host memory, cleared in stream order)
  HIP_TRY(hipGetLastError());
  c->t = 0;
  c->have_prev = false;
  c->fresh = kFreshRounds;
  c->need_begin = true;
  return REGTOPK_OK;
}

// Removes a context from its device's count of live contexts.
void gate_leave(regtopk_ctx* c) {
  if (c->internal || c->device < 0 || c->device >= kMaxDevices) return;
  DeviceGate& g = g_gate[c->device];
  std::lock_guard<std::mutex> lock(g.m);
  g.live -= 1;
}

int create_common(regtopk_ctx** out, int32_t N, int64_t d, int64_t k, float mu, void* arena,
                  size_t bytes, bool owns, hipStream_t s, bool internal = false) {
  regtopk_ctx* c = new (std::nothrow) regtopk_ctx;
  if (!c) return fail(REGTOPK_NO_MEMORY, "out of host memory");
  c->internal = internal;
  c->host_err = nullptr;
  c->N = N; c->d = d; c->k = k; c->mu = mu;
  c->owns_arena = owns;
  c->force_dense = 0;
  c->prior_roots = 0;
  c->likelihood = 0;
  c->reinit_ctl = false;
  c->gsel = nullptr;
  c->cand_target = 1.25f;
  c->profile = 0;
  c->prof_rounds = 0;
  c->arena = static_cast<char*>(arena);
  if (!make_layout(N, d, k, &c->L) || bytes < c->L.total) { delete c; return fail(REGTOPK_INVALID_ARG, "sizes have no valid layout"); }
  if (hipGetDevice(&c->device) != hipSuccess) { delete c; return fail(REGTOPK_HIP_ERROR, "hipGetDevice failed"); }
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess || cus < 1) {
    delete c;
    return fail(REGTOPK_HIP_ERROR, "cannot query the number of compute units");
  }
  // All blocks of the dense-selection kernel must be resident together (it
  // synchronises them with grid barriers): stay one block per compute unit below
  // what the occupancy calculator allows, at most 3 per unit.
  int per_cu = 0, per_cu_scalar = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_dense_all<true>, kBlock, 0) != hipSuccess || per_cu < 1 ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_scalar, k_dense_all<false>, kBlock, 0) != hipSuccess || per_cu_scalar < 1) {
    delete c;
    return fail(REGTOPK_HIP_ERROR, "cannot query the occupancy of the dense-selection kernel");
  }
  if (per_cu_scalar < per_cu) per_cu = per_cu_scalar;       // either instantiation may be the one launched
  per_cu = per_cu - 1 < 1 ? 1 : (per_cu - 1 > 3 ? 3 : per_cu - 1);
  c->dense_blocks = per_cu * cus;
  if (c->device >= kMaxDevices) { delete c; return fail(REGTOPK_INVALID_ARG, "device index %d not supported", c->device); }
  // one word of pinned host memory through which an abandoned dense selection reaches the next step
  void* hp = nullptr;
  if (hipHostMalloc(&hp, 64, hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    delete c;
    return fail(REGTOPK_NO_MEMORY, "hipHostMalloc of the error word failed");
  }
  c->host_err = static_cast<uint32_t*>(hp);
  *c->host_err = 0;
  if (!internal) {
    // from the second live context on, dense-selection launches are chained by the device's event;
    // the launches made so far were not recorded, so let them finish first
    DeviceGate& g = g_gate[c->device];
    std::lock_guard<std::mutex> lock(g.m);
    if (g.live >= 1) {
      if (!g.ev && hipEventCreateWithFlags(&g.ev, hipEventDisableTiming) != hipSuccess) {
        (void)hipHostFree(hp);
        delete c;
        return fail(REGTOPK_HIP_ERROR, "hipEventCreateWithFlags failed");
      }
      if (hipDeviceSynchronize() != hipSuccess) {
        (void)hipHostFree(hp);
        delete c;
        return fail(REGTOPK_HIP_ERROR, "hipDeviceSynchronize failed");
      }
      g.recorded = false;
    }
    g.live += 1;
  }
  k_fill_u32<<<1, 256, 0, s>>>(c->at<uint32_t>(c->L.omega), (size_t)N, __builtin_bit_cast(uint32_t, 1.0f / (float)N));
  k_fill_u32<<<1, 256, 0, s>>>(c->at<uint32_t>(c->L.kn), (size_t)N, (uint32_t)k);
  c->uniform_k = true;
  int rc = zero_state(c, s);
  if (rc == REGTOPK_OK && hipStreamSynchronize(s) != hipSuccess) rc = fail(REGTOPK_HIP_ERROR, "zeroing the state failed");
  if (rc != REGTOPK_OK) { gate_leave(c); (void)hipHostFree(c->host_err); delete c; return rc; }
  *out = c;
  return REGTOPK_OK;
}

int check_create_args(regtopk_ctx** out, int32_t N, int64_t d, int64_t k, float mu) {
  if (!out) return fail(REGTOPK_INVALID_ARG, "out is NULL");
  if (!valid_sizes(N, d, k))
    return fail(REGTOPK_INVALID_ARG, "need 1 <= N <= 65535, 1 <= d < 2^31, 1 <= k <= d (N=%d d=%lld k=%lld)", N,
                (long long)d, (long long)k);
  if (!(mu >= 0.0f) || std::isinf(mu)) return fail(REGTOPK_INVALID_ARG, "mu must be finite and >= 0");
  return REGTOPK_OK;
}

}  // namespace

extern "C" {

const char* regtopk_last_error(void) { return g_err; }

size_t regtopk_workspace_bytes(int32_t N, int64_t d, int64_t k) {
  Layout L;
  return make_layout(N, d, k, &L) ? L.total : 0;
}

int regtopk_create(regtopk_ctx** out, int32_t N, int64_t d, int64_t k, float mu) {
  int rc = check_create_args(out, N, d, k, mu);
  if (rc) return rc;
  Layout L;
  if (!make_layout(N, d, k, &L)) return fail(REGTOPK_INVALID_ARG, "sizes have no valid layout");
  const size_t bytes = L.total;
  void* p = nullptr;
  if (hipMalloc(&p, bytes) != hipSuccess) {
    (void)hipGetLastError();
    return fail(REGTOPK_NO_MEMORY, "hipMalloc of %zu bytes failed", bytes);
  }
  rc = create_common(out, N, d, k, mu, p, bytes, true, nullptr);
  if (rc) (void)hipFree(p);
  return rc;
}

int regtopk_create_in(regtopk_ctx** out, int32_t N, int64_t d, int64_t k, float mu, void* arena_dev,
                      size_t arena_bytes, void* stream) {
  int rc = check_create_args(out, N, d, k, mu);
  if (rc) return rc;
  if (!arena_dev) return fail(REGTOPK_INVALID_ARG, "arena_dev is NULL");
  if (reinterpret_cast<uintptr_t>(arena_dev) % kAlign) return fail(REGTOPK_INVALID_ARG, "arena_dev must be 256-byte aligned");
  Layout L;
  if (!make_layout(N, d, k, &L)) return fail(REGTOPK_INVALID_ARG, "sizes have no valid layout");
  const size_t need = L.total;
  if (arena_bytes < need) return fail(REGTOPK_NO_MEMORY, "arena has %zu bytes, %zu needed", arena_bytes, need);
  return create_common(out, N, d, k, mu, arena_dev, arena_bytes, false, static_cast<hipStream_t>(stream));
}

int regtopk_destroy(regtopk_ctx* c) {
  if (!c) return fail(REGTOPK_INVALID_ARG, "ctx is NULL");
  int rc = REGTOPK_OK;
  if (c->profile)
    for (auto& row : c->ev) for (auto& e : row) (void)hipEventDestroy(e);
  if (c->gsel && regtopk_destroy(c->gsel) != REGTOPK_OK) rc = REGTOPK_HIP_ERROR;
  if (c->owns_arena && hipFree(c->arena) != hipSuccess) rc = fail(REGTOPK_HIP_ERROR, "hipFree failed");
  if (c->host_err && hipHostFree(c->host_err) != hipSuccess) rc = fail(REGTOPK_HIP_ERROR, "hipHostFree failed");
  gate_leave(c);
  delete c;
  return rc;
}

int regtopk_reset(regtopk_ctx* c, void* stream) {
  if (!c) return fail(REGTOPK_INVALID_ARG, "ctx is NULL");
  DEVICE_TRY(c);
  return zero_state(c, static_cast<hipStream_t>(stream));
}

int regtopk_set_option(regtopk_ctx* c, int option, double value) {
  if (!c) return fail(REGTOPK_INVALID_ARG, "ctx is NULL");
  switch (option) {
    case REGTOPK_OPT_FORCE_DENSE:
      if ((value != 0.0) != (c->force_dense != 0)) c->need_begin = true;
      c->force_dense = value != 0.0;
      return REGTOPK_OK;
    case REGTOPK_OPT_CAND_TARGET:
      if (!(value > 1.0 && value <= 3.0)) return fail(REGTOPK_INVALID_ARG, "candidate target must be in (1, 3]");
      c->cand_target = (float)value;
      return REGTOPK_OK;
    case REGTOPK_OPT_PRIOR_ROOTS:
      if (!(value == 0.0 || value == 1.0 || value == 2.0 || value == 3.0))
        return fail(REGTOPK_INVALID_ARG, "prior roots must be 0, 1, 2 or 3");
      if ((int)value != c->prior_roots) { c->prior_roots = (int)value; c->reinit_ctl = true; c->fresh = kFreshRounds; }
      return REGTOPK_OK;
    case REGTOPK_OPT_PRIOR_EXPONENT: {
      const float y = (float)value;
      if (!(y > 0.0f && y <= 1.0f)) return fail(REGTOPK_INVALID_ARG, "prior exponent must be in (0, 1]");
      const int code = y == 1.0f ? 0 : prior_code_of_exponent(y);
      if (code != c->prior_roots) { c->prior_roots = code; c->reinit_ctl = true; c->fresh = kFreshRounds; }
      return REGTOPK_OK;
    }
    case REGTOPK_OPT_LIKELIHOOD:
      if (!(value == 0.0 || value == 1.0 || value == 2.0))
        return fail(REGTOPK_INVALID_ARG, "likelihood must be 0 (tanh), 1 (clipped linear) or 2 (erf)");
      if ((int)value != c->likelihood) { c->likelihood = (int)value; c->reinit_ctl = true; c->fresh = kFreshRounds; }
      return REGTOPK_OK;
    case REGTOPK_OPT_PROFILE:
      if (!(value == 0.0 || value == 1.0 || value == 2.0)) return fail(REGTOPK_INVALID_ARG, "profile level must be 0, 1 or 2");
      if (value != 0.0 && !c->profile) {
        // timing only: without the system-scope fence an event otherwise carries (a write-back and
        // invalidation of the caches, which the kernels after it pay for)
        for (auto& row : c->ev) for (auto& e : row) HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableSystemFence));
      }
      if (value == 0.0 && c->profile) {
        for (auto& row : c->ev) for (auto& e : row) (void)hipEventDestroy(e);
      }
      c->profile = (int)value;
      c->prof_rounds = 0;
      return REGTOPK_OK;
    default: return fail(REGTOPK_INVALID_ARG, "unknown option %d", option);
  }
}

}  // extern "C"

namespace {

// One round; G is the element type of the local gradients.  pre: the state
// already holds the accumulated values (the selector of a global Top-k round),
// grads is not read.
template <typename G>
int step_impl(regtopk_ctx* c, const G* grads, const float* gprev, void* stream, regtopk_result* out, bool pre = false) {
  if (!c || (!grads && !pre) || !out) return fail(REGTOPK_INVALID_ARG, "ctx, grads_dev and out must not be NULL");
  DEVICE_TRY(c);
  if (*static_cast<volatile uint32_t*>(c->host_err) != 0)
    return fail(REGTOPK_BAD_STATE, "an earlier round abandoned its dense selection (its blocks were not resident "
                                   "together); the state is undefined until regtopk_reset or regtopk_set_state");
  const int use_reg = (c->have_prev && c->mu > 0.0f) ? 1 : 0;
  if (use_reg && !gprev) return fail(REGTOPK_INVALID_ARG, "prev_aggregate_dev is required after round 0 when mu > 0");
  if (reinterpret_cast<uintptr_t>(grads) % sizeof(G) || reinterpret_cast<uintptr_t>(gprev) % 4)
    return fail(REGTOPK_INVALID_ARG, "device pointers must be aligned to their element type");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Layout& L = c->L;
  const int32_t N = c->N;
  const int64_t d = c->d, k = c->k;
  const uint32_t nc = L.nc;
  const int cur = (int)(c->t & 1), prv = cur ^ 1;
  const bool vec = (d % 4 == 0) && (pre || reinterpret_cast<uintptr_t>(grads) % (4 * sizeof(G)) == 0);

  WorkerCtl* ctl = c->at<WorkerCtl>(L.ctl);
  GlobalCtl* gctl = c->at<GlobalCtl>(L.gctl);
  float* e = c->at<float>(L.e);
  int32_t* cand_idx = c->at<int32_t>(L.cand_idx);
  float* cand_val = c->at<float>(L.cand_val);
  uint32_t* cand_key = c->at<uint32_t>(L.cand_key);
  uint32_t* ch_off = c->at<uint32_t>(L.ch_off);
  uint32_t* ch_cnt = c->at<uint32_t>(L.ch_cnt);
  uint32_t* ch_gt = c->at<uint32_t>(L.ch_gt);
  uint32_t* ch_tie = c->at<uint32_t>(L.ch_tie);
  uint32_t* tie_off = c->at<uint32_t>(L.tie_off);
  uint32_t* bnd_key = c->at<uint32_t>(L.bnd_key);
  uint32_t* fhist = c->at<uint32_t>(L.fhist);
  int32_t* out_idx = c->at<int32_t>(L.out_idx[cur]);
  float* out_val = c->at<float>(L.out_val[cur]);
  float* agg = c->at<float>(L.agg[cur]);
  const float* prev_val = c->at<float>(L.out_val[prv]);
  uint32_t* sel_off = c->at<uint32_t>(L.sel_off[cur]);
  const uint32_t* prev_sel_off = c->at<uint32_t>(L.sel_off[prv]);
  uint32_t* agg_hot = c->at<uint32_t>(L.agg_hot[cur]);
  uint32_t* mask = c->at<uint32_t>(L.mask);
  float* cand_prev = c->at<float>(L.cand_prev);
  const float* omega = c->at<float>(L.omega);
  const uint32_t* kn = c->at<uint32_t>(L.kn);

  const dim3 g_chunks(nc, N), g_waves((nc + 3) / 4, N);
  const dim3 g_score((L.cap_r + kScoreSlots - 1) / kScoreSlots, L.regions, N);
  hipEvent_t* ev = c->profile ? c->ev[c->prof_rounds % kProfRounds] : nullptr;
  const bool ev_all = c->profile == 1;              // else only ev[0], ev[1] around the sweep
  if (ev) c->ev_level[c->prof_rounds % kProfRounds] = c->profile;
  if (ev && ev_all) HIP_TRY(hipEventRecord(ev[4], s));
  const ScoreKind sk{c->prior_roots, c->likelihood};
  if (c->reinit_ctl) {
    k_init_ctl<<<N, 256, 0, s>>>(ctl);
    c->reinit_ctl = false;
    c->need_begin = true;
  }
  if (c->need_begin) {          // otherwise the last kernel of the previous round has done this
    k_begin<<<N, kBlock, 0, s>>>(ctl, gctl, c->force_dense);
    c->need_begin = false;
  }
  if (c->fresh > 0 && !c->force_dense) {
    // No bound from a previous round, or only the guess of a controller that has
    // not seen two rounds yet (from an empty error state the k-th score grows by
    // up to a factor of two in the second round and 3/2 in the third): take the
    // bound from a strided sample of a = eps + g.
    const uint64_t lines_all = (uint64_t)((d + 31) / 32);
    const uint32_t n_lines = (uint32_t)(lines_all < kSampleMax / 32 ? lines_all : kSampleMax / 32);
    const uint32_t line_stride = (uint32_t)(lines_all / n_lines);
    const uint32_t n_groups = n_lines * 8;
    // every sample line is whole except, possibly, the last line of the row
    const uint64_t last_start = (uint64_t)(n_lines - 1) * line_stride * 32;
    const uint64_t last_len = (uint64_t)d - last_start < 32 ? (uint64_t)d - last_start : 32;
    const uint64_t n_sampled = (uint64_t)(n_lines - 1) * 32 + last_len;
    k_fill_u32<<<64, 256, 0, s>>>(fhist, (size_t)N * 3 * kL1Bins, 0u);
    // a bounded number of blocks per worker: every block ends with one global add per occupied histogram
    // bin, and adds of many blocks to the same few words queue up (about 12 ns each)
    uint32_t sample_blocks = (n_groups + 4 * kBlock - 1) / (4 * kBlock);
    if (sample_blocks > 64) sample_blocks = 64;
    if (pre) k_sample_hist_state<<<dim3(sample_blocks, N), kBlock, 0, s>>>(e, d, fhist, n_groups, line_stride, sk.roots);
    else if (sk.roots == 0) k_sample_hist<G, true><<<dim3(sample_blocks, N), kBlock, 0, s>>>(e, grads, mask, d, nc, fhist, n_groups, line_stride, 0);
    else k_sample_hist<G, false><<<dim3(sample_blocks, N), kBlock, 0, s>>>(e, grads, mask, d, nc, fhist, n_groups, line_stride, sk.roots);
    k_sample_bound<<<N, kScanBlock, 0, s>>>(ctl, fhist, d, kn, (uint32_t)n_sampled, sk.roots);
  }
  if (c->fresh > 0) c->fresh -= 1;
  // The dominant kernel carries its two events in its own dispatch (start and stop time of the
  // kernel itself); events recorded around it would each keep the next kernel from starting back
  // to back.  The other forms of the sweep are timed by recorded events.
  const bool ev_in_launch = ev && !pre && vec;
  if (ev && !ev_in_launch) HIP_TRY(hipEventRecord(ev[0], s));
  if (pre && vec)
    k_emit_only<true><<<g_chunks, kBlock, 0, s>>>(e, d, ctl, cand_idx, cand_val, cand_prev, ch_off, ch_cnt, nc, L.cap_r, L.cap_total, L.regions);
  else if (pre)
    k_emit_only<false><<<g_chunks, kBlock, 0, s>>>(e, d, ctl, cand_idx, cand_val, cand_prev, ch_off, ch_cnt, nc, L.cap_r, L.cap_total, L.regions);
  else if (vec && ev_in_launch)
    hipExtLaunchKernelGGL((k_accum_emit_vec<G, kSweepNI>), g_chunks, dim3(1024 / kSweepNI), 0, s, ev[0], ev[1], 0,
                          e, grads, static_cast<const uint32_t*>(mask), d, ctl, cand_idx, cand_val, cand_prev, ch_off, ch_cnt, nc, L.cap_r, L.cap_total, L.regions);
  else if (vec)
    k_accum_emit_vec<G, kSweepNI><<<g_chunks, 1024 / kSweepNI, 0, s>>>(e, grads, mask, d, ctl, cand_idx, cand_val, cand_prev, ch_off, ch_cnt, nc, L.cap_r, L.cap_total, L.regions);
  else
    k_accum_emit<G><<<g_chunks, kBlock, 0, s>>>(e, grads, mask, d, ctl, cand_idx, cand_val, cand_prev, ch_off, ch_cnt, nc, L.cap_r, L.cap_total, L.regions);
  if (ev && !ev_in_launch) HIP_TRY(hipEventRecord(ev[1], s));
  if (sk.roots == 0 && sk.likelihood == 0)
    k_score<false><<<g_score, kBlock, 0, s>>>(ctl, cand_idx, cand_val, cand_prev, cand_key, bnd_key, gprev, d, L.cap_r, L.cap_total, L.bnd_cap, omega, c->mu, use_reg, sk);
  else
    k_score<true><<<g_score, kBlock, 0, s>>>(ctl, cand_idx, cand_val, cand_prev, cand_key, bnd_key, gprev, d, L.cap_r, L.cap_total, L.bnd_cap, omega, c->mu, use_reg, sk);
  k_select<<<N, kScanBlock, 0, s>>>(ctl, gctl, cand_key, bnd_key, kn, L.cap_r, L.cap_total, L.regions, L.bnd_cap, c->cand_target, c->force_dense, sk.roots, fhist);
  // dense selection for the workers whose speculation failed; returns at once if there is none
  {
    DeviceGate* gate = c->internal ? nullptr : &g_gate[c->device];
    std::unique_lock<std::mutex> lock;
    bool chain = false;
    if (gate) {
      lock = std::unique_lock<std::mutex>(gate->m);
      chain = gate->live > 1;
      if (chain && gate->recorded && gate->last != s) HIP_TRY(hipStreamWaitEvent(s, gate->ev, 0));
    }
    if (vec)
      k_dense_all<true><<<c->dense_blocks, kBlock, 0, s>>>(e, mask, prev_sel_off, d, ctl, gctl, fhist, ch_gt, ch_tie, ch_off, ch_cnt, tie_off, cand_idx, cand_val, cand_prev, cand_key, bnd_key, prev_val, gprev, k, kn, nc, N, L.cap_r, L.cap_total, L.regions, L.bnd_cap, omega, c->mu, use_reg, c->cand_target, sk, c->host_err);
    else
      k_dense_all<false><<<c->dense_blocks, kBlock, 0, s>>>(e, mask, prev_sel_off, d, ctl, gctl, fhist, ch_gt, ch_tie, ch_off, ch_cnt, tie_off, cand_idx, cand_val, cand_prev, cand_key, bnd_key, prev_val, gprev, k, kn, nc, N, L.cap_r, L.cap_total, L.regions, L.bnd_cap, omega, c->mu, use_reg, c->cand_target, sk, c->host_err);
    if (chain) {
      HIP_TRY(hipEventRecord(gate->ev, s));
      gate->last = s;
      gate->recorded = true;
    }
  }

  // ordered compaction, error update, aggregation
  if (ev && ev_all) HIP_TRY(hipEventRecord(ev[2], s));
  const uint32_t n_blk = (nc + kChunksPerBlock - 1) / kChunksPerBlock;
  const dim3 g_groups(n_blk, N);
  uint32_t* blk_gt = c->at<uint32_t>(L.blk_gt);
  uint32_t* blk_tie = c->at<uint32_t>(L.blk_tie);
  k_chunk_count<<<g_groups, kBlock, 0, s>>>(ctl, cand_key, ch_off, ch_cnt, ch_gt, ch_tie, blk_gt, blk_tie, nc, L.cap_total);
  constexpr uint32_t kCompactPerBlock = (kBlock / 64) * (64 / kCompactLanes);
  k_compact<kCompactLanes><<<dim3((nc + kCompactPerBlock - 1) / kCompactPerBlock, N), kBlock, 0, s>>>(
      ctl, gctl, cand_key, cand_idx, cand_val, ch_off, ch_cnt, ch_gt, ch_tie, blk_gt, blk_tie, n_blk, sel_off, prev_sel_off,
      out_idx, out_val, mask, k, kn, nc, L.cap_total, c->force_dense);
  k_aggregate<<<nc, kBlock, 0, s>>>(out_idx, out_val, sel_off, agg, agg_hot, d, k, nc, N, omega);
  if (ev && ev_all) HIP_TRY(hipEventRecord(ev[3], s));
  if (ev) c->prof_rounds += 1;
  HIP_TRY(hipGetLastError());

  c->t += 1;
  c->have_prev = true;
  out->idx = out_idx;
  out->val = out_val;
  out->agg = agg;
  return REGTOPK_OK;
}

}  // namespace

extern "C" {

int regtopk_step(regtopk_ctx* c, const float* grads, const float* gprev, void* stream, regtopk_result* out) {
  return step_impl<float>(c, grads, gprev, stream, out);
}

// Makes the selector of the global Top-k rounds (one row of d entries, plain
// Top-k) in `mem`.
static int bind_global_impl(regtopk_ctx* c, void* mem, size_t bytes, bool owned, hipStream_t s) {
  regtopk_ctx* g = nullptr;
  int rc = create_common(&g, 1, c->d, c->k, 0.0f, mem, bytes, owned, s, true);
  if (rc != REGTOPK_OK) return rc;
  c->gsel = g;
  return REGTOPK_OK;
}

size_t regtopk_global_workspace_bytes(int64_t d, int64_t k) {
  Layout L;
  return make_layout(1, d, k, &L) ? L.total : 0;
}

int regtopk_bind_global(regtopk_ctx* c, void* mem_dev, size_t bytes, void* stream) {
  if (!c || !mem_dev) return fail(REGTOPK_INVALID_ARG, "ctx and mem_dev must not be NULL");
  if (c->gsel) return fail(REGTOPK_BAD_STATE, "the global Top-k round already has its memory");
  DEVICE_TRY(c);
  if (reinterpret_cast<uintptr_t>(mem_dev) % kAlign) return fail(REGTOPK_INVALID_ARG, "mem_dev must be 256-byte aligned");
  const size_t need = regtopk_global_workspace_bytes(c->d, c->k);
  if (bytes < need) return fail(REGTOPK_NO_MEMORY, "memory has %zu bytes, %zu needed", bytes, need);
  return bind_global_impl(c, mem_dev, bytes, false, static_cast<hipStream_t>(stream));
}

int regtopk_step_global(regtopk_ctx* c, const float* grads, void* stream, regtopk_result* out) {
  if (!c || !grads || !out) return fail(REGTOPK_INVALID_ARG, "ctx, grads_dev and out must not be NULL");
  if (reinterpret_cast<uintptr_t>(grads) % 4) return fail(REGTOPK_INVALID_ARG, "grads_dev must be 4-byte aligned");
  if (!c->uniform_k) return fail(REGTOPK_BAD_STATE, "the global Top-k round shares one mask of k entries: per-worker k is set");
  DEVICE_TRY(c);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!c->gsel) {
    // first use.  A context that owns its arena allocates the selector's memory as well; one that
    // lives in the caller's memory never allocates: the caller binds the memory beforehand.
    if (!c->owns_arena)
      return fail(REGTOPK_BAD_STATE, "this context lives in caller-owned memory: give the global Top-k round its "
                                     "memory with regtopk_bind_global first");
    const size_t bytes = regtopk_global_workspace_bytes(c->d, c->k);
    void* ga = nullptr;
    if (bytes == 0 || hipMalloc(&ga, bytes) != hipSuccess) {
      (void)hipGetLastError();
      return fail(REGTOPK_NO_MEMORY, "hipMalloc of %zu bytes failed", bytes);
    }
    int rc = bind_global_impl(c, ga, bytes, true, s);
    if (rc != REGTOPK_OK) { (void)hipFree(ga); return rc; }
  }
  regtopk_ctx* g = c->gsel;
  const Layout& L = c->L;
  const int cur = (int)(c->t & 1), prv = cur ^ 1;
  const bool vec = (c->d % 4 == 0) && (reinterpret_cast<uintptr_t>(grads) % 16 == 0);
  float* e = c->at<float>(L.e);
  uint32_t* mask = c->at<uint32_t>(L.mask);
  const uint32_t* prev_sel_off = c->at<uint32_t>(L.sel_off[prv]);
  hipEvent_t* ev = c->profile ? c->ev[c->prof_rounds % kProfRounds] : nullptr;
  const bool ev_all = c->profile == 1;
  if (ev) c->ev_level[c->prof_rounds % kProfRounds] = c->profile;
  if (ev && ev_all) HIP_TRY(hipEventRecord(ev[4], s));
  if (ev) HIP_TRY(hipEventRecord(ev[0], s));
  // abar goes straight into the selector's state: its round neither adds nor stores anything
  float* abar = g->at<float>(g->L.e);
  const uint32_t acc_blocks = (uint32_t)((c->d + 4 * kGlobalBlock - 1) / (4 * kGlobalBlock));
  if (vec) k_global_accum<true, kGlobalRows, kGlobalBlock><<<acc_blocks, kGlobalBlock, 0, s>>>(e, grads, mask, c->d, L.nc, c->N, c->at<float>(L.omega), abar);
  else k_global_accum<false, 1, kGlobalBlock><<<acc_blocks, kGlobalBlock, 0, s>>>(e, grads, mask, c->d, L.nc, c->N, c->at<float>(L.omega), abar);
  if (ev) HIP_TRY(hipEventRecord(ev[1], s));
  HIP_TRY(hipGetLastError());
  regtopk_result sel;
  const int gcur = (int)(g->t & 1);
  int rc = step_impl<float>(g, nullptr, nullptr, stream, &sel, true);
  if (rc != REGTOPK_OK) return rc;
  if (ev && ev_all) HIP_TRY(hipEventRecord(ev[2], s));
  const uint32_t entry_blocks = (uint32_t)((c->k + kBlock - 1) / kBlock);
  k_global_apply<<<dim3(entry_blocks + (L.nc + 3) / 4, c->N), kBlock, 0, s>>>(
      e, sel.idx, g->at<uint32_t>(g->L.sel_off[gcur]), g->at<uint32_t>(g->L.mask), prev_sel_off,
      c->at<int32_t>(L.out_idx[cur]), c->at<float>(L.out_val[cur]), c->at<uint32_t>(L.sel_off[cur]), mask, c->d, c->k, L.nc,
      entry_blocks);
  if (ev && ev_all) HIP_TRY(hipEventRecord(ev[3], s));
  if (ev) c->prof_rounds += 1;
  HIP_TRY(hipGetLastError());
  c->t += 1;
  c->have_prev = true;
  c->fresh = kFreshRounds;               // bounds of earlier local rounds do not describe the next one
  out->idx = c->at<int32_t>(L.out_idx[cur]);
  out->val = c->at<float>(L.out_val[cur]);
  out->agg = sel.agg;
  return REGTOPK_OK;
}

int regtopk_step_bf16(regtopk_ctx* c, const uint16_t* grads, const float* gprev, void* stream, regtopk_result* out) {
  return step_impl<bf16_t>(c, reinterpret_cast<const bf16_t*>(grads), gprev, stream, out);
}

int regtopk_get_state(regtopk_ctx* c, float* e_dev, int32_t* pidx_dev, float* pval_dev, int64_t* t_host, void* stream) {
  if (!c) return fail(REGTOPK_INVALID_ARG, "ctx is NULL");
  DEVICE_TRY(c);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t nd = (size_t)c->N * (size_t)c->d, nk = (size_t)c->N * (size_t)c->k;
  (void)nd;
  if (e_dev) k_export_eps<<<2048, 256, 0, s>>>(e_dev, c->at<float>(c->L.e), c->at<uint32_t>(c->L.mask), c->d, c->L.nc, c->N);
  if (c->have_prev) {
    const int prv = (int)((c->t & 1) ^ 1);
    if (pidx_dev) k_copy_u32<<<512, 256, 0, s>>>(reinterpret_cast<uint32_t*>(pidx_dev), c->at<uint32_t>(c->L.out_idx[prv]), nk);
    if (pval_dev) k_copy_u32<<<512, 256, 0, s>>>(reinterpret_cast<uint32_t*>(pval_dev), c->at<uint32_t>(c->L.out_val[prv]), nk);
  }
  HIP_TRY(hipGetLastError());
  if (t_host) *t_host = c->t;
  return REGTOPK_OK;
}

int regtopk_set_state(regtopk_ctx* c, const float* e_dev, const int32_t* pidx_dev, const float* pval_dev, int64_t t, void* stream) {
  if (!c || !e_dev) return fail(REGTOPK_INVALID_ARG, "ctx and e_dev must not be NULL");
  if (t < 0) return fail(REGTOPK_INVALID_ARG, "t must be >= 0");
  if (t > 0 && (!pidx_dev || !pval_dev)) return fail(REGTOPK_INVALID_ARG, "previous lists are required when t > 0");
  DEVICE_TRY(c);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t nd = (size_t)c->N * (size_t)c->d, nk = (size_t)c->N * (size_t)c->k;
  k_copy_u32<<<2048, 256, 0, s>>>(c->at<uint32_t>(c->L.e), reinterpret_cast<const uint32_t*>(e_dev), nd);
  k_init_ctl<<<c->N, 256, 0, s>>>(c->at<WorkerCtl>(c->L.ctl));     // no bound is carried over: the next rounds sample theirs
  k_fill_u32<<<1, 64, 0, s>>>(c->at<uint32_t>(c->L.gctl), sizeof(GlobalCtl) / 4, 0u);
  k_fill_u32<<<1, 64, 0, s>>>(c->host_err, 1, 0u);
  c->t = t;
  c->have_prev = t > 0;
  c->fresh = kFreshRounds;
  c->need_begin = true;
  if (t == 0) {
    for (int b = 0; b < 2; ++b)
      k_fill_u32<<<256, 256, 0, s>>>(c->at<uint32_t>(c->L.sel_off[b]), (size_t)c->N * (c->L.nc + 1), 0u);
    k_fill_u32<<<1024, 256, 0, s>>>(c->at<uint32_t>(c->L.mask), (size_t)c->N * c->L.nc * kChunkWords, 0u);
  }
  if (t > 0) {
    const int prv = (int)((t & 1) ^ 1);
    int32_t* pi = c->at<int32_t>(c->L.out_idx[prv]);
    k_copy_u32<<<512, 256, 0, s>>>(reinterpret_cast<uint32_t*>(pi), reinterpret_cast<const uint32_t*>(pidx_dev), nk);
    k_copy_u32<<<512, 256, 0, s>>>(c->at<uint32_t>(c->L.out_val[prv]), reinterpret_cast<const uint32_t*>(pval_dev), nk);
    const dim3 g((c->L.nc + 3) / 4, c->N);
    k_build_mask<<<g, kBlock, 0, s>>>(pi, c->at<uint32_t>(c->L.mask), c->at<uint32_t>(c->L.sel_off[prv]), c->k, c->at<uint32_t>(c->L.kn), c->L.nc);
    k_scatter_prev<<<512, 256, 0, s>>>(c->at<float>(c->L.e), pi, c->at<float>(c->L.out_val[prv]), c->d, c->k, c->at<uint32_t>(c->L.kn), c->N);
    const dim3 g2(64, c->N);
    k_check_ascending<<<g2, 256, 0, s>>>(pi, c->at<WorkerCtl>(c->L.ctl), c->d, c->k, c->at<uint32_t>(c->L.kn));
  }
  HIP_TRY(hipGetLastError());
  return REGTOPK_OK;
}

int regtopk_get_stats(regtopk_ctx* c, regtopk_worker_stats* st, void* stream) {
  if (!c || !st) return fail(REGTOPK_INVALID_ARG, "ctx and stats_host must not be NULL");
  DEVICE_TRY(c);
  hipStream_t s = static_cast<hipStream_t>(stream);
  std::vector<WorkerCtl> h((size_t)c->N);
  GlobalCtl hg;
  HIP_TRY(hipMemcpyAsync(h.data(), c->at<WorkerCtl>(c->L.ctl), sizeof(WorkerCtl) * (size_t)c->N, hipMemcpyDeviceToHost, s));
  HIP_TRY(hipMemcpyAsync(&hg, c->at<GlobalCtl>(c->L.gctl), sizeof(GlobalCtl), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  uint32_t err = hg.bar_err ? 4u : 0u;
  for (int32_t n = 0; n < c->N; ++n) {
    const WorkerCtl& w = h[(size_t)n];
    st[n].tau_lo_bits = w.snap_tau_lo;
    st[n].n_candidates = w.snap_n_cand;
    st[n].used_dense = w.snap_used_dense;
    st[n].tau_bits = w.tau;
    st[n].n_greater = w.n_gt;
    st[n].n_ties_taken = w.budget;
    st[n].n_ties_total = w.ties_total;
    st[n].overflow = w.snap_overflow;
    st[n].used_window = w.snap_used_window;
    st[n].n_boundary = w.snap_n_bnd;
    st[n].n_valid = w.snap_n_valid;
    st[n].window_half = w.snap_win_half;
    err |= w.err;
  }
  if (err) return fail(REGTOPK_BAD_STATE, "device-side check failed (flags 0x%x)", err);
  return REGTOPK_OK;
}

int regtopk_set_weights(regtopk_ctx* c, const float* w_host, void* stream) {
  if (!c || !w_host) return fail(REGTOPK_INVALID_ARG, "ctx and weights_host must not be NULL");
  DEVICE_TRY(c);
  for (int32_t n = 0; n < c->N; ++n)
    if (!std::isfinite(w_host[n])) return fail(REGTOPK_INVALID_ARG, "weight %d is not finite", n);
  hipStream_t s = static_cast<hipStream_t>(stream);
  HIP_TRY(hipMemcpyAsync(c->at<float>(c->L.omega), w_host, (size_t)c->N * 4, hipMemcpyHostToDevice, s));
  HIP_TRY(hipStreamSynchronize(s));
  return REGTOPK_OK;
}

int regtopk_set_worker_k(regtopk_ctx* c, const int64_t* k_host, void* stream) {
  if (!c || !k_host) return fail(REGTOPK_INVALID_ARG, "ctx and k_host must not be NULL");
  DEVICE_TRY(c);
  std::vector<uint32_t> v((size_t)c->N);
  bool uniform = true;
  for (int32_t n = 0; n < c->N; ++n) {
    if (k_host[n] < 1 || k_host[n] > c->k)
      return fail(REGTOPK_INVALID_ARG, "k of worker %d is %lld, outside [1, %lld]", n, (long long)k_host[n], (long long)c->k);
    v[(size_t)n] = (uint32_t)k_host[n];
    uniform = uniform && k_host[n] == c->k;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  HIP_TRY(hipMemcpyAsync(c->at<uint32_t>(c->L.kn), v.data(), (size_t)c->N * 4, hipMemcpyHostToDevice, s));
  HIP_TRY(hipStreamSynchronize(s));
  c->uniform_k = uniform;
  c->reinit_ctl = true;                  // the bounds carried over belong to the old k
  c->fresh = kFreshRounds;
  return REGTOPK_OK;
}

int regtopk_mask_overlap(regtopk_ctx* c, int64_t* counts_dev, void* stream) {
  if (!c || !counts_dev) return fail(REGTOPK_INVALID_ARG, "ctx and counts_dev must not be NULL");
  if (reinterpret_cast<uintptr_t>(counts_dev) % 8) return fail(REGTOPK_INVALID_ARG, "counts_dev must be 8-byte aligned");
  DEVICE_TRY(c);
  hipStream_t s = static_cast<hipStream_t>(stream);
  int planes = 1;
  while ((1 << planes) <= c->N) ++planes;             // column sums reach N
  const size_t nw = (size_t)((c->d + 31) / 32);
  size_t blocks = (nw + kBlock - 1) / kBlock;
  if (blocks > 4096) blocks = 4096;
  unsigned long long* counts = reinterpret_cast<unsigned long long*>(counts_dev);
  // Per-block histograms go through the histogram area of the dense selection,
  // which is idle between rounds and cleared before each of its uses:
  // 4096 * (N+1) words fit into its 3 * 4096 * N words for every N >= 1.
  uint32_t* partial = c->at<uint32_t>(c->L.fhist);
  const bool staged = (uint32_t)c->N + 1u <= kOverlapBins;
  if (!staged) k_fill_u32<<<64, 256, 0, s>>>(reinterpret_cast<uint32_t*>(counts_dev), 2 * ((size_t)c->N + 1), 0u);
  k_mask_overlap<<<(uint32_t)blocks, kBlock, 0, s>>>(c->at<uint32_t>(c->L.mask), c->d, c->L.nc, c->N, planes, counts, partial);
  if (staged) k_overlap_sum<<<(uint32_t)c->N + 1u, kBlock, 0, s>>>(partial, (uint32_t)blocks, c->N, counts);
  HIP_TRY(hipGetLastError());
  return REGTOPK_OK;
}

int regtopk_mask_overlap_static(regtopk_ctx* c, int64_t* counts_dev, void* stream) {
  if (!c || !counts_dev) return fail(REGTOPK_INVALID_ARG, "ctx and counts_dev must not be NULL");
  if (reinterpret_cast<uintptr_t>(counts_dev) % 8) return fail(REGTOPK_INVALID_ARG, "counts_dev must be 8-byte aligned");
  if ((uint32_t)c->N + 1u > kOverlapBins)
    return fail(REGTOPK_INVALID_ARG, "regtopk_mask_overlap_static handles at most %u workers (N = %d); use regtopk_mask_overlap",
                kOverlapBins - 1u, c->N);
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev != c->device) return fail(REGTOPK_INVALID_ARG, "the context lives on device %d, the current device is %d", c->device, dev);
  uint32_t* scratch = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_overlap_mutex);
    if (!g_overlap_ptr[dev]) {
      void* p = nullptr;
      HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(g_overlap_scratch)));     // this device's copy of the array
      g_overlap_ptr[dev] = static_cast<uint32_t*>(p);
    }
    scratch = g_overlap_ptr[dev];
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  int planes = 1;
  while ((1 << planes) <= c->N) ++planes;
  const size_t nw = (size_t)((c->d + 31) / 32);
  size_t blocks = (nw + kBlock - 1) / kBlock;
  if (blocks > kStaticOverlapBlocks) blocks = kStaticOverlapBlocks;
  // Nothing has to be cleared: every block writes all N + 1 words of its row of the scratch before
  // k_overlap_sum reads exactly those rows, so what an earlier call left behind is never read.
  k_mask_overlap<<<(uint32_t)blocks, kBlock, 0, s>>>(c->at<uint32_t>(c->L.mask), c->d, c->L.nc, c->N, planes,
                                                     reinterpret_cast<unsigned long long*>(counts_dev), scratch);
  k_overlap_sum<<<(uint32_t)c->N + 1u, kBlock, 0, s>>>(scratch, (uint32_t)blocks, c->N,
                                                      reinterpret_cast<unsigned long long*>(counts_dev));
  HIP_TRY(hipGetLastError());
  return REGTOPK_OK;
}

int regtopk_sgd_update(float* theta_dev, const float* g_dev, float eta, int64_t d, void* stream) {
  if (d < 0 || (d > 0 && (!theta_dev || !g_dev))) return fail(REGTOPK_INVALID_ARG, "bad arguments");
  if (reinterpret_cast<uintptr_t>(theta_dev) % 4 || reinterpret_cast<uintptr_t>(g_dev) % 4)
    return fail(REGTOPK_INVALID_ARG, "device pointers must be 4-byte aligned");
  if (d == 0) return REGTOPK_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool vec = d % 4 == 0 && reinterpret_cast<uintptr_t>(theta_dev) % 16 == 0 && reinterpret_cast<uintptr_t>(g_dev) % 16 == 0;
  int64_t blocks = ((vec ? d / 4 : d) + kBlock - 1) / kBlock;
  if (blocks > 8192) blocks = 8192;
  if (vec) k_sgd_update<true><<<(uint32_t)blocks, kBlock, 0, s>>>(theta_dev, g_dev, eta, d);
  else k_sgd_update<false><<<(uint32_t)blocks, kBlock, 0, s>>>(theta_dev, g_dev, eta, d);
  HIP_TRY(hipGetLastError());
  return REGTOPK_OK;
}

int regtopk_get_timings(regtopk_ctx* c, float* out, int32_t max_rounds, int32_t* n_rounds) {
  if (!c || !out || !n_rounds || max_rounds < 0) return fail(REGTOPK_INVALID_ARG, "bad arguments");
  if (!c->profile) return fail(REGTOPK_BAD_STATE, "profiling is off (REGTOPK_OPT_PROFILE)");
  int64_t have = c->prof_rounds < kProfRounds ? c->prof_rounds : kProfRounds;
  if (have > max_rounds) have = max_rounds;
  for (int64_t i = 0; i < have; ++i) {
    const int64_t r = c->prof_rounds - have + i;      // oldest first
    hipEvent_t* ev = c->ev[r % kProfRounds];
    const bool all = c->ev_level[r % kProfRounds] == 1;
    HIP_TRY(hipEventSynchronize(all ? ev[3] : ev[1]));
    HIP_TRY(hipEventElapsedTime(&out[i * 4 + 0], ev[0], ev[1]));
    out[i * 4 + 1] = out[i * 4 + 2] = out[i * 4 + 3] = 0.0f;
    if (all) {
      HIP_TRY(hipEventElapsedTime(&out[i * 4 + 1], ev[1], ev[2]));
      HIP_TRY(hipEventElapsedTime(&out[i * 4 + 2], ev[2], ev[3]));
      HIP_TRY(hipEventElapsedTime(&out[i * 4 + 3], ev[4], ev[3]));
    }
  }
  *n_rounds = (int32_t)have;
  return REGTOPK_OK;
}

int regtopk_copy_f32(float* dst_dev, const float* src_dev, int64_t n, void* stream) {
  if (n < 0 || (n > 0 && (!dst_dev || !src_dev))) return fail(REGTOPK_INVALID_ARG, "bad arguments");
  if (n == 0) return REGTOPK_OK;
  k_copy_u32<<<2048, 256, 0, static_cast<hipStream_t>(stream)>>>(reinterpret_cast<uint32_t*>(dst_dev),
                                                                   reinterpret_cast<const uint32_t*>(src_dev), (size_t)n);
  HIP_TRY(hipGetLastError());
  return REGTOPK_OK;
}

int regtopk_pow_f32(const float* x_dev, float y, float* out_dev, int64_t n, void* stream) {
  if (n < 0 || (n > 0 && (!x_dev || !out_dev)) || !(y > 0.0f && y < 1.0f)) return fail(REGTOPK_INVALID_ARG, "bad arguments");
  if (n == 0) return REGTOPK_OK;
  k_pow<<<2048, 256, 0, static_cast<hipStream_t>(stream)>>>(x_dev, y, out_dev, n);
  HIP_TRY(hipGetLastError());
  return REGTOPK_OK;
}

int regtopk_erf_f32(const float* x_dev, float* y_dev, int64_t n, void* stream) {
  if (n < 0 || (n > 0 && (!x_dev || !y_dev))) return fail(REGTOPK_INVALID_ARG, "bad arguments");
  if (n == 0) return REGTOPK_OK;
  k_erf<<<2048, 256, 0, static_cast<hipStream_t>(stream)>>>(x_dev, y_dev, n);
  HIP_TRY(hipGetLastError());
  return REGTOPK_OK;
}

int regtopk_tanh_f32(const float* x_dev, float* y_dev, int64_t n, void* stream) {
  if (n < 0 || (n > 0 && (!x_dev || !y_dev))) return fail(REGTOPK_INVALID_ARG, "bad arguments");
  if (n == 0) return REGTOPK_OK;
  k_tanh<<<2048, 256, 0, static_cast<hipStream_t>(stream)>>>(x_dev, y_dev, n);
  HIP_TRY(hipGetLastError());
  return REGTOPK_OK;
}

}  // extern "C"
