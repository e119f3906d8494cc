// RegTop-k oracle: a plain, slow, single-threaded CPU statement of one
// communication round of Regularized Top-k gradient sparsification for N
// simulated workers plus the server-side aggregation.
//
// THIS IS TEST INFRASTRUCTURE. It is the parity reference for the HIP library
// and the timed CPU baseline of the benchmark; nothing on the product path may
// call it, and it shares no code, header, table or constant with the HIP path.
//
// What it follows (paper: "Regularized Top-k: A Bayesian Framework for
// Gradient Sparsification"):
//   * Algorithm 2 (RegTop-k sparsification at worker n): accumulate, posterior
//     distortion, regularised Top_k mask, sparsified gradient, error update.
//   * Algorithm 1 / the Top_k selector defined in the subsection "Top-k:
//     Classical Sparsification Scheme": mask with exactly k ones on the k
//     largest magnitudes.
//   * The definition of the posterior distortion Delta in the subsection
//     "Characterizing the Likelihood".
//   * The likelihood with tanh and the constant C = 1 (Section "RegTop-k
//     Algorithm", display after the cumulative function u_mu, and its footnote).
//   * The aggregation equation g^t = sum_n omega_n ghat_n^t right after
//     Algorithm 1.
//
// Precision: every quantity is IEEE-754 binary32, round to nearest even, no
// fused multiply-add, denormals kept (build with -ffp-contract=off and without
// fast-math).  The one non-elementary step, tanh, is taken as the correctly
// rounded binary32 value of the exact tanh of its binary32 argument; it is
// realised here by evaluating tanhl in x87 extended precision (64-bit
// significand) and rounding once to binary32.
//
// Readings where the paper leaves a choice (each is also listed in the design
// document of the repository):
//   R1  ties in Top_k: the lower index wins; always exactly k entries.
//   R2  omega_n = 1/N for every worker, computed as 1.0f / (float)N, unless
//       the caller sets other weights (the paper's general aggregation
//       g = sum_n omega_n g_n of the introduction); worker n then uses its own
//       omega_n in the distortion, as Algorithm 2 writes it.
//   R3  entries not sent in the previous round get the factor 1 exactly
//       (C = 1, i.e. the Q -> infinity limit); Q is never formed.
//   R4  omega * a^t == 0 in the denominator of the distortion: factor 1
//       (infinite distortion = no information).  A NaN argument: factor 1.
//   R5  mu == 0 switches the regulariser off (plain Top-k, Algorithm 1).
//   R6  round 0 has an empty previous mask, so it is plain Top-k.
//   R7  operation order of the distortion: (gprev - w*aprev) / (w*a), then
//       1 + D, abs, divide by mu, tanh, times |a|.
//   R8  aggregation: start from +0 and add w * ghat_n[j] for n = 0..N-1 in
//       ascending worker order.
//   R9  the sent values are the un-weighted entries of a; the server applies w.
//   R15 score variants of the appendix remark on sub-linear scaling and of the
//       sentence that other cumulative functions u_mu may replace tanh:
//       the prior |a|^y is offered for y = 2^-m, m = 0..3, and evaluated as m
//       successive correctly rounded binary32 square roots of |a| (so that both
//       sides of the parity check can take it bit for bit), and for a general
//       binary32 exponent 0 < y < 1 as the correctly rounded binary32 value of
//       the real power (realised by powl in x87 extended precision, rounded
//       once); besides tanh the
//       likelihood may be the cumulative function of a uniform innovation,
//       min(|1+Delta|/mu, 1), or of a Gaussian one with the constants dropped
//       as the paper drops them for tanh, erf(|1+Delta|/mu) (correctly rounded
//       binary32, realised like tanh).  The defaults (m = 0, tanh) are
//       Algorithm 2.
//   R18 Algorithm 2 is stated "at worker n" and its selector Top_k takes k as a
//       parameter of that worker's sparsifier; the paper's experiments give all
//       workers the same k.  Here worker n may be given its own k_n <= k: its
//       mask has exactly k_n ones, its lists hold k_n pairs, and the rest of its
//       row of the [N,k] outputs is filled with index -1 and value 0.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <numeric>
#include <vector>

namespace {

struct Oracle {
    int32_t N;
    int64_t d, k;
    float mu;
    std::vector<float> w;        // [N] aggregation weights omega_n (R2)
    std::vector<int64_t> kn;     // [N] entries kept by worker n, 1 <= k_n <= k (R18; default k)
    int sqrt_steps;              // prior |a|^y with y = 2^-sqrt_steps (R15)
    float exponent;              // or, when != 1, prior |a|^exponent (R15); sqrt_steps is then 0
    int likelihood;              // 0: tanh(x), 1: min(x, 1) (R15)
    int64_t t;       // rounds done so far
    std::vector<float> e;        // [N*d] sparsification error eps_n
    std::vector<float> a;        // [N*d] accumulated gradient of the last round
    std::vector<float> a_prev;   // [N*d] accumulated gradient of the round before
    std::vector<uint8_t> s_prev; // [N*d] previous mask s_n^{t-1}
    std::vector<float> score;    // [N*d] selection score of the last round
    std::vector<uint8_t> s;      // [N*d] mask of the last round
    std::vector<float> ghat;     // [N*d] sparsified gradient of the last round
};

// tanh step: correctly rounded binary32 tanh (see header).  Rounding the
// extended-precision value once more to binary32 gives the correctly rounded
// result only if the intermediate carries far more than 24 bits: the x87 format
// (64-bit significand) does, a long double that is binary64 would not be
// trusted here.
static_assert(std::numeric_limits<long double>::digits >= 64,
              "the oracle's tanh needs a long double with a 64-bit significand (x87 extended precision)");
float tanh32(float x) {
    return (float)tanhl((long double)x);
}

// erf step of the Gaussian likelihood (R15): correctly rounded binary32 erf,
// realised the same way.
float erf32(float x) {
    return (float)erfl((long double)x);
}

// Likelihood factor for an entry that WAS sent in the previous round
// (Algorithm 2, distortion line and the tanh in the mask line).  R4, R7.
float likelihood_sent(float a_now, float a_before, float g_before, float w, float mu, int kind = 0) {
    float num = g_before - w * a_before;   // g^{t-1} - omega a^{t-1}
    float den = w * a_now;                 // omega a^t
    if (den == 0.0f) return 1.0f;
    float D = num / den;                   // posterior distortion Delta
    float r = std::fabs(1.0f + D);
    float x = r / mu;
    if (x != x) return 1.0f;
    if (kind == 1) return x < 1.0f ? x : 1.0f;   // uniform innovation on [0, mu]
    if (kind == 2) return erf32(x);              // Gaussian innovation
    return tanh32(x);
}

// Prior |a|^y, y = 2^-m, as m correctly rounded square roots (R15).
float prior(float a, int m) {
    float p = std::fabs(a);
    for (int i = 0; i < m; ++i) p = std::sqrt(p);
    return p;
}

// Prior |a|^y for a general exponent 0 < y < 1: the real power rounded once to
// binary32 (R15).
float prior_pow(float a, float y) {
    return (float)powl((long double)std::fabs(a), (long double)y);
}

// Top_k selector: mask with exactly k ones on the k largest scores, lower index
// first among equal scores (R1).  Scores are non-negative and never NaN here.
void topk_mask(const float* score, int64_t d, int64_t k, uint8_t* mask) {
    std::vector<int64_t> order((size_t)d);
    std::iota(order.begin(), order.end(), (int64_t)0);
    auto before = [score](int64_t i, int64_t j) {
        if (score[i] != score[j]) return score[i] > score[j];
        return i < j;
    };
    if (k < d) std::nth_element(order.begin(), order.begin() + k, order.end(), before);
    std::fill(mask, mask + d, (uint8_t)0);
    for (int64_t i = 0; i < k; ++i) mask[order[(size_t)i]] = 1;
}

}  // namespace

extern "C" {

void* rtk_oracle_create(int32_t N, int64_t d, int64_t k, float mu) {
    if (N < 1 || d < 1 || k < 1 || k > d || !(mu >= 0.0f)) return nullptr;
    Oracle* o = new Oracle;
    o->N = N; o->d = d; o->k = k; o->mu = mu;
    o->w.assign((size_t)N, 1.0f / (float)N);
    o->kn.assign((size_t)N, k);
    o->t = 0;
    o->sqrt_steps = 0;
    o->exponent = 1.0f;
    o->likelihood = 0;
    size_t nd = (size_t)N * (size_t)d;
    o->e.assign(nd, 0.0f);           // eps^0 = 0
    o->a.assign(nd, 0.0f);
    o->a_prev.assign(nd, 0.0f);
    o->s_prev.assign(nd, 0);         // empty previous mask (R6)
    o->score.assign(nd, 0.0f);
    o->s.assign(nd, 0);
    o->ghat.assign(nd, 0.0f);
    return o;
}

void rtk_oracle_destroy(void* h) { delete (Oracle*)h; }

// One round.  grads [N*d] row-major, gprev [d] (previous aggregate g^{t-1};
// not read in round 0 and may then be NULL).  Outputs: idx [N*k] ascending per
// worker, val [N*k] = a at those indices, agg [d].
void rtk_oracle_step(void* h, const float* grads, const float* gprev,
                     int32_t* idx, float* val, float* agg) {
    Oracle* o = (Oracle*)h;
    const int64_t d = o->d, k = o->k;
    const float mu = o->mu;
    for (int32_t n = 0; n < o->N; ++n) {
        const float w = o->w[(size_t)n];
        const size_t row = (size_t)n * (size_t)d;
        float* e = &o->e[row];
        float* a = &o->a[row];
        float* ap = &o->a_prev[row];
        uint8_t* sp = &o->s_prev[row];
        float* sc = &o->score[row];
        uint8_t* s = &o->s[row];
        float* gh = &o->ghat[row];
        const float* g = grads + row;
        for (int64_t j = 0; j < d; ++j) {
            a[j] = e[j] + g[j];                              // accumulate
            float f = 1.0f;                                  // C = 1 (R3)
            if (mu != 0.0f && sp[j])                         // R5, R6
                f = likelihood_sent(a[j], ap[j], gprev[j], w, mu, o->likelihood);
            const float pr = o->exponent != 1.0f ? prior_pow(a[j], o->exponent) : prior(a[j], o->sqrt_steps);
            sc[j] = pr * f;                                  // |a|^y . u(|1 + Delta|)
        }
        topk_mask(sc, d, o->kn[(size_t)n], s);               // s^t = Top_k(.), k = k_n (R18)
        int64_t c = 0;
        for (int64_t j = 0; j < d; ++j) {
            gh[j] = (float)s[j] * a[j];                      // ghat = s . a
            e[j] = a[j] - gh[j];                             // eps^{t+1} = a - ghat
            if (s[j]) { idx[(size_t)n * k + c] = (int32_t)j; val[(size_t)n * k + c] = a[j]; ++c; }
        }
        for (; c < k; ++c) { idx[(size_t)n * k + c] = -1; val[(size_t)n * k + c] = 0.0f; }   // unused rest of the row
        std::memcpy(ap, a, sizeof(float) * (size_t)d);       // keep a^{t} for round t+1
        std::memcpy(sp, s, (size_t)d);                       // keep s^{t}
    }
    for (int64_t j = 0; j < d; ++j) {                        // server: g = sum_n w ghat_n (R8)
        float acc = 0.0f;
        for (int32_t n = 0; n < o->N; ++n) acc = acc + o->w[(size_t)n] * o->ghat[(size_t)n * d + j];
        agg[j] = acc;
    }
    o->t += 1;
}

// Aggregation weights omega_n (introduction, aggregation equation with general
// weights).  They apply from the next round on, to the distortion of worker n
// and to its term of the aggregate.
void rtk_oracle_set_weights(void* h, const float* w) {
    Oracle* o = (Oracle*)h;
    for (int32_t n = 0; n < o->N; ++n) o->w[(size_t)n] = w[n];
}

// Entries kept per worker (R18): k_n[0..N), each in [1, k].  Applies from the
// next round on.  Returns 0 on success.
int rtk_oracle_set_worker_k(void* h, const int64_t* kn) {
    Oracle* o = (Oracle*)h;
    for (int32_t n = 0; n < o->N; ++n)
        if (kn[n] < 1 || kn[n] > o->k) return -1;
    for (int32_t n = 0; n < o->N; ++n) o->kn[(size_t)n] = kn[n];
    return 0;
}

// Score variant (R15): prior exponent y = 2^-sqrt_steps (0..3) and the kind of
// likelihood (0 tanh, 1 clipped linear, 2 erf).  Returns 0 on success.
int rtk_oracle_set_score_variant(void* h, int sqrt_steps, int likelihood) {
    Oracle* o = (Oracle*)h;
    if (sqrt_steps < 0 || sqrt_steps > 3 || likelihood < 0 || likelihood > 2) return -1;
    o->sqrt_steps = sqrt_steps;
    o->exponent = 1.0f;
    o->likelihood = likelihood;
    return 0;
}

// General prior exponent 0 < y <= 1 (R15); y = 1 is Algorithm 2.  Replaces the
// square-root variant.  Returns 0 on success.
int rtk_oracle_set_prior_exponent(void* h, float y) {
    Oracle* o = (Oracle*)h;
    if (!(y > 0.0f && y <= 1.0f)) return -1;
    o->exponent = y;
    o->sqrt_steps = 0;
    return 0;
}

// How far the masks of the last round agree (appendix "Comparing Sparsification
// Masks"): counts[c], c = 0..N, is the number of entries j that exactly c
// workers selected.
void rtk_oracle_mask_overlap(void* h, int64_t* counts) {
    Oracle* o = (Oracle*)h;
    for (int32_t c = 0; c <= o->N; ++c) counts[c] = 0;
    for (int64_t j = 0; j < o->d; ++j) {
        int32_t c = 0;
        for (int32_t n = 0; n < o->N; ++n) c += o->s[(size_t)n * o->d + j];
        counts[c] += 1;
    }
}

// Model update of distributed SGD (introduction): theta <- theta - eta * g,
// binary32, the product rounded before the subtraction.
void rtk_oracle_sgd_update(float* theta, const float* g, float eta, int64_t d) {
    for (int64_t j = 0; j < d; ++j) {
        float step = eta * g[j];
        theta[j] = theta[j] - step;
    }
}

// One round of the idealised "global Top-k" of the subsection "Statistical
// Global Top-k": a genie tells every worker the aggregate of the accumulated
// gradients without sparsification, abar_j = sum_n omega_n a_{n,j}, and all
// workers apply Top_k to it, i.e. they share one mask, the k largest |abar_j|
// (lower index first among equals).  Everything else is Algorithm 1: a = eps +
// g, ghat = s . a, eps <- a - ghat, g = sum_n omega_n ghat_n.  abar is summed
// like the aggregate (R8: from +0, + omega_n a_n in ascending worker order).
// Outputs as in rtk_oracle_step (the N index rows are equal).
void rtk_oracle_step_global(void* h, const float* grads, int32_t* idx, float* val, float* agg) {
    Oracle* o = (Oracle*)h;
    const int64_t d = o->d, k = o->k;
    const size_t nd = (size_t)o->N * (size_t)d;
    for (size_t i = 0; i < nd; ++i) o->a[i] = o->e[i] + grads[i];      // accumulate
    std::vector<float> mag((size_t)d);
    for (int64_t j = 0; j < d; ++j) {
        float acc = 0.0f;
        for (int32_t n = 0; n < o->N; ++n) acc = acc + o->w[(size_t)n] * o->a[(size_t)n * d + j];
        mag[(size_t)j] = std::fabs(acc);                              // what the genie reveals
    }
    std::vector<uint8_t> s((size_t)d);
    topk_mask(mag.data(), d, k, s.data());
    for (int32_t n = 0; n < o->N; ++n) {
        const size_t row = (size_t)n * (size_t)d;
        int64_t c = 0;
        for (int64_t j = 0; j < d; ++j) {
            const float a = o->a[row + j];
            o->score[row + j] = mag[(size_t)j];
            o->s[row + j] = s[(size_t)j];
            o->ghat[row + j] = (float)s[(size_t)j] * a;
            o->e[row + j] = a - o->ghat[row + j];
            if (s[(size_t)j]) { idx[(size_t)n * k + c] = (int32_t)j; val[(size_t)n * k + c] = a; ++c; }
        }
    }
    o->a_prev = o->a;
    o->s_prev = o->s;
    for (int64_t j = 0; j < d; ++j) {
        float acc = 0.0f;
        for (int32_t n = 0; n < o->N; ++n) acc = acc + o->w[(size_t)n] * o->ghat[(size_t)n * d + j];
        agg[j] = acc;
    }
    o->t += 1;
}

// Read-only views for the tests (pointers stay valid until destroy).
const float* rtk_oracle_e(void* h) { return ((Oracle*)h)->e.data(); }
const float* rtk_oracle_a(void* h) { return ((Oracle*)h)->a.data(); }
const float* rtk_oracle_score(void* h) { return ((Oracle*)h)->score.data(); }
const uint8_t* rtk_oracle_mask(void* h) { return ((Oracle*)h)->s.data(); }
int64_t rtk_oracle_round(void* h) { return ((Oracle*)h)->t; }

// Single steps exposed so that the tests can pin them one by one.
float rtk_oracle_tanh32(float x) { return tanh32(x); }
float rtk_oracle_likelihood_sent(float a_now, float a_before, float g_before, float w, float mu) {
    return likelihood_sent(a_now, a_before, g_before, w, mu);
}
float rtk_oracle_likelihood_sent_kind(float a_now, float a_before, float g_before, float w, float mu, int kind) {
    return likelihood_sent(a_now, a_before, g_before, w, mu, kind);
}
float rtk_oracle_prior(float a, int sqrt_steps) { return prior(a, sqrt_steps); }
float rtk_oracle_prior_pow(float a, float y) { return prior_pow(a, y); }
void rtk_oracle_prior_pow_array(const float* x, float y, float* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = prior_pow(x[i], y);
}
void rtk_oracle_topk_mask(const float* score, int64_t d, int64_t k, uint8_t* mask) {
    topk_mask(score, d, k, mask);
}
void rtk_oracle_tanh32_array(const float* x, float* y, int64_t n) {
    for (int64_t i = 0; i < n; ++i) y[i] = tanh32(x[i]);
}
float rtk_oracle_erf32(float x) { return erf32(x); }
void rtk_oracle_erf32_array(const float* x, float* y, int64_t n) {
    for (int64_t i = 0; i < n; ++i) y[i] = erf32(x[i]);
}

}  // extern "C"
