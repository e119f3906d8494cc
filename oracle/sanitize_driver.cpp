// Runs the CPU oracle through its whole interface under AddressSanitizer and
// UndefinedBehaviorSanitizer (built by tests/test_oracle_sanitized.py together
// with regtopk_oracle.cpp).  TEST INFRASTRUCTURE.  The checks here are only what
// the definitions fix at any size -- exactly k_n mask bits, a = ghat + eps
// bitwise, ascending index lists, counts that add up -- the point of the run is
// that the sanitizers see every code path with ragged sizes.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

extern "C" {
void* rtk_oracle_create(int32_t N, int64_t d, int64_t k, float mu);
void rtk_oracle_destroy(void* h);
void rtk_oracle_step(void* h, const float* grads, const float* gprev, int32_t* idx, float* val, float* agg);
void rtk_oracle_step_global(void* h, const float* grads, int32_t* idx, float* val, float* agg);
void rtk_oracle_set_weights(void* h, const float* w);
int rtk_oracle_set_worker_k(void* h, const int64_t* kn);
int rtk_oracle_set_score_variant(void* h, int sqrt_steps, int likelihood);
void rtk_oracle_mask_overlap(void* h, int64_t* counts);
void rtk_oracle_sgd_update(float* theta, const float* g, float eta, int64_t d);
const float* rtk_oracle_e(void* h);
const float* rtk_oracle_a(void* h);
const uint8_t* rtk_oracle_mask(void* h);
float rtk_oracle_tanh32(float x);
void rtk_oracle_topk_mask(const float* score, int64_t d, int64_t k, uint8_t* mask);
}

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform() {
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return (double)(rng_state >> 11) / 9007199254740992.0;
}
static float draw(int pattern) {
  const double u = uniform() - 0.5;
  if (pattern == 0) return (float)(u * 4.0);
  if (pattern == 1) return (float)(std::floor(u * 7.0) * 0.25);          // few values: ties
  if (pattern == 2) return uniform() < 0.9 ? 0.0f : (float)u;            // mostly zeros
  return (float)(u * std::pow(10.0, std::floor(uniform() * 60.0) - 40.0)); // many binades, denormals
}
#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #cond, __LINE__); std::exit(1); } } while (0)

static void scenario(int32_t N, int64_t d, int64_t k, float mu, int pattern, int variant, bool weights, bool worker_k, int rounds) {
  void* h = rtk_oracle_create(N, d, k, mu);
  CHECK(h != nullptr);
  CHECK(rtk_oracle_set_score_variant(h, variant & 3, (variant >> 2) & 1) == 0);
  std::vector<float> w((size_t)N);
  if (weights) { for (auto& x : w) x = (float)uniform(); rtk_oracle_set_weights(h, w.data()); }
  std::vector<int64_t> kn((size_t)N, k);
  if (worker_k) { for (auto& x : kn) x = 1 + (int64_t)(uniform() * (double)k) % k; kn[0] = k; CHECK(rtk_oracle_set_worker_k(h, kn.data()) == 0); }
  std::vector<float> g((size_t)N * d), agg((size_t)d), val((size_t)N * k), gp((size_t)d, 0.0f);
  std::vector<int32_t> idx((size_t)N * k);
  std::vector<int64_t> counts((size_t)N + 1);
  for (int t = 0; t < rounds; ++t) {
    for (auto& x : g) x = draw(pattern);
    const bool global = !worker_k && t == rounds - 1;
    if (global) rtk_oracle_step_global(h, g.data(), idx.data(), val.data(), agg.data());
    else rtk_oracle_step(h, g.data(), gp.data(), idx.data(), val.data(), agg.data());
    const float* a = rtk_oracle_a(h);
    const float* e = rtk_oracle_e(h);
    const uint8_t* m = rtk_oracle_mask(h);
    for (int32_t n = 0; n < N; ++n) {
      const int64_t want = global ? k : kn[(size_t)n];
      int64_t bits = 0;
      for (int64_t j = 0; j < d; ++j) {
        bits += m[(size_t)n * d + j];
        const float sent = m[(size_t)n * d + j] ? a[(size_t)n * d + j] : 0.0f;
        const float sum = sent + e[(size_t)n * d + j];
        CHECK(std::memcmp(&sum, &a[(size_t)n * d + j], 4) == 0 || (sum == 0.0f && a[(size_t)n * d + j] == 0.0f));
      }
      CHECK(bits == want);
      for (int64_t i = 0; i < want; ++i) {
        const int32_t j = idx[(size_t)n * k + i];
        CHECK(j >= 0 && j < d && m[(size_t)n * d + j] == 1);
        CHECK(i == 0 || idx[(size_t)n * k + i - 1] < j);
        CHECK(std::memcmp(&val[(size_t)n * k + i], &a[(size_t)n * d + j], 4) == 0);
      }
      for (int64_t i = want; i < k; ++i) CHECK(idx[(size_t)n * k + i] == -1 && val[(size_t)n * k + i] == 0.0f);
    }
    rtk_oracle_mask_overlap(h, counts.data());
    int64_t total = 0;
    for (auto c : counts) total += c;
    CHECK(total == d);
    gp = agg;
  }
  std::vector<float> theta((size_t)d, 0.5f);
  rtk_oracle_sgd_update(theta.data(), agg.data(), 0.01f, d);
  rtk_oracle_destroy(h);
}

int main() {
  CHECK(rtk_oracle_create(0, 10, 1, 1.0f) == nullptr && rtk_oracle_create(2, 10, 11, 1.0f) == nullptr);
  CHECK(rtk_oracle_tanh32(0.0f) == 0.0f && rtk_oracle_tanh32(20.0f) == 1.0f);
  std::vector<float> sc = {1.0f, 3.0f, 3.0f, 0.0f, 3.0f};
  std::vector<uint8_t> mk(5);
  rtk_oracle_topk_mask(sc.data(), 5, 2, mk.data());
  CHECK(mk[1] == 1 && mk[2] == 1 && mk[0] + mk[3] + mk[4] == 0);          // lower index first among equals
  int cases = 0;
  for (int pattern = 0; pattern < 4; ++pattern)
    for (int variant = 0; variant < 8; variant += (pattern == 0 ? 1 : 5)) {
      scenario(1, 1, 1, 1.0f, pattern, variant, false, false, 3);
      scenario(3, 37, 5, 0.7f, pattern, variant, true, false, 5);
      scenario(4, 257, 257, 2.0f, pattern, variant, false, true, 4);
      scenario(5, 1000, 33, 0.0f, pattern, variant, true, true, 4);
      scenario(2, 4099, 400, 0.05f, pattern, variant, false, false, 4);
      cases += 5;
    }
  std::printf("oracle under sanitizers: %d scenarios ok\n", cases);
  return 0;
}
