// Driver for sanitizer builds of the library's HIP-free host code: the expert
// cache scheduler (cache_state.hpp), the host-core expert FFN and its thread
// pool (cpu_expert.cpp) and the alpha selection (alpha_select.hpp).  It feeds
// them seeded random but well-formed inputs over every policy, batch size and
// scheduling mode and checks the structural invariants; what it is for is run
// under -fsanitize=address,undefined and -fsanitize=thread (tests/test_sanitizers.py).
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "alpha_select.hpp"
#include "cache_state.hpp"
#include "cpu_expert.hpp"

using namespace smoe;

namespace {

struct Rng {
  uint64_t s;
  uint32_t next() { s = s * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(s >> 33); }
  int below(int n) { return (int)(next() % (uint32_t)n); }
  float unit() { return (next() & 0xffffff) / 16777216.0f; }
};

#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) { std::fprintf(stderr, "CHECK failed: %s (line %d)\n", #cond, __LINE__); std::exit(3); } \
  } while (0)

int popcount(uint64_t v) { return __builtin_popcountll(v); }

void scheduler_run(Rng& rng, int E, int k, int cap, int B, int policy, int window, int n_stage, int cpu_assist,
                   int prefetch_max) {
  CacheParams p{E, k, cap, window, policy, n_stage, 0.25f, prefetch_max, cpu_assist};
  CacheLayer layer;
  std::vector<int32_t> ids(cap);
  for (int s = 0; s < cap; ++s) ids[s] = s;
  layer.reset(p, ids.data());
  std::vector<int32_t> topk(B * k), fin(B * k), sub(B * k);
  std::vector<float> sc((size_t)B * E);
  int64_t refused = 0;
  for (int step = 0; step < 200; ++step) {
    StepDecision d{};
    d.B = B;
    for (int t = 0; t < B; ++t) {
      float tot = 0.f;
      for (int e = 0; e < E; ++e) { sc[(size_t)t * E + e] = 0.01f + rng.unit(); tot += sc[(size_t)t * E + e]; }
      for (int e = 0; e < E; ++e) sc[(size_t)t * E + e] /= tot;
      uint64_t used = 0;
      for (int j = 0; j < k; ++j) {                     // distinct experts per token
        int e;
        do { e = rng.below(E); } while ((used >> e) & 1ull);
        used |= 1ull << e;
        topk[t * k + j] = e;
        fin[t * k + j] = e;
        sub[t * k + j] = 0;
      }
      d.topk[t] = &topk[t * k]; d.final_[t] = &fin[t * k]; d.subst[t] = &sub[t * k]; d.scores[t] = &sc[(size_t)t * E];
    }
    if (prefetch_max && (step & 1)) {
      PrefetchPlan pp;
      layer.plan_prefetch(p, d, pp);
      CHECK(pp.n <= prefetch_max && pp.n <= pp.n_wanted);
      CHECK(popcount(layer.resident) == cap);
    }
    const moe_stats_t before = layer.st;
    const uint64_t res_before = layer.resident;
    StepPlan plan;
    const int rc = layer.plan_step(p, d, 1000, plan, 1.0 + rng.below(3), 1.0 + rng.below(3));
    if (rc != SMOE_OK) {
      ++refused;
      CHECK(rc == SMOE_ESTATE);
      CHECK(std::memcmp(&before, &layer.st, sizeof(before)) == 0 && res_before == layer.resident);
      continue;
    }
    CHECK(popcount(layer.resident) == cap);
    CHECK(plan.n_staged <= n_stage);
    for (int i = 0; i < plan.n_fetch; ++i) {
      CHECK(plan.victims[i] < 0 || !((plan.shield >> plan.victims[i]) & 1ull));   // the shield holds
      CHECK((plan.slot[i] >= 0) == (plan.victims[i] >= 0));
    }
    for (int s = 0; s < cap; ++s) CHECK(layer.slot_of[layer.expert_of_slot[s]] == s);
    CHECK(layer.st.hits + layer.st.misses == layer.st.slots);
  }
  (void)refused;
}

void cpu_expert_run(Rng& rng, int threads) {
  CpuExperts pool(threads);
  for (int rep = 0; rep < 6; ++rep) {
    const int H = 8 * (1 + rng.below(24)), F = 8 * (1 + rng.below(40)), ntok = 1 + rng.below(8);
    const int dtype = rep & 1;
    const size_t n = 3 * (size_t)H * F;
    std::vector<float> w32;
    std::vector<uint16_t> w16;
    if (dtype == 0) { w32.resize(n); for (auto& v : w32) v = (rng.unit() - 0.5f) * 0.1f; }
    else { w16.resize(n); for (auto& v : w16) { float f = (rng.unit() - 0.5f) * 0.1f; uint32_t u; std::memcpy(&u, &f, 4); v = (uint16_t)(u >> 16); } }
    std::vector<float> x((size_t)ntok * H), y((size_t)ntok * H, 0.f), wt(ntok);
    for (auto& v : x) v = rng.unit() - 0.5f;
    for (auto& v : wt) v = rng.unit();
    const float* xs[8]; float* ys[8];
    for (int t = 0; t < ntok; ++t) { xs[t] = &x[(size_t)t * H]; ys[t] = &y[(size_t)t * H]; }
    const void* expert = dtype == 0 ? (const void*)w32.data() : (const void*)w16.data();
    pool.touch(expert, n * (dtype == 0 ? 4 : 2));
    pool.run(expert, dtype, H, F, ntok, xs, wt.data(), ys);
    pool.run(expert, dtype, H, F, ntok, xs, wt.data(), ys);
    // reference for token 0, plain loops (two runs accumulate twice)
    std::vector<double> a(F), ref(H, 0.0);
    auto W = [&](size_t i) -> double {
      if (dtype == 0) return w32[i];
      uint32_t u = (uint32_t)w16[i] << 16; float f; std::memcpy(&f, &u, 4); return f;
    };
    for (int f = 0; f < F; ++f) {
      double g = 0, u = 0;
      for (int h = 0; h < H; ++h) { g += W((size_t)f * H + h) * x[h]; u += W((size_t)(F + f) * H + h) * x[h]; }
      a[f] = g / (1.0 + std::exp(-g)) * u;
    }
    for (int h = 0; h < H; ++h) {
      double s = 0;
      for (int f = 0; f < F; ++f) s += W(2 * (size_t)F * H + (size_t)h * F + f) * a[f];
      ref[h] = 2.0 * wt[0] * s;
    }
    double num = 0, den = 1e-30;
    for (int h = 0; h < H; ++h) { num += (y[h] - ref[h]) * (y[h] - ref[h]); den += ref[h] * ref[h]; }
    CHECK(num <= 1e-8 * den + 1e-20);
  }
}

void alpha_run(Rng& rng) {
  for (int rep = 0; rep < 200; ++rep) {
    const int n = 2 + rng.below(10), degree = rng.below(n < 7 ? n : 7);
    double a[12], t[12], coef[kMaxPolyDegree + 1], out = -1.0;
    for (int i = 0; i < n; ++i) { a[i] = 0.05 * i + 0.01 * rng.unit(); t[i] = 100.0 - 60.0 * a[i] + rng.unit(); }
    const int rc = select_alpha(a, t, n, 80.0 + 30.0 * rng.unit(), degree, 2 + rng.below(500), &out, coef);
    CHECK(rc == 0 || rc == 1 || rc == -1);
    if (rc == 0) CHECK(out >= a[0] - 1e-12 && out <= a[n - 1] + 1e-12);
  }
}

}  // namespace

int main() {
  Rng rng{20261128};
  for (int policy = SMOE_EVICT_SCORE; policy <= SMOE_EVICT_LFU; ++policy)
    for (int B : {1, 3, 8})
      for (int assist : {0, 1, 2}) {
        scheduler_run(rng, 8, 2, 4, B, policy, 3, B > 1 ? 4 : 0, assist, 0);
        scheduler_run(rng, 64, 8, 32, B, policy, 0, B * 8, assist, 3);
        scheduler_run(rng, 5, 5, 5, B, policy, 7, 0, assist, 2);
      }
  for (int threads : {1, 3, 8}) cpu_expert_run(rng, threads);
  alpha_run(rng);
  std::puts("host code: ok");
  return 0;
}
