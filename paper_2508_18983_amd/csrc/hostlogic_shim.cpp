// CPU-only test shim around the expert-cache bookkeeping (cache_state.hpp):
// lets the scheduler's decisions be replayed and checked without a GPU.  Built
// with g++ into libsmoe_hostlogic.so; not used by libsmoe itself.
#include <stddef.h>

#include <new>
#include <vector>

#include "cache_state.hpp"
#include "cpu_expert.hpp"
#include "alpha_select.hpp"

using namespace smoe;

struct hl_handle {
  CacheParams p;
  int n_layers;
  int64_t expert_bytes;
  double c_load = 1.0, c_cpu = 1.0;      // costs of Algorithm 2
  std::vector<CacheLayer> layers;
};

extern "C" {

// init_resident: [n_layers][cache_cap] or null for 0..cap-1.  Returns null on bad arguments.
hl_handle* smoe_hl_create(int n_layers, int n_experts, int top_k, int cache_cap, int evict_window,
                          int evict_policy, int n_stage, int64_t expert_bytes, const int32_t* init_resident,
                          float alpha, int prefetch_max, int cpu_assist, double c_load, double c_cpu) {
  if (n_layers < 1 || n_experts < 1 || n_experts > SMOE_MAX_EXPERTS || top_k < 1 || top_k > SMOE_MAX_TOPK ||
      cache_cap < top_k || cache_cap > n_experts || evict_window < 0 || n_stage < 0 ||
      evict_policy < SMOE_EVICT_SCORE || evict_policy > SMOE_EVICT_LFU)
    return nullptr;
  hl_handle* h = new (std::nothrow) hl_handle();
  if (!h) return nullptr;
  h->p = CacheParams{n_experts, top_k, cache_cap, evict_window, evict_policy, n_stage, alpha, prefetch_max,
                     cpu_assist};
  h->c_load = c_load;
  h->c_cpu = c_cpu;
  h->n_layers = n_layers;
  h->expert_bytes = expert_bytes;
  h->layers.resize(n_layers);
  std::vector<int32_t> ids(cache_cap);
  for (int l = 0; l < n_layers; ++l) {
    for (int s = 0; s < cache_cap; ++s) ids[s] = init_resident ? init_resident[(size_t)l * cache_cap + s] : s;
    h->layers[l].reset(h->p, ids.data());
  }
  return h;
}

void smoe_hl_destroy(hl_handle* h) { delete h; }

// topk / final_ / subst: [B][k] int32; scores: [B][E] fp32; inflight: bit mask of prefetched
// experts whose copy is taken to be unfinished.  Outputs (each sized B*k): fetched experts,
// victims (-1 = staged), slots (>= 0 physical slot, < 0 staging), experts left to the host
// cores (count in *n_cpu), prefetched experts taken into the cache with their victims
// (count in *n_adopted), prefetched experts dropped (count in *n_dropped).  Returns the
// number of loads, or a negative SMOE_E* code.
int smoe_hl_step(hl_handle* h, int layer, int B, const int32_t* topk, const int32_t* final_,
                 const int32_t* subst, const float* scores, uint64_t inflight, int32_t* fetched,
                 int32_t* victims, int32_t* slots, int32_t* on_cpu, int32_t* n_cpu, int32_t* adopted,
                 int32_t* adopt_victims, int32_t* n_adopted, int32_t* dropped, int32_t* n_dropped) {
  if (!h || layer < 0 || layer >= h->n_layers || B < 1 || B > SMOE_MAX_BATCH) return SMOE_EINVAL;
  StepDecision d{};
  d.B = B;
  for (int t = 0; t < B; ++t) {
    d.topk[t] = topk + (size_t)t * h->p.top_k;
    d.final_[t] = final_ + (size_t)t * h->p.top_k;
    d.subst[t] = subst + (size_t)t * h->p.top_k;
    d.scores[t] = scores + (size_t)t * h->p.n_experts;
  }
  StepPlan plan;
  const int rc = h->layers[layer].plan_step(h->p, d, h->expert_bytes, plan, h->c_load, h->c_cpu, inflight);
  if (rc != SMOE_OK) return rc;
  for (int i = 0; i < plan.n_cpu; ++i) on_cpu[i] = plan.on_cpu[i];
  *n_cpu = plan.n_cpu;
  for (int i = 0; i < plan.n_fetch; ++i) {
    fetched[i] = plan.fetched[i];
    victims[i] = plan.victims[i];
    slots[i] = plan.slot[i];
  }
  for (int i = 0; i < plan.n_adopted; ++i) {
    adopted[i] = plan.adopted[i];
    adopt_victims[i] = plan.adopt_victims[i];
  }
  *n_adopted = plan.n_adopted;
  for (int i = 0; i < plan.n_dropped; ++i) dropped[i] = plan.dropped[i];
  *n_dropped = plan.n_dropped;
  // every physical slot of the layer is in exactly one place: G, waiting, or spare
  {
    const CacheLayer& ls = h->layers[layer];
    uint64_t seen_lo = 0, seen_hi = 0;
    auto mark = [&](int phys) {
      uint64_t& w = phys < 64 ? seen_lo : seen_hi;
      const uint64_t bit = 1ull << (phys & 63);
      if (w & bit) return false;
      w |= bit;
      return true;
    };
    bool ok = true;
    for (int s = 0; s < h->p.cache_cap; ++s) ok &= mark(ls.phys_of_slot[s]);
    for (int i = 0; i < ls.n_landed; ++i) ok &= mark(ls.landed_slot[i]);
    for (int phys : ls.spare) ok &= mark(phys);
    if (!ok || __builtin_popcountll(seen_lo) + __builtin_popcountll(seen_hi) != h->p.cache_cap + h->p.prefetch_max)
      return SMOE_ESTATE;
  }
  return plan.n_fetch;
}

// Top-score prefetch on predicted scores / top-k ([B][E], [B][k]).  Outputs sized B*k:
// wanted experts and the physical slots of the loaded prefix.  Returns the number put on
// the load queue; *n_wanted gets the number of wanted experts.
int smoe_hl_prefetch(hl_handle* h, int layer, int B, const int32_t* topk, const float* scores,
                     int32_t* wanted, int32_t* n_wanted, int32_t* slots) {
  if (!h || layer < 0 || layer >= h->n_layers || B < 1 || B > SMOE_MAX_BATCH) return SMOE_EINVAL;
  StepDecision d{};
  d.B = B;
  for (int t = 0; t < B; ++t) {
    d.topk[t] = topk + (size_t)t * h->p.top_k;
    d.scores[t] = scores + (size_t)t * h->p.n_experts;
  }
  PrefetchPlan pp;
  h->layers[layer].plan_prefetch(h->p, d, pp);
  for (int i = 0; i < pp.n_wanted; ++i) wanted[i] = pp.wanted[i];
  for (int i = 0; i < pp.n; ++i) slots[i] = pp.slot[i];
  *n_wanted = pp.n_wanted;
  return pp.n;
}

// The host-core expert FFN on its own: yacc[t] += w[t] * FFN_expert(x[t]), x and yacc
// as [ntok][H] fp32 arrays.
void smoe_hl_cpu_expert(const void* expert, int dtype, int H, int F, int ntok, const float* x,
                        const float* w, float* yacc, int n_threads) {
  CpuExperts pool(n_threads);
  const float* xs[SMOE_MAX_BATCH];
  float* ys[SMOE_MAX_BATCH];
  for (int t = 0; t < ntok; ++t) { xs[t] = x + (size_t)t * H; ys[t] = yacc + (size_t)t * H; }
  pool.run(expert, dtype, H, F, ntok, xs, w, ys);
}

// A pool that outlives the call, as libsmoe keeps it.
CpuExperts* smoe_hl_pool_create(int n_threads) { return new (std::nothrow) CpuExperts(n_threads); }
void smoe_hl_pool_destroy(CpuExperts* p) { delete p; }
void smoe_hl_pool_touch(CpuExperts* p, const void* base, size_t bytes) { p->touch(base, bytes); }
void smoe_hl_pool_run(CpuExperts* pool, const void* expert, int dtype, int H, int F, int ntok, const float* x,
                      const float* w, float* yacc) {
  const float* xs[SMOE_MAX_BATCH];
  float* ys[SMOE_MAX_BATCH];
  for (int t = 0; t < ntok; ++t) { xs[t] = x + (size_t)t * H; ys[t] = yacc + (size_t)t * H; }
  pool->run(expert, dtype, H, F, ntok, xs, w, ys);
}

void smoe_hl_residency(const hl_handle* h, int layer, int32_t* out_slots) {
  for (int s = 0; s < h->p.cache_cap; ++s) out_slots[s] = h->layers[layer].expert_of_slot[s];
}

void smoe_hl_stats(const hl_handle* h, int layer, moe_stats_t* out) { *out = h->layers[layer].st; }

// alpha from a latency budget (Section V-C): 0 found, 1 no feasible alpha, -1 bad arguments
int smoe_hl_select_alpha(const double* alphas, const double* tpots, int n, double budget, int degree,
                         int resolution, double* out_alpha, double* out_coef) {
  return select_alpha(alphas, tpots, n, budget, degree, resolution, out_alpha, out_coef);
}

}  // extern "C"
