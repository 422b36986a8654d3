// Expert-cache bookkeeping of one layer: residency, score history, protection
// shield, victim selection, counters (Section IV-B "Cache eviction", Eq. 3;
// Section V-B dependency 1).  Plain C++ with no HIP dependency, so the same
// code runs inside libsmoe and inside the CPU test shim.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "smoe.h"

namespace smoe {

struct CacheParams {
  int n_experts, top_k, cache_cap, evict_window, evict_policy, n_stage;
  float alpha = 0.0f;        // threshold of the top-score / low-score split
  int prefetch_max = 0;      // experts one prefetch call may load
  int cpu_assist = 0;        // 1: Algorithm 2 splits the misses between loading and the CPU,
                             // 2: the min-max split (variant)
};

// What the router decided for one step (B tokens), as read from the mirror.
struct StepDecision {
  int B;
  const int32_t* topk[SMOE_MAX_BATCH];     // [k] experts by descending score
  const int32_t* final_[SMOE_MAX_BATCH];   // [k] expert per slot after substitution
  const int32_t* subst[SMOE_MAX_BATCH];    // [k] 1 where replaced
  const float* scores[SMOE_MAX_BATCH];     // [E]
};

// What the scheduler has to do for that step.
struct StepPlan {
  uint64_t before = 0;     // residency when the step started
  uint64_t shield = 0;     // every expert the step computes
  int n_fetch = 0, n_evict = 0, n_staged = 0;
  int fetched[SMOE_MAX_BATCH * SMOE_MAX_TOPK];   // distinct missing experts, (token, slot) order
  int victims[SMOE_MAX_BATCH * SMOE_MAX_TOPK];   // expert evicted for each, -1 = staged
  int slot[SMOE_MAX_BATCH * SMOE_MAX_TOPK];      // layer-local cache slot, or -(1 + staging index)
  int n_cpu = 0;
  int on_cpu[SMOE_MAX_BATCH * SMOE_MAX_TOPK];    // distinct missing experts left to the host cores
  int64_t raw_hits = 0, hits = 0, subs = 0;
};

// CPU-assisted task load scheduling (Section V-A, Algorithm 2).  The n missing
// experts of a step, in descending score, are shared out between the load queue
// (which takes from the front of the list) and the host cores (which take from
// the back).  Seen from the two workers: the load queue becomes free at times
// 0, C_load, 2 C_load, ..., the host cores at 0, C_CPU, 2 C_CPU, ...; the next
// expert always goes to the worker that is free first, the load queue when both
// are.  Returns how many experts are loaded; the other n - n_load are computed.
inline int split_load_cpu(int n, double c_load, double c_cpu) {
  int n_load = 0, n_cpu = 0;
  while (n_load + n_cpu < n) {
    if (n_load * c_load <= n_cpu * c_cpu) ++n_load;
    else ++n_cpu;
  }
  return n_load;
}

// What a top-score prefetch has to load (Section IV-C).
struct PrefetchPlan {
  int n_wanted = 0, n = 0;
  int wanted[SMOE_MAX_BATCH * SMOE_MAX_TOPK];    // predicted top-score experts that are not resident
  int experts[SMOE_MAX_BATCH * SMOE_MAX_TOPK];   // the ones loaded (a prefix of wanted)
  int victims[SMOE_MAX_BATCH * SMOE_MAX_TOPK];   // expert evicted for each
  int slot[SMOE_MAX_BATCH * SMOE_MAX_TOPK];      // layer-local cache slot of each
};

// Active experts of one token whose score reaches T = (1 + alpha) * S_{k+1}
// (Algorithm 1's threshold; all of them when there is no (k+1)-th expert).
inline uint64_t top_score_mask(const float* scores, const int32_t* topk, int E, int k, float alpha) {
  uint64_t active = 0;
  for (int j = 0; j < k; ++j) active |= 1ull << topk[j];
  if (E <= k) return active;
  double s_k1 = -1.0;
  for (int e = 0; e < E; ++e)
    if (!((active >> e) & 1ull) && (double)scores[e] > s_k1) s_k1 = (double)scores[e];
  const double T = (1.0 + (double)alpha) * s_k1;
  uint64_t top = 0;
  for (int j = 0; j < k; ++j)
    if ((double)scores[topk[j]] >= T) top |= 1ull << topk[j];
  return top;
}

// Variant (cpu_assist = 2): the stated objective min max(n_load C_load, n_CPU C_CPU)
// solved over all n+1 splits; of equally good splits the one that loads more.
inline int split_load_cpu_minmax(int n, double c_load, double c_cpu) {
  int best_i = 0;
  double best_t = -1.0;
  for (int i = 0; i <= n; ++i) {
    const double tl = i * c_load, tc = (n - i) * c_cpu;
    const double t = tl > tc ? tl : tc;
    if (best_t < 0.0 || t <= best_t) { best_i = i; best_t = t; }
  }
  return best_i;
}

struct CacheLayer {
  uint64_t resident = 0;
  uint64_t prefetched = 0;               // prefetched since the layer's last step, not yet judged
  int8_t slot_of[SMOE_MAX_EXPERTS];
  std::vector<int32_t> expert_of_slot;   // [cap]
  std::vector<double> hist;              // ring [(n+1)][E] of batch-mean score vectors
  int hist_count = 0, hist_head = 0;
  int64_t step = 0;                      // steps of this layer so far
  int64_t last_use[SMOE_MAX_EXPERTS];    // stamp of the latest use (recency policies)
  int64_t load_stamp[SMOE_MAX_EXPERTS];  // stamp of the load that brought the expert in
  int64_t use_count[SMOE_MAX_EXPERTS];   // uses since that load
  moe_stats_t st{};

  // Initial residency: expert ids per slot (distinct, validated by the caller).
  void reset(const CacheParams& p, const int32_t* init_ids) {
    resident = 0;
    prefetched = 0;
    for (int e = 0; e < SMOE_MAX_EXPERTS; ++e) {
      slot_of[e] = -1;
      last_use[e] = load_stamp[e] = use_count[e] = 0;
    }
    expert_of_slot.assign(p.cache_cap, -1);
    hist.assign((size_t)(p.evict_window + 1) * p.n_experts, 0.0);
    hist_count = hist_head = 0;
    step = 0;
    st = moe_stats_t{};
    for (int s = 0; s < p.cache_cap; ++s) {
      const int e = init_ids[s];
      resident |= 1ull << e;
      slot_of[e] = (int8_t)s;
      expert_of_slot[s] = e;
      last_use[e] = load_stamp[e] = (int64_t)s - p.cache_cap;   // before step 0, in slot order
    }
  }

  // Mean score of every expert over the retained window (Eq. 3); zeros while
  // the layer has no history.
  void window_means(const CacheParams& p, double* mean) const {
    for (int e = 0; e < p.n_experts; ++e) {
      double s = 0.0;
      for (int i = 0; i < hist_count; ++i) s += hist[(size_t)i * p.n_experts + e];
      mean[e] = hist_count ? s / hist_count : 0.0;
    }
  }

  // Victim among the resident experts outside `shield` under the configured
  // policy, lower id on ties; -1 when nothing is evictable.
  int choose_victim(const CacheParams& p, uint64_t shield, const double* mean) const {
    int victim = -1;
    for (int e = 0; e < p.n_experts; ++e) {
      if (!((resident >> e) & 1ull) || ((shield >> e) & 1ull)) continue;
      if (victim < 0) { victim = e; continue; }
      bool better;
      switch (p.evict_policy) {
        case SMOE_EVICT_LRU:  better = last_use[e] < last_use[victim]; break;
        case SMOE_EVICT_FIFO: better = load_stamp[e] < load_stamp[victim]; break;
        case SMOE_EVICT_LFU:
          better = use_count[e] < use_count[victim] ||
                   (use_count[e] == use_count[victim] && last_use[e] < last_use[victim]);
          break;
        default:              better = mean[e] < mean[victim]; break;   // Eq. 3
      }
      if (better) victim = e;
    }
    return victim;
  }

  // Expert m takes the cache slot of `victim`.
  int replace(int victim, int m) {
    const int s = slot_of[victim];
    resident = (resident & ~(1ull << victim)) | (1ull << m);
    slot_of[victim] = -1;
    slot_of[m] = (int8_t)s;
    expert_of_slot[s] = m;
    return s;
  }

  // Top-score prefetch (Section IV-C): `d` holds the router's scores and top-k
  // of the *predicted* hidden states.  Predicted top-score experts that are not
  // resident are loaded in rank order (token by token, repeats skipped), at most
  // prefetch_max of them; every predicted active expert is shielded while the
  // victims are chosen; loading stops when nothing is evictable.
  void plan_prefetch(const CacheParams& p, const StepDecision& d, PrefetchPlan& out) {
    out = PrefetchPlan{};
    uint64_t shield = 0, listed = 0;
    for (int t = 0; t < d.B; ++t) {
      const uint64_t top = top_score_mask(d.scores[t], d.topk[t], p.n_experts, p.top_k, p.alpha);
      for (int j = 0; j < p.top_k; ++j) {
        const int e = d.topk[t][j];
        shield |= 1ull << e;
        if (((top >> e) & 1ull) && !((resident >> e) & 1ull) && !((listed >> e) & 1ull)) {
          listed |= 1ull << e;
          out.wanted[out.n_wanted++] = e;
        }
      }
    }
    double mean[SMOE_MAX_EXPERTS];
    window_means(p, mean);
    const int64_t stamp = step * 64 - 1;              // just before the layer's next step
    for (int i = 0; i < out.n_wanted && i < p.prefetch_max; ++i) {
      const int victim = choose_victim(p, shield, mean);
      if (victim < 0) break;
      const int m = out.wanted[i];
      out.experts[out.n] = m;
      out.victims[out.n] = victim;
      out.slot[out.n] = replace(victim, m);
      ++out.n;
      load_stamp[m] = last_use[m] = stamp;
      use_count[m] = 0;
      prefetched |= 1ull << m;
      ++st.evictions;
      ++st.prefetches;
    }
  }

  // One step: push the scores into the history (before victims are chosen),
  // shield what the step computes, pick a victim for every distinct missing
  // expert, update residency and counters.  Returns SMOE_OK; SMOE_ESTATE when
  // the decision is malformed or the step needs more staging slots than exist.
  // Both are found out before anything is changed: after a refused step the
  // layer's state is what it was before the call.
  int plan_step(const CacheParams& p, const StepDecision& d, int64_t expert_bytes, StepPlan& out,
                double c_load = 1.0, double c_cpu = 1.0) {
    const int E = p.n_experts, k = p.top_k, B = d.B;
    out = StepPlan{};
    out.before = resident;
    // ---- what the step needs, read-only -------------------------------------
    for (int t = 0; t < B; ++t)
      for (int j = 0; j < k; ++j) {
        const int e = d.final_[t][j];
        const int e0 = d.topk[t][j];
        if (e < 0 || e >= E || e0 < 0 || e0 >= E) return SMOE_ESTATE;
        out.shield |= 1ull << e;
        out.raw_hits += (out.before >> e0) & 1ull;
        out.subs += d.subst[t][j] != 0;
        if ((out.before >> e) & 1ull) {
          ++out.hits;
        } else {
          bool dup = false;
          for (int i = 0; i < out.n_fetch; ++i) dup |= out.fetched[i] == e;
          if (!dup) out.fetched[out.n_fetch++] = e;
        }
      }
    int n_load = out.n_fetch;
    if (p.cpu_assist && out.n_fetch > 0) {
      // the distinct misses are in descending score (batch 1: slot order is rank order;
      // batch > 1: token by token): the tail goes to the host cores, which neither
      // load nor cache it
      n_load = p.cpu_assist == 1 ? split_load_cpu(out.n_fetch, c_load, c_cpu)
                                 : split_load_cpu_minmax(out.n_fetch, c_load, c_cpu);
    }
    {
      // every load needs an unshielded resident to replace, or a staging slot
      const int evictable = __builtin_popcountll(resident & ~out.shield);
      if (n_load - evictable > p.n_stage) return SMOE_ESTATE;
    }

    // ---- from here on the state changes --------------------------------------
    {
      double* row = &hist[(size_t)hist_head * E];
      for (int e = 0; e < E; ++e) {
        double s = 0.0;
        for (int t = 0; t < B; ++t) s += (double)d.scores[t][e];
        row[e] = s / B;
      }
      hist_head = (hist_head + 1) % (p.evict_window + 1);
      if (hist_count < p.evict_window + 1) ++hist_count;
    }
    {
      uint64_t stamped = 0;                             // first appearance of a missing expert = its load
      for (int t = 0; t < B; ++t)
        for (int j = 0; j < k; ++j) {
          const int e = d.final_[t][j];
          const int64_t stamp = step * 64 + (int64_t)t * k + j;
          if (!((out.before >> e) & 1ull) && !((stamped >> e) & 1ull)) {
            stamped |= 1ull << e;
            load_stamp[e] = stamp;
            use_count[e] = 0;
          }
          last_use[e] = stamp;
          ++use_count[e];
        }
    }
    ++step;

    if (n_load < out.n_fetch) {
      for (int i = n_load; i < out.n_fetch; ++i) out.on_cpu[out.n_cpu++] = out.fetched[i];
      out.n_fetch = n_load;
      st.cpu_computed += out.n_cpu;
    }

    if (prefetched) {
      // prefetch accuracy: was a prefetched expert computed by this step, and was
      // it one of the step's top-score experts
      uint64_t top = 0;
      for (int t = 0; t < B; ++t) top |= top_score_mask(d.scores[t], d.topk[t], E, k, p.alpha);
      st.prefetch_used += __builtin_popcountll(prefetched & out.shield);
      st.prefetch_top += __builtin_popcountll(prefetched & top);
      prefetched = 0;
    }

    if (out.n_fetch > 0) {
      double mean[SMOE_MAX_EXPERTS];
      window_means(p, mean);
      for (int i = 0; i < out.n_fetch; ++i) {
        const int victim = choose_victim(p, out.shield, mean);
        out.victims[i] = victim;
        const int m = out.fetched[i];
        if (victim >= 0) {
          out.slot[i] = replace(victim, m);
          ++out.n_evict;
        } else {
          out.slot[i] = -(1 + out.n_staged++);          // (checked above: a staging slot is left)
        }
      }
    }
    st.tokens += B;
    st.slots += (int64_t)B * k;
    st.raw_hits += out.raw_hits;
    st.hits += out.hits;
    st.misses += (int64_t)B * k - out.hits;
    st.substitutions += out.subs;
    st.evictions += out.n_evict;
    st.staged += out.n_staged;
    st.fetches += out.n_fetch;
    st.bytes_fetched += (int64_t)out.n_fetch * expert_bytes;
    return SMOE_OK;
  }
};

}  // namespace smoe
