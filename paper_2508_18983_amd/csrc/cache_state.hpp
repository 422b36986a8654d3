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
  uint64_t before = 0;     // the cache set G when the step started
  uint64_t on_gpu = 0;     // G plus the experts prefetched for this step
  uint64_t shield = 0;     // every expert the step computes
  int n_fetch = 0, n_evict = 0, n_staged = 0;
  int fetched[SMOE_MAX_BATCH * SMOE_MAX_TOPK];   // distinct missing experts, (token, slot) order
  int victims[SMOE_MAX_BATCH * SMOE_MAX_TOPK];   // expert evicted for each, -1 = staged
  int slot[SMOE_MAX_BATCH * SMOE_MAX_TOPK];      // physical slot of the layer, or -(1 + staging index)
  int n_cpu = 0;
  int on_cpu[SMOE_MAX_BATCH * SMOE_MAX_TOPK];    // experts left to the host cores (missing, or prefetched
                                                 // and still in flight)
  int n_adopted = 0;
  int adopted[SMOE_MAX_BATCH * SMOE_MAX_TOPK];        // prefetched experts the step computes, in order
  int adopt_victims[SMOE_MAX_BATCH * SMOE_MAX_TOPK];  // expert evicted for each, -1: not kept
  int adopt_slot[SMOE_MAX_BATCH * SMOE_MAX_TOPK];     // physical slot each is computed from
  int n_dropped = 0;
  int dropped[SMOE_MAX_BATCH * SMOE_MAX_TOPK];        // prefetched experts the step does not wait for
                                                      // (unused, or given to the host cores)
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
  int wanted[SMOE_MAX_BATCH * SMOE_MAX_TOPK];    // predicted top-score experts that are neither resident
                                                 // nor already prefetched
  int experts[SMOE_MAX_BATCH * SMOE_MAX_TOPK];   // the ones put on the load queue (a prefix of wanted)
  int slot[SMOE_MAX_BATCH * SMOE_MAX_TOPK];      // physical (spare) slot each is loaded into
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

// A layer owns cap + prefetch_max physical slots of the slab.  cap of them hold
// the cache set G (logical cache slot s -> physical slot phys_of_slot[s]); the
// others are spare: a prefetched expert is loaded into a spare slot and waits
// there, outside G, for the layer's next step (Section IV-C: a misprediction
// must cost nothing but the baseline).  If that step computes it, the expert
// takes the logical slot of a victim and keeps its physical slot, the victim's
// physical slot becomes spare; if not, it is dropped and its slot is spare again.
struct CacheLayer {
  uint64_t resident = 0;                 // G
  int8_t slot_of[SMOE_MAX_EXPERTS];      // logical cache slot of each member of G
  std::vector<int32_t> expert_of_slot;   // [cap]
  std::vector<int32_t> phys_of_slot;     // [cap] physical slot of each logical slot
  std::vector<int32_t> spare;            // physical slots not in use (a stack)
  int n_landed = 0;                      // experts prefetched for the next step, in load order
  int landed[SMOE_MAX_BATCH * SMOE_MAX_TOPK];
  int landed_slot[SMOE_MAX_BATCH * SMOE_MAX_TOPK];   // their physical slots
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
    n_landed = 0;
    phys_of_slot.resize(p.cache_cap);
    spare.clear();
    for (int s = 0; s < p.cache_cap; ++s) phys_of_slot[s] = s;
    for (int s = p.cache_cap + p.prefetch_max - 1; s >= p.cache_cap; --s) spare.push_back(s);
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

  uint64_t landed_mask() const {
    uint64_t m = 0;
    for (int i = 0; i < n_landed; ++i) m |= 1ull << landed[i];
    return m;
  }
  // Physical slot a member of G is computed from.
  int phys_of_expert(int e) const { return phys_of_slot[slot_of[e]]; }

  // Top-score prefetch (Section IV-C): `d` holds the router's scores and top-k
  // of the *predicted* hidden states.  Predicted top-score experts that are
  // neither in G nor already waiting are put on the load queue in rank order
  // (token by token, repeats skipped), as many as the layer has spare slots
  // left (at most prefetch_max wait at a time).  G, the history and the stamps
  // are not touched.
  void plan_prefetch(const CacheParams& p, const StepDecision& d, PrefetchPlan& out) {
    out = PrefetchPlan{};
    uint64_t listed = resident | landed_mask();
    for (int t = 0; t < d.B; ++t) {
      const uint64_t top = top_score_mask(d.scores[t], d.topk[t], p.n_experts, p.top_k, p.alpha);
      for (int j = 0; j < p.top_k; ++j) {
        const int e = d.topk[t][j];
        if (((top >> e) & 1ull) && !((listed >> e) & 1ull)) {
          listed |= 1ull << e;
          out.wanted[out.n_wanted++] = e;
        }
      }
    }
    for (int i = 0; i < out.n_wanted && n_landed < p.prefetch_max && !spare.empty(); ++i) {
      const int phys = spare.back();
      spare.pop_back();
      landed[n_landed] = out.wanted[i];
      landed_slot[n_landed] = phys;
      ++n_landed;
      out.experts[out.n] = out.wanted[i];
      out.slot[out.n] = phys;
      ++out.n;
      ++st.prefetches;
    }
  }

  // One step: push the scores into the history (before victims are chosen),
  // shield what the step computes, pick a victim for every expert that has to
  // enter G (missing ones and prefetched ones the step computes), update
  // residency and counters.  `inflight`: prefetched experts whose copy has not
  // finished (only read with CPU-assisted scheduling, which may hand them to the
  // host cores).  Returns SMOE_OK; SMOE_ESTATE when the decision is malformed or
  // the step needs more staging slots than exist.  Both are found out before
  // anything is changed: after a refused step the layer's state is what it was
  // before the call.
  int plan_step(const CacheParams& p, const StepDecision& d, int64_t expert_bytes, StepPlan& out,
                double c_load = 1.0, double c_cpu = 1.0, uint64_t inflight = 0) {
    const int E = p.n_experts, k = p.top_k, B = d.B;
    constexpr int kMaxIn = SMOE_MAX_BATCH * SMOE_MAX_TOPK;
    out = StepPlan{};
    out.before = resident;
    const uint64_t waiting_here = landed_mask();
    out.on_gpu = resident | waiting_here;
    // ---- what the step needs, read-only -------------------------------------
    int incoming[kMaxIn], n_in = 0;                     // experts outside G, (token, slot) order
    for (int t = 0; t < B; ++t)
      for (int j = 0; j < k; ++j) {
        const int e = d.final_[t][j];
        const int e0 = d.topk[t][j];
        if (e < 0 || e >= E || e0 < 0 || e0 >= E) return SMOE_ESTATE;
        out.shield |= 1ull << e;
        out.raw_hits += (out.before >> e0) & 1ull;
        out.subs += d.subst[t][j] != 0;
        out.hits += (out.on_gpu >> e) & 1ull;
        if (!((out.before >> e) & 1ull)) {
          bool dup = false;
          for (int i = 0; i < n_in; ++i) dup |= incoming[i] == e;
          if (!dup) incoming[n_in++] = e;
        }
      }
    uint64_t cpu_mask = 0;
    if (p.cpu_assist) {
      // Algorithm 2 over what the step would have to wait for, in descending score (batch 1:
      // slot order is rank order; batch > 1: token by token): the missing experts and the
      // prefetched ones still in flight.  The tail goes to the host cores, which neither
      // load nor cache it.
      int waiting[kMaxIn], n_wait = 0;
      for (int i = 0; i < n_in; ++i) {
        const uint64_t bit = 1ull << incoming[i];
        if (!(waiting_here & bit) || (inflight & bit)) waiting[n_wait++] = incoming[i];
      }
      if (n_wait > 0) {
        const int n_load = p.cpu_assist == 1 ? split_load_cpu(n_wait, c_load, c_cpu)
                                             : split_load_cpu_minmax(n_wait, c_load, c_cpu);
        for (int i = n_load; i < n_wait; ++i) {
          out.on_cpu[out.n_cpu++] = waiting[i];
          cpu_mask |= 1ull << waiting[i];
        }
      }
    }
    {
      // every expert that enters G replaces an unshielded resident; a missing expert that
      // finds none needs a staging slot (a prefetched one is computed where it landed)
      int evictable = __builtin_popcountll(resident & ~out.shield), need_stage = 0;
      for (int i = 0; i < n_in; ++i) {
        const uint64_t bit = 1ull << incoming[i];
        if (cpu_mask & bit) continue;
        if (evictable > 0) --evictable;
        else if (!(waiting_here & bit)) ++need_stage;
      }
      if (need_stage > p.n_stage) return SMOE_ESTATE;
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
      uint64_t stamped = 0;                             // first appearance outside G = the expert's load
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
    st.cpu_computed += out.n_cpu;

    if (n_landed > 0) {
      // prefetch accuracy: was a prefetched expert computed by this step, and was
      // it one of the step's top-score experts
      uint64_t top = 0;
      for (int t = 0; t < B; ++t) top |= top_score_mask(d.scores[t], d.topk[t], E, k, p.alpha);
      st.prefetch_used += __builtin_popcountll(waiting_here & out.shield);
      st.prefetch_top += __builtin_popcountll(waiting_here & top);
    }

    double mean[SMOE_MAX_EXPERTS];
    if (n_in > 0) window_means(p, mean);
    for (int i = 0; i < n_in; ++i) {
      const int m = incoming[i];
      const uint64_t bit = 1ull << m;
      if (cpu_mask & bit) continue;
      const int victim = choose_victim(p, out.shield, mean);
      if (waiting_here & bit) {
        int li = 0;
        while (landed[li] != m) ++li;
        const int phys = landed_slot[li];
        const int a = out.n_adopted++;
        out.adopted[a] = m;
        out.adopt_victims[a] = victim;
        out.adopt_slot[a] = phys;
        if (victim >= 0) {                              // m keeps its physical slot, the victim's is spare
          const int s = slot_of[victim];
          spare.push_back(phys_of_slot[s]);
          phys_of_slot[s] = phys;
          replace(victim, m);
          ++out.n_evict;
        } else {
          spare.push_back(phys);                        // computed where it landed, then given up
        }
      } else {
        const int f = out.n_fetch++;
        out.fetched[f] = m;
        out.victims[f] = victim;
        if (victim >= 0) {
          out.slot[f] = phys_of_slot[replace(victim, m)];
          ++out.n_evict;
        } else {
          out.slot[f] = -(1 + out.n_staged++);          // (checked above: a staging slot is left)
        }
      }
    }
    // prefetched experts the step does not wait for: unused ones, and those the host cores compute
    for (int i = 0; i < n_landed; ++i) {
      const uint64_t bit = 1ull << landed[i];
      if (!(out.shield & bit) || (cpu_mask & bit)) {
        out.dropped[out.n_dropped++] = landed[i];
        spare.push_back(landed_slot[i]);
      }
    }
    n_landed = 0;
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
