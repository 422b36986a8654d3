// Selection stage of the router, as device functions one wavefront executes
// with all 64 lanes active: softmax over the routed experts, top-(k+1) by rank
// counting, the alpha classes of Algorithm 1, the substitution of non-resident
// low-score experts (Section IV-B), and the decision record.  Used by the
// stand-alone selection kernel and by the prologue of the batch-1 up kernel.
//
// Input: the partial dot products the gate GEMV kernel left in device memory,
// part[(token * E + expert) * kMaxGateSeg + segment]; the segments of a row are
// added in index order, so the logits do not depend on which kernel adds them.
#pragma once
#include "smoe_dev.hpp"
#include "wave_ops.hpp"

namespace smoe {

// Shared memory of the selection; NB = tokens it can hold.
template <int NB>
struct SelectSmem {
  alignas(16) float lg[NB][kWave];   // logits; lanes >= E hold -inf
  float sc[NB][kWave];               // scores
  int rk[NB][kWave];                 // rank of each expert
  int tk[NB][SMOE_MAX_TOPK];         // E_a by rank
  unsigned long long top_m[NB];      // top-score experts of each token (read by the other tokens' waves
                                     // after a block barrier)
  int slot_of[kWave];                // cache slot of each expert (-1: not computable from the cache now)
  int fin[NB][SMOE_MAX_TOPK];        // final expert per (token, slot)
  int slt[NB][SMOE_MAX_TOPK];        // its cache slot, -1 when it has to be loaded
  float wsl[NB][SMOE_MAX_TOPK];      // combine weight per (token, slot)
};

template <> struct SelectSmem<0> {};

// Lanes of one wave hand data to each other through LDS: the stores before this
// point are ordered before the loads after it.  The hardware executes a wave's
// LDS instructions in order; the fences keep the compiler from moving a load
// above another lane's store, which it may otherwise do (a single thread never
// observes the difference).  Generates no instructions beyond a wait.
__device__ __forceinline__ void wave_lds_handoff() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// What pass 1 leaves for pass 2 besides shared memory (uniform over the wave).
struct TokenClasses {
  unsigned long long top_m;          // top-score experts: active with s >= T = (1 + alpha) S_{k+1}
  float R;                           // (1 - alpha) S_{k+1}
};

// Workspace of the expert grouping of a batched step (stand-alone kernel only).
struct GroupSmem {
  int pair_e[kWave];                          // expert of (token, slot) pair t * k + j
  int gcnt[kWave];                            // tokens per expert
  int gtok[kWave][SMOE_MAX_BATCH];            // their tokens, ascending
  float gw[kWave][SMOE_MAX_BATCH];            // and combine weights
};

// Logit of expert `lane` for token `tok` from the GEMV kernel's partial sums
// (rows of kMaxGateSeg floats: two 128-bit loads, issued together), segments
// added in index order.
__device__ __forceinline__ float logit_from_parts(const RouteArgs& a, int lane, int tok) {
  if (lane >= a.E) return -INFINITY;
  const float4* p = reinterpret_cast<const float4*>(a.gate_part + ((size_t)tok * a.E + lane) * kMaxGateSeg);
  const float4 lo = p[0];
  const float4 hi = a.nseg > 4 ? p[1] : float4{0.f, 0.f, 0.f, 0.f};
  float v = lo.x;
  if (a.nseg > 1) v += lo.y;
  if (a.nseg > 2) { v += lo.z; v += lo.w; }
  if (a.nseg > 4) { v += hi.x; v += hi.y; v += hi.z; v += hi.w; }
  return v;
}

// Rank of this lane's expert in (logit descending, id ascending) order = the number of
// experts that precede it.  The logit becomes an order-preserving 32-bit integer and every lane
// counts the larger ones, which arrive by lane broadcast: 64 x (v_readlane, compare, add), no
// memory access.  (E reads of the logits from LDS, one per loop trip, took 2.0 us of the 2.9 us
// the selection took in the up kernel's prologue; k+1 dependent wave-wide arg-max rounds are
// slower still.)  Equal logits leave equal counts, and then the counts of the E real experts no
// longer add up to 0 + 1 + ... + (E-1): only then the count is redone with 64-bit keys that
// carry 63 - id in their low bits, so that the lower id wins the tie.  Lanes >= E hold -inf and
// precede nobody.
__device__ __forceinline__ int rank_by_logit(float l, int lane, int E) {
  const float lz = l + 0.0f;                                     // -0 and +0 tie
  unsigned ub = __float_as_uint(lz);
  ub = (ub & 0x80000000u) ? ~ub : (ub | 0x80000000u);
  int myrank = 0;
#pragma unroll
  for (int j = 0; j < kWave; ++j) myrank += (unsigned)__builtin_amdgcn_readlane((int)ub, j) > ub;
  const float total = wave_sum(lane < E ? (float)myrank : 0.f);  // (exact: at most 2016)
  if (total != (float)(E * (E - 1) / 2)) {                       // ties among the real experts: rare
    const unsigned key_hi = ub >> 26, key_lo = (ub << 6) | (unsigned)(63 - lane);
    const unsigned long long key = ((unsigned long long)key_hi << 32) | key_lo;
    myrank = 0;
    for (int j = 0; j < kWave; ++j) {
      const unsigned long long kj = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)key_hi, j) << 32) |
                                    (unsigned)__builtin_amdgcn_readlane((int)key_lo, j);
      myrank += kj > key;
    }
  }
  return myrank;
}

// Scores, top-(k+1), alpha classes of one token.
template <int NB>
__device__ __forceinline__ TokenClasses select_pass1(const RouteArgs& a, SelectSmem<NB>& sm, int lane, int row) {
  const int E = a.E, k = a.k;
  const bool has_pivot = E > k;
  const bool in = lane < E;
  const float l = sm.lg[row][lane];
  const float m = wave_max(l);
  const float p = in ? expf(l - m) : 0.f;
  const float s = p / wave_sum(p);
  int myrank = rank_by_logit(l, lane, E);
  if (!in) myrank = 127;
  if (lane < k) sm.tk[row][lane] = lane;               // defined even if the logits are not numbers
  wave_lds_handoff();
  if (myrank < k) sm.tk[row][myrank] = lane;
  const unsigned long long pivot_m = __ballot(has_pivot && myrank == k);
  const int pivot = pivot_m ? (int)__ffsll((long long)pivot_m) - 1 : -1;
  float R = 0.f;
  bool top = myrank < k;
  if (has_pivot) {
    const float s_k1 = __shfl(s, pivot, kWave);
    const float T_hi = (1.0f + a.alpha) * s_k1;
    R = (1.0f - a.alpha) * s_k1;
    top = top && (s >= T_hi);
  }
  const unsigned long long top_m = __ballot(top);
  sm.sc[row][lane] = s;
  sm.rk[row][lane] = myrank;
  wave_lds_handoff();
  return TokenClasses{top_m, R};
}

// Substitution of one token against residency and the batch top-score set
// `c_mask`; leaves final expert, slot and weight of every slot in shared
// memory and, with `emit`, writes the token's decision record to device memory
// and to the host mirror.
template <int NB>
__device__ __forceinline__ void select_pass2(const RouteArgs& a, SelectSmem<NB>& sm, const TokenClasses& cls,
                                             unsigned long long c_mask, int lane, int tok, int row, bool emit) {
  const int E = a.E, k = a.k;
  const bool has_pivot = E > k;
  const unsigned long long avail = a.resident | c_mask;
  const float s = sm.sc[row][lane];
  const int myrank = sm.rk[row][lane];
  const bool active = myrank < k;
  const unsigned long long top_m = cls.top_m;
  const float R = cls.R;
  const bool is_avail = (avail >> lane) & 1ull;
  const unsigned long long need_m = __ballot(active && !((top_m >> lane) & 1ull) && !is_avail);
  unsigned long long cand_m = has_pivot ? __ballot(lane < E && !active && is_avail && s >= R) : 0ull;
  const int mytop = lane < k ? sm.tk[row][lane] : -1;   // lane r owns slot r
  int myfin = mytop, mysub = 0;
  if (need_m && cand_m) {
    for (int r = k - 1; r >= 0; --r) {                  // lowest-scoring active first
      const int b = __shfl(mytop, r, kWave);
      if (!((need_m >> b) & 1ull)) continue;
      if (!cand_m) break;
      const bool is_cand = (cand_m >> lane) & 1ull;
      float key = s;
      if (a.subst_key == 0) key = is_cand ? a.sim[(size_t)b * E + lane] : 0.f;
      const int c = wave_argmax(key, is_cand, lane);
      if (lane == r) { myfin = c; mysub = 1; }
      cand_m &= ~(1ull << c);
    }
  }
  float w = lane < k ? sm.sc[row][mytop] : 0.f;
  const float wsum = wave_sum(w);
  if (a.renorm) w = w / wsum;
  if (lane < k) {
    const int slot = ((a.resident >> myfin) & 1ull) ? sm.slot_of[myfin] : -1;
    sm.fin[row][lane] = myfin;
    sm.slt[row][lane] = slot;
    sm.wsl[row][lane] = w;
    if (emit) {
      TokRec* d = &a.rec_dev->tok[tok];
      TokRec* hrec = &a.rec_host->tok[tok];
      d->topk[lane] = mytop;   hrec->topk[lane] = mytop;
      d->final_[lane] = myfin; hrec->final_[lane] = myfin;
      d->slot[lane] = slot;    hrec->slot[lane] = slot;
      d->subst[lane] = mysub;  hrec->subst[lane] = mysub;
      d->w[lane] = w;          hrec->w[lane] = w;
    }
  }
  if (emit) a.rec_host->tok[tok].scores[lane] = lane < E ? s : 0.f;
}

// Last step, one wave, after every token's pass 2: the hidden states for the
// host cores (CPU-assisted scheduling only), then the call number, which tells
// the host that the mirror is complete.
__device__ __forceinline__ void publish_seq(const RouteArgs& a, int lane) {
  typedef unsigned int pu32x4 __attribute__((ext_vector_type(4)));
  if (a.x_mirror != nullptr) {
    const pu32x4* src = static_cast<const pu32x4*>(a.x);
    pu32x4* dst = static_cast<pu32x4*>(a.x_mirror);
    for (int u = lane; u < a.x_units; u += kWave) dst[u] = src[u];
  }
  // every store of this wave to the mirror is complete before seq changes
  __threadfence_system();
  if (lane == 0) __hip_atomic_store(&a.rec_host->seq, a.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// The whole selection of a batch-1 call by one wave.  `slot_of_lane` and
// `logit` are this lane's entries of the slot table and of the logits, loaded
// by the caller (so that it can issue those loads early).
__device__ __forceinline__ void select_single(const RouteArgs& a, SelectSmem<1>& sm, int lane, int slot_of_lane,
                                              float logit, bool emit) {
  sm.slot_of[lane] = slot_of_lane;
  sm.lg[0][lane] = logit;
  wave_lds_handoff();
  const TokenClasses cls = select_pass1(a, sm, lane, 0);
  select_pass2(a, sm, cls, cls.top_m, lane, 0, 0, emit);
  if (emit) publish_seq(a, lane);
}

// What one routed slot of a batch-1 call computes -- final expert of slot j, its cache slot (-1:
// to be loaded) and its combine weight -- by one wave, in registers only: the same steps as
// select_pass1 / select_pass2 (same arithmetic, same order of the weight sum, hence the same
// bits), with the hand-offs through LDS replaced by ballots and lane broadcasts.  The blocks
// of the up kernel that do not have to write the decision record use this; results are uniform
// over the wave.
__device__ __forceinline__ void select_slot_in_registers(const RouteArgs& a, int lane, int slot_of_lane, float l,
                                                         int j, int& expert, int& slot, float& wgt) {
  const int E = a.E, k = a.k;
  const bool has_pivot = E > k;
  const bool in = lane < E;
  const float m = wave_max(l);
  const float p = in ? expf(l - m) : 0.f;
  const float s = p / wave_sum(p);
  int myrank = rank_by_logit(l, lane, E);
  if (!in) myrank = 127;
  int t[SMOE_MAX_TOPK];                                 // E_a by rank (uniform values)
#pragma unroll
  for (int r = 0; r < SMOE_MAX_TOPK; ++r) {
    const unsigned long long mr = __ballot(myrank == r);
    t[r] = (r < k && mr) ? (int)__ffsll((long long)mr) - 1 : r;
  }
  float R = 0.f;
  bool top = myrank < k;
  if (has_pivot) {
    const unsigned long long pivot_m = __ballot(myrank == k);
    const int pivot = pivot_m ? (int)__ffsll((long long)pivot_m) - 1 : 0;
    const float s_k1 = lane_f(s, pivot);
    const float T_hi = (1.0f + a.alpha) * s_k1;
    R = (1.0f - a.alpha) * s_k1;
    top = top && (s >= T_hi);
  }
  const unsigned long long top_m = __ballot(top);
  const unsigned long long avail = a.resident | top_m;
  const bool active = myrank < k;
  const bool is_avail = (avail >> lane) & 1ull;
  const unsigned long long need_m = __ballot(active && !((top_m >> lane) & 1ull) && !is_avail);
  unsigned long long cand_m = has_pivot ? __ballot(in && !active && is_avail && s >= R) : 0ull;
  int fin[SMOE_MAX_TOPK];
#pragma unroll
  for (int r = 0; r < SMOE_MAX_TOPK; ++r) fin[r] = t[r];
  if (need_m && cand_m) {
#pragma unroll
    for (int r = SMOE_MAX_TOPK - 1; r >= 0; --r) {      // lowest-scoring active first
      if (r >= k) continue;
      const int b = t[r];
      if (!((need_m >> b) & 1ull)) continue;
      if (!cand_m) continue;
      const bool is_cand = (cand_m >> lane) & 1ull;
      float key = s;
      if (a.subst_key == 0) key = is_cand ? a.sim[(size_t)b * E + lane] : 0.f;
      const int c = wave_argmax(key, is_cand, lane);
      fin[r] = c;
      cand_m &= ~(1ull << c);
    }
  }
  // lane r < k holds the score of the expert ranked r: the same operands, in the same lanes, as
  // the weight sum of select_pass2
  float w = 0.f;
#pragma unroll
  for (int r = 0; r < SMOE_MAX_TOPK; ++r) {
    const float sr = lane_f(s, t[r]);
    if (r < k && lane == r) w = sr;
  }
  const float wsum = wave_sum(w);
  if (a.renorm) w = w / wsum;
  expert = 0;
#pragma unroll
  for (int r = 0; r < SMOE_MAX_TOPK; ++r)
    if (r == j) expert = fin[r];
  wgt = lane_f(w, j);
  slot = ((a.resident >> expert) & 1ull) ? __builtin_amdgcn_readlane(slot_of_lane, expert) : -1;
}

}  // namespace smoe
