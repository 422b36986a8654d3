// Router + expert-cache router on the GPU, one launch per layer call.
//
//   gate GEMV -> softmax over the routed experts -> top-(k+1)   (Section II-A,
//                                                     Algorithm 1 "Sort S_t desc")
//   T = (1+alpha) S_{k+1}, R = (1-alpha) S_{k+1}, top-score / low-score classes,
//   substitution of non-resident low-score experts by resident (or batch
//   top-score) inactive experts inside the score band       (Algorithm 1 and
//                                                     Section IV-B prose)
//
// The paper runs this search on the CPU; here one wavefront holds one expert
// per lane (E <= 64), the residency set is a 64-bit mask passed by value, and
// every set operation is a ballot.  The gate GEMV is spread over the 16 waves
// of the block.  Decisions go to device memory for the FFN kernels and to a
// pinned host mirror for the cache scheduler.
#include "smoe_dev.hpp"
#include "wave_ops.hpp"

namespace smoe {
namespace {

struct bf16_t { uint16_t v; };

template <typename T> struct GateUnit;
typedef unsigned int gu32x4 __attribute__((ext_vector_type(4)));
typedef float gf32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 gbf16x2 __attribute__((ext_vector_type(2)));

template <> struct GateUnit<float> {
  static constexpr int N = 4;
  using raw = gf32x4;
  __device__ static __forceinline__ float dot(const raw& w, const raw& x, float acc) {
    acc = fmaf(w.x, x.x, acc); acc = fmaf(w.y, x.y, acc);
    acc = fmaf(w.z, x.z, acc); acc = fmaf(w.w, x.w, acc);
    return acc;
  }
  __device__ static __forceinline__ void load(const float* p, float (&v)[4]) {
    const float4 q = *reinterpret_cast<const float4*>(p);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
  }
  __device__ static __forceinline__ float widen1(float s) { return s; }
};
template <> struct GateUnit<bf16_t> {
  static constexpr int N = 8;
  using raw = gu32x4;
  // packed bf16 pairs through the 2-way bf16 dot instruction (elements copied to
  // scalars before the bit cast)
  __device__ static __forceinline__ float dot(const raw& w, const raw& x, float acc) {
    const unsigned w0 = w.x, w1 = w.y, w2 = w.z, w3 = w.w;
    const unsigned x0 = x.x, x1 = x.y, x2 = x.z, x3 = x.w;
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(gbf16x2, w0), __builtin_bit_cast(gbf16x2, x0), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(gbf16x2, w1), __builtin_bit_cast(gbf16x2, x1), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(gbf16x2, w2), __builtin_bit_cast(gbf16x2, x2), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(gbf16x2, w3), __builtin_bit_cast(gbf16x2, x3), acc, false);
    return acc;
  }
  __device__ static __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const uint4 q = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
    v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
    v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
  }
  __device__ static __forceinline__ float widen1(bf16_t s) { return __uint_as_float(uint32_t(s.v) << 16); }
};

// Shared memory the selection stage works in.
struct SelectSmem {
  alignas(16) float lg[SMOE_MAX_BATCH][kWave];   // logits; lanes >= E hold -inf
  float sc[SMOE_MAX_BATCH][kWave];
  int rk[SMOE_MAX_BATCH][kWave];
  int tk[SMOE_MAX_BATCH][SMOE_MAX_TOPK];
  float thr_r[SMOE_MAX_BATCH];
  unsigned long long top_m_sh[SMOE_MAX_BATCH];
  int slot_of[kWave];
  int fin[SMOE_MAX_BATCH][SMOE_MAX_TOPK];     // final expert per (token, slot)
  float wsl[SMOE_MAX_BATCH][SMOE_MAX_TOPK];   // combine weight per (token, slot)
  // expert groups of a batched step while they are being collected
  int pair_e[kWave];                          // expert of (token, slot) pair t * k + j
  int gcnt[kWave];                            // tokens per expert
  int gtok[kWave][SMOE_MAX_BATCH];            // their tokens, ascending
  float gw[kWave][SMOE_MAX_BATCH];            // and combine weights
};

// Runs on wave 0 with all 64 lanes active: logits in sm.lg -> decision record.
// `sim` is this layer's similarity table (global or LDS).
// Pass 1 for tokens [t_begin, t_end): scores, top-(k+1), alpha classes.  Returns
// the union of their top-score masks.
__device__ __forceinline__ unsigned long long select_pass1(const RouteArgs& a, SelectSmem& sm, int lane,
                                                           int t_begin, int t_end) {
  const int E = a.E, k = a.k;
  auto& lg = sm.lg; auto& sc = sm.sc; auto& rk = sm.rk; auto& tk = sm.tk;
  auto& thr_r = sm.thr_r; auto& top_m_sh = sm.top_m_sh;
  const bool has_pivot = E > k;
  unsigned long long c_mask = 0;
  for (int t = t_begin; t < t_end; ++t) {
    const bool in = lane < E;
    const float l = in ? lg[t][lane] : -INFINITY;
    const float m = wave_max(l);
    const float p = in ? expf(l - m) : 0.f;
    const float s = p / wave_sum(p);
    // Rank of this lane's expert in (logit descending, id ascending) order, by
    // counting the experts that precede it: E broadcast reads of the logits in
    // LDS instead of k+1 dependent wave-wide arg-max rounds.
    int myrank = 0;
    for (int j = 0; j < E; j += 4) {
      const float4 q = *reinterpret_cast<const float4*>(&lg[t][j]);    // lanes >= E hold -inf
      myrank += (q.x > l) || (q.x == l && j < lane);
      myrank += (q.y > l) || (q.y == l && j + 1 < lane);
      myrank += (q.z > l) || (q.z == l && j + 2 < lane);
      myrank += (q.w > l) || (q.w == l && j + 3 < lane);
    }
    if (!in) myrank = 127;
    if (lane < k) tk[t][lane] = lane;                 // defined even if the logits are not numbers
    if (myrank < k) tk[t][myrank] = lane;
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
    c_mask |= top_m;
    sc[t][lane] = s;
    rk[t][lane] = myrank;
    if (lane == 0) { thr_r[t] = R; top_m_sh[t] = top_m; }
  }
  return c_mask;
}

// Pass 2: substitution against residency and the batch top-score set C, the
// decision record, the expert groups, and the publication to the host mirror.
__device__ __forceinline__ void select_pass2(const RouteArgs& a, SelectSmem& sm, const float* sim,
                                             unsigned long long c_mask, int lane, int t_begin, int t_end) {
  const int E = a.E, k = a.k;
  auto& sc = sm.sc; auto& rk = sm.rk; auto& tk = sm.tk;
  auto& thr_r = sm.thr_r; auto& top_m_sh = sm.top_m_sh; auto& slot_of = sm.slot_of;
  const bool has_pivot = E > k;
  const unsigned long long avail = a.resident | c_mask;
  for (int t = t_begin; t < t_end; ++t) {
    const float s = sc[t][lane];
    const int myrank = rk[t][lane];
    const bool active = myrank < k;
    const unsigned long long top_m = top_m_sh[t];
    const float R = thr_r[t];
    const bool is_avail = (avail >> lane) & 1ull;
    const unsigned long long need_m = __ballot(active && !((top_m >> lane) & 1ull) && !is_avail);
    unsigned long long cand_m =
        has_pivot ? __ballot(lane < E && !active && is_avail && s >= R) : 0ull;
    const int mytop = lane < k ? tk[t][lane] : -1;   // lane r owns slot r
    int myfin = mytop, mysub = 0;
    for (int r = k - 1; r >= 0; --r) {               // lowest-scoring active first
      const int b = __shfl(mytop, r, kWave);
      if (!((need_m >> b) & 1ull)) continue;
      if (!cand_m) break;
      const bool is_cand = (cand_m >> lane) & 1ull;
      float key = s;
      if (a.subst_key == 0) key = is_cand ? sim[(size_t)b * E + lane] : 0.f;
      const int c = wave_argmax(key, is_cand, lane);
      if (lane == r) { myfin = c; mysub = 1; }
      cand_m &= ~(1ull << c);
    }
    float w = lane < k ? sc[t][mytop] : 0.f;
    const float wsum = wave_sum(w);
    if (a.renorm) w = w / wsum;
    if (lane < k) {
      const int slot = ((a.resident >> myfin) & 1ull) ? slot_of[myfin] : -1;
      TokRec* d = &a.rec_dev->tok[t];
      TokRec* hrec = &a.rec_host->tok[t];
      d->topk[lane] = mytop;   hrec->topk[lane] = mytop;
      d->final_[lane] = myfin; hrec->final_[lane] = myfin;
      d->slot[lane] = slot;    hrec->slot[lane] = slot;
      d->subst[lane] = mysub;  hrec->subst[lane] = mysub;
      d->w[lane] = w;          hrec->w[lane] = w;
      sm.fin[t][lane] = myfin;
      sm.wsl[t][lane] = w;
    }
    a.rec_host->tok[t].scores[lane] = lane < E ? s : 0.f;
  }
}

// Last step, one wave, after every token's pass 2: the expert groups of a
// batched step, then the publication of the call number to the host mirror.
__device__ __forceinline__ void publish(const RouteArgs& a, SelectSmem& sm, int lane) {
  const int k = a.k, B = a.B;
  auto& slot_of = sm.slot_of;
  if (B > 1) {
    // Expert groups for the batched FFN.  Lane p first stands for the (token, slot) pair
    // p = t * k + j: its place in its expert's token list is the number of earlier pairs with
    // the same expert (pairs are in token order and a token uses an expert once, so the list
    // comes out ascending).  Then lane e stands for expert e and reads its list back.
    const int np = B * k;                               // <= 64
    const bool has = lane < np;
    const int pt = lane / k, pj = lane - pt * k;
    const int pe = has ? sm.fin[pt][pj] : -1;
    sm.pair_e[lane] = pe;
    sm.gcnt[lane] = 0;
    int pos = 0, cnt = 0;
    for (int q = 0; q < np; ++q) {
      const bool same = sm.pair_e[q] == pe;
      pos += same && q < lane;
      cnt += same;
    }
    if (has) {
      sm.gtok[pe][pos] = pt;
      sm.gw[pe][pos] = sm.wsl[pt][pj];
      if (pos == 0) sm.gcnt[pe] = cnt;
    }
    GroupTask g;
    g.expert = lane;
    g.slot = ((a.resident >> lane) & 1ull) ? slot_of[lane] : -1;
    g.ntok = sm.gcnt[lane];
    g.pad_ = 0;
#pragma unroll
    for (int i = 0; i < SMOE_MAX_BATCH; ++i) {
      g.tok[i] = i < g.ntok ? sm.gtok[lane][i] : 0;
      g.w[i] = i < g.ntok ? sm.gw[lane][i] : 0.f;
    }
    const unsigned long long has_m = __ballot(g.ntok > 0);
    const int idx = __popcll(has_m & ((1ull << lane) - 1ull));
    if (g.ntok > 0) a.rec_dev->grp[idx] = g;
    if (lane == 0) a.rec_dev->n_groups = __popcll(has_m);
  }
  if (a.x_mirror != nullptr) {
    // CPU-assisted scheduling: the host cores need the hidden states of this call
    const gu32x4* src = static_cast<const gu32x4*>(a.x);
    gu32x4* dst = static_cast<gu32x4*>(a.x_mirror);
    for (int u = lane; u < a.x_units; u += kWave) dst[u] = src[u];
  }
  // publish: every store of this wave to the mirror is complete before seq changes
  __threadfence_system();
  if (lane == 0) __hip_atomic_store(&a.rec_host->seq, a.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__device__ __forceinline__ void select_and_publish(const RouteArgs& a, SelectSmem& sm, const float* sim,
                                                   int lane) {
  const unsigned long long c_mask = select_pass1(a, sm, lane, 0, a.B);
  select_pass2(a, sm, sim, c_mask, lane, 0, a.B);
  publish(a, sm, lane);
}

constexpr int kMaxSeg = 8;   // a gate row is split into at most this many segments

// NTOK = tokens whose hidden states sit in LDS together (dynamic LDS: NTOK*H floats).
template <typename T, int NTOK>
__global__ __launch_bounds__(1024) void route_kernel(const RouteArgs a) {
  extern __shared__ __align__(16) float xs[];                 // [NTOK][H]
  __shared__ float part[SMOE_MAX_BATCH][kWave][kMaxSeg];
  __shared__ SelectSmem sm;

  constexpr int N = GateUnit<T>::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int nw = blockDim.x >> 6;
  const int H = a.H, E = a.E, B = a.B;
  if (tid < kWave) sm.slot_of[tid] = a.slot_of[tid];

  // ---- gate GEMV: logits[t][e] = Wg[e] . x[t] --------------------------------
  // work item = (expert row, segment of the row); segments are summed in a fixed order
  const T* wg = static_cast<const T*>(a.gate_w);
  const T* x = static_cast<const T*>(a.x);
  const int units = H / N;
  const int nseg = a.nseg;
  const int items = E * nseg;
  for (int t0 = 0; t0 < B; t0 += NTOK) {
    const int nt = min(NTOK, B - t0);
    __syncthreads();
    for (int i = tid; i < nt * H; i += blockDim.x) xs[i] = GateUnit<T>::widen1(x[(size_t)t0 * H + i]);
    __syncthreads();
    for (int it = wave; it < items; it += nw) {
      const int e = it / nseg, sg = it - e * nseg;
      const int u0 = (int)((long)units * sg / nseg), u1 = (int)((long)units * (sg + 1) / nseg);
      const T* row = wg + (size_t)e * H;
      float acc[NTOK];
#pragma unroll
      for (int q = 0; q < NTOK; ++q) acc[q] = 0.f;
#pragma unroll 4
      for (int u = u0 + lane; u < u1; u += kWave) {
        float w[N];
        GateUnit<T>::load(row + (size_t)u * N, w);
#pragma unroll
        for (int q = 0; q < NTOK; ++q) {
          if (q < nt) {
            const float* xv = xs + (size_t)q * H + (size_t)u * N;
#pragma unroll
            for (int i = 0; i < N; ++i) acc[q] = fmaf(w[i], xv[i], acc[q]);
          }
        }
      }
#pragma unroll
      for (int q = 0; q < NTOK; ++q) {
        const float v = wave_sum(acc[q]);
        if (lane == 0 && q < nt) part[t0 + q][e][sg] = v;
      }
    }
  }
  __syncthreads();
  if (wave != 0) return;
  for (int t = 0; t < B; ++t) {
    float v = 0.f;
    if (lane < E)
      for (int sg = 0; sg < nseg; ++sg) v += part[t][lane][sg];
    sm.lg[t][lane] = lane < E ? v : -INFINITY;
  }

  select_and_publish(a, sm, a.sim, lane);
}

// Batch-1 fast path.  No staging of x: a wave owns up to four gate rows (or
// row segments) at once, loads its slice of x and of those rows straight into
// registers so that all loads of the GEMV are in flight together, and the
// similarity table is copied to LDS meanwhile.  UPI = 128-bit units of one
// item per lane.
template <typename T, int UPI>
__global__ __launch_bounds__(1024) void route_b1_kernel(const RouteArgs a) {
  __shared__ SelectSmem sm;
  __shared__ float part[kWave][kMaxSeg];
  __shared__ float sim_sh[SMOE_MAX_EXPERTS * SMOE_MAX_EXPERTS];
  constexpr int N = GateUnit<T>::N;
  using raw = typename GateUnit<T>::raw;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int H = a.H, E = a.E;
  const int nseg = a.nseg;                       // power of two <= 8, divides the 16 waves
  const int items = E * nseg;
  const int units = H / N;
  const T* wg = static_cast<const T*>(a.gate_w);
  const int tok = blockIdx.x;                    // one block per token
  const T* x = static_cast<const T*>(a.x) + (size_t)tok * H;

  // this wave's segment of x (the same for all of its items: 16 is a multiple of nseg)
  const int sg = wave & (nseg - 1);
  const int u0 = (int)((long)units * sg / nseg), u1 = (int)((long)units * (sg + 1) / nseg);
  raw xr[UPI];
#pragma unroll
  for (int i = 0; i < UPI; ++i) {
    const int u = u0 + i * kWave + lane;
    xr[i] = (u < u1) ? *reinterpret_cast<const raw*>(x + (size_t)u * N) : raw{};
  }
  if (a.subst_key == 0 && gridDim.x == 1)
    for (int i = tid; i < E * E; i += 1024) sim_sh[i] = a.sim[i];
  if (tid < kWave) sm.slot_of[tid] = a.slot_of[tid];

  // RPP rows in flight per wave and pass (fewer when a row segment is long, to stay in registers)
  constexpr int RPP = UPI >= 8 ? 2 : 4;
  for (int base = 0; base < items; base += RPP * 16) {
    float acc[RPP];
#pragma unroll
    for (int r = 0; r < RPP; ++r) acc[r] = 0.f;
#pragma unroll
    for (int i = 0; i < UPI; ++i) {
      const int u = u0 + i * kWave + lane;
      raw q[RPP];
#pragma unroll
      for (int r = 0; r < RPP; ++r) {
        const int it = base + r * 16 + wave;
        q[r] = (it < items && u < u1) ? *reinterpret_cast<const raw*>(wg + (size_t)(it / nseg) * H + (size_t)u * N)
                                      : raw{};
      }
#pragma unroll
      for (int r = 0; r < RPP; ++r) acc[r] = GateUnit<T>::dot(q[r], xr[i], acc[r]);
    }
#pragma unroll
    for (int r = 0; r < RPP; ++r) {
      const int it = base + r * 16 + wave;
      const float v = wave_sum(acc[r]);
      if (lane == 0 && it < items) part[it / nseg][sg] = v;
    }
  }
  __syncthreads();
  if (wave != 0) return;
  {
    float v = 0.f;
    if (lane < E)
      for (int s2 = 0; s2 < nseg; ++s2) v += part[lane][s2];
    sm.lg[tok][lane] = lane < E ? v : -INFINITY;
  }
  if (gridDim.x == 1) {
    select_and_publish(a, sm, sim_sh, lane);
    return;
  }
  // batch > 1: leave this token's pass-1 state for the merge kernel
  select_pass1(a, sm, lane, tok, tok + 1);
  RouteTmp* o = a.tmp + tok;
  o->sc[lane] = sm.sc[tok][lane];
  o->rk[lane] = sm.rk[tok][lane];
  if (lane < SMOE_MAX_TOPK) o->tk[lane] = lane < a.k ? sm.tk[tok][lane] : -1;
  if (lane == 0) { o->thr_r = sm.thr_r[tok]; o->top_m = sm.top_m_sh[tok]; }
}

// Batch 1, gate matrix too large for one compute unit to stream quickly (a
// single block pulls a few tens of GB/s): the GEMV is spread over `split_nb`
// blocks of four waves.  Work item = (row, segment); the waves of the whole
// grid take items round-robin, RPP at a time, with their slice of x in
// registers, and write each item's partial dot product to device scratch.  The
// block that finishes last (agent-scope fence, then one atomic ticket per
// block) sums the segments of every row in fixed order and runs the selection
// and the publication exactly as the single-block kernel does; it also resets
// the ticket counter for the next launch.
template <typename T, int UPI>
__global__ __launch_bounds__(256) void route_split_kernel(const RouteArgs a) {
  __shared__ SelectSmem sm;
  __shared__ float sim_sh[SMOE_MAX_EXPERTS * SMOE_MAX_EXPERTS];
  __shared__ int is_last;
  constexpr int N = GateUnit<T>::N;
  using raw = typename GateUnit<T>::raw;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int H = a.H, E = a.E;
  const int nseg = a.nseg;                       // power of two <= 8; 4 * gridDim.x is a multiple of it
  const int items = E * nseg;
  const int units = H / N;
  const int nw = 4 * gridDim.x;
  const int gw = 4 * blockIdx.x + wave;
  const T* wg = static_cast<const T*>(a.gate_w);
  const T* x = static_cast<const T*>(a.x);

  const int sg = gw & (nseg - 1);                // the same segment for every item of this wave
  const int u0 = (int)((long)units * sg / nseg), u1 = (int)((long)units * (sg + 1) / nseg);
  raw xr[UPI];
#pragma unroll
  for (int i = 0; i < UPI; ++i) {
    const int u = u0 + i * kWave + lane;
    xr[i] = (u < u1) ? *reinterpret_cast<const raw*>(x + (size_t)u * N) : raw{};
  }
  if (a.subst_key == 0)
    for (int i = tid; i < E * E; i += 256) sim_sh[i] = a.sim[i];
  if (tid < kWave) sm.slot_of[tid] = a.slot_of[tid];

  constexpr int RPP = UPI >= 8 ? 2 : 4;
  for (int base = 0; base < items; base += RPP * nw) {
    float acc[RPP];
#pragma unroll
    for (int r = 0; r < RPP; ++r) acc[r] = 0.f;
#pragma unroll
    for (int i = 0; i < UPI; ++i) {
      const int u = u0 + i * kWave + lane;
      raw q[RPP];
#pragma unroll
      for (int r = 0; r < RPP; ++r) {
        const int it = base + r * nw + gw;
        q[r] = (it < items && u < u1) ? *reinterpret_cast<const raw*>(wg + (size_t)(it / nseg) * H + (size_t)u * N)
                                      : raw{};
      }
#pragma unroll
      for (int r = 0; r < RPP; ++r) acc[r] = GateUnit<T>::dot(q[r], xr[i], acc[r]);
    }
#pragma unroll
    for (int r = 0; r < RPP; ++r) {
      const int it = base + r * nw + gw;
      const float v = wave_sum(acc[r]);
      if (lane == 0 && it < items) a.split_part[it] = v;     // it = row * nseg + sg
    }
  }
  // This block's partial sums are visible device-wide before its ticket is drawn.  One thread
  // fences for the whole block (the barrier orders the other waves' stores before it): every
  // wave that executes an agent-scope release makes the XCD write back its L2.
  __syncthreads();
  if (tid == 0) {
    __threadfence();
    is_last = (atomicAdd(a.split_count, 1u) == gridDim.x - 1) ? 1 : 0;
  }
  __syncthreads();
  if (!is_last || wave != 0) return;
  __threadfence();                                // the other blocks' sums are visible to this wave
  if (lane == 0) *a.split_count = 0u;             // stream order: the next launch starts after this one ends
  {
    float v = 0.f;
    if (lane < E)
      for (int s2 = 0; s2 < nseg; ++s2)
        v += __builtin_nontemporal_load(a.split_part + lane * nseg + s2);
    sm.lg[0][lane] = lane < E ? v : -INFINITY;
  }
  select_and_publish(a, sm, sim_sh, lane);
}

// Batch > 1, second launch: wave t runs pass 2 for token t against the batch
// top-score set; wave 0 then builds the expert groups and publishes.
__global__ __launch_bounds__(64 * SMOE_MAX_BATCH) void route_merge_kernel(const RouteArgs a) {
  __shared__ SelectSmem sm;
  __shared__ float sim_sh[SMOE_MAX_EXPERTS * SMOE_MAX_EXPERTS];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int E = a.E;
  if (a.subst_key == 0)
    for (int i = tid; i < E * E; i += blockDim.x) sim_sh[i] = a.sim[i];
  if (tid < kWave) sm.slot_of[tid] = a.slot_of[tid];
  unsigned long long c_mask = 0;
  for (int t = 0; t < a.B; ++t) c_mask |= a.tmp[t].top_m;
  if (wave < a.B) {
    const RouteTmp* o = a.tmp + wave;
    sm.sc[wave][lane] = o->sc[lane];
    sm.rk[wave][lane] = o->rk[lane];
    if (lane < SMOE_MAX_TOPK) sm.tk[wave][lane] = o->tk[lane];
    if (lane == 0) { sm.thr_r[wave] = o->thr_r; sm.top_m_sh[wave] = o->top_m; }
  }
  __syncthreads();
  if (wave < a.B) select_pass2(a, sm, sim_sh, c_mask, lane, wave, wave + 1);
  __syncthreads();
  __threadfence_system();                       // each wave's stores to the mirror are out
  __syncthreads();
  if (wave == 0) publish(a, sm, lane);
}

}  // namespace

template <typename T>
static void launch_route_t(const RouteArgs& a, hipStream_t s) {
  if (a.fast_upi > 0 && a.B == 1 && a.split_nb > 0) {
    switch (a.fast_upi) {
      case 1: hipLaunchKernelGGL((route_split_kernel<T, 1>), dim3(a.split_nb), dim3(256), 0, s, a); return;
      case 2: hipLaunchKernelGGL((route_split_kernel<T, 2>), dim3(a.split_nb), dim3(256), 0, s, a); return;
      case 4: hipLaunchKernelGGL((route_split_kernel<T, 4>), dim3(a.split_nb), dim3(256), 0, s, a); return;
      case 8: hipLaunchKernelGGL((route_split_kernel<T, 8>), dim3(a.split_nb), dim3(256), 0, s, a); return;
      default: break;
    }
  }
  if (a.fast_upi > 0) {
    // one block per token; with more than one token a second launch merges them
    bool launched = true;
    switch (a.fast_upi) {
      case 1: hipLaunchKernelGGL((route_b1_kernel<T, 1>), dim3(a.B), dim3(1024), 0, s, a); break;
      case 2: hipLaunchKernelGGL((route_b1_kernel<T, 2>), dim3(a.B), dim3(1024), 0, s, a); break;
      case 4: hipLaunchKernelGGL((route_b1_kernel<T, 4>), dim3(a.B), dim3(1024), 0, s, a); break;
      case 8: hipLaunchKernelGGL((route_b1_kernel<T, 8>), dim3(a.B), dim3(1024), 0, s, a); break;
      default: launched = false; break;
    }
    if (launched) {
      if (a.B > 1) hipLaunchKernelGGL(route_merge_kernel, dim3(1), dim3(64 * a.B), 0, s, a);
      return;
    }
  }
  // as many tokens' hidden states in LDS together as fit in 32 KB
  int ntok = 1;
  while (ntok < a.B && ntok < SMOE_MAX_BATCH && (size_t)(2 * ntok) * a.H * sizeof(float) <= 32 * 1024)
    ntok *= 2;
  const size_t lds = (size_t)ntok * a.H * sizeof(float);
  switch (ntok) {
    case 1: hipLaunchKernelGGL((route_kernel<T, 1>), dim3(1), dim3(1024), lds, s, a); break;
    case 2: hipLaunchKernelGGL((route_kernel<T, 2>), dim3(1), dim3(1024), lds, s, a); break;
    case 4: hipLaunchKernelGGL((route_kernel<T, 4>), dim3(1), dim3(1024), lds, s, a); break;
    default: hipLaunchKernelGGL((route_kernel<T, 8>), dim3(1), dim3(1024), lds, s, a); break;
  }
}

void launch_route(const RouteArgs& a, int dtype, hipStream_t s) {
  if (dtype == SMOE_DTYPE_FP32) launch_route_t<float>(a, s);
  else launch_route_t<bf16_t>(a, s);
}

}  // namespace smoe
