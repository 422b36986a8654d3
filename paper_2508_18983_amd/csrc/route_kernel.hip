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

namespace smoe {
namespace {

struct bf16_t { uint16_t v; };

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
// Lane holding the largest value among lanes with valid set; lower lane wins
// ties; -1 when no lane is valid.  Result is uniform across the wave.
__device__ __forceinline__ int wave_argmax(float v, bool valid, int lane) {
  float val = valid ? v : -INFINITY;
  int idx = valid ? lane : kWave;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(val, o, kWave);
    int oi = __shfl_xor(idx, o, kWave);
    if (ov > val || (ov == val && oi < idx)) { val = ov; idx = oi; }
  }
  return idx == kWave ? -1 : idx;
}

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float(uint32_t(v.v) << 16); }

template <typename T>
__global__ __launch_bounds__(1024) void route_kernel(const RouteArgs a) {
  __shared__ float xs[SMOE_MAX_HIDDEN];
  __shared__ float lg[SMOE_MAX_BATCH][kWave];
  __shared__ float sc[SMOE_MAX_BATCH][kWave];
  __shared__ int rk[SMOE_MAX_BATCH][kWave];
  __shared__ int tk[SMOE_MAX_BATCH][SMOE_MAX_TOPK];
  __shared__ float thr_r[SMOE_MAX_BATCH];
  __shared__ unsigned long long top_m_sh[SMOE_MAX_BATCH];
  __shared__ int slot_of[kWave];

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int nw = blockDim.x >> 6;
  const int H = a.H, E = a.E, k = a.k, B = a.B;
  if (tid < kWave) slot_of[tid] = a.slot_of[tid];

  // ---- gate GEMV: logits[t][e] = Wg[e] . x[t] --------------------------------
  const T* wg = static_cast<const T*>(a.gate_w);
  const T* x = static_cast<const T*>(a.x);
  for (int t = 0; t < B; ++t) {
    __syncthreads();
    for (int h = tid; h < H; h += blockDim.x) xs[h] = to_f32(x[(size_t)t * H + h]);
    __syncthreads();
    for (int e = wave; e < E; e += nw) {
      const T* row = wg + (size_t)e * H;
      float acc = 0.f;
      for (int h = lane; h < H; h += kWave) acc = fmaf(to_f32(row[h]), xs[h], acc);
      acc = wave_sum(acc);
      if (lane == 0) lg[t][e] = acc;
    }
  }
  __syncthreads();
  if (wave != 0) return;

  // ---- pass 1: scores, top-(k+1), alpha classes, batch top-score set C ------
  const bool has_pivot = E > k;
  unsigned long long c_mask = 0;
  for (int t = 0; t < B; ++t) {
    const bool in = lane < E;
    const float l = in ? lg[t][lane] : -INFINITY;
    const float m = wave_max(l);
    const float p = in ? expf(l - m) : 0.f;
    const float s = p / wave_sum(p);
    bool rem = in;
    int myrank = 127, pivot = -1;
    const int nsel = has_pivot ? k + 1 : k;
    for (int r = 0; r < nsel; ++r) {
      const int idx = wave_argmax(l, rem, lane);
      if (lane == idx) { rem = false; myrank = r; }
      if (r < k) { if (lane == 0) tk[t][r] = idx; } else pivot = idx;
    }
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

  // ---- pass 2: substitution and the decision record -------------------------
  const unsigned long long avail = a.resident | c_mask;
  for (int t = 0; t < B; ++t) {
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
      if (a.subst_key == 0) key = is_cand ? a.sim[(size_t)b * E + lane] : 0.f;
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
    }
    a.rec_host->tok[t].scores[lane] = lane < E ? s : 0.f;
  }
}

}  // namespace

void launch_route(const RouteArgs& a, int dtype, hipStream_t s) {
  if (dtype == SMOE_DTYPE_FP32)
    hipLaunchKernelGGL(route_kernel<float>, dim3(1), dim3(1024), 0, s, a);
  else
    hipLaunchKernelGGL(route_kernel<bf16_t>, dim3(1), dim3(1024), 0, s, a);
}

}  // namespace smoe
