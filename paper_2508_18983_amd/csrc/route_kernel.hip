// Router + expert-cache router on the GPU.
//
//   gate GEMV -> softmax over the routed experts -> top-(k+1)   (Section II-A,
//                                                     Algorithm 1 "Sort S_t desc")
//   T = (1+alpha) S_{k+1}, R = (1-alpha) S_{k+1}, top-score / low-score classes,
//   substitution of non-resident low-score experts by resident (or batch
//   top-score) inactive experts inside the score band       (Algorithm 1 and
//                                                     Section IV-B prose)
//
// The paper runs this search on the CPU.  Here the gate GEMV is one launch
// spread over many compute units (gate_partial_kernel: one wave per row
// segment, partial dot products to device memory, no fence and no ticket: the
// kernel boundary is the barrier).  The selection works on one wavefront per
// token with one expert per lane (E <= 64), the residency set is a 64-bit mask
// passed by value and every set operation is a ballot (route_select.hpp).  At
// batch 1 it runs in the prologue of the up-projection kernel, so a layer call
// is three launches; route_select_kernel is the stand-alone form for batched
// steps (which also need the batch top-score set and the expert groups), for
// predictions, and for shapes the register up kernel does not cover.
#include "smoe_dev.hpp"
#include "wave_ops.hpp"
#include "route_select.hpp"

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
};

// Gate GEMV.  Work item = (expert row, segment of the row): one wave per item,
// grid.y = tokens.  The wave's slices of x and of the row go straight into
// registers (UPI 128-bit units per lane each), all loads in flight together.
template <typename T, int UPI>
__global__ __launch_bounds__(256) void gate_partial_kernel(const RouteArgs a) {
  constexpr int N = GateUnit<T>::N;
  using raw = typename GateUnit<T>::raw;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  const int nseg = a.nseg;
  const int item = blockIdx.x * 4 + wave;
  if (item >= a.E * nseg) return;
  const int tok = blockIdx.y;
  const int e = item / nseg, sg = item - e * nseg;
  const int units = a.H / N;
  const int u0 = (int)((long)units * sg / nseg), u1 = (int)((long)units * (sg + 1) / nseg);
  const T* x = static_cast<const T*>(a.x) + (size_t)tok * a.H;
  const T* row = static_cast<const T*>(a.gate_w) + (size_t)e * a.H;
  raw xr[UPI], wr[UPI];
#pragma unroll
  for (int i = 0; i < UPI; ++i) {
    const int u = u0 + i * kWave + lane;
    const bool live = u < u1;
    xr[i] = live ? *reinterpret_cast<const raw*>(x + (size_t)u * N) : raw{};
    wr[i] = live ? *reinterpret_cast<const raw*>(row + (size_t)u * N) : raw{};
  }
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < UPI; ++i) acc = GateUnit<T>::dot(wr[i], xr[i], acc);
  acc = wave_sum(acc);
  if (lane == 0) a.gate_part[((size_t)tok * a.E + e) * kMaxGateSeg + sg] = acc;
}

// Stand-alone selection: one block, wave t = token t.  Pass 1 per token, the
// batch top-score set C as the union of the tokens' top-score masks, pass 2 per
// token against residency and C; wave 0 then builds the expert groups of a
// batched step and publishes the call number.
__global__ __launch_bounds__(64 * SMOE_MAX_BATCH) void route_select_kernel(const RouteArgs a) {
  __shared__ SelectSmem<SMOE_MAX_BATCH> sm;
  __shared__ GroupSmem gs;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int B = a.B, k = a.k;
  if (tid < kWave) sm.slot_of[tid] = a.slot_of[tid];
  sm.lg[wave][lane] = logit_from_parts(a, lane, wave);   // (the block has exactly B waves)
  wave_lds_handoff();
  const TokenClasses cls = select_pass1(a, sm, lane, wave);
  if (lane == 0) sm.top_m[wave] = cls.top_m;
  __syncthreads();
  unsigned long long c_mask = 0;
  for (int t = 0; t < B; ++t) c_mask |= sm.top_m[t];
  select_pass2(a, sm, cls, c_mask, lane, wave, wave, true);
  __syncthreads();
  __threadfence_system();                       // each wave's stores to the mirror are out
  __syncthreads();
  if (wave != 0) return;
  if (B > 1) {
    // Expert groups for the batched FFN.  Lane p first stands for the (token, slot) pair
    // p = t * k + j: its place in its expert's token list is the number of earlier pairs with
    // the same expert (pairs are in token order and a token uses an expert once, so the list
    // comes out ascending).  Then lane e stands for expert e and reads its list back.
    const int np = B * k;                               // <= 64
    const bool has = lane < np;
    const int pt = lane / k, pj = lane - pt * k;
    const int pe = has ? sm.fin[pt][pj] : -1;
    gs.pair_e[lane] = pe;
    gs.gcnt[lane] = 0;
    wave_lds_handoff();
    int pos = 0, cnt = 0;
    for (int q = 0; q < np; ++q) {
      const bool same = gs.pair_e[q] == pe;
      pos += same && q < lane;
      cnt += same;
    }
    if (has) {
      gs.gtok[pe][pos] = pt;
      gs.gw[pe][pos] = sm.wsl[pt][pj];
      if (pos == 0) gs.gcnt[pe] = cnt;
    }
    wave_lds_handoff();
    GroupTask g;
    g.expert = lane;
    g.slot = ((a.resident >> lane) & 1ull) ? sm.slot_of[lane] : -1;
    g.ntok = gs.gcnt[lane];
    g.pad_ = 0;
#pragma unroll
    for (int i = 0; i < SMOE_MAX_BATCH; ++i) {
      g.tok[i] = i < g.ntok ? gs.gtok[lane][i] : 0;
      g.w[i] = i < g.ntok ? gs.gw[lane][i] : 0.f;
    }
    const unsigned long long has_m = __ballot(g.ntok > 0);
    const int idx = __popcll(has_m & ((1ull << lane) - 1ull));
    if (g.ntok > 0) a.rec_dev->grp[idx] = g;
    if (lane == 0) a.rec_dev->n_groups = __popcll(has_m);
  }
  publish_seq(a, lane);
}

}  // namespace

template <typename T>
static void launch_gate_t(const RouteArgs& a, hipStream_t s) {
  const dim3 grid((a.E * a.nseg + 3) / 4, a.B);
  switch (a.upi) {
    case 1: hipLaunchKernelGGL((gate_partial_kernel<T, 1>), grid, dim3(256), 0, s, a); return;
    case 2: hipLaunchKernelGGL((gate_partial_kernel<T, 2>), grid, dim3(256), 0, s, a); return;
    case 4: hipLaunchKernelGGL((gate_partial_kernel<T, 4>), grid, dim3(256), 0, s, a); return;
    default: hipLaunchKernelGGL((gate_partial_kernel<T, 8>), grid, dim3(256), 0, s, a); return;
  }
}

void launch_gate_partial(const RouteArgs& a, int dtype, hipStream_t s) {
  if (dtype == SMOE_DTYPE_FP32) launch_gate_t<float>(a, s);
  else launch_gate_t<bf16_t>(a, s);
}

void launch_route_select(const RouteArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(route_select_kernel, dim3(1), dim3(64 * a.B), 0, s, a);
}

}  // namespace smoe
