// Batch-1-style SwiGLU expert FFN for the chosen experts and the shared experts
// (Section V-B, GPU operations "Direct expert computation" and "New Expert
// Computation"; shared experts per Section II-A).  Pure weight streaming: every
// weight element is read once from HBM with non-temporal 128-bit loads, the
// activation vector sits in registers (LDS in the fallback kernels), one
// wavefront owns whole rows and reduces with cross-lane permutes, accumulation
// is fp32.
//
//   up   : act[task][f] = w_task * silu(W1[f].x) * (W3[f].x)
//   down : y[h] = sum_task sum_f W2[h][f] * act[task][f]
//          one wave produces y[h] for its rows over all tasks in a fixed
//          order: no partial buffers, atomics or fences.
#include "smoe_dev.hpp"
#include "wave_ops.hpp"
#include "route_select.hpp"

namespace smoe {
namespace {

struct bf16_t { uint16_t v; };
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

template <typename T> struct Unit;
template <> struct Unit<float> {
  static constexpr int N = 4;          // elements per 128-bit load
  using raw = f32x4;
  __device__ static __forceinline__ raw load(const float* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const raw*>(p));
  }
  __device__ static __forceinline__ void widen(const raw& q, float (&v)[4]) {
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
  }
  __device__ static __forceinline__ float widen1(float s) { return s; }
  __device__ static __forceinline__ float narrow(float s) { return s; }
  // acc + w . x for one unit, x in its stored form
  __device__ static __forceinline__ float dot(const raw& w, const raw& x, float acc) {
    acc = fmaf(w.x, x.x, acc); acc = fmaf(w.y, x.y, acc);
    acc = fmaf(w.z, x.z, acc); acc = fmaf(w.w, x.w, acc);
    return acc;
  }
};
template <> struct Unit<bf16_t> {
  static constexpr int N = 8;
  using raw = u32x4;
  __device__ static __forceinline__ raw load(const bf16_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const raw*>(p));
  }
  __device__ static __forceinline__ void widen(const raw& q, float (&v)[8]) {
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
    v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
    v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
  }
  __device__ static __forceinline__ float widen1(bf16_t s) {
    return __uint_as_float(uint32_t(s.v) << 16);
  }
  __device__ static __forceinline__ bf16_t narrow(float s) {   // round to nearest even
    uint32_t u = __float_as_uint(s);
    u += 0x7fffu + ((u >> 16) & 1u);
    return bf16_t{uint16_t(u >> 16)};
  }
  // acc + w . x for one unit of 8 bf16 pairs: both operands stay packed and go
  // through the 2-way bf16 dot instruction (products exact in fp32, fp32 sum)
  __device__ static __forceinline__ float dot(const raw& w, const raw& x, float acc) {
    // (elements are copied to scalars first: bit-casting a vector element in place
    // made the compiler read element 0 four times)
    const unsigned w0 = w.x, w1 = w.y, w2 = w.z, w3 = w.w;
    const unsigned x0 = x.x, x1 = x.y, x2 = x.z, x3 = x.w;
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w0), __builtin_bit_cast(bf16x2, x0), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w1), __builtin_bit_cast(bf16x2, x1), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w2), __builtin_bit_cast(bf16x2, x2), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w3), __builtin_bit_cast(bf16x2, x3), acc, false);
    return acc;
  }
};

// Keeps the loads written above this point above it in the instruction stream.  Without it the
// compiler may sink each load next to its first use to save registers, which turns "all loads
// of a row in flight, then the arithmetic" into one load at a time.
__device__ __forceinline__ void loads_issued_before_here() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

// Weights of task (t, j): null when the task is not part of this pass.
// PASS 0: routed slots whose expert is resident + shared experts; PASS 1: the
// slots whose expert has just been loaded (slot_override >= 0).  The pass is a
// template parameter so the two show up as separate kernels in profiles.
template <int PASS>
__device__ __forceinline__ const char* task_weights(const FfnArgs& a, int t, int j, int task,
                                                    int& F, float& wgt) {
  if (j < a.k) {
    F = a.F;
    wgt = a.rec->tok[t].w[j];
    int g;
    if (PASS == 0) {
      const int s = a.rec->tok[t].slot[j];
      if (s < 0) return nullptr;
      g = a.slot_base + s;
    } else {
      g = a.slot_override[task];
      if (g < 0) return nullptr;
    }
    return a.slab + (int64_t)g * a.expert_bytes;
  }
  if (PASS != 0) return nullptr;
  F = a.Fs;
  wgt = 1.0f;
  return a.shared + (int64_t)(j - a.k) * a.shared_bytes;
}

// Up kernels, batch-1 style: block -> (token, task j, tile of TF f-rows).  The
// shared experts' blocks come first: they need no routing decision, so with the
// selection fused into the kernel they stream weights while the routed blocks
// are still deciding.
__device__ __forceinline__ void up_block_coords(const FfnArgs& a, int bid, int& t, int& j, int& tile) {
  const int n_shared_blocks = a.ns * a.tilesS;
  const int bpt = n_shared_blocks + a.k * a.tilesR;   // blocks per token
  t = bid / bpt;
  int r = bid - t * bpt;
  if (r < n_shared_blocks) { j = a.k + r / a.tilesS; tile = r - (j - a.k) * a.tilesS; }
  else { r -= n_shared_blocks; j = r / a.tilesR; tile = r - j * a.tilesR; }
}

// acc[r] += sum_u row_r[u] . vec[u] over `units` 128-bit units, ROWS rows at a
// time, UNR independent steps in flight per row.
template <typename T, int ROWS, int UNR>
__device__ __forceinline__ void dot_rows(const T* const (&row)[ROWS], const float* __restrict__ vec,
                                         int units, int lane, float (&acc)[ROWS]) {
  constexpr int N = Unit<T>::N;
  using raw = typename Unit<T>::raw;
  int u = lane;
  for (; u + (UNR - 1) * kWave < units; u += UNR * kWave) {
    raw q[UNR][ROWS];
#pragma unroll
    for (int s = 0; s < UNR; ++s)
#pragma unroll
      for (int r = 0; r < ROWS; ++r) q[s][r] = Unit<T>::load(row[r] + (size_t)(u + s * kWave) * N);
#pragma unroll
    for (int s = 0; s < UNR; ++s) {
      const float* xv = vec + (size_t)(u + s * kWave) * N;
      float xq[N];
#pragma unroll
      for (int e = 0; e < N; ++e) xq[e] = xv[e];
#pragma unroll
      for (int r = 0; r < ROWS; ++r) {
        float w[N];
        Unit<T>::widen(q[s][r], w);
#pragma unroll
        for (int e = 0; e < N; ++e) acc[r] = fmaf(w[e], xq[e], acc[r]);
      }
    }
  }
  for (; u < units; u += kWave) {
    raw q[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) q[r] = Unit<T>::load(row[r] + (size_t)u * N);
    const float* xv = vec + (size_t)u * N;
    float xq[N];
#pragma unroll
    for (int e = 0; e < N; ++e) xq[e] = xv[e];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
      float w[N];
      Unit<T>::widen(q[r], w);
#pragma unroll
      for (int e = 0; e < N; ++e) acc[r] = fmaf(w[e], xq[e], acc[r]);
    }
  }
}

template <typename T, int PASS>
__global__ __launch_bounds__(256) void ffn_up_kernel(const FfnArgs a) {
  extern __shared__ __align__(16) float xs[];       // H floats
  constexpr int N = Unit<T>::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int nj = a.k + a.ns;
  int t, j, tile;
  up_block_coords(a, (int)blockIdx.x, t, j, tile);
  const int task = t * nj + j;
  int F; float wgt;
  const char* base = task_weights<PASS>(a, t, j, task, F, wgt);
  if (base == nullptr) return;
  const int H = a.H;
  const T* W1 = reinterpret_cast<const T*>(base);
  const T* W3 = W1 + (size_t)F * H;

  const T* x = static_cast<const T*>(a.x) + (size_t)t * H;
  for (int h = tid; h < H; h += 256) xs[h] = Unit<T>::widen1(x[h]);
  __syncthreads();

  const int units = H / N;
  const int per_wave = a.TF >> 2;
  const int f_begin = tile * a.TF + wave * per_wave;
  float* act = a.act + (size_t)task * a.Fmax;
  for (int i = 0; i < per_wave; i += 2) {
    const int f = f_begin + i;
    if (f >= F) break;
    // two f-rows at a time; when the wave's share or the matrix ends on an odd row the second
    // one repeats the first and is not stored
    const bool two = (i + 1 < per_wave) && (f + 1 < F);
    const int f2 = two ? f + 1 : f;
    const T* const rows[4] = {W1 + (size_t)f * H, W3 + (size_t)f * H,
                              W1 + (size_t)f2 * H, W3 + (size_t)f2 * H};
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    dot_rows<T, 4, 2>(rows, xs, units, lane, acc);
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = wave_sum(acc[q]);
    if (lane == 0) {
      act[f] = wgt * (acc[0] / (1.0f + expf(-acc[0]))) * acc[1];
      if (two) act[f + 1] = wgt * (acc[2] / (1.0f + expf(-acc[2]))) * acc[3];
    }
  }
}

// Down projection + combine.  A block owns 4*R consecutive output rows of one
// token (one wave = R rows) and keeps their running sums in registers while it
// walks this pass's tasks.  `stage_all` != 0: the activations of all tasks fit
// in LDS together and are loaded once; otherwise each task is processed in
// chunks of `chunk` floats.  Pass 0 writes y when the token has no missing
// expert, else fp32 sums to `ysum`; pass 1 adds the loaded experts to `ysum`
// and writes y.
template <typename T, int R, int PASS>
__global__ __launch_bounds__(256) void ffn_down_kernel(const FfnArgs a) {
  extern __shared__ __align__(16) float as[];
  constexpr int N = Unit<T>::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int nj = a.k + a.ns;
  const int t = blockIdx.x / a.htiles;
  const int ht = blockIdx.x - t * a.htiles;
  const int H = a.H;
  const int h0 = ht * (4 * R) + wave * R;

  bool any_miss = false;
  for (int q = 0; q < a.k; ++q) any_miss |= (a.rec->tok[t].slot[q] < 0);
  if (PASS == 1 && !any_miss) return;               // y of this token is already final

  float acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.f;

  if (a.stage_all) {
    int off = 0;
    for (int j = 0; j < nj; ++j) {
      int F; float wgt;
      if (task_weights<PASS>(a, t, j, t * nj + j, F, wgt) == nullptr) continue;
      const float* act = a.act + (size_t)(t * nj + j) * a.Fmax;
      for (int i = tid; i < F; i += 256) as[off + i] = act[i];
      off += F;
    }
    __syncthreads();
    off = 0;
    for (int j = 0; j < nj; ++j) {
      int F; float wgt;
      const char* base = task_weights<PASS>(a, t, j, t * nj + j, F, wgt);
      if (base == nullptr) continue;
      if (h0 < H) {
        const T* W2 = reinterpret_cast<const T*>(base) + 2 * (size_t)F * H;
        const T* rows[R];
#pragma unroll
        for (int r = 0; r < R; ++r) rows[r] = W2 + (size_t)min(h0 + r, H - 1) * F;
        dot_rows<T, R, (R >= 4 ? 2 : 4)>(rows, as + off, F / N, lane, acc);
      }
      off += F;
    }
  } else {
    for (int j = 0; j < nj; ++j) {
      int F; float wgt;
      const char* base = task_weights<PASS>(a, t, j, t * nj + j, F, wgt);
      if (base == nullptr) continue;
      const T* W2 = reinterpret_cast<const T*>(base) + 2 * (size_t)F * H;
      const float* act = a.act + (size_t)(t * nj + j) * a.Fmax;
      for (int c0 = 0; c0 < F; c0 += a.chunk) {
        const int clen = min(a.chunk, F - c0);
        __syncthreads();                              // previous chunk consumed by every wave
        for (int i = tid; i < clen; i += 256) as[i] = act[c0 + i];
        __syncthreads();
        if (h0 < H) {
          const T* rows[R];
#pragma unroll
          for (int r = 0; r < R; ++r) rows[r] = W2 + (size_t)min(h0 + r, H - 1) * F + c0;
          dot_rows<T, R, (R >= 4 ? 2 : 4)>(rows, as, clen / N, lane, acc);
        }
      }
    }
  }

#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = wave_sum(acc[r]);
  if (lane == 0) {
    T* y = static_cast<T*>(a.y) + (size_t)t * H;
    float* ysum = a.ysum + (size_t)t * H;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int h = h0 + r;
      if (h >= H) break;
      if (PASS == 0) {
        if (any_miss) ysum[h] = acc[r];
        else y[h] = Unit<T>::narrow(acc[r]);
      } else {
        y[h] = Unit<T>::narrow(ysum[h] + acc[r]);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Register-resident fast paths.  A lane always multiplies the same columns, so
// its slice of the activation vector stays in registers for every row it
// streams: no LDS traffic, no block-wide barrier inside the row loop.
// ---------------------------------------------------------------------------

// Up projection with x in registers: one wave owns whole rows (H/N <= 64*UPL
// units).  Per f it has 2*UPL independent 128-bit loads in flight.
//
// FUSED (batch 1, resident pass): there is no separate selection launch.  Every
// routed block repeats the selection for itself in its prologue (one wave,
// about a microsecond of arithmetic on E <= 64 logits that sit in L2) while its
// loads of x are in flight; the first routed block also writes the decision
// record for the down kernel and the host mirror.
template <typename T, int UPL, int PASS, bool FUSED>
__global__ __launch_bounds__(256) void ffn_up_reg_kernel(const FfnArgs a, const RouteArgs ra) {
  constexpr int N = Unit<T>::N;
  using raw = typename Unit<T>::raw;
  __shared__ SelectSmem<FUSED ? 1 : 0> sm;             // (empty when not fused)
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int nj = a.k + a.ns;
  // FUSED with ra.gate_blocks > 0: the launch starts with the blocks of the gate GEMV
  int ng = 0;
  if constexpr (FUSED) ng = ra.gate_blocks;
  const bool gate_block = (int)blockIdx.x < ng;
  int t = 0, j = 0, tile = 0;
  if (!gate_block) up_block_coords(a, (int)blockIdx.x - ng, t, j, tile);
  const int task = t * nj + j;
  const int H = a.H;
  const int units = H / N;
  // The wave that runs the selection.  A block's wave w sits on SIMD w of its compute unit, and
  // the blocks that share a compute unit at the start of a launch are 256 apart in the grid: with
  // wave 0 selecting in all of them the selections queue up on one SIMD while three idle
  // (2.2 us per selection instead of under one).
  const int sel_wave = ((int)blockIdx.x >> 8) & 3;

  // FUSED: what the selection reads from memory is requested first, together with x, so that
  // one round trip serves all of it (the scalar arguments of the selection are pinned here for
  // the same reason: fetched with the other kernel arguments instead of one by one later)
  int my_slot_of = -1;
  float my_logit = 0.f;
  if constexpr (FUSED) {
    const int e_ = ra.E, k_ = ra.k, ns_ = ra.nseg, rn_ = ra.renorm, sk_ = ra.subst_key;
    const float al_ = ra.alpha;
    const unsigned long long res_ = ra.resident;
    const float* gp_ = ra.gate_part;
    asm volatile("" ::"s"(e_), "s"(k_), "s"(ns_), "s"(rn_), "s"(sk_), "s"(al_), "s"(res_), "s"(gp_));
    if (!gate_block && j < a.k && wave == sel_wave) {
      my_slot_of = ra.slot_of[lane];
      if (ng == 0) my_logit = logit_from_parts(ra, lane, 0);
    }
  }
  raw xr[UPL];                                          // this lane's slice of x, as stored
  const T* x = static_cast<const T*>(a.x) + (size_t)t * H;
#pragma unroll
  for (int i = 0; i < UPL; ++i) {
    const int u = i * kWave + lane;
    xr[i] = (u < units) ? *reinterpret_cast<const raw*>(x + (size_t)u * N) : raw{};
  }

  if constexpr (FUSED) {
    // logit of expert e: one wave, the row against the slice of x every lane already holds
    auto gate_logit = [&](int e) -> float {
      const T* row = static_cast<const T*>(ra.gate_w) + (size_t)e * H;
      raw q[UPL];
#pragma unroll
      for (int s = 0; s < UPL; ++s) {
        if (s * kWave < units) q[s] = Unit<T>::load(row + (size_t)min(s * kWave + lane, units - 1) * N);
        else q[s] = raw{};
      }
      float acc = 0.f;
#pragma unroll
      for (int s = 0; s < UPL; ++s) acc = Unit<T>::dot(q[s], xr[s], acc);
      return wave_sum(acc);
    };
    if (gate_block) {
      // Gate GEMV (Section II-A): wave w of gate block b owns expert row 4 b + w and publishes
      // its logit with this call's epoch in one 64-bit word (one store: no fence, no counter).
      const int e = (int)blockIdx.x * 4 + wave;
      if (e < ra.E) {
        const float l = gate_logit(e);
        if (lane == 0)
          __hip_atomic_store(&ra.gate_word[e], ((unsigned long long)ra.epoch << 32) | __float_as_uint(l),
                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      return;
    }
    if (ng > 0 && j < a.k && wave == sel_wave) {
      // The selecting wave reads the E words until all of them carry this call's epoch.  The
      // gate blocks are the first blocks of this launch, so they are running or done by the
      // time any other block exists; the wait is bounded all the same, and a wave that gives
      // up computes the logits itself (slower, same values).
      unsigned long long v = 0;
      bool all_here = false;
      // (hundreds of blocks read the same few cache lines past the L2.  A block that starts when
      // the logits are long there must not wait at all, so the first read comes at once; after a
      // miss the wave stays away for a while, then reads at intervals)
      for (int spin = 0; spin < ra.gate_spin; ++spin) {
        v = lane < ra.E ? __hip_atomic_load(&ra.gate_word[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                        : ((unsigned long long)ra.epoch << 32);
        all_here = __all((unsigned)(v >> 32) == ra.epoch);
        if (all_here) break;
        if (spin == 0) __builtin_amdgcn_s_sleep(24);
        else __builtin_amdgcn_s_sleep(32);
      }
      if (all_here) {
        my_logit = lane < ra.E ? __uint_as_float((unsigned)v) : -INFINITY;
      } else {
        my_logit = -INFINITY;
        for (int e = 0; e < ra.E; ++e) {
          const float l = gate_logit(e);
          if (lane == e) my_logit = l;
        }
      }
    }
  }

  int F; float wgt;
  const char* base = nullptr;
  bool decided = false;
  if constexpr (FUSED) {
    if (j < a.k) {                                      // (uniform over the block)
      if (wave == sel_wave) {
        if (j == 0 && tile == 0) {
          select_single(ra, sm, lane, my_slot_of, my_logit, true);     // also writes the decision record
        } else {
          int e_sel, slot_sel;
          float w_sel;
          select_slot_in_registers(ra, lane, my_slot_of, my_logit, j, e_sel, slot_sel, w_sel);
          if (lane == 0) { sm.slt[0][j] = slot_sel; sm.wsl[0][j] = w_sel; }
        }
      }
      __syncthreads();
      const int slot = sm.slt[0][j];
      F = a.F;
      wgt = sm.wsl[0][j];
      base = slot < 0 ? nullptr : a.slab + (int64_t)(a.slot_base + slot) * a.expert_bytes;
      decided = true;
    }
  }
  if (!decided) base = task_weights<PASS>(a, t, j, task, F, wgt);
  if (base == nullptr) return;
  const T* W1 = reinterpret_cast<const T*>(base);
  const T* W3 = W1 + (size_t)F * H;

  // FPI f-rows (each = one W1 row + one W3 row) in flight per iteration
  constexpr int FPI = UPL >= 8 ? 1 : 2;
  const int per_wave = a.TF >> 2;
  const int f_begin = tile * a.TF + wave * per_wave;
  float* act = a.act + (size_t)task * a.Fmax;
  for (int i = 0; i < per_wave; i += FPI) {
    const int f = f_begin + i;
    if (f >= F) break;
    raw qg[FPI][UPL], qu[FPI][UPL];
#pragma unroll
    for (int p = 0; p < FPI; ++p) {
      const bool live = (i + p < per_wave) && (f + p < F);   // (the same for the whole wave)
      const T* g = W1 + (size_t)(f + p) * H;
      const T* up = W3 + (size_t)(f + p) * H;
      // (no per-lane branches around the loads: columns past the end of the row are clamped into
      // it and meet zeros in x; a row or a unit slot that nobody needs is skipped by the whole wave)
#pragma unroll
      for (int s = 0; s < UPL; ++s) {
        if (live && s * kWave < units) {
          const int u = min(s * kWave + lane, units - 1);
          qg[p][s] = Unit<T>::load(g + (size_t)u * N);
          qu[p][s] = Unit<T>::load(up + (size_t)u * N);
        } else {
          qg[p][s] = raw{};
          qu[p][s] = raw{};
        }
      }
    }
    loads_issued_before_here();
#pragma unroll
    for (int p = 0; p < FPI; ++p) {
      float ag = 0.f, au = 0.f;
#pragma unroll
      for (int s = 0; s < UPL; ++s) {
        ag = Unit<T>::dot(qg[p][s], xr[s], ag);
        au = Unit<T>::dot(qu[p][s], xr[s], au);
      }
      ag = wave_sum(ag);
      au = wave_sum(au);
      if (lane == 0 && i + p < per_wave && f + p < F) act[f + p] = wgt * (ag / (1.0f + expf(-ag))) * au;
    }
  }
}

// Down projection with the activations in registers.  A block of NW waves owns
// RB output rows of one token.  A row of task j is cut into column segments of
// <= 64*UPL units; a work item is (task, segment) and the waves take the items
// round-robin (the launch picks NW so that a wave has one or two).  For its
// item a wave loads its slice of the activations once and streams the RB rows
// R at a time through two register buffers: the loads of the next R rows are
// issued before the current R rows are reduced, so 2*R*UPL 128-bit loads per
// lane are in flight.  Every (item, row) partial sum is produced by exactly
// one wave and parked in LDS; after one barrier the block adds them in item
// order, so y does not depend on scheduling.
template <typename T, int UPL, int R, int NW, int PASS>
__global__ __launch_bounds__(64 * NW) void ffn_down_reg_kernel(const FfnArgs a) {
  extern __shared__ __align__(16) float part[];       // [items][RB]
  constexpr int N = Unit<T>::N;
  using raw = typename Unit<T>::raw;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int nj = a.k + a.ns;
  const int RB = a.RB;                                 // multiple of R
  const int t = blockIdx.x / a.htiles;
  const int ht = blockIdx.x - t * a.htiles;
  const int H = a.H;
  const int hb = ht * RB;
  // items of the shared experts first: their weights do not depend on the decision record, so
  // the waves that start with them have loads in flight while the record is still on its way
  const int items_s = a.ns * a.nsegS;
  const int n_items = items_s + a.k * a.nsegR;

  if (PASS == 1) {
    bool any_miss = false;
    for (int q = 0; q < a.k; ++q) any_miss |= (a.rec->tok[t].slot[q] < 0);
    if (!any_miss) return;                              // y of this token is already final
  }

  for (int it = wave; it < n_items; it += NW) {
    int j, seg, nseg;
    if (it < items_s) { nseg = a.nsegS; j = it / nseg; seg = it - j * nseg; j += a.k; }
    else { nseg = a.nsegR; const int q = it - items_s; j = q / nseg; seg = q - j * nseg; }
    float* prow = part + (size_t)it * RB;
    int F; float wgt;
    const char* base = task_weights<PASS>(a, t, j, t * nj + j, F, wgt);
    if (base == nullptr) {                            // not in this pass: contributes 0
      for (int r = lane; r < RB; r += kWave) prow[r] = 0.f;
      continue;
    }
    const int units = F / N;
    const int seg_units = (units + nseg - 1) / nseg;
    const int ubeg = seg * seg_units;
    const int uend = min(units, ubeg + seg_units);
    const T* W2 = reinterpret_cast<const T*>(base) + 2 * (size_t)F * H;
    const float* act = a.act + (size_t)(t * nj + j) * a.Fmax;

    // No per-lane branches around the loads: columns past the end of the segment are clamped into
    // it and meet zero activations, rows past H repeat the last one and are not written.  Only
    // whole unit slots that no lane needs are skipped, by a branch the whole wave takes together.
    float ar[UPL][N];                                   // my slice of the activations, loaded first:
#pragma unroll                                          // waiting for it must not wait for weight rows
    for (int i = 0; i < UPL; ++i) {
      const int u = ubeg + i * kWave + lane;
      const int uc = min(u, uend - 1);
      const bool slot_live = ubeg + i * kWave < uend;   // the same for the whole wave
#pragma unroll
      for (int e = 0; e < N; e += 4) {
        float4 v = {0.f, 0.f, 0.f, 0.f};
        if (slot_live) v = *reinterpret_cast<const float4*>(act + (size_t)uc * N + e);
        const bool in = u < uend;
        ar[i][e] = in ? v.x : 0.f; ar[i][e + 1] = in ? v.y : 0.f;
        ar[i][e + 2] = in ? v.z : 0.f; ar[i][e + 3] = in ? v.w : 0.f;
      }
    }
    // rows rr .. rr+R-1 of the block into one register buffer
    auto load_rows = [&](raw (&q)[R][UPL], int rr) {
#pragma unroll
      for (int r2 = 0; r2 < R; ++r2) {
        const T* row = W2 + (size_t)min(hb + rr + r2, H - 1) * F;
#pragma unroll
        for (int s2 = 0; s2 < UPL; ++s2) {
          // (a unit slot past the end of the segment is skipped by the whole wave; single lanes
          // past it re-read the segment's last unit)
          if (ubeg + s2 * kWave < uend) {
            const int u = min(ubeg + s2 * kWave + lane, uend - 1);
            q[r2][s2] = Unit<T>::load(row + (size_t)u * N);
          } else {
            q[r2][s2] = raw{};
          }
        }
      }
    };
    auto reduce_rows = [&](const raw (&q)[R][UPL], int rr) {
#pragma unroll
      for (int r2 = 0; r2 < R; ++r2) {
        float acc = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < UPL; ++s2) {
          float w[N];
          Unit<T>::widen(q[r2][s2], w);
#pragma unroll
          for (int e = 0; e < N; ++e) acc = fmaf(w[e], ar[s2][e], acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) prow[rr + r2] = acc;
      }
    };
    // two buffers, RB / R >= 2 steps: the steady loop reloads both, the last two or three steps
    // are peeled
    raw qa[R][UPL], qb[R][UPL];
    load_rows(qa, 0);
    load_rows(qb, R);
    int rr = 0;
    for (; rr + 3 * R < RB; rr += 2 * R) {
      reduce_rows(qa, rr);
      load_rows(qa, rr + 2 * R);
      reduce_rows(qb, rr + R);
      load_rows(qb, rr + 3 * R);
    }
    reduce_rows(qa, rr);
    if (rr + 2 * R < RB) {                              // three steps left
      load_rows(qa, rr + 2 * R);
      reduce_rows(qb, rr + R);
      reduce_rows(qa, rr + 2 * R);
    } else {
      reduce_rows(qb, rr + R);
    }
  }
  __syncthreads();
  bool any_miss = false;
  if (PASS == 0)
    for (int q = 0; q < a.k; ++q) any_miss |= (a.rec->tok[t].slot[q] < 0);
  for (int row = tid; row < RB; row += 64 * NW) {
    const int h = hb + row;
    if (h >= H) break;
    float sum = 0.f;
    for (int it = 0; it < n_items; ++it) sum += part[(size_t)it * RB + row];
    T* y = static_cast<T*>(a.y) + (size_t)t * H;
    float* ysum = a.ysum + (size_t)t * H;
    if (PASS == 0) {
      if (any_miss) ysum[h] = sum;
      else y[h] = Unit<T>::narrow(sum);
    } else {
      y[h] = Unit<T>::narrow(ysum[h] + sum);
    }
  }
}

// ---------------------------------------------------------------------------
// Batch > 1: grouped kernels.  A task is one distinct expert of the step (a
// record group) or a shared expert, with the list of tokens that compute it;
// the expert's weights are streamed from HBM once per group of up to kGrpTok
// tokens (a group with more tokens is done in two token passes) and every
// loaded unit is multiplied with all of those tokens' vectors.
// ---------------------------------------------------------------------------
constexpr int kGrpTok = 4;       // tokens per pass over the weights
constexpr int kGrpUpl = 2;       // down: 128-bit units of a row segment per lane
constexpr int kGrpRows = 2;      // down: rows in flight

struct GrpTask {
  const char* base;              // expert weights, null = not in this pass
  int F;
  int ntok;
  int tok[SMOE_MAX_BATCH];
  float w[SMOE_MAX_BATCH];
  float* act;                    // [SMOE_MAX_BATCH][F] activations of this task
};

// task index: [0, maxg) record groups, then the shared experts
template <int PASS>
__device__ __forceinline__ GrpTask grp_task(const FfnArgs& a, int task) {
  GrpTask g;
  g.base = nullptr;
  g.F = 0;
  g.ntok = 0;
  g.act = nullptr;
#pragma unroll
  for (int i = 0; i < SMOE_MAX_BATCH; ++i) { g.tok[i] = 0; g.w[i] = 0.f; }
  if (task < a.maxg) {
    if (task >= a.rec->n_groups) return g;
    const GroupTask& r = a.rec->grp[task];
    int gs;
    if (PASS == 0) {
      if (r.slot < 0) return g;
      gs = a.slot_base + r.slot;
    } else {
      gs = a.slot_override[task];
      if (gs < 0) return g;
    }
    g.base = a.slab + (int64_t)gs * a.expert_bytes;
    g.F = a.F;
    g.ntok = r.ntok;
#pragma unroll
    for (int i = 0; i < SMOE_MAX_BATCH; ++i) { g.tok[i] = r.tok[i]; g.w[i] = r.w[i]; }
    g.act = a.act + (size_t)task * SMOE_MAX_BATCH * a.F;
  } else {
    if (PASS != 0) return g;
    const int sidx = task - a.maxg;
    g.base = a.shared + (int64_t)sidx * a.shared_bytes;
    g.F = a.Fs;
    g.ntok = a.B;
#pragma unroll
    for (int i = 0; i < SMOE_MAX_BATCH; ++i) { g.tok[i] = i; g.w[i] = 1.0f; }
    g.act = a.act + a.act_shared_off + (size_t)sidx * SMOE_MAX_BATCH * a.Fs;
  }
  return g;
}

// Up projection for a task and one token pass.  The hidden states of the up
// to kGrpTok tokens sit in LDS as stored; a wave owns whole rows and keeps the
// 2*UPL loaded units of one f-row pair in registers while it walks the tokens.
template <typename T, int UPL, int PASS>
__global__ __launch_bounds__(256) void ffn_up_grp_kernel(const FfnArgs a) {
  extern __shared__ __align__(16) unsigned char xs_raw[];      // [kGrpTok][H] elements of T
  constexpr int N = Unit<T>::N;
  using raw = typename Unit<T>::raw;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int routed_blocks = a.maxg * 2 * a.tilesR;
  int task, tpass, tile;
  if ((int)blockIdx.x < routed_blocks) {
    task = blockIdx.x / (2 * a.tilesR);
    const int r = blockIdx.x - task * 2 * a.tilesR;
    tpass = r / a.tilesR; tile = r - tpass * a.tilesR;
  } else {
    const int b = blockIdx.x - routed_blocks;
    const int sidx = b / (2 * a.tilesS);
    const int r = b - sidx * 2 * a.tilesS;
    tpass = r / a.tilesS; tile = r - tpass * a.tilesS;
    task = a.maxg + sidx;
  }
  const GrpTask g = grp_task<PASS>(a, task);
  const int t0 = tpass * kGrpTok;
  if (g.base == nullptr || t0 >= g.ntok) return;
  const int nt = min(kGrpTok, g.ntok - t0);
  const int H = a.H, F = g.F;
  const int units = H / N;
  const T* W1 = reinterpret_cast<const T*>(g.base);
  const T* W3 = W1 + (size_t)F * H;
  raw* xs = reinterpret_cast<raw*>(xs_raw);                    // [kGrpTok][units]

  int toks[kGrpTok]; float wts[kGrpTok];
#pragma unroll
  for (int i = 0; i < kGrpTok; ++i) {
    toks[i] = 0; wts[i] = 0.f;
#pragma unroll
    for (int q = 0; q < SMOE_MAX_BATCH; ++q)
      if (q == t0 + i) { toks[i] = g.tok[q]; wts[i] = g.w[q]; }
  }
#pragma unroll
  for (int i = 0; i < kGrpTok; ++i)
    if (i < nt) {
      const T* x = static_cast<const T*>(a.x) + (size_t)toks[i] * H;
      for (int u = tid; u < units; u += 256) xs[i * units + u] = *reinterpret_cast<const raw*>(x + (size_t)u * N);
    }
  __syncthreads();

  const int per_wave = a.TF >> 2;
  const int f_begin = tile * a.TF + wave * per_wave;
  for (int fi = 0; fi < per_wave; ++fi) {
    const int f = f_begin + fi;
    if (f >= F) break;
    const T* gr = W1 + (size_t)f * H;
    const T* ur = W3 + (size_t)f * H;
    raw qg[UPL], qu[UPL];
#pragma unroll
    for (int s = 0; s < UPL; ++s) {
      const int u = s * kWave + lane;
      if (u < units) { qg[s] = Unit<T>::load(gr + (size_t)u * N); qu[s] = Unit<T>::load(ur + (size_t)u * N); }
      else { qg[s] = raw{}; qu[s] = raw{}; }
    }
#pragma unroll
    for (int i = 0; i < kGrpTok; ++i) {
      if (i < nt) {                                            // uniform
        float ag = 0.f, au = 0.f;
#pragma unroll
        for (int s = 0; s < UPL; ++s) {
          const int u = s * kWave + lane;
          const raw xv = (u < units) ? xs[i * units + u] : raw{};
          ag = Unit<T>::dot(qg[s], xv, ag);
          au = Unit<T>::dot(qu[s], xv, au);
        }
        ag = wave_sum(ag);
        au = wave_sum(au);
        if (lane == 0) {
          const float v = wts[i] * (ag / (1.0f + expf(-ag))) * au;
          if (a.mfma_down) {
            // the MFMA down kernel takes the activation as two bf16 terms, hi + lo (|error| <= 2^-17 |v|):
            // the row of F floats holds hi[F] followed by lo[F]
            uint16_t* row16 = reinterpret_cast<uint16_t*>(g.act + (size_t)(t0 + i) * F);
            const bf16_t hi = Unit<bf16_t>::narrow(v);
            row16[f] = hi.v;
            row16[F + f] = Unit<bf16_t>::narrow(v - Unit<bf16_t>::widen1(hi)).v;
          } else {
            g.act[(size_t)(t0 + i) * F + f] = v;
          }
        }
      }
    }
  }
}

// Down projection + combine for all tokens of the step.  A block owns RBG
// output rows.  Work item = (task, column segment of 64*kGrpUpl units); the
// four waves take items round-robin, keep the item's activation slices of up
// to kGrpTok tokens in registers and stream the block's rows.  Partial sums go
// to LDS [item][token slot][row]; after one barrier they are added per token
// in item order.
template <typename T, int PASS>
__global__ __launch_bounds__(256) void ffn_down_grp_kernel(const FfnArgs a) {
  extern __shared__ __align__(16) float part[];       // [items][SMOE_MAX_BATCH][RBG]
  constexpr int N = Unit<T>::N;
  constexpr int UPL = kGrpUpl, R = kGrpRows;
  using raw = typename Unit<T>::raw;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int RB = a.RBG, H = a.H;
  const int hb = blockIdx.x * RB;
  const int n_groups = min(a.rec->n_groups, a.maxg);
  const int items_r = n_groups * a.nsegGR;
  const int n_items = items_r + a.ns * a.nsegGS;

  for (int i = tid; i < n_items * SMOE_MAX_BATCH * RB; i += 256) part[i] = 0.f;
  __syncthreads();

  for (int it = wave; it < n_items; it += 4) {
    int task, seg;
    if (it < items_r) { task = it / a.nsegGR; seg = it - task * a.nsegGR; }
    else { const int q = it - items_r; const int sidx = q / a.nsegGS; seg = q - sidx * a.nsegGS; task = a.maxg + sidx; }
    const GrpTask g = grp_task<PASS>(a, task);
    if (g.base == nullptr) continue;
    const int F = g.F;
    const int units = F / N;
    const int ubeg = seg * kWave * UPL;
    const int uend = min(units, ubeg + kWave * UPL);
    const T* W2 = reinterpret_cast<const T*>(g.base) + 2 * (size_t)F * H;
    float* pitem = part + (size_t)it * SMOE_MAX_BATCH * RB;
    for (int t0 = 0; t0 < g.ntok; t0 += kGrpTok) {
      const int nt = min(kGrpTok, g.ntok - t0);
      float ar[kGrpTok][UPL][N];
#pragma unroll
      for (int i = 0; i < kGrpTok; ++i)
#pragma unroll
        for (int s = 0; s < UPL; ++s) {
          const int u = ubeg + s * kWave + lane;
          if (i < nt && u < uend) {
            const float* ap = g.act + (size_t)(t0 + i) * F + (size_t)u * N;
#pragma unroll
            for (int e = 0; e < N; e += 4) {
              const float4 v = *reinterpret_cast<const float4*>(ap + e);
              ar[i][s][e] = v.x; ar[i][s][e + 1] = v.y; ar[i][s][e + 2] = v.z; ar[i][s][e + 3] = v.w;
            }
          } else {
#pragma unroll
            for (int e = 0; e < N; ++e) ar[i][s][e] = 0.f;
          }
        }
      for (int rr = 0; rr < RB; rr += R) {
        raw q[R][UPL];
#pragma unroll
        for (int r2 = 0; r2 < R; ++r2) {
          const T* row = W2 + (size_t)min(hb + rr + r2, H - 1) * F;
#pragma unroll
          for (int s = 0; s < UPL; ++s) {
            const int u = ubeg + s * kWave + lane;
            q[r2][s] = (u < uend) ? Unit<T>::load(row + (size_t)u * N) : raw{};
          }
        }
#pragma unroll
        for (int r2 = 0; r2 < R; ++r2) {
          float w[UPL][N];
#pragma unroll
          for (int s = 0; s < UPL; ++s) Unit<T>::widen(q[r2][s], w[s]);
#pragma unroll
          for (int i = 0; i < kGrpTok; ++i) {
            if (i < nt) {                                      // uniform
              float acc = 0.f;
#pragma unroll
              for (int s = 0; s < UPL; ++s)
#pragma unroll
                for (int e = 0; e < N; ++e) acc = fmaf(w[s][e], ar[i][s][e], acc);
              acc = wave_sum(acc);
              if (lane == 0 && rr + r2 < RB) pitem[(size_t)(t0 + i) * RB + rr + r2] = acc;
            }
          }
        }
      }
    }
  }
  __syncthreads();
  for (int idx = tid; idx < a.B * RB; idx += 256) {
    const int t = idx / RB, row = idx - t * RB;
    const int h = hb + row;
    if (h >= H) continue;
    bool any_miss = false;
    for (int q = 0; q < a.k; ++q) any_miss |= (a.rec->tok[t].slot[q] < 0);
    if (PASS == 1 && !any_miss) continue;
    float sum = 0.f;
    for (int gi = 0; gi < n_groups; ++gi) {
      const GroupTask& r = a.rec->grp[gi];
      int pos = -1;
      for (int i = 0; i < r.ntok; ++i) pos = (r.tok[i] == t) ? i : pos;
      if (pos < 0) continue;
      for (int sg = 0; sg < a.nsegGR; ++sg)
        sum += part[((size_t)(gi * a.nsegGR + sg) * SMOE_MAX_BATCH + pos) * RB + row];
    }
    for (int sidx = 0; sidx < a.ns; ++sidx)
      for (int sg = 0; sg < a.nsegGS; ++sg)
        sum += part[((size_t)(items_r + sidx * a.nsegGS + sg) * SMOE_MAX_BATCH + t) * RB + row];
    T* y = static_cast<T*>(a.y) + (size_t)t * H;
    float* ysum = a.ysum + (size_t)t * H;
    if (PASS == 0) {
      if (any_miss) ysum[h] = sum;
      else y[h] = Unit<T>::narrow(sum);
    } else {
      y[h] = Unit<T>::narrow(ysum[h] + sum);
    }
  }
}

// Batch > 1, bf16: down projection + combine on the matrix cores.  With several
// tokens per expert the product W2[rows, cols] x act[cols, tokens] is a real
// contraction; on the vector ALUs it costs one cross-lane reduction per (row,
// token), on MFMA none.  A block owns RT <= 16 output rows (the M of the
// 16x16x32 tile is 16: with RT < 16 the last tile rows are neither loaded nor
// written, their LDS rows hold whatever was there and their results are dropped;
// RT is chosen so that the grid has at least one block per compute unit, which
// is what this kernel's rate scales with).  K runs over an item = (task,
// 256-column segment).  The activations
// come as two bf16 terms (hi + lo) written by the up kernel; with at most 8
// tokens per step both fit the 16 tile columns: column j holds the hi terms of
// token j, column 8 + j its lo terms, so ONE MFMA per K-step multiplies both and
// the two halves of the result tile are added in the epilogue.  Each of the
// eight waves takes a contiguous range of the items (it walks along the rows of
// one expert, segment after segment; measured 3 % faster than every eighth item,
// which a.mfma_contig = 0 keeps) and stages its 16 x 256 weight tile through a
// private, padded LDS region (coalesced 128-bit global loads in, MFMA operand
// order out) and accumulates one 16 x 16 fp32 tile over all of its items.  The
// activations of the next item and the weight tiles of the next two are in
// flight while an item is multiplied (loads retire in order, so an activation
// load that is waited for must be older than the tiles meant to stay in flight).
// The eight tiles are then added in wave order.
static_assert(SMOE_MAX_BATCH <= 8, "hi and lo terms of every token share the 16 tile columns");

// 128-bit loads through pointers that are known to point to device memory.  A pointer that went
// through LDS (the down kernel's task table) has lost its address space; loading through it is a
// generic ("flat") load, which counts on the vector-memory AND the LDS counter, and the compiler
// then waits for every outstanding load before the next LDS access: no load stays in flight
// across an item.  The explicit address space brings back global loads.
typedef const u32x4 __attribute__((address_space(1)))* global_u32x4_ptr;
__device__ __forceinline__ u32x4 load_global_stream(const void* p) {
  return __builtin_nontemporal_load((global_u32x4_ptr)p);
}
__device__ __forceinline__ u32x4 load_global(const void* p) { return *(global_u32x4_ptr)p; }
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int kMfmaCols = 256;                  // columns per item
constexpr int kMfmaRowBytes = 2 * kMfmaCols + 16;   // staged row + pad against bank conflicts
constexpr int kMfmaWaves = 8;
constexpr int kMfmaLdsBytes = kMfmaWaves * 16 * kMfmaRowBytes;
constexpr int kMfmaTaskTabBytes = (SMOE_MAX_EXPERTS + SMOE_MAX_SHARED) * 48;

// Batch > 1, bf16: up projection on the matrix cores.  A block = one task x 64
// f-rows; each of its four waves owns 16 rows of W1 and the same 16 rows of W3
// (M = 16), the tile columns are the step's tokens (B operand = x as stored,
// bf16, so one MFMA per K-step is exact), K walks H in 256-column segments.
// Both weight tiles of a segment are staged through the wave's private LDS
// region; the loads of the next segment are issued right after staging.  The
// epilogue applies w * silu(g) * u for the tokens of the task and writes the
// activation as hi + lo bf16 terms for the MFMA down kernel.
constexpr int kMfmaUpWaves = 4;
constexpr int kMfmaUpLdsBytes = kMfmaUpWaves * 2 * 16 * kMfmaRowBytes;

template <int PASS>
__global__ __launch_bounds__(64 * kMfmaUpWaves) void ffn_up_mfma_kernel(const FfnArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int i16 = lane & 15, g4 = lane >> 4;
  const int tiles_r = (a.F + 63) / 64, tiles_s = a.ns ? (a.Fs + 63) / 64 : 0;
  const int routed_blocks = a.maxg * tiles_r;
  int task, tile;
  if ((int)blockIdx.x < routed_blocks) { task = blockIdx.x / tiles_r; tile = blockIdx.x - task * tiles_r; }
  else { const int b = blockIdx.x - routed_blocks; const int sidx = b / tiles_s; tile = b - sidx * tiles_s; task = a.maxg + sidx; }
  const GrpTask g = grp_task<PASS>(a, task);
  if (g.base == nullptr) return;
  const int H = a.H, F = g.F;
  const int f0 = tile * 64 + wave * 16;
  if (f0 >= F) return;
  const bf16_t* W1 = reinterpret_cast<const bf16_t*>(g.base);
  const bf16_t* W3 = W1 + (size_t)F * H;
  const bf16_t* x = static_cast<const bf16_t*>(a.x);
  unsigned char* st1 = lds + (size_t)wave * 2 * 16 * kMfmaRowBytes;
  unsigned char* st3 = st1 + 16 * kMfmaRowBytes;
  const int unit = lane & 31, rsub = lane >> 5;
  const int nseg = (H + kMfmaCols - 1) / kMfmaCols;

  u32x4 w1reg[8], w3reg[8];
  auto load_seg = [&](int sg) {
    const int c0 = sg * kMfmaCols;
    const bool live = sg < nseg && c0 + unit * 8 < H;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const size_t roff = (size_t)min(f0 + 2 * q + rsub, F - 1) * H + c0 + unit * 8;
      w1reg[q] = live ? Unit<bf16_t>::load(W1 + roff) : u32x4{};
      w3reg[q] = live ? Unit<bf16_t>::load(W3 + roff) : u32x4{};
    }
  };
  f32x4 accg = {0.f, 0.f, 0.f, 0.f}, accu = {0.f, 0.f, 0.f, 0.f};
  load_seg(0);
  for (int sg = 0; sg < nseg; ++sg) {
    const int c0 = sg * kMfmaCols;
    u32x4 xf[8];                              // x of token i16, 8 K-steps of this segment
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      const int col = c0 + 32 * st + 8 * g4;
      xf[st] = (i16 < a.B && col < H) ? *reinterpret_cast<const u32x4*>(x + (size_t)i16 * H + col) : u32x4{};
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      *reinterpret_cast<u32x4*>(st1 + (2 * q + rsub) * kMfmaRowBytes + unit * 16) = w1reg[q];
      *reinterpret_cast<u32x4*>(st3 + (2 * q + rsub) * kMfmaRowBytes + unit * 16) = w3reg[q];
    }
    __builtin_amdgcn_wave_barrier();
    load_seg(sg + 1);
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      const u32x4 a1 = *reinterpret_cast<const u32x4*>(st1 + i16 * kMfmaRowBytes + (4 * st + g4) * 16);
      const u32x4 a3 = *reinterpret_cast<const u32x4*>(st3 + i16 * kMfmaRowBytes + (4 * st + g4) * 16);
      const u32x4 xb = xf[st];
      accg = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a1), __builtin_bit_cast(bf16x8, xb), accg, 0, 0, 0);
      accu = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a3), __builtin_bit_cast(bf16x8, xb), accu, 0, 0, 0);
    }
    __builtin_amdgcn_wave_barrier();
  }
  // lane holds rows f0 + 4*g4 + r of token i16: store if that token belongs to the task
  int pos = -1; float wgt = 0.f;
#pragma unroll
  for (int q = 0; q < SMOE_MAX_BATCH; ++q)
    if (q < g.ntok && g.tok[q] == i16) { pos = q; wgt = g.w[q]; }
  if (pos >= 0) {
    uint16_t* row16 = reinterpret_cast<uint16_t*>(g.act + (size_t)pos * F);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int f = f0 + 4 * g4 + r;
      if (f < F) {
        const float ag = accg[r], au = accu[r];
        const float v = wgt * (ag / (1.0f + expf(-ag))) * au;
        const bf16_t hi = Unit<bf16_t>::narrow(v);
        row16[f] = hi.v;
        row16[F + f] = Unit<bf16_t>::narrow(v - Unit<bf16_t>::widen1(hi)).v;
      }
    }
  }
}

template <int PASS, int RT>
__global__ __launch_bounds__(64 * kMfmaWaves) void ffn_down_mfma_kernel(const FfnArgs a) {
  static_assert(RT % 2 == 0 && RT >= 2 && RT <= 16, "a block owns RT of the tile's 16 rows, loaded two per instruction");
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // item bookkeeping stays on the scalar unit
  const int i16 = lane & 15, g4 = lane >> 4;     // tile row / column index, K sub-block
  const int H = a.H;
  const int hb = blockIdx.x * RT;
  const int n_groups = min(a.rec->n_groups, a.maxg);
  const int nsegR = (a.F + kMfmaCols - 1) / kMfmaCols;
  const int nsegS = a.ns ? (a.Fs + kMfmaCols - 1) / kMfmaCols : 0;
  const int items_r = n_groups * nsegR;
  const int n_items = items_r + a.ns * nsegS;
  unsigned char* stage = lds + (size_t)wave * 16 * kMfmaRowBytes;
  int next_it = 0;                          // item index at which describe() last stopped
  // Items of a wave: a contiguous range (a.mfma_contig), so that the wave walks along the rows of one
  // task segment after segment, or every eighth item.
  // (the pass over the freshly loaded experts has work for a few tasks only: every eighth item
  // spreads those over all waves, a contiguous range would give a task to one or two of them)
  const bool contig = PASS == 0 && a.mfma_contig;
  const int ipw = (n_items + kMfmaWaves - 1) / kMfmaWaves;
  const int it_step = contig ? 1 : kMfmaWaves;
  const int it_first = contig ? wave * ipw : wave;
  const int it_end = contig ? min(n_items, (wave + 1) * ipw) : n_items;

  // Task table in LDS (built once per block): decoding an item must not cost a
  // round trip to the decision record in the middle of the pipeline.
  struct TaskEnt {
    const char* w2;          // W2 of the task, null = not in this pass
    const float* act;        // its activation rows
    int F, ntok;
    signed char pos_of_tok[16];   // position of token j in the task's list, -1 = absent
  };
  static_assert(sizeof(TaskEnt) <= 48, "task table entry outgrew its LDS budget");
  TaskEnt* ttab = reinterpret_cast<TaskEnt*>(lds + kMfmaLdsBytes);
  const int n_tasks = a.maxg + a.ns;
  for (int task = tid; task < n_tasks; task += 64 * kMfmaWaves) {
    const GrpTask g = grp_task<PASS>(a, task);
    TaskEnt e;
    e.w2 = g.base ? g.base + 2 * (size_t)g.F * H * sizeof(bf16_t) : nullptr;
    e.act = g.act;
    e.F = g.F;
    e.ntok = g.ntok;
    for (int j = 0; j < 16; ++j) {
      int pos = -1;
#pragma unroll
      for (int q = 0; q < SMOE_MAX_BATCH; ++q) pos = (q < g.ntok && g.tok[q] == j) ? q : pos;
      e.pos_of_tok[j] = (signed char)pos;
    }
    ttab[task] = e;
  }
  __syncthreads();

  // One item: where its 16 x 256 weight tile and this lane's activation row live.  Every load
  // of the pipeline is issued unconditionally (a load inside a branch makes the number of loads
  // in flight unknown to the compiler, which then waits for all of them): columns past the end
  // of a short segment are clamped into it and multiplied by zero activations, an item past the
  // end of the list reads 16 bytes of the decision record and is never multiplied.
  struct Item {
    const bf16_t* w2;        // W2 + c0 of row 0 of the matrix
    const uint16_t* arow;    // my tile column's terms of the activation row (hi, or lo F further), at c0
    int F, ncols;
    bool has_tok;            // my column's token is in the task's list
    bool valid;
  };
  const bf16_t* const dummy_w = reinterpret_cast<const bf16_t*>(a.rec);
  auto describe = [&](int it) -> Item {
    Item d{dummy_w, reinterpret_cast<const uint16_t*>(a.rec), 0, 8, false, false};
    // skip forward over items whose task is not part of this pass
    for (; it < it_end; it += it_step) {
      int task, seg;
      if (it < items_r) { task = it / nsegR; seg = it - task * nsegR; }
      else { const int q = it - items_r; const int sidx = q / nsegS; seg = q - sidx * nsegS; task = a.maxg + sidx; }
      const TaskEnt& e = ttab[task];
      // the entry is the same for the whole wave: pointer and width go to scalar registers
      const unsigned long long w2_bits = reinterpret_cast<unsigned long long>(e.w2);
      const unsigned w2_lo = __builtin_amdgcn_readfirstlane((unsigned)w2_bits);
      const unsigned w2_hi = __builtin_amdgcn_readfirstlane((unsigned)(w2_bits >> 32));
      if ((w2_lo | w2_hi) == 0u) continue;
      const int eF = __builtin_amdgcn_readfirstlane(e.F);
      const int c0 = seg * kMfmaCols;
      const int pos = e.pos_of_tok[i16 & 7];
      d.F = eF;
      d.ncols = min(kMfmaCols, eF - c0);
      d.w2 = reinterpret_cast<const bf16_t*>(((unsigned long long)w2_hi << 32) | w2_lo) + c0;
      d.arow = reinterpret_cast<const uint16_t*>(e.act + (size_t)max(pos, 0) * eF) + (i16 >> 3) * eF + c0;
      d.has_tok = pos >= 0;
      d.valid = true;
      break;
    }
    next_it = it;
    return d;
  };
  const int unit = lane & 31, rsub = lane >> 5;
  auto load_tile = [&](const Item& d, u32x4 (&wreg)[8]) {   // RT/2 coalesced loads, two 512-byte rows each
    const int cu = min(unit * 8, d.ncols - 8);
#pragma unroll
    for (int q = 0; q < RT / 2; ++q) {
      const int r = 2 * q + rsub;
      wreg[q] = load_global_stream(d.w2 + (size_t)min(hb + r, H - 1) * d.F + cu);
    }
  };
  // B operand of item d for this lane: 8 K-steps of 8 columns of my token's hi (tile
  // columns 0..7) or lo (columns 8..15) terms
  auto load_act = [&](const Item& d, u32x4 (&areg)[8]) {
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      const int col = 32 * st + 8 * g4;
      areg[st] = load_global(d.arow + min(col, d.ncols - 8));
    }
  };
  // the item's weight tile from registers to LDS (row r at r * kMfmaRowBytes)
  auto stage_tile = [&](const u32x4 (&wreg)[8]) {
#pragma unroll
    for (int q = 0; q < RT / 2; ++q)
      *reinterpret_cast<u32x4*>(stage + (2 * q + rsub) * kMfmaRowBytes + unit * 16) = wreg[q];
    __builtin_amdgcn_wave_barrier();
  };
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  // (what was loaded for a token outside the task's list or past the end of a short segment is
  // replaced by zeros here, next to its use: a select right behind the load would wait for it)
  auto multiply_staged = [&](const u32x4 (&areg)[8], bool has_tok, int ncols) {
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      const u32x4 af = *reinterpret_cast<const u32x4*>(stage + i16 * kMfmaRowBytes + (4 * st + g4) * 16);
      const u32x4 b4 = (has_tok && 32 * st + 8 * g4 < ncols) ? areg[st] : u32x4{};
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af), __builtin_bit_cast(bf16x8, b4),
                                                    acc, 0, 0, 0);
    }
    __builtin_amdgcn_wave_barrier();
  };
  // Issue order per item n: activations of item n+1, then the tile of item n+3.  Loads retire in
  // order, so the multiply's wait for the activations of item n (issued one item earlier) lets the
  // tiles of items n+2 and n+3 stay in flight: 16 KB per wave during the multiply, and a tile has
  // two items' time to arrive.  Three tile buffers, two activation buffers, three descriptors,
  // all indexed at compile time (the loop body is six items).
  u32x4 wt[3][8], av[2][8];
  bool av_tok[2];
  int av_cols[2];
  Item q[3];
  q[0] = describe(it_first);
  load_tile(q[0], wt[0]);
  load_act(q[0], av[0]);
  av_tok[0] = q[0].has_tok;
  av_cols[0] = q[0].ncols;
  q[1] = describe(next_it + it_step);
  load_tile(q[1], wt[1]);
  q[2] = describe(next_it + it_step);
  load_tile(q[2], wt[2]);
  bool more = q[0].valid;
  while (more) {
#pragma unroll
    for (int s6 = 0; s6 < 6; ++s6) {
      const int t3 = s6 % 3, a2 = s6 & 1;
      stage_tile(wt[t3]);                         // item n (buffer n % 3)
      load_act(q[(s6 + 1) % 3], av[a2 ^ 1]);      // item n + 1
      av_tok[a2 ^ 1] = q[(s6 + 1) % 3].has_tok;
      av_cols[a2 ^ 1] = q[(s6 + 1) % 3].ncols;
      q[t3] = describe(next_it + it_step);     // item n + 3 takes over item n's buffer and descriptor
      load_tile(q[t3], wt[t3]);
      multiply_staged(av[a2], av_tok[a2], av_cols[a2]);
      if (!q[(s6 + 1) % 3].valid) { more = false; break; }
    }
  }

  // ---- add the eight tiles in wave order (hi half, then lo half); lane holds rows 4*g4 + r, column i16 ----
  __syncthreads();
  float* red = reinterpret_cast<float*>(lds);           // [wave][16 rows][16 cols]
#pragma unroll
  for (int r = 0; r < 4; ++r) red[(wave * 16 + 4 * g4 + r) * 16 + i16] = acc[r];
  __syncthreads();
  for (int idx = tid; idx < RT * a.B; idx += 64 * kMfmaWaves) {
    const int t = idx / RT, row = idx - t * RT;
    const int h = hb + row;
    if (h >= H) continue;
    bool any_miss = false;
    for (int q = 0; q < a.k; ++q) any_miss |= (a.rec->tok[t].slot[q] < 0);
    if (PASS == 1 && !any_miss) continue;
    float sum = 0.f;
    for (int w = 0; w < kMfmaWaves; ++w) sum += red[(w * 16 + row) * 16 + t] + red[(w * 16 + row) * 16 + 8 + t];
    bf16_t* y = static_cast<bf16_t*>(a.y) + (size_t)t * H;
    float* ysum = a.ysum + (size_t)t * H;
    if (PASS == 0) {
      if (any_miss) ysum[h] = sum;
      else y[h] = Unit<bf16_t>::narrow(sum);
    } else {
      y[h] = Unit<bf16_t>::narrow(ysum[h] + sum);
    }
  }
}

// Predicted input of the next MoE layer from this layer's partial output (top-
// score prefetch, Section IV-C, Fig. "prefetch": the prediction starts from what
// the experts already on the GPU have produced, before the loaded ones are
// done).  With the attention block outside this path the next layer's input is
// modelled as the RMS-normalised residual sum: xp = (x + p) / rms(x + p), where
// p is the resident pass's result -- its fp32 sums for a token that still waits
// for experts, its finished output otherwise.  One block per token.
template <typename T>
__global__ __launch_bounds__(256) void predict_state_kernel(const StepRec* rec, const T* __restrict__ x,
                                                            const T* __restrict__ y,
                                                            const float* __restrict__ ysum, T* __restrict__ xp,
                                                            int H, int k) {
  __shared__ float red[4];
  const int t = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  bool any_miss = false;
  for (int q = 0; q < k; ++q) any_miss |= (rec->tok[t].slot[q] < 0);
  const T* xt = x + (size_t)t * H;
  const T* yt = y + (size_t)t * H;
  const float* st = ysum + (size_t)t * H;
  float acc = 0.f;
  for (int h = tid; h < H; h += 256) {
    const float z = Unit<T>::widen1(xt[h]) + (any_miss ? st[h] : Unit<T>::widen1(yt[h]));
    acc = fmaf(z, z, acc);
  }
  acc = wave_sum(acc);
  if (lane == 0) red[wave] = acc;
  __syncthreads();
  const float ms = ((red[0] + red[1]) + (red[2] + red[3])) / (float)H;
  const float inv = 1.0f / sqrtf(ms);
  for (int h = tid; h < H; h += 256) {
    const float z = Unit<T>::widen1(xt[h]) + (any_miss ? st[h] : Unit<T>::widen1(yt[h]));
    xp[(size_t)t * H + h] = Unit<T>::narrow(z * inv);
  }
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst,
                                                   const uint4* __restrict__ src, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    dst[i] = src[i];
}

// ysum[i] += part[i]: `part` is what the host cores computed for the experts that
// Algorithm 2 gave to the CPU, read straight from pinned host memory.
__global__ __launch_bounds__(256) void add_partial_kernel(float4* __restrict__ ysum,
                                                          const float4* __restrict__ part, int n4) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n4) {
    float4 a = ysum[i];
    const float4 b = part[i];
    a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    ysum[i] = a;
  }
}

}  // namespace

template <typename T, int PASS>
static void launch_up_t(const FfnArgs& a, const RouteArgs& ra, hipStream_t s) {
  if (a.grouped && a.mfma_down && a.mfma_up) {
    static bool lds_opted_in[2] = {false, false};
    if (!lds_opted_in[PASS]) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_up_mfma_kernel<PASS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kMfmaUpLdsBytes);
      lds_opted_in[PASS] = true;
    }
    const int grid = a.maxg * ((a.F + 63) / 64) + a.ns * ((a.Fs + 63) / 64);
    hipLaunchKernelGGL((ffn_up_mfma_kernel<PASS>), dim3(grid), dim3(64 * kMfmaUpWaves), kMfmaUpLdsBytes, s, a);
    return;
  }
  if (a.grouped) {
    const int grid = a.maxg * 2 * a.tilesR + a.ns * 2 * a.tilesS;
    const size_t lds = (size_t)kGrpTok * a.H * sizeof(T);
    switch (a.up_upl) {
      case 1: hipLaunchKernelGGL((ffn_up_grp_kernel<T, 1, PASS>), dim3(grid), dim3(256), lds, s, a); return;
      case 2: hipLaunchKernelGGL((ffn_up_grp_kernel<T, 2, PASS>), dim3(grid), dim3(256), lds, s, a); return;
      case 4: hipLaunchKernelGGL((ffn_up_grp_kernel<T, 4, PASS>), dim3(grid), dim3(256), lds, s, a); return;
      default: hipLaunchKernelGGL((ffn_up_grp_kernel<T, 8, PASS>), dim3(grid), dim3(256), lds, s, a); return;
    }
  }
  const int grid = a.B * (a.k * a.tilesR + a.ns * a.tilesS);
  if (PASS == 0 && a.fused_select) {
    const int fgrid = grid + ra.gate_blocks;            // (the gate GEMV's blocks come first)
    switch (a.up_upl) {
      case 1: hipLaunchKernelGGL((ffn_up_reg_kernel<T, 1, 0, true>), dim3(fgrid), dim3(256), 0, s, a, ra); return;
      case 2: hipLaunchKernelGGL((ffn_up_reg_kernel<T, 2, 0, true>), dim3(fgrid), dim3(256), 0, s, a, ra); return;
      case 4: hipLaunchKernelGGL((ffn_up_reg_kernel<T, 4, 0, true>), dim3(fgrid), dim3(256), 0, s, a, ra); return;
      default: hipLaunchKernelGGL((ffn_up_reg_kernel<T, 8, 0, true>), dim3(fgrid), dim3(256), 0, s, a, ra); return;
    }
  }
  switch (a.up_upl) {
    case 1: hipLaunchKernelGGL((ffn_up_reg_kernel<T, 1, PASS, false>), dim3(grid), dim3(256), 0, s, a, ra); return;
    case 2: hipLaunchKernelGGL((ffn_up_reg_kernel<T, 2, PASS, false>), dim3(grid), dim3(256), 0, s, a, ra); return;
    case 4: hipLaunchKernelGGL((ffn_up_reg_kernel<T, 4, PASS, false>), dim3(grid), dim3(256), 0, s, a, ra); return;
    case 8: hipLaunchKernelGGL((ffn_up_reg_kernel<T, 8, PASS, false>), dim3(grid), dim3(256), 0, s, a, ra); return;
    default: break;
  }
  const size_t lds = (size_t)a.H * sizeof(float);
  hipLaunchKernelGGL((ffn_up_kernel<T, PASS>), dim3(grid), dim3(256), lds, s, a);
}

void launch_ffn_up(const FfnArgs& a, const RouteArgs& ra, int dtype, hipStream_t s) {
  if (dtype == SMOE_DTYPE_FP32) {
    if (a.pass == 0) launch_up_t<float, 0>(a, ra, s); else launch_up_t<float, 1>(a, ra, s);
  } else {
    if (a.pass == 0) launch_up_t<bf16_t, 0>(a, ra, s); else launch_up_t<bf16_t, 1>(a, ra, s);
  }
}

template <typename T, int PASS>
static void launch_down_t(const FfnArgs& a, hipStream_t s) {
  if (a.grouped) {
    if (a.mfma_down) {
      // the staging area is larger than the 64 KB default: opt in once per instance
#define SMOE_MFMA_DOWN_CASE(RT)                                                                              \
  if (a.mfma_rt == RT) {                                                                                     \
    static bool opted_in = false;                                                                            \
    if (!opted_in) {                                                                                         \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_down_mfma_kernel<PASS, RT>),              \
                                hipFuncAttributeMaxDynamicSharedMemorySize, kMfmaLdsBytes + kMfmaTaskTabBytes); \
      opted_in = true;                                                                                       \
    }                                                                                                        \
    hipLaunchKernelGGL((ffn_down_mfma_kernel<PASS, RT>), dim3((a.H + RT - 1) / RT), dim3(64 * kMfmaWaves),   \
                       kMfmaLdsBytes + kMfmaTaskTabBytes, s, a);                                             \
    return;                                                                                                  \
  }
      SMOE_MFMA_DOWN_CASE(8)
      SMOE_MFMA_DOWN_CASE(12)
      SMOE_MFMA_DOWN_CASE(14)
      SMOE_MFMA_DOWN_CASE(16)
#undef SMOE_MFMA_DOWN_CASE
      return;
    }
    const int grid = (a.H + a.RBG - 1) / a.RBG;
    hipLaunchKernelGGL((ffn_down_grp_kernel<T, PASS>), dim3(grid), dim3(256), grouped_down_lds_bytes(a), s, a);
    return;
  }
  const int grid = a.B * a.htiles;
  if (a.down_upl > 0) {
    const size_t lds = (size_t)(a.k * a.nsegR + a.ns * a.nsegS) * a.RB * sizeof(float);
#define SMOE_DOWN_CASE(U, RR)                                                                                 \
  if (a.down_upl == U && a.down_r == RR) {                                                                    \
    if (a.down_nw >= 8)                                                                                       \
      hipLaunchKernelGGL((ffn_down_reg_kernel<T, U, RR, 8, PASS>), dim3(grid), dim3(512), lds, s, a);         \
    else                                                                                                      \
      hipLaunchKernelGGL((ffn_down_reg_kernel<T, U, RR, 4, PASS>), dim3(grid), dim3(256), lds, s, a);         \
    return;                                                                                                   \
  }
    SMOE_DOWN_CASE(2, 4)
    SMOE_DOWN_CASE(4, 2)
    SMOE_DOWN_CASE(6, 2)
    SMOE_DOWN_CASE(8, 1)
#undef SMOE_DOWN_CASE
  }
  const size_t lds = (size_t)a.down_lds_floats * sizeof(float);
  if (a.R == 1) hipLaunchKernelGGL((ffn_down_kernel<T, 1, PASS>), dim3(grid), dim3(256), lds, s, a);
  else if (a.R == 2) hipLaunchKernelGGL((ffn_down_kernel<T, 2, PASS>), dim3(grid), dim3(256), lds, s, a);
  else hipLaunchKernelGGL((ffn_down_kernel<T, 4, PASS>), dim3(grid), dim3(256), lds, s, a);
}

void launch_ffn_down(const FfnArgs& a, int dtype, hipStream_t s) {
  if (dtype == SMOE_DTYPE_FP32) {
    if (a.pass == 0) launch_down_t<float, 0>(a, s); else launch_down_t<float, 1>(a, s);
  } else {
    if (a.pass == 0) launch_down_t<bf16_t, 0>(a, s); else launch_down_t<bf16_t, 1>(a, s);
  }
}

size_t grouped_down_lds_bytes(const FfnArgs& a) {
  return (size_t)(a.maxg * a.nsegGR + a.ns * a.nsegGS) * SMOE_MAX_BATCH * a.RBG * sizeof(float);
}

void launch_copy(void* dst, const void* src, int64_t n_bytes, hipStream_t s) {
  const int64_t n = n_bytes / 16;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                     static_cast<uint4*>(dst), static_cast<const uint4*>(src), n);
}

void launch_predict_state(const StepRec* rec, const void* x, const void* y, const float* ysum, void* xp, int B,
                          int H, int k, int dtype, hipStream_t s) {
  if (dtype == SMOE_DTYPE_FP32)
    hipLaunchKernelGGL(predict_state_kernel<float>, dim3(B), dim3(256), 0, s, rec, static_cast<const float*>(x),
                       static_cast<const float*>(y), ysum, static_cast<float*>(xp), H, k);
  else
    hipLaunchKernelGGL(predict_state_kernel<bf16_t>, dim3(B), dim3(256), 0, s, rec,
                       static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(y), ysum,
                       static_cast<bf16_t*>(xp), H, k);
}

void launch_add_partial(float* ysum, const float* part, int n, hipStream_t s) {
  const int n4 = n / 4;
  hipLaunchKernelGGL(add_partial_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                     reinterpret_cast<float4*>(ysum), reinterpret_cast<const float4*>(part), n4);
}

}  // namespace smoe
