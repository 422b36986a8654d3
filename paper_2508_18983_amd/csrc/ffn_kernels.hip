// Batch-1-style SwiGLU expert FFN for the chosen experts and the shared experts
// (Section V-B, GPU operations "Direct expert computation" and "New Expert
// Computation"; shared experts per Section II-A).  Pure weight streaming: every
// weight element is read once from HBM with 128-bit loads, the activation
// vector sits in LDS, one wavefront owns whole rows and reduces with
// cross-lane shuffles, accumulation is fp32.
//
//   up   : act[task][f] = w_task * silu(W1[f].x) * (W3[f].x)
//   down : y[h] = sum_task sum_f W2[h][f] * act[task][f]
//          split over F-chunks; partial sums are combined in a fixed order by
//          the last block to finish each row tile, so the result does not
//          depend on scheduling.
#include "smoe_dev.hpp"

namespace smoe {
namespace {

struct bf16_t { uint16_t v; };

template <typename T> struct Unit;
template <> struct Unit<float> {
  static constexpr int N = 4;
  __device__ static __forceinline__ void load(const float* p, float (&v)[4]) {
    const float4 q = *reinterpret_cast<const float4*>(p);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
  }
  __device__ static __forceinline__ float widen(float s) { return s; }
  __device__ static __forceinline__ float narrow(float s) { return s; }
};
template <> struct Unit<bf16_t> {
  static constexpr int N = 8;
  __device__ static __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const uint4 q = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
    v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
    v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
  }
  __device__ static __forceinline__ float widen(bf16_t s) {
    return __uint_as_float(uint32_t(s.v) << 16);
  }
  __device__ static __forceinline__ bf16_t narrow(float s) {   // round to nearest even
    uint32_t u = __float_as_uint(s);
    u += 0x7fffu + ((u >> 16) & 1u);
    return bf16_t{uint16_t(u >> 16)};
  }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Weights of task (t, j): null when the task is not part of this pass.
__device__ __forceinline__ const char* task_weights(const FfnArgs& a, int t, int j, int task,
                                                    int& F, float& wgt) {
  if (j < a.k) {
    F = a.F;
    wgt = a.rec->tok[t].w[j];
    int g;
    if (a.pass == 0) {
      const int s = a.rec->tok[t].slot[j];
      if (s < 0) return nullptr;
      g = a.slot_base + s;
    } else {
      g = a.slot_override[task];
      if (g < 0) return nullptr;
    }
    return a.slab + (int64_t)g * a.expert_bytes;
  }
  if (a.pass != 0) return nullptr;
  F = a.Fs;
  wgt = 1.0f;
  return a.shared + (int64_t)(j - a.k) * a.shared_bytes;
}

template <typename T>
__global__ __launch_bounds__(256) void ffn_up_kernel(const FfnArgs a) {
  extern __shared__ float xs[];                       // H floats
  constexpr int N = Unit<T>::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int nj = a.k + a.ns;
  const int bpt = a.k * a.tilesR + a.ns * a.tilesS;   // blocks per token
  const int t = blockIdx.x / bpt;
  int r = blockIdx.x - t * bpt, j, tile;
  if (r < a.k * a.tilesR) { j = r / a.tilesR; tile = r - j * a.tilesR; }
  else { r -= a.k * a.tilesR; j = a.k + r / a.tilesS; tile = r - (j - a.k) * a.tilesS; }
  const int task = t * nj + j;
  int F; float wgt;
  const char* base = task_weights(a, t, j, task, F, wgt);
  if (base == nullptr) return;
  const int H = a.H;
  const T* W1 = reinterpret_cast<const T*>(base);
  const T* W3 = W1 + (size_t)F * H;

  const T* x = static_cast<const T*>(a.x) + (size_t)t * H;
  for (int h = tid; h < H; h += 256) xs[h] = Unit<T>::widen(x[h]);
  __syncthreads();

  const int units = H / N;
  const int per_wave = a.TF >> 2;
  const int f_begin = tile * a.TF + wave * per_wave;
  float* act = a.act + (size_t)task * a.Fmax;
  for (int i = 0; i < per_wave; i += 2) {
    const int f = f_begin + i;
    if (f >= F) break;
    const T* g0 = W1 + (size_t)f * H;
    const T* u0 = W3 + (size_t)f * H;
    const T* g1 = g0 + H;
    const T* u1 = u0 + H;
    float ag0 = 0.f, au0 = 0.f, ag1 = 0.f, au1 = 0.f;
#pragma unroll 2
    for (int u = lane; u < units; u += kWave) {
      float a0[N], b0[N], a1[N], b1[N];
      Unit<T>::load(g0 + u * N, a0);
      Unit<T>::load(u0 + u * N, b0);
      Unit<T>::load(g1 + u * N, a1);
      Unit<T>::load(u1 + u * N, b1);
      const float* xv = xs + u * N;
#pragma unroll
      for (int q = 0; q < N; ++q) {
        const float xq = xv[q];
        ag0 = fmaf(a0[q], xq, ag0);
        au0 = fmaf(b0[q], xq, au0);
        ag1 = fmaf(a1[q], xq, ag1);
        au1 = fmaf(b1[q], xq, au1);
      }
    }
    ag0 = wave_sum(ag0); au0 = wave_sum(au0);
    ag1 = wave_sum(ag1); au1 = wave_sum(au1);
    if (lane == 0) {
      act[f] = wgt * (ag0 / (1.0f + expf(-ag0))) * au0;
      act[f + 1] = wgt * (ag1 / (1.0f + expf(-ag1))) * au1;
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void ffn_down_kernel(const FfnArgs a) {
  extern __shared__ float as[];                       // one F-chunk of act
  __shared__ int is_last;
  constexpr int N = Unit<T>::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int nj = a.k + a.ns;
  const int per_tok = a.k * a.chunksR + a.ns * a.chunksS;   // (task, chunk) pairs per token
  const int bpt = a.htiles * per_tok;
  const int t = blockIdx.x / bpt;
  int r = blockIdx.x - t * bpt;
  int tc = r / a.htiles;
  const int ht = r - tc * a.htiles;
  int j, ch, fc;
  if (tc < a.k * a.chunksR) { j = tc / a.chunksR; ch = tc - j * a.chunksR; fc = a.fcR; }
  else { tc -= a.k * a.chunksR; j = a.k + tc / a.chunksS; ch = tc - (j - a.k) * a.chunksS; fc = a.fcS; }
  const int task = t * nj + j;
  int F; float wgt;
  const char* base = task_weights(a, t, j, task, F, wgt);
  if (base == nullptr) return;                        // not in this pass: does not count
  const int H = a.H;
  const T* W2 = reinterpret_cast<const T*>(base) + 2 * (size_t)F * H;
  const int c0 = ch * fc;
  const int clen = min(fc, F - c0);

  const float* act = a.act + (size_t)task * a.Fmax + c0;
  for (int i = tid; i < clen; i += 256) as[i] = act[i];
  __syncthreads();

  const int units = clen / N;
  const int per_wave = a.RB >> 2;
  const int h_begin = ht * a.RB + wave * per_wave;
  float* part = a.partial + ((size_t)task * kMaxChunks + ch) * H;
  for (int i = 0; i < per_wave; i += 4) {
    const int h = h_begin + i;
    if (h >= H) break;
    const T* r0 = W2 + (size_t)h * F + c0;
    const T* r1 = W2 + (size_t)min(h + 1, H - 1) * F + c0;
    const T* r2 = W2 + (size_t)min(h + 2, H - 1) * F + c0;
    const T* r3 = W2 + (size_t)min(h + 3, H - 1) * F + c0;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll 2
    for (int u = lane; u < units; u += kWave) {
      float w0[N], w1[N], w2[N], w3[N];
      Unit<T>::load(r0 + u * N, w0);
      Unit<T>::load(r1 + u * N, w1);
      Unit<T>::load(r2 + u * N, w2);
      Unit<T>::load(r3 + u * N, w3);
      const float* av = as + u * N;
#pragma unroll
      for (int q = 0; q < N; ++q) {
        const float aq = av[q];
        s0 = fmaf(w0[q], aq, s0);
        s1 = fmaf(w1[q], aq, s1);
        s2 = fmaf(w2[q], aq, s2);
        s3 = fmaf(w3[q], aq, s3);
      }
    }
    s0 = wave_sum(s0); s1 = wave_sum(s1); s2 = wave_sum(s2); s3 = wave_sum(s3);
    if (lane == 0) {
      part[h] = s0;
      if (h + 1 < H) part[h + 1] = s1;
      if (h + 2 < H) part[h + 2] = s2;
      if (h + 3 < H) part[h + 3] = s3;
    }
  }

  // ---- last block of this (token, row tile) combines all partial sums -------
  __syncthreads();
  uint32_t* counter = a.counters + (size_t)t * a.htiles + ht;
  if (tid == 0) {
    __threadfence();
    const uint32_t old = atomicAdd(counter, 1u);
    is_last = (old + 1u == (uint32_t)per_tok);
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  T* y = static_cast<T*>(a.y) + (size_t)t * H;
  for (int row = tid; row < a.RB; row += 256) {
    const int h = ht * a.RB + row;
    if (h >= H) break;
    float sum = 0.f;
    for (int jj = 0; jj < nj; ++jj) {
      const int nch = jj < a.k ? a.chunksR : a.chunksS;
      const float* p = a.partial + ((size_t)(t * nj + jj) * kMaxChunks) * H + h;
      for (int c = 0; c < nch; ++c)
        sum += __hip_atomic_load(p + (size_t)c * H, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    y[h] = Unit<T>::narrow(sum);
  }
  if (tid == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst,
                                                   const uint4* __restrict__ src, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    dst[i] = src[i];
}

__global__ void fill_u32_kernel(uint32_t* p, int64_t n, uint32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace

void launch_ffn_up(const FfnArgs& a, int dtype, hipStream_t s) {
  const int grid = a.B * (a.k * a.tilesR + a.ns * a.tilesS);
  const size_t lds = (size_t)a.H * sizeof(float);
  if (dtype == SMOE_DTYPE_FP32)
    hipLaunchKernelGGL(ffn_up_kernel<float>, dim3(grid), dim3(256), lds, s, a);
  else
    hipLaunchKernelGGL(ffn_up_kernel<bf16_t>, dim3(grid), dim3(256), lds, s, a);
}

void launch_ffn_down(const FfnArgs& a, int dtype, hipStream_t s) {
  const int grid = a.B * a.htiles * (a.k * a.chunksR + a.ns * a.chunksS);
  const size_t lds = (size_t)(a.fcR > a.fcS ? a.fcR : a.fcS) * sizeof(float);
  if (dtype == SMOE_DTYPE_FP32)
    hipLaunchKernelGGL(ffn_down_kernel<float>, dim3(grid), dim3(256), lds, s, a);
  else
    hipLaunchKernelGGL(ffn_down_kernel<bf16_t>, dim3(grid), dim3(256), lds, s, a);
}

void launch_copy(void* dst, const void* src, int64_t n_bytes, hipStream_t s) {
  const int64_t n = n_bytes / 16;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                     static_cast<uint4*>(dst), static_cast<const uint4*>(src), n);
}

void launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t s) {
  if (n <= 0) return;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n, v);
}

}  // namespace smoe
