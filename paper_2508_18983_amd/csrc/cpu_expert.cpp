// Host-core expert FFN (see cpu_expert.hpp).  The work of one expert is cut
// into contiguous row ranges, one per worker: first the rows of W1 / W3 (gate
// and up projection + SwiGLU), then, behind a barrier, the rows of W2 (down
// projection).  Every worker streams its rows once, front to back, which is
// what the hardware prefetchers of the host cores like; the loops are plain
// C++ over 16 independent partial sums so that the compiler vectorises them,
// and each is built for AVX-512, AVX2+FMA and baseline x86-64, the right one
// being chosen when the library is loaded.
#include "cpu_expert.hpp"

#include <math.h>
#include <string.h>

#include <atomic>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

// (SMOE_NO_CLONES: a single baseline version.  ThreadSanitizer builds need it: the clones are
// dispatched through IFUNC resolvers, which run before that sanitizer's runtime is up.)
#if defined(__x86_64__) && defined(__GNUC__) && !defined(__clang__) && !defined(SMOE_NO_CLONES)
#define SMOE_CLONES __attribute__((target_clones("avx512f", "avx2,fma", "default")))
#else
#define SMOE_CLONES
#endif

namespace smoe {
namespace {

constexpr int kMaxTok = 8;

inline __attribute__((always_inline)) float widen1(float v) { return v; }
inline __attribute__((always_inline)) float widen1(uint16_t v) {      // bf16 = upper half of an fp32
  const uint32_t u = (uint32_t)v << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

// sum_i w[i] * x[i], n a multiple of 8
template <typename W>
inline __attribute__((always_inline)) float dot(const W* __restrict w, const float* __restrict x, int n) {
  float a[16];
  for (int j = 0; j < 16; ++j) a[j] = 0.f;
  int i = 0;
  for (; i + 16 <= n; i += 16)
    for (int j = 0; j < 16; ++j) a[j] += widen1(w[i + j]) * x[i + j];
  if (i < n)
    for (int j = 0; j < 8; ++j) a[j] += widen1(w[i + j]) * x[i + j];
  for (int s = 8; s >= 1; s >>= 1)
    for (int j = 0; j < s; ++j) a[j] += a[j + s];
  return a[0];
}

struct Job {
  const unsigned char* touch = nullptr;   // non-null: touch job over `touch_bytes` instead of an FFN
  size_t touch_bytes = 0;
  const void* expert;
  int dtype, H, F, ntok;
  const float* x[kMaxTok];
  float w[kMaxTok];
  float* yacc[kMaxTok];
  float* act;               // [ntok][F]
};

// rows [f0, f1) of W1 and W3: act[t][f] = w[t] * silu(W1[f] . x[t]) * (W3[f] . x[t])
template <typename W>
inline __attribute__((always_inline)) void up_rows(const Job& j, int f0, int f1) {
  const W* W1 = static_cast<const W*>(j.expert);
  const W* W3 = W1 + (size_t)j.F * j.H;
  for (int f = f0; f < f1; ++f) {
    const W* r1 = W1 + (size_t)f * j.H;
    const W* r3 = W3 + (size_t)f * j.H;
    for (int t = 0; t < j.ntok; ++t) {
      const float g = dot(r1, j.x[t], j.H);
      const float u = dot(r3, j.x[t], j.H);
      j.act[(size_t)t * j.F + f] = j.w[t] * (g / (1.0f + expf(-g))) * u;
    }
  }
}

// rows [h0, h1) of W2: yacc[t][h] += W2[h] . act[t]
template <typename W>
inline __attribute__((always_inline)) void down_rows(const Job& j, int h0, int h1) {
  const W* W2 = static_cast<const W*>(j.expert) + 2 * (size_t)j.F * j.H;
  for (int h = h0; h < h1; ++h) {
    const W* r = W2 + (size_t)h * j.F;
    for (int t = 0; t < j.ntok; ++t) j.yacc[t][h] += dot(r, j.act + (size_t)t * j.F, j.F);
  }
}

SMOE_CLONES void up_rows_bf16(const Job& j, int f0, int f1) { up_rows<uint16_t>(j, f0, f1); }
SMOE_CLONES void up_rows_f32(const Job& j, int f0, int f1) { up_rows<float>(j, f0, f1); }
SMOE_CLONES void down_rows_bf16(const Job& j, int h0, int h1) { down_rows<uint16_t>(j, h0, h1); }
SMOE_CLONES void down_rows_f32(const Job& j, int h0, int h1) { down_rows<float>(j, h0, h1); }

}  // namespace

struct CpuExperts::Impl {
  int n = 1;
  std::vector<std::thread> th;
  std::mutex mu;
  std::condition_variable cv;
  uint64_t gen = 0;
  bool stop = false;
  Job job{};
  std::vector<float> act;
  std::atomic<int> up_done{0}, all_done{0};
  std::atomic<unsigned> touch_sink{0};

  static void wait_for(const std::atomic<int>& c, int want) {
    int spins = 0;
    while (c.load(std::memory_order_acquire) < want)
      if (++spins > 2000) std::this_thread::yield();
  }

  void work(int id) {
    const Job& j = job;
    if (j.touch != nullptr) {
      // one read per 4 KiB page of this worker's share
      const size_t pages = (j.touch_bytes + 4095) / 4096;
      const size_t p0 = pages * id / n, p1 = pages * (id + 1) / n;
      unsigned acc = 0;
      for (size_t p = p0; p < p1; ++p) acc += *static_cast<const volatile unsigned char*>(j.touch + p * 4096);
      touch_sink.fetch_add(acc, std::memory_order_relaxed);
      all_done.fetch_add(1, std::memory_order_acq_rel);
      return;
    }
    const int f0 = (int)((int64_t)j.F * id / n), f1 = (int)((int64_t)j.F * (id + 1) / n);
    if (j.dtype == 0) up_rows_f32(j, f0, f1); else up_rows_bf16(j, f0, f1);
    up_done.fetch_add(1, std::memory_order_acq_rel);
    wait_for(up_done, n);                          // every activation is written
    const int h0 = (int)((int64_t)j.H * id / n), h1 = (int)((int64_t)j.H * (id + 1) / n);
    if (j.dtype == 0) down_rows_f32(j, h0, h1); else down_rows_bf16(j, h0, h1);
    all_done.fetch_add(1, std::memory_order_acq_rel);
  }

  void worker(int id) {
    uint64_t seen = 0;
    for (;;) {
      {
        std::unique_lock<std::mutex> lk(mu);
        cv.wait(lk, [&] { return stop || gen != seen; });
        if (stop) return;
        seen = gen;
      }
      work(id);
    }
  }
};

CpuExperts::CpuExperts(int n_threads) : impl_(new Impl()), n_threads_(n_threads < 1 ? 1 : n_threads) {
  impl_->n = n_threads_;
  for (int i = 1; i < n_threads_; ++i) impl_->th.emplace_back([this, i] { impl_->worker(i); });
}

CpuExperts::~CpuExperts() {
  {
    std::lock_guard<std::mutex> lk(impl_->mu);
    impl_->stop = true;
  }
  impl_->cv.notify_all();
  for (auto& t : impl_->th) t.join();
  delete impl_;
}

void CpuExperts::touch(const void* base, size_t bytes) {
  if (!base || bytes == 0) return;
  Impl& m = *impl_;
  {
    std::lock_guard<std::mutex> lk(m.mu);
    m.job = Job{};
    m.job.touch = static_cast<const unsigned char*>(base);
    m.job.touch_bytes = bytes;
    m.up_done.store(0, std::memory_order_relaxed);
    m.all_done.store(0, std::memory_order_relaxed);
    ++m.gen;
  }
  m.cv.notify_all();
  m.work(0);
  Impl::wait_for(m.all_done, m.n);
}

void CpuExperts::run(const void* expert, int dtype, int H, int F, int ntok, const float* const* x,
                     const float* w, float* const* yacc) {
  if (ntok < 1) return;
  if (ntok > kMaxTok) ntok = kMaxTok;
  Impl& m = *impl_;
  if (m.act.size() < (size_t)ntok * F) m.act.resize((size_t)ntok * F);
  {
    std::lock_guard<std::mutex> lk(m.mu);
    m.job.touch = nullptr;
    m.job.expert = expert;
    m.job.dtype = dtype; m.job.H = H; m.job.F = F; m.job.ntok = ntok;
    for (int t = 0; t < ntok; ++t) { m.job.x[t] = x[t]; m.job.w[t] = w[t]; m.job.yacc[t] = yacc[t]; }
    m.job.act = m.act.data();
    m.up_done.store(0, std::memory_order_relaxed);
    m.all_done.store(0, std::memory_order_relaxed);
    ++m.gen;
  }
  m.cv.notify_all();
  m.work(0);
  Impl::wait_for(m.all_done, m.n);
}

}  // namespace smoe
