// Expert FFN on the host cores, for the CPU-assisted task load scheduling of
// Section V-A (CPU operation 3 of Section V-B, "CPU expert computation"): a
// missing expert that Algorithm 2 assigns to the CPU is computed from its host
// copy instead of being loaded.  Plain C++ threads, no HIP dependency.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace smoe {

class CpuExperts {
 public:
  // n_threads workers in total, the calling thread included (>= 1).
  explicit CpuExperts(int n_threads);
  ~CpuExperts();
  CpuExperts(const CpuExperts&) = delete;
  CpuExperts& operator=(const CpuExperts&) = delete;

  int threads() const { return n_threads_; }

  // yacc[t][0..H) += w[t] * W2 ( silu(W1 x[t]) * (W3 x[t]) ) for t < ntok <= 8.
  //   expert: {W1[F][H], W3[F][H], W2[H][F]} row-major, fp32 (dtype 0) or bf16 (dtype 1)
  //   x[t]:   H fp32 values; yacc[t]: H fp32 accumulators
  // fp32 arithmetic throughout.  Blocks until done; not re-entrant.
  void run(const void* expert, int dtype, int H, int F, int ntok, const float* const* x,
           const float* w, float* const* yacc);

  // Reads one byte of every 4 KiB page of [base, base + bytes) with all workers.
  // Page-locked memory that so far only a device has written is mapped into the
  // CPU's page tables page by page on first touch; doing that once up front keeps
  // those faults (which cost several times the FFN itself) out of the decode path.
  void touch(const void* base, size_t bytes);

 private:
  struct Impl;
  Impl* impl_;
  int n_threads_;
};

}  // namespace smoe
