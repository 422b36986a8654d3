// Host side of libsmoe: the C ABI, the expert-cache bookkeeping (score history,
// Eq. 3 eviction, protection shield; Section IV-B "Cache eviction") and the
// two-stream schedule of one layer call (Section V-B: resident experts are
// computed while the misses are loaded; loaded experts are computed after
// their copy completes).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "smoe.h"
#include "smoe_dev.hpp"
#include "cache_state.hpp"
#include "cpu_expert.hpp"
#include "alpha_select.hpp"

#include <chrono>
#include <thread>

using namespace smoe;

// Scratch of moe_decode_layer_static: one array per GPU, held until the process
// ends.  In host code the name below is only a stand-in for the symbol: the
// device address is looked up once per device at init (scratch_of_device) and
// only that pointer is ever handed to kernels or runtime calls.
static __device__ __align__(256) unsigned char scratch[SMOE_STATIC_SCRATCH_BYTES];

namespace {

thread_local int g_last_hip = 0;

#define HIP_TRY(expr)                         \
  do {                                        \
    hipError_t e_ = (expr);                   \
    if (e_ != hipSuccess) {                   \
      g_last_hip = (int)e_;                   \
      return SMOE_EHIP;                       \
    }                                         \
  } while (0)

constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

struct EventPair { hipEvent_t a, b; };
struct ProfKind {
  std::vector<EventPair> ev;
  size_t used = 0;
  int64_t bytes = 0;
};

// Device address of this GPU's copy of `scratch` (each GPU holds its own);
// `dev` must be the current device.
int scratch_of_device(int dev, unsigned char** out) {
  if (dev < 0 || dev >= kMaxDevices) return SMOE_EINVAL;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return SMOE_OK;
}

// Device memory the kernels of one decode call work in besides the caller's
// inputs and outputs.
struct Scratch {
  StepRec* rec = nullptr;                // decision record
  float* act = nullptr;                  // SwiGLU activations between the up and the down kernel
  float* ysum = nullptr;                 // [B][H] fp32 sums carried from the resident to the loaded pass
  float* gate_part = nullptr;            // [B][E][kMaxGateSeg] partial dot products of the gate GEMV
  void* x_pred = nullptr;                // [B][H] dtype: predicted input of the next layer (auto_prefetch)
};
constexpr int64_t kGatePartBytes = (int64_t)SMOE_MAX_BATCH * SMOE_MAX_EXPERTS * kMaxGateSeg * sizeof(float);
// (the 64-bit {epoch, logit} words of the in-kernel gate GEMV follow the partial sums)
constexpr int64_t kGateWordBytes = (int64_t)SMOE_MAX_EXPERTS * sizeof(unsigned long long);

}  // namespace

struct moe_handle {
  moe_cfg_t cfg{};
  moe_buffers_t buf{};
  hipStream_t s_compute = nullptr, s_copy = nullptr;
  hipEvent_t ev_copy = nullptr;
  int64_t esize = 0, expert_bytes = 0, shared_bytes = 0;
  int Fmax = 0;
  std::vector<CacheLayer> layers;
  CacheParams cp{};
  std::vector<int32_t> init_resident;    // [L][cap]
  std::vector<const char*> experts_host; // [L] pinned blocks of E experts
  // device scratch
  float* sim_dev = nullptr;
  Scratch own;                           // allocated at init, used by moe_decode_layer
  Scratch fixed;                         // carved out of this GPU's static array, used by
                                         // moe_decode_layer_static (null: need > the array)
  int64_t fixed_need = 0;                // bytes of the static array this configuration needs
  int device = 0;
  StepRec* rec_host = nullptr;           // pinned
  StepRec* rec_host_dev = nullptr;       // its device-visible address
  // top-score prefetch: the prediction has a decision record of its own
  StepRec* pred_dev = nullptr;
  StepRec* pred_host = nullptr;          // pinned
  StepRec* pred_host_dev = nullptr;
  int32_t pred_seq = 0;                  // number of the last prediction launched
  int pending_layer = -1, pending_batch = 0;   // prediction launched, loads not queued yet
  // Load queue of the prefetcher (Section IV-C): prefetch copies are not handed to the copy
  // stream whole.  They wait here and are fed to it in chunks, a bounded number outstanding,
  // so that an on-demand load of the running layer never queues behind more than that, and a
  // prefetch whose layer has run without it is withdrawn before the rest of it is copied.
  struct PfEntry {
    int layer = -1, expert = -1, slot = -1;   // physical slot of the layer
    int64_t next_off = 0;                      // bytes handed to the copy stream so far
    hipEvent_t done = nullptr;                 // recorded behind the last chunk
    bool all_submitted = false;
  };
  std::vector<PfEntry> pf_entries;       // live entries (waiting for their layer's step), oldest first
  std::vector<hipEvent_t> pf_event_pool; // spare events for entries
  static constexpr int kMaxChunksOut = 8;
  hipEvent_t chunk_ev[kMaxChunksOut] = {};
  bool chunk_busy[kMaxChunksOut] = {false};
  int chunks_out_limit = 4;              // SMOE_PF_OUTSTANDING
  int64_t chunk_bytes = 64ll << 20;      // SMOE_PF_CHUNK_MB (smaller chunks cost more in submission
                                         // overhead than they gain: measured 16 MB -> 64 MB +3-5 %)
  int64_t pf_bytes_submitted = 0, pf_bytes_withdrawn = 0;
  int mfma_rt = 16;                      // output rows per block of the MFMA down kernel
  int mfma_contig = 1;                   // its waves take contiguous item ranges (SMOE_MFMA_CONTIG=0: every eighth item)
  int fused_gate = 1;                    // batch 1: gate GEMV in the first blocks of the up kernel
  int gate_spin = 8192;                  // reads of the logit words before a block computes them itself
  int uid = 0;                           // 1..255, distinguishes the epochs of handles that share scratch
  int64_t pf_yielded = 0;                // predictions skipped because the link was busy
  std::vector<int32_t> slot_guard;       // per global slot: number of the decode call whose kernels may
                                         // still read a slot that has been given up since (-1: none)
  moe_prefetch_info_t pf_last{};
  // CPU-assisted scheduling (Section V-A): host-core FFN, the hidden states and the
  // partial outputs it exchanges with the GPU, and the two costs of Algorithm 2
  CpuExperts* cpu = nullptr;
  void* x_host = nullptr;                // pinned [B][H] dtype, written by the router kernel
  void* x_host_dev = nullptr;
  float* ycpu_host = nullptr;            // pinned [B][H] fp32, read by the add kernel
  float* ycpu_host_dev = nullptr;
  std::vector<float> x_f32;              // [B][H] widened hidden states
  double c_load_us = 0.0, c_cpu_us = 0.0;
  static constexpr int kCostWindow = 8;  // both costs are means over this many recent samples
  double cpu_busy_us = 0.0;              // wall time spent in the host FFN so far
  int64_t cpu_experts = 0;
  double cpu_hist[kCostWindow] = {0};
  int cpu_hist_n = 0;
  EventPair copy_ev[kCostWindow] = {};
  bool copy_ev_pending[kCostWindow] = {false};
  double copy_hist[kCostWindow] = {0};
  int copy_ev_next = 0, copy_hist_n = 0;
  // launch geometry
  int TF = 0, tilesR = 0, tilesS = 0, R = 0, htiles = 0, stage_all = 0, chunk = 0, down_lds = 0;
  int up_upl = 0, down_upl = 0, down_nw = 4, down_r = 1, RB = 0, nsegR = 1, nsegS = 1;
  int grouped_ok = 0, nsegGR = 0, nsegGS = 0, RBG = 0;   // batch > 1: grouped kernels
  int mfma_ok = 1;                                       // SMOE_MFMA=0 keeps the vector-ALU down kernel
  int64_t act_floats = 0;
  // profiling
  int32_t seq = 0;                       // number of the last decode call
  int fused_select = 1;                  // batch 1: the up kernel runs the selection (SMOE_FUSED_SELECT=0: own launch)
  long spin_limit = 4000000;             // polls of the mirror before falling back to the event
  uint32_t prof_mask = 0;                // bit i: record kind i
  ProfKind prof[SMOE_PROF_KINDS];
};

namespace {

int env_int(const char* name, int dflt) {
  const char* v = std::getenv(name);
  if (!v || !*v) return dflt;
  return std::atoi(v);
}

void plan_geometry(moe_handle* h) {
  const moe_cfg_t& c = h->cfg;
  const long total_f = (long)c.top_k * c.ffn + (long)c.n_shared * c.shared_ffn;
  // up: TF rows of W1 and W3 per block, ~2560 blocks per token (ten per compute unit: measured
  // flat from 1000 to 2400 blocks on the 14336-wide experts, 3-4 % better than 1000 on narrow ones)
  int tf = (int)((total_f + 2559) / 2560 + 3) / 4 * 4;
  tf = std::max(8, tf);
  {
    // A small layer whose blocks do not all fit on the chip at once, but almost do, runs as one
    // full round of blocks plus a short second one that pays the whole start-up chain (kernel
    // arguments, gate sums, selection, first weights) again: take rows per block so that one
    // round holds them all.  Blocks the chip holds at once: 4 waves each, 8 / 8 / 4 / 3 waves per
    // SIMD for 1 / 2 / 4 / 8 units of x per lane (register use of the kernel instances).
    const int nx = c.dtype == SMOE_DTYPE_FP32 ? 4 : 8;
    const int xu = (c.hidden / nx + kWave - 1) / kWave;
    const long at_once = 256L * (xu <= 2 ? 8 : (xu <= 4 ? 4 : 3));
    auto blocks_of = [&](int t) {
      return (long)c.top_k * ((c.ffn + t - 1) / t) + (c.n_shared ? (long)c.n_shared * ((c.shared_ffn + t - 1) / t) : 0);
    };
    if (blocks_of(tf) > at_once && blocks_of(tf) <= 2 * at_once)
      while (blocks_of(tf) > at_once && tf < 64) tf += 4;
  }
  tf = env_int("SMOE_TF", tf);
  if (tf < 4) tf = 4;
  tf = tf / 4 * 4;
  h->TF = tf;
  h->tilesR = (c.ffn + tf - 1) / tf;
  h->tilesS = c.n_shared ? (c.shared_ffn + tf - 1) / tf : 0;
  // down: R rows per wave, 4 waves per block
  int r = (c.hidden / 4 >= 2048) ? 2 : 1;
  r = env_int("SMOE_R", r);
  h->R = r >= 4 ? 4 : (r >= 2 ? 2 : 1);
  h->htiles = (c.hidden + 4 * h->R - 1) / (4 * h->R);
  h->stage_all = total_f <= kStageElems;
  int chunk = env_int("SMOE_CHUNK", kChunkElems);
  chunk = std::max(512, std::min(kStageElems, chunk / 512 * 512));
  h->chunk = chunk;
  h->down_lds = h->stage_all ? (int)total_f : chunk;

  const int n = c.dtype == SMOE_DTYPE_FP32 ? 4 : 8;
  // batch > 1: grouped kernels stream an expert once for up to 4 of its tokens
  h->grouped_ok = 0;
  if (c.max_batch > 1 && env_int("SMOE_GROUPED", 1) != 0) {
    const int esz = c.dtype == SMOE_DTYPE_FP32 ? 4 : 2;
    const int maxg = std::min(c.n_experts, c.max_batch * c.top_k);
    h->nsegGR = (c.ffn / n + 127) / 128;
    h->nsegGS = c.n_shared ? (c.shared_ffn / n + 127) / 128 : 0;
    const long items = (long)maxg * h->nsegGR + (long)c.n_shared * h->nsegGS;
    int rbg = 4;
    while (rbg > 2 && items * SMOE_MAX_BATCH * rbg * 4 > 60 * 1024) rbg /= 2;
    const bool lds_ok = items * SMOE_MAX_BATCH * rbg * 4 <= 60 * 1024 && 4L * c.hidden * esz <= 60 * 1024;
    const int xu0 = (c.hidden / n + kWave - 1) / kWave;
    if (lds_ok && xu0 <= 8) { h->grouped_ok = 1; h->RBG = rbg; }
  }

  // MFMA down kernel: output rows per block.  Its rate scales with the number of compute
  // units that have a block (measured: 224 blocks of 16 rows at H = 3584 ran at 7/8 of the rate
  // of 256 blocks at H = 4096), so take the largest row count that still gives every unit one.
  {
    const int per_cu = c.hidden / 256;
    int rt = per_cu >= 16 ? 16 : (per_cu >= 14 ? 14 : (per_cu >= 12 ? 12 : 8));
    rt = env_int("SMOE_MFMA_RT", rt);
    h->mfma_rt = (rt == 8 || rt == 12 || rt == 14) ? rt : 16;
  }

  // register-resident fast paths (SMOE_REGPATH=0 forces the LDS kernels)
  h->up_upl = 0;
  h->down_upl = 0;
  if (env_int("SMOE_REGPATH", 1) == 0) return;
  const int xu = (c.hidden / n + kWave - 1) / kWave;           // units of x per lane
  h->up_upl = xu <= 1 ? 1 : (xu <= 2 ? 2 : (xu <= 4 ? 4 : (xu <= 8 ? 8 : 0)));
  // Column segments per row: aim at the same number of units per lane (4..8) for the
  // routed and the shared rows, so one kernel instance keeps enough loads in flight for both.
  auto per_lane_of = [&](int F) { return (F / n + kWave - 1) / kWave; };
  int target = per_lane_of(c.ffn);
  if (c.n_shared) target = std::min(target, per_lane_of(c.shared_ffn));
  target = std::max(4, std::min(8, target));
  target = std::max(1, std::min(8, env_int("SMOE_DSEG", target)));
  auto seg_plan = [&](int F, int& nseg) -> int {               // -> units per lane
    nseg = std::max(1, std::min(16, (per_lane_of(F) + target - 1) / target));
    return ((F / n + nseg - 1) / nseg + kWave - 1) / kWave;
  };
  int need = seg_plan(c.ffn, h->nsegR);
  if (c.n_shared) need = std::max(need, seg_plan(c.shared_ffn, h->nsegS));
  if (need <= 8) {
    const int upl = need <= 2 ? 2 : (need <= 4 ? 4 : (need <= 6 ? 6 : 8));
    const int rows_at_once = upl <= 2 ? 4 : (upl <= 6 ? 2 : 1);   // R of the kernel (two such buffers
                                                                  // in flight; deeper did not help)
    const int items = c.top_k * h->nsegR + c.n_shared * h->nsegS;
    // waves per block: one or two items per wave
    int nw = env_int("SMOE_DNW", items >= 8 ? 8 : 4);
    nw = nw >= 8 ? 8 : 4;
    // rows per block: about one block per compute unit (measured on the three large shapes:
    // halving the rows costs 3-8 % through the repeated activation loads, doubling them leaves
    // half of the chip idle), at least two pipeline steps
    int rb = (c.hidden + 255) / 256;
    rb = std::max(2 * rows_at_once, (rb + rows_at_once - 1) / rows_at_once * rows_at_once);
    rb = env_int("SMOE_RB", rb);
    rb = std::max(2 * rows_at_once, std::min(256, rb) / rows_at_once * rows_at_once);   // the kernel's pipeline
                                                                                        // needs two steps
    h->down_upl = upl;
    h->down_nw = nw;
    h->down_r = rows_at_once;
    h->RB = rb;
    h->htiles = (c.hidden + rb - 1) / rb;
  }
}

// Global slot numbers: layer l owns the physical slots [l * (cap + prefetch_max), ...); the
// staging slots follow the last layer.
inline int64_t layer_slot_base(const moe_handle* h, int layer) {
  return (int64_t)layer * (h->cfg.cache_cap + h->cfg.prefetch_max);
}
inline int64_t staging_slot_base(const moe_handle* h) { return layer_slot_base(h, h->cfg.n_layers); }
inline char* slot_ptr(const moe_handle* h, int64_t gslot) {
  return static_cast<char*>(h->buf.cache_slab_dev) + gslot * h->expert_bytes;
}

int upload_initial(moe_handle* h) {
  const moe_cfg_t& c = h->cfg;
  for (int l = 0; l < c.n_layers; ++l) {
    h->layers[l].reset(h->cp, &h->init_resident[(size_t)l * c.cache_cap]);
    for (int s = 0; s < c.cache_cap; ++s) {
      const int e = h->init_resident[(size_t)l * c.cache_cap + s];
      const char* src = h->experts_host[l] + (int64_t)e * h->expert_bytes;
      char* dst = slot_ptr(h, layer_slot_base(h, l) + s);
      HIP_TRY(hipMemcpyAsync(dst, src, h->expert_bytes, hipMemcpyHostToDevice, h->s_copy));
    }
  }
  HIP_TRY(hipStreamSynchronize(h->s_copy));
  return SMOE_OK;
}

void free_all(moe_handle* h) {
  if (!h) return;
  for (auto& k : h->prof)
    for (auto& p : k.ev) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  if (h->ev_copy) (void)hipEventDestroy(h->ev_copy);
  for (auto& e : h->pf_entries) if (e.done) (void)hipEventDestroy(e.done);
  for (hipEvent_t e : h->pf_event_pool) (void)hipEventDestroy(e);
  for (hipEvent_t e : h->chunk_ev) if (e) (void)hipEventDestroy(e);
  delete h->cpu;
  for (auto& p : h->copy_ev) {
    if (p.a) (void)hipEventDestroy(p.a);
    if (p.b) (void)hipEventDestroy(p.b);
  }
  if (h->x_host) (void)hipHostFree(h->x_host);
  if (h->ycpu_host) (void)hipHostFree(h->ycpu_host);
  if (h->pred_dev) (void)hipFree(h->pred_dev);
  if (h->pred_host) (void)hipHostFree(h->pred_host);
  if (h->sim_dev) (void)hipFree(h->sim_dev);
  if (h->own.rec) (void)hipFree(h->own.rec);
  if (h->rec_host) (void)hipHostFree(h->rec_host);
  if (h->own.act) (void)hipFree(h->own.act);
  if (h->own.ysum) (void)hipFree(h->own.ysum);
  if (h->own.gate_part) (void)hipFree(h->own.gate_part);
  if (h->own.x_pred) (void)hipFree(h->own.x_pred);
  delete h;
}

// Event pair around one launch while profiling; nullptr when not recording.
EventPair* prof_begin(moe_handle* h, int kind, hipStream_t s) {
  if (!((h->prof_mask >> kind) & 1u)) return nullptr;
  ProfKind& k = h->prof[kind];
  if (k.used >= k.ev.size()) return nullptr;
  EventPair* p = &k.ev[k.used++];
  (void)hipEventRecord(p->a, s);
  return p;
}
void prof_end(EventPair* p, hipStream_t s) {
  if (p) (void)hipEventRecord(p->b, s);
}


inline float bf16_bits_to_float(uint16_t v) {
  const uint32_t u = (uint32_t)v << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

// C_load of Algorithm 2 when it is measured: fold in the copies that have completed.
void refresh_load_cost(moe_handle* h) {
  if (h->cfg.load_cost_us > 0.f) return;
  for (int i = 0; i < moe_handle::kCostWindow; ++i) {
    if (!h->copy_ev_pending[i]) continue;
    if (hipEventQuery(h->copy_ev[i].b) != hipSuccess) { (void)hipGetLastError(); continue; }
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, h->copy_ev[i].a, h->copy_ev[i].b) == hipSuccess) {
      h->copy_hist[i] = ms * 1e3;
      if (h->copy_hist_n < moe_handle::kCostWindow) ++h->copy_hist_n;
    } else {
      (void)hipGetLastError();
    }
    h->copy_ev_pending[i] = false;
  }
  if (h->copy_hist_n > 0) {
    double s = 0.0;
    int n = 0;
    for (int i = 0; i < moe_handle::kCostWindow; ++i)
      if (h->copy_hist[i] > 0.0) { s += h->copy_hist[i]; ++n; }
    if (n) h->c_load_us = s / n;
  }
}

void note_cpu_cost(moe_handle* h, double us) {
  h->cpu_busy_us += us;
  ++h->cpu_experts;
  if (h->cfg.cpu_cost_us > 0.f) return;
  h->cpu_hist[h->cpu_hist_n % moe_handle::kCostWindow] = us;
  ++h->cpu_hist_n;
  const int n = std::min(h->cpu_hist_n, moe_handle::kCostWindow);
  double s = 0.0;
  for (int i = 0; i < n; ++i) s += h->cpu_hist[i];
  h->c_cpu_us = s / n;
}

// The experts Algorithm 2 left to the host cores: ycpu[t] = sum over them of
// w * FFN_e(x[t]) in fp32, from the hidden states the router kernel mirrored.
void compute_on_cpu(moe_handle* h, int layer, int B, const StepRec& rec, const int* on_cpu, int n_cpu) {
  const moe_cfg_t& c = h->cfg;
  const int H = c.hidden, k = c.top_k;
  for (int t = 0; t < B; ++t) {
    float* xf = h->x_f32.data() + (size_t)t * H;
    if (c.dtype == SMOE_DTYPE_FP32) {
      std::memcpy(xf, static_cast<const float*>(h->x_host) + (size_t)t * H, sizeof(float) * H);
    } else {
      const uint16_t* xb = static_cast<const uint16_t*>(h->x_host) + (size_t)t * H;
      for (int i = 0; i < H; ++i) xf[i] = bf16_bits_to_float(xb[i]);
    }
  }
  std::memset(h->ycpu_host, 0, sizeof(float) * (size_t)B * H);
  for (int i = 0; i < n_cpu; ++i) {
    const int e = on_cpu[i];
    const float* xs[SMOE_MAX_BATCH];
    float ws[SMOE_MAX_BATCH];
    float* ys[SMOE_MAX_BATCH];
    int ntok = 0;
    for (int t = 0; t < B; ++t)
      for (int j = 0; j < k; ++j)
        if (rec.tok[t].final_[j] == e) {
          xs[ntok] = h->x_f32.data() + (size_t)t * H;
          ws[ntok] = rec.tok[t].w[j];
          ys[ntok] = h->ycpu_host + (size_t)t * H;
          ++ntok;
        }
    const auto t0 = std::chrono::steady_clock::now();
    h->cpu->run(h->experts_host[layer] + (int64_t)e * h->expert_bytes, c.dtype, H, c.ffn, ntok, xs, ws, ys);
    const auto t1 = std::chrono::steady_clock::now();
    note_cpu_cost(h, std::chrono::duration<double, std::micro>(t1 - t0).count());
  }
}

// Arguments of one router launch for `layer` on x (the decision record and the
// call number are filled in by the caller).
void fill_route_args(const moe_handle* h, const Scratch& sc, int layer, int B, const void* x, RouteArgs& ra) {
  const moe_cfg_t& c = h->cfg;
  const int E = c.n_experts;
  const CacheLayer& ls = h->layers[layer];
  ra.gate_w = static_cast<const char*>(h->buf.gate_w_dev) + (int64_t)layer * E * c.hidden * h->esize;
  ra.x = x;
  ra.sim = h->sim_dev + (size_t)layer * E * E;
  ra.gate_part = sc.gate_part;
  ra.gate_word = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(sc.gate_part) + kGatePartBytes);
  ra.epoch = 0;
  ra.gate_blocks = 0;
  ra.gate_spin = h->gate_spin;
  ra.B = B; ra.H = c.hidden; ra.E = E; ra.k = c.top_k;
  ra.renorm = c.renorm_topk; ra.subst_key = c.subst_key; ra.alpha = c.alpha;
  // gate GEMV: one wave per (row, segment); split the rows until there are >= 128 waves of work
  // or a segment is down to one unit per lane; a segment is at most 8 units per lane
  const int gate_units = c.hidden / (c.dtype == SMOE_DTYPE_FP32 ? 4 : 8);
  int nseg = 1;
  while (nseg < kMaxGateSeg && (gate_units / nseg > 8 * kWave || E * nseg < 128) && gate_units / (nseg * 2) >= kWave)
    nseg *= 2;
  while (nseg < kMaxGateSeg && ((gate_units + nseg - 1) / nseg + kWave - 1) / kWave > 8) nseg *= 2;
  const int per_lane = ((gate_units + nseg - 1) / nseg + kWave - 1) / kWave;
  ra.nseg = nseg;
  ra.upi = per_lane <= 1 ? 1 : (per_lane <= 2 ? 2 : (per_lane <= 4 ? 4 : 8));
  // experts prefetched for this layer count as resident for every decision, but the resident
  // pass cannot use them (their copy may still be running): they have no slot here and are
  // computed in the second pass
  ra.resident = ls.resident | ls.landed_mask();
  for (int e = 0; e < SMOE_MAX_EXPERTS; ++e)
    ra.slot_of[e] = ((ls.resident >> e) & 1ull) ? (int8_t)ls.phys_of_expert(e) : (int8_t)-1;
  ra.x_mirror = nullptr;
  ra.x_units = 0;
}

// Wait until the router kernel that was given call number `want` has published
// its record to the pinned mirror: bounded polling, then the stream.
int await_record(moe_handle* h, const StepRec* mirror, int32_t want) {
  const volatile int32_t* seq = &mirror->seq;
  long spins = 0;
  while (*seq != want && spins < h->spin_limit) ++spins;
  if (*seq != want) HIP_TRY(hipStreamSynchronize(h->s_compute));
  __atomic_thread_fence(__ATOMIC_ACQUIRE);
  return *seq == want ? SMOE_OK : SMOE_ESTATE;
}

// ---- load queue of the prefetcher --------------------------------------------
// Chunks of queued prefetches go to the copy stream while fewer than
// chunks_out_limit of them are outstanding there.  Entries of `first_layer` (the
// layer that is about to need them) go first, then the oldest entry.  Called
// only at points where the host has just seen a record of a kernel that was
// launched after every kernel that could still read a slot given up earlier.
int pump_prefetch_queue(moe_handle* h, int first_layer) {
  int out = 0;
  for (int i = 0; i < moe_handle::kMaxChunksOut; ++i) {
    if (!h->chunk_busy[i]) continue;
    if (hipEventQuery(h->chunk_ev[i]) == hipSuccess) h->chunk_busy[i] = false;
    else { (void)hipGetLastError(); ++out; }           // "not ready" is not an error here
  }
  while (out < h->chunks_out_limit) {
    // (an entry whose slot was read by the kernels of the call that is still running waits)
    auto ready = [&](const moe_handle::PfEntry& c) {
      return !c.all_submitted && h->slot_guard[layer_slot_base(h, c.layer) + c.slot] < h->seq;
    };
    moe_handle::PfEntry* e = nullptr;
    for (auto& c : h->pf_entries)
      if (c.layer == first_layer && ready(c)) { e = &c; break; }
    if (!e)
      for (auto& c : h->pf_entries)
        if (ready(c)) { e = &c; break; }
    if (!e) break;
    int slot_i = 0;
    while (h->chunk_busy[slot_i]) ++slot_i;             // out < limit <= kMaxChunksOut: one is free
    const int64_t n = std::min(h->chunk_bytes, h->expert_bytes - e->next_off);
    const char* src = h->experts_host[e->layer] + (int64_t)e->expert * h->expert_bytes + e->next_off;
    char* dst = slot_ptr(h, layer_slot_base(h, e->layer) + e->slot) + e->next_off;
    EventPair* pc = prof_begin(h, SMOE_PROF_COPY, h->s_copy);
    HIP_TRY(hipMemcpyAsync(dst, src, (size_t)n, hipMemcpyHostToDevice, h->s_copy));
    prof_end(pc, h->s_copy);
    if (pc) h->prof[SMOE_PROF_COPY].bytes += n;
    e->next_off += n;
    h->pf_bytes_submitted += n;
    if (e->next_off >= h->expert_bytes) {
      e->all_submitted = true;
      HIP_TRY(hipEventRecord(e->done, h->s_copy));
    }
    HIP_TRY(hipEventRecord(h->chunk_ev[slot_i], h->s_copy));
    h->chunk_busy[slot_i] = true;
    ++out;
  }
  return SMOE_OK;
}

moe_handle::PfEntry* find_prefetch_entry(moe_handle* h, int layer, int expert) {
  for (auto& e : h->pf_entries)
    if (e.layer == layer && e.expert == expert) return &e;
  return nullptr;
}

// Hand the rest of an entry to the copy stream at once (its layer computes the expert now).
int finish_prefetch_entry(moe_handle* h, moe_handle::PfEntry* e) {
  if (e->all_submitted) return SMOE_OK;
  const int64_t n = h->expert_bytes - e->next_off;
  const char* src = h->experts_host[e->layer] + (int64_t)e->expert * h->expert_bytes + e->next_off;
  char* dst = slot_ptr(h, layer_slot_base(h, e->layer) + e->slot) + e->next_off;
  EventPair* pc = prof_begin(h, SMOE_PROF_COPY, h->s_copy);
  HIP_TRY(hipMemcpyAsync(dst, src, (size_t)n, hipMemcpyHostToDevice, h->s_copy));
  prof_end(pc, h->s_copy);
  if (pc) h->prof[SMOE_PROF_COPY].bytes += n;
  e->next_off = h->expert_bytes;
  e->all_submitted = true;
  h->pf_bytes_submitted += n;
  HIP_TRY(hipEventRecord(e->done, h->s_copy));
  return SMOE_OK;
}

// Remove an entry from the queue; what has not been handed to the copy stream is never copied.
void retire_prefetch_entry(moe_handle* h, int layer, int expert, bool withdrawn) {
  for (size_t i = 0; i < h->pf_entries.size(); ++i) {
    moe_handle::PfEntry& e = h->pf_entries[i];
    if (e.layer != layer || e.expert != expert) continue;
    if (withdrawn) h->pf_bytes_withdrawn += h->expert_bytes - e.next_off;
    h->pf_event_pool.push_back(e.done);
    h->pf_entries.erase(h->pf_entries.begin() + (long)i);
    return;
  }
}

// Prefetched experts of `layer` whose copy has not finished (queued, or on the copy stream).
uint64_t prefetches_in_flight(moe_handle* h, int layer) {
  uint64_t m = 0;
  for (auto& e : h->pf_entries) {
    if (e.layer != layer) continue;
    bool done = false;
    if (e.all_submitted) {
      if (hipEventQuery(e.done) == hipSuccess) done = true;
      else (void)hipGetLastError();
    }
    if (!done) m |= 1ull << e.expert;
  }
  return m;
}

// Are copies of earlier calls still on the host link (on-demand loads, chunks of queued
// prefetches, or prefetches not yet handed over)?  With cfg.prefetch_yield a prediction that
// would be launched now is skipped then.
bool link_busy(moe_handle* h) {
  for (auto& e : h->pf_entries) {
    if (!e.all_submitted) return true;
    if (hipEventQuery(e.done) != hipSuccess) { (void)hipGetLastError(); return true; }
  }
  for (int i = 0; i < moe_handle::kMaxChunksOut; ++i) {
    if (!h->chunk_busy[i]) continue;
    if (hipEventQuery(h->chunk_ev[i]) != hipSuccess) { (void)hipGetLastError(); return true; }
  }
  if (hipEventQuery(h->ev_copy) != hipSuccess) { (void)hipGetLastError(); return true; }   // (never recorded: ready)
  return false;
}

// A prediction for `layer` that is not made because the link is busy.
void note_yielded_prefetch(moe_handle* h, int layer) {
  h->pf_last = moe_prefetch_info_t{};
  h->pf_last.layer = layer;
  h->pf_last.yielded = 1;
  for (int i = 0; i < SMOE_MAX_BATCH * SMOE_MAX_TOPK; ++i) h->pf_last.wanted[i] = -1;
  ++h->pf_yielded;
}

// Take the decision of a pending prefetch (Section IV-C): read the predicted
// scores, pick what to load, put it on the load queue.  The prediction kernels
// precede every kernel launched since the prefetch call on the compute stream,
// so once their record is visible the only kernels that can still be running
// belong to the current call.
int settle_prefetch(moe_handle* h) {
  if (h->pending_layer < 0) return SMOE_OK;
  const int layer = h->pending_layer, B = h->pending_batch;
  h->pending_layer = -1;
  {
    const int rc = await_record(h, h->pred_host, h->pred_seq);
    if (rc != SMOE_OK) return rc;
  }
  StepDecision dec{};
  dec.B = B;
  for (int t = 0; t < B; ++t) {
    dec.topk[t] = h->pred_host->tok[t].topk;
    dec.scores[t] = h->pred_host->tok[t].scores;
  }
  PrefetchPlan pp;
  h->layers[layer].plan_prefetch(h->cp, dec, pp);
  h->pf_last.layer = layer;
  h->pf_last.yielded = 0;
  h->pf_last.n_wanted = pp.n_wanted;
  h->pf_last.n_loaded = pp.n;
  for (int i = 0; i < SMOE_MAX_BATCH * SMOE_MAX_TOPK; ++i) h->pf_last.wanted[i] = i < pp.n_wanted ? pp.wanted[i] : -1;
  for (int i = 0; i < pp.n; ++i) {
    moe_handle::PfEntry e;
    e.layer = layer;
    e.expert = pp.experts[i];
    e.slot = pp.slot[i];
    if (h->pf_event_pool.empty()) {
      HIP_TRY(hipEventCreateWithFlags(&e.done, hipEventDisableTiming));
    } else {
      e.done = h->pf_event_pool.back();
      h->pf_event_pool.pop_back();
    }
    h->pf_entries.push_back(e);
  }
  return pump_prefetch_queue(h, -1);
}

// Arguments of the FFN launches of one call (resident pass; the second pass
// changes `pass` and `slot_override` only).
void fill_ffn_args(const moe_handle* h, const Scratch& sc, int layer, int B, const void* x_dev, void* y_dev,
                   FfnArgs& fa) {
  const moe_cfg_t& c = h->cfg;
  fa.rec = sc.rec;
  fa.x = x_dev; fa.y = y_dev;
  fa.slab = static_cast<const char*>(h->buf.cache_slab_dev);
  fa.shared = c.n_shared ? static_cast<const char*>(h->buf.shared_dev) +
                               (int64_t)layer * c.n_shared * h->shared_bytes
                         : nullptr;
  fa.act = sc.act; fa.ysum = sc.ysum;
  fa.expert_bytes = h->expert_bytes; fa.shared_bytes = h->shared_bytes;
  fa.B = B; fa.H = c.hidden; fa.F = c.ffn; fa.Fs = c.n_shared ? c.shared_ffn : 0;
  fa.k = c.top_k; fa.ns = c.n_shared; fa.Fmax = h->Fmax;
  fa.slot_base = (int32_t)layer_slot_base(h, layer);
  fa.pass = 0;
  fa.TF = h->TF; fa.tilesR = h->tilesR; fa.tilesS = h->tilesS;
  fa.R = h->R; fa.htiles = h->htiles;
  fa.stage_all = h->stage_all; fa.chunk = h->chunk; fa.down_lds_floats = h->down_lds;
  fa.up_upl = h->up_upl; fa.down_upl = h->down_upl; fa.RB = h->RB;
  fa.nsegR = h->nsegR; fa.nsegS = h->nsegS; fa.down_nw = h->down_nw; fa.down_r = h->down_r;
  for (int i = 0; i < kMaxTasks; ++i) fa.slot_override[i] = -1;
  fa.grouped = (B > 1 && h->grouped_ok) ? 1 : 0;
  fa.maxg = std::min(c.n_experts, B * c.top_k);
  fa.mfma_down = (fa.grouped && c.dtype == SMOE_DTYPE_BF16 && h->mfma_ok) ? 1 : 0;
  fa.mfma_up = (fa.mfma_down && h->mfma_ok >= 2) ? 1 : 0;
  fa.mfma_rt = h->mfma_rt;
  fa.mfma_contig = h->mfma_contig;
  fa.nsegGR = h->nsegGR; fa.nsegGS = h->nsegGS; fa.RBG = h->RBG;
  fa.act_shared_off = (int64_t)fa.maxg * SMOE_MAX_BATCH * c.ffn;
  if (fa.grouped && fa.up_upl == 0) {                 // grouped up kernel needs units per lane
    const int n = c.dtype == SMOE_DTYPE_FP32 ? 4 : 8;
    const int xu = (c.hidden / n + kWave - 1) / kWave;
    fa.up_upl = xu <= 1 ? 1 : (xu <= 2 ? 2 : (xu <= 4 ? 4 : 8));
  }
}

// One up + down launch pair; *timed_up / *timed_down tell whether the profiler
// recorded them.
int launch_ffn_pair(moe_handle* h, const FfnArgs& fa, const RouteArgs& ra, int kind_up, int kind_down,
                    bool* timed_up, bool* timed_down) {
  EventPair* pu = prof_begin(h, kind_up, h->s_compute);
  launch_ffn_up(fa, ra, h->cfg.dtype, h->s_compute);
  prof_end(pu, h->s_compute);
  EventPair* pd = prof_begin(h, kind_down, h->s_compute);
  launch_ffn_down(fa, h->cfg.dtype, h->s_compute);
  prof_end(pd, h->s_compute);
  *timed_up = pu != nullptr;
  *timed_down = pd != nullptr;
  HIP_TRY(hipGetLastError());
  return SMOE_OK;
}

// Loads of the step's missing experts on the copy stream (Section V-B, "Loading
// Experts from Layer i"); gslot[i] = global slot of load i.  Records ev_copy behind
// them.  With measured Algorithm-2 costs each copy also goes into the ring of
// timed copies.
int enqueue_loads(moe_handle* h, int layer, const StepPlan& plan, int* gslot) {
  const moe_cfg_t& c = h->cfg;
  const bool time_copies = c.cpu_assist && c.load_cost_us <= 0.f;
  for (int i = 0; i < plan.n_fetch; ++i) {
    const int m = plan.fetched[i];
    gslot[i] = plan.slot[i] >= 0 ? (int)(layer_slot_base(h, layer) + plan.slot[i])
                                 : (int)(staging_slot_base(h) + (-plan.slot[i] - 1));
    const char* src = h->experts_host[layer] + (int64_t)m * h->expert_bytes;
    char* dst = static_cast<char*>(h->buf.cache_slab_dev) + (int64_t)gslot[i] * h->expert_bytes;
    EventPair* pc = prof_begin(h, SMOE_PROF_COPY, h->s_copy);
    EventPair* cost = nullptr;
    if (time_copies && !h->copy_ev_pending[h->copy_ev_next]) {
      cost = &h->copy_ev[h->copy_ev_next];
      HIP_TRY(hipEventRecord(cost->a, h->s_copy));
    }
    HIP_TRY(hipMemcpyAsync(dst, src, h->expert_bytes, hipMemcpyHostToDevice, h->s_copy));
    if (cost) {
      HIP_TRY(hipEventRecord(cost->b, h->s_copy));
      h->copy_ev_pending[h->copy_ev_next] = true;
      h->copy_ev_next = (h->copy_ev_next + 1) % moe_handle::kCostWindow;
    }
    prof_end(pc, h->s_copy);
    if (pc) h->prof[SMOE_PROF_COPY].bytes += h->expert_bytes;   // bytes of timed copies only
  }
  if (plan.n_fetch > 0) HIP_TRY(hipEventRecord(h->ev_copy, h->s_copy));
  return SMOE_OK;
}

// Second pass: which task computes from which global slot -- the experts this
// call has loaded (gslot[i] for plan.fetched[i]) and the prefetched experts it
// computes (from the physical slot they were loaded into).
void set_second_pass_slots(const moe_handle* h, int layer, int B, const StepRec& rec, const StepPlan& plan,
                           const int* gslot, FfnArgs& fa) {
  const moe_cfg_t& c = h->cfg;
  const int k = c.top_k, nj = k + c.n_shared;
  const int base = (int)layer_slot_base(h, layer);
  fa.pass = 1;
  auto slot_for = [&](int e) -> int {
    for (int i = 0; i < plan.n_fetch; ++i)
      if (plan.fetched[i] == e) return gslot[i];
    for (int i = 0; i < plan.n_adopted; ++i)
      if (plan.adopted[i] == e) return base + plan.adopt_slot[i];
    return -1;
  };
  if (fa.grouped) {
    // group index of an expert = its rank among the distinct experts of the step (ascending id)
    for (int e = 0; e < c.n_experts; ++e) {
      if (!((plan.shield >> e) & 1ull) || ((plan.before >> e) & 1ull)) continue;
      const int gi = __builtin_popcountll(plan.shield & ((1ull << e) - 1ull));
      fa.slot_override[gi] = slot_for(e);
    }
    return;
  }
  for (int t = 0; t < B; ++t)
    for (int j = 0; j < k; ++j) {
      const int e = rec.tok[t].final_[j];
      if ((plan.before >> e) & 1ull) continue;
      fa.slot_override[t * nj + j] = slot_for(e);
    }
}

// Algorithmic bytes the timed launches of this call were asked to stream
// (launches past the end of the event pool are not timed and add no bytes).
void account_profile_bytes(moe_handle* h, int B, const StepRec& rec, const StepPlan& plan, bool grouped,
                           const bool (&timed)[5]) {
  const moe_cfg_t& c = h->cfg;
  const int k = c.top_k;
  // slots computed by the resident pass (expert in G), by the second pass, by the host cores
  int64_t res_slots = 0, cpu_slots = 0;
  for (int t = 0; t < B; ++t)
    for (int j = 0; j < k; ++j) {
      const int e = rec.tok[t].final_[j];
      res_slots += (plan.before >> e) & 1ull;
      for (int i = 0; i < plan.n_cpu; ++i) cpu_slots += plan.on_cpu[i] == e;
    }
  int64_t late_slots = (int64_t)B * k - res_slots - cpu_slots, shared_times = B;
  if (grouped) {                                      // weights are streamed once per distinct expert
    res_slots = __builtin_popcountll(plan.shield & plan.before);
    late_slots = plan.n_fetch + plan.n_adopted;
    shared_times = 1;
  }
  const int64_t up_r = 2ll * c.hidden * c.ffn * h->esize, up_s = 2ll * c.hidden * c.shared_ffn * h->esize;
  const int64_t resident_up = res_slots * up_r + shared_times * c.n_shared * up_s;
  if (timed[0]) h->prof[SMOE_PROF_ROUTE].bytes += (int64_t)c.n_experts * c.hidden * h->esize;
  if (timed[1]) h->prof[SMOE_PROF_UP].bytes += resident_up;
  if (timed[2]) h->prof[SMOE_PROF_DOWN].bytes += resident_up / 2;
  if (timed[3]) h->prof[SMOE_PROF_UP_LOADED].bytes += late_slots * up_r;
  if (timed[4]) h->prof[SMOE_PROF_DOWN_LOADED].bytes += late_slots * up_r / 2;
}

void fill_trace(const moe_handle* h, int B, const StepRec& rec, const StepPlan& plan, moe_trace_t* trace) {
  const int k = h->cfg.top_k, E = h->cfg.n_experts;
  for (int t = 0; t < B; ++t)
    for (int j = 0; j < k; ++j) {
      const int o = t * k + j;
      if (trace->topk_idx) trace->topk_idx[o] = rec.tok[t].topk[j];
      if (trace->final_idx) trace->final_idx[o] = rec.tok[t].final_[j];
      if (trace->substituted) trace->substituted[o] = (uint8_t)(rec.tok[t].subst[j] != 0);
      if (trace->hit) trace->hit[o] = (uint8_t)((plan.on_gpu >> rec.tok[t].final_[j]) & 1ull);
      if (trace->weights) trace->weights[o] = rec.tok[t].w[j];
    }
  if (trace->scores)
    for (int t = 0; t < B; ++t)
      std::memcpy(trace->scores + (size_t)t * E, rec.tok[t].scores, sizeof(float) * E);
  for (int i = 0; i < B * k; ++i) {
    if (trace->fetched) trace->fetched[i] = i < plan.n_fetch ? plan.fetched[i] : -1;
    if (trace->victims) trace->victims[i] = i < plan.n_fetch ? plan.victims[i] : -1;
    if (trace->on_cpu) trace->on_cpu[i] = i < plan.n_cpu ? plan.on_cpu[i] : -1;
    if (trace->adopted) trace->adopted[i] = i < plan.n_adopted ? plan.adopted[i] : -1;
    if (trace->adopt_victims) trace->adopt_victims[i] = i < plan.n_adopted ? plan.adopt_victims[i] : -1;
  }
  trace->n_fetched = plan.n_fetch;
  trace->n_on_cpu = plan.n_cpu;
  trace->n_adopted = plan.n_adopted;
}

}  // namespace

extern "C" {

int moe_last_hip_error(void) { return g_last_hip; }

int moe_cache_init(const moe_cfg_t* cfg, const moe_buffers_t* buf, moe_handle_t** out) {
  if (!cfg || !buf || !out) return SMOE_EINVAL;
  *out = nullptr;
  const moe_cfg_t& c = *cfg;
  if (c.dtype != SMOE_DTYPE_FP32 && c.dtype != SMOE_DTYPE_BF16) return SMOE_EINVAL;
  if (c.n_layers < 1 || c.hidden < 8 || c.hidden > SMOE_MAX_HIDDEN || c.hidden % 8) return SMOE_EINVAL;
  if (c.n_experts < 1 || c.n_experts > SMOE_MAX_EXPERTS) return SMOE_EINVAL;
  if (c.ffn < 8 || c.ffn % 8) return SMOE_EINVAL;
  if (c.top_k < 1 || c.top_k > SMOE_MAX_TOPK || c.top_k > c.n_experts) return SMOE_EINVAL;
  if (c.cache_cap < c.top_k || c.cache_cap > c.n_experts) return SMOE_EINVAL;
  if (c.n_shared < 0 || c.n_shared > SMOE_MAX_SHARED) return SMOE_EINVAL;
  if (c.n_shared > 0 && (c.shared_ffn < 8 || c.shared_ffn % 8)) return SMOE_EINVAL;
  if (c.max_batch < 1 || c.max_batch > SMOE_MAX_BATCH) return SMOE_EINVAL;
  if (!(c.alpha >= 0.0f) || c.alpha >= 1.0f) return SMOE_EINVAL;
  if (c.subst_key != 0 && c.subst_key != 1) return SMOE_EINVAL;
  if (c.evict_window < 0 || c.evict_window > 1024 || c.n_stage < 0) return SMOE_EINVAL;
  if (c.evict_policy < SMOE_EVICT_SCORE || c.evict_policy > SMOE_EVICT_LFU) return SMOE_EINVAL;
  if (c.prefetch_max < 0 || c.prefetch_max > SMOE_MAX_BATCH * SMOE_MAX_TOPK - 1) return SMOE_EINVAL;
  if (c.cpu_assist < 0 || c.cpu_assist > 2 || c.cpu_threads < 0 || c.cpu_threads > 256) return SMOE_EINVAL;
  if (c.auto_prefetch < 0 || c.auto_prefetch > 1 || (c.auto_prefetch && c.prefetch_max < 1)) return SMOE_EINVAL;
  if (c.prefetch_yield < 0 || c.prefetch_yield > 1) return SMOE_EINVAL;
  if (!buf->gate_w_dev || !buf->experts_host || !buf->sim_host || !buf->cache_slab_dev) return SMOE_EINVAL;
  if (c.n_shared > 0 && !buf->shared_dev) return SMOE_EINVAL;
  if (buf->stream_compute == buf->stream_copy) return SMOE_EINVAL;
  if (reinterpret_cast<uintptr_t>(buf->cache_slab_dev) % 256) return SMOE_EINVAL;

  for (int l = 0; l < c.n_layers; ++l) {
    if (!buf->experts_host[l]) return SMOE_EINVAL;
    hipPointerAttribute_t attr;
    hipError_t pe = hipPointerGetAttributes(&attr, buf->experts_host[l]);
    if (pe != hipSuccess) { (void)hipGetLastError(); return SMOE_ENOTPINNED; }
    if (attr.type != hipMemoryTypeHost) return SMOE_ENOTPINNED;
  }

  moe_handle* h = new (std::nothrow) moe_handle();
  if (!h) return SMOE_EINVAL;
  h->cfg = c;
  h->buf = *buf;
  h->s_compute = static_cast<hipStream_t>(buf->stream_compute);
  h->s_copy = static_cast<hipStream_t>(buf->stream_copy);
  h->esize = c.dtype == SMOE_DTYPE_FP32 ? 4 : 2;
  h->expert_bytes = 3ll * c.hidden * c.ffn * h->esize;
  h->shared_bytes = 3ll * c.hidden * c.shared_ffn * h->esize;
  h->Fmax = std::max(c.ffn, c.n_shared ? c.shared_ffn : 0);
  h->layers.resize(c.n_layers);
  h->cp = CacheParams{c.n_experts, c.top_k, c.cache_cap, c.evict_window, c.evict_policy, c.n_stage,
                      c.alpha, c.prefetch_max, c.cpu_assist};
  h->pf_last.layer = -1;
  for (int l = 0; l < c.n_layers; ++l)
    h->experts_host.push_back(static_cast<const char*>(buf->experts_host[l]));
  h->buf.experts_host = nullptr;
  h->init_resident.resize((size_t)c.n_layers * c.cache_cap);
  for (int l = 0; l < c.n_layers; ++l) {
    uint64_t seen = 0;
    for (int s = 0; s < c.cache_cap; ++s) {
      const int e = buf->init_resident ? buf->init_resident[(size_t)l * c.cache_cap + s] : s;
      if (e < 0 || e >= c.n_experts || ((seen >> e) & 1ull)) { delete h; return SMOE_EINVAL; }
      seen |= 1ull << e;
      h->init_resident[(size_t)l * c.cache_cap + s] = e;
    }
  }
  h->buf.init_resident = nullptr;
  plan_geometry(h);

  const int nj = c.top_k + c.n_shared;
  const size_t sim_bytes = (size_t)c.n_layers * c.n_experts * c.n_experts * sizeof(float);
  int rc = [&]() -> int {
    HIP_TRY(hipEventCreateWithFlags(&h->ev_copy, hipEventDisableTiming));
    HIP_TRY(hipMalloc(&h->sim_dev, sim_bytes));
    HIP_TRY(hipMemcpy(h->sim_dev, buf->sim_host, sim_bytes, hipMemcpyHostToDevice));
    HIP_TRY(hipMalloc(&h->own.rec, sizeof(StepRec)));
    HIP_TRY(hipHostMalloc(&h->rec_host, sizeof(StepRec), hipHostMallocDefault));
    std::memset(h->rec_host, 0, sizeof(StepRec));
    h->spin_limit = env_int("SMOE_SPIN_LIMIT", 4000000);
    h->fused_select = env_int("SMOE_FUSED_SELECT", 1);
    // (worth it where blocks exist that can stream while the logits are on their way: the shared
    // experts'.  Without them every block of the launch waits for the gate blocks and the kernel
    // boundary it replaces was no slower: measured on the Mixtral-shaped workload)
    h->fused_gate = env_int("SMOE_FUSED_GATE", c.n_shared > 0 ? 1 : 0);
    h->gate_spin = std::max(0, env_int("SMOE_GATE_SPIN", 8192));
    {
      static std::atomic<int> next_uid{0};
      h->uid = next_uid.fetch_add(1) % 255 + 1;
    }
    h->mfma_contig = env_int("SMOE_MFMA_CONTIG", 1) != 0 ? 1 : 0;
    h->mfma_ok = env_int("SMOE_MFMA", 2);   // 0: vector ALUs, 1: MFMA down only, 2: MFMA up and down
    void* dp = nullptr;
    HIP_TRY(hipHostGetDevicePointer(&dp, h->rec_host, 0));
    h->rec_host_dev = static_cast<StepRec*>(dp);
    {
      const int64_t maxg = std::min(c.n_experts, c.max_batch * c.top_k);
      const int64_t grouped = maxg * SMOE_MAX_BATCH * c.ffn + (int64_t)c.n_shared * SMOE_MAX_BATCH * c.shared_ffn;
      h->act_floats = std::max<int64_t>((int64_t)c.max_batch * nj * h->Fmax, grouped);
    }
    HIP_TRY(hipMalloc(&h->own.act, (size_t)h->act_floats * sizeof(float)));
    HIP_TRY(hipMalloc(&h->own.ysum, (size_t)c.max_batch * c.hidden * sizeof(float)));
    HIP_TRY(hipMalloc(&h->own.gate_part, (size_t)(kGatePartBytes + kGateWordBytes)));
    HIP_TRY(hipMemset(h->own.gate_part, 0, (size_t)(kGatePartBytes + kGateWordBytes)));   // epoch 0 = never written
    HIP_TRY(hipMalloc(&h->own.x_pred, (size_t)c.max_batch * c.hidden * h->esize));
    {
      // the same buffers inside this GPU's static array, for moe_decode_layer_static
      HIP_TRY(hipGetDevice(&h->device));
      unsigned char* base = nullptr;
      const int src = scratch_of_device(h->device, &base);
      if (src != SMOE_OK) return src;
      int64_t off = 0;
      auto carve = [&](int64_t bytes) { const int64_t o = off; off += (bytes + 255) / 256 * 256; return o; };
      const int64_t o_rec = carve(sizeof(StepRec));
      const int64_t o_part = carve(kGatePartBytes + kGateWordBytes);
      const int64_t o_xp = carve((int64_t)c.max_batch * c.hidden * h->esize);
      const int64_t o_ysum = carve((int64_t)c.max_batch * c.hidden * sizeof(float));
      const int64_t o_act = carve(h->act_floats * (int64_t)sizeof(float));
      h->fixed_need = off;
      if (off <= (int64_t)SMOE_STATIC_SCRATCH_BYTES) {
        h->fixed.rec = reinterpret_cast<StepRec*>(base + o_rec);
        h->fixed.gate_part = reinterpret_cast<float*>(base + o_part);
        h->fixed.x_pred = base + o_xp;
        h->fixed.ysum = reinterpret_cast<float*>(base + o_ysum);
        h->fixed.act = reinterpret_cast<float*>(base + o_act);
      }
    }
    if (c.prefetch_max > 0) {
      HIP_TRY(hipMalloc(&h->pred_dev, sizeof(StepRec)));
      HIP_TRY(hipHostMalloc(&h->pred_host, sizeof(StepRec), hipHostMallocDefault));
      std::memset(h->pred_host, 0, sizeof(StepRec));
      HIP_TRY(hipHostGetDevicePointer(&dp, h->pred_host, 0));
      h->pred_host_dev = static_cast<StepRec*>(dp);
      h->slot_guard.assign((size_t)staging_slot_base(h), -1);
      h->chunks_out_limit = std::max(1, std::min((int)moe_handle::kMaxChunksOut, env_int("SMOE_PF_OUTSTANDING", 4)));
      h->chunk_bytes = (int64_t)std::max(1, env_int("SMOE_PF_CHUNK_MB", 64)) << 20;
      for (auto& e : h->chunk_ev) HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    }
    if (c.cpu_assist) {
      int nt = c.cpu_threads;
      if (nt == 0) nt = (int)std::min(16u, std::max(1u, std::thread::hardware_concurrency()));
      h->cpu = new CpuExperts(nt);
      // the host cores will read expert weights that may only ever have been written by a
      // device: fault their pages into the CPU mapping now, not on the first use of each expert
      for (int l = 0; l < c.n_layers; ++l) {
        bool seen = false;
        for (int q = 0; q < l; ++q) seen |= h->experts_host[q] == h->experts_host[l];
        if (!seen) h->cpu->touch(h->experts_host[l], (size_t)c.n_experts * h->expert_bytes);
      }
      HIP_TRY(hipHostMalloc(&h->x_host, (size_t)c.max_batch * c.hidden * h->esize, hipHostMallocDefault));
      HIP_TRY(hipHostGetDevicePointer(&h->x_host_dev, h->x_host, 0));
      void* yp = nullptr;
      HIP_TRY(hipHostMalloc(&yp, (size_t)c.max_batch * c.hidden * sizeof(float), hipHostMallocDefault));
      h->ycpu_host = static_cast<float*>(yp);
      HIP_TRY(hipHostGetDevicePointer(&yp, h->ycpu_host, 0));
      h->ycpu_host_dev = static_cast<float*>(yp);
      h->x_f32.assign((size_t)c.max_batch * c.hidden, 0.f);
      for (auto& p : h->copy_ev) {
        HIP_TRY(hipEventCreate(&p.a));
        HIP_TRY(hipEventCreate(&p.b));
      }
    }
    const auto up0 = std::chrono::steady_clock::now();
    const int urc = upload_initial(h);
    if (urc != SMOE_OK) return urc;
    if (c.cpu_assist) {
      // first estimates of the two costs of Algorithm 2: the initial upload gives the copy
      // time of one expert, one run of the host FFN on zeros (after a warm-up run) its own
      const auto up1 = std::chrono::steady_clock::now();
      h->c_load_us = c.load_cost_us > 0.f
                         ? c.load_cost_us
                         : std::chrono::duration<double, std::micro>(up1 - up0).count() /
                               ((double)c.n_layers * c.cache_cap);
      if (c.cpu_cost_us > 0.f) {
        h->c_cpu_us = c.cpu_cost_us;
      } else {
        const float* xs[1] = {h->x_f32.data()};
        const float ws[1] = {1.0f};
        float* ys[1] = {h->ycpu_host};
        std::memset(h->ycpu_host, 0, sizeof(float) * c.hidden);
        for (int rep = 0; rep < 2; ++rep) {
          const auto t0 = std::chrono::steady_clock::now();
          h->cpu->run(h->experts_host[0], c.dtype, c.hidden, c.ffn, 1, xs, ws, ys);
          const auto t1 = std::chrono::steady_clock::now();
          h->c_cpu_us = std::chrono::duration<double, std::micro>(t1 - t0).count();
        }
      }
    }
    return SMOE_OK;
  }();
  if (rc != SMOE_OK) { free_all(h); return rc; }
  *out = h;
  return SMOE_OK;
}

// One decode step of one layer with the kernels' scratch in `sc`: the body of
// moe_decode_layer and moe_decode_layer_static.
static int decode_layer_with(moe_handle_t* h, const Scratch& sc, int32_t layer, int32_t batch,
                             const void* x_dev, void* y_dev, moe_trace_t* trace) {
  const moe_cfg_t& c = h->cfg;
  CacheLayer& ls = h->layers[layer];
  const int B = batch;
  bool timed[5] = {false, false, false, false, false};   // route, up, down, up (2nd pass), down (2nd pass)

  // ---- a prefetch for this very layer has to be decided before it is routed ----
  if (h->pending_layer == layer) {
    const int rc = settle_prefetch(h);
    if (rc != SMOE_OK) return rc;
  } else if (!h->pf_entries.empty()) {
    // keep the link fed (slots that the previous call's kernels may still read are guarded)
    const int rc = pump_prefetch_queue(h, layer);
    if (rc != SMOE_OK) return rc;
  }

  // ---- router + expert-cache router ------------------------------------------
  RouteArgs ra{};
  fill_route_args(h, sc, layer, B, x_dev, ra);
  ra.rec_dev = sc.rec;
  ra.rec_host = h->rec_host_dev;
  ra.seq = ++h->seq;
  if (c.cpu_assist) {                    // the host cores may need x: the router kernel mirrors it
    ra.x_mirror = h->x_host_dev;
    ra.x_units = (int32_t)((int64_t)B * c.hidden * h->esize / 16);
  }
  FfnArgs fa{};
  fill_ffn_args(h, sc, layer, B, x_dev, y_dev, fa);
  // batch 1 on the register up kernel: the selection runs in that kernel's prologue
  fa.fused_select = (B == 1 && h->fused_select && fa.up_upl > 0 && !fa.grouped) ? 1 : 0;
  if (fa.fused_select && h->fused_gate) {
    // the gate GEMV runs in the first blocks of the up kernel: two launches per layer
    ra.gate_blocks = (c.n_experts + 3) / 4;
    ra.epoch = ((uint32_t)h->uid << 24) | ((uint32_t)h->seq & 0xFFFFFFu);
  } else {
    EventPair* pr = prof_begin(h, SMOE_PROF_ROUTE, h->s_compute);
    launch_gate_partial(ra, c.dtype, h->s_compute);
    if (!fa.fused_select) launch_route_select(ra, h->s_compute);
    prof_end(pr, h->s_compute);
    timed[0] = pr != nullptr;
    HIP_TRY(hipGetLastError());
  }
  // (no event after the router kernels: an event record costs several microseconds of
  // stream time between the router and the FFN; the host polls the mirror instead)

  // ---- FFN over what is already resident (+ shared experts), enqueued before
  //      the host knows the routing result ------------------------------------
  {
    const int rc = launch_ffn_pair(h, fa, ra, SMOE_PROF_UP, SMOE_PROF_DOWN, &timed[1], &timed[2]);
    if (rc != SMOE_OK) return rc;
  }

  // ---- top-score prefetch from the partial output (Section IV-C): the input of the next
  //      layer is predicted from what the resident pass has produced and that layer's gate
  //      runs on it, queued right behind the resident pass; its decision is taken when the
  //      next layer is decoded ----------------------------------------------------------
  if (c.auto_prefetch && layer + 1 < c.n_layers) {
    {
      const int rc = settle_prefetch(h);                // one prediction may wait at a time
      if (rc != SMOE_OK) return rc;
    }
    if (c.prefetch_yield && link_busy(h)) {
      note_yielded_prefetch(h, layer + 1);
    } else {
      launch_predict_state(sc.rec, x_dev, y_dev, sc.ysum, sc.x_pred, B, c.hidden, c.top_k, c.dtype, h->s_compute);
      RouteArgs pa{};
      fill_route_args(h, sc, layer + 1, B, sc.x_pred, pa);
      pa.rec_dev = h->pred_dev;
      pa.rec_host = h->pred_host_dev;
      pa.seq = ++h->pred_seq;
      launch_gate_partial(pa, c.dtype, h->s_compute);
      launch_route_select(pa, h->s_compute);
      HIP_TRY(hipGetLastError());
      h->pending_layer = layer + 1;
      h->pending_batch = B;
    }
  }

  // ---- the decision reaches the host: poll the pinned mirror (the router kernel
  //      publishes its call number last), then fall back to draining the stream ----
  {
    const int rc = await_record(h, h->rec_host, h->seq);
    if (rc != SMOE_OK) return rc;
  }
  const StepRec& rec = *h->rec_host;

  // ---- cache bookkeeping: history, shield, Algorithm 2, victims, residency, counters ----
  StepDecision dec{};
  dec.B = B;
  for (int t = 0; t < B; ++t) {
    dec.topk[t] = rec.tok[t].topk;
    dec.final_[t] = rec.tok[t].final_;
    dec.subst[t] = rec.tok[t].subst;
    dec.scores[t] = rec.tok[t].scores;
  }
  StepPlan plan;
  // prefetched experts of this layer whose copy is not complete: with CPU-assisted scheduling
  // Algorithm 2 may give them to the host cores instead of waiting (Section V-B, dependency 2)
  const uint64_t inflight = (ls.n_landed > 0) ? prefetches_in_flight(h, layer) : 0;
  {
    if (c.cpu_assist) refresh_load_cost(h);
    const int rc = ls.plan_step(h->cp, dec, h->expert_bytes, plan, h->c_load_us, h->c_cpu_us, inflight);
    if (rc != SMOE_OK) return rc;
  }
  // prefetched experts the step does not wait for leave the load queue; what was not yet
  // handed to the copy stream is never copied
  for (int i = 0; i < plan.n_dropped; ++i) retire_prefetch_entry(h, layer, plan.dropped[i], true);
  // a prefetched expert that found no victim is computed where it landed and its slot is
  // spare again at once: nothing may be copied into it while this call's kernels run
  for (int i = 0; i < plan.n_adopted; ++i)
    if (plan.adopt_victims[i] < 0) h->slot_guard[layer_slot_base(h, layer) + plan.adopt_slot[i]] = h->seq;

  if (plan.n_fetch > 0 || plan.n_adopted > 0 || plan.n_cpu > 0) {
    // ---- copies the second FFN pass waits for: first the rest of the prefetched experts
    //      this step computes (requested earlier), then the on-demand loads ------------
    hipEvent_t adopted_done[SMOE_MAX_BATCH * SMOE_MAX_TOPK];
    for (int i = 0; i < plan.n_adopted; ++i) {
      moe_handle::PfEntry* e = find_prefetch_entry(h, layer, plan.adopted[i]);
      if (!e) return SMOE_ESTATE;
      const int rc = finish_prefetch_entry(h, e);
      if (rc != SMOE_OK) return rc;
      adopted_done[i] = e->done;
    }
    int gslot[SMOE_MAX_BATCH * SMOE_MAX_TOPK];
    {
      const int rc = enqueue_loads(h, layer, plan, gslot);
      if (rc != SMOE_OK) return rc;
    }
    if (plan.n_cpu > 0) {
      // ---- CPU-assisted scheduling: while the copies run, the host cores compute the
      //      experts Algorithm 2 left to them; a prefetch that is waiting for its decision
      //      joins the load queue first so that the link stays busy meanwhile.  The result is
      //      added to the fp32 sums of the resident pass, and the second pass rounds y once.
      const bool own_prediction = c.auto_prefetch && h->pending_layer == layer + 1;
      const int rc = own_prediction ? SMOE_OK : settle_prefetch(h);
      if (rc != SMOE_OK) return rc;
      compute_on_cpu(h, layer, B, rec, plan.on_cpu, plan.n_cpu);
      launch_add_partial(sc.ysum, h->ycpu_host_dev, B * c.hidden, h->s_compute);
      HIP_TRY(hipGetLastError());
    }
    if (plan.n_fetch > 0) {
      // (recorded behind the loads, which are behind everything handed over before)
      HIP_TRY(hipStreamWaitEvent(h->s_compute, h->ev_copy, 0));
    } else {
      for (int i = 0; i < plan.n_adopted; ++i) HIP_TRY(hipStreamWaitEvent(h->s_compute, adopted_done[i], 0));
    }
    set_second_pass_slots(h, layer, B, rec, plan, gslot, fa);
    fa.fused_select = 0;
    const int rc = launch_ffn_pair(h, fa, ra, SMOE_PROF_UP_LOADED, SMOE_PROF_DOWN_LOADED, &timed[3], &timed[4]);
    if (rc != SMOE_OK) return rc;
    // the adopted experts' queue entries are done with (their events stay valid: a recorded
    // event may be re-recorded only after the wait above has been enqueued, which it has)
    for (int i = 0; i < plan.n_adopted; ++i) retire_prefetch_entry(h, layer, plan.adopted[i], false);
  }
  // ---- a prefetch waiting for its decision (for another layer) joins the load queue now,
  //      and the queue is fed: behind the loads this layer is waiting for --------------
  {
    // (a prediction this call has launched itself is left for the next call: it is queued
    // behind the resident pass, waiting for it here would stall the host)
    const bool own_prediction = c.auto_prefetch && h->pending_layer == layer + 1;
    int rc = own_prediction ? SMOE_OK : settle_prefetch(h);
    if (rc == SMOE_OK) rc = pump_prefetch_queue(h, layer + 1 < c.n_layers ? layer + 1 : 0);
    if (rc != SMOE_OK) return rc;
  }
  if (h->prof_mask) account_profile_bytes(h, B, rec, plan, fa.grouped != 0, timed);
  if (trace) {
    fill_trace(h, B, rec, plan, trace);
    trace->inflight_mask = inflight & plan.shield;
  }
  return SMOE_OK;
}

int moe_decode_layer(moe_handle_t* h, int32_t layer, int32_t batch, const void* x_dev, void* y_dev,
                     moe_trace_t* trace) {
  if (!h || !x_dev || !y_dev) return SMOE_EINVAL;
  if (layer < 0 || layer >= h->cfg.n_layers || batch < 1 || batch > h->cfg.max_batch) return SMOE_EINVAL;
  return decode_layer_with(h, h->own, layer, batch, x_dev, y_dev, trace);
}

int moe_decode_layer_static(moe_handle_t* h, int32_t layer, int32_t batch, const void* x_dev, void* y_dev,
                            moe_trace_t* trace) {
  if (!h || !x_dev || !y_dev) return SMOE_EINVAL;
  if (layer < 0 || layer >= h->cfg.n_layers || batch < 1 || batch > h->cfg.max_batch) return SMOE_EINVAL;
  if (h->fixed_need > (int64_t)SMOE_STATIC_SCRATCH_BYTES || !h->fixed.rec) return SMOE_ETOOBIG;
  // The array is shared by every handle on this GPU and keeps the previous call's contents.
  // Nothing in it has to start at zero: every part is written by this call's kernels (gate
  // partial sums, decision record, activations, carry-over sums) before it is read.
  return decode_layer_with(h, h->fixed, layer, batch, x_dev, y_dev, trace);
}

int moe_prefetch_layer(moe_handle_t* h, int32_t layer, int32_t batch, const void* x_pred_dev) {
  if (!h || !x_pred_dev) return SMOE_EINVAL;
  const moe_cfg_t& c = h->cfg;
  if (c.prefetch_max < 1 || layer < 0 || layer >= c.n_layers || batch < 1 || batch > c.max_batch)
    return SMOE_EINVAL;
  {
    const int rc = settle_prefetch(h);      // one prediction may wait at a time
    if (rc != SMOE_OK) return rc;
  }
  if (c.prefetch_yield && link_busy(h)) {
    note_yielded_prefetch(h, layer);
    return SMOE_OK;
  }
  // The prediction is the router kernel itself on the predicted hidden state,
  // writing to a record of its own; only its scores and top-k are used.
  RouteArgs ra{};
  fill_route_args(h, h->own, layer, batch, x_pred_dev, ra);
  ra.rec_dev = h->pred_dev;
  ra.rec_host = h->pred_host_dev;
  ra.seq = ++h->pred_seq;
  launch_gate_partial(ra, c.dtype, h->s_compute);
  launch_route_select(ra, h->s_compute);
  HIP_TRY(hipGetLastError());
  h->pending_layer = layer;
  h->pending_batch = batch;
  return SMOE_OK;
}

int moe_cpu_assist_costs(const moe_handle_t* h, double* c_load_us, double* c_cpu_us, double* cpu_busy_us,
                         int64_t* cpu_experts) {
  if (!h) return SMOE_EINVAL;
  if (!h->cfg.cpu_assist) return SMOE_ESTATE;
  if (c_load_us) *c_load_us = h->c_load_us;
  if (c_cpu_us) *c_cpu_us = h->c_cpu_us;
  if (cpu_busy_us) *cpu_busy_us = h->cpu_busy_us;
  if (cpu_experts) *cpu_experts = h->cpu_experts;
  return SMOE_OK;
}

int moe_prefetch_last(moe_handle_t* h, moe_prefetch_info_t* out) {
  if (!h || !out) return SMOE_EINVAL;
  const int rc = settle_prefetch(h);
  if (rc != SMOE_OK) return rc;
  *out = h->pf_last;
  out->bytes_copied = h->pf_bytes_submitted;
  out->bytes_withdrawn = h->pf_bytes_withdrawn;
  return SMOE_OK;
}

int moe_cache_stats(moe_handle_t* h, int32_t layer, moe_stats_t* out) {
  if (!h || !out || layer < -1 || layer >= h->cfg.n_layers) return SMOE_EINVAL;
  {
    const int rc = settle_prefetch(h);
    if (rc != SMOE_OK) return rc;
  }
  moe_stats_t s{};
  for (int l = 0; l < h->cfg.n_layers; ++l) {
    if (layer >= 0 && l != layer) continue;
    const moe_stats_t& a = h->layers[l].st;
    s.tokens += a.tokens; s.slots += a.slots; s.raw_hits += a.raw_hits; s.hits += a.hits;
    s.misses += a.misses; s.substitutions += a.substitutions; s.evictions += a.evictions;
    s.staged += a.staged; s.fetches += a.fetches; s.bytes_fetched += a.bytes_fetched;
    s.prefetches += a.prefetches; s.prefetch_used += a.prefetch_used; s.prefetch_top += a.prefetch_top;
    s.cpu_computed += a.cpu_computed;
  }
  *out = s;
  return SMOE_OK;
}

int moe_cache_residency(moe_handle_t* h, int32_t layer, int32_t* out_slots) {
  if (!h || !out_slots || layer < 0 || layer >= h->cfg.n_layers) return SMOE_EINVAL;
  {
    const int rc = settle_prefetch(h);
    if (rc != SMOE_OK) return rc;
  }
  const CacheLayer& ls = h->layers[layer];
  for (int s = 0; s < h->cfg.cache_cap; ++s) out_slots[s] = ls.expert_of_slot[s];
  return SMOE_OK;
}

int moe_cache_reset(moe_handle_t* h) {
  if (!h) return SMOE_EINVAL;
  HIP_TRY(hipStreamSynchronize(h->s_compute));
  HIP_TRY(hipStreamSynchronize(h->s_copy));
  h->pending_layer = -1;                     // a prediction that was not acted on is dropped
  h->pf_last.layer = -1;
  h->pf_last.n_wanted = h->pf_last.n_loaded = 0;
  for (auto& e : h->pf_entries) h->pf_event_pool.push_back(e.done);
  h->pf_entries.clear();
  for (bool& b : h->chunk_busy) b = false;
  h->pf_bytes_submitted = h->pf_bytes_withdrawn = 0;
  h->pf_yielded = 0;
  std::fill(h->slot_guard.begin(), h->slot_guard.end(), -1);
  return upload_initial(h);
}

int moe_cache_destroy(moe_handle_t* h) {
  if (!h) return SMOE_EINVAL;
  (void)hipStreamSynchronize(h->s_compute);
  (void)hipStreamSynchronize(h->s_copy);
  free_all(h);
  return SMOE_OK;
}

int moe_profile_enable(moe_handle_t* h, int32_t enable, int32_t max_launches) {
  if (!h || enable < 0 || enable >= (1 << SMOE_PROF_KINDS) || (enable && max_launches < 1)) return SMOE_EINVAL;
  HIP_TRY(hipStreamSynchronize(h->s_compute));
  HIP_TRY(hipStreamSynchronize(h->s_copy));
  if (enable) {
    for (int kind = 0; kind < SMOE_PROF_KINDS; ++kind) {
      ProfKind& k = h->prof[kind];
      while (((enable >> kind) & 1) && (int)k.ev.size() < max_launches) {
        EventPair p{};
        HIP_TRY(hipEventCreate(&p.a));
        HIP_TRY(hipEventCreate(&p.b));
        k.ev.push_back(p);
      }
      k.used = 0;
      k.bytes = 0;
    }
  }
  h->prof_mask = (uint32_t)enable;
  return SMOE_OK;
}

int moe_profile_read(moe_handle_t* h, moe_profile_t* out) {
  if (!h || !out) return SMOE_EINVAL;
  HIP_TRY(hipStreamSynchronize(h->s_compute));
  HIP_TRY(hipStreamSynchronize(h->s_copy));
  for (int kind = 0; kind < SMOE_PROF_KINDS; ++kind) {
    double ms = 0.0;
    for (size_t i = 0; i < h->prof[kind].used; ++i) {
      float t = 0.f;
      HIP_TRY(hipEventElapsedTime(&t, h->prof[kind].ev[i].a, h->prof[kind].ev[i].b));
      ms += t;
    }
    out->launches[kind] = (int64_t)h->prof[kind].used;
    out->ms[kind] = ms;
    out->bytes[kind] = h->prof[kind].bytes;
  }
  return SMOE_OK;
}

int moe_select_alpha(const double* alphas, const double* tpots, int32_t n, double budget, int32_t degree,
                     int32_t resolution, double* out_alpha, double* out_coef) {
  const int rc = smoe::select_alpha(alphas, tpots, n, budget, degree, resolution, out_alpha, out_coef);
  if (rc < 0) return SMOE_EINVAL;
  return rc == 0 ? SMOE_OK : SMOE_ESTATE;
}

int moe_host_alloc(int64_t n_bytes, void** out) {
  if (!out || n_bytes <= 0) return SMOE_EINVAL;
  *out = nullptr;
  HIP_TRY(hipHostMalloc(out, (size_t)n_bytes, hipHostMallocDefault));
  return SMOE_OK;
}

int moe_host_free(void* p) {
  if (!p) return SMOE_EINVAL;
  HIP_TRY(hipHostFree(p));
  return SMOE_OK;
}

int moe_calib_copy(void* dst_dev, const void* src_dev, int64_t n_bytes, void* stream) {
  if (!dst_dev || !src_dev || n_bytes <= 0 || n_bytes % 16) return SMOE_EINVAL;
  if (reinterpret_cast<uintptr_t>(dst_dev) % 16 || reinterpret_cast<uintptr_t>(src_dev) % 16)
    return SMOE_EINVAL;
  launch_copy(dst_dev, src_dev, n_bytes, static_cast<hipStream_t>(stream));
  HIP_TRY(hipGetLastError());
  return SMOE_OK;
}

}  // extern "C"
