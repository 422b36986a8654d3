// Device-side records and launch arguments shared by the kernels and the host
// scheduler of libsmoe.  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "smoe.h"

namespace smoe {

constexpr int kWave = 64;
constexpr int kMaxTasks = SMOE_MAX_BATCH * (SMOE_MAX_TOPK + SMOE_MAX_SHARED);
constexpr int kStageElems = 16384;     // fp32 activations a down-projection block can hold in LDS
constexpr int kChunkElems = 8192;      // default chunk when the activations do not fit at once

// Routing decision of one token, written by the router kernel to device memory
// (read by the FFN kernels) and to a pinned host mirror (read by the scheduler).
struct TokRec {
  int32_t topk[SMOE_MAX_TOPK];     // E_a by descending score
  int32_t final_[SMOE_MAX_TOPK];   // expert computed in each slot after substitution
  int32_t slot[SMOE_MAX_TOPK];     // cache slot (layer-local) of final_, -1 when not resident
  int32_t subst[SMOE_MAX_TOPK];    // 1 where final_ != topk
  float   w[SMOE_MAX_TOPK];        // combine weight
  float   scores[SMOE_MAX_EXPERTS];
};
// Batch > 1: one entry per distinct expert of the step, ascending expert id,
// with the tokens that compute it (device copy of the record only).
struct GroupTask {
  int32_t expert;
  int32_t slot;                    // layer-local cache slot, -1 when not resident
  int32_t ntok;
  int32_t pad_;
  int32_t tok[SMOE_MAX_BATCH];     // tokens using this expert, ascending
  float   w[SMOE_MAX_BATCH];       // their combine weights
};
struct StepRec {
  TokRec tok[SMOE_MAX_BATCH];
  int32_t n_groups;
  int32_t pad_[3];
  GroupTask grp[SMOE_MAX_EXPERTS];
  int32_t seq;                     // host mirror only: call number, written last
};

constexpr int kMaxGateSeg = 8;   // a gate row is split into at most this many segments

struct RouteArgs {
  const void* gate_w;   // [E][H] of this layer
  const void* x;        // [B][H]
  const float* sim;     // [E][E] of this layer (device)
  StepRec* rec_dev;
  StepRec* rec_host;    // device-visible address of the pinned mirror
  float* gate_part;     // [B][E][kMaxGateSeg] partial dot products of the gate GEMV, the first nseg of
                        // each row in use (device scratch, 32-byte aligned)
  void* x_mirror;       // device-visible pinned host copy of x for the host cores, or null
  int32_t x_units;      // 16-byte units of x ([B][H] dtype) to mirror
  int32_t B, H, E, k;
  int32_t renorm, subst_key;
  int32_t nseg;         // segments each gate row is split into (power of two, <= kMaxGateSeg)
  int32_t upi;          // 128-bit units of one row segment per lane (1, 2, 4 or 8)
  int32_t seq;          // call number published to the host mirror when the record is complete
  float alpha;
  // Gate GEMV inside the up kernel (batch 1, selection fused): the first gate_blocks blocks of
  // that launch compute the logits, one wave per expert row, and publish each as one 64-bit
  // word {epoch, logit bits} in gate_word[e]; the routed blocks read the words until all carry
  // this call's epoch (at most gate_spin times, then they compute the logits themselves).
  unsigned long long* gate_word;   // [E], device scratch
  uint32_t epoch;                  // unique per (handle, call); never 0
  int32_t gate_blocks;             // 0: the logits come from gate_part (separate gate launch)
  int32_t gate_spin;
  uint64_t resident;                  // bit e = expert e is in the HBM cache
  int8_t slot_of[SMOE_MAX_EXPERTS];   // layer-local slot of each resident expert
};

// One launch of the up (gate/up projection + SwiGLU) or down (down projection
// + combine) kernel.  Task index = token * (k + ns) + j, j < k routed slot j,
// j >= k shared expert j - k.
struct FfnArgs {
  const StepRec* rec;
  const void* x;            // [B][H]
  void* y;                  // [B][H]
  const char* slab;         // cache slab base
  const char* shared;       // this layer's shared experts, or null
  float* act;               // [task][Fmax] weighted SwiGLU activations
  float* ysum;              // [B][H] fp32 sums of pass 0 for tokens that still wait for loads
  int64_t expert_bytes;     // bytes of one routed expert
  int64_t shared_bytes;     // bytes of one shared expert
  int32_t B, H, F, Fs, k, ns;
  int32_t Fmax;
  int32_t slot_base;        // layer * cache_cap
  int32_t pass;             // 0: routed tasks whose expert is resident + shared; 1: slot_override >= 0 only
  int32_t TF, tilesR, tilesS;              // up: f-rows per block, blocks per routed / shared task
  int32_t R, htiles;                       // down: rows per wave, row tiles (4*R rows each) per token
  int32_t stage_all, chunk, down_lds_floats;  // down (LDS path): all activations in LDS at once, else chunked
  int32_t up_upl;                          // up: 128-bit units of x per lane held in registers, 0 = LDS path
  int32_t down_upl, RB, nsegR, nsegS;      // down register path: units per lane (0 = LDS path), rows per
                                           // block, column segments of a routed / shared row
  int32_t down_nw, down_r;                 // ... waves per block (4 or 8), rows per register buffer
  int32_t grouped;                         // batch > 1: tasks are the record's expert groups (+ shared)
  int32_t maxg;                            // grouped: upper bound of groups = min(E, B*k)
  int32_t mfma_down;                       // grouped, bf16: down projection on the matrix cores
  int32_t mfma_contig;                     // its waves take contiguous ranges of items
  int32_t mfma_rt;                         // its output rows per block: 8, 12, 14 or 16
  int32_t mfma_up;                         // ... and the up projection too
  int32_t nsegGR, nsegGS, RBG;             // grouped down kernel: segments per routed / shared row, rows per block
  int64_t act_shared_off;                  // grouped: float offset of the shared experts' activations in act
  int32_t fused_select;                    // batch 1, pass 0: the up kernel runs the selection itself
  int32_t slot_override[kMaxTasks];        // pass 1: global slot per task (grouped: per group), -1 = not in this pass
};

void launch_gate_partial(const RouteArgs& a, int dtype, hipStream_t s);
void launch_route_select(const RouteArgs& a, hipStream_t s);
// `ra` is read only when a.fused_select is set
void launch_ffn_up(const FfnArgs& a, const RouteArgs& ra, int dtype, hipStream_t s);
void launch_ffn_down(const FfnArgs& a, int dtype, hipStream_t s);
size_t grouped_down_lds_bytes(const FfnArgs& a);
void launch_copy(void* dst, const void* src, int64_t n_bytes, hipStream_t s);
// xp[t] = (x[t] + partial[t]) / rms(x[t] + partial[t]) for t < B: the predicted input of the next layer
void launch_predict_state(const StepRec* rec, const void* x, const void* y, const float* ysum, void* xp, int B,
                          int H, int k, int dtype, hipStream_t s);
// ysum[i] += part[i], i < n (n a multiple of 4): adds what the host cores computed
void launch_add_partial(float* ysum, const float* part, int n, hipStream_t s);

}  // namespace smoe
