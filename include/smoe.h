/*
 * smoe.h -- C ABI of the MI355X (gfx950) SMoE offloaded-MoE decode library.
 *
 * One decode step of one MoE layer under the SMoE expert scheduler
 * (arxiv 2508.18983):
 *   router            gate GEMV, softmax over the routed experts, top-k
 *                     (Section II-A; Algorithm 1, "Sort S_t desc")
 *   expert-cache      low-score active experts that are not in the HBM expert
 *   router            cache are replaced by eligible resident experts
 *                     (Section IV-B, Algorithm 1; thresholds T, L, R around the
 *                     (k+1)-th score S_{k+1}, Table "Definitions")
 *   cache update      score-history eviction (Eq. 3) with the protection shield
 *                     (Section IV-B "Cache eviction"; Section V-B dependency 1)
 *   on-demand load    remaining misses are copied host -> HBM on a side stream
 *                     (Section V-B, "Loading Experts from Layer i", dependency 2)
 *   expert FFN        SwiGLU FFN of the chosen experts + shared experts and the
 *                     weighted combine (Section V-B GPU operations 2 and 4,
 *                     Section II-A for shared experts)
 *   CPU-assisted      optional: Algorithm 2 leaves the lowest-scoring misses of a step
 *   scheduling        to the host cores, which compute them from the host copy while
 *                     the others are loaded (Section V-A; Section V-B CPU operations 2, 3)
 *   top-score         optional: the gate of a layer that has not run yet is applied
 *   prefetch          to a predicted hidden state (the caller's, or the library's own
 *                     from the running layer's partial output) and its top-score
 *                     experts go through a load queue behind the current layer's
 *                     own loads; mispredicted ones are withdrawn (Section IV-C;
 *                     Section V-B, "Prefetching Experts from Layer i+1")
 *   alpha selection   the substitution threshold from a latency budget: polynomial
 *                     fit of measured TPOT, smallest feasible alpha (Section V-C, Eq. 5)
 *
 * All entry points return 0 on success or a negative SMOE_E* code; nothing
 * throws across this boundary.  "device" pointers are HIP device pointers on
 * the current device, "host" pointers are ordinary process memory, "pinned
 * host" pointers come from hipHostMalloc (or an equivalent allocator).  The
 * library never allocates or frees expert weights: the caller owns the host
 * copy of every expert, the HBM cache slab, the gate and shared-expert weights
 * and the two streams, and must keep them alive until moe_cache_destroy.  The
 * library owns only its bookkeeping, a device copy of the similarity tables,
 * a few hundred KB of device scratch and its events.
 *
 * A handle is not thread-safe.  Work is enqueued on the caller's compute
 * stream; moe_decode_layer returns once the routing decision of this call has
 * reached the host (it waits for the router kernel only, the FFN kernels are
 * still in flight); with cpu_assist it also stays until the host cores have
 * computed the experts Algorithm 2 left to them.  Calls on one handle that
 * overlap race on its scratch.
 */
#ifndef SMOE_H_
#define SMOE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SMOE_MAX_EXPERTS 64   /* routed experts per layer: residency is one 64-bit mask */
#define SMOE_MAX_TOPK     8
#define SMOE_MAX_BATCH    8
#define SMOE_MAX_SHARED   4
#define SMOE_MAX_HIDDEN   8192

#define SMOE_OK         0
#define SMOE_EINVAL    -1   /* bad argument, shape or layout */
#define SMOE_EHIP      -2   /* a HIP runtime call failed: see moe_last_hip_error() */
#define SMOE_ENOTPINNED -3  /* an experts_host block is not pinned host memory */
#define SMOE_ESTATE    -4   /* call not valid in the handle's state */
#define SMOE_ETOOBIG   -5   /* the configuration needs more scratch than SMOE_STATIC_SCRATCH_BYTES */

/* Size of the per-GPU scratch array behind moe_decode_layer_static. */
#define SMOE_STATIC_SCRATCH_BYTES (8u << 20)

#define SMOE_DTYPE_FP32 0
#define SMOE_DTYPE_BF16 1

/* Replacement policies.  SCORE is the paper's (Eq. 3: lowest mean gate score over
 * the last n+1 steps); the others are the recency / frequency baselines its
 * ablation compares against (Section VI-C, "+CE" step).  Every policy skips the
 * experts the current step computes (protection shield) and breaks ties towards
 * the lower expert id.  A "use" is one (token, slot) of a step computing the
 * expert; uses and loads are stamped step * 64 + token * k + slot. */
#define SMOE_EVICT_SCORE 0
#define SMOE_EVICT_LRU   1   /* least recently used                                  */
#define SMOE_EVICT_FIFO  2   /* earliest loaded (initial residents: in slot order)   */
#define SMOE_EVICT_LFU   3   /* fewest uses since it was loaded, then least recent   */

typedef struct moe_handle moe_handle_t;   /* opaque, library-owned */

typedef struct {
  int32_t n_layers;      /* L                                                        */
  int32_t hidden;        /* H, multiple of 8, <= SMOE_MAX_HIDDEN                     */
  int32_t n_experts;     /* E routed experts per layer, <= SMOE_MAX_EXPERTS          */
  int32_t ffn;           /* F of a routed expert, multiple of 8                      */
  int32_t top_k;         /* k, 1 <= k <= min(E, SMOE_MAX_TOPK)                       */
  int32_t cache_cap;     /* experts resident in HBM per layer, k <= cap <= E         */
  int32_t n_shared;      /* always-resident shared experts per layer (weight 1)      */
  int32_t shared_ffn;    /* F of one shared expert, multiple of 8 (0 if none)        */
  int32_t dtype;         /* SMOE_DTYPE_*: type of weights, x and y                   */
  int32_t max_batch;     /* 1..SMOE_MAX_BATCH tokens per call                        */
  float   alpha;         /* substitution threshold of Algorithm 1; 0 disables it     */
  int32_t subst_key;     /* ranking of eligible substitutes: 0 = similarity-table
                            row of the replaced expert, 1 = gate score (Section IV-B) */
  int32_t renorm_topk;   /* 1: combine weights divided by the sum of the k selected
                            scores; 0: raw softmax scores                            */
  int32_t evict_window;  /* n of Eq. 3: the mean runs over the last n+1 steps        */
  int32_t n_stage;       /* transient slots after the L*cap cache slots, used when a
                            missing expert finds no evictable resident (batch > 1)   */
  int32_t evict_policy;  /* SMOE_EVICT_*: which unshielded resident a load replaces   */
  int32_t prefetch_max;  /* prefetched experts a layer may hold at a time (= spare slots
                            per layer; 0: prefetch is off and the call is refused), < 64 */
  int32_t cpu_assist;    /* 1: CPU-assisted task load scheduling (Section V-A): the
                            missing experts of a step are split by Algorithm 2 between
                            the load queue (highest scores, cached) and the host cores
                            (lowest scores, computed from the host copy, not cached).
                            0 (default): every miss is loaded, nothing of the method
                            runs on the CPU.  2: variant of this library -- the split
                            that minimises max(n_load C_load, n_CPU C_CPU) outright
                            (Section V-A's objective) instead of the two-pointer walk,
                            which always loads the first expert; of equal splits the
                            one that loads more                                       */
  int32_t cpu_threads;   /* host threads of the expert FFN, the caller's included;
                            0 = min(16, hardware threads)                             */
  float   load_cost_us;  /* C_load of Algorithm 2 in microseconds; <= 0: measured (mean
                            duration of the last 8 expert copies)                     */
  float   cpu_cost_us;   /* C_CPU of Algorithm 2; <= 0: measured (mean wall time of the
                            last 8 host-computed experts)                             */
  int32_t auto_prefetch; /* 1 (needs prefetch_max > 0): every moe_decode_layer of a layer
                            l < L-1 predicts the input of layer l+1 from its own partial
                            output -- the resident and shared experts' result, before
                            the loaded experts are done (Section IV-C, Fig. "prefetch")
                            -- as (x + partial) / rms(x + partial), runs layer l+1's gate
                            on it and prefetches for layer l+1 exactly as a
                            moe_prefetch_layer call with that state would; the decision
                            is taken when layer l+1 is decoded.  0: predictions come
                            from the caller through moe_prefetch_layer only           */
  int32_t prefetch_yield;/* 1: a prediction is skipped when, at the moment it would be
                            launched, copies of earlier calls (on-demand loads or
                            prefetches) are still on the host link: with the link as
                            the bottleneck a prefetch cannot arrive early and every
                            misprediction costs link time.  Such a call is reported by
                            moe_prefetch_last with yielded = 1 and prefetches nothing.
                            0: every prediction is taken (the paper's behaviour)       */
} moe_cfg_t;

typedef struct {
  const void*    gate_w_dev;      /* device  [L][E][H] dtype, row e = expert e                */
  const void* const* experts_host; /* host array of L pointers; entry l -> pinned host
                                     [E]{W1[F][H], W3[F][H], W2[H][F]} dtype of layer l:
                                     W1 gate-projection, W3 up-projection, W2 down-projection,
                                     each row-major, the three back to back.  The array itself
                                     is copied at init; the blocks it points to are borrowed  */
  const void*    shared_dev;      /* device  [L][n_shared]{W1[Fs][H], W3[Fs][H], W2[H][Fs]}
                                     or NULL when n_shared == 0                               */
  const float*   sim_host;        /* host    [L][E][E] fp32 similarity table, copied at init  */
  void*          cache_slab_dev;  /* device  (L*(cache_cap + prefetch_max) + n_stage) slots of
                                     3*H*F*sizeof(dtype) bytes: layer l owns the slots from
                                     l*(cache_cap + prefetch_max) on (its cache plus the spare
                                     slots prefetched experts are loaded into), the staging
                                     slots follow; 256-byte aligned; contents overwritten      */
  const int32_t* init_resident;   /* host    [L][cache_cap] distinct expert ids, or NULL for
                                     experts 0..cap-1 in every layer                          */
  void*          stream_compute;  /* hipStream_t all kernels run on                           */
  void*          stream_copy;     /* hipStream_t the expert loads run on (must differ)        */
} moe_buffers_t;

/* Optional per-call trace, host memory owned by the caller, every pointer may be NULL. */
typedef struct {
  int32_t* topk_idx;     /* [B][k]  experts selected by the router, by descending score   */
  int32_t* final_idx;    /* [B][k]  expert each slot computes after substitution          */
  uint8_t* substituted;  /* [B][k]  1 where final_idx differs from topk_idx                */
  uint8_t* hit;          /* [B][k]  1 where the slot was served without a load            */
  float*   scores;       /* [B][E]  gate scores                                           */
  float*   weights;      /* [B][k]  combine weight of each slot                           */
  int32_t* fetched;      /* [B*k]   distinct experts loaded by this call, in load order,
                                    -1 padded                                             */
  int32_t* victims;      /* [B*k]   expert evicted for each load, -1 = staged / padding   */
  int32_t* on_cpu;       /* [B*k]   experts computed by the host cores (cpu_assist): missing
                                    ones and prefetched ones still in flight, in list
                                    order, -1 padded                                      */
  int32_t* adopted;      /* [B*k]   prefetched experts this call computed and took into the
                                    cache, in (token, slot) order, -1 padded              */
  int32_t* adopt_victims;/* [B*k]   expert evicted for each (-1: none evictable, computed
                                    where it was loaded and not kept)                     */
  int32_t  n_fetched;    /* out: number of loads issued by this call                      */
  int32_t  n_on_cpu;     /* out: number of experts left to the host cores                 */
  int32_t  n_adopted;    /* out: number of prefetched experts taken into the cache        */
  int32_t  pad_;
  uint64_t inflight_mask;/* out: bit e = expert e was prefetched for this call, is computed
                                    by it, and its copy had not finished when the call was
                                    decided (a fact of the machine: with cpu_assist it
                                    decides whether Algorithm 2 considers the expert)     */
} moe_trace_t;

typedef struct {
  int64_t tokens;         /* tokens decoded (per layer: calls * batch)                     */
  int64_t slots;          /* tokens * k                                                    */
  int64_t raw_hits;       /* sum |G n E_a|: router choices already resident               */
  int64_t hits;           /* slots served without a load, after substitution (Eq. 1)      */
  int64_t misses;         /* slots - hits                                                  */
  int64_t substitutions;  /* slots whose expert was replaced                               */
  int64_t evictions;      /* residents replaced by a loaded expert                         */
  int64_t staged;         /* loads computed from a transient slot, not inserted            */
  int64_t fetches;        /* expert loads issued                                           */
  int64_t bytes_fetched;  /* fetches * expert bytes                                        */
  int64_t prefetches;     /* experts loaded ahead of time by moe_prefetch_layer (each also
                             counts as an eviction, none as a fetch)                       */
  int64_t prefetch_used;  /* ... that the layer's next step computed                       */
  int64_t prefetch_top;   /* ... that were top-score experts (s >= T) of that step         */
  int64_t cpu_computed;   /* missing experts computed by the host cores instead of loaded  */
} moe_stats_t;

/* What the most recent prefetch did (moe_prefetch_last). */
typedef struct {
  int32_t layer;                                       /* -1: no prefetch so far           */
  int32_t n_wanted;                                    /* predicted top-score experts that
                                                          were neither resident nor already
                                                          prefetched                       */
  int32_t n_loaded;                                    /* how many of them were put on the
                                                          load queue (a prefix of wanted)  */
  int32_t wanted[SMOE_MAX_BATCH * SMOE_MAX_TOPK];      /* in load order                    */
  int32_t yielded;                                     /* 1: skipped because the link was busy
                                                          (cfg.prefetch_yield)             */
  int64_t bytes_copied;                                /* prefetch bytes handed to the copy
                                                          stream since init / reset        */
  int64_t bytes_withdrawn;                             /* bytes of dropped prefetches that
                                                          were never copied                */
} moe_prefetch_info_t;

/* In-stream duration of the launches, measured with HIP events recorded on the
 * launching stream around every launch while profiling is enabled.  Kinds:
 * the router kernel; the up / down FFN kernels of the resident pass; the host
 * to HBM expert copies; the up / down kernels of the pass over loaded experts.
 * bytes = algorithmic bytes those launches had to move (gate matrix; expert
 * weights streamed once; expert bytes copied). */
#define SMOE_PROF_ROUTE       0
#define SMOE_PROF_UP          1
#define SMOE_PROF_DOWN        2
#define SMOE_PROF_COPY        3
#define SMOE_PROF_UP_LOADED   4
#define SMOE_PROF_DOWN_LOADED 5
#define SMOE_PROF_KINDS       6
typedef struct {
  int64_t launches[SMOE_PROF_KINDS];
  double  ms[SMOE_PROF_KINDS];      /* summed over the recorded launches */
  int64_t bytes[SMOE_PROF_KINDS];
} moe_profile_t;

/* Create a handle for one model: the expert scheduler of Section IV works per
 * layer and online (problem statement of Section IV-A: each layer has its own
 * router, cache set G and history; nothing is prepared offline), so a handle is
 * L independent layer caches over one HBM slab.  Validates cfg, uploads the
 * similarity tables, copies the initial residents into the slab (on
 * stream_copy, waited for) and zeroes history and statistics.  SMOE_EINVAL for shapes outside the limits above,
 * cap < k, duplicate ids in init_resident, NULL buffers or equal streams;
 * SMOE_ENOTPINNED when a block of experts_host is not pinned; SMOE_EHIP on HIP errors. */
int moe_cache_init(const moe_cfg_t* cfg, const moe_buffers_t* buf, moe_handle_t** out);

/* Decode `batch` tokens through MoE layer `layer`.
 *   x_dev  device [batch][H] dtype (read by kernels until the stream drains)
 *   y_dev  device [batch][H] dtype, overwritten with
 *          sum_j w_j FFN_{final_j}(x) + sum_shared FFN_s(x)
 * Enqueues router + substitution, the FFN over resident experts, and -- when
 * the step has misses -- victim selection, the loads on stream_copy and a
 * second FFN pass over the loaded experts.  With cfg.cpu_assist the misses are
 * first split by Algorithm 2 (Section V-A): the tail of the score-ordered list
 * is computed by the host cores while the head is loaded, and the call returns
 * when they are done.  y is complete when the compute stream has drained.
 * With a trace the call also fills it (host data only).  SMOE_ESTATE when a
 * step needs more staging slots than cfg.n_stage provides: the step is refused
 * before the cache state changes (history, residency and counters are those of
 * before the call), but its kernels were already queued, so y of this call is
 * undefined.
 * SMOE_EINVAL for a bad layer / batch or NULL x, y. */
int moe_decode_layer(moe_handle_t* h, int32_t layer, int32_t batch,
                     const void* x_dev, void* y_dev, moe_trace_t* trace_or_null);

/* moe_decode_layer for callers that must not allocate device memory at all
 * (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): same arguments, same results, but every device buffer its kernels
 * work in besides the caller's inputs and outputs -- the decision record, the
 * SwiGLU activations between the up and the down kernel, the fp32 sums carried
 * to the pass over loaded experts, the router's partial sums and counter --
 * lives in one file-scope device array of SMOE_STATIC_SCRATCH_BYTES (8 MiB) per
 * GPU, which the library's code object holds on every GPU it runs on until the
 * process ends.  The call itself allocates and frees nothing, on the device or
 * on the host.  The array's address on the handle's GPU is looked up once, in
 * moe_cache_init.
 * SMOE_ETOOBIG when the handle's configuration needs more than the array holds:
 * 9.5 KB of records + max_batch*H*4 bytes of sums + the activations, which are
 * max_batch*(k+n_shared)*max(F, Fs)*4 bytes, or at max_batch > 1 the larger of
 * that and (min(E, max_batch*k)*F + n_shared*Fs)*32 bytes (the c5-shaped
 * workload at batch 8 needs 6.1 MB).  All handles on one GPU share the array and
 * it keeps the last call's contents: what has to start at zero is cleared by the
 * call.  Two moe_decode_layer_static calls on one GPU whose kernels can run at
 * the same time (handles on different compute streams, or calls from different
 * threads) race on the array: the caller keeps them on one stream or orders the
 * streams itself.  moe_decode_layer is not affected (it has its own buffers). */
int moe_decode_layer_static(moe_handle_t* h, int32_t layer, int32_t batch,
                            const void* x_dev, void* y_dev, moe_trace_t* trace_or_null);

/* Top-score prefetch for a layer that has not run yet (Section IV-C).
 *   x_pred_dev  device [batch][H] dtype: the caller's prediction of the hidden
 *               state `layer` will see (read until the compute stream drains)
 * Enqueues the gate of `layer` on x_pred (GEMV + selection kernels, compute
 * stream) and returns at once.  The decision is taken by the next call on the
 * handle: a moe_decode_layer of ANOTHER layer first queues its own loads and
 * then takes the prefetch decision; any other call (a decode of `layer` itself,
 * stats, residency, another prefetch, reset) takes it first.  Wanted are the
 * experts the predicted scores rank in the top-k with score >= T = (1+alpha)
 * S_{k+1} that are neither resident nor already prefetched for the layer, in
 * rank order (token by token); as many of them as the layer has spare slots
 * left go onto the library's load queue (at most cfg.prefetch_max wait per
 * layer).
 * The load queue (Section IV-C: the paper's queue can be cleared of mispredicted
 * experts; Section V-B "Prefetching Experts from Layer i+1": prefetches must not
 * delay the running layer's loads).  A prefetched expert is copied into a spare
 * slot of its layer and does NOT enter the cache set until the layer's next
 * moe_decode_layer: nobody is evicted for it, the score history is not touched.
 * Its copy is fed to stream_copy in chunks, a bounded number outstanding, from
 * inside later calls on the handle (there is no background thread), so an
 * on-demand load never waits behind more than that.  At the layer's next decode
 * the waiting experts count as resident for every decision (hits, substitutes).
 * Those the step computes are finished first (the rest of their copy is handed
 * over at once), computed in the call's second pass, and enter the cache there,
 * each replacing a victim like any load; the others leave the queue and what
 * was not yet handed to the copy stream is never copied.  A wrong prediction
 * therefore costs at most the chunks already under way.
 * SMOE_EINVAL for a bad layer / batch, NULL x_pred or prefetch_max == 0. */
int moe_prefetch_layer(moe_handle_t* h, int32_t layer, int32_t batch, const void* x_pred_dev);

/* Settles a pending prefetch and reports what the latest one decided. */
int moe_prefetch_last(moe_handle_t* h, moe_prefetch_info_t* out);

/* The two costs Algorithm 2 currently works with (cpu_assist): C_load and C_CPU in
 * microseconds, fixed by cfg or measured over the last 8 copies / host-computed
 * experts; plus the wall time the host cores have spent on experts so far and the
 * number of experts they computed.  Any pointer may be NULL.  SMOE_ESTATE when
 * cpu_assist is off. */
int moe_cpu_assist_costs(const moe_handle_t* h, double* c_load_us, double* c_cpu_us,
                         double* cpu_busy_us, int64_t* cpu_experts);

/* Counters of one layer, or of all layers summed when layer == -1: the expert
 * cache hits of Eq. 1 (`hits`: slots served from the cache after substitution;
 * `raw_hits`: |G n E_a| before it) and what the paper's evaluation derives from
 * them (cache ratio = hits / slots, Section VI-A), plus loads, evictions and the
 * prefetch / CPU-assist counters.  (Takes a non-const handle since a pending
 * prefetch is settled first.) */
int moe_cache_stats(moe_handle_t* h, int32_t layer, moe_stats_t* out);

/* The cache set G of `layer` (Table "Definitions"): expert id held by each
 * cache slot, out_slots[cache_cap]. */
int moe_cache_residency(moe_handle_t* h, int32_t layer, int32_t* out_slots);

/* Back to the state after moe_cache_init (the start of a new sequence: the
 * history window of Eq. 3 and the cache contents belong to one decode stream):
 * drains both streams, reloads the initial residents, zeroes history and
 * counters. */
int moe_cache_reset(moe_handle_t* h);

/* Drain both streams and release everything the library owns. */
int moe_cache_destroy(moe_handle_t* h);

/* Per-kernel timing.  enable = bit mask of SMOE_PROF_* kinds to record with
 * event pairs (bit i = kind i; at most max_launches launches per kind are
 * recorded, later ones add neither time nor bytes; counters restart),
 * enable = 0 stops.
 * moe_profile_read drains the compute and copy streams and returns the totals
 * recorded since the last enable. */
int moe_profile_enable(moe_handle_t* h, int32_t enable, int32_t max_launches);
int moe_profile_read(moe_handle_t* h, moe_profile_t* out);

/* The substitution threshold from a latency budget (Section V-C, Eq. 5: minimise
 * the accuracy loss subject to T(alpha) <= R).  alphas / tpots: n measured pairs
 * (host arrays; TPOT in any unit, budget in the same).  A polynomial of `degree`
 * (0..6, n > degree) is fitted by least squares and the uniform grid of
 * `resolution` >= 2 points over [min alpha, max alpha] is scanned from its low
 * end; *out_alpha receives the first point whose predicted TPOT is <= budget
 * (accuracy loss grows with alpha, so this is the minimiser), out_coef[0..degree]
 * the coefficients, constant term first.  Host arithmetic only, no handle.
 * SMOE_OK; SMOE_ESTATE when no grid point meets the budget (out_coef is still
 * filled); SMOE_EINVAL for bad arguments or a singular fit. */
int moe_select_alpha(const double* alphas, const double* tpots, int32_t n, double budget,
                     int32_t degree, int32_t resolution, double* out_alpha, double* out_coef);

/* hipError_t of the most recent failing HIP call in this thread (0 if none). */
int moe_last_hip_error(void);

/* Page-locked host memory for expert storage (hipHostMalloc of exactly n_bytes;
 * PyTorch's pinned allocator rounds large requests up to a power of two).
 * moe_host_alloc stores the pointer in *out; SMOE_EHIP when the system cannot
 * pin that much.  Free with moe_host_free after the handles using it are gone. */
int moe_host_alloc(int64_t n_bytes, void** out);
int moe_host_free(void* p);

/* Plain device-to-device copy kernel (n_bytes multiple of 16, both pointers
 * 16-byte aligned) on `stream`: the known-size kernel hardware counters are
 * calibrated against.  Returns SMOE_EINVAL on misaligned arguments. */
int moe_calib_copy(void* dst_dev, const void* src_dev, int64_t n_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SMOE_H_ */
