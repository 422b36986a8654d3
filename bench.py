#!/usr/bin/env python3
"""Benchmark of the SMoE offloaded-MoE decode hot path on one MI355X.

A step = one decode token through every MoE layer of the workload: gate GEMV,
selection + substitution, cache bookkeeping, on-demand loads of the misses,
expert FFNs.  Inputs (weights in pinned host memory, gate / shared weights and
hidden states in HBM, initial residents in the HBM cache) are in place before
the timed region starts.  The timed region is repeated (default 3 times, each
exactly --steps tokens, continuing the token stream) and the median repeat is
reported.  Prints ONE JSON line.

Headline workload: c5 (Qwen2-57B-A14B-shaped), the largest of the five by bytes
per token; c3 and c4 are summarised in `extra.other_workloads`.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

# HBM bytes per launch / algorithmic bytes per launch of the resident-pass FFN kernels, from the
# two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, scaled by the 1 GiB calibration copy) that
# profiles/<workload>_ffn_hbm_traffic_pmc.md summarises.  bench.py cannot read counters itself;
# a workload without a committed summary reports traffic = null.
MEASURED_TRAFFIC_RATIO = {
    "c3-mixtral8x7b-shaped": 1.0022,       # profiles/c3_ffn_hbm_traffic_pmc.md
    "c4-dsv2lite-shaped": 1.0080,          # profiles/c4_ffn_hbm_traffic_pmc.md
    "c5-qwen2-57b-a14b-shaped": 1.0028,    # profiles/c5_ffn_hbm_traffic_pmc.md
}
# Names the profiler prints for the two resident-pass kernels at batch 1 (template arguments:
# up <type, 128-bit units of x per lane, pass, selection fused>; down <type, units per lane,
# rows per buffer, waves per block, pass>).
KERNEL_NAMES = {
    "c3-mixtral8x7b-shaped": ("ffn_up_reg_kernel<bf16_t, 8, 0, true>", "ffn_down_reg_kernel<bf16_t, 8, 1, 8, 0>"),
    "c4-dsv2lite-shaped": ("ffn_up_reg_kernel<bf16_t, 4, 0, true>", "ffn_down_reg_kernel<bf16_t, 4, 2, 8, 0>"),
    "c5-qwen2-57b-a14b-shaped": ("ffn_up_reg_kernel<bf16_t, 8, 0, true>", "ffn_down_reg_kernel<bf16_t, 6, 2, 8, 0>"),
}


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


PREFETCH_AHEAD = 1      # layer calls between a prefetch and the layer it is for (--prefetch-ahead)


def run_tokens(ses, x_dev, y_dev, t0: int, t1: int, n_layers: int, xp_dev=None) -> None:
    """Tokens t0..t1-1 through all layers.  With predicted states ``xp_dev`` every
    layer call is preceded by the top-score prefetch for the layer that runs
    PREFETCH_AHEAD calls later (1 = the next layer, as in the paper)."""
    n_tok = x_dev.shape[0]
    for t in range(t0, t1):
        for l in range(n_layers):
            if xp_dev is not None:
                tn, ln = divmod(t * n_layers + l + PREFETCH_AHEAD, n_layers)
                if tn < n_tok:
                    ses.prefetch(ln, xp_dev[tn, ln])
            ses.decode(l, x_dev[t, l], y_dev[l])


def run_tokens_chained(ses, x_dev, y_dev, t0: int, t1: int, n_layers: int) -> None:
    """Chained input mode: layer 0 of a token takes the workload's input, layer
    l+1 the RMS-normalised x_l + y_l (the stand-in for the blocks between two
    MoE layers, a few torch kernels on the library's compute stream).  With
    cfg.auto_prefetch the library predicts that state itself, from the partial
    output, while the layer's loads are still in flight (Section IV-C)."""
    import torch
    from smoe_inputs import chain_next_input
    with torch.cuda.stream(ses.stream_compute):
        for t in range(t0, t1):
            x = x_dev[t, 0]
            for l in range(n_layers):
                ses.decode(l, x, y_dev[l])
                x = chain_next_input(x, y_dev[l]).to(x_dev.dtype)


def predictor_reading(wl, Bt: int, L: int, warmup: int, steps: int, prefetch_max: int) -> dict:
    """Chained inputs, once without prefetch and once with the library's own
    predictor; the prefetch counters over the timed tokens next to the accuracy
    the paper reports for its predictor (Section VI-C)."""
    import torch
    from paper_2508_18983_amd.session import session_from_workload
    s = wl.shape
    out = {"inputs": "chained (layer l+1 input = RMS-normalised x_l + y_l)", "prefetch_max": prefetch_max,
           "paper_top_score_accuracy": 0.82, "paper_active_accuracy": 0.95}
    for key, auto, yld in (("off", 0, 0), ("own_predictor", 1, 0), ("own_predictor_yielding_to_a_busy_link", 1, 1)):
        with session_from_workload(wl, max_batch=Bt, n_stage=(Bt * s.top_k if Bt > 1 else 0),
                                   prefetch_max=prefetch_max if auto else 0, auto_prefetch=auto,
                                   prefetch_yield=yld) as ses:
            x_dev = wl.x.to(ses.device).contiguous()
            y_dev = torch.empty(L, Bt, s.hidden, dtype=ses.tdtype, device=ses.device)
            run_tokens_chained(ses, x_dev, y_dev, 0, warmup, L)
            ses.sync()
            st0 = ses.stats()
            t_begin = time.perf_counter()
            run_tokens_chained(ses, x_dev, y_dev, warmup, warmup + steps, L)
            ses.sync()
            dt = time.perf_counter() - t_begin
            st1 = ses.stats()
        st = {k: st1[k] - st0[k] for k in st1}
        r = {"tokens_per_s": steps * Bt / dt, "hit_rate": st["hits"] / max(st["slots"], 1),
             "loads_per_step": st["fetches"] / steps}
        if auto:
            r.update(prefetches_per_step=st["prefetches"] / steps,
                     prefetched_and_computed_frac=st["prefetch_used"] / max(st["prefetches"], 1),
                     prefetched_and_top_score_frac=st["prefetch_top"] / max(st["prefetches"], 1))
        out[key] = r
    return out


PROF_RESIDENT_AND_COPY = (1 << 1) | (1 << 2) | (1 << 3)      # up, down (resident pass), copies
PROF_ALL = (1 << 6) - 1


def timed_repeats(ses, x_dev, y_dev, warmup: int, steps: int, repeats: int, n_layers: int,
                  prof_mask: int = PROF_RESIDENT_AND_COPY, xp_dev=None):
    """`warmup` untimed tokens, then `repeats` timed regions of exactly `steps`
    tokens each, every one bracketed by a drain of both streams.  Returns the
    per-repeat wall times, the event profile and the counter deltas over all
    repeats."""
    import paper_2508_18983_amd as M
    run_tokens(ses, x_dev, y_dev, 0, warmup, n_layers, xp_dev)
    ses.sync()
    st0 = ses.stats()
    M.moe_profile_enable(ses.handle, prof_mask, repeats * steps * n_layers + 8)
    times = []
    for r in range(repeats):
        ses.sync()
        t_begin = time.perf_counter()
        run_tokens(ses, x_dev, y_dev, warmup + r * steps, warmup + (r + 1) * steps, n_layers, xp_dev)
        ses.sync()
        times.append(time.perf_counter() - t_begin)
    prof = M.moe_profile_read(ses.handle).as_dict()
    M.moe_profile_enable(ses.handle, 0, 1)
    st1 = ses.stats()
    delta = {k: st1[k] - st0[k] for k in st1}
    return times, prof, delta


def host_cores() -> int:
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def cpu_baseline(wl, budget_s: float):
    """The CPU oracle as it stands, timed on the first token's layers: once with
    its numerical library held to one thread, once with the cores this process
    may use (each for about half of ``budget_s``); scaled to tokens/s."""
    from oracle import smoe_oracle as O
    from smoe_inputs import as_numpy
    try:
        from threadpoolctl import threadpool_limits
    except Exception:
        threadpool_limits = None
    s = wl.shape
    cores = host_cores()

    def reading(n_threads, budget):
        orc = O.oracle_from_workload(wl, widen_cache_bytes=0)
        done = 0
        t0 = time.perf_counter()
        for l in range(s.n_layers):
            orc.decode_layer(l, as_numpy(wl.x[0, l]), compute_y=True)
            done += 1
            if time.perf_counter() - t0 > budget:
                break
        dt = time.perf_counter() - t0
        return 1.0 / (dt / done * s.n_layers), done, dt

    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            v1, n1, d1 = reading(1, budget_s / 2)
        with threadpool_limits(limits=cores):
            vall, nall, dall = reading(cores, budget_s / 2)
        used = cores
    else:
        v1 = n1 = d1 = None
        vall, nall, dall = reading(None, budget_s)
        used = 1
    return {"value": vall, "unit": "tokens/s", "cores": int(used), "kind": "oracle",
            "sample": f"token 0, layers 0..{nall - 1} of {s.n_layers} ({dall:.1f} s of fp64 numpy on "
                      f"{used} threads), scaled to a whole token",
            "single_thread": None if v1 is None else {
                "value": v1, "cores": 1,
                "sample": f"token 0, layers 0..{n1 - 1} of {s.n_layers} ({d1:.1f} s)"},
            "host_cores_visible": cores}


def kernel_block(prof_kind: dict, name: str, event_pair_us: float) -> dict:
    n = max(prof_kind["launches"], 1)
    avg_s = prof_kind["ms"] / n * 1e-3
    bpl = prof_kind["bytes"] / n
    ach = bpl / avg_s / 1e9 if avg_s > 0 else 0.0
    only = avg_s - event_pair_us * 1e-6
    return {"kernel": name, "launches": prof_kind["launches"], "bytes_per_launch": bpl,
            "avg_launch_us": avg_s * 1e6, "achieved": ach, "frac": ach / HBM_PEAK_GBS,
            # the event interval with the reading of an empty event pair taken off: brackets the
            # rocprofv3 kernel duration from the other side
            "kernel_only_us": only * 1e6 if only > 0 else None,
            "kernel_only_frac": (bpl / only / 1e9 / HBM_PEAK_GBS) if only > 0 else None}


def empty_event_pair_us(ses) -> float:
    """What an event pair reads with nothing between its two records on the
    compute stream: the part of an event interval that is not the kernel."""
    import torch
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(64)]
    ses.sync()
    for a_ev, b_ev in pairs:
        a_ev.record(ses.stream_compute)
        b_ev.record(ses.stream_compute)
    ses.sync()
    return sum(a_ev.elapsed_time(b_ev) for a_ev, b_ev in pairs) / len(pairs) * 1e3


def measure(args, workload: str, steps: int, warmup: int, repeats: int, headline: bool):
    """One workload: the run with misses served (the `value`), the resident-path
    roofline from it, and the all-resident reference run.  Returns a dict."""
    import torch
    import paper_2508_18983_amd as M
    from paper_2508_18983_amd.session import session_from_workload, pinned_empty, pinned_free_all
    from smoe_inputs import shape_by_name, make_workload

    shape = shape_by_name(workload)
    if headline:
        if args.cache_cap is not None:
            shape = shape.with_(cache_cap=args.cache_cap)
        if args.alpha is not None:
            shape = shape.with_(alpha=args.alpha)
        if args.evict_policy is not None:
            shape = shape.with_(evict_policy=args.evict_policy)
    Bt = args.batch if headline else 1
    prefetch = args.prefetch if headline else 0
    cpu_assist = int(args.cpu_assist) if headline else 0
    while repeats > 1 and warmup + repeats * steps > shape.tokens:
        repeats -= 1
    n_tok = warmup + repeats * steps
    if n_tok > shape.tokens:
        raise SystemExit(f"bench.py: warmup+steps must be <= {shape.tokens} tokens of {shape.name}")
    L = shape.n_layers if (args.layers is None or not headline) else args.layers
    t0 = time.perf_counter()
    log(f"drawing {shape.name}: {L} layers, {n_tok} tokens ...")
    block_bytes = shape.n_experts * shape.expert_bytes
    distinct = L
    while distinct > 1 and distinct * block_bytes > args.pin_budget_gb * 1e9:
        distinct = (distinct + 1) // 2
    host_note = "every layer has its own pinned host copy"
    if distinct < L:
        host_note = (f"host pins at most ~{args.pin_budget_gb:.0f} GB: {distinct} distinct layer blocks "
                     f"of expert weights, layer l reads block l mod {distinct} (same bytes copied per "
                     f"load, separate HBM cache slots, gate weights and inputs per layer)")
    wl = make_workload(shape, device="cuda", n_layers=L, tokens=n_tok, batch=Bt,
                       host_alloc=pinned_empty, distinct_layers=distinct,
                       pred_noise=args.pred_noise if prefetch > 0 else None)
    s = wl.shape
    log(f"inputs ready in {time.perf_counter() - t0:.1f} s (margin audit redrew {wl.redraws} token-layers)")
    out = {"shape": s, "L": L, "Bt": Bt, "host_note": host_note, "repeats": repeats}
    try:
        with session_from_workload(wl, max_batch=Bt, n_stage=(Bt * s.top_k if Bt > 1 else 0),
                                   prefetch_max=prefetch, cpu_assist=cpu_assist,
                                   prefetch_yield=int(args.prefetch_yield and prefetch > 0),
                                   cpu_threads=args.cpu_threads) as ses:
            x_dev = wl.x.to(ses.device).contiguous()
            xp_dev = wl.x_pred.to(ses.device).contiguous() if prefetch > 0 else None
            y_dev = torch.empty(L, Bt, s.hidden, dtype=ses.tdtype, device=ses.device)
            log("timed run ...")
            times, prof, st = timed_repeats(ses, x_dev, y_dev, warmup, steps, repeats, L, xp_dev=xp_dev)
            out["cpu_costs"] = M.moe_cpu_assist_costs(ses.handle) if cpu_assist else None
            out["event_pair_us"] = empty_event_pair_us(ses)
        out.update(times=times, prof=prof, st=st)
        extra = {}
        if not args.no_miss_free:
            # same tokens with every expert resident: the pure HBM path, no loads
            log("all-resident reference run ...")
            full = wl.shape.with_(cache_cap=s.n_experts)
            wl_full = type(wl)(full, wl.gate_w, wl.experts, wl.shared, wl.sim, wl.x, wl.redraws)
            try:
                with session_from_workload(wl_full, max_batch=Bt) as ses2:
                    x_dev = wl.x.to(ses2.device).contiguous()
                    y_dev = torch.empty(L, Bt, s.hidden, dtype=ses2.tdtype, device=ses2.device)
                    t2, _, _ = timed_repeats(ses2, x_dev, y_dev, min(warmup, 4), steps, repeats, L, prof_mask=0)
                    e2 = statistics.median(t2)
                    roof = HBM_PEAK_GBS * 1e9 / (s.layer_bytes() * L)
                    extra["miss_free_tokens_per_s"] = steps * Bt / e2
                    extra["miss_free_frac_of_hbm_roofline"] = (steps / e2) / roof
                    extra["miss_free_us_per_layer"] = e2 / (steps * L) * 1e6
                    # a short pass with an event pair around every launch: per-kernel durations
                    n_short = min(steps, 16)
                    _, p3, _ = timed_repeats(ses2, x_dev, y_dev, 0, n_short, 1, L, prof_mask=PROF_ALL)
                for kind in ("route", "up", "down"):
                    v = p3[kind]
                    if v["launches"]:
                        extra[f"miss_free_{kind}_us"] = v["ms"] * 1e3 / v["launches"]
                        extra[f"miss_free_{kind}_GBs"] = v["bytes"] / (v["ms"] * 1e-3) / 1e9
            except Exception as exc:            # e.g. not enough HBM for every expert
                extra["miss_free_error"] = repr(exc)
        if headline and not args.no_miss_free and not cpu_assist and prefetch == 0:
            # the same tokens with the paper's CPU-assisted scheduling switched on (reported beside
            # the headline, never as `value`): Algorithm 2 as printed, and this build's min-max variant
            for mode, key in ((1, "cpu_assist_algorithm2"), (2, "cpu_assist_minmax_variant")):
                log(f"run with cpu_assist = {mode} ...")
                try:
                    with session_from_workload(wl, max_batch=Bt, n_stage=(Bt * s.top_k if Bt > 1 else 0),
                                               cpu_assist=mode, cpu_threads=args.cpu_threads) as ses3:
                        x_dev = wl.x.to(ses3.device).contiguous()
                        y_dev = torch.empty(L, Bt, s.hidden, dtype=ses3.tdtype, device=ses3.device)
                        t3, _, st3 = timed_repeats(ses3, x_dev, y_dev, warmup, steps, 1, L, prof_mask=0)
                        costs = M.moe_cpu_assist_costs(ses3.handle)
                    extra[key] = {"tokens_per_s": steps * Bt / t3[0],
                                  "hit_rate": st3["hits"] / max(st3["slots"], 1),
                                  "loads_per_step": st3["fetches"] / steps,
                                  "host_computed_per_step": st3["cpu_computed"] / steps,
                                  "c_load_us": costs["c_load_us"], "c_cpu_us": costs["c_cpu_us"]}
                except Exception as exc:
                    extra[key] = {"error": repr(exc)}
        if headline and args.predictor > 0 and not cpu_assist and prefetch == 0:
            log("chained inputs, the library's own predictor ...")
            try:
                torch.cuda.empty_cache()
                extra["predictor_chained_inputs"] = predictor_reading(wl, Bt, L, min(warmup, 16), min(steps, 32),
                                                                      args.predictor)
            except Exception as exc:
                extra["predictor_chained_inputs"] = {"error": repr(exc)}
        out["extra"] = extra
        if headline and args.cpu_budget > 0:
            log("timing the CPU oracle ...")
            out["cpu"] = cpu_baseline(wl, args.cpu_budget)
    finally:
        del wl
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        pinned_free_all()
    return out


def summarise(m: dict, steps: int) -> dict:
    """Common figures of one measured workload."""
    s, L, Bt = m["shape"], m["L"], m["Bt"]
    elapsed = statistics.median(m["times"])
    st, prof = m["st"], m["prof"]
    n_steps = steps * len(m["times"])
    names = KERNEL_NAMES.get(s.name, ("ffn_up kernel (resident pass)", "ffn_down kernel (resident pass)"))
    if Bt > 1:      # batched steps run the grouped kernels (bf16: on the matrix cores)
        names = (("ffn_up_mfma_kernel<0>", "ffn_down_mfma_kernel<0>") if s.dtype == "bf16"
                 else ("ffn_up_grp_kernel<float, 0>", "ffn_down_grp_kernel<float, 0>"))
    up = kernel_block(prof["up"], names[0], m["event_pair_us"])
    down = kernel_block(prof["down"], names[1], m["event_pair_us"])
    both_bytes = up["bytes_per_launch"] + down["bytes_per_launch"]
    both_s = (up["avg_launch_us"] + down["avg_launch_us"]) * 1e-6
    copy = prof["copy"]
    res = {
        "tokens_per_s": steps * Bt / elapsed,
        "ms_per_step": elapsed / steps * 1e3,
        "ms_per_step_repeats": [t / steps * 1e3 for t in m["times"]],
        "hit_rate_raw": st["raw_hits"] / max(st["slots"], 1),
        "hit_rate": st["hits"] / max(st["slots"], 1),
        "substitutions_per_token": st["substitutions"] / (n_steps * Bt),
        "fetches_per_step": st["fetches"] / n_steps,
        "host_link_GBs": (copy["bytes"] / (copy["ms"] * 1e-3) / 1e9) if copy["ms"] > 0 else None,
        "layer_bytes": s.layer_bytes(),
        "hbm_roofline_tokens_per_s": HBM_PEAK_GBS * 1e9 / (s.layer_bytes() * L),
        "resident_path": {"achieved": both_bytes / both_s / 1e9 if both_s > 0 else 0.0,
                          "bytes_per_launch_pair": both_bytes, "us_per_launch_pair": both_s * 1e6},
        "up": up, "down": down,
    }
    res["resident_path"]["frac"] = res["resident_path"]["achieved"] / HBM_PEAK_GBS
    res.update(m.get("extra", {}))
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--repeats", type=int, default=3, help="timed regions of --steps tokens each; the median is reported")
    ap.add_argument("--workload", default="c5", help="c1..c5 (default c5: Qwen2-57B-A14B-shaped, the largest)")
    ap.add_argument("--others", default="c3,c4",
                    help="workloads summarised in extra.other_workloads (comma list, '' = none)")
    ap.add_argument("--layers", type=int, default=None, help="override layer count (diagnostic only)")
    ap.add_argument("--batch", type=int, default=1, help="tokens per decode step (the headline metric is batch 1)")
    ap.add_argument("--cpu-budget", type=float, default=20.0, help="seconds of oracle timing; 0 = skip")
    ap.add_argument("--no-miss-free", action="store_true", help="skip the all-resident reference run")
    ap.add_argument("--calib-copies", type=int, default=3,
                    help="launches of the known-size (1 GiB) copy kernel that hardware counters are scaled by")
    ap.add_argument("--alpha", type=float, default=None,
                    help="override the substitution threshold (diagnostic only; 0 = no substitution)")
    ap.add_argument("--evict-policy", type=int, default=None,
                    help="override the replacement policy: 0 score (Eq. 3), 1 LRU, 2 FIFO, 3 LFU (diagnostic only)")
    ap.add_argument("--cache-cap", type=int, default=None,
                    help="override the workload's HBM cache capacity per layer (diagnostic only)")
    ap.add_argument("--prefetch", type=int, default=0,
                    help="experts a top-score prefetch may load per layer (0 = off, the headline setting)")
    ap.add_argument("--predictor", type=int, default=2,
                    help="experts per layer the library's own predictor may prefetch in the extra chained-input "
                         "reading (extra.predictor_chained_inputs; 0 = skip that reading)")
    ap.add_argument("--prefetch-yield", type=int, default=0,
                    help="1: predictions are skipped while earlier copies are still on the host link")
    ap.add_argument("--cpu-assist", type=int, nargs="?", const=1, default=0,
                    help="CPU-assisted task load scheduling with measured costs: part of the misses is computed "
                         "by the host cores instead of being loaded.  1 = Algorithm 2, 2 = min-max split "
                         "(variant); 0 = off, the headline setting")
    ap.add_argument("--cpu-threads", type=int, default=0, help="host threads of the expert FFN (0 = up to 16)")
    ap.add_argument("--prefetch-ahead", type=int, default=1,
                    help="how many layer calls ahead of its layer a prefetch is issued (paper: 1)")
    ap.add_argument("--pred-noise", type=float, default=0.3,
                    help="std of the noise that turns a hidden state into the prefetcher's predicted state")
    ap.add_argument("--pin-budget-gb", type=float, default=60.0,
                    help="page-locked host memory the box lets one process hold for expert storage")
    args = ap.parse_args()
    global PREFETCH_AHEAD
    PREFETCH_AHEAD = max(1, args.prefetch_ahead)
    if args.gpus != 1:
        print("bench.py: this build is a one-GPU path (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    import paper_2508_18983_amd as M
    M.load_library()

    if args.calib_copies > 0:
        # known-size traffic for counter calibration: 1 GiB read + 1 GiB written per launch
        n_cal = 1 << 30
        src = torch.ones(n_cal, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(args.calib_copies):
            M.moe_calib_copy(dst.data_ptr(), src.data_ptr(), n_cal, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    m = measure(args, args.workload, args.steps, args.warmup, max(1, args.repeats), headline=True)
    s, L, Bt = m["shape"], m["L"], m["Bt"]
    res = summarise(m, args.steps)
    up, down = res.pop("up"), res.pop("down")
    rp = res.pop("resident_path")
    extra = {k: v for k, v in res.items() if k not in ("tokens_per_s", "ms_per_step")}
    if args.cpu_assist:
        extra["cpu_computed_per_step"] = m["st"]["cpu_computed"] / (args.steps * len(m["times"]))
        extra["cpu_assist_costs"] = m["cpu_costs"]
    if args.prefetch > 0:
        st = m["st"]
        extra.update({
            "prefetches_per_step": st["prefetches"] / (args.steps * len(m["times"])),
            "prefetch_used_frac": st["prefetch_used"] / max(st["prefetches"], 1),
            "prefetch_top_frac": st["prefetch_top"] / max(st["prefetches"], 1),
        })

    others = {}
    for name in [w for w in args.others.split(",") if w and w != args.workload and Bt == 1]:
        try:
            log(f"---- {name} (summary) ----")
            mo = measure(args, name, min(args.steps, 24), min(args.warmup, 16), 1, headline=False)
            so = summarise(mo, min(args.steps, 24))
            o_up, o_down, o_rp = so.pop("up"), so.pop("down"), so.pop("resident_path")
            so.update(resident_path_GBs=o_rp["achieved"], resident_path_frac=o_rp["frac"],
                      up_kernel=o_up["kernel"], up_GBs=o_up["achieved"], up_avg_launch_us=o_up["avg_launch_us"],
                      down_kernel=o_down["kernel"], down_GBs=o_down["achieved"],
                      down_avg_launch_us=o_down["avg_launch_us"], host_expert_storage=mo["host_note"])
            others[mo["shape"].name] = so
        except Exception as exc:
            others[name] = {"error": repr(exc)}
    if others:
        extra["other_workloads"] = others

    ratio = MEASURED_TRAFFIC_RATIO.get(s.name) if Bt == 1 else None      # counters were read at batch 1
    out = {
        "metric": f"decode tokens/s at batch {Bt} (full MoE stack)",
        "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if s.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": s.name, "layers": L, "hidden": s.hidden, "experts": s.n_experts,
                   "ffn": s.ffn, "top_k": s.top_k, "cache_cap": s.cache_cap, "alpha": s.alpha,
                   "n_shared": s.n_shared, "shared_ffn": s.shared_ffn, "batch": Bt,
                   "zipf_s": s.zipf_s, "seed": s.seed, "evict_policy": s.evict_policy,
                   "cpu_assist": int(args.cpu_assist), "prefetch_max": args.prefetch,
                   "prefetch_ahead": PREFETCH_AHEAD if args.prefetch > 0 else None,
                   "prefetch_yield": args.prefetch_yield if args.prefetch > 0 else None,
                   "pred_noise": args.pred_noise if args.prefetch > 0 else None,
                   "timed_repeats": len(m["times"]), "reported": "median repeat",
                   "host_expert_storage": m["host_note"]},
        # the resident-expert FFN path = the two kernels that stream the resident and shared
        # experts' weights in every call (up: W1, W3; down: W2); the first is the dominant one
        "roofline": {"bound": "hbm",
                     "kernel": f"{up['kernel']} + {down['kernel']} (resident pass)",
                     "achieved": rp["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": rp["frac"],
                     "traffic": ratio * rp["bytes_per_launch_pair"] if ratio is not None else None,
                     "bytes_per_launch": rp["bytes_per_launch_pair"],
                     "avg_launch_us": rp["us_per_launch_pair"],
                     "empty_event_pair_us": m["event_pair_us"],
                     "kernels": [up, down]},
        "cpu_baseline": m.get("cpu"),
        "extra": extra,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
