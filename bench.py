#!/usr/bin/env python3
"""Benchmark of the SMoE offloaded-MoE decode hot path on one MI355X.

A step = one decode token through every MoE layer of the workload: router,
substitution, cache bookkeeping, on-demand loads of the misses, expert FFNs.
Inputs (weights in pinned host memory, gate / shared weights and hidden states
in HBM, initial residents in the HBM cache) are in place before the timed
region starts.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes per launch of the resident-pass up kernel / its algorithmic bytes, from the two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) summarised in profiles/c3_ffn_hbm_traffic_pmc.md
MEASURED_TRAFFIC_RATIO = {"c3-mixtral8x7b-shaped": 1.0003}


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


PROF_UP_AND_COPY = (1 << 1) | (1 << 3)
PROF_ALL = (1 << 6) - 1


def timed_run(ses, x_dev, y_dev, warmup: int, steps: int, n_layers: int, prof_launches: int,
              prof_mask: int = PROF_UP_AND_COPY, xp_dev=None):
    import paper_2508_18983_amd as M
    run_tokens(ses, x_dev, y_dev, 0, warmup, n_layers, xp_dev)
    ses.sync()
    st0 = ses.stats()
    M.moe_profile_enable(ses.handle, prof_mask, prof_launches)
    ses.sync()
    t_begin = time.perf_counter()
    run_tokens(ses, x_dev, y_dev, warmup, warmup + steps, n_layers, xp_dev)
    ses.sync()
    elapsed = time.perf_counter() - t_begin
    prof = M.moe_profile_read(ses.handle).as_dict()
    M.moe_profile_enable(ses.handle, 0, 1)
    st1 = ses.stats()
    delta = {k: st1[k] - st0[k] for k in st1}
    return elapsed, prof, delta


def cpu_baseline(wl, budget_s: float):
    """Time the CPU oracle, as it stands, on the first token's layers until
    about ``budget_s`` seconds are spent; scale to tokens/s."""
    from oracle import smoe_oracle as O
    from smoe_inputs import as_numpy
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    s = wl.shape
    orc = O.oracle_from_workload(wl, widen_cache_bytes=0)
    done = 0
    t0 = time.perf_counter()
    for l in range(s.n_layers):
        orc.decode_layer(l, as_numpy(wl.x[0, l]), compute_y=True)
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    per_token = dt / done * s.n_layers
    return {"value": 1.0 / per_token, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"token 0, layers 0..{done - 1} of {s.n_layers} ({dt:.1f} s of fp64 numpy), "
                      f"scaled to a whole token"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=96)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="c3", help="c1..c5 (default c3: Mixtral-8x7B-shaped)")
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
    from paper_2508_18983_amd.session import session_from_workload, pinned_empty
    from smoe_inputs import shape_by_name, make_workload

    M.load_library()
    shape = shape_by_name(args.workload)
    if args.cache_cap is not None:
        shape = shape.with_(cache_cap=args.cache_cap)
    if args.alpha is not None:
        shape = shape.with_(alpha=args.alpha)
    if args.evict_policy is not None:
        shape = shape.with_(evict_policy=args.evict_policy)
    n_tok = args.warmup + args.steps
    if n_tok > shape.tokens:
        print(f"bench.py: warmup+steps must be <= {shape.tokens} tokens of {shape.name}", file=sys.stderr)
        return 2
    t0 = time.perf_counter()
    log(f"drawing {shape.name}: {shape.n_layers if args.layers is None else args.layers} layers, "
        f"{n_tok} tokens ...")
    L = shape.n_layers if args.layers is None else args.layers
    block_bytes = shape.n_experts * shape.expert_bytes
    distinct = L
    while distinct > 1 and distinct * block_bytes > args.pin_budget_gb * 1e9:
        distinct = (distinct + 1) // 2
    host_note = "every layer has its own pinned host copy"
    if distinct < L:
        host_note = (f"host pins at most ~{args.pin_budget_gb:.0f} GB: {distinct} distinct layer blocks "
                     f"of expert weights, layer l reads block l mod {distinct} (same bytes copied per "
                     f"load, separate HBM cache slots, gate weights and inputs per layer)")
    Bt = args.batch
    wl = make_workload(shape, device="cuda", n_layers=args.layers, tokens=n_tok, batch=Bt,
                       host_alloc=pinned_empty, distinct_layers=distinct,
                       pred_noise=args.pred_noise if args.prefetch > 0 else None)
    s = wl.shape
    log(f"inputs ready in {time.perf_counter() - t0:.1f} s (margin audit redrew {wl.redraws} token-layers)")

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

    prof_launches = args.steps * L + 8
    with session_from_workload(wl, max_batch=Bt, n_stage=(Bt * s.top_k if Bt > 1 else 0),
                               prefetch_max=args.prefetch, cpu_assist=int(args.cpu_assist),
                               cpu_threads=args.cpu_threads) as ses:
        x_dev = wl.x.to(ses.device)[:, :, :, :].contiguous()
        xp_dev = wl.x_pred.to(ses.device).contiguous() if args.prefetch > 0 else None
        y_dev = torch.empty(L, Bt, s.hidden, dtype=ses.tdtype, device=ses.device)
        log("timed run ...")
        elapsed, prof, st = timed_run(ses, x_dev, y_dev, args.warmup, args.steps, L, prof_launches,
                                      xp_dev=xp_dev)
        cpu_costs = M.moe_cpu_assist_costs(ses.handle) if args.cpu_assist else None
        # what an event pair reads with nothing between its two records on the compute stream:
        # the part of `avg_launch_us` that is not the kernel (reported, not subtracted)
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(64)]
        ses.sync()
        for a_ev, b_ev in pairs:
            a_ev.record(ses.stream_compute)
            b_ev.record(ses.stream_compute)
        ses.sync()
        event_pair_us = sum(a_ev.elapsed_time(b_ev) for a_ev, b_ev in pairs) / len(pairs) * 1e3
    tok_s = args.steps * Bt / elapsed
    up = prof["up"]
    up_avg_s = up["ms"] / max(up["launches"], 1) * 1e-3
    up_bytes_per_launch = up["bytes"] / max(up["launches"], 1)
    achieved = up_bytes_per_launch / up_avg_s / 1e9 if up_avg_s > 0 else 0.0
    copy = prof["copy"]
    host_link = (copy["bytes"] / (copy["ms"] * 1e-3) / 1e9) if copy["ms"] > 0 else None

    extra = {
        "hit_rate_raw": st["raw_hits"] / max(st["slots"], 1),
        "hit_rate": st["hits"] / max(st["slots"], 1),
        "substitutions_per_token": st["substitutions"] / (args.steps * Bt),
        "fetches_per_step": st["fetches"] / args.steps,
        "host_link_GBs": host_link,
        "layer_bytes": s.layer_bytes(),
        "hbm_roofline_tokens_per_s": HBM_PEAK_GBS * 1e9 / (s.layer_bytes() * L),
    }
    if args.cpu_assist:
        extra["cpu_computed_per_step"] = st["cpu_computed"] / args.steps
        extra["cpu_assist_costs"] = cpu_costs
    if args.prefetch > 0:
        extra.update({
            "prefetches_per_step": st["prefetches"] / args.steps,
            "prefetch_used_frac": st["prefetch_used"] / max(st["prefetches"], 1),
            "prefetch_top_frac": st["prefetch_top"] / max(st["prefetches"], 1),
        })

    if not args.no_miss_free:
        # same tokens with every expert resident: the pure HBM path, no loads
        log("all-resident reference run ...")
        full = wl.shape.with_(cache_cap=s.n_experts)
        wl_full = type(wl)(full, wl.gate_w, wl.experts, wl.shared, wl.sim, wl.x, wl.redraws)
        try:
            with session_from_workload(wl_full, max_batch=Bt) as ses2:
                x_dev = wl.x.to(ses2.device).contiguous()
                y_dev = torch.empty(L, Bt, s.hidden, dtype=ses2.tdtype, device=ses2.device)
                e2, p2, _ = timed_run(ses2, x_dev, y_dev, min(args.warmup, 4), args.steps, L, prof_launches,
                                      prof_mask=0)
                extra["miss_free_tokens_per_s"] = args.steps * Bt / e2
                extra["miss_free_frac_of_hbm_roofline"] = (args.steps / e2) / extra["hbm_roofline_tokens_per_s"]
                # a short pass with an event pair around every launch: per-kernel durations
                n_short = min(args.steps, 16)
                _, p3, _ = timed_run(ses2, x_dev, y_dev, 0, n_short, L, n_short * L + 8, prof_mask=PROF_ALL)
            for kind in ("route", "up", "down"):
                v = p3[kind]
                if v["launches"]:
                    extra[f"miss_free_{kind}_us"] = v["ms"] * 1e3 / v["launches"]
                    extra[f"miss_free_{kind}_GBs"] = v["bytes"] / (v["ms"] * 1e-3) / 1e9
        except Exception as exc:            # e.g. not enough HBM for every expert
            extra["miss_free_error"] = repr(exc)

    if not args.no_miss_free and not args.cpu_assist and args.prefetch == 0:
        # the same tokens with the paper's CPU-assisted scheduling switched on (reported beside the
        # headline, never as `value`): Algorithm 2 as printed, and this build's min-max variant
        for mode, key in ((1, "cpu_assist_algorithm2"), (2, "cpu_assist_minmax_variant")):
            log(f"run with cpu_assist = {mode} ...")
            try:
                with session_from_workload(wl, max_batch=Bt, n_stage=(Bt * s.top_k if Bt > 1 else 0),
                                           cpu_assist=mode, cpu_threads=args.cpu_threads) as ses3:
                    x_dev = wl.x.to(ses3.device).contiguous()
                    y_dev = torch.empty(L, Bt, s.hidden, dtype=ses3.tdtype, device=ses3.device)
                    e3, _, st3 = timed_run(ses3, x_dev, y_dev, args.warmup, args.steps, L, 1, prof_mask=0)
                    costs = M.moe_cpu_assist_costs(ses3.handle)
                extra[key] = {"tokens_per_s": args.steps * Bt / e3,
                              "hit_rate": st3["hits"] / max(st3["slots"], 1),
                              "loads_per_step": st3["fetches"] / args.steps,
                              "host_computed_per_step": st3["cpu_computed"] / args.steps,
                              "c_load_us": costs["c_load_us"], "c_cpu_us": costs["c_cpu_us"]}
            except Exception as exc:
                extra[key] = {"error": repr(exc)}

    cpu = None
    if args.cpu_budget > 0:
        log("timing the CPU oracle ...")
        cpu = cpu_baseline(wl, args.cpu_budget)

    out = {
        "metric": f"decode tokens/s at batch {Bt} (full MoE stack)",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if s.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": s.name, "layers": L, "hidden": s.hidden, "experts": s.n_experts,
                   "ffn": s.ffn, "top_k": s.top_k, "cache_cap": s.cache_cap, "alpha": s.alpha,
                   "n_shared": s.n_shared, "shared_ffn": s.shared_ffn, "batch": Bt,
                   "zipf_s": s.zipf_s, "seed": s.seed, "evict_policy": s.evict_policy, "cpu_assist": int(args.cpu_assist), "prefetch_max": args.prefetch,
                   "prefetch_ahead": PREFETCH_AHEAD if args.prefetch > 0 else None,
                   "pred_noise": args.pred_noise if args.prefetch > 0 else None,
                   "host_expert_storage": host_note},
        "roofline": {"bound": "hbm", "kernel": "ffn_up_kernel (resident pass)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": (MEASURED_TRAFFIC_RATIO[s.name] * up_bytes_per_launch
                                 if s.name in MEASURED_TRAFFIC_RATIO else None),
                     "bytes_per_launch": up_bytes_per_launch, "avg_launch_us": up_avg_s * 1e6,
                     "empty_event_pair_us": event_pair_us,
                     # the same with the empty-pair reading taken off the interval: what the kernel
                     # itself takes (agrees with the rocprofv3 kernel duration)
                     "kernel_only": {"avg_us": up_avg_s * 1e6 - event_pair_us,
                                     "achieved": (up_bytes_per_launch / (up_avg_s - event_pair_us * 1e-6) / 1e9
                                                  if up_avg_s * 1e6 > event_pair_us else None),
                                     "frac": (up_bytes_per_launch / (up_avg_s - event_pair_us * 1e-6) / 1e9
                                              / HBM_PEAK_GBS if up_avg_s * 1e6 > event_pair_us else None)},
                     "launches": up["launches"]},
        "cpu_baseline": cpu,
        "extra": extra,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
