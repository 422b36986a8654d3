"""Choosing the substitution threshold alpha from a latency budget (Section V-C).

The paper minimises the accuracy loss subject to T(alpha) <= R (Eq. 5) by
fitting a low-degree polynomial to measured (alpha, TPOT) pairs and taking,
by a one-dimensional search, the smallest alpha whose predicted TPOT meets the
budget (accuracy loss grows with alpha, so the smallest feasible alpha is the
minimiser).  The arithmetic lives in the library (moe_select_alpha); this module
measures TPOT for a list of alphas (needs a GPU) and forwards the pairs.

    python -m paper_2508_18983_amd.alpha_select c3 --budget-frac 0.9
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from typing import Optional, Sequence, Tuple

import numpy as np


def select_alpha(alphas: Sequence[float], tpots: Sequence[float], budget: float, degree: int = 2,
                 resolution: int = 2001) -> Tuple[Optional[float], np.ndarray]:
    """Forwards to the library's moe_select_alpha (the fit and the scan are done
    there).  Returns (alpha or None, polynomial coefficients constant term first)."""
    from . import binding as B
    return B.moe_select_alpha(alphas, tpots, budget, degree, resolution)


def measure_tpot(name: str, alphas: Sequence[float], steps: int = 32, warmup: int = 16,
                 pin_budget_gb: float = 60.0):
    """Milliseconds per output token of the library on one workload for each alpha
    (same inputs, same initial cache; loads of missing experts included)."""
    import torch
    from smoe_inputs import shape_by_name, make_workload
    from .session import session_from_workload, pinned_empty

    shape = shape_by_name(name)
    L = shape.n_layers
    distinct = L
    while distinct > 1 and distinct * shape.n_experts * shape.expert_bytes > pin_budget_gb * 1e9:
        distinct = (distinct + 1) // 2
    wl = make_workload(shape, device="cuda", tokens=warmup + steps, host_alloc=pinned_empty,
                       distinct_layers=distinct)
    base = wl.shape
    out = []
    for a in alphas:
        wl.shape = base.with_(alpha=float(a))
        with session_from_workload(wl) as ses:
            x = wl.x.to(ses.device)
            y = torch.empty(L, 1, base.hidden, dtype=ses.tdtype, device=ses.device)
            for t in range(warmup):
                for l in range(L):
                    ses.decode(l, x[t, l], y[l])
            ses.sync()
            t0 = time.perf_counter()
            for t in range(warmup, warmup + steps):
                for l in range(L):
                    ses.decode(l, x[t, l], y[l])
            ses.sync()
            ms = (time.perf_counter() - t0) / steps * 1e3
            st = ses.stats()
        out.append(dict(alpha=float(a), tpot_ms=ms, hit_rate=st["hits"] / st["slots"]))
        print(json.dumps(out[-1]), flush=True)
    return out


def main(argv) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("workload", nargs="?", default="c3")
    ap.add_argument("--alphas", default="0,0.1,0.2,0.3,0.4,0.5,0.6")
    ap.add_argument("--budget-frac", type=float, default=0.9, help="TPOT budget as a fraction of T(0)")
    ap.add_argument("--degree", type=int, default=2)
    ap.add_argument("--steps", type=int, default=32)
    args = ap.parse_args(argv)
    alphas = [float(v) for v in args.alphas.split(",")]
    rows = measure_tpot(args.workload, alphas, steps=args.steps)
    tp = [r["tpot_ms"] for r in rows]
    budget = args.budget_frac * tp[0]
    chosen, coef = select_alpha(alphas, tp, budget, args.degree)
    print(json.dumps(dict(workload=args.workload, budget_ms=budget, chosen_alpha=chosen,
                          poly_coef_low_to_high=[float(c) for c in coef])), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
