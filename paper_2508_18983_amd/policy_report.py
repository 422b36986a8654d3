"""Hit-rate ladder of the paper's ablation on the synthetic traces (Section VI-C):
recency cache -> score-based eviction ("+CE", Eq. 3) -> expert-cache router
("+CR", Algorithm 1 substitution) -> top-score prefetch ("+Pre", Section IV-C,
from predicted states with noise 0.3) -> CPU-assisted scheduling ("+BA",
Algorithm 2 with the fixed cost ratio C_load : C_CPU = 3 : 1 of the paper's S3
remark, since measured costs mean nothing at a shrunk FFN width).  Runs the
HIP library (decisions depend only on the gate logits and the cache state, so
the expert FFN width is shrunk to keep the run short) and prints one table row
per workload and configuration.

    python -m paper_2508_18983_amd.policy_report [c3 c4 c5]
"""
from __future__ import annotations

import json
import sys

import torch

from smoe_inputs import SHAPES, make_workload
from .session import session_from_workload

LADDER = (("LRU", dict(evict_policy=1, alpha=0.0)),
          ("FIFO", dict(evict_policy=2, alpha=0.0)),
          ("LFU", dict(evict_policy=3, alpha=0.0)),
          ("+CE score eviction", dict(evict_policy=0, alpha=0.0)),
          ("+CR substitution", dict(evict_policy=0)),
          ("+Pre top-score prefetch", dict(evict_policy=0)),
          ("+BA CPU-assisted scheduling", dict(evict_policy=0)))
PRED_NOISE = 0.3


def run(name: str) -> list:
    if name not in SHAPES:
        raise SystemExit(f"unknown workload {name!r}; known: {sorted(SHAPES)}")
    base = SHAPES[name]
    small = base.with_(ffn=64, shared_ffn=64 if base.n_shared else 0)
    rows = []
    for label, kw in LADDER:
        shp = small.with_(**kw)
        # the inputs (and their margin audit) are those of the workload's own alpha
        prefetch = label.startswith(("+Pre", "+BA"))
        assist = label.startswith("+BA")
        wl = make_workload(small, device="cuda" if torch.cuda.is_available() else "cpu",
                           pred_noise=PRED_NOISE if prefetch else None)
        wl.shape = shp.with_(n_layers=wl.shape.n_layers, tokens=wl.shape.tokens, batch=wl.shape.batch)
        cfg = dict(prefetch_max=2) if prefetch else {}
        if assist:
            cfg.update(cpu_assist=1, cpu_threads=2, load_cost_us=3.0, cpu_cost_us=1.0)
        with session_from_workload(wl, **cfg) as ses:
            x = wl.x.to(ses.device)
            xp = wl.x_pred.to(ses.device) if prefetch else None
            y = torch.empty_like(x[0, 0])
            L = shp.n_layers
            for t in range(shp.tokens):
                for l in range(L):
                    tn, ln = divmod(t * L + l + 1, L)
                    if prefetch and tn < shp.tokens:
                        ses.prefetch(ln, xp[tn, ln])
                    ses.decode(l, x[t, l], y)
            ses.sync()
            st = ses.stats()
        rows.append(dict(workload=base.name, config=label, alpha=shp.alpha,
                         hit_rate=st["hits"] / st["slots"], raw_hit_rate=st["raw_hits"] / st["slots"],
                         loads_per_token=(st["fetches"] + st["prefetches"]) / shp.tokens,
                         host_computed_per_token=st["cpu_computed"] / shp.tokens,
                         prefetch_used=(st["prefetch_used"] / st["prefetches"]) if st["prefetches"] else None,
                         substitutions_per_token=st["substitutions"] / shp.tokens))
    return rows


def main(argv) -> int:
    names = argv or ["c3", "c4", "c5"]
    for n in names:
        for row in run(n):
            print(json.dumps(row), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
