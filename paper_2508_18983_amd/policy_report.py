"""Hit-rate ladder of the paper's ablation on the synthetic traces (Section VI-C):
recency cache -> score-based eviction ("+CE", Eq. 3) -> expert-cache router
("+CR", Algorithm 1 substitution).  Runs the HIP library (decisions depend only
on the gate logits and the cache state, so the expert FFN width is shrunk to
keep the run short) and prints one table row per workload and configuration.

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
          ("+CR substitution", dict(evict_policy=0)))


def run(name: str) -> list:
    base = SHAPES[name]
    small = base.with_(ffn=64, shared_ffn=64 if base.n_shared else 0)
    rows = []
    for label, kw in LADDER:
        shp = small.with_(**kw)
        # the inputs (and their margin audit) are those of the workload's own alpha
        wl = make_workload(small, device="cuda" if torch.cuda.is_available() else "cpu")
        wl.shape = shp.with_(n_layers=wl.shape.n_layers, tokens=wl.shape.tokens, batch=wl.shape.batch)
        with session_from_workload(wl) as ses:
            x = wl.x.to(ses.device)
            y = torch.empty_like(x[0, 0])
            for t in range(shp.tokens):
                for l in range(shp.n_layers):
                    ses.decode(l, x[t, l], y)
            ses.sync()
            st = ses.stats()
        rows.append(dict(workload=base.name, config=label, alpha=shp.alpha,
                         hit_rate=st["hits"] / st["slots"], raw_hit_rate=st["raw_hits"] / st["slots"],
                         loads_per_token=st["fetches"] / shp.tokens,
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
