"""The five workload shapes the build is measured on.

They are synthetic stand-ins for the paper's model/GPU settings (Table "Model
and GPU Configurations") and public-suite prompts (Section VI "Workloads"),
neither of which is available offline: same layer shapes, expert counts and
top-k as the named model families, random weights, gate logits with the
"few high scores, flat tail" profile of Fig. "obser".
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class MoEShape:
    name: str
    n_layers: int
    hidden: int          # H
    n_experts: int       # E routed experts per layer
    ffn: int             # F per routed expert
    top_k: int           # k
    cache_cap: int       # experts resident in HBM per layer
    alpha: float         # substitution threshold (Table "Definitions")
    tokens: int          # decode steps
    dtype: str = "bf16"  # "fp32" | "bf16": weights, x and y
    batch: int = 1
    n_shared: int = 0    # always-resident shared experts per layer
    shared_ffn: int = 0  # F of each shared expert
    renorm_topk: int = 1
    subst_key: int = 0   # 0: similarity table ranks candidates, 1: gate score
    evict_window: int = 3  # n of Eq. 3
    evict_policy: int = 0  # 0 score (Eq. 3), 1 LRU, 2 FIFO, 3 LFU
    prior: str = "normal"  # "normal": x ~ N(0,1); "zipf": logits from a Zipf prior
    zipf_s: float = 0.0
    locality_p: float = 0.0      # P(boost previous token's top-k) per token-layer
    locality_boost: float = 4.0
    sim: str = "cosine"          # "cosine" of flattened weights | seeded "uniform"
    seed: int = 0

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    @property
    def expert_elems(self) -> int:
        return 3 * self.hidden * self.ffn

    @property
    def expert_bytes(self) -> int:
        return self.expert_elems * self.elem_bytes

    @property
    def shared_elems(self) -> int:
        return 3 * self.hidden * self.shared_ffn

    def layer_bytes(self) -> int:
        """Algorithmic HBM bytes one batch-1 decode of one layer must read:
        gate matrix + k routed experts + the shared experts, each once."""
        eb = self.elem_bytes
        return eb * (self.n_experts * self.hidden
                     + self.top_k * self.expert_elems
                     + self.n_shared * self.shared_elems)

    def with_(self, **kw) -> "MoEShape":
        return replace(self, **kw)


SHAPES = {
    # tiny fp32 case the oracle finishes in well under a second
    "c1": MoEShape("c1-tiny-fp32", 2, 256, 8, 512, 2, 4, 0.3, 16, dtype="fp32"),
    # small bf16 case, gate logits drawn with a minimum top-k gap
    "c2": MoEShape("c2-small-bf16", 4, 1024, 16, 2816, 2, 8, 0.25, 128),
    # Mixtral-8x7B-shaped
    "c3": MoEShape("c3-mixtral8x7b-shaped", 32, 4096, 8, 14336, 2, 4, 0.2, 256,
                   prior="zipf", zipf_s=1.1, sim="uniform"),
    # DeepSeek-V2-Lite-shaped: 64 routed + 2 shared
    "c4": MoEShape("c4-dsv2lite-shaped", 26, 2048, 64, 1408, 6, 24, 0.15, 256,
                   n_shared=2, shared_ffn=1408, renorm_topk=0,
                   prior="zipf", zipf_s=1.0, sim="uniform"),
    # Qwen2-57B-A14B-shaped: 64 routed + one wide shared FFN
    "c5": MoEShape("c5-qwen2-57b-a14b-shaped", 28, 3584, 64, 2560, 8, 32, 0.25, 512,
                   n_shared=1, shared_ffn=20480, renorm_topk=0,
                   prior="zipf", zipf_s=1.2, locality_p=0.6, sim="uniform"),
}


def shape_by_name(name: str) -> MoEShape:
    key = name.lower()
    if key in SHAPES:
        return SHAPES[key]
    for s in SHAPES.values():
        if s.name == name:
            return s
    raise KeyError(f"unknown workload shape {name!r}; known: {sorted(SHAPES)}")
