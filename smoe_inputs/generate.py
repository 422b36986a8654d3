"""Seeded generator of weights, similarity tables and hidden states.

Recipe (all draws are functions of ``shape.seed`` only):

* every weight matrix is i.i.d. N(0, 0.02) rounded once to the storage dtype;
* ``prior == "normal"``: hidden states x ~ N(0, 1);
* ``prior == "zipf"``: per layer a random permutation pi of the experts and a
  popularity prior p[pi(r)] ~ r^-s.  Target logits are log p + Gumbel(0, 1)
  noise (so the top-k set is a draw without replacement from the prior, with a
  few large scores and a flat tail), optionally boosted on the previous
  token's top-k experts (temporal locality).  The hidden state that realises
  them is the minimum-norm correction of a N(0, 1) vector:
  x = z - Wg^T (Wg Wg^T)^-1 (Wg z - l*), then rounded to the storage dtype;
* *margin audit*: the logits the rounded x really produces (Wg x in fp64) are
  inspected and the token-layer is redrawn when a comparison the decode path
  turns into an integer decision sits closer than ``delta`` to equality
  (top-(k+1) order, the two alpha thresholds around the (k+1)-th logit, the
  order of experts inside the substitution band).  This is the "min top-k gap"
  the workload definitions ask for; it keeps fp32 and fp64 evaluations of the
  same comparison on the same side.

The audit only multiplies the gate matrix with x to look at the inputs it has
just drawn; it takes no routing decision and nothing downstream reads the
logits it computed.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from .shapes import MoEShape

WEIGHT_STD = 0.02
LOGIT_DELTA = 1e-3


def _tdtype(shape: MoEShape) -> torch.dtype:
    return torch.float32 if shape.dtype == "fp32" else torch.bfloat16


def as_numpy(t: torch.Tensor) -> np.ndarray:
    """Zero-copy numpy view of a host tensor; bf16 comes back as raw uint16."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def _to_f64(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.float64).numpy()


def chain_next_input(x: torch.Tensor, y: torch.Tensor) -> torch.Tensor:
    """Chained input mode: the next MoE layer's input from this layer's input x
    and output y, both [B, H].  The blocks between two MoE layers (attention,
    norms) are outside this path; their stand-in is the RMS-normalised residual
    sum z / rms(z), z = x + y, per token.  Computed in fp64 when y is fp64 (the
    tests' checking side), else in fp32; the caller rounds to the storage type."""
    acc = torch.float64 if y.dtype == torch.float64 else torch.float32
    z = x.to(acc) + y.to(acc)
    return z * torch.rsqrt(z.square().mean(dim=-1, keepdim=True))


def logit_margin_ok(logits: np.ndarray, k: int, alpha: float,
                    delta: float = LOGIT_DELTA) -> np.ndarray:
    """Row-wise audit of gate logits [N, E]: True where every comparison the
    decode path will take has at least ``delta`` of slack in logit space."""
    logits = np.asarray(logits, dtype=np.float64)
    n, e = logits.shape
    srt = -np.sort(-logits, axis=1)
    gaps = srt[:, :-1] - srt[:, 1:]
    if e <= k:
        return (gaps >= delta).all(axis=1)
    ok = (gaps[:, :min(e - 1, k + 1)] >= delta).all(axis=1)
    pivot = srt[:, k:k + 1]
    # active experts against T = (1+alpha) S_{k+1}
    ok &= (np.abs(srt[:, :k] - pivot - np.log1p(alpha)) >= delta).all(axis=1)
    if 0.0 < alpha < 1.0 and e > k + 1:
        # inactive experts below the (k+1)-th against R = (1-alpha) S_{k+1}, and the
        # order of those that fall inside the band
        lo = np.log1p(-alpha)
        below = srt[:, k + 1:] - pivot
        ok &= (np.abs(below - lo) >= delta).all(axis=1)
        lower_in_band = (srt[:, 1:] - pivot) >= (lo - delta)
        ok &= ((gaps >= delta) | ~lower_in_band).all(axis=1)
    return ok


@dataclass
class Workload:
    shape: MoEShape
    gate_w: torch.Tensor              # [L, E, H] storage dtype, host
    experts: list                     # L host tensors [E, 3*H*F]: W1[F][H] | W3[F][H] | W2[H][F];
                                      # entries may alias when fewer distinct layers were drawn
    shared: Optional[torch.Tensor]    # [L, n_shared, 3*H*Fs] or None, host
    sim: torch.Tensor                 # [L, E, E] fp32, host
    x: torch.Tensor                   # [T, L, B, H] storage dtype, host
    redraws: int                      # token-layers the margin audit redrew
    x_pred: Optional[torch.Tensor] = None   # [T, L, B, H] predicted hidden states (prefetch input)

    def expert_mats(self, layer: int, e: int):
        s = self.shape
        hf = s.hidden * s.ffn
        flat = self.experts[layer][e]
        return (flat[:hf].view(s.ffn, s.hidden),
                flat[hf:2 * hf].view(s.ffn, s.hidden),
                flat[2 * hf:].view(s.hidden, s.ffn))

    def shared_mats(self, layer: int, j: int):
        s = self.shape
        hf = s.hidden * s.shared_ffn
        flat = self.shared[layer, j]
        return (flat[:hf].view(s.shared_ffn, s.hidden),
                flat[hf:2 * hf].view(s.shared_ffn, s.hidden),
                flat[2 * hf:].view(s.hidden, s.shared_ffn))


def _draw_weights(n: int, dtype: torch.dtype, gen: torch.Generator, device: str,
                  out: torch.Tensor, chunk: int = 1 << 28) -> None:
    """Fill flat host tensor ``out`` (n elements) with N(0, WEIGHT_STD)."""
    flat = out.view(-1)
    for lo in range(0, n, chunk):
        m = min(chunk, n - lo)
        w = torch.randn(m, generator=gen, device=device, dtype=torch.float32)
        w.mul_(WEIGHT_STD)
        flat[lo:lo + m].copy_(w.to(dtype))


def _cosine_table(flat: torch.Tensor) -> torch.Tensor:
    """Cosine between rows of [E, N] (each row = one expert's W1|W3|W2),
    accumulated in fp64, stored fp32, exactly symmetric, unit diagonal."""
    e, n = flat.shape
    g = torch.zeros(e, e, dtype=torch.float64)
    step = 1 << 20
    for lo in range(0, n, step):
        blk = flat[:, lo:lo + step].to(torch.float64)
        g += blk @ blk.T
    nrm = torch.sqrt(torch.diagonal(g))
    c = g / (nrm[:, None] * nrm[None, :])
    c = 0.5 * (c + c.T)
    c.fill_diagonal_(1.0)
    return c.to(torch.float32)


def _uniform_table(e: int, rng: np.random.Generator) -> torch.Tensor:
    u = rng.uniform(-0.05, 0.05, size=(e, e))
    u = np.triu(u, 1)
    u = u + u.T
    np.fill_diagonal(u, 1.0)
    return torch.from_numpy(u.astype(np.float32))


def make_workload(shape: MoEShape, device: str = "cpu", n_layers: int | None = None,
                  tokens: int | None = None, batch: int | None = None,
                  host_alloc=None, distinct_layers: int | None = None,
                  delta: float = LOGIT_DELTA, pred_noise: float | None = None) -> Workload:
    """Draw one workload.  ``device`` is where the normal deviates for the
    weights are drawn ("cuda" makes the 100 GB shapes practical); everything
    is returned in host memory.  ``host_alloc(n_elems, dtype)`` may supply the
    (pinned) storage of each layer's experts.  With ``distinct_layers = D < L``
    only D layers of expert weights are drawn and layer l uses the block of
    layer l mod D (for hosts that cannot pin the whole model); gate weights,
    similarity tables and hidden states stay distinct per layer.

    ``pred_noise = sigma`` also draws the *predicted* hidden states a prefetcher
    would be given (a stand-in for a predictor that sees the layer's input
    before it exists): x_pred = x + sigma * N(0, 1), rounded to the storage
    dtype, from a generator of its own so that x does not depend on it, and
    audited like x (top-(k+1) order and the threshold T of the predicted
    scores)."""
    L = shape.n_layers if n_layers is None else n_layers
    T = shape.tokens if tokens is None else tokens
    B = shape.batch if batch is None else batch
    E, H, F, k = shape.n_experts, shape.hidden, shape.ffn, shape.top_k
    dt = _tdtype(shape)
    gen = torch.Generator(device=device)
    rng = np.random.default_rng([shape.seed, 0x5E0E])
    rng_pred = np.random.default_rng([shape.seed, 0x9FE7])

    gate_w = torch.empty(L, E, H, dtype=dt)
    D = L if distinct_layers is None else max(1, min(L, distinct_layers))
    if host_alloc is None:
        host_alloc = lambda n, dtype: torch.empty(n, dtype=dtype)
    blocks = [host_alloc(E * shape.expert_elems, dt).view(E, shape.expert_elems) for _ in range(D)]
    experts = [blocks[l % D] for l in range(L)]
    shared = None
    if shape.n_shared:
        shared = torch.empty(L, shape.n_shared, shape.shared_elems, dtype=dt)
    sim = torch.empty(L, E, E, dtype=torch.float32)
    for l in range(L):
        gen.manual_seed(shape.seed * 1_000_003 + 7919 * l + 1)
        _draw_weights(E * H, dt, gen, device, gate_w[l])
        if l < D:
            _draw_weights(E * shape.expert_elems, dt, gen, device, experts[l])
        if shared is not None:
            _draw_weights(shape.n_shared * shape.shared_elems, dt, gen, device, shared[l])
        if shape.sim == "cosine":
            sim[l] = _cosine_table(experts[l])
        else:
            sim[l] = _uniform_table(E, rng)

    # ---- hidden states -------------------------------------------------
    wg64 = _to_f64(gate_w)                                   # [L, E, H]
    x = torch.empty(T, L, B, H, dtype=dt)
    x_pred = torch.empty(T, L, B, H, dtype=dt) if pred_noise is not None else None
    redraws = 0
    if shape.prior == "zipf":
        ranks = np.arange(1, E + 1, dtype=np.float64)
        logp = np.empty((L, E))
        for l in range(L):
            perm = rng.permutation(E)
            p = ranks ** (-shape.zipf_s)
            logp[l, perm] = np.log(p / p.sum())
        gram_inv = np.linalg.inv(np.einsum("leh,lfh->lef", wg64, wg64))
        pinv = np.einsum("leh,lef->lhf", wg64, gram_inv)    # Wg^T (Wg Wg^T)^-1 : [L, H, E]
    prev_top = None                                          # [L, B, k] realised top-k of previous token
    for t in range(T):
        todo = np.ones((L, B), dtype=bool)
        xt = np.empty((L, B, H))
        lt = np.empty((L, B, E))
        attempt = 0
        boost = None
        if shape.prior == "zipf" and shape.locality_p > 0 and prev_top is not None:
            boost = rng.random((L, B)) < shape.locality_p
        while todo.any():
            attempt += 1
            if attempt > 200:
                raise RuntimeError("margin audit keeps failing; delta too large for this shape")
            li, bi = np.nonzero(todo)
            m = li.size
            z = rng.standard_normal((m, H))
            if shape.prior == "zipf":
                tgt = logp[li] + rng.gumbel(size=(m, E))
                if boost is not None:
                    rows = np.nonzero(boost[li, bi])[0]
                    if rows.size:
                        cols = prev_top[li[rows], bi[rows]]              # [r, k]
                        tgt[rows[:, None], cols] += shape.locality_boost
                tgt -= tgt.mean(axis=1, keepdims=True)
                resid = np.einsum("meh,mh->me", wg64[li], z) - tgt
                z = z - np.einsum("mhe,me->mh", pinv[li], resid)
            zq = torch.from_numpy(z).to(dt)
            z64 = zq.to(torch.float64).numpy()
            logit = np.einsum("meh,mh->me", wg64[li], z64)
            ok = logit_margin_ok(logit, k, shape.alpha, delta)
            redraws += int((~ok).sum())
            good = np.nonzero(ok)[0]
            xt[li[good], bi[good]] = z64[good]
            lt[li[good], bi[good]] = logit[good]
            todo[li[good], bi[good]] = False
        x[t] = torch.from_numpy(xt).to(dt)
        prev_top = np.argsort(-lt, axis=2, kind="stable")[:, :, :k]
        if x_pred is not None:
            xq = x[t].to(torch.float64).numpy()                      # [L, B, H]
            xp = np.empty((L, B, H))
            todo = np.ones((L, B), dtype=bool)
            attempt = 0
            while todo.any():
                attempt += 1
                if attempt > 200:
                    raise RuntimeError("margin audit of the predicted states keeps failing")
                li, bi = np.nonzero(todo)
                cand = xq[li, bi] + pred_noise * rng_pred.standard_normal((li.size, H))
                c64 = torch.from_numpy(cand).to(dt).to(torch.float64).numpy()
                logit = np.einsum("meh,mh->me", wg64[li], c64)
                ok = logit_margin_ok(logit, k, shape.alpha, delta)
                redraws += int((~ok).sum())
                good = np.nonzero(ok)[0]
                xp[li[good], bi[good]] = c64[good]
                todo[li[good], bi[good]] = False
            x_pred[t] = torch.from_numpy(xp).to(dt)
    return Workload(shape.with_(n_layers=L, tokens=T, batch=B), gate_w, experts, shared, sim, x, redraws,
                    x_pred)
