"""Device-memory plumbing around the C ABI: allocates the HBM cache slab and
the I/O tensors with PyTorch, owns the two streams and forwards every call to
libsmoe.  No arithmetic of the method happens here."""
from __future__ import annotations

from typing import Optional

import ctypes as C

import numpy as np
import torch

from . import binding as B

_PINNED_BLOCKS = {}     # data_ptr -> owner: blocks handed out by pinned_empty()


def pinned_empty(n_elems: int, dtype: torch.dtype) -> torch.Tensor:
    """Host tensor of exactly n_elems elements in page-locked memory obtained
    from moe_host_alloc (freed at process exit)."""
    nbytes = n_elems * torch.empty(0, dtype=dtype).element_size()
    ptr = B.moe_host_alloc(nbytes)
    raw = (C.c_uint8 * nbytes).from_address(ptr)
    t = torch.frombuffer(raw, dtype=torch.uint8).view(dtype)
    _PINNED_BLOCKS[t.data_ptr()] = raw
    return t


def pinned_free_all() -> None:
    """Release every block handed out by pinned_empty().  Tensors created from
    them must not be touched afterwards."""
    for ptr in list(_PINNED_BLOCKS):
        _PINNED_BLOCKS.pop(ptr)
        B.moe_host_free(ptr)


def _is_pinned(t: torch.Tensor) -> bool:
    return t.data_ptr() in _PINNED_BLOCKS or any(
        base <= t.data_ptr() < base + len(raw) for base, raw in _PINNED_BLOCKS.items()) or t.is_pinned()


class DecodeSession:
    """One moe_handle_t plus the buffers it borrows.

    ``shape`` needs the attributes n_layers, hidden, n_experts, ffn, top_k,
    cache_cap, n_shared, shared_ffn, dtype ("fp32" | "bf16"), alpha, subst_key,
    renorm_topk, evict_window.  ``experts`` holds one host tensor [E, 3*H*F]
    per layer (entries may alias); blocks that are not pinned are copied into
    pinned memory here."""

    def __init__(self, shape, gate_w: torch.Tensor, experts,
                 shared: Optional[torch.Tensor], sim: torch.Tensor, *, max_batch: int = 1,
                 n_stage: int = 0, init_resident: Optional[np.ndarray] = None,
                 device: str = "cuda:0", **cfg_override):
        B.load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("libsmoe needs a GPU: there is no CPU path")
        self.shape = shape
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.tdtype = torch.float32 if shape.dtype == "fp32" else torch.bfloat16
        esize = 4 if shape.dtype == "fp32" else 2
        # expert blocks that are not page-locked yet are copied into blocks of exactly their size
        # from moe_host_alloc, owned by this session and released in close() (PyTorch's pinned
        # allocator rounds sizes up and keeps what it has handed out for the life of the process)
        self._owned_pinned = []
        pinned = {}
        for blk in experts:
            if id(blk) not in pinned:
                if _is_pinned(blk):
                    pinned[id(blk)] = blk
                else:
                    mine = pinned_empty(blk.numel(), blk.dtype).view(blk.shape)
                    mine.copy_(blk)
                    self._owned_pinned.append(mine.data_ptr())
                    pinned[id(blk)] = mine
        self.experts_host = [pinned[id(blk)] for blk in experts]
        self._expert_ptrs = (C.c_void_p * len(self.experts_host))(
            *[blk.data_ptr() for blk in self.experts_host])
        self.gate_w = gate_w.to(self.device).contiguous()
        self.shared = shared.to(self.device).contiguous() if shared is not None else None
        self.sim = sim.contiguous()
        self.stream_compute = torch.cuda.Stream(self.device)
        self.stream_copy = torch.cuda.Stream(self.device)
        cfg = dict(n_layers=shape.n_layers, hidden=shape.hidden, n_experts=shape.n_experts,
                   ffn=shape.ffn, top_k=shape.top_k, cache_cap=shape.cache_cap,
                   n_shared=shape.n_shared, shared_ffn=shape.shared_ffn,
                   dtype=0 if shape.dtype == "fp32" else 1, max_batch=max_batch,
                   alpha=float(shape.alpha), subst_key=shape.subst_key,
                   renorm_topk=shape.renorm_topk, evict_window=shape.evict_window, n_stage=n_stage,
                   evict_policy=getattr(shape, "evict_policy", 0), prefetch_max=0,
                   cpu_assist=0, cpu_threads=0, load_cost_us=0.0, cpu_cost_us=0.0, auto_prefetch=0,
                   prefetch_yield=0)
        cfg.update(cfg_override)
        self.cfg = B.MoeCfg(**cfg)
        self.expert_bytes = 3 * cfg["hidden"] * cfg["ffn"] * esize
        n_slots = cfg["n_layers"] * (cfg["cache_cap"] + cfg["prefetch_max"]) + n_stage
        self.slab = torch.empty(n_slots * self.expert_bytes, dtype=torch.uint8, device=self.device)
        self._init_res = None
        if init_resident is not None:
            self._init_res = np.ascontiguousarray(init_resident, dtype=np.int32)
        buf = B.MoeBuffers(
            self.gate_w.data_ptr(), C.cast(self._expert_ptrs, C.c_void_p),
            self.shared.data_ptr() if self.shared is not None else None,
            self.sim.data_ptr(), self.slab.data_ptr(),
            self._init_res.ctypes.data if self._init_res is not None else None,
            self.stream_compute.cuda_stream, self.stream_copy.cuda_stream)
        torch.cuda.synchronize(self.device)
        self.handle = B.moe_cache_init(self.cfg, buf)
        self.max_batch = max_batch

    # ------------------------------------------------------------------
    def new_trace(self, batch: int = 1) -> B.Trace:
        return B.Trace(batch, self.cfg.top_k, self.cfg.n_experts)

    def decode(self, layer: int, x_dev: torch.Tensor, y_dev: Optional[torch.Tensor] = None,
               trace: Optional[B.Trace] = None, static: bool = False) -> torch.Tensor:
        """x_dev [B, H] on the device (produced on any stream that has been
        synchronised).  Returns y_dev; valid after ``sync()``.  ``static``
        forwards to moe_decode_layer_static (y_dev must then be supplied: that
        entry point exists for callers that do not allocate)."""
        batch = x_dev.shape[0]
        if y_dev is None:
            if static:
                raise ValueError("the static entry point needs a caller-owned y_dev")
            y_dev = torch.empty_like(x_dev)
        fn = B.moe_decode_layer_static if static else B.moe_decode_layer
        fn(self.handle, layer, batch, x_dev.data_ptr(), y_dev.data_ptr(), trace)
        return y_dev

    def prefetch(self, layer: int, x_pred_dev: torch.Tensor) -> None:
        """Top-score prefetch for ``layer`` from the predicted states [B, H]."""
        B.moe_prefetch_layer(self.handle, layer, x_pred_dev.shape[0], x_pred_dev.data_ptr())

    def prefetch_last(self) -> dict:
        return B.moe_prefetch_last(self.handle).as_dict()

    def prefetch_yielded(self) -> bool:
        """Was the last prediction skipped because the link was busy (cfg.prefetch_yield)?
        Like prefetch_last, this takes the decision of a prediction that is still pending."""
        return bool(B.moe_prefetch_last(self.handle).yielded)

    def prefetch_bytes(self) -> dict:
        """Bytes of prefetch copies handed to the copy stream / withdrawn before they were copied."""
        info = B.moe_prefetch_last(self.handle)
        return dict(copied=int(info.bytes_copied), withdrawn=int(info.bytes_withdrawn))

    def sync(self) -> None:
        self.stream_compute.synchronize()
        self.stream_copy.synchronize()

    def stats(self, layer: int = -1) -> dict:
        return B.moe_cache_stats(self.handle, layer).as_dict()

    def residency(self, layer: int) -> np.ndarray:
        return B.moe_cache_residency(self.handle, layer, self.cfg.cache_cap)

    def reset(self) -> None:
        B.moe_cache_reset(self.handle)

    def close(self) -> None:
        if getattr(self, "handle", None):
            B.moe_cache_destroy(self.handle)
            self.handle = None
        for ptr in getattr(self, "_owned_pinned", []):
            if _PINNED_BLOCKS.pop(ptr, None) is not None:
                B.moe_host_free(ptr)
        self._owned_pinned = []
        self.experts_host = []
        # the HBM cache slab goes back to the allocator with the handle (a closed session
        # that is still referenced must not keep tens of GB of device memory)
        self.slab = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def session_from_workload(wl, **kw) -> DecodeSession:
    return DecodeSession(wl.shape, wl.gate_w, wl.experts, wl.shared, wl.sim, **kw)
