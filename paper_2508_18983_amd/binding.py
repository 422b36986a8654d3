"""ctypes binding of libsmoe.so.  Argument marshalling only: every function
here has the name and arguments of the C entry point it forwards to (see
include/smoe.h); pointers are passed as integers (``tensor.data_ptr()``,
``stream.cuda_stream``).  There is no fallback: a missing library raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libsmoe.so")
_lib = None

PROF_KINDS = ("route", "up", "down", "copy", "up_loaded", "down_loaded")
ERRORS = {-1: "SMOE_EINVAL", -2: "SMOE_EHIP", -3: "SMOE_ENOTPINNED", -4: "SMOE_ESTATE", -5: "SMOE_ETOOBIG"}


class SmoeError(RuntimeError):
    def __init__(self, fn: str, code: int):
        self.code = code
        hip = moe_last_hip_error() if code == -2 else 0
        super().__init__(f"{fn} failed: {ERRORS.get(code, code)}" + (f" (hipError {hip})" if hip else ""))


class MoeCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "hidden", "n_experts", "ffn", "top_k", "cache_cap", "n_shared",
        "shared_ffn", "dtype", "max_batch")] + [("alpha", C.c_float)] + [(n, C.c_int32) for n in (
        "subst_key", "renorm_topk", "evict_window", "n_stage", "evict_policy", "prefetch_max",
        "cpu_assist", "cpu_threads")] + [("load_cost_us", C.c_float), ("cpu_cost_us", C.c_float),
                                            ("auto_prefetch", C.c_int32), ("prefetch_yield", C.c_int32)]


class MoeBuffers(C.Structure):
    _fields_ = [("gate_w_dev", C.c_void_p), ("experts_host", C.c_void_p), ("shared_dev", C.c_void_p),
                ("sim_host", C.c_void_p), ("cache_slab_dev", C.c_void_p), ("init_resident", C.c_void_p),
                ("stream_compute", C.c_void_p), ("stream_copy", C.c_void_p)]


class MoeTrace(C.Structure):
    _fields_ = [("topk_idx", C.c_void_p), ("final_idx", C.c_void_p), ("substituted", C.c_void_p),
                ("hit", C.c_void_p), ("scores", C.c_void_p), ("weights", C.c_void_p),
                ("fetched", C.c_void_p), ("victims", C.c_void_p), ("on_cpu", C.c_void_p),
                ("adopted", C.c_void_p), ("adopt_victims", C.c_void_p),
                ("n_fetched", C.c_int32), ("n_on_cpu", C.c_int32), ("n_adopted", C.c_int32), ("pad_", C.c_int32),
                ("inflight_mask", C.c_uint64)]


class MoeStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "tokens", "slots", "raw_hits", "hits", "misses", "substitutions", "evictions", "staged",
        "fetches", "bytes_fetched", "prefetches", "prefetch_used", "prefetch_top", "cpu_computed")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class MoePrefetchInfo(C.Structure):
    _fields_ = [("layer", C.c_int32), ("n_wanted", C.c_int32), ("n_loaded", C.c_int32),
                ("wanted", C.c_int32 * 64), ("yielded", C.c_int32),
                ("bytes_copied", C.c_int64), ("bytes_withdrawn", C.c_int64)]

    def as_dict(self):
        return dict(layer=int(self.layer), wanted=[int(v) for v in self.wanted[:self.n_wanted]],
                    loaded=[int(v) for v in self.wanted[:self.n_loaded]])


class MoeProfile(C.Structure):
    _fields_ = [("launches", C.c_int64 * 6), ("ms", C.c_double * 6), ("bytes", C.c_int64 * 6)]

    def as_dict(self):
        return {k: dict(launches=int(self.launches[i]), ms=float(self.ms[i]), bytes=int(self.bytes[i]))
                for i, k in enumerate(PROF_KINDS)}


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the in-tree libsmoe.so; raise if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2508_18983_amd.build` "
            "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    P, I = C.c_void_p, C.c_int32
    lib.moe_cache_init.argtypes = [C.POINTER(MoeCfg), C.POINTER(MoeBuffers), C.POINTER(P)]
    lib.moe_decode_layer.argtypes = [P, I, I, P, P, C.POINTER(MoeTrace)]
    lib.moe_decode_layer_static.argtypes = [P, I, I, P, P, C.POINTER(MoeTrace)]
    lib.moe_prefetch_layer.argtypes = [P, I, I, P]
    lib.moe_prefetch_last.argtypes = [P, C.POINTER(MoePrefetchInfo)]
    lib.moe_cpu_assist_costs.argtypes = [P, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                         C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.moe_cache_stats.argtypes = [P, I, C.POINTER(MoeStats)]
    lib.moe_cache_residency.argtypes = [P, I, P]
    lib.moe_cache_reset.argtypes = [P]
    lib.moe_cache_destroy.argtypes = [P]
    lib.moe_profile_enable.argtypes = [P, I, I]
    lib.moe_profile_read.argtypes = [P, C.POINTER(MoeProfile)]
    lib.moe_last_hip_error.argtypes = []
    lib.moe_calib_copy.argtypes = [P, P, C.c_int64, P]
    lib.moe_host_alloc.argtypes = [C.c_int64, C.POINTER(P)]
    lib.moe_host_free.argtypes = [P]
    lib.moe_select_alpha.argtypes = [P, P, I, C.c_double, I, I, C.POINTER(C.c_double), P]
    for fn in ("moe_cache_init", "moe_decode_layer", "moe_decode_layer_static", "moe_prefetch_layer", "moe_prefetch_last", "moe_cpu_assist_costs", "moe_cache_stats", "moe_cache_residency",
               "moe_cache_reset", "moe_cache_destroy", "moe_profile_enable", "moe_profile_read",
               "moe_last_hip_error", "moe_calib_copy", "moe_host_alloc", "moe_host_free", "moe_select_alpha"):
        getattr(lib, fn).restype = C.c_int
    _lib = lib
    return lib


def _check(fn: str, rc: int) -> None:
    if rc != 0:
        raise SmoeError(fn, rc)


class Trace:
    """Host arrays for one call's moe_trace_t."""

    def __init__(self, batch: int, k: int, n_experts: int):
        self.topk_idx = np.full((batch, k), -1, np.int32)
        self.final_idx = np.full((batch, k), -1, np.int32)
        self.substituted = np.zeros((batch, k), np.uint8)
        self.hit = np.zeros((batch, k), np.uint8)
        self.scores = np.zeros((batch, n_experts), np.float32)
        self.weights = np.zeros((batch, k), np.float32)
        self.fetched = np.full(batch * k, -1, np.int32)
        self.victims = np.full(batch * k, -1, np.int32)
        self.on_cpu = np.full(batch * k, -1, np.int32)
        self.adopted = np.full(batch * k, -1, np.int32)
        self.adopt_victims = np.full(batch * k, -1, np.int32)
        self.c = MoeTrace(*(a.ctypes.data for a in (
            self.topk_idx, self.final_idx, self.substituted, self.hit, self.scores, self.weights,
            self.fetched, self.victims, self.on_cpu, self.adopted, self.adopt_victims)), 0, 0, 0, 0, 0)

    @property
    def n_fetched(self) -> int:
        return int(self.c.n_fetched)

    @property
    def n_on_cpu(self) -> int:
        return int(self.c.n_on_cpu)

    @property
    def n_adopted(self) -> int:
        return int(self.c.n_adopted)

    @property
    def inflight(self) -> set:
        m = int(self.c.inflight_mask)
        return {e for e in range(64) if (m >> e) & 1}


def moe_last_hip_error() -> int:
    return int(load_library().moe_last_hip_error())


def moe_cache_init(cfg: MoeCfg, buf: MoeBuffers) -> int:
    handle = C.c_void_p()
    _check("moe_cache_init", load_library().moe_cache_init(C.byref(cfg), C.byref(buf), C.byref(handle)))
    return handle.value


def moe_decode_layer(handle: int, layer: int, batch: int, x_dev: int, y_dev: int,
                     trace: Optional[Trace] = None) -> None:
    tp = C.byref(trace.c) if trace is not None else None
    _check("moe_decode_layer", load_library().moe_decode_layer(handle, layer, batch, x_dev, y_dev, tp))


def moe_decode_layer_static(handle: int, layer: int, batch: int, x_dev: int, y_dev: int,
                            trace: Optional[Trace] = None) -> None:
    tp = C.byref(trace.c) if trace is not None else None
    _check("moe_decode_layer_static",
           load_library().moe_decode_layer_static(handle, layer, batch, x_dev, y_dev, tp))


def moe_prefetch_layer(handle: int, layer: int, batch: int, x_pred_dev: int) -> None:
    _check("moe_prefetch_layer", load_library().moe_prefetch_layer(handle, layer, batch, x_pred_dev))


def moe_prefetch_last(handle: int) -> MoePrefetchInfo:
    info = MoePrefetchInfo()
    _check("moe_prefetch_last", load_library().moe_prefetch_last(handle, C.byref(info)))
    return info


def moe_cpu_assist_costs(handle: int) -> dict:
    cl, cc, busy, n = C.c_double(), C.c_double(), C.c_double(), C.c_int64()
    _check("moe_cpu_assist_costs", load_library().moe_cpu_assist_costs(
        handle, C.byref(cl), C.byref(cc), C.byref(busy), C.byref(n)))
    return dict(c_load_us=cl.value, c_cpu_us=cc.value, cpu_busy_us=busy.value, cpu_experts=n.value)


def moe_cache_stats(handle: int, layer: int = -1) -> MoeStats:
    st = MoeStats()
    _check("moe_cache_stats", load_library().moe_cache_stats(handle, layer, C.byref(st)))
    return st


def moe_cache_residency(handle: int, layer: int, cache_cap: int) -> np.ndarray:
    out = np.zeros(cache_cap, np.int32)
    _check("moe_cache_residency", load_library().moe_cache_residency(handle, layer, out.ctypes.data))
    return out


def moe_cache_reset(handle: int) -> None:
    _check("moe_cache_reset", load_library().moe_cache_reset(handle))


def moe_cache_destroy(handle: int) -> None:
    _check("moe_cache_destroy", load_library().moe_cache_destroy(handle))


def moe_profile_enable(handle: int, enable: int, max_launches: int = 1) -> None:
    _check("moe_profile_enable", load_library().moe_profile_enable(handle, enable, max_launches))


def moe_profile_read(handle: int) -> MoeProfile:
    p = MoeProfile()
    _check("moe_profile_read", load_library().moe_profile_read(handle, C.byref(p)))
    return p


def moe_calib_copy(dst_dev: int, src_dev: int, n_bytes: int, stream: int) -> None:
    _check("moe_calib_copy", load_library().moe_calib_copy(dst_dev, src_dev, n_bytes, stream))


def moe_host_alloc(n_bytes: int) -> int:
    p = C.c_void_p()
    _check("moe_host_alloc", load_library().moe_host_alloc(n_bytes, C.byref(p)))
    return p.value


def moe_host_free(ptr: int) -> None:
    _check("moe_host_free", load_library().moe_host_free(ptr))


def moe_select_alpha(alphas, tpots, budget: float, degree: int = 2, resolution: int = 2001):
    """-> (alpha or None when no grid point meets the budget, coefficients constant term first)."""
    a = np.ascontiguousarray(alphas, dtype=np.float64)
    t = np.ascontiguousarray(tpots, dtype=np.float64)
    if a.ndim != 1 or a.shape != t.shape:
        raise ValueError("alphas and tpots must be one-dimensional and of equal length")
    coef = np.zeros(degree + 1, np.float64)
    out = C.c_double()
    rc = load_library().moe_select_alpha(a.ctypes.data, t.ctypes.data, a.size, float(budget), degree,
                                         resolution, C.byref(out), coef.ctypes.data)
    if rc == -4:
        return None, coef
    _check("moe_select_alpha", rc)
    return out.value, coef
