"""The host-core expert FFN of the CPU-assisted scheduling (Section V-A),
checked on its own against the oracle's FFN on the same stored weights."""
import ctypes as C
import os

import numpy as np
import pytest
import torch

from oracle import smoe_oracle as O
from smoe_inputs import as_numpy

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SHIM = os.path.join(ROOT, "paper_2508_18983_amd", "libsmoe_hostlogic.so")


@pytest.fixture(scope="module")
def shim():
    if not os.path.exists(SHIM):
        pytest.fail(f"{SHIM} missing: run python -m paper_2508_18983_amd.build")
    lib = C.CDLL(SHIM)
    lib.smoe_hl_cpu_expert.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_int]
    lib.smoe_hl_cpu_expert.restype = None
    return lib


@pytest.mark.parametrize("dtype,H,F,ntok,threads", [
    ("fp32", 256, 512, 1, 1), ("fp32", 264, 520, 3, 4), ("bf16", 1024, 2816, 1, 8),
    ("bf16", 8, 8, 2, 3), ("bf16", 2048, 1408, 8, 5),
])
def test_host_expert_ffn_matches_oracle_ffn(shim, dtype, H, F, ntok, threads):
    g = torch.Generator().manual_seed(H + F)
    tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
    flat = (torch.randn(3 * H * F, generator=g) * 0.05).to(tdt)
    x = torch.randn(ntok, H, generator=g).to(tdt)
    w = torch.rand(ntok, generator=g).to(torch.float32)
    y0 = torch.randn(ntok, H, generator=g).to(torch.float32)            # accumulated into
    y = y0.clone()
    x32 = x.to(torch.float32).contiguous()
    shim.smoe_hl_cpu_expert(flat.data_ptr(), 0 if dtype == "fp32" else 1, H, F, ntok, x32.data_ptr(),
                            w.data_ptr(), y.data_ptr(), threads)
    wf = O.widen(as_numpy(flat))
    w1, w3, w2 = wf[:H * F].reshape(F, H), wf[H * F:2 * H * F].reshape(F, H), wf[2 * H * F:].reshape(H, F)
    for t in range(ntok):
        ref = y0[t].numpy().astype(np.float64) + float(w[t]) * O.swiglu_expert(w1, w3, w2, O.widen(as_numpy(x[t])))
        got = y[t].numpy().astype(np.float64)
        err = np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30)
        assert err < 2e-6, (t, err)


def test_pool_is_reused_across_jobs_and_touch_passes(shim):
    """The library keeps one pool for its lifetime: FFN jobs, a page-touch pass
    and more FFN jobs in a row, with tokens sharing one expert, give the same
    result as fresh single-threaded runs."""
    shim.smoe_hl_pool_create.restype = C.c_void_p
    shim.smoe_hl_pool_create.argtypes = [C.c_int]
    shim.smoe_hl_pool_destroy.argtypes = [C.c_void_p]
    shim.smoe_hl_pool_touch.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
    shim.smoe_hl_pool_run.argtypes = [C.c_void_p, C.c_void_p] + [C.c_int] * 4 + [C.c_void_p] * 3
    H, F = 512, 384
    g = torch.Generator().manual_seed(5)
    experts = [(torch.randn(3 * H * F, generator=g) * 0.05).to(torch.bfloat16) for _ in range(3)]
    x = torch.randn(2, H, generator=g)
    w = torch.rand(2, generator=g)
    pool = shim.smoe_hl_pool_create(5)
    got = torch.zeros(2, H)
    ref = torch.zeros(2, H)
    for rep in range(3):
        for e in experts:
            shim.smoe_hl_pool_run(pool, e.data_ptr(), 1, H, F, 2, x.data_ptr(), w.data_ptr(), got.data_ptr())
            shim.smoe_hl_cpu_expert(e.data_ptr(), 1, H, F, 2, x.data_ptr(), w.data_ptr(), ref.data_ptr(), 1)
        shim.smoe_hl_pool_touch(pool, experts[rep].data_ptr(), experts[rep].numel() * 2)
    shim.smoe_hl_pool_destroy(pool)
    assert torch.isfinite(got).all() and float(got.abs().max()) > 0
    # row ranges differ between 5 workers and 1, the per-row arithmetic does not
    torch.testing.assert_close(got, ref, rtol=0, atol=0)
