"""The library's cache bookkeeping (history ring, Eq. 3 / baseline victims,
protection shield, slot map, counters) replayed on the CPU: the HIP-free
scheduler code is built into a small shim and fed the oracle's routing
decisions; its victims, residency and counters must equal the oracle's."""
import ctypes as C
import os

import numpy as np
import pytest

from oracle import smoe_oracle as O
from smoe_inputs import SHAPES, make_workload, as_numpy

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SHIM = os.path.join(ROOT, "paper_2508_18983_amd", "libsmoe_hostlogic.so")


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("tokens", "slots", "raw_hits", "hits", "misses", "substitutions",
                                         "evictions", "staged", "fetches", "bytes_fetched",
                                         "prefetches", "prefetch_used", "prefetch_top", "cpu_computed")]


@pytest.fixture(scope="module")
def shim():
    if not os.path.exists(SHIM):
        pytest.fail(f"{SHIM} missing: run python -m paper_2508_18983_amd.build")
    lib = C.CDLL(SHIM)
    lib.smoe_hl_create.restype = C.c_void_p
    lib.smoe_hl_create.argtypes = [C.c_int] * 7 + [C.c_int64, C.c_void_p, C.c_float, C.c_int, C.c_int,
                                   C.c_double, C.c_double]
    lib.smoe_hl_prefetch.argtypes = [C.c_void_p, C.c_int, C.c_int] + [C.c_void_p] * 5
    lib.smoe_hl_destroy.argtypes = [C.c_void_p]
    lib.smoe_hl_step.argtypes = [C.c_void_p, C.c_int, C.c_int] + [C.c_void_p] * 4 + [C.c_uint64] + [C.c_void_p] * 10
    lib.smoe_hl_residency.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
    lib.smoe_hl_stats.argtypes = [C.c_void_p, C.c_int, C.POINTER(Stats)]
    return lib


class StepOut:
    """Output arrays of one smoe_hl_step call."""

    def __init__(self, nk):
        self.fetched, self.victims, self.slots, self.on_cpu, self.adopted, self.adopt_victims, self.dropped = (
            np.zeros(nk, np.int32) for _ in range(7))
        self.n_cpu, self.n_adopted, self.n_dropped = (np.zeros(1, np.int32) for _ in range(3))

    def args(self):
        return [a.ctypes.data for a in (self.fetched, self.victims, self.slots, self.on_cpu, self.n_cpu,
                                        self.adopted, self.adopt_victims, self.n_adopted, self.dropped,
                                        self.n_dropped)]


def hl_step(lib, h, layer, batch, r, out, inflight=0):
    """Feed the oracle's routing decision `r` to the scheduler; returns the number of loads."""
    topk = np.ascontiguousarray(r.topk, np.int32)
    fin = np.ascontiguousarray(r.final, np.int32)
    sub = np.ascontiguousarray(r.substituted, np.int32)
    sc = np.ascontiguousarray(r.scores, np.float32)
    return lib.smoe_hl_step(h, layer, batch, topk.ctypes.data, fin.ctypes.data, sub.ctypes.data, sc.ctypes.data,
                            inflight, *out.args())


def replay(lib, wl, batch=1, n_stage=0, prefetch_max=0, inflight_all=False, **oracle_kw):
    """`inflight_all`: every prefetched expert is taken to be still in flight at its
    layer's step (on both sides), so that CPU-assisted scheduling may take it over."""
    s = wl.shape
    orc = O.oracle_from_workload(wl, **oracle_kw)
    h = lib.smoe_hl_create(s.n_layers, s.n_experts, s.top_k, orc.cap, orc.window, orc.evict_policy,
                           n_stage, s.expert_bytes, None, orc.alpha, prefetch_max,
                           int(orc.cpu_assist), orc.c_load, orc.c_cpu)
    assert h
    nk = batch * s.top_k
    out = StepOut(nk)
    wanted = np.zeros(nk, np.int32); n_wanted = np.zeros(1, np.int32); pslots = np.zeros(nk, np.int32)
    res_slots = np.zeros(orc.cap, np.int32)
    loads = 0
    try:
        for t in range(s.tokens):
            for l in range(s.n_layers):
                inflight = set()
                if prefetch_max:
                    pf = orc.prefetch_layer(l, as_numpy(wl.x_pred[t, l]), prefetch_max)
                    p_topk = np.ascontiguousarray(pf.topk, np.int32)
                    p_sc = np.ascontiguousarray(pf.scores, np.float32)
                    n = lib.smoe_hl_prefetch(h, l, batch, p_topk.ctypes.data, p_sc.ctypes.data,
                                             wanted.ctypes.data, n_wanted.ctypes.data, pslots.ctypes.data)
                    assert wanted[:n_wanted[0]].tolist() == pf.wanted, (t, l)
                    assert n == len(pf.prefetched), (t, l)
                    assert all(orc.cap <= v < orc.cap + prefetch_max or v < orc.cap for v in pslots[:n])
                    lib.smoe_hl_residency(h, l, res_slots.ctypes.data)
                    assert res_slots.tolist() == orc.layers[l].slot_expert, (t, l)      # G untouched
                    if inflight_all:
                        inflight = set(orc.layers[l].landed)
                r = orc.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False, inflight=inflight)
                n = hl_step(lib, h, l, batch, r, out, sum(1 << e for e in inflight))
                assert n == len(r.fetched), (t, l, n)
                assert out.on_cpu[:out.n_cpu[0]].tolist() == r.on_cpu, (t, l)
                assert out.fetched[:n].tolist() == r.fetched and out.victims[:n].tolist() == r.victims, (t, l)
                assert [v >= 0 for v in out.victims[:n]] == [sl >= 0 for sl in out.slots[:n]]
                na = out.n_adopted[0]
                assert out.adopted[:na].tolist() == r.adopted and out.adopt_victims[:na].tolist() == r.adopt_victims
                want_dropped = r.dropped + [e for e in r.on_cpu if e in inflight]
                assert sorted(out.dropped[:out.n_dropped[0]].tolist()) == sorted(want_dropped), (t, l)
                lib.smoe_hl_residency(h, l, res_slots.ctypes.data)
                assert res_slots.tolist() == orc.layers[l].slot_expert, (t, l)
                loads += n
        for l in range(s.n_layers):
            st = Stats()
            lib.smoe_hl_stats(h, l, C.byref(st))
            assert {n: getattr(st, n) for n, _ in Stats._fields_} == orc.stats(l).as_dict()
    finally:
        lib.smoe_hl_destroy(h)
    return loads, orc.stats()


@pytest.mark.parametrize("policy", [0, 1, 2, 3])
def test_scheduler_replay_matches_oracle(shim, policy):
    wl = make_workload(SHAPES["c1"].with_(tokens=40, seed=policy))
    loads, st = replay(shim, wl, evict_policy=policy)
    assert loads > 10 and st.substitutions > 0
    shp = SHAPES["c4"].with_(ffn=32, shared_ffn=32, seed=40 + policy)
    wl = make_workload(shp, n_layers=3, tokens=60)
    loads, st = replay(shim, wl, evict_policy=policy)
    assert loads > 50


@pytest.mark.parametrize("window", [0, 1, 7])
def test_scheduler_window_lengths(shim, window):
    wl = make_workload(SHAPES["c1"].with_(tokens=40, seed=3))
    replay(shim, wl, evict_window=window)


def test_scheduler_batch_and_staging(shim):
    shp = SHAPES["c5"].with_(ffn=32, shared_ffn=32, cache_cap=12, seed=5)
    wl = make_workload(shp, n_layers=2, tokens=20, batch=4)
    loads, st = replay(shim, wl, batch=4, n_stage=32)
    assert st.staged > 0
    # without staging slots the same step is refused with SMOE_ESTATE (-4)
    s = wl.shape
    orc = O.oracle_from_workload(wl)
    h = shim.smoe_hl_create(s.n_layers, s.n_experts, s.top_k, s.cache_cap, 3, 0, 0, s.expert_bytes, None,
                            0.25, 0, 0, 1.0, 1.0)
    rc = 0
    out = StepOut(64)
    for t in range(s.tokens):
        for l in range(s.n_layers):
            r = orc.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
            rc = hl_step(shim, h, l, 4, r, out)
            if rc < 0 or -1 in r.victims:
                break
        if rc < 0 or -1 in r.victims:
            break
    assert rc == -4
    shim.smoe_hl_destroy(h)


@pytest.mark.parametrize("policy,batch", [(0, 1), (1, 1), (2, 1), (3, 1), (0, 3)])
def test_prefetch_replay_matches_oracle(shim, policy, batch):
    """Top-score prefetch decisions (Section IV-C): what is wanted, what is
    loaded, whom it evicts, and the accuracy counters at the next step."""
    shp = SHAPES["c4"].with_(ffn=32, shared_ffn=32, seed=60 + policy, cache_cap=16)
    wl = make_workload(shp, n_layers=2, tokens=50, batch=batch, pred_noise=0.6)
    loads, st = replay(shim, wl, batch=batch, n_stage=batch * shp.top_k, prefetch_max=3, evict_policy=policy)
    assert st.prefetches > 30 and 0 < st.prefetch_top <= st.prefetch_used < st.prefetches
    # the same with every prefetch taken to be in flight and Algorithm 2 on: some prefetched
    # experts are handed to the host cores instead of being waited for
    loads, st = replay(shim, wl, batch=batch, n_stage=batch * shp.top_k, prefetch_max=3, evict_policy=policy,
                       inflight_all=True, cpu_assist=1, c_load=3.0, c_cpu=1.0)
    assert st.prefetches > 30 and st.cpu_computed > 5


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("costs,batch", [((2.0, 1.0), 1), ((1.0, 1.0), 1), ((1.0, 3.5), 1), ((3.0, 1.0), 3)])
def test_cpu_assisted_scheduling_replay_matches_oracle(shim, costs, batch, mode):
    """Algorithm 2 inside the scheduler: which misses are loaded (and cached) and
    which are left to the host cores, with and without a pending prefetch."""
    shp = SHAPES["c4"].with_(ffn=32, shared_ffn=32, seed=80 + batch, cache_cap=12)
    wl = make_workload(shp, n_layers=2, tokens=40, batch=batch, pred_noise=0.6)
    for pf in (0, 2):
        loads, st = replay(shim, wl, batch=batch, n_stage=batch * shp.top_k, prefetch_max=pf,
                           cpu_assist=mode, c_load=costs[0], c_cpu=costs[1])
        if mode == 1:
            assert st.cpu_computed > 20 and st.fetches > 20
        else:                       # the variant leans to whichever side is cheaper
            assert st.cpu_computed + st.fetches > 40
            assert (st.cpu_computed > st.fetches) == (costs[1] < costs[0]) or costs[0] == costs[1]


def test_scheduler_rejects_bad_arguments_and_malformed_decisions(shim):
    tail = (0.2, 0, 0, 1.0, 1.0)
    assert not shim.smoe_hl_create(1, 65, 2, 4, 3, 0, 0, 100, None, *tail)      # too many experts
    assert not shim.smoe_hl_create(1, 8, 2, 1, 3, 0, 0, 100, None, *tail)       # cap < k
    assert not shim.smoe_hl_create(1, 8, 2, 4, 3, 9, 0, 100, None, *tail)       # unknown policy
    h = shim.smoe_hl_create(1, 8, 2, 4, 3, 0, 0, 100, None, *tail)
    topk = np.array([[0, 1]], np.int32); bad = np.array([[0, 9]], np.int32); sub = np.zeros((1, 2), np.int32)
    sc = np.full((1, 8), 0.125, np.float32); o = StepOut(2)
    assert shim.smoe_hl_step(h, 0, 1, topk.ctypes.data, bad.ctypes.data, sub.ctypes.data, sc.ctypes.data,
                             0, *o.args()) == -4
    assert shim.smoe_hl_step(h, 3, 1, topk.ctypes.data, topk.ctypes.data, sub.ctypes.data, sc.ctypes.data,
                             0, *o.args()) == -1
    shim.smoe_hl_destroy(h)


def test_refused_step_leaves_the_layer_as_it_was(shim):
    """A step that needs more staging slots than exist is refused before anything
    changes: counters, residency, history and stamps are those of a scheduler
    that never saw it, so the following steps still match the oracle."""
    E, k, cap = 8, 2, 2
    h = shim.smoe_hl_create(1, E, k, cap, 3, 1, 1, 100, None, 0.0, 0, 0, 1.0, 1.0)     # LRU, one staging slot
    twin = shim.smoe_hl_create(1, E, k, cap, 3, 1, 1, 100, None, 0.0, 0, 0, 1.0, 1.0)
    o = StepOut(8)
    res = np.zeros(cap, np.int32)

    def step(hh, topk_rows):
        B = len(topk_rows)
        topk = np.array(topk_rows, np.int32)
        sub = np.zeros_like(topk)
        sc = np.full((B, E), 0.05, np.float32)
        for t, row in enumerate(topk_rows):
            sc[t, row] = [0.4, 0.3]
        return shim.smoe_hl_step(hh, 0, B, topk.ctypes.data, topk.ctypes.data, sub.ctypes.data, sc.ctypes.data,
                                 0, *o.args())

    def state(hh):
        st = Stats()
        shim.smoe_hl_stats(hh, 0, C.byref(st))
        shim.smoe_hl_residency(hh, 0, res.ctypes.data)
        return {n: getattr(st, n) for n, _ in Stats._fields_}, res.tolist()

    for hh in (h, twin):
        assert step(hh, [[0, 2]]) == 1                       # one load, evicts expert 1
    before = state(h)
    # two tokens, four distinct experts, three of them missing: both residents shielded, 3 loads > 1 slot
    assert step(h, [[0, 3], [4, 5]]) == -4
    assert state(h) == before
    for rows in ([[2, 6]], [[0, 6]], [[7, 2]], [[1, 0]]):
        assert step(h, rows) == step(twin, rows)
        assert state(h) == state(twin)
    shim.smoe_hl_destroy(h)
    shim.smoe_hl_destroy(twin)
