"""Pins for the CPU oracle: each checks it against something other than itself
(values the paper states, closed forms, library routines, brute force)."""
import itertools
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import smoe_oracle as O
from smoe_inputs import SHAPES, make_workload, as_numpy

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- formats
def test_widen_bf16_matches_library_conversion():
    t = (torch.randn(4096, generator=torch.Generator().manual_seed(1)) * 3).to(torch.bfloat16)
    t[0], t[1], t[2] = 0.0, -0.0, 1.0
    got = O.widen(as_numpy(t))
    assert got.dtype == np.float64
    np.testing.assert_array_equal(got, t.to(torch.float64).numpy())


# ---------------------------------------------------------------- router
def test_scores_are_library_softmax():
    rng = np.random.default_rng(0)
    for e in (2, 8, 64):
        l = rng.normal(size=e) * 5
        np.testing.assert_allclose(O.softmax_scores(l), scipy.special.softmax(l), rtol=1e-14)
        assert abs(O.softmax_scores(l).sum() - 1) < 1e-14
    # shift invariance and overflow safety
    np.testing.assert_allclose(O.softmax_scores(np.array([1000.0, 999.0])),
                               scipy.special.softmax([1.0, 0.0]), rtol=1e-14)


def test_gate_logits_is_matvec_with_rows_as_experts():
    rng = np.random.default_rng(1)
    wg = rng.normal(size=(5, 7)).astype(np.float32)
    x = rng.normal(size=7).astype(np.float32)
    want = [sum(float(wg[e, h]) * float(x[h]) for h in range(7)) for e in range(5)]
    np.testing.assert_allclose(O.gate_logits(wg, x), want, rtol=1e-14)


def test_topk_matches_full_sort_and_library_topk():
    rng = np.random.default_rng(2)
    for trial in range(200):
        e = int(rng.integers(2, 65))
        k = int(rng.integers(1, e + 1))
        s = scipy.special.softmax(rng.normal(size=e) * 2)
        info = O.route(s, k, 0.25)
        brute = sorted(range(e), key=lambda i: (-s[i], i))[:k]
        assert info.topk == brute
        lib = torch.topk(torch.from_numpy(s), k).indices.tolist()
        assert info.topk == lib
        if e > k:
            assert info.s_k1 == sorted(s, reverse=True)[k]


def test_topk_tie_rule_lower_id_first():
    s = np.array([0.1, 0.3, 0.3, 0.1, 0.2])
    assert O.route(s, 3, 0.0).topk == [1, 2, 4]
    assert O.route(np.array([0.25, 0.25, 0.25, 0.25]), 2, 0.0).topk == [0, 1]


def test_alpha_classification_thresholds():
    # S_{k+1} = 0.10; T = 0.13; R = 0.07  (Algorithm 1, threshold line)
    s = np.array([0.40, 0.14, 0.12, 0.10, 0.08, 0.06, 0.10 - 1e-9])
    s = s / 1.0
    info = O.route(s, 3, 0.3)
    assert info.topk == [0, 1, 2]
    assert info.s_k1 == 0.10
    assert info.T == pytest.approx(0.13) and info.R == pytest.approx(0.07)
    assert info.top_score == [0, 1] and info.low_score == [2]


# ---------------------------------------------------------------- Algorithm 1
def _read_golden(name):
    d = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            d[key] = vals
    return d


def test_intro_worked_example_hit_rate_2_of_5_to_4_of_5():
    g = _read_golden("intro_example.txt")
    names = g["experts"]
    idx = {n: i for i, n in enumerate(names)}
    active = [idx[n] for n in g["active"]]
    resident = {idx[n] for n in g["resident"]}
    # scores realising the example's structure: a,b,c clearly high; d,e just above
    # the (k+1)-th score; f,g just below it; h far below
    score = dict(a=0.30, b=0.25, c=0.20, d=0.062, e=0.060, f=0.055, g=0.054, h=0.019)
    s = np.array([score[n] for n in names])
    k = len(active)
    alpha = 0.3
    info = O.route(s, k, alpha)
    assert sorted(info.topk) == sorted(active)
    assert sorted(info.low_score) == sorted(idx[n] for n in g["low_score"])
    hits_before = len(set(info.topk) & resident)
    assert hits_before == int(g["hits_before"][0])
    assert k - hits_before == int(g["loads_before"][0])
    for key in (0, 1):
        sim = np.eye(len(names))
        r = O.cache_router(info, resident, set(), sim, key)
        served = [e for e in r.final if e in resident]
        assert len(served) == int(g["hits_after"][0])
        assert k - len(served) == int(g["loads_after"][0])
        subs = sorted(e for e, f in zip(r.final, r.substituted) if f)
        assert subs == sorted(idx[n] for n in g["substitutes"])
        assert O.hit_count_eq1(resident, info, len(r.cand)) == int(g["hits_after"][0])


def _random_case(rng, e_max=8):
    e = int(rng.integers(3, e_max + 1))
    k = int(rng.integers(1, e))
    s = scipy.special.softmax(rng.normal(size=e) * rng.choice([0.3, 1.0, 3.0]))
    alpha = float(rng.choice([0.0, 0.1, 0.3, 0.6, 0.9]))
    resident = {int(i) for i in np.nonzero(rng.random(e) < rng.choice([0.2, 0.5, 0.8]))[0]}
    sim = rng.uniform(-1, 1, size=(e, e))
    return e, k, s, alpha, resident, sim


def test_hit_count_equals_eq1_closed_form_bruteforce_sets():
    """Eq. 1 evaluated on sets built here from the definitions (Table
    "Definitions" + the two score-band constraints) equals the number of slots
    the router serves from the GPU."""
    rng = np.random.default_rng(3)
    for _ in range(3000):
        e, k, s, alpha, G, sim = _random_case(rng)
        rank = sorted(range(e), key=lambda i: (-s[i], i))
        Ea = set(rank[:k])
        sk1 = s[rank[k]]
        El = {i for i in Ea if s[i] < (1 + alpha) * sk1}
        Es = {i for i in range(e) if i not in Ea and i in G and s[i] >= (1 - alpha) * sk1}
        want = len(G & Ea) + min(len(El - G), len(Es))
        for key in (0, 1):
            r = O.cache_router(O.route(s, k, alpha), G, set(), sim, key)
            assert sum(1 for x in r.final if x in G) == want
            assert sum(r.substituted) == min(len(El - G), len(Es))
            assert len(set(r.final)) == k                      # no expert used twice
            # top-score experts and resident lows are never touched
            for slot, orig in enumerate(rank[:k]):
                if orig not in El or orig in G:
                    assert r.final[slot] == orig and not r.substituted[slot]
                if r.substituted[slot]:
                    assert r.final[slot] in Es


def test_score_key_takes_highest_scoring_substitutes_and_keeps_highest_lows():
    """Section IV-B: the |E_l \\ G| highest-scoring members of E_s are used; when
    E_s is short, the lows that remain for loading are the highest-scoring."""
    rng = np.random.default_rng(4)
    seen_short = 0
    for _ in range(3000):
        e, k, s, alpha, G, sim = _random_case(rng)
        info = O.route(s, k, alpha)
        r = O.cache_router(info, G, set(), sim, 1)
        rank = sorted(range(e), key=lambda i: (-s[i], i))
        sk1 = s[rank[k]]
        Es = sorted((i for i in rank[k:] if i in G and s[i] >= (1 - alpha) * sk1),
                    key=lambda i: (-s[i], i))
        need = [i for i in rank[:k] if s[i] < (1 + alpha) * sk1 and i not in G]
        m = min(len(need), len(Es))
        used = [r.final[j] for j in range(k) if r.substituted[j]]
        assert sorted(used) == sorted(Es[:m])
        replaced = [rank[j] for j in range(k) if r.substituted[j]]
        assert sorted(replaced) == sorted(need[len(need) - m:])   # the m lowest-scoring
        if m < len(need):
            seen_short += 1
            kept = [rank[j] for j in range(k) if rank[j] in need and not r.substituted[j]]
            assert sorted(kept) == sorted(need[:len(need) - m])
        # the lowest low gets the best substitute ("closest ranked first")
        if m:
            assert r.final[rank.index(need[-1])] == Es[0]
    assert seen_short > 20


def test_sim_key_is_greedy_argmax_over_all_assignments():
    """With the similarity key the first expert processed gets its most similar
    eligible candidate, the next one the best of what is left, ... : check
    against enumeration of every injective assignment in that lexicographic
    order."""
    rng = np.random.default_rng(5)
    checked = 0
    for _ in range(1500):
        e, k, s, alpha, G, sim = _random_case(rng)
        info = O.route(s, k, alpha)
        r = O.cache_router(info, G, set(), sim, 0)
        if not r.need or not r.cand:
            continue
        m = min(len(r.need), len(r.cand))
        best = max(itertools.permutations(r.cand, m),
                   key=lambda p: tuple(sim[b][c] for b, c in zip(r.need, p)))
        got = tuple(r.final[info.topk.index(b)] for b in r.need[:m])
        assert got == best
        checked += 1
    assert checked > 100


def test_no_candidate_keeps_original_expert():
    s = scipy.special.softmax(np.array([3.0, 1.0, 0.9, 0.8, -4.0, -5.0]))
    info = O.route(s, 3, 0.3)
    # residents are all far below the band
    r = O.cache_router(info, {4, 5}, set(), np.eye(6), 0)
    assert r.final == info.topk and not any(r.substituted)
    # alpha = 0: nothing is low-score, nothing is replaced even with residents in reach
    info0 = O.route(s, 3, 0.0)
    r0 = O.cache_router(info0, {3, 4, 5}, set(), np.eye(6), 0)
    assert info0.low_score == [] and r0.final == info0.topk


def test_batch_top_score_set_keeps_and_offers_experts():
    """Section IV-B / VI-B: a low-score expert that another token of the batch
    uses as a top-score expert is kept, and such experts can serve as
    substitutes although they are not resident."""
    s = scipy.special.softmax(np.array([3.0, 1.0, 0.95, 0.9, 0.85, -3.0]))
    info = O.route(s, 3, 0.3)            # actives 0,1,2 ; lows 1,2 ; pivot 3
    assert info.low_score == [1, 2]
    r = O.cache_router(info, set(), {2, 4}, np.eye(6), 1)
    assert r.need == [1]                 # 2 is in C: retained
    assert r.final == [0, 4, 2] and r.substituted == [False, True, False]


# ---------------------------------------------------------------- eviction
def test_eviction_is_eq3_on_the_full_score_log():
    """Replay a trace and recompute Eq. 3 from the complete log with the
    printed 1-based window max(1, j-n) .. j."""
    wl = make_workload(SHAPES["c1"].with_(tokens=48, seed=3))
    for n in (0, 1, 3, 7):
        orc = O.oracle_from_workload(wl, evict_window=n)
        log = {l: [] for l in range(wl.shape.n_layers)}
        fetches = 0
        for t in range(wl.shape.tokens):
            for l in range(wl.shape.n_layers):
                before = list(orc.layers[l].slot_expert)
                res = orc.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
                log[l].append(res.scores[0])
                j = len(log[l])                                    # 1-based iteration index
                lo = max(1, j - n)
                avg = sum(log[l][i - 1] for i in range(lo, j + 1)) / (j - lo + 1)
                resident = list(before)
                shield = set(res.final[0].tolist())
                for m, v in zip(res.fetched, res.victims):
                    cand = [e for e in resident if e not in shield]
                    want = min(cand, key=lambda e: (avg[e], e))
                    assert v == want
                    resident[resident.index(v)] = m
                    fetches += 1
                assert resident == orc.layers[l].slot_expert
        assert fetches > 10


def test_residency_invariants_and_counters_follow_the_trace(c1_workload):
    wl = c1_workload
    orc = O.oracle_from_workload(wl)
    s = wl.shape
    hits = misses = subs = raw = 0
    for t in range(s.tokens):
        for l in range(s.n_layers):
            before = set(orc.layers[l].slot_expert)
            res = orc.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
            after = set(orc.layers[l].slot_expert)
            assert len(orc.layers[l].slot_expert) == s.cache_cap == len(after)
            final = set(res.final[0].tolist())
            assert final <= after                       # everything used is resident after the loads
            assert not (set(res.victims) & final)       # shield: nothing in use was evicted
            assert set(res.victims) <= before
            assert res.fetched == [e for e in res.final[0] if e not in before]
            hits += len(final & before)
            misses += len(final - before)
            raw += len(set(res.topk[0].tolist()) & before)
            subs += int(res.substituted.sum())
            for j in range(s.top_k):
                if res.substituted[0, j]:
                    assert res.final[0, j] in before and res.topk[0, j] not in before
    st = orc.stats()
    assert (st.hits, st.misses, st.raw_hits, st.substitutions) == (hits, misses, raw, subs)
    assert st.hits + st.misses == st.slots == s.tokens * s.n_layers * s.top_k
    assert st.evictions == st.fetches == misses and st.staged == 0
    assert st.bytes_fetched == misses * s.expert_bytes
    assert subs > 0 and misses > 0


def test_staging_when_every_resident_expert_is_shielded():
    wl = make_workload(SHAPES["c1"].with_(cache_cap=2, tokens=4), batch=4)
    orc = O.oracle_from_workload(wl, alpha=0.0)
    staged = 0
    for t in range(4):
        res = orc.decode_layer(0, as_numpy(wl.x[t, 0]), compute_y=False)
        assert len(orc.layers[0].slot_expert) == 2
        assert res.victims.count(-1) == max(0, len(res.fetched) - len(
            [v for v in res.victims if v >= 0]))
        staged += res.victims.count(-1)
    assert staged == orc.stats().staged and staged > 0


# ---------------------------------------------------------------- FFN + output
def test_swiglu_expert_matches_library_ops():
    g = torch.Generator().manual_seed(7)
    H, F = 24, 40
    w1 = torch.randn(F, H, generator=g, dtype=torch.float64)
    w3 = torch.randn(F, H, generator=g, dtype=torch.float64)
    w2 = torch.randn(H, F, generator=g, dtype=torch.float64)
    x = torch.randn(H, generator=g, dtype=torch.float64)
    want = torch.nn.functional.linear(
        torch.nn.functional.silu(torch.nn.functional.linear(x, w1)) * torch.nn.functional.linear(x, w3), w2)
    got = O.swiglu_expert(w1.numpy(), w3.numpy(), w2.numpy(), x.numpy())
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-14)
    # silu at known points
    np.testing.assert_allclose(O.silu(np.array([0.0, 1.0, -1.0])),
                               [0.0, 1 / (1 + np.exp(-1)), -1 / (1 + np.exp(1))], rtol=1e-15)


def _dense_plain_moe(wl, layer, x_row, renorm):
    """Plain MoE layer with library ops: run every expert, mask by top-k."""
    s = wl.shape
    x = x_row.to(torch.float64)
    logits = wl.gate_w[layer].to(torch.float64) @ x
    p = torch.softmax(logits, dim=0)
    top = torch.topk(p, s.top_k)
    mask = torch.zeros(s.n_experts, dtype=torch.float64)
    mask[top.indices] = top.values / (top.values.sum() if renorm else 1.0)
    y = torch.zeros(s.hidden, dtype=torch.float64)
    for e in range(s.n_experts):
        w1, w3, w2 = (m.to(torch.float64) for m in wl.expert_mats(layer, e))
        y += mask[e] * (w2 @ (torch.nn.functional.silu(w1 @ x) * (w3 @ x)))
    for j in range(s.n_shared):
        w1, w3, w2 = (m.to(torch.float64) for m in wl.shared_mats(layer, j))
        y += w2 @ (torch.nn.functional.silu(w1 @ x) * (w3 @ x))
    return y.numpy()


@pytest.mark.parametrize("renorm", [0, 1])
def test_alpha_zero_and_full_capacity_reduce_to_plain_moe(c1_workload, renorm):
    wl = c1_workload
    s = wl.shape
    for kw in (dict(alpha=0.0), dict(cache_cap=s.n_experts)):
        orc = O.oracle_from_workload(wl, renorm_topk=renorm, **kw)
        for t in range(6):
            for l in range(s.n_layers):
                res = orc.decode_layer(l, as_numpy(wl.x[t, l]))
                assert not res.substituted.any()
                np.testing.assert_array_equal(res.final, res.topk)
                want = _dense_plain_moe(wl, l, wl.x[t, l, 0], renorm)
                np.testing.assert_allclose(res.y[0], want, rtol=1e-11, atol=1e-15)
        st = orc.stats()
        assert st.substitutions == 0
        if "cache_cap" in kw:
            assert st.misses == 0 and st.hits == st.slots


def test_substituted_slot_keeps_weight_and_uses_substitute_expert(c1_workload):
    """Output with substitutions = plain combine with the final experts and the
    original gate weights (stated convention for the slot weight)."""
    wl = c1_workload
    s = wl.shape
    orc = O.oracle_from_workload(wl)
    n_sub = 0
    for t in range(s.tokens):
        for l in range(s.n_layers):
            res = orc.decode_layer(l, as_numpy(wl.x[t, l]))
            if not res.substituted.any():
                continue
            n_sub += 1
            x = wl.x[t, l, 0].to(torch.float64)
            p = torch.softmax(wl.gate_w[l].to(torch.float64) @ x, dim=0)
            w = p[torch.from_numpy(res.topk[0])]
            w = w / w.sum()
            y = torch.zeros(s.hidden, dtype=torch.float64)
            for j in range(s.top_k):
                w1, w3, w2 = (m.to(torch.float64) for m in wl.expert_mats(l, int(res.final[0, j])))
                y += w[j] * (w2 @ (torch.nn.functional.silu(w1 @ x) * (w3 @ x)))
            np.testing.assert_allclose(res.y[0], y.numpy(), rtol=1e-11, atol=1e-15)
    assert n_sub >= 3


def test_shared_experts_and_bf16_path_against_dense_library_moe():
    shp = SHAPES["c4"].with_(hidden=128, ffn=96, shared_ffn=64, n_experts=16, cache_cap=16,
                             top_k=4, sim="uniform")
    wl = make_workload(shp, n_layers=2, tokens=3)
    orc = O.oracle_from_workload(wl)
    for t in range(3):
        for l in range(2):
            res = orc.decode_layer(l, as_numpy(wl.x[t, l]))
            want = _dense_plain_moe(wl, l, wl.x[t, l, 0], shp.renorm_topk)
            np.testing.assert_allclose(res.y[0], want, rtol=1e-11, atol=1e-15)


# ---------------------------------------------------------------- baseline replacement policies
def _route_trace(wl):
    """Experts the plain router activates per (token, layer): library top-k."""
    s = wl.shape
    logits = torch.einsum("leh,tlbh->tlbe", wl.gate_w.double(), wl.x.double())
    return torch.topk(logits, s.top_k, dim=-1).indices[:, :, 0].tolist()      # [T][L][k]


def test_lru_and_fifo_match_textbook_caches_when_nothing_is_substituted():
    """alpha = 0, batch 1: the expert cache is an ordinary cache over the router's
    access sequence (with the current step's experts pinned), so LRU must equal an
    OrderedDict LRU and FIFO a queue."""
    from collections import OrderedDict, deque
    wl = make_workload(SHAPES["c1"].with_(tokens=64, seed=8, alpha=0.0))
    s = wl.shape
    trace = _route_trace(wl)
    for policy in (O.EVICT_LRU, O.EVICT_FIFO):
        orc = O.oracle_from_workload(wl, evict_policy=policy)
        caches = []
        for l in range(s.n_layers):
            caches.append(OrderedDict((e, None) for e in range(s.cache_cap)) if policy == O.EVICT_LRU
                          else deque(range(s.cache_cap)))
        misses = 0
        for t in range(s.tokens):
            for l in range(s.n_layers):
                res = orc.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
                want_victims = []
                c = caches[l]
                cur = trace[t][l]
                # the step's experts are pinned (protection shield): evict from the old end,
                # skipping them; afterwards they become the most recent, in slot order
                for e in cur:
                    if e not in c:
                        v = next(x for x in c if x not in cur)
                        want_victims.append(v)
                        if policy == O.EVICT_LRU:
                            del c[v]
                            c[e] = None
                        else:
                            c.remove(v)
                            c.append(e)
                if policy == O.EVICT_LRU:
                    for e in cur:
                        c.move_to_end(e)
                assert res.victims == want_victims, (policy, t, l)
                assert set(orc.layers[l].slot_expert) == set(c)
                misses += len(want_victims)
        assert misses > 20 and orc.stats().misses == misses


def test_lfu_evicts_fewest_uses_bruteforce():
    wl = make_workload(SHAPES["c1"].with_(tokens=64, seed=8, alpha=0.0))
    s = wl.shape
    trace = _route_trace(wl)
    orc = O.oracle_from_workload(wl, evict_policy=O.EVICT_LFU)
    for l in range(s.n_layers):
        cached = {e: dict(cnt=0, last=e - s.cache_cap) for e in range(s.cache_cap)}
        n = 0
        for t in range(s.tokens):
            res = orc.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
            cur = set(trace[t][l])
            want = []
            for j, e in enumerate(trace[t][l]):
                stamp = t * 64 + j
                if e not in cached:
                    cand = [c for c in cached if c not in cur]
                    v = min(cand, key=lambda c: (cached[c]["cnt"], cached[c]["last"], c))
                    want.append(v)
                    del cached[v]
                    cached[e] = dict(cnt=0, last=stamp)
                cached[e]["cnt"] += 1
                cached[e]["last"] = stamp
            assert res.victims == want, (t, l)
            n += len(want)
        assert n > 5


def test_score_eviction_beats_lru_on_skewed_popularity():
    """Shape of the ablation's "+CE" step: with a Zipf-skewed router the score
    history keeps popular experts better than recency does."""
    shp = SHAPES["c4"].with_(ffn=32, shared_ffn=32, alpha=0.0, seed=12)
    wl = make_workload(shp, n_layers=4, tokens=160)
    rates = {}
    for policy in (O.EVICT_LRU, O.EVICT_SCORE):
        orc = O.oracle_from_workload(wl, evict_policy=policy)
        for t in range(160):
            for l in range(4):
                orc.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
        st = orc.stats()
        rates[policy] = st.hits / st.slots
    assert rates[O.EVICT_SCORE] > rates[O.EVICT_LRU]


# ---------------------------------------------------------------- top-score prefetch (Section IV-C)
def _prefetch_workload(alpha, pred_noise, tokens=24, seed=3):
    shp = SHAPES["c4"].with_(n_layers=2, hidden=256, ffn=8, shared_ffn=8, n_shared=0, n_experts=16,
                             top_k=3, cache_cap=6, alpha=alpha, tokens=tokens, seed=seed)
    return make_workload(shp, pred_noise=pred_noise)


def test_prefetch_with_exact_prediction_leaves_only_low_score_misses():
    """If the predicted state equals the real one and up to k experts may be
    prefetched, every top-score expert is on the GPU when its layer runs: what
    is still loaded on demand are low-score experts only, every prefetched
    expert is used, and each one is a top-score expert of the step."""
    wl = _prefetch_workload(0.3, 0.0)
    orc = O.oracle_from_workload(wl)
    s = wl.shape
    n_pref = 0
    for t in range(s.tokens):
        for l in range(s.n_layers):
            x = as_numpy(wl.x[t, l])
            pf = orc.prefetch_layer(l, x, s.top_k)
            n_pref += len(pf.prefetched)
            on_gpu = orc.layers[l].resident | set(orc.layers[l].landed)
            res = orc.decode_layer(l, x, compute_y=False)
            info = O.route(res.scores[0], s.top_k, orc.alpha)
            assert set(info.top_score) <= on_gpu
            assert set(res.fetched) <= set(info.low_score)
            assert pf.topk[0].tolist() == info.topk
            assert res.adopted == pf.prefetched and res.dropped == []
            assert set(res.final[0].tolist()) <= orc.layers[l].resident
    st = orc.stats()
    assert n_pref == st.prefetches > 0
    assert st.prefetch_used == st.prefetch_top == st.prefetches


def test_prefetch_alpha_zero_exact_prediction_removes_every_miss():
    """alpha = 0 makes every active expert top-score (s >= S_{k+1}), so an exact
    prediction with a cap of k prefetches leaves nothing to load on demand."""
    wl = _prefetch_workload(0.0, 0.0)
    orc = O.oracle_from_workload(wl)
    s = wl.shape
    for t in range(s.tokens):
        for l in range(s.n_layers):
            x = as_numpy(wl.x[t, l])
            orc.prefetch_layer(l, x, s.top_k)
            res = orc.decode_layer(l, x, compute_y=False)
            assert res.fetched == [] and res.hit.all()
    st = orc.stats()
    assert st.misses == 0 and st.fetches == 0 and st.hits == st.slots
    assert st.evictions == st.prefetches


def test_prefetch_cap_zero_changes_nothing():
    wl = _prefetch_workload(0.25, 0.4)
    a = O.oracle_from_workload(wl)
    b = O.oracle_from_workload(wl)
    s = wl.shape
    for t in range(s.tokens):
        for l in range(s.n_layers):
            pf = b.prefetch_layer(l, as_numpy(wl.x_pred[t, l]), 0)
            assert pf.prefetched == [] and b.layers[l].landed == []
            ra = a.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
            rb = b.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
            assert ra.final.tolist() == rb.final.tolist() and ra.victims == rb.victims
            assert a.layers[l].slot_expert == b.layers[l].slot_expert
    assert a.stats().as_dict() == b.stats().as_dict()


def test_prefetch_never_touches_the_cache_set_and_a_useless_one_is_free():
    """Section IV-C: a misprediction must cost nothing but the baseline.  The
    prefetch itself leaves G, history and stamps alone; a step that does not use
    the prefetched experts drops them, and from then on the layer is exactly
    where a run without prefetch is -- residency, victims and counters (other
    than the prefetch counters) included."""
    wl = _prefetch_workload(0.25, 0.0, tokens=30, seed=9)
    s = wl.shape
    a = O.oracle_from_workload(wl)               # no prefetch
    b = O.oracle_from_workload(wl)               # prefetches experts the step never computes
    dropped = 0
    for t in range(s.tokens):
        for l in range(s.n_layers):
            x = as_numpy(wl.x[t, l])
            sc = scipy.special.softmax(O.widen(as_numpy(wl.gate_w[l])) @ O.widen(x[0]))
            # a fake prediction: make the three LOWEST-scoring experts look best
            worst = np.argsort(sc)[:3]
            x_fake = np.zeros_like(O.widen(x))
            x_fake[0] = O.widen(as_numpy(wl.gate_w[l]))[worst].sum(axis=0) * 50.0
            before = (list(b.layers[l].slot_expert), list(b.layers[l].history), dict(b.layers[l].last_use))
            pf = b.prefetch_layer(l, x_fake.astype(np.float32), 3)
            assert (list(b.layers[l].slot_expert), list(b.layers[l].history), dict(b.layers[l].last_use)) == before
            ra = a.decode_layer(l, x, compute_y=False)
            rb = b.decode_layer(l, x, compute_y=False)
            if not set(pf.prefetched) & set(ra.final[0].tolist()):
                assert rb.adopted == [] and rb.dropped == pf.prefetched
                dropped += len(rb.dropped)
            assert rb.final.tolist() == ra.final.tolist() or set(pf.prefetched) & set(rb.final[0].tolist())
            if rb.adopted:
                pytest.skip("the fake prediction hit an expert the step used: the case no longer isolates drops")
            assert (rb.fetched, rb.victims) == (ra.fetched, ra.victims)
            assert a.layers[l].slot_expert == b.layers[l].slot_expert
    sa, sb = a.stats().as_dict(), b.stats().as_dict()
    assert dropped == sb["prefetches"] > 20 and sb["prefetch_used"] == 0
    for key in ("hits", "misses", "fetches", "evictions", "substitutions", "raw_hits"):
        assert sa[key] == sb[key]


def test_prefetch_step_rebuilt_from_the_definitions_bruteforce():
    """Brute force over a replay with a noisy predictor.  Prefetch: the wanted
    experts are the predicted top-k members whose predicted score reaches
    (1+alpha) x the (k+1)-th and that are neither in G nor already waiting, by
    descending score, up to the free spare slots.  Step: the waiting experts
    count as resident for the expert-cache router; the ones the step computes
    enter G in (token, slot) order together with the on-demand loads, each
    replacing the unshielded resident with the smallest Eq. 3 mean; the others
    are dropped."""
    wl = _prefetch_workload(0.25, 0.5, tokens=40, seed=5)
    orc = O.oracle_from_workload(wl)
    s = wl.shape
    k, cap_pf = s.top_k, 2
    log = [[] for _ in range(s.n_layers)]            # full score log per layer
    seen = adopted = dropped = 0
    for t in range(s.tokens):
        for l in range(s.n_layers):
            G0 = list(orc.layers[l].slot_expert)
            pf = orc.prefetch_layer(l, as_numpy(wl.x_pred[t, l]), cap_pf)
            sc = scipy.special.softmax(
                O.widen(as_numpy(wl.gate_w[l])) @ O.widen(as_numpy(wl.x_pred[t, l, 0])))
            ranked = sorted(range(s.n_experts), key=lambda e: (-sc[e], e))
            act, pivot = ranked[:k], sc[ranked[k]]
            want = [e for e in act if sc[e] >= (1 + orc.alpha) * pivot and e not in G0]
            assert pf.wanted == want and pf.prefetched == want[:cap_pf]
            assert orc.layers[l].slot_expert == G0 and orc.layers[l].landed == want[:cap_pf]
            seen += len(pf.prefetched)
            waiting = want[:cap_pf]
            res = orc.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
            # the router saw G0 + waiting as resident
            s_true = scipy.special.softmax(O.widen(as_numpy(wl.gate_w[l])) @ O.widen(as_numpy(wl.x[t, l, 0])))
            info = O.route(s_true, k, orc.alpha)
            r = O.cache_router(info, set(G0) | set(waiting), set(), wl.sim[l].numpy(), s.subst_key)
            assert res.final[0].tolist() == r.final
            assert res.hit[0].tolist() == [e in set(G0) | set(waiting) for e in r.final]
            log[l].append(s_true)
            window = log[l][-(s.evict_window + 1):]
            mean = sum(window) / len(window)
            G = list(G0)
            want_fetch, want_vict, want_adopt, want_avict = [], [], [], []
            for e in r.final:
                if e in G0:
                    continue
                ev = [g for g in G if g not in r.final]
                v = min(ev, key=lambda g: (mean[g], g)) if ev else -1
                if v >= 0:
                    G[G.index(v)] = e
                if e in waiting:
                    want_adopt.append(e); want_avict.append(v)
                else:
                    want_fetch.append(e); want_vict.append(v)
            assert (res.fetched, res.victims) == (want_fetch, want_vict)
            assert (res.adopted, res.adopt_victims) == (want_adopt, want_avict)
            assert res.dropped == [e for e in waiting if e not in r.final]
            assert orc.layers[l].slot_expert == G and orc.layers[l].landed == []
            adopted += len(res.adopted); dropped += len(res.dropped)
    st = orc.stats()
    assert seen == st.prefetches == adopted + dropped > 10
    assert adopted == st.prefetch_used and dropped > 0               # noisy prediction: some are wasted
    assert 0 < st.prefetch_top <= st.prefetch_used


def test_prefetch_raises_hit_rate_with_a_good_predictor():
    """Section VI-C (+Pre): with an accurate predictor fewer experts are loaded
    on demand and the cache hit rate goes up."""
    wl = _prefetch_workload(0.2, 0.15, tokens=64, seed=7)
    base = O.oracle_from_workload(wl)
    pre = O.oracle_from_workload(wl)
    s = wl.shape
    for t in range(s.tokens):
        for l in range(s.n_layers):
            pre.prefetch_layer(l, as_numpy(wl.x_pred[t, l]), s.top_k)
            base.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
            pre.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
    assert pre.stats().hits > base.stats().hits
    assert pre.stats().fetches < base.stats().fetches
    assert pre.stats().prefetch_used / pre.stats().prefetches > 0.7


# ---------------------------------------------------------------- Algorithm 2 (CPU-assisted scheduling)
def test_algorithm2_hand_worked_cases():
    # equal costs: alternate, starting with a load
    assert O.split_load_cpu(5, 1.0, 1.0) == (3, 2)
    assert O.split_load_cpu(1, 1.0, 1e-9) == (1, 0)            # the first expert is always loaded
    assert O.split_load_cpu(0, 1.0, 1.0) == (0, 0)
    # a CPU expert costs a third of a load (the paper's S3 remark): load, cpu x3, load, cpu x3
    assert O.split_load_cpu(8, 3.0, 1.0) == (2, 6)
    assert O.split_load_cpu(4, 3.0, 1.0) == (1, 3)
    # a CPU expert costs three loads: load, cpu, then loads until they catch up
    assert O.split_load_cpu(5, 1.0, 3.0) == (4, 1)
    assert O.split_load_cpu(6, 1.0, 3.0) == (4, 2)


def test_algorithm2_split_is_the_one_both_workers_would_accept():
    """Property that singles out Algorithm 2's split among all n+1 candidates
    without replaying it: the last expert the load queue took, it took while it
    was not behind the CPU -- (n_load - 1) C_load <= n_CPU C_CPU -- and the last
    expert the CPU took, it took while the load queue was strictly behind --
    (n_CPU - 1) C_CPU < n_load C_load.  Exactly one split satisfies both."""
    rng = np.random.default_rng(11)
    for trial in range(400):
        n = int(rng.integers(1, 17))
        c_load = float(rng.choice([0.5, 1.0, 2.0, 3.0, 6.25])) * float(rng.choice([1.0, 1.0, 0.37]))
        c_cpu = float(rng.choice([0.5, 1.0, 1.75, 2.0, 9.0]))
        ok = []
        for a in range(n + 1):
            b = n - a
            load_fine = a == 0 or (a - 1) * c_load <= b * c_cpu
            cpu_fine = b == 0 or (b - 1) * c_cpu < a * c_load
            if load_fine and cpu_fine:
                ok.append((a, b))
        assert len(ok) == 1, (n, c_load, c_cpu, ok)
        assert O.split_load_cpu(n, c_load, c_cpu) == ok[0]
    assert O.split_load_cpu(0, 1.0, 1.0) == (0, 0)


def test_algorithm2_balances_both_sides_and_is_near_the_best_split():
    """Section V-A: the goal is min max(n_load C_load, n_CPU C_CPU).  The
    two-pointer walk keeps the two sides within one item of each other and ends
    within one item of the brute-force optimum."""
    rng = np.random.default_rng(12)
    for _ in range(500):
        n = int(rng.integers(0, 65))
        cl, cc = float(rng.uniform(0.1, 10)), float(rng.uniform(0.1, 10))
        nl, ncpu = O.split_load_cpu(n, cl, cc)
        assert nl + ncpu == n and nl >= min(n, 1)
        big = max(cl, cc)
        if ncpu > 0:
            assert abs(nl * cl - ncpu * cc) <= big + 1e-9
        best = min(max(i * cl, (n - i) * cc) for i in range(n + 1))
        assert max(nl * cl, ncpu * cc) <= best + big + 1e-9


def test_cpu_assist_keeps_top_of_the_list_for_loading_and_cache_untouched_by_the_rest():
    """The highest-scoring missing experts are loaded (and cached), the
    lowest-scoring ones are computed on the CPU: they evict nobody, stay
    non-resident, and the layer output does not depend on where an expert ran."""
    shp = SHAPES["c4"].with_(n_layers=2, hidden=64, ffn=16, shared_ffn=16, n_experts=24, top_k=6,
                             cache_cap=8, alpha=0.1, tokens=30, seed=17)
    wl = make_workload(shp)
    a = O.oracle_from_workload(wl)
    b = O.oracle_from_workload(wl, cpu_assist=True, c_load=2.0, c_cpu=1.0)
    s = wl.shape
    seen_cpu = 0
    for t in range(s.tokens):
        for l in range(s.n_layers):
            G0 = set(b.layers[l].slot_expert)
            rb = b.decode_layer(l, as_numpy(wl.x[t, l]))
            missing = [int(e) for e in rb.final[0] if int(e) not in G0]
            assert rb.fetched + rb.on_cpu == missing               # slot order = descending score
            assert (len(rb.fetched), len(rb.on_cpu)) == O.split_load_cpu(len(missing), 2.0, 1.0)
            sc = rb.scores[0]
            if rb.fetched and rb.on_cpu:
                assert min(sc[e] for e in rb.topk[0][[list(rb.final[0]).index(m) for m in rb.fetched]]) > \
                       max(sc[e] for e in rb.topk[0][[list(rb.final[0]).index(m) for m in rb.on_cpu]])
            G1 = set(b.layers[l].slot_expert)
            assert not (set(rb.on_cpu) & G1) and set(rb.fetched) <= G1
            assert len(rb.victims) == len(rb.fetched) and len(G1) == s.cache_cap
            seen_cpu += len(rb.on_cpu)
            if t == 0:
                # before the caches diverge both oracles compute the same experts: same output
                ra = a.decode_layer(l, as_numpy(wl.x[t, l]))
                assert ra.final.tolist() == rb.final.tolist()
                np.testing.assert_array_equal(ra.y, rb.y)
    st = b.stats()
    assert seen_cpu == st.cpu_computed > 20
    assert st.fetches + st.cpu_computed == st.misses      # batch 1: every miss is loaded or computed
    assert st.evictions == st.fetches


def test_minmax_split_variant_is_the_brute_force_optimum_and_prefers_loading_on_ties():
    rng = np.random.default_rng(21)
    for _ in range(300):
        n = int(rng.integers(0, 40))
        cl, cc = float(rng.uniform(0.1, 10)), float(rng.uniform(0.1, 10))
        nl, ncpu = O.split_load_cpu_minmax(n, cl, cc)
        assert nl + ncpu == n
        times = [max(i * cl, (n - i) * cc) for i in range(n + 1)]
        assert max(nl * cl, ncpu * cc) == min(times)
        assert nl == max(i for i, t in enumerate(times) if t == min(times))
        # never worse than the two-pointer walk of Algorithm 2
        al, ac = O.split_load_cpu(n, cl, cc)
        assert max(nl * cl, ncpu * cc) <= max(al * cl, ac * cc) + 1e-12
    assert O.split_load_cpu_minmax(1, 3.0, 1.0) == (0, 1)      # a single miss goes to the faster side
    assert O.split_load_cpu_minmax(1, 1.0, 3.0) == (1, 0)
    assert O.split_load_cpu_minmax(2, 1.0, 1.0) == (1, 1)
    assert O.split_load_cpu_minmax(4, 3.0, 1.0) == (1, 3)


def test_adopted_prefetch_is_stamped_like_a_load_for_recency_policies():
    """LRU / FIFO with prefetch: a prefetched expert enters the cache at the step
    that uses it, so it carries that step's stamps -- under FIFO it is then the
    youngest load, not an old one."""
    E, H, k = 6, 8, 1
    gate = np.zeros((1, E, H), np.float32)
    for e in range(E):
        gate[0, e, e] = 1.0

    def x_for(e):
        x = np.zeros((1, H), np.float32)
        x[0, e] = 8.0
        return x
    experts = [np.zeros((E, 3 * H * 8), np.float32)]
    for policy, first_victim in ((O.EVICT_LRU, 2), (O.EVICT_FIFO, 0)):
        orc = O.SMoEOracle(n_layers=1, hidden=H, n_experts=E, ffn=8, top_k=k, cache_cap=3, alpha=0.0,
                           gate_w=gate, experts=experts, sim=np.eye(E, dtype=np.float32)[None],
                           init_resident=np.array([[0, 1, 2]]), elem_bytes=4, evict_policy=policy)
        orc.decode_layer(0, x_for(1), compute_y=False)             # step 0 uses 1
        orc.decode_layer(0, x_for(0), compute_y=False)             # step 1 uses 0
        pf = orc.prefetch_layer(0, x_for(4), 1)                    # predicts 4: not resident
        assert pf.prefetched == [4] and orc.layers[0].slot_expert == [0, 1, 2]
        r = orc.decode_layer(0, x_for(4), compute_y=False)         # step 2 uses 4: adopted, evicts 2
        assert r.adopted == [4] and r.fetched == [] and r.hit.all()
        # LRU: 2 was never used; FIFO: 0 is the earliest of the initial loads
        assert r.adopt_victims == [first_victim]
        r = orc.decode_layer(0, x_for(5), compute_y=False)         # step 3 loads 5
        # either way 1 goes next (LRU: last used at step 0; FIFO: the oldest load left);
        # expert 4 carries the stamps of step 2 and stays
        assert r.fetched == [5] and r.victims == [1]
        r = orc.decode_layer(0, x_for(3), compute_y=False)         # step 4 loads 3
        assert r.victims == [0 if policy == O.EVICT_LRU else 2]
        r = orc.decode_layer(0, x_for(1), compute_y=False)         # step 5 loads 1: now 4 is the oldest
        assert r.victims == [4]
        assert orc.stats().prefetches == 1 and orc.stats().prefetch_used == 1



# ---------------------------------------------------------------- batch > 1: the step as a whole
def _batch_step_from_definitions(scores, G, k, alpha, sim, subst_key):
    """One batched step rebuilt from the definitions (Table "Definitions",
    Algorithm 1's thresholds, Section IV-B / VI-B prose) without any oracle
    routine: per-token ranking by a full sort, the batch top-score set as the
    union over ALL tokens, substitution by exhaustive search of the greedy
    order, and the distinct misses in (token, slot) order."""
    B, E = scores.shape
    order = [sorted(range(E), key=lambda e: (-scores[t, e], e)) for t in range(B)]
    topk = [o[:k] for o in order]
    s_k1 = [scores[t, order[t][k]] for t in range(B)]
    top = [{e for e in topk[t] if scores[t, e] >= (1 + alpha) * s_k1[t]} for t in range(B)]
    C = set().union(*top)
    avail = set(G) | C
    final = []
    for t in range(B):
        f = list(topk[t])
        lows = [e for e in topk[t] if e not in top[t] and e not in avail]
        lows.sort(key=lambda e: (scores[t, e], -topk[t].index(e)))        # lowest score first
        cand = [c for c in range(E) if c not in topk[t] and c in avail
                and scores[t, c] >= (1 - alpha) * s_k1[t]]
        for b in lows:
            if not cand:
                break
            key = (lambda c: scores[t, c]) if subst_key == 1 else (lambda c: float(sim[b][c]))
            pick = max(cand, key=lambda c: (key(c), -c))
            f[topk[t].index(b)] = pick
            cand.remove(pick)
        final.append(f)
    distinct_misses = []
    for t in range(B):
        for e in final[t]:
            if e not in G and e not in distinct_misses:
                distinct_misses.append(e)
    hit = [[e in G for e in final[t]] for t in range(B)]
    return topk, final, C, distinct_misses, hit


@pytest.mark.parametrize("B", [2, 4])
@pytest.mark.parametrize("subst_key", [0, 1])
def test_batched_step_matches_the_definitions_bruteforce(B, subst_key):
    """Batch > 1 (Section IV-B prose "top-score experts of other tokens in the same
    batch", Section VI-B): every step of a replay is rebuilt from the definitions
    -- C = union over all tokens (not grown token by token), the history entry of
    Eq. 3 = the batch mean of the score vectors, distinct misses in (token, slot)
    order of first appearance, per-slot hits against G before the step."""
    shp = SHAPES["c4"].with_(hidden=64, ffn=16, shared_ffn=8, n_experts=14, top_k=3, cache_cap=6,
                             alpha=0.35, subst_key=subst_key, seed=60 + B)
    wl = make_workload(shp, n_layers=2, tokens=60, batch=B)
    s = wl.shape
    n = 2
    orc = O.oracle_from_workload(wl, evict_window=n)
    log = {l: [] for l in range(s.n_layers)}
    totals = dict(slots=0, hits=0, subs=0, fetches=0, staged=0, c_mattered=0, mean_mattered=0)
    for t in range(s.tokens):
        for l in range(s.n_layers):
            G = list(orc.layers[l].slot_expert)
            res = orc.decode_layer(l, as_numpy(wl.x[t, l]), compute_y=False)
            wg = wl.gate_w[l].to(torch.float64).numpy()
            xs = wl.x[t, l].to(torch.float64).numpy()
            sc = scipy.special.softmax(xs @ wg.T, axis=1)                  # [B, E]
            topk, final, C, misses, hit = _batch_step_from_definitions(
                sc, set(G), s.top_k, float(np.float32(s.alpha)), wl.sim[l].numpy(), subst_key)
            assert res.topk.tolist() == topk
            assert res.final.tolist() == final, (t, l)
            assert res.hit.tolist() == hit
            assert res.substituted.tolist() == [[a != b for a, b in zip(f, k_)] for f, k_ in zip(final, topk)]
            assert res.fetched == misses
            # would a C grown in token order have decided differently?  (sensitivity of this pin)
            grown = []
            for tt in range(B):
                tk1, fin1, _, _, _ = _batch_step_from_definitions(
                    sc[:tt + 1], set(G), s.top_k, float(np.float32(s.alpha)), wl.sim[l].numpy(), subst_key)
                grown.append(fin1[tt])
            totals["c_mattered"] += grown != final
            # Eq. 3 on the complete log, one entry per step = the batch mean
            log[l].append(sc.mean(axis=0))
            j = len(log[l])
            lo = max(1, j - n)
            avg = sum(log[l][i - 1] for i in range(lo, j + 1)) / (j - lo + 1)
            resident = list(G)
            shield = {e for f in final for e in f}
            for m, v in zip(res.fetched, res.victims):
                cand = [e for e in resident if e not in shield]
                if not cand:
                    assert v == -1
                    totals["staged"] += 1
                    continue
                want = min(cand, key=lambda e: (avg[e], e))
                assert v == want, (t, l)
                resident[resident.index(v)] = m
            assert resident == orc.layers[l].slot_expert
            totals["slots"] += B * s.top_k
            totals["hits"] += sum(map(sum, hit))
            totals["subs"] += int(res.substituted.sum())
            totals["fetches"] += len(misses)
    st = orc.stats()
    assert (st.slots, st.hits, st.substitutions, st.fetches) == (
        totals["slots"], totals["hits"], totals["subs"], totals["fetches"])
    assert st.misses == st.slots - st.hits and st.misses >= st.fetches
    assert totals["subs"] > 10 and totals["fetches"] > 20
    assert totals["c_mattered"] > 0       # the trace contains steps where the two readings of C differ


def test_batch_top_score_set_is_the_union_over_all_tokens_not_a_running_set():
    """Hand-made step (Algorithm 1 grows C inside the token loop, the prose
    speaks of the other tokens of the batch; the two-pass union is this build's
    reading): token 0's low-score expert 2 is not resident but is a top-score
    expert of token 1, which comes LATER in the batch.  Under the union it is
    kept; a C grown in token order would have replaced it by resident expert 3."""
    E, H, k = 6, 8, 2
    gate = np.zeros((1, E, H), np.float32)
    for e in range(E):
        gate[0, e, e] = 1.0
    x = np.zeros((2, H), np.float32)
    x[0, :E] = [3.0, -9.0, 1.00, 0.95, -9.0, -9.0]      # actives 0 (top), 2 (low); pivot 3
    x[1, :E] = [-9.0, -9.0, 4.0, -9.0, 3.0, 0.0]        # actives 2, 4: both top-score
    experts = [np.zeros((E, 3 * H * 8), np.float32)]
    orc = O.SMoEOracle(n_layers=1, hidden=H, n_experts=E, ffn=8, top_k=k, cache_cap=3, alpha=0.3,
                       gate_w=gate, experts=experts, sim=np.tile(np.eye(E, dtype=np.float32), (1, 1, 1)),
                       subst_key=1, init_resident=np.array([[0, 3, 5]]), elem_bytes=4)
    res = orc.decode_layer(0, x, compute_y=False)
    assert res.topk.tolist() == [[0, 2], [2, 4]]
    assert res.final.tolist() == [[0, 2], [2, 4]] and not res.substituted.any()
    assert res.fetched == [2, 4]                          # one load of expert 2 serves both tokens
    assert res.hit.tolist() == [[True, False], [False, False]]
    st = orc.stats()
    assert (st.hits, st.misses, st.fetches) == (1, 3, 2)  # hits and misses per slot, loads per distinct expert
    # the same token alone (batch 1: no C) does get the substitute
    orc.reset()
    alone = orc.decode_layer(0, x[:1], compute_y=False)
    assert alone.final.tolist() == [[0, 3]] and alone.substituted.tolist() == [[False, True]]


def test_batch_history_entry_is_the_batch_mean():
    """Eq. 3 at batch > 1 (the paper defines it per iteration j; one entry per
    decode step holding the batch mean is this build's reading): two tokens with
    opposite preferences, so that the victim differs depending on whose scores
    enter the history."""
    E, H, k = 5, 8, 1
    gate = np.zeros((1, E, H), np.float32)
    for e in range(E):
        gate[0, e, e] = 1.0
    # residents 0,1,2; both tokens activate resident 0 in step 1 (no load), then step 2 loads
    # expert 4 and must evict 1 or 2.  token 0 scores expert 1 high and 2 low; token 1 scores
    # 2 much higher than token 0 scores 1: batch mean says evict 1, token 0 alone says evict 2.
    x1 = np.zeros((2, H), np.float32)
    x1[0, :E] = [5.0, 2.0, 0.0, -5.0, -5.0]
    x1[1, :E] = [5.0, 0.0, 4.0, -5.0, -5.0]
    x2 = np.zeros((2, H), np.float32)
    x2[0, :E] = [-5.0, 2.0, 0.0, -5.0, 6.0]
    x2[1, :E] = [-5.0, 0.0, 4.0, -5.0, 6.0]
    experts = [np.zeros((E, 3 * H * 8), np.float32)]
    orc = O.SMoEOracle(n_layers=1, hidden=H, n_experts=E, ffn=8, top_k=k, cache_cap=3, alpha=0.0,
                       gate_w=gate, experts=experts, sim=np.eye(E, dtype=np.float32)[None],
                       init_resident=np.array([[0, 1, 2]]), elem_bytes=4, evict_window=3)
    r1 = orc.decode_layer(0, x1, compute_y=False)
    assert r1.fetched == []
    r2 = orc.decode_layer(0, x2, compute_y=False)
    assert r2.fetched == [4]
    s1 = scipy.special.softmax(x1[:, :E].astype(np.float64), axis=1)
    s2 = scipy.special.softmax(x2[:, :E].astype(np.float64), axis=1)
    mean = (s1.mean(axis=0) + s2.mean(axis=0)) / 2
    tok0 = (s1[0] + s2[0]) / 2
    by_mean = min([0, 1, 2], key=lambda e: mean[e])
    by_tok0 = min([0, 1, 2], key=lambda e: tok0[e])
    assert by_mean != by_tok0                     # the case separates the two readings
    assert r2.victims == [by_mean]


def test_batch_recency_stamps_follow_token_slot_order_lru_textbook():
    """alpha = 0, batch 2, LRU: the step's accesses are the (token, slot) pairs in
    order; an OrderedDict cache fed with that access sequence (the step's experts
    pinned while its misses are placed, misses placed in first-appearance order)
    must evict the same experts."""
    from collections import OrderedDict
    shp = SHAPES["c4"].with_(hidden=64, ffn=16, shared_ffn=8, n_experts=12, top_k=2, cache_cap=7,
                             alpha=0.0, evict_policy=O.EVICT_LRU, seed=77)
    wl = make_workload(shp, n_layers=1, tokens=80, batch=2)
    orc = O.oracle_from_workload(wl)
    cache = OrderedDict((e, None) for e in range(shp.cache_cap))
    logits = torch.einsum("eh,tbh->tbe", wl.gate_w[0].double(), wl.x[:, 0].double())
    top = torch.topk(logits, shp.top_k, dim=-1).indices.tolist()            # [T][B][k]
    evictions = 0
    for t in range(wl.shape.tokens):
        res = orc.decode_layer(0, as_numpy(wl.x[t, 0]), compute_y=False)
        accesses = [e for tok in top[t] for e in tok]
        pinned = set(accesses)
        before = set(cache)
        for e in accesses:                       # recency of everything the step touches
            if e in cache:
                cache.move_to_end(e)
        want_victims, loaded = [], []
        for e in accesses:
            if e in before or e in loaded:
                continue
            victim = next(c for c in cache if c not in pinned)
            del cache[victim]
            want_victims.append(victim)
            loaded.append(e)
        # loaded experts enter with the recency of their first access in the step
        for e in accesses:
            if e in loaded and e not in cache:
                cache[e] = None
        for e in accesses:
            cache.move_to_end(e)
        assert res.fetched == loaded and res.victims == want_victims, t
        assert set(orc.layers[0].slot_expert) == set(cache)
        evictions += len(loaded)
    assert evictions > 30


# ---------------------------------------------------------------- the predictor's state (Section IV-C)
def test_partial_output_is_the_output_minus_the_experts_that_had_to_be_loaded(c1_workload):
    """y_partial (what the prediction starts from) = shared experts + the slots
    whose expert was in G before the step; recomputed here from the dense
    expert outputs and the returned weights.  With nothing to load it is y."""
    wl = c1_workload
    s = wl.shape
    orc = O.oracle_from_workload(wl)
    saw_loaded = saw_equal = 0
    for t in range(s.tokens):
        for l in range(s.n_layers):
            G = set(orc.layers[l].resident)
            x = as_numpy(wl.x[t, l])
            res = orc.decode_layer(l, x)
            xt = torch.from_numpy(O.widen(x[0]))
            want = np.zeros(s.hidden)
            for j, e in enumerate(res.final[0]):
                if int(e) in G:
                    w1, w3, w2 = (m.to(torch.float64) for m in wl.expert_mats(l, int(e)))
                    want += res.weights[0, j] * (w2 @ (torch.nn.functional.silu(w1 @ xt) * (w3 @ xt))).numpy()
            np.testing.assert_allclose(res.y_partial[0], want, rtol=1e-10, atol=1e-14)
            if res.fetched:
                saw_loaded += 1
                assert not np.allclose(res.y_partial, res.y, rtol=1e-6, atol=0)
            else:
                saw_equal += 1
                np.testing.assert_array_equal(res.y_partial, res.y)
    assert saw_loaded > 3 and saw_equal > 3
    # shared experts are always on the GPU: with every routed expert resident too, the partial
    # output is the whole output (which the dense-library pin above fixes, shared experts included)
    shp = SHAPES["c4"].with_(hidden=128, ffn=96, shared_ffn=64, n_experts=16, cache_cap=16, top_k=4, sim="uniform")
    wl = make_workload(shp, n_layers=1, tokens=2)
    res = O.oracle_from_workload(wl).decode_layer(0, as_numpy(wl.x[0, 0]))
    np.testing.assert_array_equal(res.y_partial, res.y)
    assert np.abs(res.y).max() > 0


def test_predicted_state_is_the_unit_rms_residual_sum():
    rng = np.random.default_rng(2)
    orc = O.oracle_from_workload(make_workload(SHAPES["c1"].with_(tokens=1)))
    x = rng.normal(size=(3, 64)).astype(np.float32)
    yp = rng.normal(size=(3, 64)) * 0.3
    xp = orc.predict_state(x, yp)
    np.testing.assert_allclose(np.sqrt((xp ** 2).mean(axis=1)), 1.0, rtol=1e-13)           # unit RMS
    z = x.astype(np.float64) + yp
    cos = (xp * z).sum(axis=1) / np.linalg.norm(xp, axis=1) / np.linalg.norm(z, axis=1)
    np.testing.assert_allclose(cos, 1.0, rtol=1e-13)                                       # direction of x + y
    np.testing.assert_allclose(orc.predict_state(4.0 * x, 4.0 * yp), xp, rtol=1e-13)       # scale-free
    unit = x / np.sqrt((x.astype(np.float64) ** 2).mean(axis=1, keepdims=True))
    np.testing.assert_allclose(orc.predict_state(unit, np.zeros_like(yp)), unit, rtol=1e-6)  # fixed point
    # hand case: x + y = (3, 4, 0, 0): rms = sqrt(25/4) = 2.5
    np.testing.assert_allclose(orc.predict_state(np.array([[1.0, 4.0, 0.0, -1.0]], np.float32),
                                                 np.array([[2.0, 0.0, 0.0, 1.0]])), [[1.2, 1.6, 0.0, 0.0]])


# ---------------------------------------------------------------- Algorithm 2 and prefetches in flight
def _identity_gate_oracle(E, k, cap, **kw):
    """Gate = identity on the first E coordinates: the logits are x[:E], so a test
    chooses the score order directly."""
    H = max(8, E)
    gate = np.zeros((1, E, H), np.float32)
    for e in range(E):
        gate[0, e, e] = 1.0
    rng = np.random.default_rng(3)
    experts = [rng.normal(0, 0.05, size=(E, 3 * H * 8)).astype(np.float32)]
    return O.SMoEOracle(n_layers=1, hidden=H, n_experts=E, ffn=8, top_k=k, cache_cap=cap, alpha=0.0,
                        gate_w=gate, experts=experts, sim=np.eye(E, dtype=np.float32)[None],
                        init_resident=np.array([list(range(cap))]), elem_bytes=4, **kw), H


def _x_with_order(H, order):
    x = np.zeros((1, H), np.float32)
    for r, e in enumerate(order):
        x[0, e] = 6.0 - 0.5 * r                    # order[0] scores highest
    return x


def test_in_flight_prefetches_join_algorithm_2_hand_case():
    """Section V-A with Section V-B dependency 2.  E = 8, top-4, G = {0, 1, 2, 3}.  The step
    computes 5, 4, 0, 6 (descending score); 5 and 6 were prefetched, 4 is missing.
    With equal costs the two workers of Algorithm 2 alternate, the loader first:
      * both prefetches complete: only 4 waits -> it is loaded; 5 and 6 are adopted;
      * both still in flight: the step waits for 5, 4, 6 -> 5 stays on the link and is
        adopted, 6 (tail of the list) goes to the host cores and its prefetch is
        dropped -- never adopted, never cached -- and 4 is loaded;
      * only 6 in flight: the step waits for 4, 6 -> 4 is loaded, 6 goes to the host cores."""
    E, k, cap = 8, 4, 4
    order = [5, 4, 0, 6]
    for inflight, want_cpu, want_fetched, want_adopted in (
            (set(), [], [4], [5, 6]),
            ({5, 6}, [6], [4], [5]),
            ({6}, [6], [4], [5])):
        orc, H = _identity_gate_oracle(E, k, cap, cpu_assist=1, c_load=1.0, c_cpu=1.0)
        pf = orc.prefetch_layer(0, _x_with_order(H, [5, 6, 0, 1]), 2)
        assert pf.prefetched == [5, 6]
        r = orc.decode_layer(0, _x_with_order(H, order), inflight=inflight)
        assert r.final[0].tolist() == order
        assert r.hit[0].tolist() == [True, False, True, True]      # prefetched experts count as on the GPU
        assert (r.on_cpu, r.fetched, r.adopted) == (want_cpu, want_fetched, want_adopted)
        G = set(orc.layers[0].slot_expert)
        assert len(G) == cap and set(want_fetched + want_adopted + [0]) <= G and not (set(want_cpu) & G)
        assert orc.layers[0].landed == [] and all(v in (1, 2, 3) for v in r.victims + r.adopt_victims)
        st = orc.stats()
        assert (st.cpu_computed, st.fetches, st.prefetch_used) == (len(want_cpu), 1, 2)


def test_in_flight_takeover_rebuilt_from_the_definitions_bruteforce():
    """Random steps: the waiting list is, in descending score, every expert the step
    computes that is neither in G nor a prefetch whose copy has finished; Algorithm 2
    splits it head / tail; the head is loaded or adopted, the tail computed on the
    host cores; prefetched experts the step does not compute, or that went to the
    host cores, leave the queue."""
    rng = np.random.default_rng(12)
    E, k, cap = 12, 5, 6
    seen_takeover = 0
    for trial in range(200):
        cl, cc = float(rng.uniform(0.5, 4)), float(rng.uniform(0.5, 4))
        orc, H = _identity_gate_oracle(E, k, cap, cpu_assist=1, c_load=cl, c_cpu=cc)
        pred = list(rng.permutation(E)[:k])
        pf = orc.prefetch_layer(0, _x_with_order(H, pred), 3)
        landed = list(pf.prefetched)
        order = [int(e) for e in rng.permutation(E)[:k]]
        inflight = set(e for e in landed if rng.random() < 0.5)
        G0 = set(orc.layers[0].slot_expert)
        r = orc.decode_layer(0, _x_with_order(H, order), inflight=inflight)
        assert r.final[0].tolist() == order                          # alpha = 0: no substitution
        waiting = [e for e in order if e not in G0 and (e not in landed or e in inflight)]
        n_load, n_cpu = O.split_load_cpu(len(waiting), cl, cc)
        head, tail = waiting[:n_load], waiting[n_load:]
        assert r.on_cpu == tail
        assert r.fetched == [e for e in order if e not in G0 and e not in landed and e not in tail]
        assert r.adopted == [e for e in order if e in landed and e not in tail]
        assert sorted(r.dropped) == sorted(e for e in landed if e not in order)
        assert not (set(tail) & set(orc.layers[0].slot_expert))
        seen_takeover += len(set(tail) & inflight)
    assert seen_takeover > 20


def test_batched_prefetch_list_is_token_by_token_without_repeats_and_capped_by_the_spare_slots():
    """Hand case, batch 3, G = {0, 1, 2, 3}, alpha = 0 (every predicted top-k expert is
    top-score).  Predicted top-3 per token: (5, 0, 6), (6, 7, 1), (8, 5, 9).  Wanted, in
    load order: 5, 6 from token 0 (0 is resident), then 7 (6 is a repeat, 1 resident),
    then 8, 9 (5 a repeat).  Three spare slots take 5, 6, 7; a second prediction for the
    same layer wants only what is not waiting yet and finds no room."""
    orc, H = _identity_gate_oracle(10, 3, 4)
    xp = np.concatenate([_x_with_order(H, o) for o in ([5, 0, 6], [6, 7, 1], [8, 5, 9])])
    pf = orc.prefetch_layer(0, xp, 3)
    assert pf.wanted == [5, 6, 7, 8, 9] and pf.prefetched == [5, 6, 7]
    assert pf.topk.tolist() == [[5, 0, 6], [6, 7, 1], [8, 5, 9]]
    again = orc.prefetch_layer(0, xp, 3)
    assert again.wanted == [8, 9] and again.prefetched == []
    assert orc.layers[0].landed == [5, 6, 7] and orc.layers[0].slot_expert == [0, 1, 2, 3]
    assert orc.stats().prefetches == 3
    # the batched step then adopts what it computes, in (token, slot) order, and drops the rest
    x = np.concatenate([_x_with_order(H, o) for o in ([6, 0, 1], [2, 5, 0], [0, 1, 2])])
    r = orc.decode_layer(0, x)
    assert r.adopted == [6, 5] and r.dropped == [7] and r.fetched == []
    assert r.adopt_victims == [3, -1]            # shield {6,0,1,2,5}: only 3 is evictable, 5 is not kept
    assert orc.layers[0].slot_expert == [0, 1, 2, 6]
