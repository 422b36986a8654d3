"""The seeded input generator: determinism, shapes, the logit margin audit."""
import numpy as np
import torch

from smoe_inputs import SHAPES, make_workload, logit_margin_ok


def test_shapes_and_determinism():
    s = SHAPES["c1"]
    a, b = make_workload(s), make_workload(s)
    assert a.x.shape == (16, 2, 1, 256) and a.x.dtype == torch.float32
    assert len(a.experts) == 2 and a.experts[0].shape == (8, 3 * 256 * 512)
    for f in ("gate_w", "sim", "x"):
        assert torch.equal(getattr(a, f), getattr(b, f))
    assert all(torch.equal(p, q) for p, q in zip(a.experts, b.experts))
    c = make_workload(s.with_(seed=1))
    assert not torch.equal(a.x, c.x)
    assert abs(float(a.experts[0].std()) - 0.02) < 1e-4
    al = make_workload(s.with_(n_layers=4), distinct_layers=2)
    assert al.experts[2] is al.experts[0] and al.experts[3] is al.experts[1]
    assert not torch.equal(al.gate_w[0], al.gate_w[2])


def test_byte_counts_match_the_workload_table():
    assert SHAPES["c1"].expert_bytes == 1_572_864
    assert SHAPES["c2"].expert_bytes == 17_301_504
    assert SHAPES["c3"].expert_bytes == 352_321_536
    assert SHAPES["c5"].expert_bytes == 55_050_240
    assert abs(SHAPES["c3"].layer_bytes() - 704.7e6) < 0.1e6
    assert abs(SHAPES["c4"].layer_bytes() - 138.7e6) < 0.1e6
    assert abs(SHAPES["c5"].layer_bytes() - 881.3e6) < 0.1e6


def test_cosine_table_properties():
    wl = make_workload(SHAPES["c1"])
    sim = wl.sim.numpy()
    assert np.array_equal(sim, np.transpose(sim, (0, 2, 1)))
    assert (np.diagonal(sim, axis1=1, axis2=2) == 1).all()
    e0 = wl.experts[0][0].double()
    e3 = wl.experts[0][3].double()
    want = float(e0 @ e3 / (e0.norm() * e3.norm()))
    assert abs(sim[0, 0, 3] - want) < 1e-7


def test_margin_audit_holds_on_realised_logits():
    for name, kw in (("c1", {}), ("c2", dict(n_layers=1, tokens=24)),
                     ("c4", dict(n_layers=2, tokens=24)), ("c5", dict(n_layers=2, tokens=24, batch=2))):
        shp = SHAPES[name]
        if name in ("c4", "c5"):
            shp = shp.with_(ffn=32, shared_ffn=32)
        wl = make_workload(shp, **kw)
        s = wl.shape
        logits = torch.einsum("leh,tlbh->tlbe", wl.gate_w.double(), wl.x.double()).numpy()
        ok = logit_margin_ok(logits.reshape(-1, s.n_experts), s.top_k, s.alpha)
        assert ok.all()


def test_margin_audit_rejects_near_ties_and_threshold_grazes():
    base = np.array([[3.0, 2.0, 1.0, 0.0, -1.0, -6.0]])
    assert logit_margin_ok(base, 2, 0.3).all()
    tie = base.copy(); tie[0, 1] = 3.0 - 1e-5
    assert not logit_margin_ok(tie, 2, 0.3).any()
    graze_hi = base.copy(); graze_hi[0, 1] = 1.0 + np.log1p(0.3) + 1e-5
    assert not logit_margin_ok(graze_hi, 2, 0.3).any()
    graze_lo = base.copy(); graze_lo[0, 3] = 1.0 + np.log1p(-0.3) - 1e-5
    assert not logit_margin_ok(graze_lo, 2, 0.3).any()


def test_zipf_prior_skews_expert_popularity_and_locality_repeats():
    shp = SHAPES["c5"].with_(ffn=32, shared_ffn=32)
    wl = make_workload(shp, n_layers=1, tokens=200)
    logits = torch.einsum("eh,tbh->tbe", wl.gate_w[0].double(), wl.x[:, 0].double())
    top = torch.topk(logits, shp.top_k, dim=-1).indices[:, 0]       # [T, k]
    counts = torch.bincount(top.reshape(-1), minlength=shp.n_experts).double()
    srt = torch.sort(counts, descending=True).values
    assert srt[:8].sum() > 3 * srt[-32:].sum()                      # heavy head
    reuse = np.mean([len(set(top[t].tolist()) & set(top[t - 1].tolist())) for t in range(1, 200)])
    nolocal = make_workload(shp.with_(locality_p=0.0), n_layers=1, tokens=200)
    l2 = torch.einsum("eh,tbh->tbe", nolocal.gate_w[0].double(), nolocal.x[:, 0].double())
    t2 = torch.topk(l2, shp.top_k, dim=-1).indices[:, 0]
    reuse0 = np.mean([len(set(t2[t].tolist()) & set(t2[t - 1].tolist())) for t in range(1, 200)])
    assert reuse > reuse0 + 1.0


def test_predicted_states_are_seeded_audited_and_leave_x_unchanged():
    from smoe_inputs.generate import logit_margin_ok
    shp = SHAPES["c4"].with_(n_layers=2, hidden=256, ffn=8, shared_ffn=8, n_shared=0, tokens=12, seed=9)
    base = make_workload(shp)
    a = make_workload(shp, pred_noise=0.4)
    b = make_workload(shp, pred_noise=0.4)
    assert base.x_pred is None
    assert torch.equal(base.x, a.x) and torch.equal(base.gate_w, a.gate_w)      # x does not depend on the request
    assert torch.equal(a.x_pred, b.x_pred)                                       # seeded
    assert a.x_pred.shape == a.x.shape and a.x_pred.dtype == a.x.dtype
    diff = (a.x_pred.double() - a.x.double())
    assert 0.3 < float(diff.std()) < 0.5                                         # sigma = 0.4 plus rounding
    # every predicted token-layer passes the same logit-margin audit as x
    wg = a.gate_w.double().numpy()
    for l in range(shp.n_layers):
        logits = a.x_pred[:, l, 0].double().numpy() @ wg[l].T
        assert logit_margin_ok(logits, shp.top_k, shp.alpha).all()
    zero = make_workload(shp, pred_noise=0.0)
    assert torch.equal(zero.x_pred, zero.x)


def test_chained_input_is_the_unit_rms_residual_sum_in_the_checking_and_the_running_precision():
    import torch
    from smoe_inputs import chain_next_input
    g = torch.Generator().manual_seed(5)
    x = torch.randn(3, 96, generator=g).to(torch.bfloat16)
    y64 = torch.randn(3, 96, generator=g, dtype=torch.float64) * 0.1
    z = x.double() + y64
    want = z / z.pow(2).mean(dim=1, keepdim=True).sqrt()
    got64 = chain_next_input(x, y64)
    assert got64.dtype == torch.float64 and torch.allclose(got64, want, rtol=1e-13, atol=0)
    got32 = chain_next_input(x, y64.to(torch.bfloat16))          # what a run on the device computes
    assert got32.dtype == torch.float32
    z32 = x.double() + y64.to(torch.bfloat16).double()
    assert torch.allclose(got32.double(), z32 / z32.pow(2).mean(dim=1, keepdim=True).sqrt(), rtol=1e-5)
    assert torch.allclose(got64.pow(2).mean(dim=1), torch.ones(3, dtype=torch.float64), rtol=1e-13)
