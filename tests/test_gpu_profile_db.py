"""The install-phase benchmark suite that fills the profile database (Section 3: kernels timed as
a batch of asynchronous launches), and plans priced from it, on the GPU."""
import numpy as np
import pytest

import synth_inputs as S
from tests import harness as Hn
from oracle import oracle as O

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def test_benchmark_suite_fills_the_database_and_prices_a_plan():
    import torch
    from paper_2604_26334_amd import binding as B
    cfg = dict(Hn.small_dense_cfg(2), vocab=2064)
    H, I = cfg["hidden"], cfg["ffn_inter"]
    db = B.ProfileDB()
    db.measure(cfg, scratch_bytes=768 << 20)
    ent = db.entries()
    _say("  %d entries" % len(ent))
    assert all(e[6] > 0 and np.isfinite(e[6]) for e in ent)
    shapes = {((cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * 128, H), (H, cfg["n_q_heads"] * 128), (2 * I, H), (H, I), (2064, H)}
    gemv = {(e[3], e[4]) for e in ent if e[0] == B.PS_OPK_GEMV}
    assert gemv == shapes
    tiers = sorted({e[5] for e in ent if e[0] == B.PS_OPK_GEMM})
    assert tiers == [4, 16, 32, 64, 512, 1024, 2048]
    assert len([e for e in ent if e[0] == B.PS_OPK_GEMM]) == len(shapes) * len(tiers)
    assert sorted(e[3] for e in ent if e[0] == B.PS_OPK_H2D) == [1 << 20, 4 << 20, 16 << 20, 64 << 20]
    cpu = [e for e in ent if e[0] == B.PS_OPK_CPU]
    if cpu:   # hosts with AVX-512: the FFN and head matrices at four token counts, one thread count
        assert {(e[3], e[4]) for e in cpu} == {(2 * I, H), (H, I), (2064, H)} and len({e[2] for e in cpu}) == 1
        assert sorted({e[5] for e in cpu}) == [1, 2, 4, 8, 16, 64]
    # larger copies are not slower per byte; the 64 MiB copy runs at a plausible PCIe rate
    h2d = {e[3]: e[6] for e in ent if e[0] == B.PS_OPK_H2D}
    rate = (64 << 20) / (h2d[64 << 20] * 1e-3) / 1e9
    _say("  H2D 64 MiB: %.1f GB/s; GEMV %s" % (rate, {(e[3], e[4]): round(e[6] * 1e3, 1) for e in ent if e[0] == B.PS_OPK_GEMV}))
    assert 5.0 < rate < 200.0
    # the model's own shapes are exact matches; a slab of one is a neighbour
    r = db.estimate(5000.0, B.PS_OPK_GEMV, 4, 0, 2 * I, H, 1)
    assert r.match == B.PS_MATCH_EXACT
    r2 = db.estimate(5000.0, B.PS_OPK_GEMV, 4, 0, I, H, 1)
    assert r2.match == B.PS_MATCH_NEIGHBOUR and 0 < r2.ms < r.ms * 10     # (kernels this small are launch-bound)
    # a plan priced from the database runs like any other
    prof = B.make_profile(h2d_gbps=rate, gemv_gbps=5000.0, cpu_gbps=150.0 if cpu else 0.0, cpu_sync_us=40.0)
    full = B.Plan(cfg, 1 << 40, 1).summary()
    budget = full.workspace_bytes + full.weight_bytes // 2
    kinds = [B.PS_PLAN_GPU_ONLY] + ([B.PS_PLAN_AUTO] if cpu else [])
    W = Hn.WeightCache(cfg, 21)
    head = S.head_matrix(21, cfg)
    x = S.activations(21, 0, 1, H)
    ref = O.stack_forward(x, cfg, W, mirror=True)
    for kind in kinds:
        plan = B.Plan(cfg, budget, 1, profile=prof, kind=kind, db=db)
        s = plan.summary()
        _say("  kind %d -> plan %d, estimate %.3f ms (estimates per kind %s)" % (kind, s.plan_kind, s.est_step_ms, [round(v, 3) for v in s.est_kind_ms]))
        assert s.est_step_ms > 0
        st = B.Stack(plan)
        for layer in range(cfg["n_layers"]):
            for k, e, N, K in S.matrix_shapes(cfg):
                st.load_matrix(layer, k, e, *W(layer, k, e))
        st.load_matrix(cfg["n_layers"], S.MAT_OUT, None, *head)
        xin = torch.from_numpy(x).to(st.device)
        xout = torch.empty_like(xin)
        st.forward(xin, xout)
        st.synchronize()
        assert Hn.rel_err(xout.cpu().numpy(), ref) <= 5e-3
        st.close()
        plan.close()


def test_tier_table_priced_from_the_measured_database_serves_one_stack():
    """Overview steps 1-4 in one go: the benchmark suite fills the database, the planning phase prices every
    tier's schedule from it (HeuristicSplit per tier where the host has the CPU back-end), PickTier chooses
    the prefill tier from those estimates, and one stack runs the prefill in that tier and a decode step in
    the one-token tier, each against the oracle."""
    import torch
    from paper_2604_26334_amd import binding as B
    cfg = Hn.small_dense_cfg(3)
    db = B.ProfileDB()
    db.measure(cfg, scratch_bytes=768 << 20)
    has_cpu = any(e[0] == B.PS_OPK_CPU for e in db.entries())
    prof = B.make_profile(h2d_gbps=50.0, gemv_gbps=5000.0, cpu_gbps=150.0 if has_cpu else 0.0, cpu_gbps_busy=140.0 if has_cpu else 0.0,
                          h2d_gbps_busy=48.0, cpu_sync_us=40.0)
    wb, _ = Hn.total_weight_bytes(cfg)
    full = B.Plan(cfg, 1 << 40, 512).summary()
    budget = full.workspace_bytes + int(wb * 0.25)
    table = B.TierTable(cfg, budget, profile=prof, db=db, kind=B.PS_PLAN_AUTO if has_cpu else None)
    ents = [e for e in table.entries() if e.feasible]
    assert {1, 512} <= {e.tier_tokens for e in ents}
    for e in ents:   # every tier's estimate is the database-priced plan's
        alone = B.Plan(cfg, budget, e.tier_tokens, profile=prof, db=db,
                       kind=B.PS_PLAN_AUTO if (has_cpu and e.tier_tokens <= 64) else B.PS_PLAN_GPU_ONLY).summary()
        assert e.summary.est_step_ms == alone.est_step_ms and e.summary.est_step_ms > 0
    n = 600
    c = table.pick(n)
    _say("  tiers %s; PickTier for %d tokens: %d x %d trips, estimate %.3f ms" % (
        [(e.tier_tokens, e.summary.plan_kind, round(e.summary.est_step_ms, 3)) for e in ents], n, c.tier_tokens, c.iterations, c.est_total_ms))
    best = min(-(-n // e.tier_tokens) * e.summary.est_step_ms for e in ents)
    assert c.est_total_ms == pytest.approx(best)
    W = Hn.WeightCache(cfg, 29)
    st = B.Stack(table)
    for layer in range(cfg["n_layers"]):
        for k, e, N, K in S.matrix_shapes(cfg):
            st.load_matrix(layer, k, e, *W(layer, k, e))
    x = S.activations(29, 0, n, cfg["hidden"])
    st.set_tier(c.tier)
    xin = torch.from_numpy(x).to(st.device)
    xout = torch.zeros_like(xin)
    assert B.chunked_forward(st, xin, xout) == c.iterations
    st.synchronize()
    assert Hn.rel_err(xout.cpu().numpy(), O.stack_forward(x, cfg, W, mirror=True)) <= 5e-3
    st.set_tier(0)
    x1 = S.activations(29, 1, 1, cfg["hidden"])
    xin = torch.from_numpy(x1).to(st.device)
    xout = torch.zeros_like(xin)
    st.forward(xin, xout)
    st.synchronize()
    assert Hn.rel_err(xout.cpu().numpy(), O.stack_forward(x1, cfg, W, mirror=True)) <= 5e-3
    st.close()
