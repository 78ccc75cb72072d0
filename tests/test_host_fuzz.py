"""Seeded sweep over model shapes, budgets, token counts and plan kinds: whatever the planner
accepts must cover every matrix exactly once, stay inside the budget, and give a schedule the
vector-clock checker accepts.  Host only."""
import numpy as np
import pytest

import synth_inputs as S
from paper_2604_26334_amd import binding as B


def _random_cfg(rng):
    moe = rng.random() < 0.35
    attn = rng.random() < 0.8
    hidden = int(rng.choice([128, 256, 512, 1024]))
    n_kv = int(rng.choice([1, 2, 4]))
    cfg = dict(n_layers=int(rng.integers(1, 5)), hidden=hidden, n_q_heads=n_kv * int(rng.choice([1, 2, 4])) if attn else 0,
               n_kv_heads=n_kv if attn else 0, head_dim=128 if attn else 0,
               ffn_inter=0 if moe else 128 * int(rng.integers(1, 12)), n_experts=int(rng.choice([4, 8, 16])) if moe else 0,
               top_k=0, expert_inter=128 * int(rng.integers(1, 4)) if moe else 0, rms_eps=1e-6,
               no_attn=not attn, no_residual=bool(rng.random() < 0.2) and not moe)   # (the flag is the bare dense FFN block's)
    if moe:
        cfg["top_k"] = int(rng.integers(1, min(4, cfg["n_experts"]) + 1))
    if rng.random() < 0.4:
        cfg["vocab"] = 16 * int(rng.integers(1, 300))
    if attn and rng.random() < 0.3:
        cfg["kv_context"] = int(rng.integers(1, 600))
    return cfg


def _check_plan(cfg, plan, M, logits):
    s = plan.summary()
    sh = plan.shards()
    assert s.resident_bytes + s.streamed_bytes + s.cpu_bytes == s.weight_bytes == sum(x.bytes for x in sh)
    assert s.workspace_bytes + s.scratch_bytes + s.resident_bytes <= s.budget_bytes
    # every matrix: its shards tile [0, ntiles) once, in order; whole shards appear once
    groups = {}
    for x in sh:
        groups.setdefault((x.layer, x.kind, x.expert), []).append(x)
    for (layer, kind, expert), v in groups.items():
        if kind in (B.PS_SHARD_EXPERT, B.PS_SHARD_KV):
            assert len(v) == 1
        else:
            assert [y.tile0 for y in v] == [sum(z.ntiles for z in v[:i]) for i in range(len(v))]
            order = [{1: 0, 0: 1, 2: 2}[y.resident] for y in v]
            assert order == sorted(order)                       # pinned head, streamed slabs, CPU tail
        for y in v:
            if y.resident == 0:
                assert s.n_slots == 2 and y.bytes <= s.slot_bytes
            if y.resident == 2:
                assert kind in (B.PS_SHARD_GATE_UP, B.PS_SHARD_DOWN, B.PS_SHARD_OUT, B.PS_SHARD_EXPERT)
                assert s.plan_kind != B.PS_PLAN_GPU_ONLY
    # pinned shards do not overlap, start the arena in priority order, and end before scratch and workspace
    res = sorted((x.offset, x.bytes) for x in sh if x.resident == 1)
    for (o0, b0), (o1, _) in zip(res, res[1:]):
        assert o0 + b0 <= o1
    if res:
        assert res[0][0] == 0 and res[-1][0] + res[-1][1] + s.scratch_bytes + s.workspace_bytes <= s.budget_bytes
        by_rank = sorted((x.priority_rank, x.offset) for x in sh if x.resident == 1)
        assert [o for _, o in by_rank] == sorted(o for _, o in by_rank)
    sched = plan.schedule(logits)
    assert sched.validate() is None
    ops = sched.ops()
    assert sum(o.bytes for o in ops if o.type == B.PS_OP_COPY) <= s.streamed_bytes
    if not cfg["n_experts"]:
        assert sum(o.bytes for o in ops if o.type == B.PS_OP_COPY) == s.streamed_bytes
        assert sum(o.bytes for o in ops if o.type == B.PS_OP_CPU) == s.cpu_bytes
    assert s.est_step_ms >= 0 and np.isfinite(s.est_step_ms)


@pytest.mark.parametrize("seed", range(6))
def test_random_models_budgets_and_plan_kinds(seed):
    rng = np.random.default_rng(1000 + seed)
    prof = B.make_profile(h2d_gbps=50.0, gemv_gbps=4000.0, cpu_gbps=float(rng.choice([20.0, 150.0, 2000.0])),
                          cpu_gbps_busy=float(rng.choice([0.0, 100.0])), h2d_gbps_busy=40.0, cpu_tokens_free=3.0,
                          cpu_sync_us=float(rng.choice([0.5, 40.0])))
    built = rejected = 0
    for _ in range(60):
        cfg = _random_cfg(rng)
        M = 1 if cfg.get("kv_context") else int(rng.choice([1, 1, 3, 16, 64, 200]))
        logits = S.router_logits(int(rng.integers(1 << 30)), 0, cfg["n_layers"], M, cfg["n_experts"]) if cfg["n_experts"] else None
        freq = rng.random((cfg["n_layers"], cfg["n_experts"])).astype(np.float32) if cfg["n_experts"] and rng.random() < 0.5 else None
        full = B.Plan(cfg, 1 << 40, M).summary()
        budget = full.workspace_bytes + int(full.weight_bytes * rng.choice([0.02, 0.1, 0.3, 0.6, 0.95, 1.2]))
        for kind in (None, B.PS_PLAN_GPU_ONLY, B.PS_PLAN_STATIC, B.PS_PLAN_DYNAMIC, B.PS_PLAN_AUTO):
            try:
                plan = B.Plan(cfg, budget, M, profile=prof, expert_freq=freq, kind=kind)
            except B.PshardError as e:
                # too small for the workspace plus two slots, or a CPU plan asked for more than 64 tokens
                assert e.code in (B.PS_E_BUDGET, B.PS_E_ARG), (cfg, budget, M, kind, str(e))
                if e.code == B.PS_E_ARG:
                    assert M > 64 and kind in (B.PS_PLAN_STATIC, B.PS_PLAN_DYNAMIC)
                rejected += 1
                continue
            _check_plan(cfg, plan, M, logits)
            if kind == B.PS_PLAN_AUTO:
                est = [e for e in plan.summary().est_kind_ms if e >= 0]
                assert plan.summary().est_step_ms == pytest.approx(min(est))
            built += 1
            plan.close()
    assert built > 100, (built, rejected)
