"""GPU parity of the plans that leave shards in system memory and run them on the CPU (Section 3,
Plan Two "static" and Plan Three "dynamic", and HeuristicSplit's choice among the three): the
whole stack through the C ABI against the CPU oracle at max|err| / max|ref| <= 5e-3.  Rows computed
by the CPU back-end and by a GPU kernel sum in different orders, so across plan kinds outputs
agree to the tolerance, not bit for bit; one plan kind run twice must repeat its bits."""
import numpy as np
import pytest

import synth_inputs as S
from tests import harness as Hn
from oracle import oracle as O

pytestmark = pytest.mark.gpu
TOL = 5e-3


def _say(*a):
    print(*a, flush=True)


def _prof(B):
    return B.make_profile(h2d_gbps=50.0, gemv_gbps=4000.0, cpu_gbps=200.0, cpu_gbps_busy=150.0, h2d_gbps_busy=45.0,
                          cpu_tokens_free=4.0, cpu_sync_us=0.5)


def _run(cfg, W, head, budget, kind, xs, rows=None, threads=None):
    import torch
    from paper_2604_26334_amd import binding as B
    M = xs[0].shape[0]
    plan = B.Plan(cfg, int(budget), M, profile=_prof(B), kind=kind)
    st = B.Stack(plan)
    if threads and plan.summary().cpu_bytes:
        st.set_cpu_threads(threads)
    for layer in range(cfg["n_layers"]):
        for k, e, N, K in S.matrix_shapes(cfg):
            st.load_matrix(layer, k, e, *W(layer, k, e))
    if head is not None:
        st.load_matrix(cfg["n_layers"], S.MAT_OUT, None, *head)
    outs = []
    for x in xs:
        xin = torch.from_numpy(np.ascontiguousarray(x)).to(st.device)
        xout = torch.empty_like(xin)
        lo = None
        if head is not None:
            lo = torch.zeros((rows if rows else 1, cfg["vocab"]), dtype=torch.float16, device=st.device)
            st.set_logits_out(lo, 0 if rows == M else M - 1, rows if rows else 1)
        torch.cuda.synchronize()
        st.forward(xin, xout)
        st.synchronize()
        outs.append((xout.cpu().numpy(), None if lo is None else lo.cpu().numpy()))
    s, stats = plan.summary(), st.stats()
    st.close()
    plan.close()
    return outs, s, stats


@pytest.mark.parametrize("M", [1, 3, 16])
def test_static_and_dynamic_plans_match_the_oracle(M):
    from paper_2604_26334_amd import binding as B
    cfg = dict(Hn.small_dense_cfg(3), vocab=1040)
    seed = 60 + M
    W = Hn.WeightCache(cfg, seed)
    head = S.head_matrix(seed, cfg)
    xs = [S.activations(seed, t, M, cfg["hidden"]) for t in range(2)]
    refs = []
    for x in xs:
        rx = O.stack_forward(x, cfg, W, mirror=True)
        refs.append((rx, O.output_head(rx, cfg, head, mirror=True)))
    full = B.Plan(cfg, 1 << 40, M).summary()
    for frac in (0.6, 0.25):
        budget = full.workspace_bytes + int(full.weight_bytes * frac)
        for kind in (B.PS_PLAN_GPU_ONLY, B.PS_PLAN_STATIC, B.PS_PLAN_DYNAMIC, B.PS_PLAN_AUTO):
            outs, s, stats = _run(cfg, W, head, budget, kind, xs, rows=M)
            _say("  M %d frac %.2f kind %d -> plan %d: pinned %d streamed %d cpu %d (share %.2f), step: %d B on the CPU in %.2f ms, waited %.2f ms" % (
                M, frac, kind, s.plan_kind, s.resident_bytes, s.streamed_bytes, s.cpu_bytes, s.cpu_fraction,
                stats.cpu_bytes_step, stats.cpu_ms, stats.cpu_wait_ms))
            if kind in (B.PS_PLAN_STATIC, B.PS_PLAN_DYNAMIC):
                assert s.cpu_bytes > 0 and stats.cpu_bytes_step == s.cpu_bytes
            for (xo, lo), (rx, rl) in zip(outs, refs):
                e_x, e_l = Hn.rel_err(xo, rx), Hn.rel_err(lo, rl)
                _say("      err x %.3e logits %.3e" % (e_x, e_l))
                assert np.isfinite(xo.astype(np.float64)).all() and e_x <= TOL and e_l <= TOL
            if kind == B.PS_PLAN_STATIC:   # same plan, other thread counts: same bits
                again, _, _ = _run(cfg, W, head, budget, kind, xs, rows=M, threads=3)
                for (xo, lo), (xo2, lo2) in zip(outs, again):
                    np.testing.assert_array_equal(xo.view(np.uint16), xo2.view(np.uint16))
                    np.testing.assert_array_equal(lo.view(np.uint16), lo2.view(np.uint16))


def test_cpu_plans_on_the_ffn_block_and_last_token_logits():
    """No attention, no residual (the FFN input is the caller's tensor); and a head that serves one
    token of a 16-token plan from the CPU."""
    from paper_2604_26334_amd import binding as B
    cfg = S.cfg_ffn_block()
    W = Hn.WeightCache(cfg, 7)
    x = S.activations(7, 0, 1, cfg["hidden"])
    ref = O.stack_forward(x, cfg, W, mirror=True)
    full = B.Plan(cfg, 1 << 40, 1).summary()
    for kind in (B.PS_PLAN_STATIC, B.PS_PLAN_DYNAMIC):
        outs, s, stats = _run(cfg, W, None, full.workspace_bytes + full.weight_bytes // 2, kind, [x])
        e = Hn.rel_err(outs[0][0], ref)
        _say("  ffn block kind %d: cpu %d B of %d, err %.3e" % (kind, s.cpu_bytes, s.weight_bytes, e))
        assert s.cpu_bytes > 0 and e <= TOL
    cfg = dict(Hn.small_dense_cfg(2), vocab=2064)
    W = Hn.WeightCache(cfg, 8)
    head = S.head_matrix(8, cfg)
    x = S.activations(8, 0, 16, cfg["hidden"])
    rx = O.stack_forward(x, cfg, W, mirror=True)
    rl = O.output_head(rx[15:], cfg, head, mirror=True)
    full = B.Plan(cfg, 1 << 40, 16).summary()
    outs, s, stats = _run(cfg, W, head, full.workspace_bytes + full.weight_bytes // 3, B.PS_PLAN_STATIC, [x], rows=None)
    e_x, e_l = Hn.rel_err(outs[0][0], rx), Hn.rel_err(outs[0][1], rl)
    _say("  last token of 16 from a CPU head: err x %.3e logits %.3e" % (e_x, e_l))
    assert e_x <= TOL and e_l <= TOL


@pytest.mark.parametrize("M", [1, 4, 16])
def test_moe_experts_on_the_cpu_match_the_oracle(M):
    """Unpinned experts run by the CPU back-end (static), or split between PCIe and the CPU (dynamic)."""
    import torch
    from paper_2604_26334_amd import binding as B
    cfg = Hn.small_moe_cfg(3)
    seed = 80 + M
    W = Hn.WeightCache(cfg, seed)
    steps = 3
    xs = [S.activations(seed, t, M, cfg["hidden"]) for t in range(steps)]
    lgs = [S.router_logits(seed, t, cfg["n_layers"], M, cfg["n_experts"]) for t in range(steps)]
    refs = [O.stack_forward(x, cfg, W, logits=lg, mirror=True) for x, lg in zip(xs, lgs)]
    full = B.Plan(cfg, 1 << 40, M).summary()
    for frac in (0.6, 0.2):
        budget = full.workspace_bytes + int(full.weight_bytes * frac) + 65536
        for kind in (B.PS_PLAN_STATIC, B.PS_PLAN_DYNAMIC, B.PS_PLAN_AUTO):
            plan = B.Plan(cfg, budget, M, profile=_prof(B), kind=kind)
            st = B.Stack(plan)
            for layer in range(cfg["n_layers"]):
                for k, e, N, K in S.matrix_shapes(cfg):
                    st.load_matrix(layer, k, e, *W(layer, k, e))
            s = plan.summary()
            cpu_seen = 0
            for x, lg, ref in zip(xs, lgs, refs):
                xin = torch.from_numpy(x).to(st.device)
                xout = torch.empty_like(xin)
                torch.cuda.synchronize()
                st.forward(xin, xout, lg)
                st.synchronize()
                e = Hn.rel_err(xout.cpu().numpy(), ref)
                cpu_seen += st.stats().cpu_bytes_step
                assert e <= TOL, (M, frac, kind, e)
            _say("  MoE M %d frac %.1f kind %d -> plan %d: pinned %d streamed %d cpu %d; %d B went through the CPU in %d steps, last err %.3e" % (
                M, frac, kind, s.plan_kind, s.resident_bytes, s.streamed_bytes, s.cpu_bytes, cpu_seen, steps, e))
            if kind == B.PS_PLAN_STATIC:
                assert s.cpu_bytes > 0 and cpu_seen > 0
            st.close()
            plan.close()


def test_cpu_plans_beside_a_streamed_kv_cache():
    """Decode attention over a KV cache whose shards are partly streamed, with the FFN on the CPU:
    the cache and the attention matrices never leave the GPU side of the plan, the static plan keeps
    its two slots for the cache shards that do not fit."""
    import torch
    from paper_2604_26334_amd import binding as B
    ctx0, steps = 300, 2
    cfg = dict(Hn.small_dense_cfg(3), kv_context=ctx0 + steps + 3)
    W = Hn.WeightCache(cfg, 31)
    n_kv, hd, L = cfg["n_kv_heads"], cfg["head_dim"], cfg["n_layers"]
    caches = [S.kv_cache(31, l, n_kv, ctx0, hd) for l in range(L)]
    xs = [S.activations(31, t, 1, cfg["hidden"]) for t in range(steps)]
    oK = [np.zeros((n_kv, cfg["kv_context"], hd), np.float16) for _ in range(L)]
    oV = [np.zeros((n_kv, cfg["kv_context"], hd), np.float16) for _ in range(L)]
    for l in range(L):
        oK[l][:, :ctx0], oV[l][:, :ctx0] = caches[l]
    refs = []
    for t in range(steps):
        rows = []
        refs.append(O.stack_forward(xs[t], cfg, W, mirror=True, kv=lambda l: (oK[l], oV[l]), ctx=ctx0 + t, new_rows=rows))
        for l, (kn, vn) in enumerate(rows):
            oK[l][:, ctx0 + t], oV[l][:, ctx0 + t] = kn.astype(np.float16), vn.astype(np.float16)
    full = B.Plan(cfg, 1 << 40, 1)
    sh = full.shards()
    attn_b = sum(s.bytes for s in sh if s.kind in (B.PS_SHARD_QKV, B.PS_SHARD_O))
    kv_b = sum(s.bytes for s in sh if s.kind == B.PS_SHARD_KV)
    ws = full.summary().workspace_bytes
    # budgets: attention + the whole cache pinned (FFN elsewhere); attention + about half the cache
    for budget in (ws + attn_b + kv_b + (1 << 18), ws + attn_b + kv_b // 2 + (1 << 20)):
        for kind in (B.PS_PLAN_STATIC, B.PS_PLAN_DYNAMIC):
            plan = B.Plan(cfg, budget, 1, profile=_prof(B), kind=kind)
            s = plan.summary()
            shards = plan.shards()
            assert all(x.resident != 2 for x in shards if x.kind in (B.PS_SHARD_QKV, B.PS_SHARD_O, B.PS_SHARD_KV))
            kv_streamed = sum(1 for x in shards if x.kind == B.PS_SHARD_KV and x.resident == 0)
            st = B.Stack(plan)
            for layer in range(L):
                for k, e, N, K in S.matrix_shapes(cfg):
                    st.load_matrix(layer, k, e, *W(layer, k, e))
                for g in range(n_kv):
                    st.load_kv(layer, g, caches[layer][0][g], caches[layer][1][g])
            for t in range(steps):
                st.set_context(ctx0 + t)
                xin = torch.from_numpy(xs[t]).to(st.device)
                xout = torch.empty_like(xin)
                st.forward(xin, xout)
                st.synchronize()
                e = Hn.rel_err(xout.cpu().numpy(), refs[t])
                assert e <= TOL, (budget, kind, t, e)
            _say("  budget %d kind %d: slots %d, cache shards streamed %d, cpu %d B, streamed %d B, last err %.3e" % (
                budget, kind, s.n_slots, kv_streamed, s.cpu_bytes, s.streamed_bytes, e))
            assert s.cpu_bytes > 0
            st.close()
            plan.close()


@pytest.mark.parametrize("kind_name", ["static", "dynamic", "auto"])
def test_one_stack_prefills_on_the_gpu_and_decodes_with_a_cpu_plan(kind_name):
    """The paper's phase-adaptive use of one budget (Algorithm 1: SetupForSched after PickTier; Section 3,
    the three plans per tier): a tier table whose low tiers are planned with CPU shares and whose many-token
    tiers stream everything through the GPU, served by ONE stack.  Prefill runs in a chunk tier (Plan One),
    the stack switches to the one-token tier (static / dynamic / HeuristicSplit's pick) and decodes; then a
    second prompt piece goes back through the chunk tier.  Every output against the oracle; the decode steps
    bit-identical to a stack built for the one-token plan alone."""
    import torch
    from paper_2604_26334_amd import binding as B
    kind = {"static": B.PS_PLAN_STATIC, "dynamic": B.PS_PLAN_DYNAMIC, "auto": B.PS_PLAN_AUTO}[kind_name]
    cfg = Hn.small_dense_cfg(3)
    W = Hn.WeightCache(cfg, 23)
    wb, _ = Hn.total_weight_bytes(cfg)
    full = B.Plan(cfg, 1 << 40, 512).summary()
    budget = full.workspace_bytes + int(wb * 0.25)     # the 512-token tier streams every matrix; the one-token tier pins most
    table = B.TierTable(cfg, budget, profile=_prof(B), kind=kind)
    ents = table.entries()
    t_dec, t_pre = 0, [e.tier for e in ents if e.feasible and e.tier_tokens == 512][0]
    assert ents[t_pre].summary.cpu_bytes == 0 and ents[t_pre].summary.streamed_bytes > 0
    assert ents[t_dec].summary.cpu_bytes > 0 and ents[t_dec].summary.plan_kind == (B.PS_PLAN_STATIC if kind == B.PS_PLAN_AUTO else kind)
    _say("one-token tier: plan kind %d, %d B on the CPU, %d B streamed; 512-token tier: %d B streamed" % (
        ents[t_dec].summary.plan_kind, ents[t_dec].summary.cpu_bytes, ents[t_dec].summary.streamed_bytes, ents[t_pre].summary.streamed_bytes))
    st = B.Stack(table)
    alone = B.Stack(table.plan(t_dec))
    for s_ in (st, alone):
        for layer in range(cfg["n_layers"]):
            for k, e, N, K in S.matrix_shapes(cfg):
                s_.load_matrix(layer, k, e, *W(layer, k, e))

    def run(stack, xnp, chunked):
        xin = torch.from_numpy(np.ascontiguousarray(xnp)).to(stack.device)
        xout = torch.zeros_like(xin)
        if chunked:
            B.chunked_forward(stack, xin, xout)
        else:
            stack.forward(xin, xout)
        stack.synchronize()
        return xout.cpu().numpy()

    x = S.activations(23, 0, 700, cfg["hidden"])          # two trips, the second ragged
    st.set_tier(t_pre)
    e = Hn.rel_err(run(st, x, True), O.stack_forward(x, cfg, W, mirror=True))
    _say("prefill of 700 tokens in the 512-token tier: err %.2e" % e)
    assert e <= TOL
    st.set_tier(t_dec)
    for t in range(3):
        xt = S.activations(23, 1 + t, 1, cfg["hidden"])
        got = run(st, xt, False)
        e = Hn.rel_err(got, O.stack_forward(xt, cfg, W, mirror=True))
        _say("  decode step %d in the one-token tier: err %.2e, CPU bytes %d" % (t, e, st.stats().cpu_bytes_step))
        assert e <= TOL
        if ents[t_dec].summary.cpu_bytes:
            assert st.stats().cpu_bytes_step == ents[t_dec].summary.cpu_bytes
        np.testing.assert_array_equal(got.view(np.uint16), run(alone, xt, False).view(np.uint16))
    st.set_tier(t_pre)
    x2 = S.activations(23, 9, 300, cfg["hidden"])
    e = Hn.rel_err(run(st, x2, True), O.stack_forward(x2, cfg, W, mirror=True))
    _say("second prompt piece of 300 tokens: err %.2e" % e)
    assert e <= TOL
    st.close()
    alone.close()


@pytest.mark.parametrize("kind_name", ["static", "dynamic"])
def test_one_moe_stack_switches_between_tiers_with_cpu_experts(kind_name):
    """An MoE stack of several tiers whose plans leave experts to the CPU (Plan Two / Plan Three in every tier of
    up to 64 tokens, each with its own pinned set): a 100-token prompt in the 64-token tier (two trips), decode in
    the one-token tier, the 16-token tier after that; each against the oracle, decode bit-identical to a stack
    built for the one-token plan alone."""
    import torch
    from paper_2604_26334_amd import binding as B
    kind = {"static": B.PS_PLAN_STATIC, "dynamic": B.PS_PLAN_DYNAMIC}[kind_name]
    cfg = Hn.small_moe_cfg(3)
    L, E = cfg["n_layers"], cfg["n_experts"]
    W = Hn.WeightCache(cfg, 31)
    wb, _ = Hn.total_weight_bytes(cfg)
    budget = B.Plan(cfg, 1 << 40, 64).summary().workspace_bytes + int(wb * 0.3)
    table = B.TierTable(cfg, budget, profile=_prof(B), kind=kind)
    ents = {e.tier_tokens: e for e in table.entries() if e.feasible}
    assert all(ents[t].summary.cpu_bytes > 0 and ents[t].summary.plan_kind == kind for t in (1, 16, 64))
    assert ents[1].summary.resident_bytes > ents[64].summary.resident_bytes
    st = B.Stack(table)
    alone = B.Stack(table.plan(ents[1].tier))
    for s_ in (st, alone):
        for layer in range(L):
            for k, e, N, K in S.matrix_shapes(cfg):
                s_.load_matrix(layer, k, e, *W(layer, k, e))

    def run(stack, xnp, lg, chunked):
        xin = torch.from_numpy(np.ascontiguousarray(xnp)).to(stack.device)
        xout = torch.zeros_like(xin)
        if chunked:
            B.chunked_forward(stack, xin, xout, router_logits=lg)
        else:
            stack.forward(xin, xout, lg)
        stack.synchronize()
        return xout.cpu().numpy()

    x, lg = S.activations(31, 0, 100, cfg["hidden"]), S.router_logits(31, 0, L, 100, E)
    st.set_tier(ents[64].tier)
    e = Hn.rel_err(run(st, x, lg, True), O.stack_forward(x, cfg, W, logits=lg, mirror=True))
    _say("prompt of 100 tokens in the 64-token tier (%d B of experts on the CPU): err %.2e" % (ents[64].summary.cpu_bytes, e))
    assert e <= TOL
    st.set_tier(ents[1].tier)
    for t in range(3):
        xt, lt = S.activations(31, 1 + t, 1, cfg["hidden"]), S.router_logits(31, 1 + t, L, 1, E)
        got = run(st, xt, lt, False)
        e = Hn.rel_err(got, O.stack_forward(xt, cfg, W, logits=lt, mirror=True))
        _say("  decode step %d in the one-token tier: err %.2e, CPU bytes %d" % (t, e, st.stats().cpu_bytes_step))
        assert e <= TOL
        np.testing.assert_array_equal(got.view(np.uint16), run(alone, xt, lt, False).view(np.uint16))
    st.set_tier(ents[16].tier)
    x2, l2 = S.activations(31, 9, 16, cfg["hidden"]), S.router_logits(31, 9, L, 16, E)
    e = Hn.rel_err(run(st, x2, l2, False), O.stack_forward(x2, cfg, W, logits=l2, mirror=True))
    _say("16 tokens in the 16-token tier: err %.2e" % e)
    assert e <= TOL
    st.close()
    alone.close()
