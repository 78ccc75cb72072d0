"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element, on the
same seeded inputs, plus bit-exact invariance of the output to shard placement.

Tolerance (fp16 activations, fp32 accumulation): max|err| / max|ref| <= 5e-3, asserted against BOTH
forms of the oracle on these few-layer stacks: the pure fp64 definition (no rounding anywhere) and the
one that rounds to fp16 where the GPU stores fp16."""
import numpy as np
import pytest

import synth_inputs as S
from tests import harness as Hn
from oracle import oracle as O

pytestmark = pytest.mark.gpu
TOL = 5e-3


def _say(*a):
    print(*a, flush=True)


def test_mfma_operand_layout_probe():
    import ctypes as C
    import torch
    from paper_2604_26334_amd import binding as B
    out = torch.zeros(64 * 4, dtype=torch.float32, device="cuda:0")
    for pi, pk, pj in [(0, 0, 0), (5, 13, 9), (15, 31, 15), (7, 8, 2), (12, 23, 0), (3, 16, 14)]:
        out.zero_()
        torch.cuda.synchronize()
        rc = B.lib().ps_mfma_probe(pi, pk, pj, out.data_ptr(), None)
        assert rc == 0
        torch.cuda.synchronize()
        c = out.cpu().numpy().reshape(64, 4)
        nz = np.argwhere(c != 0)
        _say("probe", (pi, pk, pj), "->", nz.tolist())
        assert nz.tolist() == [[pj + 16 * (pi // 4), pi % 4]]
        assert c[pj + 16 * (pi // 4), pi % 4] == 1.0


def test_lds_transpose_read_lane_layout():
    """The LDS transpose read the chunk-attention kernels build their V operand with: within each group of 16
    lanes, lane L names 4 consecutive 16-bit numbers and lane m receives number m % 4 of lanes m / 4 + 4 e,
    e = 0 .. 3.  Checked with index numbers as data, for rows of the staged-V pitch and for packed chunks."""
    import torch
    from paper_2604_26334_amd import binding as B
    for pitch in (8, 288):                      # bytes between the rows the four lanes of a column name
        addr = np.zeros(64, dtype=np.uint32)
        for l in range(64):
            g, L = divmod(l, 16)
            addr[l] = (3 * g + L // 4) * pitch + (L % 4) * 8 if pitch > 8 else 8 * l    # (inside the 4 KB table)
        a = torch.from_numpy(addr.view(np.int32)).cuda()
        out = torch.zeros(256, dtype=torch.int16, device="cuda")
        assert B.lib().ps_lds_tr_probe(a.data_ptr(), out.data_ptr(), None) == 0
        torch.cuda.synchronize()
        got = out.cpu().numpy().view(np.uint16).reshape(64, 4)
        want = np.zeros((64, 4), dtype=np.uint16)
        for l in range(64):
            g, m = divmod(l, 16)
            for e in range(4):
                src = 16 * g + 4 * e + m // 4               # the lane whose 8 bytes hold the number
                want[l, e] = addr[src] // 2 + m % 4
        np.testing.assert_array_equal(got, want)


def _check(cfg, seed, M, budgets, logits=None, tol=TOL):
    W = Hn.WeightCache(cfg, seed)
    x = S.activations(seed, 0, M, cfg["hidden"])
    ref_m = O.stack_forward(x, cfg, W, logits=logits, mirror=True)
    ref_p = O.stack_forward(x, cfg, W, logits=logits, mirror=False)
    outs = []
    for b in budgets:
        _say("  budget", b, "M", M)
        y, info = Hn.run_gpu(cfg, W, b, x, logits=logits)
        e_m, e_p = Hn.rel_err(y, ref_m), Hn.rel_err(y, ref_p)
        _say("    resident %d streamed %d copies %d kernels %d  err(mirror) %.3e err(pure) %.3e" % (
            info["resident"], info["streamed"], info["stats"].n_copies, info["stats"].n_kernels, e_m, e_p))
        assert np.isfinite(y.astype(np.float64)).all()
        assert e_m <= tol, (b, e_m)
        assert e_p <= tol, (b, e_p)        # the plain fp64 definition, no rounding anywhere
        outs.append(y)
        if M == 1 and info["streamed"] == 0 and not cfg["n_experts"]:
            # the HIP-graph replay of the same launch sequence must agree bit for bit
            y2, info2 = Hn.run_gpu(cfg, W, b, x, logits=logits, mode=1)
            outs.append(y2)
    for y in outs[1:]:
        np.testing.assert_array_equal(y.view(np.uint16), outs[0].view(np.uint16))
    return outs[0]


def _budgets(cfg, M, fracs):
    wb, _ = Hn.total_weight_bytes(cfg)
    from paper_2604_26334_amd import binding as B
    ws = B.Plan(cfg, 1 << 62, M).summary().workspace_bytes
    return [int(wb * f) + ws + 4096 for f in fracs]


def test_ffn_block_decode_half_budget():
    """Config 1: RMSNorm -> gate/up -> SwiGLU -> down, one token, budget = 50% of the weight bytes."""
    cfg = S.cfg_ffn_block()
    wb, _ = Hn.total_weight_bytes(cfg)
    _check(cfg, 0, 1, [wb // 2, 1 << 30, wb // 3, int(wb * 0.8)])


def test_small_dense_decode_placements():
    cfg = Hn.small_dense_cfg(3)
    _check(cfg, 1, 1, _budgets(cfg, 1, [1.0, 0.7, 0.45, 0.3]))


@pytest.mark.parametrize("M", [2, 16, 37, 64, 150])
def test_small_dense_batched_and_prefill(M):
    cfg = Hn.small_dense_cfg(2)
    _check(cfg, 2, M, _budgets(cfg, M, [1.0, 0.5]))


@pytest.mark.parametrize("M", [2, 3, 4])
@pytest.mark.parametrize("ffn", [2048, 1408])
def test_few_token_decode_kernel(M, ffn):
    """Two to four tokens through matrices whose K is a multiple of 1024 take the few-token form of the decode
    kernel (MFMA dot products in the one-token kernel's launch shape, RMS factors computed in the kernel);
    with ffn 1408 the down projection (K = 1408) stays on the GEMM path and the two forms alternate inside a layer.
    Against the oracle, and bit-identical across placements."""
    cfg = dict(Hn.small_dense_cfg(2), hidden=1024, n_q_heads=8, n_kv_heads=2, ffn_inter=ffn)
    _check(cfg, 11, M, _budgets(cfg, M, [1.0, 0.6, 0.35]))


def test_few_token_kernel_in_chunked_trips():
    """Seven tokens through a four-token plan: a full trip and a short last one (three valid rows of four) in the
    few-token kernel, eager and replayed from a graph; every row against the oracle, and a row's bits do not
    depend on the trip it rode in (chunks are independent: attention is the identity on V)."""
    import torch
    from paper_2604_26334_amd import binding as B
    cfg = dict(Hn.small_dense_cfg(2), hidden=1024, n_q_heads=8, n_kv_heads=2, ffn_inter=2048)
    W = Hn.WeightCache(cfg, 13)
    x = S.activations(13, 0, 7, cfg["hidden"])
    ref = O.stack_forward(x, cfg, W, mirror=True)
    wb, _ = Hn.total_weight_bytes(cfg)
    outs = []
    for frac, mode in ((1.0, 0), (1.0, 1), (0.5, 0)):
        plan = B.Plan(cfg, _budgets(cfg, 4, [frac])[0], 4)
        st = B.Stack(plan)
        st.set_decode_mode(mode)
        for layer in range(cfg["n_layers"]):
            for kind, expert, N, K in S.matrix_shapes(cfg):
                st.load_matrix(layer, kind, expert, *W(layer, kind, expert))
        xin = torch.from_numpy(x).to(st.device)
        y = torch.zeros_like(xin)
        assert B.chunked_forward(st, xin, y) == 2
        st.synchronize()
        outs.append(y.cpu().numpy())
        # the last three rows alone, as a trip of their own
        y3 = torch.zeros_like(xin[4:])
        B.chunked_forward(st, xin[4:].contiguous(), y3)
        st.synchronize()
        np.testing.assert_array_equal(y3.cpu().numpy().view(np.uint16), outs[-1][4:].view(np.uint16))
        st.close()
        plan.close()
    assert Hn.rel_err(outs[0], ref) <= TOL
    for y in outs[1:]:
        np.testing.assert_array_equal(y.view(np.uint16), outs[0].view(np.uint16))


def test_few_token_decode_kernel_under_moe_layers():
    """The attention matrices of an MoE stack take the few-token kernel too; the experts' grouped GEMM still gets
    its RMS factors from their own launch."""
    cfg = dict(Hn.small_moe_cfg(2), hidden=1024, n_q_heads=8, n_kv_heads=2)
    M = 3
    lg = S.router_logits(5, 0, cfg["n_layers"], M, cfg["n_experts"])
    _check(cfg, 5, M, _budgets(cfg, M, [1.0, 0.5]), logits=lg)


@pytest.mark.parametrize("M", [1, 5, 16])
def test_small_moe(M):
    cfg = Hn.small_moe_cfg(2)
    lg = S.router_logits(3, 0, cfg["n_layers"], M, cfg["n_experts"])
    _check(cfg, 3, M, _budgets(cfg, M, [1.0, 0.6, 0.35]), logits=lg)


@pytest.mark.parametrize("kind,M", [("dense", 1), ("dense", 4), ("dense", 37), ("moe", 1), ("moe", 5)])
def test_copy_modes_move_the_same_bytes(kind, M):
    """Streamed shards cross PCIe by hipMemcpyAsync (mode 0), by the gather kernel where the library's rule
    picks it (mode 1, the default) or by the gather kernel throughout (mode 2): the outputs are bit-identical,
    match the oracle, and the same number of bytes is streamed.  Three forwards in a row, so slots are reused
    and the gather's descriptors are written again."""
    if kind == "dense":
        cfg, lgs = Hn.small_dense_cfg(3), None
    else:
        cfg = Hn.small_moe_cfg(2)
        lgs = [S.router_logits(17, t, cfg["n_layers"], M, cfg["n_experts"]) for t in range(3)]
    W = Hn.WeightCache(cfg, 17)
    xs = [S.activations(17, t, M, cfg["hidden"]) for t in range(3)]
    budget = _budgets(cfg, M, [0.4])[0]
    res = {m: Hn.run_gpu(cfg, W, budget, xs, logits=lgs, copy_mode=m) for m in (0, 1, 2)}
    assert res[0][1]["streamed"] > 0
    for t in range(3):
        ref = O.stack_forward(xs[t], cfg, W, logits=None if lgs is None else lgs[t], mirror=True)
        assert Hn.rel_err(res[0][0][t], ref) <= TOL
        for m in (1, 2):
            np.testing.assert_array_equal(res[0][0][t].view(np.uint16), res[m][0][t].view(np.uint16))
    for m in (1, 2):
        assert res[m][1]["stats"].streamed_bytes_step == res[0][1]["stats"].streamed_bytes_step


@pytest.mark.parametrize("M", [1, 5])
def test_small_moe_hot_experts_ranked_by_frequency(M):
    """Planner's expert ranking on the device: biased router logits make some experts hot; with the
    selection frequencies of a host warm-up the hot ones are pinned first.  Outputs are bit-identical
    with and without the ranking and match the oracle; no more bytes cross PCIe with it."""
    from paper_2604_26334_amd import binding as B
    cfg = Hn.small_moe_cfg(3)
    L, E, k = cfg["n_layers"], cfg["n_experts"], cfg["top_k"]
    W = Hn.WeightCache(cfg, 13)
    warm = S.router_logits(13, 999, L, 512, E, bias_seed=5)
    freq = np.stack([np.bincount(B.route_host(warm[l], k).reshape(-1), minlength=E) / 512.0 for l in range(L)]).astype(np.float32)
    xs = [S.activations(13, t, M, cfg["hidden"]) for t in range(3)]
    lgs = [S.router_logits(13, t, L, M, E, bias_seed=5) for t in range(3)]
    budget = _budgets(cfg, M, [0.5])[0]
    res = {}
    for name, f in (("unranked", None), ("ranked", freq)):
        ys, info = Hn.run_gpu(cfg, W, budget, xs, logits=lgs, expert_freq=f)
        res[name] = (ys, info)
    for t in range(3):
        ref_m = O.stack_forward(xs[t], cfg, W, logits=lgs[t], mirror=True)
        ref_p = O.stack_forward(xs[t], cfg, W, logits=lgs[t], mirror=False)
        a, b = res["unranked"][0][t], res["ranked"][0][t]
        np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16))
        assert Hn.rel_err(b, ref_m) <= TOL and Hn.rel_err(b, ref_p) <= TOL
    # bytes the three steps would stream, from each plan's residency marks and the host routing rule
    def streamed(expert_freq):
        plan = B.Plan(cfg, budget, M, expert_freq=expert_freq)
        pinned = {(s.layer, s.expert) for s in plan.shards() if s.kind == B.PS_SHARD_EXPERT and s.resident == 1}
        eb = next(s.bytes for s in plan.shards() if s.kind == B.PS_SHARD_EXPERT)
        n = 0
        for lg in lgs:
            for l in range(L):
                n += sum(1 for e in np.unique(B.route_host(lg[l], k)) if (l, int(e)) not in pinned)
        return n * eb
    s0, s1 = streamed(None), streamed(freq)
    _say("M", M, "expert bytes streamed over three steps: unranked", s0, "ranked", s1,
         "last step measured:", res["unranked"][1]["stats"].streamed_bytes_step, res["ranked"][1]["stats"].streamed_bytes_step)
    assert s1 <= s0 and s1 < s0 + 1      # ranking by the measured frequencies never costs bytes on these draws
    assert res["ranked"][1]["stats"].streamed_bytes_step <= res["unranked"][1]["stats"].streamed_bytes_step


@pytest.mark.parametrize("M", [2, 16, 37, 64])
@pytest.mark.parametrize("moe", [False, True])
def test_rms_factor_left_by_the_residual_epilogue_matches_its_own_launch(M, moe):
    """2..64 tokens, every shard resident: the split-K epilogue of O and down leaves the RMS factor of
    the rows it stores (modes 0/1) instead of a launch of its own (mode 2).  Same bits, fewer launches,
    and the second forward in a row (a smaller activation scale) agrees as well."""
    import torch
    from paper_2604_26334_amd import binding as B
    cfg = Hn.small_moe_cfg(2) if moe else Hn.small_dense_cfg(2)
    W = Hn.WeightCache(cfg, 11)
    wb, _ = Hn.total_weight_bytes(cfg)
    plan = B.Plan(cfg, wb + B.Plan(cfg, 1 << 62, M).summary().workspace_bytes + (1 << 20), M)
    st = B.Stack(plan)
    for layer in range(cfg["n_layers"]):
        for kind, expert, N, K in S.matrix_shapes(cfg):
            st.load_matrix(layer, kind, expert, *W(layer, kind, expert))
    lg = S.router_logits(11, 0, cfg["n_layers"], M, cfg["n_experts"]) if moe else None
    xs = [torch.from_numpy(S.activations(11, 0, M, cfg["hidden"])).cuda()]
    xs.append((xs[0] * 0.25).contiguous())
    res, launches = {}, {}
    for mode in (2, 0):
        st.set_decode_mode(mode)
        outs = []
        for x in xs:
            y = torch.empty_like(x)
            st.forward(x, y, lg)
            st.synchronize()
            outs.append(y.cpu().numpy().view(np.uint16))
        res[mode], launches[mode] = outs, st.stats().n_kernels
    _say("M", M, "moe", moe, "kernel ops", launches)
    for a, b in zip(res[0], res[2]):
        np.testing.assert_array_equal(a, b)
    st.close()


@pytest.mark.parametrize("M,hidden", [(1, 512), (4, 1024), (16, 512)])
def test_graph_replay_matches_eager_on_every_replay(M, hidden):
    """HIP-graph decode mode (one token; batched-decode steps of a few tokens, in the few-token kernel and in
    the GEMM form): several replays, with eager work and synchronisation in between, each compared bit for
    bit with the eager launch-per-shard result."""
    import torch
    from paper_2604_26334_amd import binding as B
    cfg = dict(Hn.small_dense_cfg(3), hidden=hidden)
    W = Hn.WeightCache(cfg, 5)
    wb, _ = Hn.total_weight_bytes(cfg)
    plan = B.Plan(cfg, wb + (4 << 20), M)
    st = B.Stack(plan)
    for layer in range(cfg["n_layers"]):
        for kind, expert, N, K in S.matrix_shapes(cfg):
            st.load_matrix(layer, kind, expert, *W(layer, kind, expert))
    xs = [torch.from_numpy(S.activations(5, t, M, cfg["hidden"])).cuda() for t in range(3)]
    eager = []
    st.set_decode_mode(0)
    for x in xs:
        y = torch.empty_like(x)
        st.forward(x, y)
        st.synchronize()
        eager.append(y.cpu().numpy().view(np.uint16))
    st.set_decode_mode(1)
    y = torch.empty_like(xs[0])
    for rep in range(4):
        for x, ref in zip(xs, eager):
            y.zero_()                       # eager work between replays
            torch.cuda.synchronize()
            st.forward(x, y)
            st.synchronize()
            assert st.stats().graph_replay == 1    # the graph path, not a silent launch-per-shard run
            np.testing.assert_array_equal(y.cpu().numpy().view(np.uint16), ref)
        (torch.ones(1 << 20, device="cuda") * 2).sum().item()
    st.close()


@pytest.mark.parametrize("kind", ["dense", "moe"])
def test_chunked_prefill_through_the_tier_table(kind):
    """Tier table + PickTier + chunked prefill (Section 3, inference phase): a prompt of n tokens runs
    as ceil(n / T) trips through the schedule of the picked tier T (last trip zero-padded); every row
    against the oracle, for the picked tier and for two forced ones."""
    import torch
    from paper_2604_26334_amd import binding as B
    n = 150
    if kind == "dense":
        cfg, logits = Hn.small_dense_cfg(2), None
    else:
        cfg = Hn.small_moe_cfg(2)
        logits = S.router_logits(3, 0, cfg["n_layers"], n, cfg["n_experts"])
    W = Hn.WeightCache(cfg, 7)
    wb, _ = Hn.total_weight_bytes(cfg)
    ws64 = B.Plan(cfg, 1 << 62, 64).summary().workspace_bytes
    table = B.TierTable(cfg, int(wb * 0.6) + ws64)
    choice = table.pick(n)
    _say("picked tier", choice.tier_tokens, "x", choice.iterations, "est %.3f ms" % choice.est_total_ms)
    x = S.activations(7, 0, n, cfg["hidden"])
    ref = O.stack_forward(x, cfg, W, logits=logits, mirror=True)
    tiers = sorted({choice.tier, 2, 4})            # picked, 16 and 64 tokens per trip
    streamed = []
    for t in tiers:
        e = table.entry(t)
        assert e.feasible
        streamed.append(e.summary.streamed_bytes)
        st = B.Stack(table.plan(t))
        for layer in range(cfg["n_layers"]):
            for k, ex, N, K in S.matrix_shapes(cfg):
                st.load_matrix(layer, k, ex, *W(layer, k, ex))
        xin = torch.from_numpy(x).cuda()
        xout = torch.zeros_like(xin)
        torch.cuda.synchronize()
        trips = B.chunked_forward(st, xin, xout, logits)
        st.synchronize()
        assert trips == -(-n // e.tier_tokens)
        got = xout.cpu().numpy()
        err = Hn.rel_err(got, ref)
        _say("tier", e.tier_tokens, "trips", trips, "rel err %.2e" % err)
        assert np.isfinite(got).all() and err <= TOL
        # a last chunk shorter than the tier: the bits of the same rows in a zero-padded full trip
        T, H = e.tier_tokens, cfg["hidden"]
        r0 = (n // T) * T
        if r0 < n:
            xi = torch.zeros((T, H), dtype=torch.float16, device=st.device)
            xi[:n - r0] = xin[r0:]
            xo = torch.empty_like(xi)
            lp = None
            if logits is not None:
                lp = np.zeros((cfg["n_layers"], T, cfg["n_experts"]), np.float32)
                lp[:, :n - r0] = logits[:, r0:]
            st.forward(xi, xo, lp)
            st.synchronize()
            np.testing.assert_array_equal(xo[:n - r0].cpu().numpy().view(np.uint16), got[r0:].view(np.uint16))
        if logits is not None:   # routing kernel reading the caller's device copy of the logits: same bits
            ld = torch.from_numpy(np.ascontiguousarray(logits)).to(st.device)
            xo2 = torch.zeros_like(xin)
            torch.cuda.synchronize()
            B.chunked_forward(st, xin, xo2, logits, router_logits_dev=ld)
            st.synchronize()
            np.testing.assert_array_equal(xo2.cpu().numpy().view(np.uint16), got.view(np.uint16))
        st.close()
    # the larger tier's workspace displaces pinned shards, the smaller tier pins more (or all)
    assert streamed[-1] > 0 and streamed == sorted(streamed)


@pytest.mark.parametrize("kind", ["dense", "moe"])
def test_one_stack_serves_the_prefill_tier_and_the_decode_tier(kind):
    """Algorithm 1's inference phase on ONE stack and one arena: SetupForSched for the prefill tier,
    a chunked prefill, SetupForSched for the one-token tier (shards that the larger workspace had
    displaced are pinned again from the host images), decode steps, and back again.  Every result
    against the oracle and bit-identical to a stack built for that tier alone."""
    import torch
    from paper_2604_26334_amd import binding as B
    n, steps = 150, 4
    if kind == "dense":
        cfg = Hn.small_dense_cfg(3)
        lg_p, lg_d = None, [None] * steps
    else:
        cfg = Hn.small_moe_cfg(3)
        lg_p = S.router_logits(21, 0, cfg["n_layers"], n, cfg["n_experts"])
        lg_d = [S.router_logits(21, 1 + t, cfg["n_layers"], 1, cfg["n_experts"]) for t in range(steps)]
    W = Hn.WeightCache(cfg, 21)
    wb, _ = Hn.total_weight_bytes(cfg)
    ws64 = B.Plan(cfg, 1 << 62, 64).summary().workspace_bytes
    budget = int(wb * 0.7) + ws64
    table = B.TierTable(cfg, budget)
    t_pre, t_dec = 4, 0                                   # 64 tokens per trip; one token
    e_pre, e_dec = table.entry(t_pre), table.entry(t_dec)
    assert e_pre.feasible and e_dec.feasible and e_dec.summary.resident_bytes > e_pre.summary.resident_bytes
    x = S.activations(21, 0, n, cfg["hidden"])
    xd = [S.activations(21, 1 + t, 1, cfg["hidden"]) for t in range(steps)]
    ref_p = O.stack_forward(x, cfg, W, logits=lg_p, mirror=True)
    ref_d = [O.stack_forward(xd[t], cfg, W, logits=lg_d[t], mirror=True) for t in range(steps)]

    def load(st):
        for layer in range(cfg["n_layers"]):
            for k, ex, N, K in S.matrix_shapes(cfg):
                st.load_matrix(layer, k, ex, *W(layer, k, ex))

    def prefill(st):
        xin = torch.from_numpy(x).to(st.device)
        xout = torch.zeros_like(xin)
        torch.cuda.synchronize()
        B.chunked_forward(st, xin, xout, lg_p)
        st.synchronize()
        return xout.cpu().numpy()

    def decode(st):
        outs = []
        for t in range(steps):
            xin = torch.from_numpy(xd[t]).to(st.device)
            xout = torch.zeros_like(xin)
            st.forward(xin, xout, lg_d[t])
            st.synchronize()
            outs.append(xout.cpu().numpy())
        return outs

    alone = {}
    for t, run in ((t_pre, prefill), (t_dec, decode)):    # the per-tier stacks
        st = B.Stack(table.plan(t))
        load(st)
        alone[t] = run(st)
        st.close()
    st = B.Stack(table)
    load(st)
    assert st.tier() == (0, 1)                            # the lowest tier is installed first
    for rnd in range(2):
        up = st.set_tier(t_pre)
        assert st.tier() == (t_pre, 64)
        got = prefill(st)
        np.testing.assert_array_equal(got.view(np.uint16), alone[t_pre].view(np.uint16))
        assert Hn.rel_err(got, ref_p) <= TOL
        up = st.set_tier(t_dec)
        _say(kind, "round", rnd, "back to the one-token tier: %d B pinned again (tier pins %d B, prefill tier %d B)" % (
            up, e_dec.summary.resident_bytes, e_pre.summary.resident_bytes))
        assert 0 < up <= e_dec.summary.resident_bytes     # only what the prefill tier's workspace displaced
        for a, b, r in zip(decode(st), alone[t_dec], ref_d):
            np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16))
            assert Hn.rel_err(a, r) <= TOL
    with pytest.raises(B.PshardError):
        st.set_tier(10)                                   # 16384 tokens: no plan under this budget
    st.close()


def _kv_cfg(n_layers, cap):
    return dict(Hn.small_dense_cfg(n_layers), kv_context=cap)


@pytest.mark.parametrize("ctx0", [0, 1, 127, 128, 255, 700])
def test_decode_attention_over_kv_cache(ctx0):
    """KV cache as a shard class + real decode attention: three consecutive decode steps at context
    ctx0, ctx0 + 1, ctx0 + 2 (each step attends over the rows the earlier ones appended), every step
    against the oracle, bit-identical across cache placements (all pinned / some streamed / all
    streamed), appended rows checked through the next step's result."""
    import torch
    from paper_2604_26334_amd import binding as B
    steps = 3
    cfg = _kv_cfg(3, ctx0 + steps + 5)
    W = Hn.WeightCache(cfg, 9)
    n_kv, hd, L = cfg["n_kv_heads"], cfg["head_dim"], cfg["n_layers"]
    caches = [S.kv_cache(9, l, n_kv, ctx0, hd) for l in range(L)]
    xs = [S.activations(9, t, 1, cfg["hidden"]) for t in range(steps)]
    # oracle: its own copy of the caches, rows appended as stored (fp16)
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
    wsb, allb = full.summary().workspace_bytes, full.summary().weight_bytes
    slot = B.Plan(cfg, wsb + allb - 4096, 1).summary().slot_bytes
    budgets = [wsb + allb + 4096, wsb + 2 * slot + 4096]
    n_pinned = lambda b: sum(s.resident for s in B.Plan(cfg, b, 1).shards() if s.kind == B.PS_SHARD_KV)
    for k in range(1, 40):      # a budget in between that pins some of the cache shards but not all
        b = budgets[1] + (budgets[0] - budgets[1]) * k // 40
        if 0 < n_pinned(b) < L * n_kv:
            budgets.insert(1, b)
            break
    outs = []
    for b in budgets:
        plan = B.Plan(cfg, b, 1)
        kvs = [s for s in plan.shards() if s.kind == B.PS_SHARD_KV]
        _say("budget", b, "cache shards pinned", sum(s.resident for s in kvs), "of", len(kvs))
        st = B.Stack(plan)
        for layer in range(L):
            for k, ex, N, K in S.matrix_shapes(cfg):
                st.load_matrix(layer, k, ex, *W(layer, k, ex))
            for g in range(n_kv):
                st.load_kv(layer, g, caches[layer][0][g], caches[layer][1][g])
        got = []
        for t in range(steps):
            xin = torch.from_numpy(xs[t]).cuda()
            xout = torch.empty_like(xin)
            st.set_context(ctx0 + t)
            st.forward(xin, xout)
            st.synchronize()
            got.append(xout.cpu().numpy())
            err = Hn.rel_err(got[-1], refs[t])
            _say("  step", t, "ctx", ctx0 + t, "rel err %.2e" % err)
            assert np.isfinite(got[-1]).all() and err <= TOL
        outs.append(got)
        st.close()
    pinned = [sum(s.resident for s in B.Plan(cfg, b, 1).shards() if s.kind == B.PS_SHARD_KV) for b in budgets]
    assert pinned[0] == L * n_kv
    if ctx0 >= 255:     # caches big enough that the budgets are three different placements
        assert len(budgets) == 3 and pinned[-1] == 0 and 0 < pinned[1] < L * n_kv
    for got in outs[1:]:
        for a, b in zip(got, outs[0]):
            np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16))


@pytest.mark.parametrize("ctx0,M", [(0, 5), (3, 37), (300, 64), (250, 16), (10, 300), (0, 256), (300, 520)])
def test_chunk_of_new_tokens_attends_over_the_kv_cache(ctx0, M):
    """Chunked prefill over the cache: a forward of M new tokens at context ctx0 (causal attention inside
    the chunk, rows appended at ctx0 .. ctx0 + M - 1), then a one-token step at ctx0 + M that attends over
    what the chunk appended.
    Oracle parity is taken layer by layer, each layer fed the GPU's own output of the layer before (softmax
    over scores of this size is sharp: a rounding-sized difference in one layer's rows can move weight
    between positions in the next, so the end-to-end error of a deeper stack says little about a kernel);
    the two-layer stack must then give exactly the bits of that chain, on every cache placement."""
    import torch
    from paper_2604_26334_amd import binding as B
    L = 2
    cfg = _kv_cfg(L, ctx0 + M + 9)
    one = dict(cfg, n_layers=1)
    Wall = Hn.WeightCache(cfg, 29)
    n_kv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    caches = [S.kv_cache(29, l, n_kv, ctx0, hd) for l in range(L)]
    x = S.activations(29, 0, M, cfg["hidden"])
    xd = S.activations(29, 1, 1, cfg["hidden"])

    def load(st, layers, weights):
        for layer in layers:
            for k, ex, N, K in S.matrix_shapes(cfg):
                st.load_matrix(layer, k, ex, *weights(layer, k, ex))

    def run(st, kv_of_layer, n_layers, xin_np, xd_np):
        for layer in range(n_layers):
            for g in range(n_kv):
                st.load_kv(layer, g, kv_of_layer(layer)[0][g], kv_of_layer(layer)[1][g])
        xin = torch.from_numpy(xin_np).to(st.device)
        xout = torch.zeros_like(xin)
        st.set_context(ctx0)
        st.forward(xin, xout)
        st.synchronize()
        streamed = st.stats().streamed_bytes_step
        qkv = st.debug_buffer(0, np.float16, (M, (cfg["n_q_heads"] + 2 * n_kv) * hd)).copy()    # last layer's QKV rows
        xdi = torch.from_numpy(xd_np).to(st.device)
        xdo = torch.zeros_like(xdi)
        st.set_context(ctx0 + M)
        B.chunked_forward(st, xdi, xdo)          # one token through the chunk plan's schedule
        st.synchronize()
        qkv_d = st.debug_buffer(0, np.float16, (M, (cfg["n_q_heads"] + 2 * n_kv) * hd))[0].copy()   # the token's own QKV row
        return xout.cpu().numpy(), xdo.cpu().numpy(), streamed, (qkv, qkv_d)

    # layer by layer on one-layer stacks, against the oracle on the same inputs
    cur, cur_d = x, xd
    for l in range(L):
        Wl = lambda layer, k, e, l=l: Wall(l, k, e)
        oK = np.zeros((n_kv, cfg["kv_context"], hd), np.float16)
        oV = np.zeros_like(oK)
        oK[:, :ctx0], oV[:, :ctx0] = caches[l]
        rows = []
        ref = O.stack_forward(cur, one, Wl, mirror=True, kv=lambda _l: (oK, oV), ctx=ctx0, new_rows=rows)
        ref_pure = O.stack_forward(cur, one, Wl, mirror=False, kv=lambda _l: (oK, oV), ctx=ctx0)
        st = B.Stack(B.Plan(one, 1 << 30, M))
        load(st, [0], Wl)
        got, got_d, _, (qkv, qkv_d) = run(st, lambda _l: caches[l], 1, cur, cur_d)
        st.close()
        # the next token attends over the rows the GPU appended: the oracle gets exactly those rows (a
        # last-bit difference in a row can move softmax weight between positions; the chunk's rows
        # themselves are checked here and, through `ref`, by the chunk's own attention)
        nq = cfg["n_q_heads"]
        assert Hn.rel_err(qkv[:, nq * hd:], np.concatenate([rows[0][0].reshape(M, -1), rows[0][1].reshape(M, -1)], axis=1)) <= TOL
        oK[:, ctx0:ctx0 + M] = qkv[:, nq * hd:(nq + n_kv) * hd].reshape(M, n_kv, hd).transpose(1, 0, 2)
        oV[:, ctx0:ctx0 + M] = qkv[:, (nq + n_kv) * hd:].reshape(M, n_kv, hd).transpose(1, 0, 2)
        # ... and its own QKV row: the projection against the oracle's, the rest of the layer on the GPU's row
        y_d = O.linear(O.rmsnorm(cur_d, cfg["rms_eps"]), *Wl(0, S.MAT_QKV, None))
        assert Hn.rel_err(qkv_d[None, :], y_d) <= TOL
        ref_d = Hn.kv_token_reference_from_gpu_qkv(one, Wl, cur_d, qkv_d, oK, oV, ctx0 + M)
        e, ep, ed = Hn.rel_err(got, ref), Hn.rel_err(got, ref_pure), Hn.rel_err(got_d, ref_d)
        _say("ctx", ctx0, "M", M, "layer", l, "err %.2e (pure %.2e)  next token %.2e" % (e, ep, ed))
        assert np.isfinite(got).all() and e <= TOL and ep <= TOL and ed <= TOL
        cur, cur_d = got, got_d
    # the whole stack, three placements of the cache: the chain's bits
    full = B.Plan(cfg, 1 << 40, M).summary()
    slot = B.Plan(cfg, full.workspace_bytes + full.weight_bytes - 4096, M).summary().slot_bytes
    budgets = [full.workspace_bytes + full.weight_bytes + 4096,
               full.workspace_bytes + (full.weight_bytes + 2 * slot) // 2 + 4096,
               full.workspace_bytes + 2 * slot + 4096]
    for b in budgets:
        plan = B.Plan(cfg, b, M)
        kvs = [s for s in plan.shards() if s.kind == B.PS_SHARD_KV]
        st = B.Stack(plan)
        load(st, range(L), Wall)
        got, got_d, streamed, _ = run(st, lambda l: caches[l], L, x, xd)
        _say("  budget", b, "cache shards pinned", sum(s.resident for s in kvs), "of", len(kvs), "streamed %d B" % streamed)
        np.testing.assert_array_equal(got.view(np.uint16), cur.view(np.uint16))
        np.testing.assert_array_equal(got_d.view(np.uint16), cur_d.view(np.uint16))
        st.close()
        plan.close()


def test_chunked_prefill_fills_the_cache_it_then_decodes_over():
    """150 prompt tokens through a 64-token tier of a stack with a KV cache (three trips, each attending
    over the cache and the rows the earlier trips appended), then decode steps over the filled cache.
    Causal attention does not depend on how the prompt is chunked: the oracle takes it in one piece."""
    import torch
    from paper_2604_26334_amd import binding as B
    ctx0, n, steps = 40, 150, 3
    cfg = _kv_cfg(1, ctx0 + n + steps + 4)      # one layer: this is about chunking and the context, not depth
    W = Hn.WeightCache(cfg, 37)
    n_kv, hd, L = cfg["n_kv_heads"], cfg["head_dim"], cfg["n_layers"]
    caches = [S.kv_cache(37, l, n_kv, ctx0, hd) for l in range(L)]
    x = S.activations(37, 0, n, cfg["hidden"])
    xs = [S.activations(37, 1 + t, 1, cfg["hidden"]) for t in range(steps)]
    oK = [np.zeros((n_kv, cfg["kv_context"], hd), np.float16) for _ in range(L)]
    oV = [np.zeros((n_kv, cfg["kv_context"], hd), np.float16) for _ in range(L)]
    for l in range(L):
        oK[l][:, :ctx0], oV[l][:, :ctx0] = caches[l]
    rows = []
    ref = O.stack_forward(x, cfg, W, mirror=True, kv=lambda l: (oK[l], oV[l]), ctx=ctx0, new_rows=rows)
    for l, (kn, vn) in enumerate(rows):
        oK[l][:, ctx0:ctx0 + n] = kn.transpose(1, 0, 2).astype(np.float16)
        oV[l][:, ctx0:ctx0 + n] = vn.transpose(1, 0, 2).astype(np.float16)
    refs_d = []
    for t in range(steps):
        rows = []
        refs_d.append(O.stack_forward(xs[t], cfg, W, mirror=True, kv=lambda l: (oK[l], oV[l]), ctx=ctx0 + n + t, new_rows=rows))
        for l, (kn, vn) in enumerate(rows):
            oK[l][:, ctx0 + n + t], oV[l][:, ctx0 + n + t] = kn.astype(np.float16), vn.astype(np.float16)
    table = B.TierTable(cfg, 1 << 30)
    assert table.entry(4).feasible and table.entry(0).feasible
    st = B.Stack(table.plan(4))                   # the 64-token tier
    for layer in range(L):
        for k, ex, N, K in S.matrix_shapes(cfg):
            st.load_matrix(layer, k, ex, *W(layer, k, ex))
        for g in range(n_kv):
            st.load_kv(layer, g, caches[layer][0][g], caches[layer][1][g])
    xin = torch.from_numpy(x).to(st.device)
    xout = torch.zeros_like(xin)
    st.set_context(ctx0)
    assert B.chunked_forward(st, xin, xout) == 3
    st.synchronize()
    e = Hn.rel_err(xout.cpu().numpy(), ref)
    _say("chunked prefill over the cache: err %.2e" % e)
    assert e <= TOL
    for t in range(steps):                        # the context has advanced past the prompt by itself
        xi = torch.from_numpy(xs[t]).to(st.device)
        xo = torch.zeros_like(xi)
        B.chunked_forward(st, xi, xo)
        st.synchronize()
        ed = Hn.rel_err(xo.cpu().numpy(), refs_d[t])
        _say("  decode step", t, "err %.2e" % ed)
        assert ed <= TOL
    st.close()


def test_one_stack_prefills_into_the_cache_and_decodes_in_the_one_token_tier():
    """The whole inference phase with a KV cache on ONE stack: the 64-token tier is installed, the prompt
    is prefilled in chunks (its rows go into the cache, part of which this tier streams), the one-token
    tier is installed (cache shards it pins move into the arena with their rows) and decode steps attend
    over everything; then back to the chunk tier for more prompt tokens.  One layer at a time against the
    oracle would repeat the tests above: here a one-layer stack, end to end."""
    import torch
    from paper_2604_26334_amd import binding as B
    ctx0, n, steps, n2 = 40, 150, 3, 20
    cfg = _kv_cfg(1, ctx0 + n + steps + n2 + 4)
    W = Hn.WeightCache(cfg, 41)
    n_kv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    cache = S.kv_cache(41, 0, n_kv, ctx0, hd)
    oK = np.zeros((n_kv, cfg["kv_context"], hd), np.float16)
    oV = np.zeros_like(oK)
    oK[:, :ctx0], oV[:, :ctx0] = cache
    kvf = lambda _l: (oK, oV)

    def oracle(x, ctx):
        rows = []
        ref = O.stack_forward(x, cfg, W, mirror=True, kv=kvf, ctx=ctx, new_rows=rows)
        kn, vn = rows[0]
        if x.shape[0] == 1:
            oK[:, ctx], oV[:, ctx] = kn.astype(np.float16), vn.astype(np.float16)
        else:
            oK[:, ctx:ctx + x.shape[0]] = kn.transpose(1, 0, 2).astype(np.float16)
            oV[:, ctx:ctx + x.shape[0]] = vn.transpose(1, 0, 2).astype(np.float16)
        return ref

    x = S.activations(41, 0, n, cfg["hidden"])
    xs = [S.activations(41, 1 + t, 1, cfg["hidden"]) for t in range(steps)]
    x2 = S.activations(41, 9, n2, cfg["hidden"])
    full64 = B.Plan(cfg, 1 << 40, 64).summary()
    table = B.TierTable(cfg, full64.workspace_bytes + int(full64.weight_bytes * 0.7))
    pinned = {t: sum(s.resident for s in table.plan(t).shards() if s.kind == B.PS_SHARD_KV) for t in (0, 4)}
    _say("cache shards pinned: one-token tier %d, 64-token tier %d of %d" % (pinned[0], pinned[4], n_kv))
    assert pinned[0] == n_kv and pinned[4] < n_kv
    st = B.Stack(table)
    for k, ex, N, K in S.matrix_shapes(cfg):
        st.load_matrix(0, k, ex, *W(0, k, ex))
    for g in range(n_kv):
        st.load_kv(0, g, cache[0][g], cache[1][g])

    def gpu(xnp):
        xin = torch.from_numpy(xnp).to(st.device)
        xout = torch.zeros_like(xin)
        B.chunked_forward(st, xin, xout)
        st.synchronize()
        return xout.cpu().numpy()

    st.set_tier(4)
    st.set_context(ctx0)
    e = Hn.rel_err(gpu(x), oracle(x, ctx0))
    _say("prefill of %d tokens in the 64-token tier: err %.2e" % (n, e))
    assert e <= TOL
    up = st.set_tier(0)
    _say("switch to the one-token tier moved / pinned again %d B" % up)
    assert up > 0
    for t in range(steps):
        e = Hn.rel_err(gpu(xs[t]), oracle(xs[t], ctx0 + n + t))
        _say("  decode step %d: err %.2e" % (t, e))
        assert e <= TOL
    st.set_tier(4)                               # more prompt tokens: the cache moves back with its new rows
    e = Hn.rel_err(gpu(x2), oracle(x2, ctx0 + n + steps))
    _say("second prompt piece of %d tokens: err %.2e" % (n2, e))
    assert e <= TOL
    st.close()


def test_error_paths_return_codes_and_leave_the_stack_usable():
    """Misuse through the C ABI: every case returns an error code with a text, none faults, and the
    stack still computes the right result afterwards."""
    import ctypes as C
    import torch
    from paper_2604_26334_amd import binding as B
    cfg = Hn.small_dense_cfg(2)
    W = Hn.WeightCache(cfg, 4)
    wb, _ = Hn.total_weight_bytes(cfg)
    plan = B.Plan(cfg, wb + (1 << 20), 1)
    L = B.lib()
    arena = torch.empty(int(plan.summary().budget_bytes) // 2, dtype=torch.uint8, device="cuda")
    h = C.c_void_p()
    assert L.ps_stack_create(plan.h, arena.data_ptr(), arena.numel(), None, None, C.byref(h)) == B.PS_E_ARG   # arena < budget
    assert b"arena" in L.ps_last_error()
    assert L.ps_stack_create(plan.h, None, 0, None, None, C.byref(h)) == B.PS_E_ARG
    st = B.Stack(plan)
    x = torch.from_numpy(S.activations(4, 0, 1, cfg["hidden"])).cuda()
    y = torch.empty_like(x)
    with pytest.raises(B.PshardError) as e:            # forward before the weights are loaded
        st.forward(x, y)
    assert e.value.code == B.PS_E_STATE
    for layer in range(cfg["n_layers"]):
        for k, ex, N, K in S.matrix_shapes(cfg):
            st.load_matrix(layer, k, ex, *W(layer, k, ex))
    sc, cd = W(0, S.MAT_QKV, None)
    for bad in ((9, S.MAT_QKV), (0, 17)):               # layer / matrix kind out of range
        with pytest.raises(B.PshardError) as e:
            st.load_matrix(bad[0], bad[1], None, sc, cd)
        assert e.value.code == B.PS_E_ARG
    assert L.ps_stack_forward(st.h, x.data_ptr(), x.data_ptr(), None, None) == B.PS_E_ARG      # aliasing
    assert L.ps_stack_forward(st.h, None, y.data_ptr(), None, None) == B.PS_E_ARG
    with pytest.raises(B.PshardError) as e:            # no KV cache in this stack
        st.set_context(3)
    assert e.value.code == B.PS_E_STATE
    with pytest.raises(B.PshardError):
        st.load_kv(0, 0, np.zeros((4, 128), np.float16), np.zeros((4, 128), np.float16))
    with pytest.raises(B.PshardError):
        st.set_decode_mode(7)
    with pytest.raises(B.PshardError) as e:
        st.set_copy_mode(3)
    assert e.value.code == B.PS_E_ARG
    st.forward(x, y)
    st.synchronize()
    ref = O.stack_forward(S.activations(4, 0, 1, cfg["hidden"]), cfg, W, mirror=True)
    assert Hn.rel_err(y.cpu().numpy(), ref) <= TOL
    st.close()
    # KV stack: context must leave room for the new row; more positions than the cache holds are refused
    kcfg = dict(cfg, kv_context=16)
    kst = B.Stack(B.Plan(kcfg, 1 << 26, 1))
    with pytest.raises(B.PshardError) as e:
        kst.set_context(16)
    assert e.value.code == B.PS_E_ARG
    with pytest.raises(B.PshardError):
        kst.load_kv(0, 0, np.zeros((17, 128), np.float16), np.zeros((17, 128), np.float16))
    with pytest.raises(B.PshardError):
        kst.load_kv(0, 5, np.zeros((4, 128), np.float16), np.zeros((4, 128), np.float16))
    kst.close()


def test_kv_decode_graph_replay_matches_launch_per_shard():
    """Decode over a resident KV cache replayed from a HIP graph: the context length is read from device
    memory, so one captured graph serves every step; bits must equal the launch-per-shard mode at each
    of several consecutive steps, after a jump back to a shorter context, and at an empty cache."""
    import torch
    from paper_2604_26334_amd import binding as B
    ctx0, cap = 300, 700
    cfg = _kv_cfg(3, cap)
    W = Hn.WeightCache(cfg, 19)
    n_kv, hd, L = cfg["n_kv_heads"], cfg["head_dim"], cfg["n_layers"]
    caches = [S.kv_cache(19, l, n_kv, ctx0, hd) for l in range(L)]
    xs = [S.activations(19, t, 1, cfg["hidden"]) for t in range(8)]
    contexts = [ctx0, ctx0 + 1, ctx0 + 2, ctx0 + 3, 5, 6, 0, 1]      # rows appended by earlier steps are reused
    outs = {}
    for mode in (0, 1):
        plan = B.Plan(cfg, 1 << 30, 1)
        assert plan.summary().streamed_bytes == 0
        st = B.Stack(plan)
        st.set_decode_mode(mode)
        for layer in range(L):
            for k, e, N, K in S.matrix_shapes(cfg):
                st.load_matrix(layer, k, e, *W(layer, k, e))
            for g in range(n_kv):
                st.load_kv(layer, g, caches[layer][0][g], caches[layer][1][g])
        xin = [torch.from_numpy(x).to(st.device) for x in xs]
        xout = torch.empty_like(xin[0])
        res = []
        for t, c in enumerate(contexts):
            st.set_context(c)
            torch.cuda.synchronize()
            st.forward(xin[t % 2], xout)          # two input buffers: two captured graphs, each replayed
            st.synchronize()
            assert st.stats().graph_replay == mode    # mode 1 really is the graph path on this stack
            res.append(xout.cpu().numpy().copy())
        outs[mode] = res
        st.close()
        plan.close()
    for t, (a, b) in enumerate(zip(outs[0], outs[1])):
        assert np.isfinite(a.astype(np.float64)).all()
        np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16), err_msg="step %d" % t)


@pytest.mark.parametrize("n_experts,top_k", [(48, 6), (200, 8), (1024, 8)])
def test_routing_kernel_indices_and_weights_with_ties(n_experts, top_k):
    """The routing step on its own, read back from the workspace after a one-layer MoE forward: the
    top_k largest logits per token, ties to the lower expert index, listed in descending order,
    and the softmax over them.  Logits are drawn from a handful of values, so ties are everywhere;
    the three expert counts take the three register shapes of the kernel (up to 128, 256, 1024)."""
    import torch
    from paper_2604_26334_amd import binding as B
    M = 5
    cfg = dict(Hn.small_moe_cfg(1), hidden=128, n_q_heads=1, n_kv_heads=1, n_experts=n_experts, top_k=top_k, expert_inter=128)
    W = Hn.WeightCache(cfg, 23, keep=False)
    rng = np.random.default_rng(n_experts)
    lg = rng.integers(-3, 4, size=(1, M, n_experts)).astype(np.float32) * 0.5
    lg[0, 1, :] = 0.25                    # one token with every logit equal: experts 0 .. top_k-1
    lg[0, 2, -1] = 9.0                    # the largest in the last position
    wb, ws = Hn.total_weight_bytes(cfg)
    plan = B.Plan(cfg, wb + ws + (4 << 20), M)
    st = B.Stack(plan)
    for kind, expert, N, K in S.matrix_shapes(cfg):
        st.load_matrix(0, kind, expert, *W(0, kind, expert))
    x = torch.from_numpy(S.activations(23, 0, M, cfg["hidden"])).to(st.device)
    y = torch.empty_like(x)
    st.forward(x, y, lg)
    st.synchronize()
    idx = st.debug_buffer(3, np.int32, (M, top_k)).copy()
    w = st.debug_buffer(4, np.float32, (M, top_k)).copy()
    st.close()
    plan.close()
    ref_idx, ref_w = O.route_topk(lg[0], top_k)
    np.testing.assert_array_equal(idx, ref_idx)
    np.testing.assert_array_equal(idx[1], np.arange(top_k))
    assert idx[2, 0] == n_experts - 1
    np.testing.assert_allclose(w, ref_w, rtol=2e-6, atol=1e-7)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=1e-6)
