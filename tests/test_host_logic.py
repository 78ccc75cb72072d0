"""CPU tests of the host side of the library: C-ABI exports, the packer's layout, the planner
(priority order, budget, monotonicity, estimate -- paper Section 3, Algorithm 1 and the timing
estimate) and the schedule checker.  No GPU compute is called."""
import ctypes as C
import itertools
import os
import re

import numpy as np
import pytest

import synth_inputs as S
from paper_2604_26334_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)          # declarations only, not the comments about them
    declared = set(re.findall(r"\b(ps_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_struct_sizes_match_header_layout():
    assert C.sizeof(B.ps_model_desc) == 52
    assert C.sizeof(B.ps_profile) == 8 * (3 + B.PS_NTIERS + 5)
    assert C.sizeof(B.ps_shard_info) == 48
    assert C.sizeof(B.ps_op_info) == 48
    assert C.sizeof(B.ps_stats) == 96


def test_tiers_are_the_papers_set():
    # Section 3, inference phase: J = {1, 4, 16, 32, 64, 512, 1K, 2K, 4K, 8K, 16K}
    lines = open(os.path.join(ROOT, "tests", "golden", "token_tiers.txt")).read().splitlines()
    want = [int(x) for ln in lines if not ln.startswith("#") for x in ln.split()]
    got = [B.lib().ps_tier_tokens(t) for t in range(B.PS_NTIERS)]
    assert got == want
    assert B.lib().ps_tier_for_tokens(1) == 0 and B.lib().ps_tier_for_tokens(2) == 1
    assert B.lib().ps_tier_for_tokens(2048) == 7 and B.lib().ps_tier_for_tokens(65) == 5


# ------------------------------------------------------------------ packer

def _unpack(img, rows, K):
    """Decode the documented layout back to (scales, codes) with plain index arithmetic."""
    nsb, ngroups = K // 128, (K // 128 + 7) // 8
    tile_bytes = (nsb + ngroups) * 1024
    codes = np.zeros((rows, K), dtype=np.uint8)
    scales = np.zeros((rows, K // 32), dtype=np.uint16)
    for T in range(rows // 16):
        tile = img[T * tile_bytes:(T + 1) * tile_bytes]
        for g in range(ngroups):
            nsb_g = min(8, nsb - 8 * g)
            gb = tile[g * 9 * 1024:]
            for s in range(nsb_g):
                dw = gb[s * 1024:(s + 1) * 1024].view(np.uint32).reshape(64, 4)
                for lane in range(64):
                    i, c = lane & 15, lane >> 4
                    b = 4 * (8 * g + s) + c
                    for kk in range(4):
                        v = int(dw[lane, kk])
                        for t in range(8):
                            codes[16 * T + i, 32 * b + 8 * kk + t] = (v >> (4 * ((t >> 1) + 4 * (t & 1)))) & 15
            sc = gb[nsb_g * 1024:(nsb_g + 1) * 1024].view(np.uint16).reshape(64, 8)
            for lane in range(64):
                i, c = lane & 15, lane >> 4
                for s in range(nsb_g):
                    scales[16 * T + i, 4 * (8 * g + s) + c] = sc[lane, s]
    return scales, codes


@pytest.mark.parametrize("rows,K", [(16, 128), (32, 1024), (48, 1408), (16, 2816)])
def test_pack_layout_round_trip(rows, K):
    sc, cd = S.weight_matrix(7, 0, S.MAT_QKV, None, rows, K)
    img = B.pack_matrix(sc, cd)
    assert img.size == B.lib().ps_packed_bytes(rows, K) == rows // 16 * (K // 128 + (K // 128 + 7) // 8) * 1024
    s2, c2 = _unpack(img, rows, K)
    np.testing.assert_array_equal(c2, cd)
    np.testing.assert_array_equal(s2, sc.view(np.uint16))


def test_packed_bytes_equal_algorithmic_bytes_when_k_is_a_multiple_of_1024():
    for rows, K in [(6144, 4096), (4096, 14336), (28672, 4096)]:
        assert B.lib().ps_packed_bytes(rows, K) * 32 == rows * K * 18   # 18 bytes per 32 weights


# ------------------------------------------------------------------ planner

def _plan(cfg, budget, M=1, **kw):
    p = B.Plan(cfg, int(budget), M, **kw)
    return p, p.summary(), p.shards()


def test_budget_is_honoured_and_accounts_add_up():
    for cfg, M, budgets in [(S.cfg_ffn_block(), 1, [2433024, 10 ** 7]),
                            (S.cfg_dense8b(), 1, [2e9, 4e9, 8e9]), (S.cfg_dense8b(), 2048, [4e9]),
                            (S.cfg_moe(), 16, [6e9])]:
        for b in budgets:
            p, s, sh = _plan(cfg, b, M)
            assert s.workspace_bytes + s.scratch_bytes + s.resident_bytes <= s.budget_bytes
            assert s.resident_bytes + s.streamed_bytes == s.weight_bytes
            assert sum(x.bytes for x in sh) == s.weight_bytes
            hi = s.budget_bytes - s.workspace_bytes - s.scratch_bytes     # pinned region: the head of the arena
            for x in sh:
                if x.resident:
                    assert x.offset + x.bytes <= hi
                else:
                    assert x.bytes <= s.slot_bytes
            # resident shards do not overlap
            iv = sorted((x.offset, x.offset + x.bytes) for x in sh if x.resident)
            assert all(a[1] <= b_[0] for a, b_ in zip(iv, iv[1:]))


def test_dense_8b_expected_splits():
    _, s, _ = _plan(S.cfg_dense8b(), 4e9, 1)
    assert s.weight_bytes == 3925868544 and s.streamed_bytes == 0 and s.n_slots == 0
    _, s, sh = _plan(S.cfg_dense8b(), 2e9, 1)
    attn = sum(x.bytes for x in sh if x.cls == B.PS_CLASS_ATTN)
    assert attn == 32 * (14155776 + 9437184)
    assert all(x.resident for x in sh if x.cls == B.PS_CLASS_ATTN)
    assert 1.9e9 < s.streamed_bytes < 2.1e9
    _, s, _ = _plan(S.cfg_dense8b(), 4e9, 2048)
    assert 0 < s.streamed_bytes < 0.35e9


def test_priority_attention_before_ffn_and_first_fit():
    # Section 3: attention sub-layers are pinned before FFN sub-layers, dense and MoE alike
    for cfg, b, M in [(S.cfg_dense8b(), 1.0e9, 1), (S.cfg_moe(), 6e9, 1), (S.cfg_moe(4), 0.3e9, 16)]:
        _, s, sh = _plan(cfg, b, M)
        attn_streamed = [x for x in sh if x.cls == B.PS_CLASS_ATTN and not x.resident]
        ffn_resident = [x for x in sh if x.cls == B.PS_CLASS_FFN and x.resident]
        if attn_streamed:
            free = s.budget_bytes - s.workspace_bytes - s.scratch_bytes - s.resident_bytes
            assert not ffn_resident or all(x.bytes > free for x in attn_streamed)
        ranks = [x.priority_rank for x in sh if x.cls == B.PS_CLASS_ATTN]
        assert max(ranks) < min(x.priority_rank for x in sh if x.cls == B.PS_CLASS_FFN)


def test_pinned_layers_of_a_class_are_spread_over_the_stack():
    # Algorithm 1 fixes the order of the classes only (SortByPriority).  Inside a class this planner ranks the
    # layers in a spread walk, so that whatever prefix of the class a budget pins lies evenly between the
    # streamed layers (their kernels then run beside the next streamed layer's copies), and the ranking does
    # not depend on the token count (every tier of a budget pins a prefix of the same list).
    for L in (32, 12, 5):
        cfg = S.cfg_dense8b(L)
        per_layer = 122683392
        rank_by_tokens = []
        for M in (1, 64, 2048):
            _, s, sh = _plan(cfg, 0.5 * L * per_layer + 0.35e9, M)   # room for the workspace and the two slots
            rank_by_tokens.append({(x.layer, x.kind): x.priority_rank for x in sh if x.tile0 == 0 or x.resident == 1})
            pinned = sorted({x.layer for x in sh if x.kind == B.PS_SHARD_GATE_UP and x.resident == 1 and x.ntiles == 14336 * 2 // 16})
            assert len(pinned) >= 2
            # no run of streamed layers longer than twice the even spacing, at the ends included
            gaps = [b - a for a, b in zip([-1] + pinned, pinned + [L])]
            assert max(gaps) <= 2 * -(-L // len(pinned)), (L, M, pinned)
            assert pinned[0] == 0
        assert rank_by_tokens[0] == rank_by_tokens[1] == rank_by_tokens[2]
        # a class's ranks: one permutation of the layers, matrices of a layer next to each other
        ffn = sorted((r, k) for k, r in rank_by_tokens[0].items() if k[1] in (B.PS_SHARD_GATE_UP, B.PS_SHARD_DOWN))
        layers = [k[0] for _, k in ffn]
        assert layers[0::2] == layers[1::2] and sorted(layers[0::2]) == list(range(L))


def test_streamed_bytes_monotone_in_budget():
    # the paper's evaluation appendix: throughput rises with budget; here: streamed bytes never rise
    cfg = S.cfg_dense8b(8)
    prev = None
    for b in np.linspace(0.2e9, 1.2e9, 21):
        _, s, _ = _plan(cfg, b, 1)
        if prev is not None:
            assert s.streamed_bytes <= prev
        prev = s.streamed_bytes
    assert prev == 0


def test_budget_too_small_is_an_error_not_a_crash():
    with pytest.raises(B.PshardError) as e:
        B.Plan(S.cfg_dense8b(), 10 ** 6, 1)
    assert e.value.code == B.PS_E_BUDGET
    with pytest.raises(B.PshardError) as e:
        B.Plan(dict(S.cfg_dense8b(), hidden=4000), 10 ** 9, 1)
    assert e.value.code == B.PS_E_ARG
    with pytest.raises(B.PshardError):
        B.Plan(S.cfg_dense8b(), 10 ** 9, 0)
    # the no-residual flag is the bare dense FFN block's (benchmark config 1): an MoE layer's combine keeps its residual
    with pytest.raises(B.PshardError) as e:
        B.Plan(dict(S.cfg_moe(2), no_residual=True), 10 ** 10, 1)
    assert e.value.code == B.PS_E_ARG


def test_expert_frequency_ranks_hot_experts_first():
    cfg = S.cfg_moe(2)
    rng = np.random.default_rng(0)
    freq = rng.random((2, 128)).astype(np.float32)
    freq *= 8 / freq.sum(1, keepdims=True)
    p, s, sh = _plan(cfg, 0.2e9, 1, expert_freq=freq)
    ex = [x for x in sh if x.kind == B.PS_SHARD_EXPERT]
    res = [freq[x.layer, x.expert] for x in ex if x.resident]
    non = [freq[x.layer, x.expert] for x in ex if not x.resident]
    assert res and non and min(res) >= max(non)
    # without frequencies: (layer, expert) order
    _, _, sh2 = _plan(cfg, 0.2e9, 1)
    ex2 = [x for x in sh2 if x.kind == B.PS_SHARD_EXPERT]
    flags = [x.resident for x in ex2]
    assert flags == sorted(flags, reverse=True)


def test_estimate_is_sum_of_max_compute_next_copy_on_a_toy():
    # Section 3, timing estimation: shard time = max(own compute, concurrent copy of the next shard);
    # plan time = sum.  Toy: FFN block, 1 layer, hand-computed from the shard list.
    cfg = S.cfg_ffn_block()
    prof = B.make_profile(h2d_gbps=10.0, gemv_gbps=100.0, gemm_tflops=1000.0, launch_us=2.0)
    p, s, sh = _plan(cfg, 2433024, 1, profile=prof)
    comp = [x.bytes / 100e9 * 1e3 + 2e-3 for x in sh]
    copy = [0.0 if x.resident else x.bytes / 10e9 * 1e3 for x in sh]
    want = copy[0] + sum(max(comp[i], copy[i + 1] if i + 1 < len(sh) else 0.0) for i in range(len(sh)))
    assert abs(s.est_step_ms - want) < 1e-9 * max(1, want)
    # compute-bound pricing takes over when the GEMM rate is the smaller roof
    prof2 = B.make_profile(h2d_gbps=10.0, gemv_gbps=1e6, gemm_tflops=1e-3, launch_us=0.0)
    _, s2, sh2 = _plan(cfg, 10 ** 8, 1, profile=prof2)
    want2 = sum(2.0 * (x.bytes / 0.5625) / 1e9 * 1e3 for x in sh2)
    assert abs(s2.est_step_ms - want2) < 1e-6 * want2


def test_greedy_pinning_vs_brute_force_on_few_shards():
    # with <= 12 whole shards: the pinned set respects priority (no lower-priority shard pinned
    # while a higher-priority one that would fit in its place is streamed) and the budget
    cfg = dict(S.cfg_dense8b(3), hidden=512, n_q_heads=4, n_kv_heads=2, ffn_inter=1408)
    for b in [0.6e6, 1.2e6, 2.5e6, 4e6, 9e6]:
        try:
            _, s, sh = _plan(cfg, b, 1)
        except B.PshardError:
            continue
        cap = s.budget_bytes - s.workspace_bytes - s.scratch_bytes
        assert s.resident_bytes <= cap
        whole = {}
        for x in sh:
            whole.setdefault((x.layer, x.kind), []).append(x)
        order = sorted(whole, key=lambda k: whole[k][0].priority_rank)
        # replay first-fit by hand
        rem, split = cap, False
        for k in order:
            tot = sum(x.bytes for x in whole[k])
            pinned = sum(x.bytes for x in whole[k] if x.resident)
            if tot <= rem:
                assert pinned == tot
                rem -= tot
            elif not split:
                split = True
                assert pinned <= rem
                rem -= pinned
            else:
                assert pinned == 0


# ------------------------------------------------------------------ schedule

def test_schedules_validate_and_copy_every_streamed_shard_once():
    for cfg, b, M in [(S.cfg_ffn_block(), 2433024, 1), (S.cfg_dense8b(), 2e9, 1), (S.cfg_dense8b(4), 0.25e9, 64)]:
        p, s, sh = _plan(cfg, b, M)
        sc = p.schedule()
        sc.validate()
        ops = sc.ops()
        copies = [o for o in ops if o.type == B.PS_OP_COPY]
        assert sorted(o.shard0 for o in copies) == [i for i, x in enumerate(sh) if not x.resident]
        assert sum(o.bytes for o in copies) == s.streamed_bytes
        for o in copies:
            assert o.slot in (0, 1) and o.slot_offset + o.bytes <= s.slot_bytes


def test_moe_schedule_copies_only_selected_nonresident_experts_after_routing():
    cfg = S.cfg_moe(3)
    M = 4
    lg = S.router_logits(1, 0, 3, M, 128)
    p, s, sh = _plan(cfg, 0.4e9, M)
    sc = p.schedule(lg)
    sc.validate()
    ops = sc.ops()
    routed = set()
    for l in range(3):
        idx = B.route_host(lg[l], 8)
        routed |= {(l, int(e)) for e in idx.ravel()}
    want = sorted(i for i, x in enumerate(sh) if x.kind == B.PS_SHARD_EXPERT and not x.resident
                  and (x.layer, x.expert) in routed)
    copies = [o for o in ops if o.type == B.PS_OP_COPY and sh[o.shard0].kind == B.PS_SHARD_EXPERT]
    assert sorted(o.shard0 for o in copies) == want
    seen_route = set()
    for o in ops:
        if o.type == B.PS_OP_KERNEL and o.kernel == B.PS_K_ROUTE:
            seen_route.add(o.layer)
        if o.type == B.PS_OP_COPY and sh[o.shard0].kind == B.PS_SHARD_EXPERT:
            assert o.flags & B.PS_OPF_WAIT_ROUTER and o.layer in seen_route


def test_route_host_matches_sort_rule():
    lg = S.router_logits(5, 0, 1, 9, 128)[0]
    lg[0, :] = 0.0
    lg[1, [7, 90]] = 10.0
    idx = B.route_host(lg, 8)
    for m in range(9):
        assert list(idx[m]) == sorted(range(128), key=lambda e: (-float(lg[m, e]), e))[:8]


# ------------------------------------------------------------------ token-tier table, PickTier

def test_tier_table_plans_every_tier_and_smaller_tiers_pin_more():
    cfg = S.cfg_dense8b(32)
    tb = B.TierTable(cfg, int(2e9))
    ents = tb.entries()
    assert [e.tier_tokens for e in ents] == [B.lib().ps_tier_tokens(t) for t in range(B.PS_NTIERS)]
    assert all(e.feasible for e in ents)
    for e in ents:
        assert e.summary.n_tokens == e.tier_tokens and e.summary.budget_bytes == int(2e9)
        one = B.Plan(cfg, int(2e9), e.tier_tokens).summary()     # same as planning that tier alone
        assert (one.resident_bytes, one.workspace_bytes, one.est_step_ms) == \
               (e.summary.resident_bytes, e.summary.workspace_bytes, e.summary.est_step_ms)
    res = [e.summary.resident_bytes for e in ents]
    assert all(a >= b for a, b in zip(res, res[1:])) and res[0] > res[-1]   # Section 3: lower tiers pin more
    p = tb.plan(5)
    assert p.summary().n_tokens == 512 and len(p.shards()) == ents[5].summary.n_shards


def test_tier_table_marks_tiers_that_do_not_fit():
    cfg = S.cfg_dense8b(32)
    tb = B.TierTable(cfg, int(3e8))
    feas = [e.feasible for e in tb.entries()]
    assert feas[0] == 1 and feas[-1] == 0 and feas == sorted(feas, reverse=True)
    with pytest.raises(B.PshardError):
        tb.plan(B.PS_NTIERS - 1)
    c = tb.pick(16384)          # must fall back to a feasible tier and iterate
    assert tb.entry(c.tier).feasible and c.iterations == -(-16384 // c.tier_tokens)
    none = B.TierTable(cfg, 1000)
    assert not any(e.feasible for e in none.entries())
    with pytest.raises(B.PshardError) as ei:
        none.pick(1)
    assert ei.value.code == B.PS_E_BUDGET
    with pytest.raises(B.PshardError):
        tb.pick(0)


def test_pick_tier_matches_the_definition():
    from oracle import oracle as O
    rng = np.random.default_rng(5)
    for cfg, budgets in ((S.cfg_dense8b(32), (3e8, 2e9, 4e9)), (S.cfg_moe(4), (3e8, 2e9))):
        for budget in budgets:
            for gemm in (50.0, 400.0, 1000.0):
                tb = B.TierTable(cfg, int(budget), profile=B.make_profile(gemm_tflops=gemm))
                est = [e.summary.est_step_ms if e.feasible else None for e in tb.entries()]
                for n in [1, 2, 4, 5, 63, 64, 65, 100, 512, 2048, 3000, 16384, 50000] + list(rng.integers(1, 40000, 20)):
                    c = tb.pick(int(n))
                    t, iters, total = O.pick_tier(est, int(n))
                    assert (c.tier, c.iterations) == (t, iters), (budget, gemm, n)
                    assert c.tier_tokens == O.TIER_TOKENS[t] and c.est_iter_ms == est[t]
                    assert c.est_total_ms == pytest.approx(total, rel=1e-12)


# ------------------------------------------------------------------ KV cache as a shard class

def _kv_cfg(n_layers=3, ctx=700):
    return dict(n_layers=n_layers, hidden=512, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_inter=1408,
                n_experts=0, top_k=0, expert_inter=0, rms_eps=1e-6, no_attn=False, no_residual=False, kv_context=ctx)


def test_kv_cache_shards_rank_between_attention_and_ffn():
    # Section 3, planning phase: priority attention > KV cache > FFN > outputs
    cfg = _kv_cfg()
    full = B.Plan(cfg, 1 << 40, 1)
    sh = full.shards()
    kv = [s for s in sh if s.kind == B.PS_SHARD_KV]
    assert len(kv) == cfg["n_layers"] * cfg["n_kv_heads"]
    assert all(s.bytes == cfg["kv_context"] * 128 * 2 * 2 and s.cls == B.PS_CLASS_KVCACHE for s in kv)
    rank = lambda kind: [s.priority_rank for s in sh if s.kind == kind]
    assert max(rank(B.PS_SHARD_QKV) + rank(B.PS_SHARD_O)) < min(rank(B.PS_SHARD_KV))
    assert max(rank(B.PS_SHARD_KV)) < min(rank(B.PS_SHARD_GATE_UP) + rank(B.PS_SHARD_DOWN))
    # execution order inside a layer: QKV, the kv heads, O, gate/up, down
    kinds = [s.kind for s in sh if s.layer == 1]
    first = {k: kinds.index(k) for k in set(kinds)}
    assert first[B.PS_SHARD_QKV] < first[B.PS_SHARD_KV] < first[B.PS_SHARD_O] < first[B.PS_SHARD_GATE_UP]
    # a budget that holds attention and part of the caches: caches fill before any FFN shard is pinned
    attn = sum(s.bytes for s in sh if s.kind in (B.PS_SHARD_QKV, B.PS_SHARD_O))
    kvb = sum(s.bytes for s in kv)
    ws = full.summary().workspace_bytes
    slot = B.Plan(cfg, ws + attn + kvb, 1).summary().slot_bytes       # what two scratch slots take here
    plan = B.Plan(cfg, ws + attn + kvb // 2 + 2 * slot + 4096, 1)
    got = plan.shards()
    res_kv = [s for s in got if s.kind == B.PS_SHARD_KV and s.resident]
    assert 0 < len(res_kv) < len(kv)
    assert all(s.resident for s in got if s.kind in (B.PS_SHARD_QKV, B.PS_SHARD_O))
    big_ffn = [s for s in got if s.kind in (B.PS_SHARD_GATE_UP, B.PS_SHARD_DOWN) and s.resident and s.bytes > kv[0].bytes]
    assert not big_ffn     # first fit: only FFN slabs smaller than the cache shard that missed may slip in
    sched = plan.schedule()
    sched.validate()
    ops = sched.ops()
    attn_ops = [o for o in ops if o.type == B.PS_OP_KERNEL and o.kernel == B.PS_K_ATTN]
    comb_ops = [o for o in ops if o.type == B.PS_OP_KERNEL and o.kernel == B.PS_K_ATTN_COMBINE]
    assert len(comb_ops) == cfg["n_layers"] and sum(o.nshards for o in attn_ops) == len(kv)
    copied = [o.shard0 for o in ops if o.type == B.PS_OP_COPY]
    assert sorted(copied) == [i for i, s in enumerate(got) if not s.resident]


def test_kv_cache_plans_take_chunks_that_fit_the_cache():
    """With a KV cache a plan takes one token, or a chunk of new tokens (chunked prefill over the cache);
    the chunk must leave room in the cache, and its attention partials count as workspace, so the
    tier table has a schedule for every tier that fits."""
    cfg = _kv_cfg()
    cap = cfg["kv_context"]
    p1, p16 = B.Plan(cfg, 1 << 40, 1).summary(), B.Plan(cfg, 1 << 40, 16).summary()
    assert p16.workspace_bytes > p1.workspace_bytes
    with pytest.raises(B.PshardError) as e:
        B.Plan(cfg, 1 << 40, cap)               # a chunk as long as the cache leaves no room
    assert e.value.code == B.PS_E_BUDGET
    tb = B.TierTable(cfg, 1 << 40)
    feas = [bool(x.feasible) for x in tb.entries()]
    assert feas == [B.lib().ps_tier_tokens(t) < cap for t in range(B.PS_NTIERS)] and feas[0] and feas[2]
    assert tb.pick(1).tier == 0
    prof = B.make_profile(cpu_gbps=150.0)
    with pytest.raises(B.PshardError):          # chunks over a cache keep the GPU-only plan
        B.Plan(cfg, 1 << 40, 16, profile=prof, kind=B.PS_PLAN_STATIC)
    bad = dict(cfg, no_attn=True)
    with pytest.raises(B.PshardError):
        B.Plan(bad, 1 << 40, 1)


# ---------------------------------------------------------------- output head ("outputs" class)

def _head_cfg(vocab=1040, **kw):
    return dict(_kv_cfg(**kw), kv_context=0, vocab=vocab)


def test_output_head_is_the_lowest_priority_class_and_runs_last():
    # Section 3, planning phase: priority attention > KV cache > FFN > outputs
    cfg = _head_cfg(vocab=8192)   # the head is the largest matrix: a small shortfall costs only head slabs
    full = B.Plan(cfg, 1 << 40, 1)
    sh = full.shards()
    out = [s for s in sh if s.kind == B.PS_SHARD_OUT]
    assert len(out) == 1 and out[0].cls == B.PS_CLASS_OUTS and out[0].layer == cfg["n_layers"]
    assert out[0].bytes == B.lib().ps_packed_bytes(cfg["vocab"], cfg["hidden"])
    assert out[0].priority_rank == len(sh) - 1 and sh[-1].kind == B.PS_SHARD_OUT
    base = B.Plan(dict(cfg, vocab=0), 1 << 40, 1).summary()
    assert full.summary().weight_bytes == base.weight_bytes + out[0].bytes
    # a budget just short of everything: head slabs are what gets streamed, nothing else
    need = full.summary().workspace_bytes + full.summary().weight_bytes
    lo = None
    for budget in range(need - 1, need // 2, -4096):
        try:
            lo = B.Plan(cfg, budget, 1)
        except B.PshardError:
            continue
        if lo.summary().n_slots:
            break
    streamed = [s for s in lo.shards() if not s.resident]
    assert streamed and all(s.kind == B.PS_SHARD_OUT for s in streamed)
    ops = lo.schedule().ops()
    assert lo.schedule().validate() is None
    kern = [o for o in ops if o.type == B.PS_OP_KERNEL]
    head = [o for o in kern if o.kernel == B.PS_K_OUT]
    assert head and all(o.layer == cfg["n_layers"] for o in head)
    assert kern.index(head[0]) == len(kern) - len(head)          # nothing after the head's kernels
    tiles = sum(lo.shards()[o.shard0].ntiles for o in head)
    assert tiles == cfg["vocab"] // 16
    # several tokens: the head gets its own RMS factors right before it
    ops16 = [o for o in B.Plan(cfg, 1 << 40, 16).schedule().ops() if o.type == B.PS_OP_KERNEL]
    i = [o.kernel for o in ops16].index(B.PS_K_OUT)
    assert ops16[i - 1].kernel == B.PS_K_RINV and ops16[i - 1].layer == cfg["n_layers"]


def test_output_head_streams_through_the_slots_when_nothing_is_pinned():
    cfg = _head_cfg(vocab=4096)
    full = B.Plan(cfg, 1 << 40, 1).summary()
    tight = B.Plan(cfg, full.workspace_bytes + full.weight_bytes // 6, 1)
    sched = tight.schedule()
    assert sched.validate() is None
    ops = sched.ops()
    copies = [o for o in ops if o.type == B.PS_OP_COPY and o.layer == cfg["n_layers"]]
    kern = [o for o in ops if o.type == B.PS_OP_KERNEL and o.kernel == B.PS_K_OUT]
    assert copies and sum(o.bytes for o in copies) == sum(o.bytes for o in kern if o.slot >= 0)
    moe = dict(S.cfg_moe(2), n_experts=8, top_k=2, vocab=2048)
    lg = S.router_logits(1, 0, 2, 4, 8)
    pm = B.Plan(moe, 1 << 40, 4)
    assert pm.shards()[-1].kind == B.PS_SHARD_OUT
    assert pm.schedule(lg).validate() is None


def test_output_head_argument_checks():
    for vocab in (1000, 8, (1 << 20) + 16):
        with pytest.raises(B.PshardError):
            B.Plan(_head_cfg(vocab=vocab), 1 << 40, 1)


# ---------------------------------------------------------------- the three schedule plans (Section 3)

def _cpu_prof(**kw):
    d = dict(h2d_gbps=50.0, gemv_gbps=4000.0, cpu_gbps=200.0, cpu_gbps_busy=150.0, h2d_gbps_busy=45.0,
             cpu_tokens_free=4.0, cpu_sync_us=20.0)
    d.update(kw)
    return B.make_profile(**d)


def _plans(cfg, budget, M=1, prof=None):
    prof = prof or _cpu_prof()
    return {k: B.Plan(cfg, budget, M, profile=prof, kind=k) for k in (B.PS_PLAN_GPU_ONLY, B.PS_PLAN_STATIC, B.PS_PLAN_DYNAMIC)}


def test_static_plan_keeps_unpinned_ffn_on_the_cpu_and_needs_no_scratch():
    # Plan Two: the unpinned low-priority sub-layers stay in system memory and run on the CPU
    cfg = _head_cfg(vocab=2048)
    full = B.Plan(cfg, 1 << 40, 1).summary()
    budget = full.workspace_bytes + full.weight_bytes // 2
    pl = _plans(cfg, budget)
    g, s = pl[B.PS_PLAN_GPU_ONLY].summary(), pl[B.PS_PLAN_STATIC].summary()
    assert s.plan_kind == B.PS_PLAN_STATIC and s.n_slots == 0 and s.scratch_bytes == 0 and s.streamed_bytes == 0
    assert s.cpu_bytes > 0 and s.resident_bytes + s.cpu_bytes == s.weight_bytes
    assert s.resident_bytes > g.resident_bytes            # the scratch went to the pinned region
    sh = pl[B.PS_PLAN_STATIC].shards()
    cpu = [x for x in sh if x.resident == 2]
    assert cpu and all(x.kind in (B.PS_SHARD_GATE_UP, B.PS_SHARD_DOWN, B.PS_SHARD_OUT) for x in cpu)
    # priority: whatever is on the CPU ranks below everything pinned whole
    whole = {}
    for x in sh:
        whole.setdefault((x.layer, x.kind), []).append(x)
    pinned_whole = [v[0].priority_rank for v in whole.values() if all(y.resident == 1 for y in v)]
    assert max(pinned_whole) < min(x.priority_rank for x in cpu) or len(cpu) == 0
    # every matrix is covered exactly once: pinned head then CPU tail
    for (layer, kind), v in whole.items():
        assert [y.tile0 for y in v] == [sum(z.ntiles for z in v[:i]) for i in range(len(v))]
        assert [y.resident for y in v] in ([1], [2], [1, 2])
    sched = pl[B.PS_PLAN_STATIC].schedule()
    assert sched.validate() is None
    ops = sched.ops()
    assert not [o for o in ops if o.type == B.PS_OP_COPY]
    ncpu = [o for o in ops if o.type == B.PS_OP_CPU]
    assert len(ncpu) == len(cpu) and sum(o.bytes for o in ncpu) == s.cpu_bytes
    for i, o in enumerate(ops):
        if o.type != B.PS_OP_CPU:
            continue
        # the activations were fetched before the GPU's kernels of the same matrix were launched
        j = i
        while j > 0 and ops[j - 1].layer == o.layer and ops[j - 1].kernel == o.kernel and ops[j - 1].type == B.PS_OP_KERNEL:
            j -= 1
        want = {B.PS_K_GATE_UP: B.PS_BUF_H, B.PS_K_DOWN: B.PS_BUF_S | B.PS_BUF_H, B.PS_K_OUT: B.PS_BUF_X}[o.kernel]
        assert o.buffers == want
        if ops[j - 1].type == B.PS_OP_FETCH and ops[j - 1].kernel == o.kernel:
            assert ops[j - 1].buffers & want


def test_dynamic_plan_splits_unpinned_matrices_between_pcie_and_cpu():
    # Plan Three: fewer sub-layers on the CPU, the rest time-share the scratch double buffer
    cfg = _kv_cfg(n_layers=4, ctx=0)
    cfg = dict(cfg, kv_context=0)
    full = B.Plan(cfg, 1 << 40, 1).summary()
    budget = full.workspace_bytes + full.weight_bytes // 3
    pl = _plans(cfg, budget, prof=_cpu_prof(cpu_sync_us=0.5))   # matrices of under 1 MB: keep the fixed cost small too
    d = pl[B.PS_PLAN_DYNAMIC].summary()
    s = pl[B.PS_PLAN_STATIC].summary()
    assert d.n_slots == 2 and d.cpu_bytes > 0 and d.streamed_bytes > 0
    assert s.streamed_bytes == 0 and d.cpu_bytes < d.weight_bytes - d.resident_bytes   # only part of the unpinned bytes
    assert d.resident_bytes + d.streamed_bytes + d.cpu_bytes == d.weight_bytes
    assert 0.0 < d.cpu_fraction < 1.0
    # with the CPU three times as fast as PCIe, most of the unpinned bytes are the CPU's
    assert d.cpu_bytes > d.streamed_bytes
    sh = pl[B.PS_PLAN_DYNAMIC].shards()
    by = {}
    for x in sh:
        by.setdefault((x.layer, x.kind), []).append(x)
    for v in by.values():   # pinned head, streamed slabs, CPU tail, contiguous
        res = [y.resident for y in v]
        assert res == sorted(res, key=lambda r: {1: 0, 0: 1, 2: 2}[r])
        assert [y.tile0 for y in v] == [sum(z.ntiles for z in v[:i]) for i in range(len(v))]
    sched = pl[B.PS_PLAN_DYNAMIC].schedule()
    assert sched.validate() is None
    ops = sched.ops()
    assert [o for o in ops if o.type == B.PS_OP_COPY] and [o for o in ops if o.type == B.PS_OP_CPU]
    # a slower CPU gets a smaller share
    slow = B.Plan(cfg, budget, 1, profile=_cpu_prof(cpu_gbps=60.0, cpu_gbps_busy=40.0, cpu_sync_us=0.5), kind=B.PS_PLAN_DYNAMIC).summary()
    assert slow.cpu_fraction < d.cpu_fraction


def test_heuristic_split_returns_the_plan_with_the_lowest_estimate():
    cfg = _kv_cfg(n_layers=4, ctx=0)
    cfg = dict(cfg, kv_context=0)
    full = B.Plan(cfg, 1 << 40, 1).summary()
    budget = full.workspace_bytes + full.weight_bytes // 3
    for prof in (_cpu_prof(), _cpu_prof(cpu_gbps=10.0, cpu_gbps_busy=8.0), _cpu_prof(cpu_gbps=2000.0, cpu_gbps_busy=2000.0)):
        pl = _plans(cfg, budget, prof=prof)
        est = [pl[k].summary().est_step_ms for k in range(3)]
        auto = B.Plan(cfg, budget, 1, profile=prof, kind=B.PS_PLAN_AUTO).summary()
        assert list(auto.est_kind_ms) == pytest.approx(est)
        assert auto.plan_kind == int(np.argmin(est)) and auto.est_step_ms == pytest.approx(min(est))
    # a CPU far slower than PCIe: Plan One; everything fits: nothing to split, Plan One as well
    assert B.Plan(cfg, budget, 1, profile=_cpu_prof(cpu_gbps=5.0, cpu_gbps_busy=5.0), kind=B.PS_PLAN_AUTO).summary().plan_kind == B.PS_PLAN_GPU_ONLY
    roomy = B.Plan(cfg, 1 << 40, 1, profile=_cpu_prof(), kind=B.PS_PLAN_AUTO).summary()
    assert roomy.plan_kind == B.PS_PLAN_GPU_ONLY and roomy.cpu_bytes == 0
    # prefill-sized tiers never go to the CPU back-end; no CPU rate in the profile: Plan One only
    big = B.Plan(cfg, budget * 4, 512, profile=_cpu_prof(), kind=B.PS_PLAN_AUTO).summary()
    assert big.plan_kind == B.PS_PLAN_GPU_ONLY and list(big.est_kind_ms)[1:] == [-1.0, -1.0]
    none = B.Plan(cfg, budget, 1, kind=B.PS_PLAN_AUTO).summary()
    assert none.plan_kind == B.PS_PLAN_GPU_ONLY
    with pytest.raises(B.PshardError):
        B.Plan(cfg, budget, 1, kind=B.PS_PLAN_STATIC)          # default profile has no CPU rate
    with pytest.raises(B.PshardError):
        B.Plan(cfg, budget, 1, profile=_cpu_prof(), kind=7)


def test_cpu_plan_estimates_follow_the_papers_rule():
    """A matrix costs max(GPU side, CPU side); the CPU side is bytes / rate (+ fixed cost), slower
    beyond cpu_tokens_free tokens; contended rates apply only when a plan both streams and computes."""
    cfg = _kv_cfg(n_layers=2, ctx=0)
    cfg = dict(cfg, kv_context=0)
    full = B.Plan(cfg, 1 << 40, 1).summary()
    budget = full.workspace_bytes + full.weight_bytes // 2
    prof = _cpu_prof(cpu_sync_us=0.0, launch_us=0.0, gemv_gbps=1e9)       # GPU side ~ free
    s = B.Plan(cfg, budget, 1, profile=prof, kind=B.PS_PLAN_STATIC).summary()
    assert s.est_step_ms == pytest.approx(s.cpu_bytes / 200e9 * 1e3, rel=1e-3)
    s16 = B.Plan(cfg, budget + (1 << 20), 16, profile=prof, kind=B.PS_PLAN_STATIC).summary()
    assert s16.est_step_ms >= s16.cpu_bytes / 200e9 * 1e3 * 4 * 0.999
    d = B.Plan(cfg, budget, 1, profile=prof, kind=B.PS_PLAN_DYNAMIC)
    ds = d.summary()
    # lower bound: both resources busy the whole time at their contended rates
    lo = max(ds.cpu_bytes / 150e9, ds.streamed_bytes / 45e9) * 1e3
    assert ds.est_step_ms >= lo * 0.999
    assert ds.est_step_ms <= (ds.cpu_bytes / 150e9 + ds.streamed_bytes / 45e9) * 1e3 * 1.001


def test_cpu_plans_put_cold_unpinned_experts_on_the_cpu():
    cfg = dict(S.cfg_moe(3), n_experts=16, top_k=4)
    M = 4
    lg = S.router_logits(3, 0, 3, M, 16)
    full = B.Plan(cfg, 1 << 40, M).summary()
    budget = full.workspace_bytes + full.weight_bytes // 2
    freq = np.random.default_rng(0).random((3, 16)).astype(np.float32)
    prof = _cpu_prof(cpu_sync_us=0.5)
    st = B.Plan(cfg, budget, M, profile=prof, expert_freq=freq, kind=B.PS_PLAN_STATIC)
    s = st.summary()
    sh = st.shards()
    ex = [x for x in sh if x.kind == B.PS_SHARD_EXPERT]
    assert s.n_slots == 0 and s.streamed_bytes == 0 and s.cpu_bytes == sum(x.bytes for x in ex if x.resident == 2) > 0
    assert all(x.resident == 1 for x in sh if x.kind != B.PS_SHARD_EXPERT)
    # the pinned experts are the frequent ones
    assert min(freq[x.layer, x.expert] for x in ex if x.resident == 1) >= max(freq[x.layer, x.expert] for x in ex if x.resident == 2)
    sched = st.schedule(lg)
    assert sched.validate() is None
    ops = sched.ops()
    assert not [o for o in ops if o.type == B.PS_OP_COPY]
    for layer in range(3):
        kinds = [(o.type, o.kernel) for o in ops if o.layer == layer]
        if (B.PS_OP_CPU, B.PS_K_EXPERT_GATE_UP) in kinds:
            i_f, i_c = kinds.index((B.PS_OP_FETCH, B.PS_K_EXPERT_GATE_UP)), kinds.index((B.PS_OP_CPU, B.PS_K_EXPERT_GATE_UP))
            i_r, i_m = kinds.index((B.PS_OP_KERNEL, B.PS_K_ROUTE)), kinds.index((B.PS_OP_KERNEL, B.PS_K_COMBINE))
            assert i_r < i_f < i_c < i_m
            gpu = [i for i, k in enumerate(kinds) if k == (B.PS_OP_KERNEL, B.PS_K_EXPERT_GATE_UP)]
            assert all(i_f < i < i_c for i in gpu)     # the GPU's experts are in flight while the host computes
    dy = B.Plan(cfg, budget, M, profile=prof, expert_freq=freq, kind=B.PS_PLAN_DYNAMIC)
    d = dy.summary()
    assert d.n_slots == 2 and d.cpu_bytes > 0 and d.resident_bytes + d.streamed_bytes + d.cpu_bytes == d.weight_bytes
    dex = [x for x in dy.shards() if x.kind == B.PS_SHARD_EXPERT]
    if d.streamed_bytes:   # streamed experts outrank the CPU's
        assert max(x.priority_rank for x in dex if x.resident == 0) < min(x.priority_rank for x in dex if x.resident == 2)
    assert dy.schedule(lg).validate() is None
    auto = B.Plan(cfg, budget, M, profile=prof, expert_freq=freq, kind=B.PS_PLAN_AUTO).summary()
    assert auto.est_step_ms == pytest.approx(min(e for e in auto.est_kind_ms if e >= 0))


def test_tier_table_plans_each_small_tier_with_heuristic_split():
    # Algorithm 1: for every tier, HeuristicSplit; the CPU back-end serves tiers of at most 64 tokens
    cfg = _kv_cfg(n_layers=4, ctx=0)
    cfg = dict(cfg, kv_context=0)
    full = B.Plan(cfg, 1 << 40, 1).summary()
    budget = full.workspace_bytes + full.weight_bytes // 3 + (1 << 20)
    prof = _cpu_prof(cpu_sync_us=0.5)
    tb = B.TierTable(cfg, budget, profile=prof, kind=B.PS_PLAN_AUTO)
    base = B.TierTable(cfg, budget, profile=prof)
    for e, b in zip(tb.entries(), base.entries()):
        assert e.feasible == b.feasible
        if not e.feasible:
            continue
        if e.tier_tokens > 64:
            assert e.summary.plan_kind == B.PS_PLAN_GPU_ONLY and e.summary.est_step_ms == b.summary.est_step_ms
        else:
            want = B.Plan(cfg, budget, e.tier_tokens, profile=prof, kind=B.PS_PLAN_AUTO).summary()
            assert e.summary.plan_kind == want.plan_kind and e.summary.est_step_ms == pytest.approx(want.est_step_ms)
            assert e.summary.est_step_ms <= b.summary.est_step_ms * (1 + 1e-12)
    assert tb.entry(0).summary.plan_kind != B.PS_PLAN_GPU_ONLY        # one token, CPU 4x PCIe: a CPU plan wins
    assert tb.pick(1).est_total_ms <= base.pick(1).est_total_ms
    with pytest.raises(B.PshardError):
        B.TierTable(cfg, budget, profile=prof, kind=9)


# ---------------------------------------------------------------- profile database (Section 3)

def _golden_db():
    from tests.test_oracle_pins import _profile_golden
    ent, qs = _profile_golden()
    db = B.ProfileDB()
    for e in ent:
        db.add(*e)
    return db, ent, qs


def test_profile_db_lookup_matches_the_papers_rule():
    from oracle import oracle as O
    db, ent, qs = _golden_db()
    assert db.entries() == ent
    names = {B.PS_MATCH_NONE: "none", B.PS_MATCH_EXACT: "exact", B.PS_MATCH_NEIGHBOUR: "neighbour"}
    for bw, q, want_ms, want_match in qs:           # the hand-worked examples
        r = db.estimate(bw, *q)
        assert names[r.match] == want_match and r.ms == pytest.approx(want_ms, rel=1e-9)
    rng = np.random.default_rng(5)                  # and a seeded sweep against the oracle
    ent2 = []
    db2 = B.ProfileDB()
    for _ in range(40):
        e = (int(rng.integers(0, 3)), 4, int(rng.choice([0, 8, 16])), int(2 ** rng.integers(4, 15)), int(128 * rng.integers(1, 64)),
             int(rng.choice([1, 4, 16, 64, 512])), float(rng.uniform(0.01, 5.0)))
        if any(o[:6] == e[:6] for o in ent2):
            continue
        ent2.append(e)
        db2.add(*e)
    for _ in range(300):
        q = (int(rng.integers(0, 3)), 4, int(rng.choice([0, 8, 16])), int(16 * rng.integers(1, 2000)), int(128 * rng.integers(1, 64)),
             int(rng.integers(1, 600)))
        bw = float(rng.choice([0.5, 50.0, 5000.0]))
        want_ms, want_match = O.profile_estimate(ent2, bw, *q)
        r = db2.estimate(bw, *q)
        assert names[r.match] == want_match and r.ms == pytest.approx(want_ms, rel=1e-9), q
    for e in ent2[:5]:
        assert db2.estimate(1.0, *e[:6]).match == B.PS_MATCH_EXACT
    # the same key again replaces the measurement; bad entries are refused
    db2.add(*ent2[0][:6], 9.0)
    assert db2.estimate(1.0, *ent2[0][:6]).ms == 9.0 and len(db2.entries()) == len(ent2)
    for bad in ((7, 4, 0, 16, 128, 1, 1.0), (0, 4, 0, 0, 128, 1, 1.0), (0, 4, 0, 16, 128, 1, 0.0)):
        with pytest.raises(B.PshardError):
            db2.add(*bad)


def test_profile_db_file_round_trip(tmp_path):
    db, ent, _ = _golden_db()
    path = tmp_path / "profile.txt"
    db.save(path)
    other = B.ProfileDB()
    other.load(path)
    assert other.entries() == ent
    (tmp_path / "bad.txt").write_text("0 4 0 16 not-a-number\n")
    with pytest.raises(B.PshardError):
        other.load(tmp_path / "bad.txt")
    with pytest.raises(B.PshardError):
        other.load(tmp_path / "missing.txt")


def test_plans_priced_from_a_profile_database():
    cfg = _kv_cfg(n_layers=2, ctx=0)
    cfg = dict(cfg, kv_context=0)
    H, I = cfg["hidden"], cfg["ffn_inter"]
    full = B.Plan(cfg, 1 << 40, 1).summary()
    budget = full.workspace_bytes + full.weight_bytes // 2
    prof = _cpu_prof(cpu_sync_us=0.0, launch_us=0.0)
    db = B.ProfileDB()
    # every matrix of the model as a one-token GPU kernel, 1 ms each: an all-resident plan sums them
    qkv_rows = (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"]
    for n, k in ((qkv_rows, H), (H, cfg["n_q_heads"] * cfg["head_dim"]), (2 * I, H), (H, I)):
        db.add(B.PS_OPK_GEMV, 4, 0, n, k, 1, 1.0)
    roomy = B.Plan(cfg, 1 << 40, 1, profile=prof, kind=B.PS_PLAN_GPU_ONLY, db=db).summary()
    assert roomy.est_step_ms == pytest.approx(4.0 * cfg["n_layers"])
    base = B.Plan(cfg, 1 << 40, 1, profile=prof).summary()
    assert base.est_step_ms != pytest.approx(roomy.est_step_ms)
    # a CPU that the database shows to be very slow keeps HeuristicSplit on the GPU; a fast one does not
    for cpu_ms, want_gpu in ((1000.0, True), (1e-4, False)):
        d2 = B.ProfileDB()
        for e in db.entries():
            d2.add(*e)
        for n, k in ((2 * I, H), (H, I)):
            d2.add(B.PS_OPK_CPU, 4, 16, n, k, 1, cpu_ms)
        auto = B.Plan(cfg, budget, 1, profile=prof, kind=B.PS_PLAN_AUTO, db=d2).summary()
        assert (auto.plan_kind == B.PS_PLAN_GPU_ONLY) == want_gpu
    # copies priced from H2D entries: a streamed plan's estimate follows the database's copy rate
    slow_copy, fast_copy = B.ProfileDB(), B.ProfileDB()
    slow_copy.add(B.PS_OPK_H2D, 0, 0, 1 << 20, 1, 1, 1.0)       # 1 GB/s
    fast_copy.add(B.PS_OPK_H2D, 0, 0, 1 << 20, 1, 1, 0.001)     # 1 TB/s
    a = B.Plan(cfg, budget, 1, profile=prof, kind=B.PS_PLAN_GPU_ONLY, db=slow_copy).summary()
    b = B.Plan(cfg, budget, 1, profile=prof, kind=B.PS_PLAN_GPU_ONLY, db=fast_copy).summary()
    assert a.est_step_ms == pytest.approx(a.streamed_bytes / (1 << 20) * 1.0, rel=0.05) and b.est_step_ms < a.est_step_ms / 50


def test_tier_table_priced_from_a_profile_database():
    # The paper's overview: the install-time profile database feeds the estimator that fills the
    # (token tier, schedule) table.  Every tier of the table carries the estimate of the plan built for
    # that tier alone from the same database, and PickTier follows those estimates: with 64-token GEMMs
    # priced absurdly slow in the database the pick moves off that tier, which the profile alone would take.
    cfg = dict(_kv_cfg(n_layers=2, ctx=0), kv_context=0)
    H, I = cfg["hidden"], cfg["ffn_inter"]
    prof = _cpu_prof(cpu_sync_us=0.0, launch_us=0.0)
    qkv_rows = (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"]
    mats = ((qkv_rows, H), (H, cfg["n_q_heads"] * cfg["head_dim"]), (2 * I, H), (H, I))
    db = B.ProfileDB()
    for n, k in mats:
        db.add(B.PS_OPK_GEMV, 4, 0, n, k, 1, 0.5)
        for m, ms in ((4, 0.6), (16, 0.7), (32, 0.8), (64, 1000.0), (512, 3.0)):
            db.add(B.PS_OPK_GEMM, 4, 0, n, k, m, ms)
    budget = 1 << 34
    table = B.TierTable(cfg, budget, profile=prof, db=db)
    plain = B.TierTable(cfg, budget, profile=prof)
    for e in table.entries():
        if not e.feasible:
            continue
        alone = B.Plan(cfg, budget, e.tier_tokens, profile=prof, kind=B.PS_PLAN_GPU_ONLY, db=db).summary()
        assert e.summary.est_step_ms == alone.est_step_ms
    by_tokens = {e.tier_tokens: e.summary.est_step_ms for e in table.entries() if e.feasible}
    assert by_tokens[1] == pytest.approx(0.5 * 4 * cfg["n_layers"]) and by_tokens[64] == pytest.approx(1000.0 * 4 * cfg["n_layers"])
    fair = B.ProfileDB()
    for e in db.entries():
        fair.add(*e[:6], 0.9 if e[5] == 64 else e[6])
    assert B.TierTable(cfg, budget, profile=prof, db=fair).pick(64).tier_tokens == 64     # 0.9 x 1 trip < 0.8 x 2 trips
    assert plain.entry(0).summary.est_step_ms != pytest.approx(by_tokens[1])
    c = table.pick(64)
    assert c.tier_tokens == 32 and c.iterations == 2 and c.est_total_ms == pytest.approx(2 * 0.8 * 4 * cfg["n_layers"])
    with pytest.raises(B.PshardError):     # a NULL database is refused
        B._check(B.lib().ps_tier_table_create_db(B.C.byref(table.desc), budget, B.C.byref(prof), None, None, 0, B.C.byref(B.C.c_void_p())))


# ------------------------------------------------------------------ build-time checks

def _fake_gemm_isa(prologue_wait, step_loads, step_wait):
    lds = "\tbuffer_load_dwordx4 v1, s[4:7], 0 offen lds\n"
    w4, w1 = "\tbuffer_load_dwordx4 v[2:5], v1, s[4:7], 0 offen\n", "\tbuffer_load_dword v6, v1, s[4:7], 0 offen\n"
    kinds = {"lds": lds, "w4": w4, "w1": w1, "g": "\tglobal_load_dword v7, v[8:9], off\n"}
    step = "".join(kinds[k] for k in step_loads) + "\ts_waitcnt vmcnt(%d) lgkmcnt(0)\n\ts_barrier\n" % step_wait
    return ("_ZN2ps14gemm_w4_kernelILi0ELi2ELi16ELb0ELi4EEEvNS_8GemmArgsE: ; @x\n" + lds + lds + lds + w4 + w4 +
            "\ts_waitcnt vmcnt(%d)\n\ts_barrier\n" % prologue_wait + step + step +
            "\tglobal_store_dword v[8:9], v7, off\n\ts_endpgm\n.Lfunc_end0:\n")


def test_build_check_of_the_gemm_wait_counts(tmp_path):
    """The build refuses generated code in which the GEMM's hand-counted waits would not name the loads
    they are meant to: an opening wait that is not vmcnt(0), a counted step with a load too few or too
    many, fills that do not come first, or a foreign memory operation inside the ring."""
    from paper_2604_26334_amd import build as Bd
    assert Bd.gemm_wait_counts(16, 4) == (3, 1, 3)        # 1 fill + 2 weight loads, one prefetch may be in flight
    assert Bd.gemm_wait_counts(64, 4) == (6, 4, 6)
    assert Bd.gemm_wait_counts(128, 4) == (10, 8, 0)      # one super-block of lookahead: every step waits for all
    assert Bd.gemm_wait_counts(128, 8) == (6, 4, 8)       # three of lookahead: one prefetch and the next one's weights
    good = ["lds", "w4", "w4"]
    scales = ["lds", "lds"] + good                         # the prefetch that carries a scale fill per tile
    cases = [(0, good, 3, True), (0, scales, 3, True), (3, good, 3, False), (0, good[:-1], 3, False), (0, good + ["w4"], 3, False),
             (0, ["w4", "lds", "w4"], 3, False), (0, good, 2, False), (0, good, 5, False), (0, ["lds", "w4", "g"], 3, False),
             (0, ["lds"] + good, 3, False),                # one scale fill for two tiles
             (0, good[:1], 0, True)]                       # a step that waits for everything may issue anything
    for i, (pw, loads, sw, ok) in enumerate(cases):
        p = tmp_path / ("k%d.s" % i)
        p.write_text(_fake_gemm_isa(pw, loads, sw))
        if ok:
            assert Bd.check_gemm_isa(str(p)) == 1
        else:
            with pytest.raises(RuntimeError):
                Bd.check_gemm_isa(str(p))
    with pytest.raises(RuntimeError):
        Bd.check_resource_usage("remark: Function Name: _ZN2ps14gemm_w4_kernelILi0EEE\nremark:     ScratchSize [bytes/lane]: 8 [-R]\n")
    gather = "remark: Function Name: _ZN2ps17h2d_gather_kernelEPKNS_8CopyDescEj\nremark:     LDS Size [bytes/block]: %d [-R]\n"
    clean = "remark: Function Name: _ZN2ps14gemm_w4_kernelILi0EEE\nremark:     ScratchSize [bytes/lane]: 0 [-R]\n"
    Bd.check_resource_usage(clean + gather % 163840)
    for lds in (3072, 65536):       # the gather kernel no longer holds its CU's whole LDS
        with pytest.raises(RuntimeError):
            Bd.check_resource_usage(clean + gather % lds)
    with pytest.raises(RuntimeError):
        Bd.check_resource_usage(clean)
