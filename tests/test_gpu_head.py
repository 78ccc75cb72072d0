"""GPU parity of the output head (final RMSNorm + projection to the vocabulary, the "outputs"
class of the priority list in Section 3's planning phase) through the C ABI against the CPU oracle.

Two comparisons per case: end to end (oracle stack, then oracle head) and the head alone (oracle
head applied to the hidden state the GPU produced), both at max|err| / max|ref| <= 5e-3; logits are
bit-identical across shard placements."""
import numpy as np
import pytest

import synth_inputs as S
from tests import harness as Hn
from oracle import oracle as O

pytestmark = pytest.mark.gpu
TOL = 5e-3


def _say(*a):
    print(*a, flush=True)


def _load_all(st, cfg, W, head):
    for layer in range(cfg["n_layers"]):
        for kind, expert, N, K in S.matrix_shapes(cfg):
            st.load_matrix(layer, kind, expert, *W(layer, kind, expert))
    st.load_matrix(cfg["n_layers"], S.MAT_OUT, None, *head)


def _budgets(cfg, M, fracs):
    from paper_2604_26334_amd import binding as B
    s = B.Plan(cfg, 1 << 62, M).summary()
    return [int(s.weight_bytes * f) + s.workspace_bytes + 4096 for f in fracs]


def _run(cfg, W, head, budget, x, lg, requests, mode=0):
    """One stack; for every (first_token, rows) request one forward -> (x_out, logits or None)."""
    import torch
    from paper_2604_26334_amd import binding as B
    M, V = x.shape[0], cfg["vocab"]
    plan = B.Plan(cfg, int(budget), M)
    st = B.Stack(plan)
    st.set_decode_mode(mode)
    _load_all(st, cfg, W, head)
    kinds = {}
    for s in plan.shards():
        if s.kind == B.PS_SHARD_OUT:
            kinds[bool(s.resident)] = kinds.get(bool(s.resident), 0) + s.ntiles
    xin = torch.from_numpy(np.ascontiguousarray(x)).to(st.device)
    res = []
    for first, rows in requests:
        xout = torch.empty_like(xin)
        logits = torch.full((max(rows, 1), V), 7.0, dtype=torch.float16, device=st.device)
        torch.cuda.synchronize()
        st.set_logits_out(logits if rows else None, first, rows)
        st.forward(xin, xout, lg)
        st.synchronize()
        res.append((xout.cpu().numpy(), logits.cpu().numpy()))
    st.close()
    plan.close()
    return res, kinds


@pytest.mark.parametrize("case", ["dense-1", "dense-16", "dense-80", "dense-600", "moe-4"])
def test_output_head_logits_match_the_oracle(case):
    from paper_2604_26334_amd import binding as B
    fam, M = case.split("-")
    M = int(M)
    if fam == "dense":
        cfg = dict(Hn.small_dense_cfg(2), vocab=1040)     # 65 row tiles: ragged against 8-tile workgroups
        lg = None
    else:
        cfg = dict(Hn.small_moe_cfg(2), vocab=1040)
        lg = S.router_logits(5, 0, cfg["n_layers"], M, cfg["n_experts"])
    seed = 40 + M
    W = Hn.WeightCache(cfg, seed)
    head = S.head_matrix(seed, cfg)
    x = S.activations(seed, 0, M, cfg["hidden"])
    ref_x = O.stack_forward(x, cfg, W, logits=lg, mirror=True)
    ref_l = O.output_head(ref_x, cfg, head, mirror=True)
    pure_x = O.stack_forward(x, cfg, W, logits=lg, mirror=False)         # the plain fp64 definition
    pure_l = O.output_head(pure_x, cfg, head, mirror=False)
    requests = [(0, M), (M - 1, 1), (M // 2, 1), (0, 0)] if M > 1 else [(0, 1), (0, 0)]
    first = None
    ran = 0
    for budget in _budgets(cfg, M, [1.0, 0.8, 0.4, 0.15]):
        try:
            res, kinds = _run(cfg, W, head, budget, x, lg, requests)
        except B.PshardError as e:      # many tokens: the workspace alone can exceed the smallest budgets
            assert e.code == B.PS_E_BUDGET
            continue
        ran += 1
        _say("  %s budget %d head tiles pinned %d streamed %d" % (case, budget, kinds.get(True, 0), kinds.get(False, 0)))
        for (tok, rows), (xo, lo) in zip(requests, res):
            assert Hn.rel_err(xo, ref_x) <= TOL and Hn.rel_err(xo, pure_x) <= TOL
            if rows == 0:
                assert (lo == np.float16(7.0)).all()      # the head was left out
                continue
            assert np.isfinite(lo.astype(np.float64)).all()
            want = ref_l[tok:tok + rows]
            alone = O.output_head(xo[tok:tok + rows], cfg, head, mirror=True)
            e2e, e1 = Hn.rel_err(lo, want), Hn.rel_err(lo, alone)
            _say("    tokens %d+%d  err end-to-end %.3e  head alone %.3e" % (tok, rows, e2e, e1))
            assert e2e <= TOL and e1 <= TOL, (case, budget, tok, rows, e2e, e1)
            assert Hn.rel_err(lo, pure_l[tok:tok + rows]) <= TOL
        if first is None:
            first = res
        else:
            for (xo, lo), (xo0, lo0) in zip(res, first):
                np.testing.assert_array_equal(xo.view(np.uint16), xo0.view(np.uint16))
                np.testing.assert_array_equal(lo.view(np.uint16), lo0.view(np.uint16))
    assert ran >= 3
    if M == 1:   # HIP-graph replay: same launches, same bits, also when the request changes between replays
        res, _ = _run(cfg, W, head, _budgets(cfg, 1, [1.0])[0], x, lg, [(0, 1), (0, 0), (0, 1), (0, 1)], mode=1)
        for i in (0, 2, 3):
            np.testing.assert_array_equal(res[i][1].view(np.uint16), first[0][1].view(np.uint16))
            np.testing.assert_array_equal(res[i][0].view(np.uint16), first[0][0].view(np.uint16))
        assert (res[1][1] == np.float16(7.0)).all()


def test_chunked_prefill_gives_the_last_tokens_logits():
    """45 tokens through a 16-token stack: three trips, the head runs on the third only, on its row 12."""
    import torch
    from paper_2604_26334_amd import binding as B
    cfg = dict(Hn.small_dense_cfg(2), vocab=2064)
    W = Hn.WeightCache(cfg, 71)
    head = S.head_matrix(71, cfg)
    n = 45
    x = S.activations(71, 0, n, cfg["hidden"])
    ref_x = O.stack_forward(x, cfg, W, mirror=True)
    ref_l = O.output_head(ref_x[n - 1:], cfg, head, mirror=True)[0]
    for frac in (1.0, 0.3):
        plan = B.Plan(cfg, _budgets(cfg, 16, [frac])[0], 16)
        st = B.Stack(plan)
        _load_all(st, cfg, W, head)
        xin = torch.from_numpy(x).to(st.device)
        xout = torch.empty_like(xin)
        logits = torch.zeros(cfg["vocab"], dtype=torch.float16, device=st.device)
        torch.cuda.synchronize()
        trips = B.chunked_forward(st, xin, xout, logits_out=logits)
        st.synchronize()
        torch.cuda.synchronize()
        assert trips == 3
        streamed = st.stats().streamed_bytes_step
        e_x, e_l = Hn.rel_err(xout.cpu().numpy(), ref_x), Hn.rel_err(logits.cpu().numpy(), ref_l)
        _say("  frac %.1f  streamed/step %d  err x %.3e logits %.3e" % (frac, streamed, e_x, e_l))
        assert e_x <= TOL and e_l <= TOL
        assert int(np.argmax(logits.cpu().numpy().astype(np.float64))) == int(np.argmax(ref_l)) or \
            np.sort(ref_l)[-1] - np.sort(ref_l)[-2] < 2 * TOL * np.abs(ref_l).max()
        st.close()
        plan.close()


def test_output_head_error_paths():
    import torch
    from paper_2604_26334_amd import binding as B
    L = B.lib()
    cfg = dict(Hn.small_dense_cfg(1), vocab=1040)
    W = Hn.WeightCache(cfg, 3)
    head = S.head_matrix(3, cfg)
    plan = B.Plan(cfg, 1 << 28, 16)
    st = B.Stack(plan)
    buf = torch.zeros((16, 1040), dtype=torch.float16, device=st.device)
    x = torch.zeros((16, cfg["hidden"]), dtype=torch.float16, device=st.device)
    y = torch.empty_like(x)
    for layer in range(cfg["n_layers"]):
        for kind, expert, N, K in S.matrix_shapes(cfg):
            st.load_matrix(layer, kind, expert, *W(layer, kind, expert))
    assert L.ps_stack_forward(st.h, x.data_ptr(), y.data_ptr(), None, None) == B.PS_E_STATE   # head not loaded yet
    sc, cd = head
    assert L.ps_stack_load_matrix(st.h, 0, B.PS_MAT_OUT, B.NO_EXPERT, sc.ctypes.data, cd.ctypes.data) == B.PS_E_ARG
    assert L.ps_stack_load_matrix(st.h, 1, B.PS_MAT_OUT, 0, sc.ctypes.data, cd.ctypes.data) == B.PS_E_ARG
    st.load_matrix(1, B.PS_MAT_OUT, None, sc, cd)
    assert L.ps_stack_set_logits_out(st.h, buf.data_ptr(), 0, 2) == B.PS_E_ARG      # neither 0, 1 nor 16 rows
    assert L.ps_stack_set_logits_out(st.h, buf.data_ptr(), 16, 1) == B.PS_E_ARG     # token out of range
    assert L.ps_stack_set_logits_out(st.h, buf.data_ptr(), 1, 16) == B.PS_E_ARG
    assert L.ps_stack_set_logits_out(st.h, None, 0, 1) == B.PS_E_ARG
    assert L.ps_stack_set_logits_out(st.h, buf.data_ptr() + 2, 0, 1) == B.PS_E_ARG  # misaligned
    assert L.ps_stack_set_logits_out(st.h, None, 0, 0) == B.PS_OK
    st.set_logits_out(buf, 0, 16)
    st.forward(x, y)
    st.synchronize()
    assert (buf.cpu().numpy() == 0).all()      # zero hidden state -> zero logits, and the stack still runs
    st.close()
    plan.close()
    nohead = B.Plan(Hn.small_dense_cfg(1), 1 << 28, 1)
    st2 = B.Stack(nohead)
    assert L.ps_stack_set_logits_out(st2.h, buf.data_ptr(), 0, 1) == B.PS_E_STATE
    assert L.ps_stack_load_matrix(st2.h, 1, B.PS_MAT_OUT, B.NO_EXPERT, sc.ctypes.data, cd.ctypes.data) == B.PS_E_ARG
    st2.close()
    nohead.close()
