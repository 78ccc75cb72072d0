"""ps_stack_forward_noalloc (the forward whose workspace is the library's static device array) against
ps_stack_forward, through the C ABI: bit-identical outputs and oracle parity on two calls in a row,
the second with a smaller input; oversize and unsupported stacks are refused with an error code."""
import ctypes as C

import numpy as np
import pytest

import synth_inputs as S
from oracle import oracle as O
from tests import harness as Hn

pytestmark = pytest.mark.gpu
TOL = 5e-3


def _stack(B, cfg, W, M, frac):
    full = B.Plan(cfg, 1 << 40, M).summary()
    plan = B.Plan(cfg, full.workspace_bytes + int(full.weight_bytes * frac) + (1 << 16), M)
    st = B.Stack(plan)
    for layer in range(cfg["n_layers"]):
        for kind, expert, N, K in S.matrix_shapes(cfg):
            st.load_matrix(layer, kind, expert, *W(layer, kind, expert))
    return plan, st


def test_noalloc_forward_matches_the_arena_forward_twice_in_a_row():
    import torch
    from paper_2604_26334_amd import binding as B
    cfg = Hn.small_dense_cfg(3)
    W = Hn.WeightCache(cfg, 31)
    # first call: 37 tokens (split-K planes, RMS factors, all activation buffers in the static array),
    # part of the FFN streamed; second call, right behind it: one token, all resident; third: 5 tokens
    for M, frac in ((37, 0.5), (1, 1.0), (5, 1.0)):
        plan, st = _stack(B, cfg, W, M, frac)
        x = S.activations(31, M, M, cfg["hidden"])
        ref = O.stack_forward(x, cfg, W, mirror=True)
        xin = torch.from_numpy(x).to(st.device)
        y_arena, y_static = torch.zeros_like(xin), torch.zeros_like(xin)
        print("case: %d tokens, budget fraction %.1f, workspace %d B" % (M, frac, plan.summary().workspace_bytes), flush=True)
        st.forward(xin, y_arena)
        st.synchronize()
        st.forward_noalloc(xin, y_static)
        st.synchronize()
        a, s = y_arena.cpu().numpy(), y_static.cpu().numpy()
        np.testing.assert_array_equal(s.view(np.uint16), a.view(np.uint16))
        assert np.isfinite(s.astype(np.float64)).all() and Hn.rel_err(s, ref) <= TOL
        # and once more: the array keeps the previous call's contents, nothing may depend on them
        y_static.zero_()
        st.forward_noalloc(xin, y_static)
        st.synchronize()
        np.testing.assert_array_equal(y_static.cpu().numpy().view(np.uint16), a.view(np.uint16))
        st.close()
        plan.close()


def test_noalloc_forward_with_the_few_token_kernel():
    """Four tokens through matrices of whole scale groups (the few-token form of the decode kernel: no RMS-factor
    buffer, no partial planes; its activations in the static array), then three: same bits as the arena forward."""
    import torch
    from paper_2604_26334_amd import binding as B
    cfg = dict(Hn.small_dense_cfg(2), hidden=1024, n_q_heads=8, n_kv_heads=2, ffn_inter=2048)
    W = Hn.WeightCache(cfg, 34)
    for M, frac in ((4, 0.6), (3, 1.0)):
        plan, st = _stack(B, cfg, W, M, frac)
        x = S.activations(34, M, M, cfg["hidden"])
        ref = O.stack_forward(x, cfg, W, mirror=True)
        xin = torch.from_numpy(x).to(st.device)
        y_arena, y_static = torch.zeros_like(xin), torch.zeros_like(xin)
        st.forward(xin, y_arena)
        st.synchronize()
        for rep in range(2):
            y_static.zero_()
            st.forward_noalloc(xin, y_static)
            st.synchronize()
            np.testing.assert_array_equal(y_static.cpu().numpy().view(np.uint16), y_arena.cpu().numpy().view(np.uint16))
        assert Hn.rel_err(y_static.cpu().numpy(), ref) <= TOL
        st.close()
        plan.close()


def test_noalloc_forward_refuses_what_it_cannot_hold():
    import torch
    from paper_2604_26334_amd import binding as B
    L = B.lib()
    cfg = Hn.small_dense_cfg(1)
    W = Hn.WeightCache(cfg, 32)
    plan, st = _stack(B, cfg, W, 16384, 1.0)          # workspace of 16384 tokens: far beyond 32 MiB
    assert plan.summary().workspace_bytes > (32 << 20)
    x = torch.zeros((16384, cfg["hidden"]), dtype=torch.float16, device=st.device)
    y = torch.empty_like(x)
    assert L.ps_stack_forward_noalloc(st.h, x.data_ptr(), y.data_ptr()) == B.PS_E_ARG
    assert b"static scratch" in L.ps_last_error()
    st.close()
    plan.close()
    mcfg = Hn.small_moe_cfg(1)
    mplan, mst = _stack(B, mcfg, Hn.WeightCache(mcfg, 33), 1, 1.0)
    xm = torch.zeros((1, mcfg["hidden"]), dtype=torch.float16, device=mst.device)
    assert L.ps_stack_forward_noalloc(mst.h, xm.data_ptr(), torch.empty_like(xm).data_ptr()) == B.PS_E_STATE
    mst.close()
    mplan.close()
