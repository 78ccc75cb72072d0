"""The CPU back-end's matrix kernel (shards that a plan leaves in system memory and runs on the
CPU; Section 3, Plans Two and Three) against the oracle, on the host.  Same tolerance as the GPU
path: max|err| / max|ref| <= 5e-3 against the oracle that rounds the stored fp16 result."""
import ctypes as C

import numpy as np
import pytest

import synth_inputs as S
from oracle import oracle as O
from paper_2604_26334_amd import binding as B

TOL = 5e-3


def _cpu(packed, rows, K, mode, x, eps, res, threads):
    M = x.shape[0]
    out = np.zeros((M, rows // 2 if mode == 2 else rows), dtype=np.float16)
    x = np.ascontiguousarray(x, dtype=np.float16)
    r = None if res is None else np.ascontiguousarray(res, dtype=np.float16)
    rc = B.lib().ps_cpu_matmul(packed.ctypes.data, rows, K, mode, x.ctypes.data, M, eps,
                               None if r is None else r.ctypes.data, out.ctypes.data, threads)
    if rc == B.PS_E_STATE:
        pytest.skip("no AVX-512 on this host")
    assert rc == B.PS_OK, B.lib().ps_last_error()
    return out


def _rel(got, ref):
    return float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())


@pytest.mark.parametrize("rows,K,M,threads", [(16, 128, 1, 1), (48, 640, 1, 3), (256, 4096, 1, 8), (208, 1408, 5, 4),
                                               (64, 2176, 7, 2), (32, 1024, 64, 8)])
def test_cpu_matmul_plain_and_residual_match_the_oracle(rows, K, M, threads):
    sc, cd = S.weight_matrix(90, 0, 0, None, rows, K)
    packed = B.pack_matrix(sc, cd)
    x = S.activations(91, rows + M, M, K)
    eps = 1e-6
    ref = O.linear(O.rmsnorm(x, eps), sc, cd)
    got = _cpu(packed, rows, K, 0, x, eps, None, threads)
    assert _rel(got, ref) <= TOL
    res = S.activations(92, 1, M, rows)
    ref = O.linear(x, sc, cd) + res.astype(np.float64)
    assert _rel(_cpu(packed, rows, K, 1, x, eps, res, threads), ref) <= TOL
    ref = O.linear(x, sc, cd)
    assert _rel(_cpu(packed, rows, K, 1, x, eps, None, threads), ref) <= TOL
    # any thread count, same bits: a row is summed by one thread in a fixed order
    np.testing.assert_array_equal(got.view(np.uint16), _cpu(packed, rows, K, 0, x, eps, None, 1).view(np.uint16))


@pytest.mark.parametrize("I,K,M", [(16, 128, 1), (176, 512, 1), (96, 1024, 3)])
def test_cpu_matmul_gate_up_swiglu_matches_the_oracle(I, K, M):
    gs, gc = S.weight_matrix(93, 0, S.MAT_GATE, None, I, K)
    us, uc = S.weight_matrix(93, 0, S.MAT_UP, None, I, K)
    # gate and up row-tiles alternate in the packed image
    sc = np.empty((2 * I, K // 32), dtype=np.float16)
    cd = np.empty((2 * I, K), dtype=np.uint8)
    for t in range(I // 16):
        sc[32 * t:32 * t + 16], sc[32 * t + 16:32 * t + 32] = gs[16 * t:16 * t + 16], us[16 * t:16 * t + 16]
        cd[32 * t:32 * t + 16], cd[32 * t + 16:32 * t + 32] = gc[16 * t:16 * t + 16], uc[16 * t:16 * t + 16]
    packed = B.pack_matrix(sc, cd)
    x = S.activations(94, I, M, K)
    eps = 1e-6
    n = O.rmsnorm(x, eps)
    ref = O.swiglu(O.linear(n, gs, gc), O.linear(n, us, uc))
    assert _rel(_cpu(packed, 2 * I, K, 2, x, eps, None, 4), ref) <= TOL


def test_cpu_matmul_argument_checks():
    L = B.lib()
    buf = np.zeros(1 << 16, dtype=np.uint8)
    p = buf.ctypes.data
    assert L.ps_cpu_matmul(p, 24, 128, 0, p, 1, 1e-6, None, p, 1) == B.PS_E_ARG      # rows not a multiple of 16
    assert L.ps_cpu_matmul(p, 16, 96, 0, p, 1, 1e-6, None, p, 1) == B.PS_E_ARG       # K not a multiple of 128
    assert L.ps_cpu_matmul(p, 16, 128, 3, p, 1, 1e-6, None, p, 1) == B.PS_E_ARG
    assert L.ps_cpu_matmul(p, 16, 128, 2, p, 1, 1e-6, None, p, 1) == B.PS_E_ARG      # gate/up needs tile pairs
    assert L.ps_cpu_matmul(p, 16, 128, 0, p, 0, 1e-6, None, p, 1) == B.PS_E_ARG
    assert L.ps_cpu_matmul(p, 16, 128, 0, p, 1, 1e-6, None, p, 0) == B.PS_E_ARG
    assert L.ps_cpu_matmul(None, 16, 128, 0, p, 1, 1e-6, None, p, 1) == B.PS_E_ARG


@pytest.mark.parametrize("rows,K", [(48, 1024), (32, 2048), (32, 4096)])
def test_one_token_forms_agree_bit_for_bit(rows, K):
    """One token takes a single pass over a tile when rows are short (K <= 2048) and the four-pass
    form otherwise; a token's result must not depend on which form computed it, nor on whether it
    was computed alone or as one of two tokens (per row the blocks are added in one fixed order)."""
    sc, cd = S.weight_matrix(95, 0, 0, None, rows, K)
    packed = B.pack_matrix(sc, cd)
    x = S.activations(96, 3, 2, K)
    both = _cpu(packed, rows, K, 1, x, 1e-6, None, 2)
    for t in range(2):
        alone = _cpu(packed, rows, K, 1, x[t:t + 1], 1e-6, None, 3)
        np.testing.assert_array_equal(alone.view(np.uint16)[0], both.view(np.uint16)[t])
