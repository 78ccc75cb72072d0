"""Pins for the CPU oracle: each oracle function is checked against something
other than itself -- pure-Python brute force on tiny shapes, closed forms,
numpy's independent fp16 conversion, and textbook special cases.  A dropped
term, a wrong sign/index or a transposed operand fails at least one of them.
(The paper prints no numeric tensor example, so there is no printed-value pin.)
"""
import math
import os

import numpy as np
import pytest

import synth_inputs as S
from oracle import oracle as O


# ---------------------------------------------------------------- fp16 helpers

def test_half_to_double_all_bit_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    for b in range(0, 65536, 7):  # every 7th pattern plus the specials below
        v = O.half_to_double(b)
        r = ref[b]
        assert (math.isnan(v) and math.isnan(r)) or v == r, b
    for b in (0, 1, 0x3FF, 0x400, 0x7BFF, 0x7C00, 0x8000, 0x8001, 0xFBFF, 0xFC00, 0x3C00, 0xBC00):
        assert O.half_to_double(b) == ref[b]


def test_round_f16_matches_numpy_and_ties_to_even():
    rng = np.random.default_rng(1)
    xs = np.concatenate([rng.standard_normal(2000) * s for s in (1e-7, 1e-4, 1.0, 300.0, 40000.0)])
    for x in xs:
        assert O.round_f16(x) == float(np.float64(x).astype(np.float16)), x
    # exact ties: 2049 is halfway between 2048 and 2050 -> even mantissa (2048); 2051 -> 2052
    assert O.round_f16(2049.0) == 2048.0
    assert O.round_f16(2051.0) == 2052.0
    assert O.round_f16(-2049.0) == -2048.0
    assert O.round_f16(65519.9) == 65504.0 and math.isinf(O.round_f16(65520.0))
    assert O.round_f16(2.0 ** -25) == 0.0 and O.round_f16(2.0 ** -25 * 1.0001) == 2.0 ** -24


# ---------------------------------------------------------------- dequant

def test_dequant_closed_form_all_codes():
    for d in (1.0, 0.5, 0.0234375, 2.0 ** -14, 0.0):
        scales = np.full((1, 1), d, dtype=np.float16)
        codes = (np.arange(32, dtype=np.uint8) % 16).reshape(1, 32)
        W = O.dequant(scales, codes)
        for k in range(32):
            assert W[0, k] == float(np.float16(d)) * ((k % 16) - 8)


def test_dequant_block_indexing():
    # scale varies per (row, block): W[n][k] must pick scales[n][k // 32]
    N, K = 3, 96
    scales = (np.arange(N * 3, dtype=np.float32).reshape(N, 3) + 1).astype(np.float16)
    codes = np.full((N, K), 9, dtype=np.uint8)
    W = O.dequant(scales, codes)
    for n in range(N):
        for k in range(K):
            assert W[n, k] == float(scales[n, k // 32])


# ---------------------------------------------------------------- linear

def _py_linear(X, scales, codes):
    """Pure-Python brute force of Y[m][n] = sum_k X[m][k] * d[n][k//32] * (q[n][k] - 8)."""
    M, K = len(X), len(X[0])
    N = len(codes)
    Y = [[0.0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += float(X[m][k]) * (float(scales[n][k // 32]) * (int(codes[n][k]) - 8))
            Y[m][n] = acc
    return Y


@pytest.mark.parametrize("M,N,K", [(1, 5, 32), (3, 7, 64), (2, 33, 96)])
def test_linear_vs_pure_python_bruteforce(M, N, K):
    s, c = S.weight_matrix(11, 0, S.MAT_QKV, None, N, K)
    X = S.activations(11, 0, M, K).astype(np.float64)
    Y = O.linear(X, s, c)
    ref = np.array(_py_linear(X.tolist(), s.astype(np.float64).tolist(), c.tolist()))
    assert Y.shape == (M, N)
    np.testing.assert_allclose(Y, ref, rtol=1e-13, atol=1e-13)


def test_linear_one_hot_identity_zero_and_constant():
    K = 64
    X = S.activations(3, 0, 2, K).astype(np.float64)
    ones = np.ones((K, K // 32), dtype=np.float16)
    # identity: q=9 on the diagonal, q=8 elsewhere, d=1 -> Y = X
    c = np.full((K, K), 8, dtype=np.uint8)
    c[np.arange(K), np.arange(K)] = 9
    np.testing.assert_array_equal(O.linear(X, ones, c), X)
    # one-hot rows at a non-symmetric position: row n picks X[:, (5 n + 3) % K]
    c = np.full((K, K), 8, dtype=np.uint8)
    pick = (5 * np.arange(K) + 3) % K
    c[np.arange(K), pick] = 9
    np.testing.assert_array_equal(O.linear(X, ones, c), X[:, pick])
    # all q=8 -> 0
    np.testing.assert_array_equal(O.linear(X, ones, np.full((K, K), 8, dtype=np.uint8)), np.zeros((2, K)))
    # all q=9, d=c -> c * sum(X); q=7 flips the sign
    cst = np.full((4, K // 32), 0.25, dtype=np.float16)
    Y = O.linear(X, cst, np.full((4, K), 9, dtype=np.uint8))
    np.testing.assert_allclose(Y, np.repeat(0.25 * X.sum(1, keepdims=True), 4, 1), rtol=1e-14)
    Y = O.linear(X, cst, np.full((4, K), 7, dtype=np.uint8))
    np.testing.assert_allclose(Y, np.repeat(-0.25 * X.sum(1, keepdims=True), 4, 1), rtol=1e-14)


def test_linear_matches_numpy_matmul_of_independent_dequant():
    N, K, M = 48, 256, 5
    s, c = S.weight_matrix(5, 1, S.MAT_DOWN, None, N, K)
    X = S.activations(5, 1, M, K).astype(np.float64)
    W = np.repeat(s.astype(np.float64), 32, axis=1) * (c.astype(np.float64) - 8.0)
    np.testing.assert_allclose(O.linear(X, s, c), X @ W.T, rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(O.dequant(s, c), W)


def test_generator_statistics_band():
    # sanity band for the generator: E[q-8] = -0.5, E[(q-8)^2] = 21.5, E[d^2] = 4e-4
    s, c = S.weight_matrix(0, 0, S.MAT_GATE, None, 512, 1024)
    q = c.astype(np.float64) - 8
    assert abs(q.mean() + 0.5) < 0.05 and abs((q * q).mean() - 21.5) < 0.2
    assert abs((s.astype(np.float64) ** 2).mean() - 4e-4) < 2e-5
    assert c.min() == 0 and c.max() == 15


# ---------------------------------------------------------------- norm / swiglu

def test_rmsnorm_closed_forms():
    eps = 1e-6
    for cval in (0.5, -3.0, 100.0):
        y = O.rmsnorm(np.full((2, 64), cval), eps)
        np.testing.assert_allclose(y, cval / math.sqrt(cval * cval + eps), rtol=1e-15)
    x = S.activations(2, 0, 3, 128).astype(np.float64)
    y = O.rmsnorm(x, eps)
    ms = (x * x).mean(1)
    np.testing.assert_allclose((y * y).mean(1), ms / (ms + eps), rtol=1e-13)
    # direction preserved, rows independent
    np.testing.assert_allclose(y[1] * math.sqrt(ms[1] + eps), x[1], rtol=1e-13)


def test_swiglu_closed_forms():
    g = np.array([0.0, 40.0, -40.0, 1.5, -1.5, 0.3])
    u = np.array([2.0, 1.0, 1.0, -2.0, 1.0, 7.0])
    s = O.swiglu(g, u)
    assert s[0] == 0.0
    assert abs(s[1] - 40.0) < 1e-12 and abs(s[2]) < 1e-14
    for i in range(len(g)):
        assert abs(s[i] - g[i] / (1.0 + math.exp(-g[i])) * u[i]) < 1e-15
    # silu(-x) = silu(x) - x
    x = np.linspace(-6, 6, 25)
    one = np.ones_like(x)
    np.testing.assert_allclose(O.swiglu(-x, one), O.swiglu(x, one) - x, atol=1e-14)
    # gate and up are not interchangeable
    assert O.swiglu(np.array([1.0]), np.array([3.0]))[0] != O.swiglu(np.array([3.0]), np.array([1.0]))[0]


# ---------------------------------------------------------------- attention stand-in

def test_identity_v_equals_softmax_attention_with_one_key():
    n_q, n_kv, hd, M = 8, 2, 16, 3
    rng = np.random.default_rng(4)
    qkv = rng.standard_normal((M, (n_q + 2 * n_kv) * hd))
    A = O.attn_identity_v(qkv, n_q, n_kv, hd)
    # textbook grouped-query attention with context length 1 (each token attends to itself only)
    q = qkv[:, : n_q * hd].reshape(M, n_q, hd)
    k = qkv[:, n_q * hd:(n_q + n_kv) * hd].reshape(M, n_kv, hd)
    v = qkv[:, (n_q + n_kv) * hd:].reshape(M, n_kv, hd)
    ref = np.empty((M, n_q, hd))
    for m in range(M):
        for h in range(n_q):
            kvh = h // (n_q // n_kv)
            score = np.array([q[m, h] @ k[m, kvh] / math.sqrt(hd)])
            p = np.exp(score - score.max())
            p /= p.sum()
            ref[m, h] = p[0] * v[m, kvh]
    np.testing.assert_array_equal(A, ref.reshape(M, n_q * hd))


# ---------------------------------------------------------------- routing

def test_route_topk_vs_sort_bruteforce_and_invariants():
    lg = S.router_logits(9, 0, 1, 6, 128)[0]
    idx, w = O.route_topk(lg, 8)
    for m in range(6):
        order = sorted(range(128), key=lambda e: (-float(lg[m, e]), e))[:8]
        assert list(idx[m]) == order
        ex = [math.exp(float(lg[m, e]) - float(lg[m, order[0]])) for e in order]
        np.testing.assert_allclose(w[m], np.array(ex) / sum(ex), rtol=1e-14)
        # equals the full softmax renormalised over the selection
        full = np.exp(lg[m].astype(np.float64) - lg[m].max())
        full /= full.sum()
        np.testing.assert_allclose(w[m], full[order] / full[order].sum(), rtol=1e-12)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=1e-14)
    idx2, w2 = O.route_topk(lg + np.float32(4.0), 8)   # exact shift in fp32 for these magnitudes? compare loosely
    np.testing.assert_array_equal(idx2[:, :1], idx[:, :1])
    # equal logits -> 1/8 each and the lowest indices win
    idx3, w3 = O.route_topk(np.zeros((1, 128), dtype=np.float32), 8)
    assert list(idx3[0]) == list(range(8))
    np.testing.assert_allclose(w3, 1.0 / 8)
    # ties inside the selection boundary go to the lower index
    t = np.zeros((1, 16), dtype=np.float32)
    t[0, [3, 9, 12]] = 1.0
    t[0, 5] = 2.0
    idx4, _ = O.route_topk(t, 4)
    assert list(idx4[0]) == [5, 3, 9, 12]


# ---------------------------------------------------------------- layer composition

def _numpy_dequant(sc):
    s, c = sc
    return np.repeat(s.astype(np.float64), 32, axis=1) * (c.astype(np.float64) - 8.0)


def _tiny_dense_cfg():
    return dict(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn_inter=96,
                n_experts=0, top_k=0, expert_inter=0, rms_eps=1e-6, no_attn=False, no_residual=False)


def _weights(seed, cfg):
    shapes = {(k, e): (N, K) for (k, e, N, K) in S.matrix_shapes(cfg)}

    def get(layer, kind, expert):
        N, K = shapes[(kind, expert)]
        return S.weight_matrix(seed, layer, kind, expert, N, K)
    return get


def test_dense_stack_pure_matches_numpy_composition():
    cfg = _tiny_dense_cfg()
    W = _weights(21, cfg)
    x0 = S.activations(21, 0, 3, cfg["hidden"]).astype(np.float64)
    got = O.stack_forward(x0, cfg, W, mirror=False)
    x = x0
    eps = cfg["rms_eps"]
    for l in range(cfg["n_layers"]):
        n = x / np.sqrt((x * x).mean(1, keepdims=True) + eps)
        qkv = n @ _numpy_dequant(W(l, S.MAT_QKV, None)).T
        v = qkv[:, (4 + 2) * 32:].reshape(3, 2, 32)
        A = np.repeat(v, 2, axis=1).reshape(3, 4 * 32)        # q head h reads kv head h // 2
        h = x + A @ _numpy_dequant(W(l, S.MAT_O, None)).T
        n2 = h / np.sqrt((h * h).mean(1, keepdims=True) + eps)
        g = n2 @ _numpy_dequant(W(l, S.MAT_GATE, None)).T
        u = n2 @ _numpy_dequant(W(l, S.MAT_UP, None)).T
        s = g / (1 + np.exp(-g)) * u
        x = h + s @ _numpy_dequant(W(l, S.MAT_DOWN, None)).T
    np.testing.assert_allclose(got, x, rtol=1e-10, atol=1e-10)


def test_ffn_block_config_has_no_residual():
    cfg = dict(S.cfg_ffn_block(), hidden=64, ffn_inter=96)
    W = _weights(22, cfg)
    x = S.activations(22, 0, 1, 64).astype(np.float64)
    got = O.stack_forward(x, cfg, W, mirror=False)
    n = x / np.sqrt((x * x).mean(1, keepdims=True) + 1e-6)
    g = n @ _numpy_dequant(W(0, S.MAT_GATE, None)).T
    u = n @ _numpy_dequant(W(0, S.MAT_UP, None)).T
    ref = (g / (1 + np.exp(-g)) * u) @ _numpy_dequant(W(0, S.MAT_DOWN, None)).T
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_mirror_mode_rounds_only_to_fp16_grid_and_stays_close():
    cfg = _tiny_dense_cfg()
    W = _weights(23, cfg)
    x0 = S.activations(23, 0, 2, cfg["hidden"])
    pure = O.stack_forward(x0, cfg, W, mirror=False)
    mir = O.stack_forward(x0, cfg, W, mirror=True)
    np.testing.assert_array_equal(mir, mir.astype(np.float16).astype(np.float64))
    assert np.abs(mir - pure).max() / np.abs(pure).max() < 5e-3
    assert np.abs(mir - pure).max() > 0


def _r16(v):
    return v.astype(np.float16).astype(np.float64)


def _mirror_rebuild(x, cfg, W, logits=None, drop=None):
    """The stack with an explicit fp16 store at each point where the device path stores fp16 (after the
    QKV projection, after O + residual, after SwiGLU, after down + residual or the expert combine) and
    nowhere else; the point named by `drop` is left unrounded.  Every arithmetic step is one of the
    separately pinned pieces, called in the order of the definition."""
    r = lambda name, v: v if name == drop else _r16(v)
    eps, H = cfg["rms_eps"], cfg["hidden"]
    x = np.asarray(x, dtype=np.float64)
    for l in range(cfg["n_layers"]):
        qkv = r("qkv", O.linear(O.rmsnorm(x, eps), *W(l, S.MAT_QKV, None)))
        A = O.attn_identity_v(qkv, cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"])
        h = r("h", O.linear(A, *W(l, S.MAT_O, None)) + x)
        n = O.rmsnorm(h, eps)
        if cfg["n_experts"] == 0:
            s = r("s", O.swiglu(O.linear(n, *W(l, S.MAT_GATE, None)), O.linear(n, *W(l, S.MAT_UP, None))))
            x = r("out", O.linear(s, *W(l, S.MAT_DOWN, None)) + h)
            continue
        idx, w = O.route_topk(logits[l], cfg["top_k"])
        out = np.zeros_like(h)
        for m in range(h.shape[0]):
            for j in range(cfg["top_k"]):
                e = int(idx[m, j])
                s = r("s", O.swiglu(O.linear(n[m:m + 1], *W(l, S.MAT_GATE, e)), O.linear(n[m:m + 1], *W(l, S.MAT_UP, e))))
                out[m] += w[m, j] * O.linear(s, *W(l, S.MAT_DOWN, e))[0]      # expert outputs are not rounded
            out[m] += h[m]
        x = r("out", out)
    return x


@pytest.mark.parametrize("kind", ["dense", "moe"])
def test_mirror_mode_rounds_at_exactly_the_documented_points(kind):
    """Mirror mode = fp16 stores after QKV, after O + residual, after SwiGLU and after down + residual /
    the expert combine.  The rebuild with numpy's own fp16 conversion at those points must equal the
    oracle bit for bit, and leaving any single point out must change the result: so a rounding that the
    oracle dropped, moved or added would fail here."""
    if kind == "dense":
        cfg, lg = dict(_tiny_dense_cfg(), n_layers=2), None
    else:
        cfg = dict(_tiny_moe_cfg(), n_layers=1)
        lg = S.router_logits(24, 0, 1, 3, cfg["n_experts"])
    W = _weights(24, cfg)
    x0 = S.activations(24, 0, 3, cfg["hidden"])
    mir = O.stack_forward(x0, cfg, W, logits=lg, mirror=True)
    np.testing.assert_array_equal(mir, _mirror_rebuild(x0, cfg, W, lg))
    for point in ("qkv", "h", "s", "out"):
        other = _mirror_rebuild(x0, cfg, W, lg, drop=point)
        assert np.any(other != mir), "dropping the fp16 store after %r changes nothing" % point
    # and pure mode rounds nowhere
    pure = O.stack_forward(x0, cfg, W, logits=lg, mirror=False)
    assert np.any(pure != _r16(pure))


def test_mirror_mode_rounding_points_of_the_cached_attention_half():
    """With a KV cache the stored tensors are the QKV row (hence the appended K and V rows), the
    attention output and O + residual."""
    cfg = dict(n_layers=1, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_inter=256, n_experts=0,
               top_k=0, expert_inter=0, rms_eps=1e-6, no_attn=False, no_residual=False)
    H, n_q, n_kv, hd = 256, 4, 2, 128
    qkv_w = S.weight_matrix(5, 0, S.MAT_QKV, None, (n_q + 2 * n_kv) * hd, H)
    o_w = S.weight_matrix(5, 0, S.MAT_O, None, H, n_q * hd)
    x = S.activations(5, 0, 1, H)
    rng = np.random.default_rng(17)
    cap, ctx = 12, 9
    Kc = rng.standard_normal((n_kv, cap, hd)).astype(np.float16)
    Vc = rng.standard_normal((n_kv, cap, hd)).astype(np.float16)
    h, kn, vn = O.attn_kv_half(x, cfg, qkv_w, o_w, Kc, Vc, ctx, True)

    def rebuild(drop=None):
        r = lambda name, v: v if name == drop else _r16(v)
        y = r("qkv", O.linear(O.rmsnorm(x, cfg["rms_eps"]), *qkv_w))[0]
        k_new, v_new = y[n_q * hd:(n_q + n_kv) * hd].reshape(n_kv, hd), y[(n_q + n_kv) * hd:].reshape(n_kv, hd)
        K = np.concatenate([Kc[:, :ctx].astype(np.float64), k_new[:, None, :]], axis=1)
        V = np.concatenate([Vc[:, :ctx].astype(np.float64), v_new[:, None, :]], axis=1)
        A = r("attn", O.attn_decode(y[:n_q * hd], K, V, n_q, n_kv, hd))
        return r("h", O.linear(A[None, :], *o_w) + x.astype(np.float64)), k_new, v_new

    h2, k2, v2 = rebuild()
    np.testing.assert_array_equal(h, h2)
    np.testing.assert_array_equal(kn, k2)
    np.testing.assert_array_equal(vn, v2)
    for point in ("qkv", "attn", "h"):
        assert np.any(rebuild(point)[0] != h), point


def _tiny_moe_cfg():
    return dict(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn_inter=0,
                n_experts=8, top_k=3, expert_inter=32, rms_eps=1e-6, no_attn=False, no_residual=False)


def test_moe_with_identical_experts_equals_dense_ffn():
    cfg = _tiny_moe_cfg()
    H, I = cfg["hidden"], cfg["expert_inter"]
    gate = S.weight_matrix(31, 0, S.MAT_GATE, None, I, H)
    up = S.weight_matrix(31, 0, S.MAT_UP, None, I, H)
    down = S.weight_matrix(31, 0, S.MAT_DOWN, None, H, I)
    h = S.activations(31, 0, 4, H).astype(np.float64)
    lg = S.router_logits(31, 0, 1, 4, cfg["n_experts"])[0]
    experts = {e: (gate, up, down) for e in range(cfg["n_experts"])}
    moe = O.moe_ffn_half(h, cfg, lg, experts, mirror=False)
    dense_cfg = dict(cfg, ffn_inter=I, n_experts=0)
    dense = O.dense_ffn_half(h, dense_cfg, gate, up, down, mirror=False)
    np.testing.assert_allclose(moe, dense, rtol=1e-12, atol=1e-12)


def test_moe_layer_matches_python_composition():
    cfg = _tiny_moe_cfg()
    W = _weights(32, cfg)
    H, E, k = cfg["hidden"], cfg["n_experts"], cfg["top_k"]
    h = S.activations(32, 0, 3, H).astype(np.float64)
    lg = S.router_logits(32, 0, 1, 3, E)[0]
    experts = {e: (W(0, S.MAT_GATE, e), W(0, S.MAT_UP, e), W(0, S.MAT_DOWN, e)) for e in range(E)}
    got = O.moe_ffn_half(h, cfg, lg, experts, mirror=False)
    n = h / np.sqrt((h * h).mean(1, keepdims=True) + 1e-6)
    ref = h.copy()
    for m in range(3):
        order = sorted(range(E), key=lambda e: (-float(lg[m, e]), e))[:k]
        ex = np.exp(lg[m, order].astype(np.float64) - float(lg[m, order[0]]))
        w = ex / ex.sum()
        for j, e in enumerate(order):
            g = n[m] @ _numpy_dequant(experts[e][0]).T
            u = n[m] @ _numpy_dequant(experts[e][1]).T
            ref[m] += w[j] * ((g / (1 + np.exp(-g)) * u) @ _numpy_dequant(experts[e][2]).T)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-10)


# ------------------------------------------------------------------ PickTier

def _golden_pick_cases():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "pick_tier_example.txt")
    est, cases = None, []
    for ln in open(path).read().splitlines():
        f = ln.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "est":
            est = [float(v) for v in f[1:]]
        elif f[0] == "case":
            cases.append((int(f[1]), int(f[2]), int(f[3]), float(f[4])))
    return est, cases


def test_pick_tier_hand_worked_example():
    est, cases = _golden_pick_cases()
    assert len(est) == len(O.TIER_TOKENS) and len(cases) >= 6
    for tokens, want_tok, want_iters, want_ms in cases:
        t, iters, total = O.pick_tier(est, tokens)
        assert (O.TIER_TOKENS[t], iters, total) == (want_tok, want_iters, want_ms), tokens


def test_pick_tier_closed_forms_and_ties():
    J = O.TIER_TOKENS
    # the same time for every tier: only the trip count matters -> the smallest tier that holds
    # all tokens in one trip (ties go to the lowest tier); beyond the largest tier, the largest
    for n in (1, 2, 4, 5, 17, 64, 65, 513, 16384):
        t, iters, total = O.pick_tier([5.0] * len(J), n)
        assert J[t] == min(T for T in J if T >= n) and iters == 1 and total == 5.0
    t, iters, _ = O.pick_tier([5.0] * len(J), 16385)
    assert (J[t], iters) == (16384, 2)
    # time exactly proportional to the tier size: total = a * (tokens padded up to a multiple of the
    # tier) >= a * tokens, with equality for every tier that divides the token count -> tier 1
    for n in (1, 7, 64, 100, 4096):
        t, iters, total = O.pick_tier([0.25 * T for T in J], n)
        assert (J[t], iters, total) == (1, n, 0.25 * n)
    # a fixed cost per trip on top makes the lowest-padding LARGE tier win: tokens = 1024 exactly
    t, iters, total = O.pick_tier([10.0 + 0.25 * T for T in J], 1024)
    assert (J[t], iters, total) == (1024, 1, 266.0)
    # tiers without a schedule are skipped; none at all is an error
    est = [None] * len(J)
    est[3], est[6] = 1.0, 20.0
    assert O.pick_tier(est, 40)[:2] == (3, 2) and O.pick_tier(est, 4000)[:2] == (6, 4)
    with pytest.raises(ValueError):
        O.pick_tier([None] * len(J), 5)


# ------------------------------------------------------------------ decode attention over a KV cache

def test_attn_decode_closed_forms():
    rng = np.random.default_rng(11)
    n_q, n_kv, hd, T = 4, 2, 128, 9
    q = rng.standard_normal(n_q * hd)
    K = rng.standard_normal((n_kv, T, hd))
    V = rng.standard_normal((n_kv, T, hd))
    # a single position: weight 1 -> the value row of the head's kv head (the identity-on-V stand-in)
    A1 = O.attn_decode(q, K[:, :1], V[:, :1], n_q, n_kv, hd)
    qkv = np.concatenate([q, K[:, 0].reshape(-1), V[:, 0].reshape(-1)])[None, :]
    np.testing.assert_array_equal(A1, O.attn_identity_v(qkv, n_q, n_kv, hd)[0])
    # equal keys: every score equal -> uniform weights -> the mean of the values
    Ke = np.repeat(K[:, :1], T, axis=1)
    Au = O.attn_decode(q, Ke, V, n_q, n_kv, hd).reshape(n_q, hd)
    for h in range(n_q):
        np.testing.assert_allclose(Au[h], V[h // 2].mean(axis=0), rtol=0, atol=1e-12)
    # one key aligned with a huge query: its weight -> 1 (the others underflow to 0 exactly)
    qb = np.zeros((n_q, hd)); qb[:, 0] = 1e4
    Kb = np.zeros((n_kv, T, hd)); Kb[:, 5, 0] = 1.0
    Ab = O.attn_decode(qb, Kb, V, n_q, n_kv, hd).reshape(n_q, hd)
    for h in range(n_q):
        np.testing.assert_array_equal(Ab[h], V[h // 2, 5])
    # scaling by 1/sqrt(hd): with hd-dimensional unit keys e_0 and q = sqrt(hd) * ln(3) * e_0 against a zero
    # key, the weights are 3/4 and 1/4
    K2 = np.zeros((n_kv, 2, hd)); K2[:, 0, 0] = 1.0
    q2 = np.zeros((n_q, hd)); q2[:, 0] = math.sqrt(hd) * math.log(3.0)
    A2 = O.attn_decode(q2, K2, V[:, :2], n_q, n_kv, hd).reshape(n_q, hd)
    for h in range(n_q):
        np.testing.assert_allclose(A2[h], 0.75 * V[h // 2, 0] + 0.25 * V[h // 2, 1], rtol=1e-13, atol=1e-13)


def test_attn_decode_vs_scipy_softmax_and_invariances():
    from scipy.special import softmax
    rng = np.random.default_rng(12)
    for n_q, n_kv, hd, T in ((4, 2, 128, 37), (8, 1, 128, 5), (2, 2, 128, 64)):
        q = rng.standard_normal(n_q * hd)
        K = rng.standard_normal((n_kv, T, hd))
        V = rng.standard_normal((n_kv, T, hd))
        A = O.attn_decode(q, K, V, n_q, n_kv, hd).reshape(n_q, hd)
        g = n_q // n_kv
        for h in range(n_q):
            p = softmax(K[h // g] @ q.reshape(n_q, hd)[h] / math.sqrt(hd))
            np.testing.assert_allclose(A[h], p @ V[h // g], rtol=1e-12, atol=1e-13)
        perm = rng.permutation(T)       # attention does not depend on the order of the positions
        np.testing.assert_allclose(O.attn_decode(q, K[:, perm], V[:, perm], n_q, n_kv, hd).reshape(n_q, hd), A,
                                   rtol=1e-12, atol=1e-13)
        Vs = V + 2.5                    # weights sum to 1: shifting every value shifts the output
        np.testing.assert_allclose(O.attn_decode(q, K, Vs, n_q, n_kv, hd).reshape(n_q, hd), A + 2.5, rtol=1e-12, atol=1e-12)


def test_attn_kv_half_composition_and_empty_cache():
    cfg = dict(n_layers=1, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_inter=256, n_experts=0,
               top_k=0, expert_inter=0, rms_eps=1e-6, no_attn=False, no_residual=False)
    H, n_q, n_kv, hd = 256, 4, 2, 128
    qkv = S.weight_matrix(3, 0, S.MAT_QKV, None, (n_q + 2 * n_kv) * hd, H)
    o = S.weight_matrix(3, 0, S.MAT_O, None, H, n_q * hd)
    x = S.activations(3, 0, 1, H)
    rng = np.random.default_rng(13)
    cap, ctx = 12, 7
    Kc = rng.standard_normal((n_kv, cap, hd)).astype(np.float16)
    Vc = rng.standard_normal((n_kv, cap, hd)).astype(np.float16)
    # empty cache: the token attends to itself only -> identical to the identity-on-V half
    for mirror in (False, True):
        h0, _, _ = O.attn_kv_half(x, cfg, qkv, o, Kc, Vc, 0, mirror)
        np.testing.assert_array_equal(h0, O.attn_half(x, cfg, qkv, o, mirror))
    # ctx positions: the composition of the separately pinned pieces
    h, kn, vn = O.attn_kv_half(x, cfg, qkv, o, Kc, Vc, ctx, False)
    y = O.linear(O.rmsnorm(x, cfg["rms_eps"]), *qkv)[0]
    np.testing.assert_array_equal(kn.reshape(-1), y[n_q * hd:(n_q + n_kv) * hd])
    np.testing.assert_array_equal(vn.reshape(-1), y[(n_q + n_kv) * hd:])
    K = np.concatenate([Kc[:, :ctx].astype(np.float64), kn[:, None, :]], axis=1)
    V = np.concatenate([Vc[:, :ctx].astype(np.float64), vn[:, None, :]], axis=1)
    A = O.attn_decode(y[:n_q * hd], K, V, n_q, n_kv, hd)
    np.testing.assert_allclose(h[0], x[0].astype(np.float64) + O.linear(A[None, :], *o)[0], rtol=1e-13, atol=1e-13)
    # rows at and beyond ctx are never read
    Kd, Vd = Kc.copy(), Vc.copy()
    Kd[:, ctx:] = 9.0; Vd[:, ctx:] = -9.0
    h2, _, _ = O.attn_kv_half(x, cfg, qkv, o, Kd, Vd, ctx, False)
    np.testing.assert_array_equal(h2, h)


def test_attn_kv_chunk_equals_token_by_token_decode_and_is_causal():
    """A chunk of M new tokens over the cache, by the definition of causal attention, is what M
    one-token steps give when each step's rows join the cache before the next: pinned against the
    separately pinned one-token half.  Also: a one-token chunk is that half; a later token's input
    never changes an earlier token's output; rows past ctx + M are never read."""
    cfg = dict(n_layers=1, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_inter=256, n_experts=0,
               top_k=0, expert_inter=0, rms_eps=1e-6, no_attn=False, no_residual=False)
    H, n_q, n_kv, hd = 256, 4, 2, 128
    qkv = S.weight_matrix(6, 0, S.MAT_QKV, None, (n_q + 2 * n_kv) * hd, H)
    o = S.weight_matrix(6, 0, S.MAT_O, None, H, n_q * hd)
    rng = np.random.default_rng(19)
    cap, ctx, M = 20, 6, 5
    Kc = rng.standard_normal((n_kv, cap, hd)).astype(np.float16)
    Vc = rng.standard_normal((n_kv, cap, hd)).astype(np.float16)
    x = S.activations(6, 0, M, H)
    for mirror in (False, True):
        h, kn, vn = O.attn_kv_chunk_half(x, cfg, qkv, o, Kc, Vc, ctx, mirror)
        K2, V2 = Kc.copy(), Vc.copy()
        for m in range(M):
            hm, k1, v1 = O.attn_kv_half(x[m:m + 1], cfg, qkv, o, K2, V2, ctx + m, mirror)
            if mirror:      # rows are stored as fp16: the running cache holds exactly what the chunk call used
                np.testing.assert_array_equal(h[m], hm[0])
                np.testing.assert_array_equal(kn[m], k1)
                K2[:, ctx + m], V2[:, ctx + m] = k1.astype(np.float16), v1.astype(np.float16)
            else:           # pure mode keeps the chunk's rows in fp64; a fp16 cache would round them
                np.testing.assert_array_equal(kn[m], k1)
                if m == 0:
                    np.testing.assert_array_equal(h[0], hm[0])
        # one-token chunk
        h1, k1, v1 = O.attn_kv_chunk_half(x[:1], cfg, qkv, o, Kc, Vc, ctx, mirror)
        h0, k0, v0 = O.attn_kv_half(x[:1], cfg, qkv, o, Kc, Vc, ctx, mirror)
        np.testing.assert_array_equal(h1, h0)
        np.testing.assert_array_equal(k1[0], k0)
        np.testing.assert_array_equal(v1[0], v0)
        # causal: perturbing the last token leaves the earlier ones alone
        x2 = x.copy()
        x2[M - 1] = -x2[M - 1]
        hp, _, _ = O.attn_kv_chunk_half(x2, cfg, qkv, o, Kc, Vc, ctx, mirror)
        np.testing.assert_array_equal(hp[:M - 1], h[:M - 1])
        assert np.any(hp[M - 1] != h[M - 1])
        # cache rows at and beyond ctx are not read
        Kd, Vd = Kc.copy(), Vc.copy()
        Kd[:, ctx:] = 7.0; Vd[:, ctx:] = -7.0
        hd2, _, _ = O.attn_kv_chunk_half(x, cfg, qkv, o, Kd, Vd, ctx, mirror)
        np.testing.assert_array_equal(hd2, h)
    # pure mode against brute force softmax attention for the middle token of the chunk
    h, kn, vn = O.attn_kv_chunk_half(x, cfg, qkv, o, Kc, Vc, ctx, False)
    y = O.linear(O.rmsnorm(x, cfg["rms_eps"]), *qkv)
    m = 2
    A = np.zeros(n_q * hd)
    for hq in range(n_q):
        g = hq // (n_q // n_kv)
        Ks = np.concatenate([Kc[g, :ctx].astype(np.float64), y[:m + 1, (n_q + g) * hd:(n_q + g + 1) * hd]])
        Vs = np.concatenate([Vc[g, :ctx].astype(np.float64), y[:m + 1, (n_q + n_kv + g) * hd:(n_q + n_kv + g + 1) * hd]])
        sc = Ks @ y[m, hq * hd:(hq + 1) * hd] / math.sqrt(hd)
        p = np.exp(sc - sc.max()); p /= p.sum()
        A[hq * hd:(hq + 1) * hd] = p @ Vs
    np.testing.assert_allclose(h[m], x[m].astype(np.float64) + O.linear(A[None, :], *o)[0], rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- output head

def test_output_head_closed_forms():
    """logits = W_out RMSNorm(x): cases whose value is known without running the formula."""
    H, V = 128, 48
    cfg = dict(rms_eps=0.0)
    sc, co = S.weight_matrix(11, 0, S.MAT_OUT, None, V, H)
    Wd = O.dequant(sc, co)
    # a one-hot hidden state of any size selects sqrt(H) * one column of W (with its sign):
    # fails for a transposed operand, a missing norm, or a norm over the wrong axis
    for j, a in ((0, 3.0), (77, -0.25), (127, 1e3)):
        x = np.zeros((1, H)); x[0, j] = a
        np.testing.assert_allclose(O.output_head(x, cfg, (sc, co), mirror=False)[0],
                                   math.copysign(math.sqrt(H), a) * Wd[:, j], rtol=1e-13)
    # constant hidden state, constant matrix: K * d * (q - 8) * sign(c)
    d = np.full((V, H // 32), 0.5, dtype=np.float16)
    q = np.full((V, H), 11, dtype=np.uint8)
    for cval in (2.0, -7.0):
        y = O.output_head(np.full((2, H), cval), cfg, (d, q), mirror=False)
        np.testing.assert_allclose(y, math.copysign(H * 0.5 * 3, cval), rtol=1e-13)
    # without eps the logits do not depend on the scale of x; rows are independent
    x = S.activations(12, 0, 3, H).astype(np.float64)
    y = O.output_head(x, cfg, (sc, co), mirror=False)
    np.testing.assert_allclose(O.output_head(x * 37.5, cfg, (sc, co), mirror=False), y, rtol=1e-12)
    np.testing.assert_allclose(O.output_head(x[1:2], cfg, (sc, co), mirror=False)[0], y[1], rtol=1e-13)
    # the row of W most aligned with x wins the argmax once it is planted there
    sc2, co2 = sc.copy(), co.copy()
    sc2[5] = np.float16(0.05)
    co2[5] = np.where(x[0] > 0, 15, 0).astype(np.uint8)   # sign pattern of x, largest magnitude
    assert int(np.argmax(O.output_head(x[:1], cfg, (sc2, co2), mirror=False)[0])) == 5
    # eps enters as in RMSNorm: x = c * ones gives c / sqrt(c^2 + eps) per element
    y = O.output_head(np.full((1, H), 0.5), dict(rms_eps=0.75), (d, q), mirror=False)
    np.testing.assert_allclose(y, H * 1.5 * 0.5 / math.sqrt(0.25 + 0.75), rtol=1e-13)


def test_output_head_mirror_rounds_logits_to_fp16_only():
    H, V = 256, 64
    cfg = dict(rms_eps=1e-6)
    head = S.weight_matrix(13, 2, S.MAT_OUT, None, V, H)
    x = S.activations(14, 0, 4, H)
    pure = O.output_head(x, cfg, head, mirror=False)
    mir = O.output_head(x, cfg, head, mirror=True)
    assert np.array_equal(mir, pure.astype(np.float16).astype(np.float64))
    assert np.abs(mir - pure).max() <= np.abs(pure).max() * 2.0 ** -11


# ---------------------------------------------------------------- profile database estimate

def _profile_golden():
    ent, qs = [], []
    for ln in open(os.path.join(os.path.dirname(__file__), "golden", "profile_db_example.txt")):
        f = ln.split()
        if not f or f[0] == "#":
            continue
        if f[0] == "E":
            ent.append(tuple(int(v) for v in f[1:7]) + (float(f[7]),))
        else:
            qs.append((float(f[1]), tuple(int(v) for v in f[2:8]), float(f[9]), f[10]))
    return ent, qs


def test_profile_estimate_hand_worked_examples():
    ent, qs = _profile_golden()
    assert len(ent) == 5 and len(qs) == 7
    for bw, q, want_ms, want_match in qs:
        ms, match = O.profile_estimate(ent, bw, *q)
        assert match == want_match, (q, match)
        assert ms == pytest.approx(want_ms, rel=1e-9), (q, ms)


def test_profile_estimate_properties():
    ent = [(O.OPK_GEMM, 4, 0, 4096, 4096, 512, 2.0), (O.OPK_GEMM, 4, 0, 4096, 4096, 16, 0.3)]
    # compute-bound side: time scales with the work, at the neighbour's rate
    t1, _ = O.profile_estimate(ent, 1e9, O.OPK_GEMM, 4, 0, 8192, 4096, 512)
    t2, _ = O.profile_estimate(ent, 1e9, O.OPK_GEMM, 4, 0, 16384, 4096, 512)
    assert t2 == pytest.approx(2 * t1) and t1 == pytest.approx(4.0)
    # memory-bound side: bytes over the bandwidth, whatever the neighbour's time
    t3, _ = O.profile_estimate(ent, 100.0, O.OPK_GEMM, 4, 0, 8192, 4096, 2)
    assert t3 == pytest.approx((8192 * 4096 * 0.5625 + 2 * 2 * (4096 + 8192)) / 100e9 * 1e3)
    # the order of the entries does not matter unless two are equally near
    t4, _ = O.profile_estimate(ent[::-1], 1e9, O.OPK_GEMM, 4, 0, 8192, 4096, 512)
    assert t4 == t1
    # work of an operation: one multiply-add per weight and token; 4.5 bits per weight
    assert O.op_work(O.OPK_GEMV, 4, 4096, 4096, 1) == (2.0 * 4096 * 4096, 4096 * 4096 * 0.5625 + 2 * 8192)


def test_golden_files_are_what_the_oracle_writes():
    """tests/golden/make_golden.py (which calls only oracle/) regenerates the stored expected values:
    the committed files must be exactly its output."""
    import importlib.util
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    for name, make in mod.FILES.items():
        assert open(os.path.join(here, name)).read() == make(), name
