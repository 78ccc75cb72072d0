"""ctypes front-end of the CPU oracle (pshard_oracle.c): TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
It shares nothing with the HIP library and never imports it.  The layer-stack
loops live here in plain Python; every arithmetic step is a call into the C
file, which follows the plain definition of each operation in fp64.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pshard_oracle.c")
_LIB = os.path.join(_HERE, "libpshard_oracle.so")
_lib = None

MAT_QKV, MAT_O, MAT_GATE, MAT_UP, MAT_DOWN = 0, 1, 2, 3, 4


def build(force=False):
    """Compile the C oracle with gcc (OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.orc_half_to_double.restype = C.c_double
        _lib.orc_half_to_double.argtypes = [C.c_uint16]
        _lib.orc_round_f16.restype = C.c_double
        _lib.orc_round_f16.argtypes = [C.c_double]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _sc(scales, codes):
    s = np.ascontiguousarray(scales)
    assert s.dtype == np.float16
    c = np.ascontiguousarray(codes)
    assert c.dtype == np.uint8
    return s, c


def half_to_double(bits):
    return lib().orc_half_to_double(int(bits))


def round_f16(x):
    return lib().orc_round_f16(float(x))


def dequant(scales, codes):
    s, c = _sc(scales, codes)
    N, K = c.shape
    W = np.empty((N, K), dtype=np.float64)
    lib().orc_dequant(_p(s), _p(c), C.c_int64(N), C.c_int64(K), _p(W))
    return W


def linear(X, scales, codes):
    X = _f64(X)
    s, c = _sc(scales, codes)
    N, K = c.shape
    M = X.shape[0]
    assert X.shape == (M, K) and s.shape == (N, K // 32)
    Y = np.empty((M, N), dtype=np.float64)
    lib().orc_linear(_p(X), C.c_int64(M), _p(s), _p(c), C.c_int64(N), C.c_int64(K), _p(Y))
    return Y


def rmsnorm(x, eps):
    x = _f64(x)
    y = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), C.c_int64(x.shape[0]), C.c_int64(x.shape[1]), C.c_double(eps), _p(y))
    return y


def swiglu(g, u):
    g, u = _f64(g), _f64(u)
    s = np.empty_like(g)
    lib().orc_swiglu(_p(g), _p(u), C.c_int64(g.size), _p(s))
    return s


def attn_identity_v(qkv, n_q, n_kv, hd):
    qkv = _f64(qkv)
    M = qkv.shape[0]
    A = np.empty((M, n_q * hd), dtype=np.float64)
    lib().orc_attn_identity_v(_p(qkv), C.c_int64(M), n_q, n_kv, hd, _p(A))
    return A


def route_topk(logits, top_k):
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    M, E = lg.shape
    idx = np.empty((M, top_k), dtype=np.int32)
    w = np.empty((M, top_k), dtype=np.float64)
    lib().orc_route_topk(_p(lg), C.c_int64(M), E, top_k, _p(idx), _p(w))
    return idx, w


def attn_half(x, cfg, qkv, o, mirror):
    x = _f64(x)
    M, H = x.shape
    (qs, qc), (os_, oc) = _sc(*qkv), _sc(*o)
    h = np.empty_like(x)
    lib().orc_attn_half(_p(x), C.c_int64(M), H, cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                        C.c_double(cfg["rms_eps"]), _p(qs), _p(qc), _p(os_), _p(oc), int(mirror), _p(h))
    return h


def attn_decode(q, K, V, n_q, n_kv, hd):
    """Softmax attention of one token: q [n_q*hd], K, V [n_kv][T][hd] -> A [n_q*hd] (fp64)."""
    q, K, V = _f64(q).reshape(-1), _f64(K), _f64(V)
    T = K.shape[1]
    assert K.shape == (n_kv, T, hd) and V.shape == K.shape and q.size == n_q * hd
    A = np.empty(n_q * hd, dtype=np.float64)
    lib().orc_attn_decode(_p(q), _p(K), _p(V), C.c_int64(T), n_q, n_kv, hd, _p(A))
    return A


def attn_kv_half(x, cfg, qkv, o, Kc, Vc, ctx, mirror):
    """Attention half at one new token with ctx cached positions.  Kc, Vc: float16 [n_kv][cap][hd];
    row ctx of every head is left as it was (the new rows are returned, as stored, in k_new, v_new)."""
    x = _f64(x)
    assert x.shape[0] == 1
    H = x.shape[1]
    n_q, n_kv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    (qs, qc), (os_, oc) = _sc(*qkv), _sc(*o)
    Kb = np.ascontiguousarray(Kc, dtype=np.float16).view(np.uint16)
    Vb = np.ascontiguousarray(Vc, dtype=np.float16).view(np.uint16)
    cap = Kb.shape[1]
    assert Kb.shape == (n_kv, cap, hd) and Vb.shape == Kb.shape and 0 <= ctx < cap
    h = np.empty_like(x)
    k_new = np.empty((n_kv, hd), dtype=np.float64)
    v_new = np.empty((n_kv, hd), dtype=np.float64)
    lib().orc_attn_kv_half(_p(x), H, n_q, n_kv, hd, C.c_double(cfg["rms_eps"]), _p(qs), _p(qc), _p(os_), _p(oc),
                           _p(Kb), _p(Vb), C.c_int64(cap), C.c_int64(ctx), int(mirror), _p(k_new), _p(v_new), _p(h))
    return h, k_new, v_new


def attn_kv_chunk_half(x, cfg, qkv, o, Kc, Vc, ctx, mirror):
    """Attention half for a chunk of M new tokens over ctx cached positions (causal inside the chunk).
    Kc, Vc: float16 [n_kv][cap][hd], cap >= ctx + M, left as they were; returns (h [M][H],
    k_new [M][n_kv][hd], v_new [M][n_kv][hd]): the chunk's rows as stored."""
    x = _f64(x)
    M, H = x.shape
    n_q, n_kv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    (qs, qc), (os_, oc) = _sc(*qkv), _sc(*o)
    Kb = np.ascontiguousarray(Kc, dtype=np.float16).view(np.uint16)
    Vb = np.ascontiguousarray(Vc, dtype=np.float16).view(np.uint16)
    cap = Kb.shape[1]
    assert Kb.shape == (n_kv, cap, hd) and Vb.shape == Kb.shape and 0 <= ctx and ctx + M <= cap
    h = np.empty_like(x)
    k_new = np.empty((M, n_kv, hd), dtype=np.float64)
    v_new = np.empty((M, n_kv, hd), dtype=np.float64)
    lib().orc_attn_kv_chunk_half(_p(x), C.c_int64(M), H, n_q, n_kv, hd, C.c_double(cfg["rms_eps"]), _p(qs), _p(qc), _p(os_), _p(oc),
                                 _p(Kb), _p(Vb), C.c_int64(cap), C.c_int64(ctx), int(mirror), _p(k_new), _p(v_new), _p(h))
    return h, k_new, v_new


def dense_ffn_half(h, cfg, gate, up, down, mirror):
    h = _f64(h)
    M, H = h.shape
    (gs, gc), (us, uc), (ds, dc) = _sc(*gate), _sc(*up), _sc(*down)
    out = np.empty_like(h)
    lib().orc_dense_ffn_half(_p(h), C.c_int64(M), H, cfg["ffn_inter"], C.c_double(cfg["rms_eps"]),
                             _p(gs), _p(gc), _p(us), _p(uc), _p(ds), _p(dc),
                             int(not cfg["no_residual"]), int(mirror), _p(out))
    return out


def moe_ffn_half(h, cfg, logits, experts, mirror):
    """experts: dict expert_id -> ((gs,gc),(us,uc),(ds,dc)); must hold every selected expert."""
    h = _f64(h)
    M, H = h.shape
    E, k = cfg["n_experts"], cfg["top_k"]
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    assert lg.shape == (M, E)
    keep = []
    arrs = [(C.c_void_p * E)() for _ in range(6)]
    for e, mats in experts.items():
        flat = []
        for s, c in mats:
            s, c = _sc(s, c)
            flat += [s, c]
        keep.append(flat)
        for i in range(6):
            arrs[i][e] = flat[i].ctypes.data
    out = np.empty_like(h)
    lib().orc_moe_ffn_half(_p(h), C.c_int64(M), H, cfg["expert_inter"], E, k, C.c_double(cfg["rms_eps"]),
                           _p(lg), arrs[0], arrs[1], arrs[2], arrs[3], arrs[4], arrs[5], int(mirror), _p(out))
    return out


def stack_forward(x, cfg, weights, logits=None, mirror=True, per_layer=None, kv=None, ctx=0, new_rows=None):
    """Run the whole decoder weight stack on x [M][H].

    weights(layer, kind, expert) -> (scales, codes) for one logical matrix (called
    on demand so the full model never has to be resident).  logits: fp32 [L][M][E]
    for MoE stacks.  per_layer, if a list, receives each layer's output.
    kv: None (attention = identity on V) or kv(layer) -> (K, V) float16 [n_kv][cap][hd] caches holding
    ctx earlier positions: the new tokens (one, or a chunk with causal attention inside it) attend over
    them and themselves; new_rows, if a list, receives each layer's (k_new, v_new) ([n_kv][hd] for one
    token, [M][n_kv][hd] for a chunk).
    """
    x = _f64(x)
    for l in range(cfg["n_layers"]):
        h = x
        if not cfg["no_attn"] and kv is not None:
            Kc, Vc = kv(l)
            if x.shape[0] == 1:
                h, kn, vn = attn_kv_half(x, cfg, weights(l, MAT_QKV, None), weights(l, MAT_O, None), Kc, Vc, ctx, mirror)
            else:   # a chunk of new tokens: causal inside the chunk; rows come back as [M][n_kv][hd]
                h, kn, vn = attn_kv_chunk_half(x, cfg, weights(l, MAT_QKV, None), weights(l, MAT_O, None), Kc, Vc, ctx, mirror)
            if new_rows is not None:
                new_rows.append((kn, vn))
        elif not cfg["no_attn"]:
            h = attn_half(x, cfg, weights(l, MAT_QKV, None), weights(l, MAT_O, None), mirror)
        if cfg["n_experts"] == 0:
            x = dense_ffn_half(h, cfg, weights(l, MAT_GATE, None), weights(l, MAT_UP, None),
                               weights(l, MAT_DOWN, None), mirror)
        else:
            idx, _ = route_topk(logits[l], cfg["top_k"])
            experts = {int(e): (weights(l, MAT_GATE, int(e)), weights(l, MAT_UP, int(e)),
                                weights(l, MAT_DOWN, int(e))) for e in np.unique(idx)}
            x = moe_ffn_half(h, cfg, logits[l], experts, mirror)
        if per_layer is not None:
            per_layer.append(x.copy())
    return x


def output_head(x, cfg, head, mirror=True):
    """Output projection after the last layer (the "outputs" entry of the priority list, Section 3
    planning phase): logits = Linear_head(RMSNorm(x)), x [M][H] the stack's final hidden state,
    head = (scales, codes) of the [vocab][H] matrix.  mirror rounds the logits to fp16, as stored."""
    y = linear(rmsnorm(x, cfg["rms_eps"]), *head)
    if mirror:
        y = y.astype(np.float16).astype(np.float64)
    return y


TIER_TOKENS = (1, 4, 16, 32, 64, 512, 1024, 2048, 4096, 8192, 16384)   # the tier set of Section 3


def pick_tier(est_ms, new_tokens, tier_tokens=TIER_TOKENS):
    """PickTier (Section 3, inference phase), written out: over the tiers that have a schedule
    (est_ms[t] is not None), the one minimising ceil(new_tokens / tier_tokens[t]) * est_ms[t];
    among equal products the lowest tier.  Returns (tier, iterations, total_ms).
    Exact: the products are compared as rationals, not as rounded floats."""
    from fractions import Fraction
    best = None
    for t, (tok, est) in enumerate(zip(tier_tokens, est_ms)):
        if est is None:
            continue
        iters = -(-int(new_tokens) // tok)
        total = iters * Fraction(est)
        if best is None or total < best[2]:
            best = (t, iters, total)
    if best is None:
        raise ValueError("no tier has a schedule")
    return best[0], best[1], float(best[2])


# ---- profile database (Section 3, profiler-based timing estimation) -----------------------------

OPK_GEMV, OPK_GEMM, OPK_CPU, OPK_H2D = 0, 1, 2, 3


def op_work(op, quant, n, k, m):
    """(floating point operations, bytes moved) of one benchmarked operation: a [n][k] block-format
    matrix (quant bits per weight plus one fp16 scale per 32 weights) times m fp16 activation rows,
    or, for a copy, n bytes."""
    if op == OPK_H2D:
        return 0.0, float(n)
    flops = 2.0 * n * k * m
    nbytes = n * k * (quant / 8.0 + 2.0 / 32.0) + 2.0 * m * (k + n)
    return flops, nbytes


def profile_estimate(entries, bandwidth_gbps, op, quant, threads, n, k, m):
    """Time estimate of one kernel from a profile database, as the paper's estimator does it.

    entries: list of (op, quant, threads, n, k, m, ms).  Returns (ms, match) with match
    'exact' (same op, quantisation, thread count and dimensions: the entry's own rate),
    'neighbour' (same op, quantisation and thread count, other dimensions: the entry nearest in
    the space of dimensions gives the FLOPS roof of a roofline whose memory roof is
    bandwidth_gbps; the kernel is priced compute-bound or memory-bound by where its arithmetic
    intensity falls), or 'none' (no entry of that op, quantisation and thread count: skipped, 0 ms).
    Distance: Euclidean in (log2 n, log2 k, log2 m); equal distances keep the earlier entry.
    A copy has no FLOPS: its rate in bytes/s takes that place."""
    import math
    flops, nbytes = op_work(op, quant, n, k, m)
    same = [e for e in entries if e[0] == op and e[1] == quant and e[2] == threads]
    for e in same:
        if (e[3], e[4], e[5]) == (n, k, m):
            return float(e[6]), "exact"
    if not same:
        return 0.0, "none"
    def dist(e):
        return math.sqrt(sum((math.log2(a) - math.log2(b)) ** 2 for a, b in zip((e[3], e[4], e[5]), (n, k, m))))
    best = min(same, key=dist)      # min keeps the first of equal keys
    e_flops, e_bytes = op_work(best[0], best[1], best[3], best[4], best[5])
    if op == OPK_H2D:
        return nbytes / (e_bytes / best[6]), "neighbour"
    roof_flops = e_flops / (best[6] * 1e-3)             # flop/s of the neighbour
    roof_bw = bandwidth_gbps * 1e9
    if flops / nbytes >= roof_flops / roof_bw:          # right of the ridge: compute-bound
        return flops / roof_flops * 1e3, "neighbour"
    return nbytes / roof_bw * 1e3, "neighbour"
