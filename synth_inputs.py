"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU harness.

This module only draws random numbers with the shapes and distributions of the
workloads (4-bit block-quantised decoder weight stacks, fp16 activations, fp32
router logits).  It holds none of the method's arithmetic: no dequantisation,
no matmul, no routing.  Every array is keyed by (seed, layer, kind, expert) or
(seed, step), so any single matrix can be regenerated alone.

Logical weight format (the only format that crosses the library boundary):
  scales : float16 [N][K/32]   d = |N(0,1)| * 0.02, one per 32 weights along K
  codes  : uint8   [N][K]      q ~ U{0..15}, one code per byte
  meaning: w[n][k] = d[n][k/32] * (q[n][k] - 8)
"""
import numpy as np

BLOCK = 32

# matrix kinds; numeric values match the C header's PS_MAT_* constants
MAT_QKV, MAT_O, MAT_GATE, MAT_UP, MAT_DOWN = 0, 1, 2, 3, 4
MAT_OUT = 5   # output head, addressed as a matrix of layer n_layers
NO_EXPERT = 0xFFFF


def _gen(seed, stream, a=0, b=0, c=0):
    key = [np.uint64(seed), np.uint64((stream << 56) | (a << 32) | (b << 16) | c)]
    return np.random.Generator(np.random.Philox(key=key))


def weight_matrix(seed, layer, kind, expert, N, K):
    """Return (scales f16 [N][K/32], codes u8 [N][K]) for one logical matrix."""
    assert K % BLOCK == 0
    e = NO_EXPERT if expert is None else expert
    g = _gen(seed, 1, layer, kind, e)
    scales = (np.abs(g.standard_normal((N, K // BLOCK), dtype=np.float32)) * np.float32(0.02)).astype(np.float16)
    raw = g.bit_generator.random_raw((N * K // 2 + 7) // 8).view(np.uint8)[: N * K // 2]
    codes = np.empty(N * K, dtype=np.uint8)
    codes[0::2] = raw & 15
    codes[1::2] = raw >> 4
    return scales, codes.reshape(N, K)


def head_matrix(seed, cfg):
    """(scales, codes) of the output head [vocab][hidden], drawn like every other weight matrix."""
    return weight_matrix(seed, cfg["n_layers"], MAT_OUT, None, cfg["vocab"], cfg["hidden"])


def activations(seed, step, M, H):
    """fp16 N(0,1) activations [M][H] for decode/prefill step `step`."""
    g = _gen(seed, 2, step)
    return g.standard_normal((M, H), dtype=np.float32).astype(np.float16)


def kv_cache(seed, layer, n_kv, n_pos, head_dim=128):
    """Synthetic KV cache of one layer: (K, V) fp16 [n_kv][n_pos][head_dim], N(0,1) entries (keys of
    unit variance per dimension give scores q.k / sqrt(d) of order |q|, i.e. a softmax that is
    neither flat nor one-hot for the normalised queries of this stack)."""
    g = _gen(seed, 5, layer)
    K = g.standard_normal((n_kv, n_pos, head_dim), dtype=np.float32).astype(np.float16)
    V = g.standard_normal((n_kv, n_pos, head_dim), dtype=np.float32).astype(np.float16)
    return K, V


def router_logits(seed, step, L, M, E, bias_seed=None):
    """fp32 N(0,1) router logits [L][M][E].  With bias_seed, a fixed
    per-(layer, expert) N(0,1) bias is added so that some experts are hot."""
    g = _gen(seed, 3, step)
    lg = g.standard_normal((L, M, E), dtype=np.float32)
    if bias_seed is not None:
        b = _gen(bias_seed, 4).standard_normal((L, 1, E), dtype=np.float32)
        lg = (lg + b).astype(np.float32)
    return lg


# ---- workload shapes (synthetic stand-ins; no trained weights) ----------------

def cfg_ffn_block():
    """Single dense FFN block: hidden 1024, intermediate 2816, no attention, no residual."""
    return dict(n_layers=1, hidden=1024, n_q_heads=0, n_kv_heads=0, head_dim=0,
                ffn_inter=2816, n_experts=0, top_k=0, expert_inter=0,
                rms_eps=1e-6, no_attn=True, no_residual=True)


def cfg_dense8b(n_layers=32):
    return dict(n_layers=n_layers, hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                ffn_inter=14336, n_experts=0, top_k=0, expert_inter=0,
                rms_eps=1e-6, no_attn=False, no_residual=False)


def cfg_moe(n_layers=48):
    return dict(n_layers=n_layers, hidden=2048, n_q_heads=32, n_kv_heads=4, head_dim=128,
                ffn_inter=0, n_experts=128, top_k=8, expert_inter=768,
                rms_eps=1e-6, no_attn=False, no_residual=False)


def matrix_shapes(cfg):
    """List of (kind, expert, N, K) logical matrices in one layer."""
    H = cfg["hidden"]
    out = []
    if not cfg["no_attn"]:
        nq, nkv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
        out.append((MAT_QKV, None, (nq + 2 * nkv) * hd, H))
        out.append((MAT_O, None, H, nq * hd))
    if cfg["n_experts"] == 0:
        I = cfg["ffn_inter"]
        out += [(MAT_GATE, None, I, H), (MAT_UP, None, I, H), (MAT_DOWN, None, H, I)]
    else:
        I = cfg["expert_inter"]
        for e in range(cfg["n_experts"]):
            out += [(MAT_GATE, e, I, H), (MAT_UP, e, I, H), (MAT_DOWN, e, H, I)]
    return out
