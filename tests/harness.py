"""Shared helpers for the GPU parity tests: run the HIP stack and the CPU oracle on the same
seeded inputs.  The oracle and the HIP library never see each other; only this test code does."""
import numpy as np

import synth_inputs as S
from oracle import oracle as O


def small_dense_cfg(n_layers=2):
    # 8B-shaped in miniature: several row-tiles per matrix, K not a multiple of 1024 for down
    return dict(n_layers=n_layers, hidden=512, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_inter=1408,
                n_experts=0, top_k=0, expert_inter=0, rms_eps=1e-6, no_attn=False, no_residual=False)


def small_moe_cfg(n_layers=2):
    return dict(n_layers=n_layers, hidden=256, n_q_heads=4, n_kv_heads=1, head_dim=128, ffn_inter=0,
                n_experts=8, top_k=2, expert_inter=128, rms_eps=1e-6, no_attn=False, no_residual=False)


class WeightCache:
    """weights(layer, kind, expert) -> (scales, codes), generated on demand and memoised."""

    def __init__(self, cfg, seed, keep=True):
        self.shapes = {(k, e): (N, K) for (k, e, N, K) in S.matrix_shapes(cfg)}
        self.seed, self.keep, self.mem = seed, keep, {}

    def __call__(self, layer, kind, expert):
        key = (layer, kind, expert)
        if key in self.mem:
            return self.mem[key]
        N, K = self.shapes[(kind, expert)]
        w = S.weight_matrix(self.seed, layer, kind, expert, N, K)
        if self.keep:
            self.mem[key] = w
        return w


def total_weight_bytes(cfg):
    from paper_2604_26334_amd import binding as B
    p = B.Plan(cfg, 1 << 62, 1)
    return p.summary().weight_bytes, p.summary().workspace_bytes


def run_gpu(cfg, weights, budget, x_np, logits=None, expert_freq=None, steps=1, profile=None, mode=0, copy_mode=None):
    """Plan for budget, load, run one forward per x in x_np (list) -> list of fp16 numpy outputs."""
    import torch
    from paper_2604_26334_amd import binding as B
    xs = x_np if isinstance(x_np, list) else [x_np]
    M = xs[0].shape[0]
    plan = B.Plan(cfg, int(budget), M, profile=profile, expert_freq=expert_freq)
    st = B.Stack(plan)
    st.set_decode_mode(mode)
    if copy_mode is not None:
        st.set_copy_mode(copy_mode)
    for layer in range(cfg["n_layers"]):
        for kind, expert, N, K in S.matrix_shapes(cfg):
            sc, cd = weights(layer, kind, expert)
            st.load_matrix(layer, kind, expert, sc, cd)
    outs = []
    for i, x in enumerate(xs):
        xin = torch.from_numpy(np.ascontiguousarray(x)).to(st.device)
        xout = torch.empty_like(xin)
        lg = None if logits is None else (logits[i] if isinstance(logits, list) else logits)
        torch.cuda.synchronize()
        st.forward(xin, xout, lg)
        st.synchronize()
        outs.append(xout.cpu().numpy())
    summary = plan.summary()
    info = dict(resident=summary.resident_bytes, streamed=summary.streamed_bytes, slots=summary.n_slots,
                slot_bytes=summary.slot_bytes, stats=st.stats())
    st.close()
    plan.close()
    return outs if isinstance(x_np, list) else outs[0], info


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / np.abs(ref).max())


def kv_token_reference_from_gpu_qkv(cfg, weights, x_row, qkv_row, Kc, Vc, ctx):
    """One-layer reference for ONE new token at context ctx that takes the token's QKV row as the GPU
    stored it (fp16) instead of projecting it again: h = x + Linear_O(fp16(Attention(q, cache rows +
    own k, v))), out = FFN half of h, rounding where the GPU stores fp16.  Softmax over scores of the
    size this stack produces is sharp: a last-bit difference in q or k moves weight between positions,
    so the attention kernel is checked on the very q, k, v it read (the projection that made them is
    checked on its own).  Kc, Vc: float16 [n_kv][cap][hd] with rows 0 .. ctx - 1 valid."""
    n_q, n_kv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    y = np.asarray(qkv_row, dtype=np.float16).astype(np.float64).reshape(-1)
    k_new = y[n_q * hd:(n_q + n_kv) * hd].reshape(n_kv, 1, hd)
    v_new = y[(n_q + n_kv) * hd:].reshape(n_kv, 1, hd)
    K = np.concatenate([np.asarray(Kc)[:, :ctx].astype(np.float64), k_new], axis=1)
    V = np.concatenate([np.asarray(Vc)[:, :ctx].astype(np.float64), v_new], axis=1)
    A = O.attn_decode(y[:n_q * hd], K, V, n_q, n_kv, hd).astype(np.float16).astype(np.float64)
    h = O.linear(A[None, :], *weights(0, S.MAT_O, None)) + np.asarray(x_row, dtype=np.float64).reshape(1, -1)
    h = h.astype(np.float16).astype(np.float64)
    return O.dense_ffn_half(h, cfg, weights(0, S.MAT_GATE, None), weights(0, S.MAT_UP, None), weights(0, S.MAT_DOWN, None), True)
