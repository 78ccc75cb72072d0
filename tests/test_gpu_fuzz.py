"""Seeded sweep on the GPU: random small models (dense / MoE, with or without attention, residual,
output head), budgets, token counts and plan kinds, each forward against the CPU oracle at
max|err| / max|ref| <= 5e-3, both the oracle that rounds where the GPU stores fp16 and the pure fp64 one."""
import numpy as np
import pytest

import synth_inputs as S
from oracle import oracle as O
from tests import harness as Hn

pytestmark = pytest.mark.gpu
TOL = 5e-3


def _random_cfg(rng, hiddens=(128, 256, 512), max_layers=3):
    moe = rng.random() < 0.4
    attn = rng.random() < 0.8
    n_kv = int(rng.choice([1, 2]))
    cfg = dict(n_layers=int(rng.integers(1, max_layers + 1)), hidden=int(rng.choice(list(hiddens))),
               n_q_heads=n_kv * int(rng.choice([1, 2, 4])) if attn else 0, n_kv_heads=n_kv if attn else 0,
               head_dim=128 if attn else 0, ffn_inter=0 if moe else 128 * int(rng.integers(1, 9)),
               n_experts=int(rng.choice([4, 8])) if moe else 0, top_k=0,
               expert_inter=128 * int(rng.integers(1, 3)) if moe else 0, rms_eps=1e-6, no_attn=not attn,
               no_residual=bool(rng.random() < 0.2) and not moe)     # (the flag is the bare dense FFN block's)
    if moe:
        cfg["top_k"] = int(rng.integers(1, 4))
    if rng.random() < 0.5:
        cfg["vocab"] = 16 * int(rng.integers(4, 120))
    return cfg


@pytest.mark.parametrize("seed", range(4))
def test_random_models_match_the_oracle(seed):
    _sweep(4000 + seed, 8, (128, 256, 512), 3, [1, 1, 2, 5, 16, 33, 64, 130])


@pytest.mark.parametrize("seed", range(2))
def test_random_models_of_whole_scale_groups_and_few_tokens(seed):
    """Hidden sizes that are multiples of 1024 with two to four tokens: the few-token form of the decode kernel
    on the attention matrices and the dense gate/up (and on the down projection where the intermediate size is a
    multiple of 1024 too), next to the GEMM path, the CPU plans and the output head."""
    _sweep(5000 + seed, 6, (1024, 2048), 2, [2, 3, 4, 4])


def _sweep(seed0, cases, hiddens, max_layers, token_counts):
    import torch
    from paper_2604_26334_amd import binding as B
    seed = seed0
    rng = np.random.default_rng(seed0)
    prof = B.make_profile(h2d_gbps=50.0, gemv_gbps=4000.0, cpu_gbps=150.0, cpu_gbps_busy=120.0, h2d_gbps_busy=45.0,
                          cpu_tokens_free=3.0, cpu_sync_us=0.5)
    for case in range(cases):
        cfg = _random_cfg(rng, hiddens, max_layers)
        M = int(rng.choice(token_counts))
        wseed = int(rng.integers(1 << 20))
        W = Hn.WeightCache(cfg, wseed)
        head = S.head_matrix(wseed, cfg) if cfg.get("vocab") else None
        x = S.activations(wseed, 0, M, cfg["hidden"])
        lg = S.router_logits(wseed, 0, cfg["n_layers"], M, cfg["n_experts"]) if cfg["n_experts"] else None
        ref_x = O.stack_forward(x, cfg, W, logits=lg, mirror=True)
        ref_l = O.output_head(ref_x, cfg, head, mirror=True) if head else None
        pure_x = O.stack_forward(x, cfg, W, logits=lg, mirror=False)      # the plain fp64 definition
        pure_l = O.output_head(pure_x, cfg, head, mirror=False) if head else None
        full = B.Plan(cfg, 1 << 40, M).summary()
        frac = float(rng.choice([0.1, 0.3, 0.6, 1.1]))
        budget = full.workspace_bytes + int(full.weight_bytes * frac) + (1 << 16)
        kinds = [B.PS_PLAN_GPU_ONLY] + ([B.PS_PLAN_STATIC, B.PS_PLAN_DYNAMIC] if M <= 64 else [])
        for kind in kinds:
            try:
                plan = B.Plan(cfg, budget, M, profile=prof, kind=kind)
            except B.PshardError as e:
                assert e.code == B.PS_E_BUDGET
                continue
            st = B.Stack(plan)
            for layer in range(cfg["n_layers"]):
                for k, e, N, K in S.matrix_shapes(cfg):
                    st.load_matrix(layer, k, e, *W(layer, k, e))
            lo = None
            if head:
                st.load_matrix(cfg["n_layers"], S.MAT_OUT, None, *head)
                lo = torch.zeros((M, cfg["vocab"]), dtype=torch.float16, device=st.device)
                st.set_logits_out(lo, 0, M)
            xin = torch.from_numpy(x).to(st.device)
            xout = torch.empty_like(xin)
            torch.cuda.synchronize()
            st.forward(xin, xout, lg)
            st.synchronize()
            s = plan.summary()
            e_x = Hn.rel_err(xout.cpu().numpy(), ref_x)
            e_l = Hn.rel_err(lo.cpu().numpy(), ref_l) if head else 0.0
            p_x = Hn.rel_err(xout.cpu().numpy(), pure_x)
            p_l = Hn.rel_err(lo.cpu().numpy(), pure_l) if head else 0.0
            print("  seed %d case %d kind %d: L%d H%d %s M%d frac %.1f pinned %d streamed %d cpu %d  err %.2e %.2e" % (
                seed, case, kind, cfg["n_layers"], cfg["hidden"], "moe" if cfg["n_experts"] else "dense", M, frac,
                s.resident_bytes, s.streamed_bytes, s.cpu_bytes, e_x, e_l), flush=True)
            assert e_x <= TOL and e_l <= TOL, (cfg, M, budget, kind)
            assert p_x <= TOL and p_l <= TOL, (cfg, M, budget, kind, p_x, p_l)
            st.close()
            plan.close()
