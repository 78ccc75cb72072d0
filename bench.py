"""Benchmark of the pipelined-sharding hot path on one MI355X.

A step is one pass of the whole path (every sub-layer matmul of the 32-layer 8B-shaped dense
stack, streamed shards included) over one batch of synthetic activations already in HBM.
Headline: decode tokens/s at batch 1 with a 4 GB VRAM budget (all shards resident, HBM-bound);
the same line carries the 2 GB (PCIe-bound) and 8 GB budgets, prefill TTFT at 2048 tokens, the
roofline of the dominant kernel and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_steps(torch, st, xs, xout, steps, warmup):
    for i in range(warmup):
        st.forward(xs[i % len(xs)], xout)
    st.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        st.forward(xs[i % len(xs)], xout)
    st.synchronize()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


def kernel_breakdown(B, st, plan, xs, xout, reps=3):
    """Per-kernel-kind average duration (ms) from HIP events recorded on the compute stream
    around each launch, averaged over `reps` profiled forwards."""
    ops = plan.schedule().ops()
    acc = {}
    st.set_profiling(True)
    for r in range(reps + 1):
        st.forward(xs[r % len(xs)], xout)
        st.synchronize()
        stats = st.stats()
        if stats.n_kernels == 1 and len(ops) > 1:   # persistent decode: the whole pass is one kernel
            if r > 0:
                a = acc.setdefault(("persistent", 0), [0.0, 0, 0])
                a[0] += st.op_times(1)[0][1]
                a[1] += 1
                a[2] += stats.resident_bytes_step
            continue
        times = st.op_times(len(ops))
        if r == 0:
            continue  # first profiled pass creates the events
        for o, (t0, dur) in zip(ops, times):
            key = ("copy", 0) if o.type == B.PS_OP_COPY else ("kernel", o.kernel)
            a = acc.setdefault(key, [0.0, 0, 0])
            a[0] += dur
            a[1] += 1
            a[2] += o.bytes
    st.set_profiling(False)
    return {k: dict(avg_ms=v[0] / v[1], launches=v[1] // reps, bytes_per_launch=v[2] / v[1]) for k, v in acc.items()}, stats


def cpu_baseline(cfg, seed, layers, S, O):
    """The oracle as it stands on the host cores: `layers` layers of the stack at one token."""
    import numpy as np
    sub = dict(cfg, n_layers=layers)
    shapes = {(k, e): (N, K) for (k, e, N, K) in S.matrix_shapes(sub)}
    mats = {(l, k): S.weight_matrix(seed, l, k, None, *shapes[(k, None)]) for l in range(layers) for (k, _e) in shapes}
    x = S.activations(seed, 0, 1, cfg["hidden"])
    O.lib()
    t0 = time.perf_counter()
    O.stack_forward(x, sub, lambda l, k, e: mats[(l, k)], mirror=True)
    dt = time.perf_counter() - t0
    return dt, os.cpu_count()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--layers", type=int, default=32, help="layers of the 8B-shaped stack (32 = the named config)")
    ap.add_argument("--budgets-gb", type=str, default="4,2,8", help="first one is the headline")
    ap.add_argument("--prefill-tokens", type=int, default=2048, help="0 skips the TTFT leg")
    ap.add_argument("--cpu-layers", type=int, default=4, help="oracle sample size, 0 skips")
    ap.add_argument("--measure-profile", type=int, default=1)
    ap.add_argument("--decode-mode", type=int, default=0, help="0 launch per shard, 1 persistent kernel, 2 HIP-graph replay")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1")

    import numpy as np
    import torch
    import synth_inputs as S
    from paper_2604_26334_amd import binding as B

    B.lib()  # fails loudly if libpshard.so is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    seed = 0
    cfg = S.cfg_dense8b(args.layers)
    budgets = [float(b) * 1e9 for b in args.budgets_gb.split(",")]

    prof = None
    if args.measure_profile:
        prof = B.profile_measure(1 << 30)
        log("profile: h2d %.1f GB/s, gemv %.0f GB/s, launch %.2f us, gemm TFLOP/s %s" % (
            prof.h2d_gbps, prof.gemv_gbps, prof.launch_us, ["%.0f" % v for v in prof.gemm_tflops]))

    plans = [B.Plan(cfg, int(b), 1, profile=prof) for b in budgets]
    if args.prefill_tokens:
        plans.append(B.Plan(cfg, int(budgets[0]), args.prefill_tokens, profile=prof))
    stacks = [B.Stack(p) for p in plans]
    for st in stacks:
        st.set_decode_mode(args.decode_mode)
    t0 = time.perf_counter()
    B.load_synthetic(stacks, cfg, seed, threads=min(16, os.cpu_count() or 8), progress=40)
    log("loaded %d stacks in %.1f s" % (len(stacks), time.perf_counter() - t0))

    dev = stacks[0].device
    H = cfg["hidden"]
    xs = [torch.from_numpy(S.activations(seed, t, 1, H)).to(dev) for t in range(8)]
    xout = torch.empty_like(xs[0])
    torch.cuda.synchronize()

    results = {}
    for b, plan, st in zip(budgets, plans, stacks):
        s = plan.summary()
        steps = args.steps if s.streamed_bytes == 0 else max(5, min(args.steps, 20))
        warm = args.warmup if s.streamed_bytes == 0 else 2
        ms = time_steps(torch, st, xs, xout, steps, warm)
        kb, stats = kernel_breakdown(B, st, plan, xs, xout)
        r = dict(budget_bytes=int(b), ms_per_token=ms, tokens_per_s=1e3 / ms, resident_bytes=s.resident_bytes,
                 streamed_bytes_per_token=stats.streamed_bytes_step, est_ms=s.est_step_ms, steps=steps)
        if stats.streamed_bytes_step:
            r["h2d_gbps_in_copies"] = stats.h2d_gbps
            r["pcie_gbps_whole_step"] = stats.streamed_bytes_step / (ms * 1e-3) / 1e9
            r["frac_of_measured_h2d"] = (r["pcie_gbps_whole_step"] / prof.h2d_gbps) if prof else None
            r["overlap_fraction"] = stats.overlap
        else:
            r["hbm_gbps_whole_step"] = s.weight_bytes / (ms * 1e-3) / 1e9
            r["frac_of_hbm_peak"] = r["hbm_gbps_whole_step"] / HBM_PEAK_GBS
        r["kernels"] = {("%s_%d" % k): v for k, v in kb.items()}
        results["%g" % (b / 1e9)] = r
        log("budget %.0f GB: %.3f ms/token, %.1f tok/s" % (b / 1e9, ms, 1e3 / ms), {k: round(v["avg_ms"] * 1e3, 2) for k, v in r["kernels"].items()})

    head = results["%g" % (budgets[0] / 1e9)]
    # dominant kernel of the headline run: the fused gate/up + SwiGLU GEMV (54% of the bytes)
    gu = head["kernels"].get("kernel_%d" % B.PS_K_GATE_UP)
    roof = None
    pk = head["kernels"].get("persistent_0")
    if pk:   # one persistent kernel reads every weight byte of the stack once per token
        ach = pk["bytes_per_launch"] / (pk["avg_ms"] * 1e-3) / 1e9
        roof = dict(bound="hbm", kernel="decode_persistent_kernel", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=ach / HBM_PEAK_GBS, traffic=None, bytes_per_launch=pk["bytes_per_launch"],
                    avg_launch_us=pk["avg_ms"] * 1e3)
    elif gu:
        ach = gu["bytes_per_launch"] / (gu["avg_ms"] * 1e-3) / 1e9
        roof = dict(bound="hbm", kernel="gemv_w4_kernel<GATE_UP>", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=ach / HBM_PEAK_GBS, traffic=None, bytes_per_launch=gu["bytes_per_launch"],
                    avg_launch_us=gu["avg_ms"] * 1e3)

    prefill = None
    if args.prefill_tokens:
        plan, st = plans[-1], stacks[-1]
        Mp = args.prefill_tokens
        xp = [torch.from_numpy(S.activations(seed, 100 + t, Mp, H)).to(dev) for t in range(2)]
        xpo = torch.empty_like(xp[0])
        torch.cuda.synchronize()
        ms = time_steps(torch, st, xp, xpo, 5, 2)
        s = plan.summary()
        flops = 2.0 * Mp * (s.weight_bytes / 0.5625)
        prefill = dict(tokens=Mp, budget_bytes=int(budgets[0]), ttft_ms=ms, tflops=flops / (ms * 1e-3) / 1e12,
                       frac_of_mfma_peak=flops / (ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS,
                       streamed_bytes=s.streamed_bytes, est_ms=s.est_step_ms)
        log("prefill %d tokens: TTFT %.2f ms, %.1f TFLOP/s" % (Mp, ms, prefill["tflops"]))

    cpu = None
    if args.cpu_layers:
        from oracle import oracle as O
        dt, cores = cpu_baseline(cfg, seed, args.cpu_layers, S, O)
        cpu = dict(value=1.0 / (dt * cfg["n_layers"] / args.cpu_layers), unit="tokens/s", cores=cores, kind="oracle",
                   sample="%d of %d layers of the same stack at one token, %.2f s, scaled to the full stack" % (
                       args.cpu_layers, cfg["n_layers"], dt))

    line = dict(metric="decode tokens/s at fixed VRAM budget (batch 1)", value=head["tokens_per_s"], unit="tokens/s",
                n_gpus=1, steps=head["steps"], warmup=args.warmup, ms_per_step=head["ms_per_token"],
                higher_is_better=True, scaling="weak", vs_baseline=None, dtype="w4 x f16 -> f32 accumulate",
                data="synthetic",
                config=dict(workload="dense 8B-shaped stack, %d layers, decode batch 1, budget %g GB" % (
                    cfg["n_layers"], budgets[0] / 1e9), hidden=4096, ffn=14336, weight_bytes=plans[0].summary().weight_bytes),
                roofline=roof, cpu_baseline=cpu, budgets=results, prefill=prefill,
                profile=None if prof is None else dict(h2d_gbps=prof.h2d_gbps, gemv_gbps=prof.gemv_gbps,
                                                       launch_us=prof.launch_us, gemm_tflops=list(prof.gemm_tflops)))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
