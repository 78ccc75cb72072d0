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
    for i in range(max(warmup, len(xs))):  # every input buffer once: graph mode captures one graph per buffer
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


def cpu_baseline(cfg, seed, layers, reps, S, O):
    """The oracle as it stands on the host cores: `layers` layers of the stack, one token, `reps`
    tokens one after the other.  Weights are generated beforehand (not timed)."""
    from concurrent.futures import ThreadPoolExecutor
    sub = dict(cfg, n_layers=layers)
    shapes = {(k, e): (N, K) for (k, e, N, K) in S.matrix_shapes(sub)}
    keys = [(l, k) for l in range(layers) for (k, _e) in shapes]
    with ThreadPoolExecutor(max_workers=8) as ex:
        vals = list(ex.map(lambda lk: S.weight_matrix(seed, lk[0], lk[1], None, *shapes[(lk[1], None)]), keys))
    mats = dict(zip(keys, vals))
    O.lib()
    t0 = time.perf_counter()
    for r in range(reps):
        O.stack_forward(S.activations(seed, r, 1, cfg["hidden"]), sub, lambda l, k, e: mats[(l, k)], mirror=True)
    dt = (time.perf_counter() - t0) / reps
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return dt, min(threads, os.cpu_count() or threads)


def batched_leg(B, S, torch, cfg, seed, prof, tokens, budgets, steps, decode_mode=1):
    """Batched decode (config 5): `tokens` tokens per step, `steps` steps of fresh activations (decode mode 1:
    the step's launches replayed from a HIP graph where every shard is resident)."""
    out = {}
    plans = [B.Plan(cfg, int(b), tokens, profile=prof) for b in budgets]
    stacks = [B.Stack(p) for p in plans]
    B.load_synthetic(stacks, cfg, seed, threads=min(16, os.cpu_count() or 8))
    dev = stacks[0].device
    xs = [torch.from_numpy(S.activations(seed, 200 + t, tokens, cfg["hidden"])).to(dev) for t in range(4)]
    xo = torch.empty_like(xs[0])
    torch.cuda.synchronize()
    for b, plan, st in zip(budgets, plans, stacks):
        s = plan.summary()
        st.set_decode_mode(decode_mode)
        ms = time_steps(torch, st, xs, xo, steps, 3)
        flops = 2.0 * tokens * (s.weight_bytes / 0.5625)
        out["%g" % (b / 1e9)] = dict(budget_bytes=int(b), tokens_per_step=tokens, steps=steps, ms_per_step=ms,
                                     graph_replay=int(st.stats().graph_replay),
                                     tokens_per_s=tokens * 1e3 / ms, resident_bytes=s.resident_bytes,
                                     streamed_bytes_per_step=st.stats().streamed_bytes_step,
                                     hbm_gbps=s.weight_bytes / (ms * 1e-3) / 1e9,
                                     frac_of_hbm_peak=s.weight_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                     tflops=flops / (ms * 1e-3) / 1e12)
        log("batch %d, budget %.0f GB: %.3f ms/step, %.0f tok/s" % (tokens, b / 1e9, ms, tokens * 1e3 / ms))
        st.close()
    return out


def expert_frequencies(B, S, cfg, seed, bias_seed, tokens=1024):
    """Selection frequency of every (layer, expert) over a host warm-up of `tokens` tokens routed with
    the library's own rule (ps_route_host): the share of tokens that select the expert."""
    import numpy as np
    lg = S.router_logits(seed, 999, cfg["n_layers"], tokens, cfg["n_experts"], bias_seed=bias_seed)
    freq = np.zeros((cfg["n_layers"], cfg["n_experts"]), dtype=np.float32)
    for l in range(cfg["n_layers"]):
        idx = B.route_host(lg[l], cfg["top_k"])
        freq[l] = np.bincount(idx.reshape(-1), minlength=cfg["n_experts"]) / float(tokens)
    return freq


def moe_leg(B, S, torch, seed, prof, budget, token_counts, steps, bias_seed=7):
    """MoE stack (config 4): 48 layers, 128 experts, top-8; decode at each token count.  Three runs per
    token count: the config's own router logits (i.i.d. N(0,1): every expert equally hot) on the plan
    without frequencies; and, as this build's variant of "hot experts", logits with a fixed
    per-(layer, expert) N(0,1) bias on that same plan and on a plan whose experts are ranked by the
    selection frequencies of a 1024-token host warm-up."""
    import numpy as np
    cfg = S.cfg_moe()
    out = {}
    names = ["gpu_only", "static", "dynamic"]
    plans, tags = [], []
    db = None
    if prof is not None and prof.cpu_gbps > 0:
        db = B.ProfileDB()
        db.measure(cfg)
    db_est = {}
    freq = expert_frequencies(B, S, cfg, seed, bias_seed) if bias_seed is not None else None
    for m in token_counts:
        plans.append(B.Plan(cfg, int(budget), m, profile=prof))
        tags.append((m, "batch_%d" % m, None))
        if freq is not None:
            tags.append((m, "batch_%d_hot_experts_unranked" % m, bias_seed))     # same plan, biased logits
            plans.append(plans[-1])
            plans.append(B.Plan(cfg, int(budget), m, profile=prof, expert_freq=freq))
            tags.append((m, "batch_%d_hot_experts_ranked" % m, bias_seed))
        if prof is not None and prof.cpu_gbps > 0:   # HeuristicSplit's pick, if it is not Plan One again
            auto = B.Plan(cfg, int(budget), m, profile=prof, kind=B.PS_PLAN_AUTO)
            auto_db = B.Plan(cfg, int(budget), m, profile=prof, kind=B.PS_PLAN_AUTO, db=db).summary()
            db_est[m] = dict(picked=names[auto_db.plan_kind], est_ms={names[k]: auto_db.est_kind_ms[k] for k in range(3)})
            log("MoE batch %d: HeuristicSplit estimates %s -> %s; priced from the profile database %s -> %s" % (
                m, ["%.1f" % e for e in auto.summary().est_kind_ms], names[auto.summary().plan_kind],
                ["%.1f" % e for e in auto_db.est_kind_ms], names[auto_db.plan_kind]))
            if auto.summary().plan_kind != B.PS_PLAN_GPU_ONLY:
                plans.append(auto)
                tags.append((m, "batch_%d_%s" % (m, names[auto.summary().plan_kind]), None))
    stacks, cur_m = {}, None
    for (m, tag, bias), plan in zip(tags, plans):
        if m != cur_m:      # one token count at a time: each stack keeps its unpinned experts (11 GB) in pinned host memory
            for st in stacks.values():
                st.close()
            uniq = []
            for (m2, _t, _b), p2 in zip(tags, plans):
                if m2 == m and not any(p2 is q for q in uniq):
                    uniq.append(p2)
            stacks = {id(p2): B.Stack(p2) for p2 in uniq}
            t0 = time.perf_counter()
            B.load_synthetic(list(stacks.values()), cfg, seed, threads=min(16, os.cpu_count() or 8), progress=6000)
            log("loaded %d MoE stacks (%d token(s) per step) in %.1f s" % (len(stacks), m, time.perf_counter() - t0))
            dev = next(iter(stacks.values())).device
            cur_m = m
        st = stacks[id(plan)]
        s = plan.summary()
        xs = [torch.from_numpy(S.activations(seed, 300 + t, m, cfg["hidden"])).to(dev) for t in range(4)]
        lgs = [S.router_logits(seed, 300 + t, cfg["n_layers"], m, cfg["n_experts"], bias_seed=bias) for t in range(4)]
        # share of the routed (token, expert) pairs whose expert is pinned in VRAM
        res = np.zeros((cfg["n_layers"], cfg["n_experts"]), dtype=bool)
        for sh in plan.shards():
            if sh.kind == B.PS_SHARD_EXPERT:
                res[sh.layer, sh.expert] = sh.resident == 1
        hits = pairs = 0
        for lg in lgs:
            for l in range(cfg["n_layers"]):
                idx = B.route_host(lg[l], cfg["top_k"])
                hits += int(res[l][idx.reshape(-1)].sum())
                pairs += idx.size
        xo = torch.empty_like(xs[0])
        torch.cuda.synchronize()
        for i in range(2):
            st.forward(xs[i], xo, lgs[i])
        st.synchronize()
        streamed = on_cpu = 0
        cpu_ms = 0.0
        t0 = time.perf_counter()
        for i in range(steps):
            st.forward(xs[i % 4], xo, lgs[i % 4])
            stt = st.stats()
            streamed += stt.streamed_bytes_step
            on_cpu += stt.cpu_bytes_step
            cpu_ms += stt.cpu_ms
        st.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        out[tag] = dict(budget_bytes=int(budget), tokens_per_step=m, ms_per_step=ms, tokens_per_s=m * 1e3 / ms,
                        plan=names[s.plan_kind], resident_bytes=s.resident_bytes, streamed_bytes_per_step=streamed / steps,
                        cpu_bytes_per_step=on_cpu / steps, cpu_ms_per_step=cpu_ms / steps,
                        pcie_gbps_whole_step=streamed / steps / (ms * 1e-3) / 1e9,
                        frac_of_measured_h2d=(streamed / steps / (ms * 1e-3) / 1e9 / prof.h2d_gbps) if prof else None,
                        est_ms=s.est_step_ms, heuristic_split_with_database=db_est.get(m),
                        router_logits="N(0,1)" if bias is None else "N(0,1) + fixed per-(layer, expert) N(0,1) bias (this build's hot-expert variant)",
                        resident_hit_rate=hits / max(1, pairs))
        log("MoE batch %d (%s), budget %.0f GB, plan %s: %.2f ms/step (estimate %.2f), %.1f tok/s, resident hit rate %.3f, %.2f GB streamed/step, %.2f GB/step on the CPU in %.2f ms" % (
            m, tag, budget / 1e9, names[s.plan_kind], ms, s.est_step_ms, m * 1e3 / ms, hits / max(1, pairs), streamed / steps / 1e9,
            on_cpu / steps / 1e9, cpu_ms / steps))
    for st in stacks.values():
        st.close()
    return out


def tier_leg(B, S, torch, cfg, seed, prof, budget, tokens, db=None):
    """Token-tier table + PickTier + chunked prefill: plan every tier under `budget` (priced from the
    profile database when one is given), pick the tier for a prompt of `tokens` tokens, and time the
    chunked prefill with the picked tier and its two neighbours (estimate against measurement for each)."""
    table = B.TierTable(cfg, int(budget), profile=prof, db=db)
    choice = table.pick(tokens)
    ents = table.entries()
    cand = [t for t in (choice.tier - 1, choice.tier, choice.tier + 1)
            if 0 <= t < B.PS_NTIERS and ents[t].feasible and ents[t].tier_tokens >= 64]
    stacks = [B.Stack(table.plan(t)) for t in cand]
    B.load_synthetic(stacks, cfg, seed, threads=min(16, os.cpu_count() or 8))
    dev = stacks[0].device
    x = torch.from_numpy(S.activations(seed, 400, tokens, cfg["hidden"])).to(dev)
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    out = dict(budget_bytes=int(budget), tokens=tokens, picked_tier_tokens=choice.tier_tokens, tiers={},
               estimates="profile database" if db is not None else "profile rates")
    for t, st in zip(cand, stacks):
        e = ents[t]
        B.chunked_forward(st, x, y)
        st.synchronize()
        reps = 3
        t0 = time.perf_counter()
        for _ in range(reps):
            trips = B.chunked_forward(st, x, y)
        st.synchronize()
        ms = (time.perf_counter() - t0) / reps * 1e3
        out["tiers"]["%d" % e.tier_tokens] = dict(trips=trips, ttft_ms=ms, est_ms=trips * e.summary.est_step_ms,
                                                  resident_bytes=e.summary.resident_bytes,
                                                  workspace_bytes=e.summary.workspace_bytes)
        log("prefill %d tokens, budget %.0f GB, tier %d x %d trips: TTFT %.1f ms (estimate %.1f ms)%s" % (
            tokens, budget / 1e9, e.tier_tokens, trips, ms, trips * e.summary.est_step_ms,
            "  <- picked" if t == choice.tier else ""))
        st.close()
    best = min(out["tiers"], key=lambda k: out["tiers"][k]["ttft_ms"])
    out["measured_best_tier_tokens"] = int(best)
    return out


def session_leg(B, S, torch, cfg, seed, prof, budget, prompt, decode_steps, decode_mode, db=None, kind=None):
    """The paper's operating mode under ONE budget on ONE stack: the tier table is planned once,
    PickTier chooses the prefill tier for a prompt of `prompt` tokens, the chunked prefill runs (TTFT),
    the one-token tier is installed (SetupForSched: shards that the prefill tier's workspace displaced
    are pinned again from the host images) and `decode_steps` tokens are decoded (TPS)."""
    # the install-time database prices every tier; kind = PS_PLAN_AUTO lets HeuristicSplit plan each tier of up to
    # 64 tokens with a CPU share (prefill then streams through the GPU, decode runs its unpinned FFN on the CPU)
    table = B.TierTable(cfg, int(budget), profile=prof, db=db, kind=kind)
    choice = table.pick(prompt)
    by_rates = B.TierTable(cfg, int(budget), profile=prof, kind=kind).pick(prompt)
    st = B.Stack(table)
    st.set_decode_mode(decode_mode)
    B.load_synthetic([st], cfg, seed, threads=min(16, os.cpu_count() or 8))
    dev = st.device
    x = torch.from_numpy(S.activations(seed, 600, prompt, cfg["hidden"])).to(dev)
    y = torch.empty_like(x)
    xs = [torch.from_numpy(S.activations(seed, 601 + t, 1, cfg["hidden"])).to(dev) for t in range(4)]
    yo = torch.empty_like(xs[0])
    res = []
    for rep in range(3):                      # the first round warms up (graph capture, first touches)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        up_pre = st.set_tier(choice.tier)
        t1 = time.perf_counter()
        trips = B.chunked_forward(st, x, y)
        st.synchronize()
        t2 = time.perf_counter()
        up_dec = st.set_tier(0)
        t3 = time.perf_counter()
        for i in range(decode_steps):
            st.forward(xs[i % 4], yo)
        st.synchronize()
        t4 = time.perf_counter()
        res.append(dict(setup_prefill_ms=(t1 - t0) * 1e3, ttft_ms=(t2 - t1) * 1e3, setup_decode_ms=(t3 - t2) * 1e3,
                        decode_ms_per_token=(t4 - t3) * 1e3 / decode_steps, pinned_again_bytes_prefill=up_pre,
                        pinned_again_bytes_decode=up_dec, trips=trips))
    r = res[-1]
    e_pre, e_dec = table.entry(choice.tier), table.entry(0)
    r.update(budget_bytes=int(budget), prompt_tokens=prompt, picked_tier_tokens=choice.tier_tokens, decode_steps=decode_steps,
             tokens_per_s=1e3 / r["decode_ms_per_token"], est_ttft_ms=choice.est_total_ms, est_decode_ms=e_dec.summary.est_step_ms,
             resident_bytes_prefill_tier=e_pre.summary.resident_bytes, resident_bytes_decode_tier=e_dec.summary.resident_bytes,
             e2el_ms_100_tokens=r["ttft_ms"] + r["setup_decode_ms"] + 100 * r["decode_ms_per_token"],
             estimates="profile database" if db is not None else "profile rates",
             decode_plan=["gpu_only", "static", "dynamic"][e_dec.summary.plan_kind], decode_cpu_bytes=e_dec.summary.cpu_bytes,
             pick_from_profile_rates_alone=dict(tier_tokens=by_rates.tier_tokens, trips=by_rates.iterations, est_ttft_ms=by_rates.est_total_ms))
    log("one stack, budget %.0f GB: PickTier estimate %.1f ms (from the profile's rates alone it picks %d x %d, %.1f ms)" % (
        budget / 1e9, choice.est_total_ms, by_rates.tier_tokens, by_rates.iterations, by_rates.est_total_ms))
    log("one stack, budget %.0f GB: prefill %d tokens in tier %d x %d trips: TTFT %.1f ms; switch to the one-token tier (plan %s) %.2f ms (%.1f MB pinned again); decode %.3f ms/token = %.1f tok/s" % (
        budget / 1e9, prompt, choice.tier_tokens, r["trips"], r["ttft_ms"], r["decode_plan"], r["setup_decode_ms"], r["pinned_again_bytes_decode"] / 1e6,
        r["decode_ms_per_token"], r["tokens_per_s"]))
    st.close()
    return r


def kv_leg(B, S, torch, cfg, seed, prof, context, budgets, steps, decode_mode=1):
    """Decode at a context of `context` cached positions: the KV cache is a shard class of its own
    (pinned after the attention weights, before the FFN), attention is real softmax attention."""
    kcfg = dict(cfg, kv_context=context + 64)
    plans = [B.Plan(kcfg, int(b), 1, profile=prof) for b in budgets]
    tags = ["%g" % (b / 1e9) for b in budgets]
    budgets = list(budgets)
    if prof is not None and prof.cpu_gbps > 0:   # the tightest budget again, planned by HeuristicSplit
        auto = B.Plan(kcfg, int(budgets[-1]), 1, profile=prof, kind=B.PS_PLAN_AUTO)
        if auto.summary().plan_kind != B.PS_PLAN_GPU_ONLY:
            plans.append(auto)
            tags.append("%g_heuristic_split" % (budgets[-1] / 1e9))
            budgets.append(budgets[-1])
    stacks = [B.Stack(p) for p in plans]
    for st in stacks:
        st.set_decode_mode(decode_mode)    # graph replay where everything is resident
    B.load_synthetic(stacks, kcfg, seed, threads=min(16, os.cpu_count() or 8))
    K, V = S.kv_cache(seed, 0, kcfg["n_kv_heads"], context, kcfg["head_dim"])   # same contents in every layer
    for st in stacks:
        for layer in range(kcfg["n_layers"]):
            for g in range(kcfg["n_kv_heads"]):
                st.load_kv(layer, g, K[g], V[g])
    dev = stacks[0].device
    xs = [torch.from_numpy(S.activations(seed, 500 + t, 1, kcfg["hidden"])).to(dev) for t in range(4)]
    xo = torch.empty_like(xs[0])
    kv_bytes_layer = context * kcfg["n_kv_heads"] * kcfg["head_dim"] * 2 * 2
    out = {}
    for b, tag, plan, st in zip(budgets, tags, plans, stacks):
        s = plan.summary()
        st.set_context(context)            # every timed step attends over the same `context` positions
        n = steps if s.streamed_bytes == 0 else max(3, min(steps, 10))
        ms = time_steps(torch, st, xs, xo, n, 2)
        kb, stats = kernel_breakdown(B, st, plan, xs, xo)
        at = kb.get(("kernel", B.PS_K_ATTN))
        kv_res = sum(sh.bytes for sh in plan.shards() if sh.kind == B.PS_SHARD_KV and sh.resident)
        r = dict(budget_bytes=int(b), context=context, ms_per_token=ms, tokens_per_s=1e3 / ms,
                 resident_bytes=s.resident_bytes, kv_cache_bytes=kv_bytes_layer * kcfg["n_layers"],
                 kv_cache_resident_bytes=kv_res, streamed_bytes_per_token=stats.streamed_bytes_step, est_ms=s.est_step_ms,
                 plan=["gpu_only", "static", "dynamic"][s.plan_kind], cpu_bytes_per_token=stats.cpu_bytes_step)
        if at:   # launches of one layer cover all its kv heads when they sit together
            per_layer_ms = at["avg_ms"] * at["launches"] / kcfg["n_layers"]
            r["attn_ms_per_layer"] = per_layer_ms
            r["attn_kv_gbps"] = kv_bytes_layer / (per_layer_ms * 1e-3) / 1e9
            r["attn_frac_of_hbm_peak"] = r["attn_kv_gbps"] / HBM_PEAK_GBS
        out[tag] = r
        log("context %d, budget %.0f GB, plan %s: %.3f ms/token, %.1f tok/s, cache %.2f of %.2f GB pinned, %.2f GB streamed/token, %.2f GB/token on the CPU%s" % (
            context, b / 1e9, r["plan"], ms, 1e3 / ms, kv_res / 1e9, r["kv_cache_bytes"] / 1e9, stats.streamed_bytes_step / 1e9,
            stats.cpu_bytes_step / 1e9,
            (", attention %.1f us/layer = %.0f GB/s" % (r["attn_ms_per_layer"] * 1e3, r["attn_kv_gbps"])) if at else ""))
        st.close()
    return out


def kv_prefill_leg(B, S, torch, cfg, seed, prof, context, prompt, tier_tokens, budget):
    """Chunked prefill OVER a KV cache: `prompt` new tokens at a context of `context` cached positions,
    in chunks of `tier_tokens` (causal attention inside a chunk, rows appended to the cache), then decode
    steps over the filled cache through the same schedule."""
    kcfg = dict(cfg, kv_context=context + prompt + 64)
    plan = B.Plan(kcfg, int(budget), tier_tokens, profile=prof)
    st = B.Stack(plan)
    B.load_synthetic([st], kcfg, seed, threads=min(16, os.cpu_count() or 8))
    K, V = S.kv_cache(seed, 0, kcfg["n_kv_heads"], context, kcfg["head_dim"])
    for layer in range(kcfg["n_layers"]):
        for g in range(kcfg["n_kv_heads"]):
            st.load_kv(layer, g, K[g], V[g])
    dev = st.device
    x = torch.from_numpy(S.activations(seed, 800, prompt, kcfg["hidden"])).to(dev)
    y = torch.empty_like(x)
    xd = torch.from_numpy(S.activations(seed, 801, 1, kcfg["hidden"])).to(dev)
    yd = torch.empty_like(xd)
    times = []
    for rep in range(3):
        st.set_context(context)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        trips = B.chunked_forward(st, x, y)
        st.synchronize()
        times.append((time.perf_counter() - t0) * 1e3)
    t0 = time.perf_counter()
    nd = 8
    for i in range(nd):
        B.chunked_forward(st, xd, yd)
    st.synchronize()
    dec = (time.perf_counter() - t0) * 1e3 / nd
    s = plan.summary()
    r = dict(budget_bytes=int(budget), context=context, prompt_tokens=prompt, chunk_tokens=tier_tokens, trips=trips,
             ttft_ms=min(times[1:]), ms_per_chunk=min(times[1:]) / trips, decode_ms_per_token_in_this_tier=dec,
             resident_bytes=s.resident_bytes, workspace_bytes=s.workspace_bytes, streamed_bytes=s.streamed_bytes,
             kv_cache_bytes=context * kcfg["n_kv_heads"] * kcfg["head_dim"] * 4 * kcfg["n_layers"])
    log("prefill over a cache of %d positions: %d tokens in chunks of %d: %.1f ms (%.2f ms per chunk); decode in the same tier %.2f ms/token" % (
        context, prompt, tier_tokens, r["ttft_ms"], r["ms_per_chunk"], dec))
    st.close()
    return r


def head_leg(B, S, torch, cfg, seed, prof, vocab, budgets, steps):
    """Decode with the output head (final RMSNorm + projection to `vocab` logits, lowest priority
    class): at a budget that holds everything it is one more resident GEMV, at a tight one it is the
    first thing the planner streams."""
    hcfg = dict(cfg, vocab=vocab)
    plans = [B.Plan(hcfg, int(b), 1, profile=prof) for b in budgets]
    stacks = [B.Stack(p) for p in plans]
    B.load_synthetic(stacks, hcfg, seed, threads=min(16, os.cpu_count() or 8))
    dev = stacks[0].device
    xs = [torch.from_numpy(S.activations(seed, 700 + t, 1, hcfg["hidden"])).to(dev) for t in range(4)]
    xo = torch.empty_like(xs[0])
    logits = torch.empty(vocab, dtype=torch.float16, device=dev)
    out = {}
    for b, plan, st in zip(budgets, plans, stacks):
        s = plan.summary()
        st.set_logits_out(logits, 0, 1)
        n = steps if s.streamed_bytes == 0 else max(3, min(steps, 10))
        ms = time_steps(torch, st, xs, xo, n, 2)
        kb, stats = kernel_breakdown(B, st, plan, xs, xo)
        hk = kb[("kernel", B.PS_K_OUT)]
        head_bytes = sum(sh.bytes for sh in plan.shards() if sh.kind == B.PS_SHARD_OUT)
        head_res = sum(sh.bytes for sh in plan.shards() if sh.kind == B.PS_SHARD_OUT and sh.resident)
        head_ms = hk["avg_ms"] * hk["launches"]
        r = dict(budget_bytes=int(b), vocab=vocab, ms_per_token=ms, tokens_per_s=1e3 / ms, head_bytes=head_bytes,
                 head_resident_bytes=head_res, streamed_bytes_per_token=stats.streamed_bytes_step,
                 head_kernel_ms=head_ms, head_launches=hk["launches"], est_ms=s.est_step_ms)
        if head_res == head_bytes:
            r["head_gbps"] = head_bytes / (head_ms * 1e-3) / 1e9
            r["head_frac_of_hbm_peak"] = r["head_gbps"] / HBM_PEAK_GBS
        out["%g" % (b / 1e9)] = r
        log("output head %d, budget %.0f GB: %.3f ms/token, head %.2f of %.2f GB pinned, head kernels %.1f us in %d launches%s, %.2f GB streamed/token" % (
            vocab, b / 1e9, ms, head_res / 1e9, head_bytes / 1e9, head_ms * 1e3, hk["launches"],
            (" = %.0f GB/s" % r["head_gbps"]) if "head_gbps" in r else "", stats.streamed_bytes_step / 1e9))
        st.close()
    return out


def plans_leg(B, S, torch, cfg, seed, prof, budget, tokens, steps):
    """The three schedule plans at one tight budget: all on the GPU through the scratch double buffer,
    unpinned FFN on the CPU, a split of both; and which one HeuristicSplit picks from its estimates."""
    names = {B.PS_PLAN_GPU_ONLY: "gpu_only", B.PS_PLAN_STATIC: "static", B.PS_PLAN_DYNAMIC: "dynamic"}
    out = {}
    # the same three plans priced from a profile database filled by the install-phase benchmark suite
    db = B.ProfileDB()
    t0 = time.perf_counter()
    db.measure(cfg)
    log("profile database: %d entries measured in %.1f s" % (len(db.entries()), time.perf_counter() - t0))
    for M in tokens:
        plans = {k: B.Plan(cfg, int(budget), M, profile=prof, kind=k) for k in names}
        auto = B.Plan(cfg, int(budget), M, profile=prof, kind=B.PS_PLAN_AUTO).summary()
        stacks = {k: B.Stack(p) for k, p in plans.items()}
        B.load_synthetic(list(stacks.values()), cfg, seed, threads=min(16, os.cpu_count() or 8))
        dev = stacks[B.PS_PLAN_GPU_ONLY].device
        xs = [torch.from_numpy(S.activations(seed, 900 + t, M, cfg["hidden"])).to(dev) for t in range(4)]
        xo = torch.empty_like(xs[0])
        auto_db = B.Plan(cfg, int(budget), M, profile=prof, kind=B.PS_PLAN_AUTO, db=db).summary()
        r = dict(budget_bytes=int(budget), tokens=M, picked=names[auto.plan_kind], picked_with_database=names[auto_db.plan_kind],
                 est_ms_with_database={names[k]: auto_db.est_kind_ms[k] for k in names})
        for k, st in stacks.items():
            s = plans[k].summary()
            ms = time_steps(torch, st, xs, xo, steps, 2)
            stats = st.stats()
            r[names[k]] = dict(ms_per_step=ms, tokens_per_s=M * 1e3 / ms, est_ms=s.est_step_ms, resident_bytes=s.resident_bytes,
                               streamed_bytes=s.streamed_bytes, cpu_bytes=s.cpu_bytes, cpu_fraction=s.cpu_fraction,
                               cpu_ms=stats.cpu_ms, cpu_wait_ms=stats.cpu_wait_ms,
                               cpu_gbps=(stats.cpu_bytes_step / (stats.cpu_ms * 1e-3) / 1e9) if stats.cpu_ms else None)
            log("plans at %.0f GB, %d token(s), %s: %.2f ms/step (estimate %.2f), pinned %.2f GB, streamed %.2f GB, on the CPU %.2f GB%s" % (
                budget / 1e9, M, names[k], ms, s.est_step_ms, s.resident_bytes / 1e9, s.streamed_bytes / 1e9, s.cpu_bytes / 1e9,
                (" at %.0f GB/s inside the kernel, %.2f ms waiting for the GPU" % (r[names[k]]["cpu_gbps"], stats.cpu_wait_ms)) if stats.cpu_ms else ""))
            st.close()
        best = min(names.values(), key=lambda n: r[n]["ms_per_step"])
        r["measured_best"] = best
        log("plans at %.0f GB, %d token(s): HeuristicSplit picks %s (priced from the database: %s, estimates %s), measured best %s" % (
            budget / 1e9, M, r["picked"], r["picked_with_database"],
            {n: round(v, 2) for n, v in r["est_ms_with_database"].items()}, best))
        out["%d" % M] = r
    return out


def measured_traffic(tag):
    """HBM bytes per launch of the named kernel from the committed rocprofv3 PMC summary
    (profiles/dense8b_decode_prefill_pmc_hbm_traffic.txt); None if the summary is absent."""
    path = os.path.join(ROOT, "profiles", "dense8b_decode_prefill_pmc_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch %s:" % tag):
                return int(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--layers", type=int, default=32, help="layers of the 8B-shaped stack (32 = the named config)")
    ap.add_argument("--budgets-gb", type=str, default="4,2,8", help="first one is the headline")
    ap.add_argument("--prefill-tokens", type=int, default=2048, help="0 skips the TTFT leg")
    ap.add_argument("--cpu-layers", type=int, default=32, help="layers the oracle baseline runs, 0 skips")
    ap.add_argument("--cpu-reps", type=int, default=4, help="tokens the oracle baseline runs")
    ap.add_argument("--extra", type=str, default="batch64,moe,tiers,session,kv,head,plans",
                    help="further legs: batch64 (config 5, plus 4 and 16 tokens), moe (config 4, with the hot-expert variant), tiers (tier table + chunked prefill at 2 GB), "
                         "session (prefill then decode on one stack: tier table, PickTier, tier switch), "
                         "kv (decode over a 16K-position KV cache), head (decode with a 128256-row output head), "
                         "plans (GPU-only / static / dynamic plan and HeuristicSplit's pick at 2 GB)")
    ap.add_argument("--measure-profile", type=int, default=1)
    ap.add_argument("--calibrate-copy", type=int, default=0,
                    help="also run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--decode-mode", type=int, default=1,
                    help="0 launch per shard, 1 HIP-graph replay where every shard is resident (others fall back to 0)")
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

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    prof = None
    if args.measure_profile:
        prof = B.profile_measure(1 << 30)
        log("profile: h2d %.1f GB/s, gemv %.0f GB/s, launch %.2f us, gemm TFLOP/s %s" % (
            prof.h2d_gbps, prof.gemv_gbps, prof.launch_us, ["%.0f" % v for v in prof.gemm_tflops]))
        log("profile, CPU back-end: %.0f GB/s alone, %.0f GB/s beside H2D copies (which then run at %.1f GB/s), memory-bound up to %.1f tokens, %.0f us per CPU shard" % (
            prof.cpu_gbps, prof.cpu_gbps_busy, prof.h2d_gbps_busy, prof.cpu_tokens_free, prof.cpu_sync_us))

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

    # which of the cycled activation draws keep the fp16 residual stream finite through all layers (the
    # prescribed weights have a non-zero mean; the others end in inf/NaN rows, on the GPU as in the oracle)
    finite_draws = []
    for i, x in enumerate(xs):
        stacks[0].forward(x, xout)
        stacks[0].synchronize()
        if bool(torch.isfinite(xout).all().item()):
            finite_draws.append(i)
    head = results["%g" % (budgets[0] / 1e9)]
    # dominant kernel of the headline run: the fused gate/up + SwiGLU GEMV (54% of the bytes)
    gu = head["kernels"].get("kernel_%d" % B.PS_K_GATE_UP)
    roof = None
    if gu:
        # the kernel's own launch duration: its 32 launches (one per layer, different weights each) back
        # to back between two events, so the event bracket's dispatch gap is amortised away
        iso_ms, iso_n = stacks[0].time_kernel(B.PS_K_GATE_UP, 10)
        gu = dict(gu, avg_ms=iso_ms, bracketed_avg_ms=gu["avg_ms"])
        ach = gu["bytes_per_launch"] / (gu["avg_ms"] * 1e-3) / 1e9
        ach_in_step = gu["bytes_per_launch"] / (gu["bracketed_avg_ms"] * 1e-3) / 1e9
        roof = dict(bound="hbm", kernel="gemv_w4_kernel<GATE_UP>", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=ach / HBM_PEAK_GBS, traffic=measured_traffic("gemv_gate_up"),
                    traffic_source="profiles/dense8b_decode_prefill_pmc_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                   "command, committed with the kernels they measure; not re-measured in this run)",
                    bytes_per_launch=gu["bytes_per_launch"],
                    # two timings of the same launches: `frac` uses the kernel's 32 launches (one per layer)
                    # back to back between two events; the in-step figure brackets each launch inside a
                    # whole forward and includes the gap to its neighbours
                    avg_launch_us=gu["avg_ms"] * 1e3, timing="32 launches back to back between two HIP events on the compute stream",
                    bracketed_launch_us=gu["bracketed_avg_ms"] * 1e3, achieved_in_step=ach_in_step,
                    frac_in_step=ach_in_step / HBM_PEAK_GBS,
                    whole_step_frac=head.get("frac_of_hbm_peak"))

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

    for st in stacks:
        st.close()
    extra = {}
    # each leg starts from memory handed back to the driver: an arena carved out of blocks the caching
    # allocator kept from earlier legs measured up to 9 % slower on the 8 GB stacks
    import gc

    def fresh():
        gc.collect()
        torch.cuda.empty_cache()
    fresh()
    if "batch64" in args.extra and args.layers == 32:
        extra["batched_decode_64"] = batched_leg(B, S, torch, cfg, seed, prof, 64, [4e9, 12e9], 128, args.decode_mode)
        fresh()
        # the other batch sizes of the paper's batching table (1 is the headline leg)
        extra["batched_decode_4"] = batched_leg(B, S, torch, cfg, seed, prof, 4, [4e9], 128, args.decode_mode)
        fresh()
        extra["batched_decode_16"] = batched_leg(B, S, torch, cfg, seed, prof, 16, [4e9], 128, args.decode_mode)
    fresh()
    tier_db = None
    if ("tiers" in args.extra or "session" in args.extra) and args.layers == 32:
        tier_db = B.ProfileDB()      # the install phase's benchmark suite: every matrix of the model at every tier
        tier_db.measure(cfg)
    if "tiers" in args.extra and args.layers == 32:
        extra["chunked_prefill_2gb"] = tier_leg(B, S, torch, cfg, seed, prof, 2e9, 2048, db=tier_db)
    fresh()
    if "session" in args.extra and args.layers == 32:
        extra["prefill_then_decode_one_stack"] = {"%g" % (b / 1e9): session_leg(B, S, torch, cfg, seed, prof, b, 2048, 64 if b > 3e9 else 8, args.decode_mode, db=tier_db)
                                                  for b in (4e9, 2e9)}
        if prof is not None and prof.cpu_gbps > 0:   # the same at 2 GB with HeuristicSplit planning the low tiers
            extra["prefill_then_decode_one_stack"]["2_heuristic_split"] = session_leg(B, S, torch, cfg, seed, prof, 2e9, 2048, 16, args.decode_mode,
                                                                                      db=tier_db, kind=B.PS_PLAN_AUTO)
    fresh()
    if "kv" in args.extra and args.layers == 32:
        extra["decode_context_16k"] = kv_leg(B, S, torch, cfg, seed, prof, 16384, [8e9, 4e9], 50, args.decode_mode)
    fresh()
    if "kv" in args.extra and args.layers == 32:
        extra["prefill_over_cache_4k"] = {"chunks_of_64": kv_prefill_leg(B, S, torch, cfg, seed, prof, 4096, 256, 64, 8e9)}
        fresh()
        extra["prefill_over_cache_4k"]["chunks_of_512"] = kv_prefill_leg(B, S, torch, cfg, seed, prof, 4096, 1024, 512, 8e9)
    fresh()
    if "head" in args.extra and args.layers == 32:
        extra["decode_output_head_128k"] = head_leg(B, S, torch, cfg, seed, prof, 128256, [8e9, 4e9], 100)
    fresh()
    if "plans" in args.extra and args.layers == 32 and prof is not None and prof.cpu_gbps > 0:
        extra["schedule_plans_2gb"] = plans_leg(B, S, torch, cfg, seed, prof, 2e9, [1, 16], 8)
    fresh()
    if "moe" in args.extra:
        extra["moe_decode_6gb"] = moe_leg(B, S, torch, seed, prof, 6e9, [1, 16], 10)

    cpu = None
    if args.cpu_layers:
        from oracle import oracle as O
        dt, cores = cpu_baseline(cfg, seed, min(args.cpu_layers, cfg["n_layers"]), args.cpu_reps, S, O)
        nl = min(args.cpu_layers, cfg["n_layers"])
        cpu = dict(value=1.0 / (dt * cfg["n_layers"] / nl), unit="tokens/s", cores=cores, kind="oracle",
                   sample="%d of %d layers of the same stack, %d tokens one after the other, %.2f s per token" % (
                       nl, cfg["n_layers"], args.cpu_reps, dt))

    line = dict(metric="decode tokens/s at fixed VRAM budget (batch 1)", value=head["tokens_per_s"], unit="tokens/s",
                n_gpus=1, steps=head["steps"], warmup=args.warmup, ms_per_step=head["ms_per_token"],
                higher_is_better=True, scaling="weak", vs_baseline=None, dtype="f16",
                data="synthetic",
                config=dict(workload="dense 8B-shaped stack, %d layers, decode batch 1, budget %g GB" % (
                    cfg["n_layers"], budgets[0] / 1e9), hidden=4096, ffn=14336, weight_bytes=plans[0].summary().weight_bytes,
                    decode_mode="hip graph replay of the resident forward" if args.decode_mode == 1 else "one launch per shard",
                    activation_draws=len(xs), finite_activation_draws=finite_draws),
                roofline=roof, cpu_baseline=cpu, budgets=results, prefill=prefill, extra=extra,
                profile=None if prof is None else dict(h2d_gbps=prof.h2d_gbps, gemv_gbps=prof.gemv_gbps,
                                                       launch_us=prof.launch_us, gemm_tflops=list(prof.gemm_tflops),
                                                       cpu_gbps=prof.cpu_gbps, cpu_gbps_busy=prof.cpu_gbps_busy,
                                                       h2d_gbps_busy=prof.h2d_gbps_busy, cpu_tokens_free=prof.cpu_tokens_free,
                                                       cpu_sync_us=prof.cpu_sync_us))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
