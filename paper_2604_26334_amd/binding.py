"""ctypes binding of libpshard.so: same names as include/pshard.h (and include/pshard_test.h for the
test-only entry points), argument marshalling only.

The library must have been built (python -m paper_2604_26334_amd.build, or
__graft_entry__.build()); loading fails loudly otherwise -- there is no CPU fallback.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("PS_LIB", os.path.join(_HERE, "libpshard.so"))

PS_OK, PS_E_ARG, PS_E_BUDGET, PS_E_HIP, PS_E_STATE, PS_E_NOMEM = 0, -1, -2, -3, -4, -5
PS_MAT_QKV, PS_MAT_O, PS_MAT_GATE, PS_MAT_UP, PS_MAT_DOWN, PS_MAT_OUT = 0, 1, 2, 3, 4, 5
PS_SHARD_QKV, PS_SHARD_O, PS_SHARD_GATE_UP, PS_SHARD_DOWN, PS_SHARD_EXPERT, PS_SHARD_KV, PS_SHARD_OUT = 0, 1, 2, 3, 4, 5, 6
PS_CLASS_ATTN, PS_CLASS_KVCACHE, PS_CLASS_FFN, PS_CLASS_OUTS = 0, 1, 2, 3
PS_FLAG_NO_ATTN, PS_FLAG_NO_RESIDUAL = 1, 2
PS_PLAN_GPU_ONLY, PS_PLAN_STATIC, PS_PLAN_DYNAMIC, PS_PLAN_AUTO = 0, 1, 2, 3
PS_OP_COPY, PS_OP_KERNEL, PS_OP_CPU, PS_OP_FETCH = 0, 1, 2, 3
PS_BUF_H, PS_BUF_S, PS_BUF_X = 1, 2, 4
PS_OPK_GEMV, PS_OPK_GEMM, PS_OPK_CPU, PS_OPK_H2D = 0, 1, 2, 3
PS_MATCH_NONE, PS_MATCH_EXACT, PS_MATCH_NEIGHBOUR = 0, 1, 2
PS_NTIERS = 11
(PS_K_RINV, PS_K_QKV, PS_K_O, PS_K_GATE_UP, PS_K_DOWN, PS_K_ROUTE, PS_K_EXPERT_GATE_UP,
 PS_K_EXPERT_DOWN, PS_K_COMBINE, PS_K_ATTN, PS_K_ATTN_COMBINE, PS_K_OUT) = range(12)
(PS_OPF_WAIT_SLOT_FREE, PS_OPF_WAIT_ROUTER, PS_OPF_RECORD_READY, PS_OPF_WAIT_READY,
 PS_OPF_RECORD_FREE, PS_OPF_RECORD_ROUTER) = 1, 2, 4, 8, 16, 32
NO_EXPERT = 0xFFFFFFFF


class ps_model_desc(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim",
                                          "ffn_inter", "n_experts", "top_k", "expert_inter", "flags")] + \
               [("rms_eps", C.c_float), ("kv_context", C.c_uint32), ("vocab", C.c_uint32)]


class ps_profile(C.Structure):
    _fields_ = [("h2d_gbps", C.c_double), ("gemv_gbps", C.c_double),
                ("gemm_tflops", C.c_double * PS_NTIERS), ("launch_us", C.c_double)] + \
               [(n, C.c_double) for n in ("cpu_gbps", "cpu_gbps_busy", "h2d_gbps_busy", "cpu_tokens_free", "cpu_sync_us")]


class ps_shard_info(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("layer", "kind", "expert", "cls", "tile0", "ntiles", "resident",
                                          "priority_rank")] + [("bytes", C.c_uint64), ("offset", C.c_uint64)]


class ps_plan_summary_t(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("budget_bytes", "weight_bytes", "resident_bytes", "streamed_bytes",
                                          "scratch_bytes", "workspace_bytes", "slot_bytes")] + \
               [(n, C.c_uint32) for n in ("n_slots", "n_shards", "n_tokens", "tier")] + \
               [("est_step_ms", C.c_double), ("est_streamed_bytes_per_step", C.c_double),
                ("cpu_bytes", C.c_uint64), ("plan_kind", C.c_uint32), ("pad", C.c_uint32),
                ("cpu_fraction", C.c_double), ("est_kind_ms", C.c_double * 3)]


class ps_prof_entry(C.Structure):
    _fields_ = [("op", C.c_uint32), ("quant", C.c_uint32), ("threads", C.c_uint32), ("pad", C.c_uint32),
                ("n", C.c_uint64), ("k", C.c_uint64), ("m", C.c_uint64), ("ms", C.c_double)]


class ps_prof_estimate(C.Structure):
    _fields_ = [("ms", C.c_double), ("flops", C.c_double), ("bytes", C.c_double), ("match", C.c_uint32),
                ("compute_bound", C.c_uint32), ("neighbour", C.c_int32), ("pad", C.c_uint32)]


class ps_tier_entry(C.Structure):
    _fields_ = [("tier", C.c_uint32), ("tier_tokens", C.c_uint32), ("feasible", C.c_int32), ("pad", C.c_uint32),
                ("summary", ps_plan_summary_t)]


class ps_tier_choice(C.Structure):
    _fields_ = [("tier", C.c_uint32), ("tier_tokens", C.c_uint32), ("iterations", C.c_uint32), ("pad", C.c_uint32),
                ("est_iter_ms", C.c_double), ("est_total_ms", C.c_double)]


class ps_stats(C.Structure):
    _fields_ = [("resident_bytes_step", C.c_uint64), ("streamed_bytes_step", C.c_uint64),
                ("n_copies", C.c_uint32), ("n_kernels", C.c_uint32)] + \
               [(n, C.c_double) for n in ("copy_ms", "compute_ms", "wall_ms", "overlap", "h2d_gbps")] + \
               [("cpu_bytes_step", C.c_uint64), ("cpu_ms", C.c_double), ("cpu_wait_ms", C.c_double),
                ("graph_replay", C.c_uint32), ("reserved", C.c_uint32)]


class ps_op_info(C.Structure):
    _fields_ = [("type", C.c_uint32), ("kernel", C.c_uint32), ("layer", C.c_uint32), ("flags", C.c_uint32),
                ("slot", C.c_int32), ("shard0", C.c_uint32), ("nshards", C.c_uint32), ("buffers", C.c_uint32),
                ("slot_offset", C.c_uint64), ("bytes", C.c_uint64)]


EXPORTS = ["ps_stack_create_tiers", "ps_stack_set_tier", "ps_stack_tier", "ps_stack_forward_noalloc", "ps_plan_num_shards", "ps_stack_forward_chunked", "ps_last_error", "ps_tier_tokens", "ps_tier_for_tokens", "ps_packed_bytes", "ps_plan_create",
           "ps_plan_summary", "ps_plan_get_shard", "ps_plan_destroy", "ps_schedule_create",
           "ps_schedule_num_ops", "ps_schedule_get_op", "ps_schedule_validate", "ps_schedule_destroy",
           "ps_route_host", "ps_profile_measure", "ps_stack_create", "ps_stack_load_matrix",
           "ps_stack_forward", "ps_stack_set_decode_mode", "ps_stack_set_copy_mode", "ps_stack_sync_check", "ps_stack_set_profiling", "ps_stack_stats", "ps_stack_op_time", "ps_stack_time_kernel", "ps_stack_debug_buffer",
           "ps_stack_destroy", "ps_mfma_probe", "ps_lds_tr_probe", "ps_pack_matrix", "ps_tier_table_create", "ps_tier_table_entry",
           "ps_tier_table_plan", "ps_tier_pick", "ps_tier_table_destroy", "ps_stack_load_kv", "ps_stack_set_context",
           "ps_stack_set_logits_out", "ps_cpu_matmul", "ps_plan_create_kind", "ps_stack_set_cpu_threads",
           "ps_tier_table_create_kind", "ps_tier_table_create_db", "ps_profile_db_create", "ps_profile_db_destroy", "ps_profile_db_add",
           "ps_profile_db_count", "ps_profile_db_get", "ps_profile_db_estimate", "ps_profile_db_save",
           "ps_profile_db_load", "ps_profile_db_measure", "ps_plan_create_db"]

_lib = None


def lib():
    """Load libpshard.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libpshard.so is not built: run `python -m paper_2604_26334_amd.build`")
        # torch ships its own HIP runtime; it must be in the process before libpshard.so so
        # that both resolve libamdhip64 to the same loaded copy (two runtimes cannot share a GPU)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, u32, u64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int32
        L.ps_last_error.restype = C.c_char_p
        L.ps_last_error.argtypes = []
        L.ps_tier_tokens.restype = u32
        L.ps_tier_tokens.argtypes = [u32]
        L.ps_tier_for_tokens.restype = u32
        L.ps_tier_for_tokens.argtypes = [u32]
        L.ps_packed_bytes.restype = u64
        L.ps_packed_bytes.argtypes = [u32, u32]
        sig = {
            "ps_plan_create": [C.POINTER(ps_model_desc), u64, C.POINTER(ps_profile), u32, vp, C.POINTER(vp)],
            "ps_plan_create_kind": [C.POINTER(ps_model_desc), u64, C.POINTER(ps_profile), u32, vp, u32, C.POINTER(vp)],
            "ps_stack_set_cpu_threads": [vp, u32],
            "ps_plan_summary": [vp, C.POINTER(ps_plan_summary_t)],
            "ps_plan_get_shard": [vp, u32, C.POINTER(ps_shard_info)],
            "ps_plan_num_shards": [vp, C.POINTER(u32)],
            "ps_stack_forward_chunked": [vp, vp, vp, u32, vp, vp, vp, C.POINTER(u32)],
            "ps_schedule_create": [vp, vp, C.POINTER(vp)],
            "ps_schedule_num_ops": [vp, C.POINTER(u32)],
            "ps_schedule_get_op": [vp, u32, C.POINTER(ps_op_info)],
            "ps_schedule_validate": [vp],
            "ps_route_host": [vp, u32, u32, u32, vp],
            "ps_profile_measure": [vp, u64, vp, vp, C.POINTER(ps_profile)],
            "ps_stack_create": [vp, vp, u64, vp, vp, C.POINTER(vp)],
            "ps_stack_load_matrix": [vp, u32, u32, u32, vp, vp],
            "ps_stack_forward": [vp, vp, vp, vp, vp],
            "ps_stack_forward_noalloc": [vp, vp, vp],
            "ps_stack_create_tiers": [vp, vp, u64, vp, vp, C.POINTER(vp)],
            "ps_stack_set_tier": [vp, u32, C.POINTER(u64)],
            "ps_stack_tier": [vp, C.POINTER(u32), C.POINTER(u32)],
            "ps_stack_set_profiling": [vp, i32],
            "ps_stack_set_decode_mode": [vp, i32],
            "ps_stack_sync_check": [vp],
            "ps_stack_set_copy_mode": [vp, i32],
            "ps_stack_stats": [vp, C.POINTER(ps_stats)],
            "ps_stack_op_time": [vp, u32, C.POINTER(C.c_double), C.POINTER(C.c_double)],
            "ps_stack_time_kernel": [vp, u32, u32, C.POINTER(C.c_double), C.POINTER(u32)],
            "ps_stack_debug_buffer": [vp, u32, C.POINTER(vp), C.POINTER(u64)],
            "ps_mfma_probe": [i32, i32, i32, vp, vp],
            "ps_lds_tr_probe": [vp, vp, vp],
            "ps_pack_matrix": [vp, vp, u32, u32, vp],
            "ps_tier_table_create": [C.POINTER(ps_model_desc), u64, C.POINTER(ps_profile), vp, C.POINTER(vp)],
            "ps_tier_table_create_kind": [C.POINTER(ps_model_desc), u64, C.POINTER(ps_profile), vp, u32, C.POINTER(vp)],
            "ps_tier_table_create_db": [C.POINTER(ps_model_desc), u64, C.POINTER(ps_profile), vp, vp, u32, C.POINTER(vp)],
            "ps_tier_table_entry": [vp, u32, C.POINTER(ps_tier_entry)],
            "ps_profile_db_create": [C.POINTER(vp)],
            "ps_profile_db_add": [vp, C.POINTER(ps_prof_entry)],
            "ps_profile_db_count": [vp, C.POINTER(u32)],
            "ps_profile_db_get": [vp, u32, C.POINTER(ps_prof_entry)],
            "ps_profile_db_estimate": [vp, C.c_double, u32, u32, u32, u64, u64, u64, C.POINTER(ps_prof_estimate)],
            "ps_profile_db_save": [vp, C.c_char_p],
            "ps_profile_db_load": [vp, C.c_char_p],
            "ps_profile_db_measure": [vp, C.POINTER(ps_model_desc), vp, u64, vp, vp],
            "ps_plan_create_db": [C.POINTER(ps_model_desc), u64, C.POINTER(ps_profile), vp, u32, vp, u32, C.POINTER(vp)],
            "ps_tier_table_plan": [vp, u32, C.POINTER(vp)],
            "ps_tier_pick": [vp, u32, C.POINTER(ps_tier_choice)],
            "ps_stack_load_kv": [vp, u32, u32, vp, vp, u32],
            "ps_stack_set_context": [vp, u32],
            "ps_stack_set_logits_out": [vp, vp, u32, u32],
            "ps_cpu_matmul": [vp, u32, u32, i32, vp, u32, C.c_float, vp, vp, u32],
        }
        for name, args in sig.items():
            f = getattr(L, name)
            f.restype = i32
            f.argtypes = args
        for name in ("ps_plan_destroy", "ps_schedule_destroy", "ps_stack_destroy", "ps_tier_table_destroy", "ps_profile_db_destroy"):
            f = getattr(L, name)
            f.restype = None
            f.argtypes = [vp]
        _lib = L
    return _lib


class PshardError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("pshard error %d: %s" % (code, text))
        self.code = code


def _check(rc):
    if rc != PS_OK:
        raise PshardError(rc, lib().ps_last_error().decode())


def model_desc(cfg):
    """ps_model_desc from a config dict (keys as in synth_inputs.cfg_*)."""
    flags = (PS_FLAG_NO_ATTN if cfg.get("no_attn") else 0) | (PS_FLAG_NO_RESIDUAL if cfg.get("no_residual") else 0)
    return ps_model_desc(cfg["n_layers"], cfg["hidden"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                         cfg["ffn_inter"], cfg["n_experts"], cfg["top_k"], cfg["expert_inter"], flags,
                         cfg["rms_eps"], int(cfg.get("kv_context", 0)), int(cfg.get("vocab", 0)))


def make_profile(h2d_gbps=55.0, gemv_gbps=4000.0, gemm_tflops=400.0, launch_us=3.0, cpu_gbps=0.0,
                 cpu_gbps_busy=0.0, h2d_gbps_busy=0.0, cpu_tokens_free=4.0, cpu_sync_us=30.0):
    p = ps_profile()
    p.h2d_gbps, p.gemv_gbps, p.launch_us = h2d_gbps, gemv_gbps, launch_us
    p.cpu_gbps, p.cpu_gbps_busy, p.h2d_gbps_busy = cpu_gbps, cpu_gbps_busy, h2d_gbps_busy
    p.cpu_tokens_free, p.cpu_sync_us = cpu_tokens_free, cpu_sync_us
    for t in range(PS_NTIERS):
        p.gemm_tflops[t] = gemm_tflops[t] if hasattr(gemm_tflops, "__len__") else gemm_tflops
    return p


def _ptr(a):
    if a is None:
        return None
    return a.ctypes.data_as(C.c_void_p)


class Plan:
    """ps_plan_create / ps_plan_summary / ps_plan_get_shard / ps_plan_destroy."""

    def __init__(self, cfg, budget_bytes, n_tokens, profile=None, expert_freq=None, kind=None, db=None):
        """kind: None (ps_plan_create: Plan One) or PS_PLAN_* (ps_plan_create_kind); db: a ProfileDB whose
        entries price the shards (ps_plan_create_db)."""
        self.cfg = cfg
        self.desc = model_desc(cfg)
        self.profile = profile if profile is not None else make_profile()
        self.h = C.c_void_p()
        freq = None if expert_freq is None else np.ascontiguousarray(expert_freq, dtype=np.float32)
        if db is not None:
            _check(lib().ps_plan_create_db(C.byref(self.desc), int(budget_bytes), C.byref(self.profile), db.h,
                                           int(n_tokens), _ptr(freq), int(kind or 0), C.byref(self.h)))
        elif kind is None:
            _check(lib().ps_plan_create(C.byref(self.desc), int(budget_bytes), C.byref(self.profile), int(n_tokens),
                                        _ptr(freq), C.byref(self.h)))
        else:
            _check(lib().ps_plan_create_kind(C.byref(self.desc), int(budget_bytes), C.byref(self.profile),
                                             int(n_tokens), _ptr(freq), int(kind), C.byref(self.h)))

    def summary(self):
        s = ps_plan_summary_t()
        _check(lib().ps_plan_summary(self.h, C.byref(s)))
        return s

    def shards(self):
        n = C.c_uint32()
        _check(lib().ps_plan_num_shards(self.h, C.byref(n)))
        out = []
        for i in range(n.value):
            s = ps_shard_info()
            _check(lib().ps_plan_get_shard(self.h, i, C.byref(s)))
            out.append(s)
        return out

    def schedule(self, router_logits=None):
        return Schedule(self, router_logits)

    def close(self):
        if self.h:
            lib().ps_plan_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Schedule:
    """ps_schedule_create / ps_schedule_get_op / ps_schedule_validate."""

    def __init__(self, plan, router_logits=None):
        self.h = C.c_void_p()
        lg = None if router_logits is None else np.ascontiguousarray(router_logits, dtype=np.float32)
        _check(lib().ps_schedule_create(plan.h, _ptr(lg), C.byref(self.h)))

    def ops(self):
        n = C.c_uint32()
        _check(lib().ps_schedule_num_ops(self.h, C.byref(n)))
        out = []
        for i in range(n.value):
            o = ps_op_info()
            _check(lib().ps_schedule_get_op(self.h, i, C.byref(o)))
            out.append(o)
        return out

    def validate(self):
        _check(lib().ps_schedule_validate(self.h))

    def __del__(self):
        try:
            if self.h:
                lib().ps_schedule_destroy(self.h)
        except Exception:
            pass


def pack_matrix(scales, codes):
    s = np.ascontiguousarray(scales)
    c = np.ascontiguousarray(codes)
    assert s.dtype == np.float16 and c.dtype == np.uint8
    rows, K = c.shape
    out = np.empty(lib().ps_packed_bytes(rows, K), dtype=np.uint8)
    _check(lib().ps_pack_matrix(_ptr(s), _ptr(c), rows, K, _ptr(out)))
    return out


def route_host(logits, top_k):
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    M, E = lg.shape
    idx = np.empty((M, top_k), dtype=np.int32)
    _check(lib().ps_route_host(_ptr(lg), M, E, top_k, _ptr(idx)))
    return idx


class _TierPlan(Plan):
    """A plan owned by a tier table: same queries as Plan, never destroyed from here."""

    def __init__(self, table, handle):
        self.cfg, self.desc, self.profile = table.cfg, table.desc, table.profile
        self.h = handle
        self._table = table   # keeps the owner alive

    def close(self):
        self.h = C.c_void_p()


class ProfileDB:
    """ps_profile_db_*: benchmarked kernels and the paper's look-up rule (exact, nearest neighbour, skip)."""

    def __init__(self):
        self.h = C.c_void_p()
        _check(lib().ps_profile_db_create(C.byref(self.h)))

    def add(self, op, quant, threads, n, k, m, ms):
        e = ps_prof_entry(op, quant, threads, 0, n, k, m, ms)
        _check(lib().ps_profile_db_add(self.h, C.byref(e)))

    def entries(self):
        n = C.c_uint32()
        _check(lib().ps_profile_db_count(self.h, C.byref(n)))
        out = []
        for i in range(n.value):
            e = ps_prof_entry()
            _check(lib().ps_profile_db_get(self.h, i, C.byref(e)))
            out.append((e.op, e.quant, e.threads, e.n, e.k, e.m, e.ms))
        return out

    def estimate(self, bandwidth_gbps, op, quant, threads, n, k, m):
        r = ps_prof_estimate()
        _check(lib().ps_profile_db_estimate(self.h, float(bandwidth_gbps), op, quant, threads, n, k, m, C.byref(r)))
        return r

    def save(self, path):
        _check(lib().ps_profile_db_save(self.h, str(path).encode()))

    def load(self, path):
        _check(lib().ps_profile_db_load(self.h, str(path).encode()))

    def measure(self, cfg, scratch_bytes=1 << 30, device="cuda:0"):
        """Run the benchmark suite for cfg on the device (allocates a torch scratch buffer and two streams)."""
        import torch
        dev = torch.device(device)
        desc = model_desc(cfg)
        with torch.cuda.device(dev):
            scratch = torch.empty(int(scratch_bytes), dtype=torch.uint8, device=dev)
            cs, cp = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
            torch.cuda.synchronize()
            _check(lib().ps_profile_db_measure(self.h, C.byref(desc), scratch.data_ptr(), scratch.numel(),
                                               cs.cuda_stream, cp.cuda_stream))
            torch.cuda.synchronize()
        del scratch

    def close(self):
        if self.h:
            lib().ps_profile_db_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class TierTable:
    """ps_tier_table_*: one plan per token tier under one budget, and PickTier."""

    def __init__(self, cfg, budget_bytes, profile=None, expert_freq=None, kind=None, db=None):
        self.cfg = cfg
        self.desc = model_desc(cfg)
        self.profile = profile if profile is not None else make_profile()
        self.h = C.c_void_p()
        freq = None if expert_freq is None else np.ascontiguousarray(expert_freq, dtype=np.float32)
        if db is not None:
            _check(lib().ps_tier_table_create_db(C.byref(self.desc), int(budget_bytes), C.byref(self.profile), db.h, _ptr(freq),
                                                 PS_PLAN_GPU_ONLY if kind is None else int(kind), C.byref(self.h)))
        elif kind is None:
            _check(lib().ps_tier_table_create(C.byref(self.desc), int(budget_bytes), C.byref(self.profile), _ptr(freq),
                                              C.byref(self.h)))
        else:
            _check(lib().ps_tier_table_create_kind(C.byref(self.desc), int(budget_bytes), C.byref(self.profile),
                                                   _ptr(freq), int(kind), C.byref(self.h)))

    def entry(self, tier):
        e = ps_tier_entry()
        _check(lib().ps_tier_table_entry(self.h, int(tier), C.byref(e)))
        return e

    def entries(self):
        return [self.entry(t) for t in range(PS_NTIERS)]

    def plan(self, tier):
        h = C.c_void_p()
        _check(lib().ps_tier_table_plan(self.h, int(tier), C.byref(h)))
        return _TierPlan(self, h)

    def pick(self, new_tokens):
        c = ps_tier_choice()
        _check(lib().ps_tier_pick(self.h, int(new_tokens), C.byref(c)))
        return c

    def close(self):
        if self.h:
            lib().ps_tier_table_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def chunked_forward(stack, x_in, x_out, router_logits=None, logits_out=None, router_logits_dev=None):
    """ps_stack_forward_chunked: n = x_in.shape[0] tokens through a stack planned for T = stack.M tokens
    in ceil(n / T) trips (chunked prefill with the tier size as chunk size).  logits_out (fp16 [vocab],
    models with an output head): the head runs on the last trip only, for the last token.
    Asynchronous on stack.compute like Stack.forward; returns the number of trips."""
    n = int(x_in.shape[0])
    assert x_in.dtype == stack.torch.float16 and x_out.dtype == stack.torch.float16
    assert x_in.is_contiguous() and x_out.is_contiguous()
    assert tuple(x_in.shape) == (n, stack.H) and tuple(x_out.shape) == (n, stack.H)
    lg = None if router_logits is None else np.ascontiguousarray(router_logits, dtype=np.float32)
    if lg is not None:
        assert lg.shape[1] == n
    if logits_out is not None:
        assert logits_out.dtype == stack.torch.float16 and logits_out.is_contiguous()
        assert logits_out.numel() == stack.plan.cfg["vocab"]
    trips = C.c_uint32()
    with stack.torch.cuda.device(stack.device):
        _check(lib().ps_stack_forward_chunked(stack.h, x_in.data_ptr(), x_out.data_ptr(), n, _ptr(lg),
                                              None if router_logits_dev is None else router_logits_dev.data_ptr(),
                                              None if logits_out is None else logits_out.data_ptr(), C.byref(trips)))
    return trips.value


class Stack:
    """ps_stack_*: binds a plan to a torch-owned VRAM arena and two torch streams."""

    def __init__(self, plan, device="cuda:0"):
        """plan: a Plan (ps_stack_create), or a TierTable (ps_stack_create_tiers: every feasible tier of
        the table on one arena; the lowest feasible tier is installed, set_tier installs another)."""
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.table = plan if isinstance(plan, TierTable) else None
        if self.table is not None:
            plan = self.table.plan(next(t for t in range(PS_NTIERS) if self.table.entry(t).feasible))
        self.plan = plan
        s = plan.summary()
        self.M = s.n_tokens
        self.H = plan.cfg["hidden"]
        self.arena = torch.empty(int(s.budget_bytes), dtype=torch.uint8, device=self.device)
        self.compute = torch.cuda.Stream(device=self.device)
        self.copy = torch.cuda.Stream(device=self.device)
        self.h = C.c_void_p()
        with torch.cuda.device(self.device):
            if self.table is not None:
                _check(lib().ps_stack_create_tiers(self.table.h, self.arena.data_ptr(), self.arena.numel(),
                                                   self.compute.cuda_stream, self.copy.cuda_stream, C.byref(self.h)))
            else:
                _check(lib().ps_stack_create(plan.h, self.arena.data_ptr(), self.arena.numel(),
                                             self.compute.cuda_stream, self.copy.cuda_stream, C.byref(self.h)))

    def set_tier(self, tier):
        """ps_stack_set_tier: install another tier's schedule; returns the bytes pinned again from the host."""
        up = C.c_uint64()
        with self.torch.cuda.device(self.device):
            _check(lib().ps_stack_set_tier(self.h, int(tier), C.byref(up)))
        self.plan = self.table.plan(tier)
        self.M = self.plan.summary().n_tokens
        return up.value

    def tier(self):
        t, n = C.c_uint32(), C.c_uint32()
        _check(lib().ps_stack_tier(self.h, C.byref(t), C.byref(n)))
        return t.value, n.value

    def load_matrix(self, layer, mat, expert, scales, codes):
        s = np.ascontiguousarray(scales)
        c = np.ascontiguousarray(codes)
        assert s.dtype == np.float16 and c.dtype == np.uint8
        e = NO_EXPERT if expert is None else int(expert)
        with self.torch.cuda.device(self.device):
            _check(lib().ps_stack_load_matrix(self.h, layer, mat, e, _ptr(s), _ptr(c)))

    def load_kv(self, layer, kv_head, K, V):
        """K, V: float16 [n_pos][head_dim] rows of one kv head's cache (positions 0 .. n_pos - 1)."""
        k = np.ascontiguousarray(K, dtype=np.float16)
        v = np.ascontiguousarray(V, dtype=np.float16)
        assert k.shape == v.shape and k.ndim == 2
        with self.torch.cuda.device(self.device):
            _check(lib().ps_stack_load_kv(self.h, int(layer), int(kv_head), _ptr(k), _ptr(v), k.shape[0]))

    def set_context(self, context):
        _check(lib().ps_stack_set_context(self.h, int(context)))

    def set_cpu_threads(self, threads):
        _check(lib().ps_stack_set_cpu_threads(self.h, int(threads)))

    def set_logits_out(self, logits, first_token=0, rows=1):
        """logits: torch fp16 CUDA tensor of rows * vocab elements (kept alive by the caller), or None
        with rows = 0 to leave the output head out of the following forwards."""
        if rows:
            assert logits.dtype == self.torch.float16 and logits.is_contiguous()
            assert logits.numel() == rows * self.plan.cfg["vocab"]
        _check(lib().ps_stack_set_logits_out(self.h, logits.data_ptr() if rows else None, int(first_token), int(rows)))

    def forward(self, x_in, x_out, router_logits=None, router_logits_dev=None):
        """x_in, x_out: torch fp16 CUDA tensors [M][H]; asynchronous on self.compute.
        router_logits_dev: optional torch fp32 CUDA tensor holding the same values as router_logits."""
        assert x_in.dtype == self.torch.float16 and x_out.dtype == self.torch.float16
        assert x_in.is_contiguous() and x_out.is_contiguous()
        assert tuple(x_in.shape) == (self.M, self.H) and tuple(x_out.shape) == (self.M, self.H)
        lg = None if router_logits is None else np.ascontiguousarray(router_logits, dtype=np.float32)
        ld = None
        if router_logits_dev is not None:
            assert router_logits_dev.dtype == self.torch.float32 and router_logits_dev.is_contiguous()
            assert lg is not None and tuple(router_logits_dev.shape) == lg.shape
            ld = router_logits_dev.data_ptr()
        with self.torch.cuda.device(self.device):
            _check(lib().ps_stack_forward(self.h, x_in.data_ptr(), x_out.data_ptr(), _ptr(lg), ld))

    def forward_noalloc(self, x_in, x_out):
        """ps_stack_forward_noalloc: the same pass with the workspace in the library's static device array."""
        assert x_in.dtype == self.torch.float16 and x_out.dtype == self.torch.float16
        assert x_in.is_contiguous() and x_out.is_contiguous()
        assert tuple(x_in.shape) == (self.M, self.H) and tuple(x_out.shape) == (self.M, self.H)
        with self.torch.cuda.device(self.device):
            _check(lib().ps_stack_forward_noalloc(self.h, x_in.data_ptr(), x_out.data_ptr()))

    def synchronize(self):
        with self.torch.cuda.device(self.device):
            _check(lib().ps_stack_sync_check(self.h))

    def set_copy_mode(self, gather):
        _check(lib().ps_stack_set_copy_mode(self.h, int(gather)))

    def set_decode_mode(self, mode):
        """0: launch per shard, 1: HIP-graph replay, 2: mode 0 with every RMS factor from a launch of its own (see pshard_test.h)."""
        with self.torch.cuda.device(self.device):
            _check(lib().ps_stack_set_decode_mode(self.h, int(mode)))

    def set_profiling(self, on):
        _check(lib().ps_stack_set_profiling(self.h, 1 if on else 0))

    def stats(self):
        s = ps_stats()
        with self.torch.cuda.device(self.device):
            _check(lib().ps_stack_stats(self.h, C.byref(s)))
        return s

    def op_times(self, n_ops):
        """[(start_ms, dur_ms)] of the last profiled forward, one per schedule op."""
        out = []
        a, b = C.c_double(), C.c_double()
        with self.torch.cuda.device(self.device):
            for i in range(n_ops):
                _check(lib().ps_stack_op_time(self.h, i, C.byref(a), C.byref(b)))
                out.append((a.value, b.value))
        return out

    def time_kernel(self, kernel, reps=5):
        """(avg ms per launch, launches per pass) of one kernel kind launched back to back."""
        ms, n = C.c_double(), C.c_uint32()
        with self.torch.cuda.device(self.device):
            _check(lib().ps_stack_time_kernel(self.h, kernel, reps, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def debug_buffer(self, which, dtype, shape):
        """Copy of a workspace buffer as a numpy array (synchronises first)."""
        self.synchronize()
        p, n = C.c_void_p(), C.c_uint64()
        _check(lib().ps_stack_debug_buffer(self.h, which, C.byref(p), C.byref(n)))
        off = p.value - self.arena.data_ptr()
        raw = self.arena[off:off + n.value].cpu().numpy()
        return raw.view(dtype)[: int(np.prod(shape))].reshape(shape)

    def close(self):
        if self.h:
            with self.torch.cuda.device(self.device):
                lib().ps_stack_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def profile_measure(scratch_bytes=1 << 30, device="cuda:0"):
    import torch
    dev = torch.device(device)
    scratch = torch.empty(scratch_bytes, dtype=torch.uint8, device=dev)
    s1, s2 = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
    p = ps_profile()
    with torch.cuda.device(dev):
        _check(lib().ps_profile_measure(scratch.data_ptr(), scratch_bytes, s1.cuda_stream, s2.cuda_stream, C.byref(p)))
    torch.cuda.synchronize(dev)
    return p


def load_synthetic(stacks, cfg, seed, threads=8, lookahead=12, progress=None):
    """Generate every logical matrix of cfg with synth_inputs.weight_matrix (a pool of generator
    threads, bounded look-ahead so the whole model is never resident on the host) and load it
    into each stack of `stacks`."""
    import collections
    from concurrent.futures import ThreadPoolExecutor
    import synth_inputs as S
    stacks = stacks if isinstance(stacks, (list, tuple)) else [stacks]
    todo = [(layer, kind, expert, N, K) for layer in range(cfg["n_layers"])
            for (kind, expert, N, K) in S.matrix_shapes(cfg)]
    if cfg.get("vocab"):   # output head: a matrix of the layer after the last
        todo.append((cfg["n_layers"], S.MAT_OUT, None, cfg["vocab"], cfg["hidden"]))
    with ThreadPoolExecutor(max_workers=threads) as ex:
        q = collections.deque()
        it = iter(todo)

        def submit():
            t = next(it, None)
            if t is not None:
                q.append((t, ex.submit(S.weight_matrix, seed, t[0], t[1], t[2], t[3], t[4])))
        for _ in range(lookahead):
            submit()
        done = 0
        while q:
            (layer, kind, expert, N, K), fut = q.popleft()
            sc, cd = fut.result()
            submit()
            for st in stacks:
                st.load_matrix(layer, kind, expert, sc, cd)
            done += 1
            if progress and (done % progress == 0 or done == len(todo)):
                import sys
                print("  loaded %d / %d matrices" % (done, len(todo)), file=sys.stderr, flush=True)
