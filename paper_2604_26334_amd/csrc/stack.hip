// Executor of the GPU-only plan (paper Section 3, "Plan One", and Algorithm 1's
// SetupForSched / RunInTopologicalOrder): resident shards are computed in place, host
// shards are copied with hipMemcpyAsync on the copy stream into a two-slot VRAM scratch
// while the compute stream works on the other slot.  Also: weight loading (packing into
// the private layout) and the machine-profile measurement.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <functional>
#include <chrono>
#include <map>
#include <memory>
#include <mutex>
#include <thread>
#include <tuple>

#include "cpu_backend.h"
#include "kernels.h"
#include "ps_internal.h"

#define PS_HIP(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            ps::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
            return PS_E_HIP;                                                           \
        }                                                                              \
    } while (0)

struct ps_stack {
    ps_plan plan;
    uint8_t *arena = nullptr;
    uint64_t arena_bytes = 0;
    // several token tiers on one arena (ps_stack_create_tiers): every tier's plan, the packed image of
    // every matrix in pinned host memory, and what each stretch of the pinned region holds right now
    bool multi = false;
    std::vector<ps_plan> tiers;               // by tier index; a plan with M == 0 marks an infeasible tier
    uint32_t active_tier = 0;
    std::map<std::tuple<uint32_t, uint32_t, uint32_t>, uint8_t *> image;   // (layer, shard kind, expert) -> whole matrix
    struct Content { uint64_t off, bytes, tile_bytes; uint32_t layer, kind, expert, tile0; };
    std::vector<Content> content;
    uint8_t *static_ws = nullptr;             // this device's address of the library's static scratch
    uint8_t *ws_base = nullptr;               // where the workspace offsets of the plan count from: the arena,
                                              // or the library's static scratch during ps_stack_forward_noalloc
    hipStream_t compute = nullptr, copy = nullptr;
    std::vector<void *> host_chunks;          // hipHostMalloc'ed pools of streamed shards
    std::vector<uint8_t *> shard_host;        // per shard: host image (streamed) or null
    std::map<std::tuple<uint32_t, uint32_t, uint32_t>, std::vector<uint32_t>> cover;  // (layer, shard kind, expert)
    std::vector<uint8_t> loaded;              // per (layer, logical matrix slot)
    uint64_t n_loaded = 0, n_expected = 0;
    hipEvent_t ev_ready[2] = {nullptr, nullptr}, ev_free[2] = {nullptr, nullptr};
    std::vector<hipEvent_t> ev_router;
    hipEvent_t ev_upload[2] = {nullptr, nullptr};   // per table buffer: its uploads / gathers are done
    bool upload_pending[2] = {false, false};
    uint32_t table_idx = 0;                   // table buffer of the current forward
    bool gather_copy = true;                  // expert batches: one gather kernel instead of one memcpy each
    int32_t copy_mode = 1;                    // as set by ps_stack_set_copy_mode
    bool gather_dense = false;                // this plan's dense slabs go through the gather kernel as well
    bool inline_fill = true;                  // a layer's only expert fill is issued on the compute stream
    ps::CopyDesc *dense_descs = nullptr;      // pinned: one descriptor per op of the dense schedule (copies use theirs)
    size_t dense_descs_cap = 0;
    uint64_t descs_off = 0;                   // offset of the copy descriptors in a table buffer
    uint32_t n_descs = 0;                     // descriptors written in the current forward
    ps_schedule dense_sched;
    bool have_dense_sched = false;
    void *stage = nullptr;                    // pinned staging for resident loads
    uint64_t stage_bytes = 0;
    void *tables_host[2] = {nullptr, nullptr};   // pinned: logits | tasks | pairs | copy descriptors of one forward (MoE)
    uint64_t tables_bytes = 0;
    int32_t decode_mode = 0;                  // as set by ps_stack_set_decode_mode (re-evaluated when a tier is installed)
    bool use_graph = false;                   // all-resident one-token forward replayed from a HIP graph
    std::map<std::tuple<const void *, void *, void *, uint32_t>, hipGraphExec_t> graphs;   // per (x_in, x_out, logits, valid rows and head rows)
    // CPU back-end (plans with shards left in system memory): worker threads, pinned host copies of
    // the activations it reads (FFN input, SwiGLU output, final hidden state) and of what it writes
    std::unique_ptr<ps::CpuPool> pool;
    uint16_t *host_h = nullptr, *host_s = nullptr, *host_x = nullptr, *host_out = nullptr;
    std::vector<float> cpu_scratch;
    std::vector<uint16_t> cpu_xg, cpu_sg;     // MoE: the CPU experts' gathered inputs and SwiGLU outputs, per pair
    bool out_upload_pending = false;          // host_out is still being read by an upload
    __half *logits = nullptr;                 // output head: caller's logits buffer
    uint32_t head_rows = 0, head_row0 = 0;    // 0: head skipped, 1: token head_row0 only, n_tokens: every token
    uint32_t n_valid = 0;                     // token rows of the current forward that carry data (<= plan.M)
    const float *route_logits = nullptr;      // device: router logits the routing kernel of this forward reads
    uint64_t route_layer_stride = 0;          // elements between two layers' logits there
    uint32_t ctx = 0;                         // cached positions the next forward attends over (KV stacks)
    hipEvent_t ev_step = nullptr;             // KV stacks: end of the previous forward's compute
    bool step_pending = false;
    bool kv_copied = false;                   // some kv shard is not resident: the copy stream reads appended rows
    uint32_t kv_rows = 0;                     // cache positions written so far (loaded or appended): what a tier switch moves
    bool profiling = false;
    bool own_rinv_launch = false;             // decode mode 2: RMS factors always from rinv_kernel
    const void *rinv_of = nullptr;            // rows whose RMS factors the last residual epilogue left in the workspace
    std::vector<hipEvent_t> prof_ev;          // 2 per op of the last profiled forward
    std::vector<uint8_t> prof_is_copy;
    std::vector<double> prof_start, prof_dur;
    bool prof_valid = false;
    ps_stats stats{};
};

// Workspace of ps_stack_forward_noalloc: one array per GPU, in the library's own device image, so
// that entry point needs no memory from its caller beyond inputs, outputs and the arena's weights.
// In host code the array's name stands for the symbol, not for a device address: the address on a
// device comes from hipGetSymbolAddress with that device current, once, and is kept per device.
constexpr uint64_t kStaticWsBytes = 32ull << 20;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

namespace {

using namespace ps;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up on first use there)
int32_t static_scratch(uint8_t **out) {
    int dev = -1;
    PS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { ps::set_error("device index %d out of range", dev); return PS_E_HIP; }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        PS_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || (uintptr_t)ptr % kAlign) { ps::set_error("static scratch has no usable device address"); return PS_E_HIP; }
        g_scratch_ptr[dev] = ptr;
    }
    *out = static_cast<uint8_t *>(g_scratch_ptr[dev]);
    return PS_OK;
}

constexpr uint64_t kHostChunk = 1ull << 30;

uint8_t *slot_ptr(const ps_stack *st, int slot) {
    return st->arena + st->plan.scratch_off + (uint64_t)slot * st->plan.slot_bytes;
}

void parallel_for(uint32_t n, const std::function<void(uint32_t)> &fn) {
    unsigned hw = std::thread::hardware_concurrency();
    uint32_t nt = std::max(1u, std::min<uint32_t>(std::min<uint32_t>(hw ? hw : 4, 16), n));
    if (nt == 1) { for (uint32_t i = 0; i < n; ++i) fn(i); return; }
    std::atomic<uint32_t> next{0};
    std::vector<std::thread> th;
    for (uint32_t t = 0; t < nt; ++t)
        th.emplace_back([&]() { for (uint32_t i; (i = next.fetch_add(1)) < n;) fn(i); });
    for (auto &t : th) t.join();
}

const MatGeom &geom_of(const ModelGeom &g, uint32_t mat) {
    switch (mat) {
        case PS_MAT_QKV: return g.qkv;
        case PS_MAT_O: return g.o;
        case PS_MAT_DOWN: return g.down;
        case PS_MAT_OUT: return g.head;
        default: return g.gate_up;
    }
}

// A dense matmul op of a plan of two to kGemvMtTokens tokens runs in the few-token form of the decode
// kernel when the matrix's K is a multiple of 1024 (whole scale groups); it computes its own RMS factors
static bool few_token_gemv(const ps_plan &p, const MatGeom &mg) {
    return p.M >= 2 && p.M <= (uint32_t)kGemvMtTokens && mg.ntiles && mg.nsb % 8 == 0;
}

// GEMV launch description of a dense matmul op (QKV, O, GATE_UP, DOWN) of one or a few tokens
bool dense_gemv_args(const ps_stack *st, const Op &op, const __half *x_in, __half *x_out, GemvArgs *out, int *mode,
                     uint32_t *ks) {
    const ps_plan &p = st->plan;
    const ModelGeom &g = p.g;
    const auto &m = g.m;
    const uint32_t l = op.info.layer;
    uint8_t *A = st->arena;       // weights: pinned shards and scratch slots
    uint8_t *WS = st->ws_base;    // activations, RMS factors, partial sums, tables
    const __half *xin = l == 0 ? x_in : reinterpret_cast<const __half *>(WS + ((l - 1) & 1 ? p.ws.x1 : p.ws.x0));
    __half *xout = l == m.n_layers - 1 ? x_out : reinterpret_cast<__half *>(WS + (l & 1 ? p.ws.x1 : p.ws.x0));
    __half *hbuf = g.has_attn ? reinterpret_cast<__half *>(WS + p.ws.h) : const_cast<__half *>(xin);
    __half *qkv = reinterpret_cast<__half *>(WS + p.ws.qkv);
    __half *sbuf = reinterpret_cast<__half *>(WS + p.ws.s);
    const bool resid = !(m.flags & PS_FLAG_NO_RESIDUAL);
    const Shard &s = p.shards[op.info.shard0];
    const uint4 *W = s.resident == 1 ? reinterpret_cast<const uint4 *>(A + s.offset)
                                : reinterpret_cast<const uint4 *>(slot_ptr(st, op.info.slot) + op.info.slot_offset);
    const MatGeom *mg = nullptr;
    GemvArgs a{};
    a.x_group = 1; a.eps = m.rms_eps; a.top_k = 1; a.W = W;
    switch (op.info.kernel) {
        case PS_K_QKV:
            mg = &g.qkv; *mode = GEMV_PLAIN; *ks = gemv_ksplit(mg->ngroups, mg->ntiles);
            a.nunits = s.ntiles; a.x = xin; a.out = qkv; a.out_row0 = s.tile0 * 16;
            a.x_stride = m.hidden; a.out_stride = g.qkv_w;
            break;
        case PS_K_O:
            mg = &g.o; *mode = GEMV_RESID; *ks = gemv_ksplit(mg->ngroups, mg->ntiles);
            a.nunits = s.ntiles; a.res = xin; a.out = hbuf; a.out_row0 = s.tile0 * 16;
            if (g.kv) {   // the attention output
                a.x = reinterpret_cast<const __half *>(WS + p.ws.attn); a.x_stride = g.attn_w;
            } else {      // identity on V, read in place from the QKV row
                a.x = qkv; a.x_off = (m.n_q_heads + m.n_kv_heads) * m.head_dim; a.x_group = m.n_q_heads / m.n_kv_heads;
                a.x_stride = g.qkv_w;
            }
            a.out_stride = m.hidden;
            break;
        case PS_K_GATE_UP:
            mg = &g.gate_up; *mode = GEMV_GATE_UP; *ks = gemv_ksplit(mg->ngroups, mg->ntiles / 2);
            a.nunits = s.ntiles / 2; a.x = hbuf; a.out = sbuf; a.out_row0 = s.tile0 / 2 * 16;
            a.x_stride = m.hidden; a.out_stride = g.ffn_i;
            break;
        case PS_K_DOWN:
            mg = &g.down; *mode = GEMV_RESID; *ks = gemv_ksplit(mg->ngroups, mg->ntiles);
            a.nunits = s.ntiles; a.x = sbuf; a.res = resid ? hbuf : nullptr; a.out = xout; a.out_row0 = s.tile0 * 16;
            a.x_stride = g.ffn_i; a.out_stride = m.hidden;
            break;
        default: return false;
    }
    a.tile_u4 = (uint32_t)(mg->tile_bytes / 16); a.nsb = mg->nsb; a.ngroups = mg->ngroups; a.K = mg->K;
    *out = a;
    return true;
}

int32_t issue_kernel(ps_stack *st, const ps_schedule &sc, const Op &op, const __half *x_in, __half *x_out) {
    const ps_plan &p = st->plan;
    const ModelGeom &g = p.g;
    const auto &m = g.m;
    // M: token rows that carry data in this forward (the last chunk of a chunked prefill has fewer
    // than the plan's MP).  Launch shapes, tile sizes and the K split go by MP alone, so a row's bits
    // do not depend on how many rows came with it; rows past M are neither read nor written.
    const uint32_t M = st->n_valid, MP = p.M, H = m.hidden, l = op.info.layer;
    uint8_t *A = st->arena;       // weights: pinned shards and scratch slots
    uint8_t *WS = st->ws_base;    // activations, RMS factors, partial sums, tables
    const __half *xin = l == 0 ? x_in : reinterpret_cast<const __half *>(WS + ((l - 1) & 1 ? p.ws.x1 : p.ws.x0));
    __half *xout = l == m.n_layers - 1 ? x_out : reinterpret_cast<__half *>(WS + (l & 1 ? p.ws.x1 : p.ws.x0));
    __half *hbuf = g.has_attn ? reinterpret_cast<__half *>(WS + p.ws.h) : const_cast<__half *>(xin);
    __half *qkv = reinterpret_cast<__half *>(WS + p.ws.qkv);
    __half *sbuf = reinterpret_cast<__half *>(WS + p.ws.s);
    float *rinv = reinterpret_cast<float *>(WS + p.ws.rinv);
    const bool resid = !(m.flags & PS_FLAG_NO_RESIDUAL);
    hipStream_t cs = st->compute;

    auto wptr = [&](const Op &o) -> const uint4 * {
        const Shard &s = p.shards[o.info.shard0];
        if (s.resident == 1) return reinterpret_cast<const uint4 *>(A + s.offset);
        return reinterpret_cast<const uint4 *>(slot_ptr(st, o.info.slot) + o.info.slot_offset);
    };
    auto gemv_base = [&](const MatGeom &mg) {
        GemvArgs a{};
        a.tile_u4 = (uint32_t)(mg.tile_bytes / 16); a.nsb = mg.nsb; a.ngroups = mg.ngroups; a.K = mg.K;
        a.x_group = 1; a.eps = m.rms_eps; a.top_k = std::max(1u, m.top_k);
        return a;
    };
    auto gemm_base = [&](const MatGeom &mg) {
        GemmArgs a{};
        a.tile_u4 = (uint32_t)(mg.tile_bytes / 16); a.nsb = mg.nsb; a.M = M; a.total_tiles = mg.ntiles;
        a.x_group = 1; a.rinv = rinv; a.top_k = std::max(1u, m.top_k);
        return a;
    };

    if (op.info.kernel == PS_K_OUT && st->head_rows == 1) {
        // logits of one token: fused RMSNorm + GEMV over its row of the final hidden state
        const Shard &s = p.shards[op.info.shard0];
        GemvArgs a = gemv_base(g.head);
        a.top_k = 1; a.W = wptr(op); a.nunits = s.ntiles; a.x = x_out + (size_t)st->head_row0 * H;
        a.out = st->logits; a.out_row0 = s.tile0 * 16;
        PS_HIP(launch_gemv(GEMV_PLAIN, gemv_ksplit(g.head.ngroups, g.head.ntiles), a, 0, cs));
        return PS_OK;
    }
    if (MP == 1 && op.info.kernel >= PS_K_QKV && op.info.kernel <= PS_K_DOWN) {
        GemvArgs a;
        int mode;
        uint32_t ks;
        dense_gemv_args(st, op, x_in, x_out, &a, &mode, &ks);
        PS_HIP(launch_gemv(mode, ks, a, 0, cs));
        return PS_OK;
    }
    if (op.info.kernel >= PS_K_QKV && op.info.kernel <= PS_K_DOWN &&
        few_token_gemv(p, op.info.kernel == PS_K_QKV ? g.qkv : op.info.kernel == PS_K_O ? g.o : op.info.kernel == PS_K_GATE_UP ? g.gate_up : g.down)) {
        GemvArgs a;
        int mode;
        uint32_t ks;
        dense_gemv_args(st, op, x_in, x_out, &a, &mode, &ks);
        PS_HIP(launch_gemv_mt(mode, ks, a, M, cs));
        return PS_OK;
    }
    // batched decode (2..64 tokens) of a narrow matrix: split K over blockIdx.z into fp32 partial
    // planes, then one epilogue kernel sums them in order and applies the mode's epilogue
    auto run_gemm = [&](int mode, GemmArgs a, const MatGeom &mg) -> int32_t {
        const uint32_t per = gemm_sb_per_part(mg, MP);
        if (!per) { PS_HIP(launch_gemm(mode, a, 0, MP, cs)); return PS_OK; }
        GemmArgs pa = a;
        float *partial = reinterpret_cast<float *>(WS + p.ws.partial);
        const uint32_t ncols = a.ntiles * 16;
        pa.out_f32 = partial; pa.out = nullptr; pa.out_stride = ncols; pa.out_row0 = 0;
        pa.sb_per_part = per; pa.part_stride = MP * ncols;
        PS_HIP(launch_gemm(GEMM_F32, pa, 0, MP, cs));
        if (mode == GEMM_RESID && ncols == H && a.out_row0 == 0 && a.out_stride == H && !st->own_rinv_launch) {
            // the launch covers whole rows of the hidden state: its epilogue also leaves their RMS
            // factors (the bits rinv_kernel gives), and the PS_K_RINV op that follows is skipped
            PS_HIP(launch_splitk_epilogue_resid_rinv(partial, (mg.nsb + per - 1) / per, pa.part_stride, M, H, a.res, a.out,
                                                     m.rms_eps, rinv, cs));
            st->rinv_of = a.out;
            return PS_OK;
        }
        PS_HIP(launch_splitk_epilogue(mode, partial, (mg.nsb + per - 1) / per, pa.part_stride, M, ncols, rinv, a.res,
                                      a.out, a.out_stride, a.out_row0, cs));
        return PS_OK;
    };
    switch (op.info.kernel) {
        case PS_K_RINV: {
            const __half *rows = op.info.shard0 == 2 ? x_out : op.info.shard0 == 0 && g.has_attn ? xin : hbuf;   // 2: output head
            const bool have = st->rinv_of == rows;
            st->rinv_of = nullptr;
            // the few-token kernels of QKV (factors of kind 0) and of a dense gate/up (kind 1) compute their own
            if (op.info.shard0 == 0 && few_token_gemv(p, g.qkv)) return PS_OK;
            if (op.info.shard0 == 1 && !g.moe && few_token_gemv(p, g.gate_up)) return PS_OK;
            if (!have) PS_HIP(launch_rinv(rows, M, H, m.rms_eps, rinv, cs));
            return PS_OK;
        }
        case PS_K_OUT: {   // every token's logits (head_rows == MP > 1)
            const Shard &s = p.shards[op.info.shard0];
            GemmArgs a = gemm_base(g.head);
            a.W = wptr(op); a.ntiles = s.ntiles; a.x = x_out; a.x_stride = H; a.out = st->logits;
            a.out_stride = m.vocab; a.out_row0 = s.tile0 * 16;
            return run_gemm(GEMM_PLAIN, a, g.head);
        }
        case PS_K_QKV: {
            const Shard &s = p.shards[op.info.shard0];
            GemmArgs a = gemm_base(g.qkv);
            a.W = wptr(op); a.ntiles = s.ntiles; a.x = xin; a.x_stride = H; a.out = qkv;
            a.out_stride = g.qkv_w; a.out_row0 = s.tile0 * 16;
            return run_gemm(GEMM_PLAIN, a, g.qkv);
        }
        case PS_K_O: {
            const Shard &s = p.shards[op.info.shard0];
            GemmArgs a = gemm_base(g.o);
            a.W = wptr(op); a.ntiles = s.ntiles;
            if (g.kv) {   // the attention output rows
                a.x = reinterpret_cast<const __half *>(WS + p.ws.attn); a.x_stride = g.attn_w;
            } else {      // identity on V, read in place from the QKV rows
                a.x = qkv; a.x_stride = g.qkv_w;
                a.x_off = (m.n_q_heads + m.n_kv_heads) * m.head_dim; a.x_group = m.n_q_heads / m.n_kv_heads;
            }
            a.res = xin; a.out = hbuf; a.out_stride = H; a.out_row0 = s.tile0 * 16;
            return run_gemm(GEMM_RESID, a, g.o);
        }
        case PS_K_GATE_UP: {
            const Shard &s = p.shards[op.info.shard0];
            GemmArgs a = gemm_base(g.gate_up);
            a.W = wptr(op); a.ntiles = s.ntiles; a.x = hbuf; a.x_stride = H; a.out = sbuf;
            a.out_stride = g.ffn_i; a.out_row0 = s.tile0 / 2 * 16;
            return run_gemm(GEMM_GATE_UP, a, g.gate_up);
        }
        case PS_K_DOWN: {
            const Shard &s = p.shards[op.info.shard0];
            GemmArgs a = gemm_base(g.down);
            a.W = wptr(op); a.ntiles = s.ntiles; a.x = sbuf; a.x_stride = g.ffn_i;
            a.res = resid ? hbuf : nullptr; a.out = xout; a.out_stride = H; a.out_row0 = s.tile0 * 16;
            return run_gemm(GEMM_RESID, a, g.down);
        }
        case PS_K_ATTN: {
            const Shard &s = p.shards[op.info.shard0];
            const uint32_t ccap = (m.kv_context + kAttnChunk - 1) / kAttnChunk + (MP > 1 ? (MP + kAttnChunk - 1) / kAttnChunk : 0);
            if (MP >= kAttnOnePassTokens) {   // many tokens: cache and own rows in one walk, finished rows out
                AttnChunkArgs c{};
                c.k_base = reinterpret_cast<const __half *>(wptr(op)); c.head_stride = g.kv_shard_bytes;
                c.cap = m.kv_context; c.ctx = st->ctx; c.head0 = s.expert; c.nheads = op.info.nshards;
                c.group = m.n_q_heads / m.n_kv_heads; c.n_q = m.n_q_heads; c.row_stride = m.head_dim;
                c.ntok = M; c.q_stride = g.qkv_w; c.q = qkv;
                c.k_own = qkv + (size_t)m.n_q_heads * m.head_dim; c.v_own = qkv + (size_t)(m.n_q_heads + m.n_kv_heads) * m.head_dim;
                c.own_stride = g.qkv_w; c.out = reinterpret_cast<__half *>(WS + p.ws.attn); c.out_stride = g.attn_w;
                PS_HIP(launch_attn_chunk_onepass(c, cs));
                return PS_OK;
            }
            if (MP > 1) {   // a chunk of tokens over the cached positions of this run of kv heads
                AttnChunkArgs c{};
                c.k_base = reinterpret_cast<const __half *>(wptr(op)); c.head_stride = g.kv_shard_bytes;
                c.cap = m.kv_context; c.ctx = st->ctx; c.head0 = s.expert; c.nheads = op.info.nshards;
                c.group = m.n_q_heads / m.n_kv_heads; c.n_q = m.n_q_heads; c.row_stride = m.head_dim; c.causal = 0;
                c.ntok = M; c.q_stride = g.qkv_w; c.chunk0 = 0; c.chunk_cap = ccap; c.q = qkv;
                c.part = reinterpret_cast<float *>(WS + p.ws.apart);
                PS_HIP(launch_attn_chunk(c, cs));
                return PS_OK;
            }
            AttnArgs a{};
            a.kv = reinterpret_cast<const __half *>(wptr(op));
            a.head_stride = g.kv_shard_bytes; a.cap = m.kv_context; a.ctx = st->ctx;
            a.head0 = s.expert; a.nheads = op.info.nshards; a.group = m.n_q_heads / m.n_kv_heads;
            a.chunk_cap = (m.kv_context + kAttnChunk - 1) / kAttnChunk;
            a.q = qkv; a.part = reinterpret_cast<float *>(WS + p.ws.apart);
            a.ctx_dev = st->use_graph ? reinterpret_cast<const uint32_t *>(WS + p.ws.ctx) : nullptr;
            PS_HIP(launch_attn_decode(a, cs));
            return PS_OK;
        }
        case PS_K_ATTN_COMBINE:
            if (MP >= kAttnOnePassTokens) {   // the attention rows are finished: only the chunk's rows remain to be appended
                PS_HIP(launch_kv_append_rows(st->ctx, m.kv_context, qkv, g.qkv_w, m.n_q_heads, m.n_kv_heads, M,
                                             reinterpret_cast<const uint64_t *>(WS + p.ws.kvhome) + (size_t)l * m.n_kv_heads, cs));
                return PS_OK;
            }
            if (MP > 1) {   // the chunk's own rows (causal), then every token's chunks merged and its rows appended
                const uint32_t ccap = (m.kv_context + kAttnChunk - 1) / kAttnChunk + (MP + kAttnChunk - 1) / kAttnChunk;
                AttnChunkArgs c{};
                c.k_base = qkv + (size_t)m.n_q_heads * m.head_dim; c.v_base = qkv + (size_t)(m.n_q_heads + m.n_kv_heads) * m.head_dim;
                c.cap = m.kv_context; c.ctx = st->ctx; c.head0 = 0; c.nheads = m.n_kv_heads;
                c.group = m.n_q_heads / m.n_kv_heads; c.n_q = m.n_q_heads; c.row_stride = g.qkv_w; c.causal = 1;
                c.ntok = M; c.q_stride = g.qkv_w; c.chunk0 = (st->ctx + kAttnPosPerWg - 1) / kAttnPosPerWg; c.chunk_cap = ccap; c.q = qkv;
                c.part = reinterpret_cast<float *>(WS + p.ws.apart);
                PS_HIP(launch_attn_chunk(c, cs));
                PS_HIP(launch_attn_combine_chunk(c.part, ccap, st->ctx, m.kv_context, qkv, g.qkv_w, m.n_q_heads, m.n_kv_heads, M,
                                                 reinterpret_cast<const uint64_t *>(WS + p.ws.kvhome) + (size_t)l * m.n_kv_heads,
                                                 reinterpret_cast<__half *>(WS + p.ws.attn), g.attn_w, cs));
                return PS_OK;
            }
            PS_HIP(launch_attn_combine(reinterpret_cast<const float *>(WS + p.ws.apart),
                                       (m.kv_context + kAttnChunk - 1) / kAttnChunk, st->ctx,
                                       st->use_graph ? reinterpret_cast<const uint32_t *>(WS + p.ws.ctx) : nullptr, m.kv_context, qkv,
                                       m.n_q_heads, m.n_kv_heads,
                                       reinterpret_cast<const uint64_t *>(WS + p.ws.kvhome) + (size_t)l * m.n_kv_heads,
                                       reinterpret_cast<__half *>(WS + p.ws.attn), cs));
            return PS_OK;
        case PS_K_ROUTE:
            PS_HIP(launch_route(st->route_logits + (size_t)l * st->route_layer_stride, M,
                                m.n_experts, m.top_k, reinterpret_cast<int32_t *>(WS + p.ws.ridx),
                                reinterpret_cast<float *>(WS + p.ws.rw), cs));
            return PS_OK;
        case PS_K_EXPERT_GATE_UP:
        case PS_K_EXPERT_DOWN: {
            const bool gu = op.info.kernel == PS_K_EXPERT_GATE_UP;
            const DeviceTask *tasks = reinterpret_cast<const DeviceTask *>(WS + p.ws.tasks) + op.task0;
            const int32_t *pairs = reinterpret_cast<const int32_t *>(WS + p.ws.pairs);
            float *y = reinterpret_cast<float *>(WS + p.ws.y);
            uint32_t max_tok = 0;
            for (uint32_t t = op.task0; t < op.task0 + op.ntasks; ++t) max_tok = std::max(max_tok, sc.tasks[t].npairs);
            const MatGeom &mg = gu ? g.gate_up : g.down;
            if (MP == 1) {
                GemvArgs a = gemv_base(mg);
                a.tasks = tasks; a.pairs = pairs;
                if (gu) { a.nunits = mg.ntiles / 2; a.x = hbuf; a.x_stride = H; a.out = sbuf; a.out_stride = g.ffn_i; }
                else { a.nunits = mg.ntiles; a.x = sbuf; a.x_stride = g.ffn_i; a.out_f32 = y; a.out_stride = H; }
                const uint32_t units = gu ? mg.ntiles / 2 : mg.ntiles;
                PS_HIP(launch_gemv(gu ? GEMV_GATE_UP : GEMV_F32, gemv_ksplit(mg.ngroups, units * m.top_k), a, op.ntasks, cs));
            } else {
                GemmArgs a = gemm_base(mg);
                a.tasks = tasks; a.pairs = pairs; a.ntiles = mg.ntiles;
                if (gu) { a.x = hbuf; a.x_stride = H; a.out = sbuf; a.out_stride = g.ffn_i; }
                else { a.x = sbuf; a.x_stride = g.ffn_i; a.out_f32 = y; a.out_stride = H; }
                PS_HIP(launch_gemm(gu ? GEMM_GATE_UP : GEMM_F32, a, op.ntasks, max_tok, cs));
            }
            return PS_OK;
        }
        case PS_K_COMBINE:
            PS_HIP(launch_combine(hbuf, reinterpret_cast<const float *>(WS + p.ws.y),
                                  reinterpret_cast<const float *>(WS + p.ws.rw), M, H, m.top_k, resid ? 1 : 0, xout, cs));
            return PS_OK;
    }
    set_error("unknown kernel id %u", op.info.kernel);
    return PS_E_STATE;
}

double now_ms() {
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// FETCH: the activation buffers a CPU shard reads go to their pinned host copies on the compute
// stream, and the host waits for them (this also retires every earlier upload from host_out).
int32_t issue_fetch(ps_stack *st, const Op &op, const __half *x_in, __half *x_out) {
    const ps_plan &p = st->plan;
    const ModelGeom &g = p.g;
    const uint32_t M = st->n_valid, H = g.m.hidden, l = op.info.layer;
    const double t0 = now_ms();
    if (op.info.buffers & PS_BUF_H) {
        const __half *xin = l == 0 ? x_in : reinterpret_cast<const __half *>(st->ws_base + ((l - 1) & 1 ? p.ws.x1 : p.ws.x0));
        const void *src = g.has_attn ? static_cast<const void *>(st->ws_base + p.ws.h) : static_cast<const void *>(xin);
        PS_HIP(hipMemcpyAsync(st->host_h, src, (size_t)M * H * 2, hipMemcpyDeviceToHost, st->compute));
    }
    if (op.info.buffers & PS_BUF_S)
        PS_HIP(hipMemcpyAsync(st->host_s, st->ws_base + p.ws.s, (size_t)M * g.ffn_i * 2, hipMemcpyDeviceToHost, st->compute));
    if (op.info.buffers & PS_BUF_X) {
        // the head reads every token's final state, or only the requested token's row
        const size_t row0 = st->head_rows == 1 ? st->head_row0 : 0, rows = st->head_rows == 1 ? 1 : M;
        PS_HIP(hipMemcpyAsync(st->host_x, x_out + row0 * H, rows * H * 2, hipMemcpyDeviceToHost, st->compute));
    }
    PS_HIP(hipStreamSynchronize(st->compute));
    st->out_upload_pending = false;
    st->stats.cpu_wait_ms += now_ms() - t0;
    return PS_OK;
}

// The CPU's experts of one MoE layer: for every such expert its routed (token, rank) pairs go
// through gate/up + SwiGLU and the down projection on the host; all experts share two passes over
// the worker pool.  The fp32 result rows travel in one upload, followed by their pair numbers, and
// a scatter kernel puts them where the combine step reads them.
int32_t issue_cpu_experts(ps_stack *st, const ps_schedule &sc, const Op &op) {
    const ps_plan &p = st->plan;
    const ModelGeom &g = p.g;
    const auto &m = g.m;
    const uint32_t H = m.hidden, I = g.ffn_i, P = p.M * m.top_k;
    if (st->out_upload_pending) { PS_HIP(hipStreamSynchronize(st->compute)); st->out_upload_pending = false; }
    std::vector<CpuMatArgs> gu(op.ntasks), dn(op.ntasks);
    std::vector<size_t> scr(op.ntasks + 1, 0);
    float *yrows = reinterpret_cast<float *>(st->host_out);
    uint32_t row = 0, nrows = 0;
    uint64_t bytes = 0;
    for (uint32_t k = 0; k < op.ntasks; ++k) nrows += sc.tasks[op.task0 + k].npairs;
    if (nrows > P) { set_error("internal: CPU expert pairs exceed the workspace"); return PS_E_STATE; }
    // result rows [nrows][H] fp32, directly followed by their pair numbers: one upload
    int32_t *ypairs = reinterpret_cast<int32_t *>(yrows + (size_t)nrows * H);
    for (uint32_t k = 0; k < op.ntasks; ++k) {
        const TaskHost &t = sc.tasks[op.task0 + k];
        for (uint32_t q = 0; q < t.npairs; ++q) {
            const int32_t pair = sc.pairs[t.pair0 + q];
            if (pair < 0 || (uint32_t)pair >= P) { set_error("internal: pair index out of range"); return PS_E_STATE; }
            std::memcpy(st->cpu_xg.data() + (size_t)(row + q) * H, st->host_h + (size_t)(pair / m.top_k) * H, (size_t)H * 2);
            ypairs[row + q] = pair;
        }
        CpuMatArgs a;
        a.W = st->shard_host[t.shard]; a.ntiles = g.gate_up.ntiles; a.tile_bytes = g.gate_up.tile_bytes;
        a.nsb = g.gate_up.nsb; a.ngroups = g.gate_up.ngroups; a.K = H; a.M = t.npairs; a.eps = m.rms_eps;
        a.mode = CPU_GATE_UP; a.x = st->cpu_xg.data() + (size_t)row * H; a.x_stride = H;
        a.out = st->cpu_sg.data() + (size_t)row * I; a.out_stride = I; a.out_col0 = 0;
        gu[k] = a;
        CpuMatArgs b;
        b.W = st->shard_host[t.shard] + g.gate_up.bytes; b.ntiles = g.down.ntiles; b.tile_bytes = g.down.tile_bytes;
        b.nsb = g.down.nsb; b.ngroups = g.down.ngroups; b.K = I; b.M = t.npairs; b.mode = CPU_F32;
        b.x = a.out; b.x_stride = I; b.out_f32 = yrows + (size_t)row * H; b.out_stride = H; b.out_col0 = 0;
        dn[k] = b;
        scr[k + 1] = scr[k] + cpu_scratch_floats(t.npairs, std::max(H, I));
        row += t.npairs;
        bytes += p.shards[t.shard].bytes;
    }
    if (st->cpu_scratch.size() < scr[op.ntasks]) st->cpu_scratch.resize(scr[op.ntasks]);
    const double t0 = now_ms();
    scr.pop_back();
    cpu_matmul_many(gu, *st->pool, st->cpu_scratch.data(), scr);   // gate/up + SwiGLU of every expert
    cpu_matmul_many(dn, *st->pool, st->cpu_scratch.data(), scr);   // then the down projections
    st->stats.cpu_ms += now_ms() - t0;
    st->stats.cpu_bytes_step += bytes;
    uint8_t *land = st->ws_base + p.ws.cpu_y;
    PS_HIP(hipMemcpyAsync(land, yrows, (size_t)row * H * 4 + (size_t)row * 4, hipMemcpyHostToDevice, st->compute));
    PS_HIP(launch_scatter_rows(reinterpret_cast<const float *>(land), reinterpret_cast<const int32_t *>(land + (size_t)row * H * 4), row, H,
                               reinterpret_cast<float *>(st->ws_base + p.ws.y), st->compute));
    st->out_upload_pending = true;
    return PS_OK;
}

// CPU: one shard on the CPU back-end, straight from its packed image in the pinned host pool; the
// finished columns are uploaded on the compute stream, in order with the GPU's work on them.
int32_t issue_cpu(ps_stack *st, const ps_schedule &sc, const Op &op, __half *x_out) {
    if (op.info.kernel == PS_K_EXPERT_GATE_UP) return issue_cpu_experts(st, sc, op);
    const ps_plan &p = st->plan;
    const ModelGeom &g = p.g;
    const auto &m = g.m;
    const uint32_t M = st->n_valid, H = m.hidden, l = op.info.layer;
    const Shard &s = p.shards[op.info.shard0];
    if (st->out_upload_pending) { PS_HIP(hipStreamSynchronize(st->compute)); st->out_upload_pending = false; }
    CpuMatArgs a;
    a.W = st->shard_host[op.info.shard0];
    a.ntiles = s.ntiles; a.M = M; a.eps = m.rms_eps; a.out = st->host_out;
    __half *dst = nullptr;       // device buffer the columns go to
    const MatGeom *mg = nullptr;
    switch (op.info.kernel) {
        case PS_K_GATE_UP:
            mg = &g.gate_up; a.mode = CPU_GATE_UP; a.x = st->host_h; a.x_stride = H;
            a.out_stride = g.ffn_i; a.out_col0 = s.tile0 / 2 * 16;
            dst = reinterpret_cast<__half *>(st->ws_base + p.ws.s);
            break;
        case PS_K_DOWN:
            mg = &g.down; a.mode = CPU_RESID; a.x = st->host_s; a.x_stride = g.ffn_i;
            a.res = (m.flags & PS_FLAG_NO_RESIDUAL) ? nullptr : st->host_h;
            a.out_stride = H; a.out_col0 = s.tile0 * 16;
            dst = l == m.n_layers - 1 ? x_out : reinterpret_cast<__half *>(st->ws_base + (l & 1 ? p.ws.x1 : p.ws.x0));
            break;
        case PS_K_OUT:
            mg = &g.head; a.mode = CPU_PLAIN; a.x = st->host_x; a.x_stride = H;
            if (st->head_rows == 1) a.M = 1;
            a.out_stride = m.vocab; a.out_col0 = s.tile0 * 16;
            dst = st->logits;
            break;
        default: set_error("kernel %u has no CPU form", op.info.kernel); return PS_E_STATE;
    }
    a.tile_bytes = mg->tile_bytes; a.nsb = mg->nsb; a.ngroups = mg->ngroups; a.K = mg->K;
    const uint32_t ncols = (a.mode == CPU_GATE_UP ? s.ntiles / 2 : s.ntiles) * 16;
    const double t0 = now_ms();
    cpu_matmul_w4(a, *st->pool, st->cpu_scratch.data());
    st->stats.cpu_ms += now_ms() - t0;
    st->stats.cpu_bytes_step += s.bytes;
    PS_HIP(hipMemcpy2DAsync(dst + a.out_col0, (size_t)a.out_stride * 2, st->host_out + a.out_col0, (size_t)a.out_stride * 2,
                            (size_t)ncols * 2, a.M, hipMemcpyHostToDevice, st->compute));
    st->out_upload_pending = true;
    return PS_OK;
}

// Ops of the output head (layer index n_layers) that this forward leaves out: all of them, copies
// included, when no logits are asked for; the RMS factors of every token when only one token's
// is.  The head's slot fills hold head shards only and nothing follows them, so leaving a fill out
// together with its kernels keeps every event wait paired with the record it was built for.
bool skip_head_op(const ps_stack *st, const Op &op) {
    if (op.info.layer != st->plan.g.m.n_layers) return false;
    if (st->head_rows == 0) return true;
    return st->head_rows == 1 && op.info.type == PS_OP_KERNEL && op.info.kernel == PS_K_RINV;
}

// Plans whose forward is a fixed sequence of kernels and nothing else: dense, every shard resident, no CPU
// share; one token (with or without a KV cache) or a batched-decode step of up to 64 tokens without one
// (a chunk's attention takes its context as a launch argument)
static bool graph_eligible(const ps_plan &p) {
    return !p.g.moe && p.n_slots == 0 && p.cpu_bytes == 0 && (p.M == 1 || (p.M <= 64 && !p.g.kv));
}

// True when the copy op at index i opens the only slot fill of its layer (the schedule lists a layer's
// expert copies between its routing kernel and the next layer's ops; a fill ends at its ready record).
bool only_fill_of_layer(const ps_schedule &sc, size_t i) {
    const uint32_t layer = sc.ops[i].info.layer;
    for (size_t j = i; j-- > 0 && sc.ops[j].info.layer == layer;)
        if (sc.ops[j].info.type == PS_OP_COPY) return false;   // an earlier fill of this layer
    bool past_ready = false;
    for (size_t j = i; j < sc.ops.size() && sc.ops[j].info.layer == layer; ++j) {
        const ps_op_info &c = sc.ops[j].info;
        if (c.type != PS_OP_COPY) continue;
        if (past_ready) return false;
        if (c.flags & PS_OPF_RECORD_READY) past_ready = true;
    }
    return true;
}

int32_t run_schedule(ps_stack *st, const ps_schedule &sc, const __half *x_in, __half *x_out) {
    const ps_plan &p = st->plan;
    const bool prof = st->profiling;
    if (prof) {
        while (st->prof_ev.size() < 2 * sc.ops.size()) {
            hipEvent_t e;
            PS_HIP(hipEventCreate(&e));
            st->prof_ev.push_back(e);
        }
        st->prof_is_copy.assign(sc.ops.size(), 0);
    }
    st->prof_valid = false;
    st->rinv_of = nullptr;
    ps_stats &ss = st->stats;
    ss = ps_stats{};
    // graph mode with a KV cache: the context length travels in device memory, where the attention
    // kernels of this mode read it (set here, outside any capture, so a replay sees this step's value)
    if (st->use_graph && p.g.kv) PS_HIP(launch_set_u32(reinterpret_cast<uint32_t *>(st->ws_base + p.ws.ctx), st->ctx, st->compute));
    if (st->use_graph && !prof) {
        // Launch-bound case (every shard resident; one token or a batched-decode step): the kernel
        // sequence is captured once per (x_in, x_out, logits, rows) and replayed.  Kernel nodes only.
        auto key = std::make_tuple(static_cast<const void *>(x_in), static_cast<void *>(x_out),
                                   static_cast<void *>(st->head_rows ? st->logits : nullptr),
                                   st->n_valid | (st->head_rows << 8) | (st->head_row0 << 16));
        auto it = st->graphs.find(key);
        if (it == st->graphs.end()) {
            if (st->graphs.size() >= 32) {
                // forward is asynchronous: the latest replays may still be running, and an executable
                // graph must not be destroyed while it is in flight
                PS_HIP(hipStreamSynchronize(st->compute));
                for (auto &g : st->graphs) (void)hipGraphExecDestroy(g.second);
                st->graphs.clear();
            }
            hipGraph_t graph = nullptr;
            PS_HIP(hipStreamBeginCapture(st->compute, hipStreamCaptureModeThreadLocal));
            int32_t rc = PS_OK;
            for (const Op &op : sc.ops) {
                if (skip_head_op(st, op)) continue;
                rc = issue_kernel(st, sc, op, x_in, x_out);
                if (rc) break;
            }
            hipError_t e = hipStreamEndCapture(st->compute, &graph);
            if (rc) { if (graph) (void)hipGraphDestroy(graph); return rc; }
            if (e != hipSuccess) { ps::set_error("hipStreamEndCapture failed: %s", hipGetErrorString(e)); return PS_E_HIP; }
            hipGraphExec_t exec = nullptr;
            e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
            (void)hipGraphDestroy(graph);
            if (e != hipSuccess) { ps::set_error("hipGraphInstantiate failed: %s", hipGetErrorString(e)); return PS_E_HIP; }
            it = st->graphs.emplace(key, exec).first;
        }
        PS_HIP(hipGraphLaunch(it->second, st->compute));
        ss.graph_replay = 1;
        for (const Op &op : sc.ops)
            if (!skip_head_op(st, op)) { ss.resident_bytes_step += op.info.bytes; ss.n_kernels++; }
        return PS_OK;
    }
    for (size_t i = 0; i < sc.ops.size(); ++i) {
        const Op &op = sc.ops[i];
        const ps_op_info &o = op.info;
        if (skip_head_op(st, op)) {
            if (prof) {   // keeps one (empty) interval per op
                PS_HIP(hipEventRecord(st->prof_ev[2 * i], st->compute));
                PS_HIP(hipEventRecord(st->prof_ev[2 * i + 1], st->compute));
            }
            continue;
        }
        if (o.type == PS_OP_COPY) {
            // One-token steps: a streamed expert fill that is its layer's only one goes out on the
            // compute stream.  It can start only when the router has run and the layer's streamed
            // experts can start only when it has landed, so the copy stream would add two cross-stream
            // event hand-overs and hide only the launch of the resident experts, which at one token is
            // shorter than the hand-overs (with more tokens it is not, and the copy stream keeps the
            // fill).  Stream order stands in for both waits.
            const bool inl = st->inline_fill && st->n_valid == 1 && (o.flags & PS_OPF_WAIT_ROUTER) && only_fill_of_layer(sc, i);
            const hipStream_t cps = inl ? st->compute : st->copy;
            if (!inl) {
                if (o.flags & PS_OPF_WAIT_SLOT_FREE) PS_HIP(hipStreamWaitEvent(st->copy, st->ev_free[o.slot], 0));
                if (o.flags & PS_OPF_WAIT_ROUTER) PS_HIP(hipStreamWaitEvent(st->copy, st->ev_router[o.layer], 0));
            }
            if (prof) { PS_HIP(hipEventRecord(st->prof_ev[2 * i], cps)); st->prof_is_copy[i] = 1; }
            size_t last = i;
            const bool expert_gather = st->gather_copy && p.shards[o.shard0].kind == PS_SHARD_EXPERT && st->tables_host[0];
            const bool dense_gather = st->gather_dense && st->dense_descs && &sc == &st->dense_sched && p.shards[o.shard0].kind != PS_SHARD_KV;
            if (expert_gather || dense_gather) {
                // the rest of this slot fill follows in the op list: one gather launch for all of it
                // (a dense schedule never changes between forwards: its descriptors sit at the ops' own
                // indices and are rewritten with the same values)
                ps::CopyDesc *descs = dense_gather ? st->dense_descs + i : reinterpret_cast<ps::CopyDesc *>(
                    static_cast<uint8_t *>(st->tables_host[st->table_idx]) + st->descs_off) + st->n_descs;
                uint32_t n = 0;
                for (size_t j = i; j < sc.ops.size(); ++j) {
                    const ps_op_info &c = sc.ops[j].info;
                    if (c.type != PS_OP_COPY || c.slot != o.slot || (j > i && (c.flags & PS_OPF_WAIT_SLOT_FREE))) break;
                    if (dense_gather && p.shards[c.shard0].kind == PS_SHARD_KV) break;
                    descs[n].src = (uint64_t)(uintptr_t)st->shard_host[c.shard0];
                    descs[n].dst = (uint64_t)(uintptr_t)(slot_ptr(st, c.slot) + c.slot_offset);
                    descs[n].n16 = (uint32_t)(c.bytes / 16);
                    ++n;
                    last = j;
                    ss.streamed_bytes_step += c.bytes;
                    ss.n_copies++;
                    if (prof && j > i) {   // the batch's time is booked on its first op
                        PS_HIP(hipEventRecord(st->prof_ev[2 * j], cps));
                        PS_HIP(hipEventRecord(st->prof_ev[2 * j + 1], cps));
                        st->prof_is_copy[j] = 1;
                    }
                    if (c.flags & PS_OPF_RECORD_READY) break;
                }
                if (!dense_gather) st->n_descs += n;
                PS_HIP(launch_h2d_gather(descs, n, cps));
            } else if (p.shards[o.shard0].kind == PS_SHARD_KV) {
                // a cache shard: only the rows the step attends over cross PCIe (K rows, then V rows)
                const uint64_t rows_b = (uint64_t)st->ctx * p.g.m.head_dim * 2, vbase = (uint64_t)p.g.m.kv_context * p.g.m.head_dim * 2;
                if (rows_b) {
                    uint8_t *dst = slot_ptr(st, o.slot) + o.slot_offset;
                    PS_HIP(hipMemcpyAsync(dst, st->shard_host[o.shard0], rows_b, hipMemcpyHostToDevice, cps));
                    PS_HIP(hipMemcpyAsync(dst + vbase, st->shard_host[o.shard0] + vbase, rows_b, hipMemcpyHostToDevice, cps));
                    ss.streamed_bytes_step += 2 * rows_b;
                    ss.n_copies += 2;
                }
            } else {
                PS_HIP(hipMemcpyAsync(slot_ptr(st, o.slot) + o.slot_offset, st->shard_host[o.shard0], o.bytes,
                                      hipMemcpyHostToDevice, cps));
                ss.streamed_bytes_step += o.bytes;
                ss.n_copies++;
            }
            if (prof) PS_HIP(hipEventRecord(st->prof_ev[2 * i + 1], cps));
            if (sc.ops[last].info.flags & PS_OPF_RECORD_READY) PS_HIP(hipEventRecord(st->ev_ready[o.slot], cps));
            i = last;
        } else {
            if (o.flags & PS_OPF_WAIT_READY) PS_HIP(hipStreamWaitEvent(st->compute, st->ev_ready[o.slot], 0));
            if (prof) PS_HIP(hipEventRecord(st->prof_ev[2 * i], st->compute));
            // RMS factors left by a residual epilogue are good only for the PS_K_RINV op right behind it
            if (!(o.type == PS_OP_KERNEL && o.kernel == PS_K_RINV)) st->rinv_of = nullptr;
            int32_t rc = o.type == PS_OP_FETCH ? issue_fetch(st, op, x_in, x_out)
                         : o.type == PS_OP_CPU ? issue_cpu(st, sc, op, x_out) : issue_kernel(st, sc, op, x_in, x_out);
            if (rc) return rc;
            if (prof) PS_HIP(hipEventRecord(st->prof_ev[2 * i + 1], st->compute));
            if (o.flags & PS_OPF_RECORD_FREE) PS_HIP(hipEventRecord(st->ev_free[o.slot], st->compute));
            if (o.flags & PS_OPF_RECORD_ROUTER) PS_HIP(hipEventRecord(st->ev_router[o.layer], st->compute));
            if (o.type == PS_OP_KERNEL) {
                if (o.slot < 0) ss.resident_bytes_step += o.bytes;
                ss.n_kernels++;
            }
        }
    }
    st->prof_valid = prof;
    return PS_OK;
}

}  // namespace

extern "C" {

}  // extern "C"

namespace {

// Whether a dense plan's streamed slabs should cross PCIe through the gather kernel rather than
// hipMemcpyAsync.  Measured on the 8B-shaped stack: the kernel keeps the link at 98 % of the pinned
// H2D rate where back-to-back hipMemcpyAsync calls leave about 60 us between copies (90 %), but a
// kernel that runs beside it is several times slower (its loads queue behind the PCIe reads on the
// CUs the gather occupies).  So it pays where the step is copy time almost alone: the plan's copy
// estimate at least ten times its kernel estimate (one-token decode at 2 GB: 36 ms against 1 ms,
// 40.3 -> 37.0 ms per token; the 295 MB head beside 1 ms of resident decode, ratio 5: 6.4 -> 7.1 ms).
// mode: 0 never, 1 by this rule, 2 always.
bool dense_gather_pays(const ps_plan &p, int32_t mode) {
    if (mode != 1) return mode == 2;
    if (!(p.prof.h2d_gbps > 0) || !(p.prof.gemv_gbps > 0) || p.streamed_bytes == 0) return false;
    const double tf = p.prof.gemm_tflops[p.tier];
    double copy_ms = 0, kernel_ms = 0;
    for (const ps::Shard &sh : p.shards) {
        if (sh.resident == 2) continue;
        const double t_mem = (double)sh.bytes / (p.prof.gemv_gbps * 1e9);
        const double t_cmp = tf > 0 ? 2.0 * p.M * ((double)sh.bytes / 0.5625) / (tf * 1e12) : 0;
        kernel_ms += std::max(t_mem, t_cmp) * 1e3;
        if (!sh.resident) copy_ms += (double)sh.bytes / (p.prof.h2d_gbps * 1e9) * 1e3;
    }
    return copy_ms >= 10.0 * kernel_ms;
}

// tile size of the matrix a shard is cut from (0: whole shards, never split)
uint64_t shard_tile_bytes(const ps::ModelGeom &g, uint32_t kind) {
    switch (kind) {
        case PS_SHARD_QKV: return g.qkv.tile_bytes;
        case PS_SHARD_O: return g.o.tile_bytes;
        case PS_SHARD_GATE_UP: return g.gate_up.tile_bytes;
        case PS_SHARD_DOWN: return g.down.tile_bytes;
        case PS_SHARD_OUT: return g.head.tile_bytes;
    }
    return 0;
}

// Everything a stack derives from its current plan (Algorithm 1, SetupForSched): where the workspace
// lies, where each shard's host copy is, which shards cover which matrix, the dense schedule.
int32_t bind_plan(ps_stack *st) {
    const ps_plan &p = st->plan;
    st->n_valid = p.M;
    st->ws_base = st->arena + p.ws_off;
    st->cover.clear();
    for (size_t i = 0; i < p.shards.size(); ++i)
        st->cover[std::make_tuple(p.shards[i].layer, p.shards[i].kind, p.shards[i].expert)].push_back((uint32_t)i);
    if (st->multi) {   // every shard is a run of tiles of its matrix's image
        st->shard_host.assign(p.shards.size(), nullptr);
        for (size_t i = 0; i < p.shards.size(); ++i) {
            const ps::Shard &sh = p.shards[i];
            auto it = st->image.find(std::make_tuple(sh.layer, sh.kind, sh.expert));
            if (it == st->image.end()) { ps::set_error("internal: shard without a matrix image"); return PS_E_STATE; }
            st->shard_host[i] = it->second + (uint64_t)sh.tile0 * shard_tile_bytes(p.g, sh.kind);
        }
    }
    if (p.g.moe) {
        st->descs_off = ps::align_up(p.ws.logits_bytes + p.ws.tasks_bytes + p.ws.pairs_bytes, 256);
    } else {
        st->dense_sched = ps_schedule();
        int32_t rc = ps::build_schedule(&st->plan, nullptr, &st->dense_sched);
        if (rc) return rc;
        rc = ps::validate_schedule(&st->dense_sched);
        if (rc) return rc;
        st->have_dense_sched = true;
        st->gather_dense = dense_gather_pays(p, st->copy_mode);
        if (st->dense_sched.ops.size() > st->dense_descs_cap) {
            if (st->dense_descs) (void)hipHostFree(st->dense_descs);
            st->dense_descs = nullptr;
            st->dense_descs_cap = 0;
            void *d = nullptr;
            if (hipHostMalloc(&d, st->dense_sched.ops.size() * sizeof(ps::CopyDesc), hipHostMallocDefault) != hipSuccess) {
                ps::set_error("hipHostMalloc for copy descriptors failed"); return PS_E_HIP;
            }
            st->dense_descs = static_cast<ps::CopyDesc *>(d);
            st->dense_descs_cap = st->dense_sched.ops.size();
        }
    }
    st->use_graph = st->decode_mode == 1 && graph_eligible(p) && st->have_dense_sched;
    if (p.g.kv) {
        // home of every kv head's cache: where its rows live between steps (arena or pinned pool)
        const auto &m = p.g.m;
        std::vector<uint64_t> home((size_t)m.n_layers * m.n_kv_heads, 0);
        st->kv_copied = false;
        for (size_t i = 0; i < p.shards.size(); ++i) {
            const ps::Shard &s = p.shards[i];
            if (s.kind != PS_SHARD_KV) continue;
            if (!s.resident) st->kv_copied = true;
            home[(size_t)s.layer * m.n_kv_heads + s.expert] =
                (uint64_t)(uintptr_t)(s.resident ? st->arena + s.offset : st->shard_host[i]);
        }
        PS_HIP(hipMemcpy(st->ws_base + p.ws.kvhome, home.data(), home.size() * 8, hipMemcpyHostToDevice));
    }
    return PS_OK;
}

// plans: one plan (ps_stack_create), or the PS_NTIERS plans of a tier table (null where infeasible)
int32_t stack_create_impl(const std::vector<const ps_plan *> &plans, bool multi, void *vram_arena, uint64_t arena_bytes,
                          void *compute_stream, void *copy_stream, ps_stack **out) {
    const ps_plan *plan = nullptr;       // the plan installed first: the lowest feasible tier (it pins the most)
    uint32_t first = 0;
    for (uint32_t t = 0; t < plans.size() && !plan; ++t)
        if (plans[t]) { plan = plans[t]; first = t; }
    if (!plan) { ps::set_error("no feasible tier"); return PS_E_BUDGET; }
    if (arena_bytes < plan->budget) {
        ps::set_error("arena of %llu B is smaller than the plan's budget %llu B", (unsigned long long)arena_bytes,
                      (unsigned long long)plan->budget);
        return PS_E_ARG;
    }
    if ((uintptr_t)vram_arena % ps::kAlign) { ps::set_error("arena must be 256-byte aligned"); return PS_E_ARG; }
    bool any_slots = false;
    for (const ps_plan *q : plans) {
        if (!q) continue;
        any_slots |= q->n_slots != 0;
    }
    if (compute_stream == copy_stream && any_slots) {
        ps::set_error("streamed shards need distinct compute and copy streams"); return PS_E_ARG;
    }
    ps_stack *st = new (std::nothrow) ps_stack();
    if (!st) { ps::set_error("out of host memory"); return PS_E_NOMEM; }
    st->plan = *plan;
    st->multi = multi;
    if (multi) {
        st->tiers.resize(plans.size());
        for (size_t t = 0; t < plans.size(); ++t)
            if (plans[t]) st->tiers[t] = *plans[t];
        st->active_tier = first;
    }
    st->n_valid = plan->M;
    st->arena = static_cast<uint8_t *>(vram_arena);
    st->ws_base = st->arena + plan->ws_off;
    {   // set-up for ps_stack_forward_noalloc: this device's address of the static scratch
        const int32_t rc = static_scratch(&st->static_ws);
        if (rc) { delete st; return rc; }
    }
    st->arena_bytes = arena_bytes;
    st->compute = static_cast<hipStream_t>(compute_stream);
    st->copy = static_cast<hipStream_t>(copy_stream);
    auto fail = [&](int32_t rc) { ps_stack_destroy(st); return rc; };

    const ps_plan &p = st->plan;
    const auto &m = p.g.m;
    // host pools for streamed shards: chunks of at most 1 GiB, a shard never straddles chunks
    st->shard_host.assign(p.shards.size(), nullptr);
    if (multi) {
        // one image per matrix (per expert), whatever the tiers do with it: any tier's shard is a run
        // of its tiles, and a shard that another tier's workspace displaced can be pinned again from it
        std::vector<std::pair<std::tuple<uint32_t, uint32_t, uint32_t>, uint64_t>> mats;
        for (uint32_t l = 0; l < m.n_layers; ++l) {
            if (p.g.has_attn) {
                mats.push_back({std::make_tuple(l, (uint32_t)PS_SHARD_QKV, ps::kNoExpert), p.g.qkv.bytes});
                mats.push_back({std::make_tuple(l, (uint32_t)PS_SHARD_O, ps::kNoExpert), p.g.o.bytes});
                // a cache shard's host home, used by the tiers that do not pin it
                if (p.g.kv) for (uint32_t h = 0; h < m.n_kv_heads; ++h) mats.push_back({std::make_tuple(l, (uint32_t)PS_SHARD_KV, h), p.g.kv_shard_bytes});
            }
            if (!p.g.moe) {
                mats.push_back({std::make_tuple(l, (uint32_t)PS_SHARD_GATE_UP, ps::kNoExpert), p.g.gate_up.bytes});
                mats.push_back({std::make_tuple(l, (uint32_t)PS_SHARD_DOWN, ps::kNoExpert), p.g.down.bytes});
            } else {
                for (uint32_t e = 0; e < m.n_experts; ++e) mats.push_back({std::make_tuple(l, (uint32_t)PS_SHARD_EXPERT, e), p.g.expert_bytes});
            }
        }
        if (m.vocab) mats.push_back({std::make_tuple(m.n_layers, (uint32_t)PS_SHARD_OUT, ps::kNoExpert), p.g.head.bytes});
        std::vector<uint64_t> chunk_bytes;
        std::vector<std::pair<size_t, uint64_t>> place(mats.size());
        for (size_t i = 0; i < mats.size(); ++i) {
            if (chunk_bytes.empty() || chunk_bytes.back() + mats[i].second > kHostChunk) chunk_bytes.push_back(0);
            place[i] = {chunk_bytes.size() - 1, chunk_bytes.back()};
            chunk_bytes.back() += mats[i].second;
        }
        for (uint64_t b : chunk_bytes) {
            void *ptr = nullptr;
            hipError_t e = hipHostMalloc(&ptr, b, hipHostMallocDefault);
            if (e != hipSuccess) { ps::set_error("hipHostMalloc(%llu) failed: %s", (unsigned long long)b, hipGetErrorString(e)); return fail(PS_E_HIP); }
            st->host_chunks.push_back(ptr);
        }
        for (size_t i = 0; i < mats.size(); ++i)
            st->image[mats[i].first] = static_cast<uint8_t *>(st->host_chunks[place[i].first]) + place[i].second;
    } else {
        std::vector<std::pair<size_t, uint64_t>> place(p.shards.size());  // chunk, offset
        std::vector<uint64_t> chunk_bytes;
        for (size_t i = 0; i < p.shards.size(); ++i) {
            if (p.shards[i].resident == 1) continue;
            if (chunk_bytes.empty() || chunk_bytes.back() + p.shards[i].bytes > kHostChunk) chunk_bytes.push_back(0);
            place[i] = {chunk_bytes.size() - 1, chunk_bytes.back()};
            chunk_bytes.back() += p.shards[i].bytes;
        }
        for (uint64_t b : chunk_bytes) {
            void *ptr = nullptr;
            hipError_t e = hipHostMalloc(&ptr, b, hipHostMallocDefault);
            if (e != hipSuccess) { ps::set_error("hipHostMalloc(%llu) failed: %s", (unsigned long long)b, hipGetErrorString(e)); return fail(PS_E_HIP); }
            st->host_chunks.push_back(ptr);
        }
        for (size_t i = 0; i < p.shards.size(); ++i)
            if (p.shards[i].resident != 1) st->shard_host[i] = static_cast<uint8_t *>(st->host_chunks[place[i].first]) + place[i].second;
    }
    const uint32_t per_layer = (p.g.has_attn ? 2 : 0) + 3 * (p.g.moe ? m.n_experts : 1);
    st->n_expected = (uint64_t)per_layer * m.n_layers + (m.vocab ? 1 : 0);
    st->loaded.assign(st->n_expected, 0);

    for (int s = 0; s < 2; ++s) {
        if (hipEventCreateWithFlags(&st->ev_ready[s], hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&st->ev_free[s], hipEventDisableTiming) != hipSuccess) {
            ps::set_error("hipEventCreate failed"); return fail(PS_E_HIP);
        }
    }
    if (p.g.moe) {
        st->ev_router.resize(m.n_layers);
        for (auto &e : st->ev_router)
            if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) { ps::set_error("hipEventCreate failed"); return fail(PS_E_HIP); }
        for (const ps_plan *q : plans) {   // room for the largest tier's tables
            if (!q) continue;
            const uint64_t d = ps::align_up(q->ws.logits_bytes + q->ws.tasks_bytes + q->ws.pairs_bytes, 256);
            st->tables_bytes = std::max(st->tables_bytes, d + (q->ws.tasks_bytes / sizeof(ps::DeviceTask)) * sizeof(ps::CopyDesc));
        }
        for (int b = 0; b < 2; ++b) {
            if (hipEventCreateWithFlags(&st->ev_upload[b], hipEventDisableTiming) != hipSuccess) { ps::set_error("hipEventCreate failed"); return fail(PS_E_HIP); }
            if (hipHostMalloc(&st->tables_host[b], st->tables_bytes, hipHostMallocDefault) != hipSuccess) {
                ps::set_error("hipHostMalloc for routing tables failed"); return fail(PS_E_HIP);
            }
        }
    }
    {
        const int32_t rc = bind_plan(st);
        if (rc) return fail(rc);
    }
    uint32_t cpu_M = 0;     // most tokens of any plan that leaves shards to the CPU (several tiers: each may)
    for (const ps_plan *q : plans)
        if (q && q->cpu_bytes) cpu_M = std::max(cpu_M, q->M);
    if (cpu_M) {
        if (!ps::cpu_backend_supported()) { ps::set_error("the CPU back-end needs AVX-512 (F, BW, VL, DQ) and F16C"); return fail(PS_E_STATE); }
        const uint32_t H = m.hidden, I = p.g.ffn_i;
        const size_t widest = std::max<size_t>(std::max(H, I), m.vocab);
        const size_t P = (size_t)cpu_M * std::max(1u, m.top_k);
        void *bufs[4] = {};
        // host_out doubles as the CPU experts' landing image: fp32 rows [P][H], then P pair numbers
        const size_t sizes[4] = {(size_t)cpu_M * H * 2, (size_t)cpu_M * I * 2, (size_t)cpu_M * H * 2,
                                 std::max((size_t)cpu_M * widest * 2, p.g.moe ? P * H * 4 + P * 4 : 0)};
        if (p.g.moe) { st->cpu_xg.resize(P * H); st->cpu_sg.resize(P * I); }
        for (int b = 0; b < 4; ++b)
            if (hipHostMalloc(&bufs[b], sizes[b], hipHostMallocDefault) != hipSuccess) {
                for (int c = 0; c < b; ++c) (void)hipHostFree(bufs[c]);
                ps::set_error("hipHostMalloc for the CPU back-end's activation copies failed"); return fail(PS_E_HIP);
            }
        st->host_h = static_cast<uint16_t *>(bufs[0]); st->host_s = static_cast<uint16_t *>(bufs[1]);
        st->host_x = static_cast<uint16_t *>(bufs[2]); st->host_out = static_cast<uint16_t *>(bufs[3]);
        st->cpu_scratch.resize(ps::cpu_scratch_floats(cpu_M, std::max(H, I)));
        const unsigned hw = std::thread::hardware_concurrency();
        st->pool.reset(new ps::CpuPool(std::min(hw ? hw : 4u, 16u)));
    }
    st->stage_bytes = 32ull << 20;
    if (hipHostMalloc(&st->stage, st->stage_bytes, hipHostMallocDefault) != hipSuccess) {
        ps::set_error("hipHostMalloc for staging failed"); return fail(PS_E_HIP);
    }
    if (p.g.kv && hipEventCreateWithFlags(&st->ev_step, hipEventDisableTiming) != hipSuccess) {
        ps::set_error("KV cache set-up failed"); return fail(PS_E_HIP);
    }
    *out = st;
    return PS_OK;
}

// [C, end of arena) is about to be, or has been, used as scratch and workspace: what was pinned there is gone
void clobber_from(ps_stack *st, uint64_t C) {
    std::vector<ps_stack::Content> keep;
    for (ps_stack::Content r : st->content) {
        if (r.off + r.bytes <= C) { keep.push_back(r); continue; }
        if (r.off >= C || !r.tile_bytes) continue;
        const uint64_t nt = (C - r.off) / r.tile_bytes;      // whole tiles in front of C survive
        if (!nt) continue;
        r.bytes = nt * r.tile_bytes;
        keep.push_back(r);
    }
    st->content.swap(keep);
}

void note_content(ps_stack *st, const ps::Shard &sh) {
    const uint64_t tb = shard_tile_bytes(st->plan.g, sh.kind);
    for (const ps_stack::Content &r : st->content)
        if (r.off == sh.offset && r.bytes == sh.bytes && r.layer == sh.layer && r.kind == sh.kind && r.expert == sh.expert && r.tile0 == sh.tile0) return;
    std::vector<ps_stack::Content> keep;
    for (const ps_stack::Content &r : st->content)
        if (r.off + r.bytes <= sh.offset || r.off >= sh.offset + sh.bytes) keep.push_back(r);
    keep.push_back(ps_stack::Content{sh.offset, sh.bytes, tb, sh.layer, sh.kind, sh.expert, sh.tile0});
    st->content.swap(keep);
}

}  // namespace

extern "C" {

int32_t ps_stack_create(const ps_plan *plan, void *vram_arena, uint64_t arena_bytes, void *compute_stream,
                        void *copy_stream, ps_stack **out) {
    if (!plan || !vram_arena || !out) { ps::set_error("NULL argument"); return PS_E_ARG; }
    *out = nullptr;
    return stack_create_impl({plan}, false, vram_arena, arena_bytes, compute_stream, copy_stream, out);
}

int32_t ps_stack_create_tiers(const ps_tier_table *table, void *vram_arena, uint64_t arena_bytes, void *compute_stream,
                              void *copy_stream, ps_stack **out) {
    if (!table || !vram_arena || !out) { ps::set_error("NULL argument"); return PS_E_ARG; }
    *out = nullptr;
    std::vector<const ps_plan *> plans(table->plans, table->plans + PS_NTIERS);
    return stack_create_impl(plans, true, vram_arena, arena_bytes, compute_stream, copy_stream, out);
}

int32_t ps_stack_tier(const ps_stack *st, uint32_t *tier, uint32_t *n_tokens) {
    if (!st || !tier || !n_tokens) { ps::set_error("NULL argument"); return PS_E_ARG; }
    *tier = st->multi ? st->active_tier : st->plan.tier;
    *n_tokens = st->plan.M;
    return PS_OK;
}

int32_t ps_stack_set_tier(ps_stack *st, uint32_t tier, uint64_t *uploaded_bytes) {
    if (!st) { ps::set_error("NULL argument"); return PS_E_ARG; }
    if (uploaded_bytes) *uploaded_bytes = 0;
    if (!st->multi) { ps::set_error("this stack was created for one plan (use ps_stack_create_tiers)"); return PS_E_STATE; }
    if (tier >= st->tiers.size() || st->tiers[tier].M == 0) { ps::set_error("tier %u has no plan under this budget", tier); return PS_E_ARG; }
    if (st->n_loaded != st->n_expected) { ps::set_error("set the tier once all matrices are loaded"); return PS_E_STATE; }
    // no forward of the old tier may be in flight while its workspace moves and shards are pinned again
    PS_HIP(hipStreamSynchronize(st->copy));
    PS_HIP(hipStreamSynchronize(st->compute));
    if (tier == st->active_tier) return PS_OK;
    for (auto &g : st->graphs) (void)hipGraphExecDestroy(g.second);
    st->graphs.clear();
    // KV caches are state, not copies of something on the host: a cache shard whose home changes
    // with the tier (pinned in one, streamed in the other) moves with its rows, through its host home
    std::map<std::pair<uint32_t, uint32_t>, std::pair<uint32_t, uint64_t>> old_kv;   // (layer, head) -> (resident, offset)
    const uint64_t kv_rows_b = (uint64_t)st->kv_rows * st->plan.g.m.head_dim * 2;
    const uint64_t kv_vbase = (uint64_t)st->plan.g.m.kv_context * st->plan.g.m.head_dim * 2;
    uint64_t moved = 0;
    if (st->plan.g.kv) {
        const ps_plan &np = st->tiers[tier];
        std::map<std::pair<uint32_t, uint32_t>, std::pair<uint32_t, uint64_t>> new_kv;
        for (const ps::Shard &sh : np.shards)
            if (sh.kind == PS_SHARD_KV) new_kv[{sh.layer, sh.expert}] = {sh.resident, sh.offset};
        for (size_t i = 0; i < st->plan.shards.size(); ++i) {
            const ps::Shard &sh = st->plan.shards[i];
            if (sh.kind != PS_SHARD_KV) continue;
            old_kv[{sh.layer, sh.expert}] = {sh.resident, sh.offset};
            const auto nk = new_kv[{sh.layer, sh.expert}];
            if (sh.resident == 1 && kv_rows_b && (nk.first != 1 || nk.second != sh.offset)) {
                PS_HIP(hipMemcpy(st->shard_host[i], st->arena + sh.offset, kv_rows_b, hipMemcpyDeviceToHost));
                PS_HIP(hipMemcpy(st->shard_host[i] + kv_vbase, st->arena + sh.offset + kv_vbase, kv_rows_b, hipMemcpyDeviceToHost));
                moved += 2 * kv_rows_b;
            }
        }
    }
    // the tier that ran until now used the tail of the arena from its slots on; so will the new one
    clobber_from(st, std::min(st->plan.scratch_off, st->tiers[tier].scratch_off));
    st->plan = st->tiers[tier];
    st->active_tier = tier;
    const int32_t rc = bind_plan(st);
    if (rc) return rc;
    const ps_plan &p = st->plan;
    uint64_t up = moved;
    for (size_t i = 0; i < p.shards.size(); ++i) {
        const ps::Shard &sh = p.shards[i];
        if (sh.resident != 1) continue;
        if (sh.kind == PS_SHARD_KV) {   // back into the arena if it was not there, or not at this place
            const auto ok = old_kv[{sh.layer, sh.expert}];
            if (kv_rows_b && (ok.first != 1 || ok.second != sh.offset)) {
                PS_HIP(hipMemcpyAsync(st->arena + sh.offset, st->shard_host[i], kv_rows_b, hipMemcpyHostToDevice, st->compute));
                PS_HIP(hipMemcpyAsync(st->arena + sh.offset + kv_vbase, st->shard_host[i] + kv_vbase, kv_rows_b, hipMemcpyHostToDevice, st->compute));
                up += 2 * kv_rows_b;
            }
            note_content(st, sh);
            continue;
        }
        // bytes of the shard already in place: a record of the same matrix under the same tile -> address map
        uint64_t have = 0;
        const uint64_t tb = shard_tile_bytes(p.g, sh.kind);
        for (const ps_stack::Content &r : st->content) {
            if (r.layer != sh.layer || r.kind != sh.kind || r.expert != sh.expert) continue;
            if (r.off - (uint64_t)r.tile0 * tb != sh.offset - (uint64_t)sh.tile0 * tb) continue;
            if (r.off <= sh.offset && r.off + r.bytes > sh.offset) have = std::max(have, std::min(sh.bytes, r.off + r.bytes - sh.offset));
        }
        if (have < sh.bytes) {
            PS_HIP(hipMemcpyAsync(st->arena + sh.offset + have, st->shard_host[i] + have, sh.bytes - have, hipMemcpyHostToDevice, st->compute));
            up += sh.bytes - have;
        }
        note_content(st, sh);
    }
    PS_HIP(hipStreamSynchronize(st->compute));
    if (uploaded_bytes) *uploaded_bytes = up;
    return PS_OK;
}

int32_t ps_stack_load_matrix(ps_stack *st, uint32_t layer, uint32_t mat, uint32_t expert,
                             const uint16_t *scales, const uint8_t *codes) {
    if (!st || !scales || !codes) { ps::set_error("NULL argument"); return PS_E_ARG; }
    const ps_plan &p = st->plan;
    const ps::ModelGeom &g = p.g;
    const auto &m = g.m;
    const bool is_head = mat == PS_MAT_OUT;
    if (is_head ? (!m.vocab || layer != m.n_layers) : (layer >= m.n_layers || mat > PS_MAT_DOWN)) {
        ps::set_error("bad layer/matrix id"); return PS_E_ARG;
    }
    const bool is_attn = mat == PS_MAT_QKV || mat == PS_MAT_O;
    if (is_attn && !g.has_attn) { ps::set_error("model has no attention matrices"); return PS_E_ARG; }
    if (g.moe && !is_attn && !is_head) {
        if (expert >= m.n_experts) { ps::set_error("expert id %u out of range", expert); return PS_E_ARG; }
    } else if (expert != ps::kNoExpert) {
        ps::set_error("expert must be 0xFFFFFFFF for this matrix"); return PS_E_ARG;
    }
    uint32_t kind;
    if (is_attn) kind = mat == PS_MAT_QKV ? PS_SHARD_QKV : PS_SHARD_O;
    else if (is_head) kind = PS_SHARD_OUT;
    else if (g.moe) kind = PS_SHARD_EXPERT;
    else kind = mat == PS_MAT_DOWN ? PS_SHARD_DOWN : PS_SHARD_GATE_UP;
    auto it = st->cover.find(std::make_tuple(layer, kind, kind == PS_SHARD_EXPERT ? expert : ps::kNoExpert));
    if (it == st->cover.end()) { ps::set_error("internal: no shard covers this matrix"); return PS_E_STATE; }
    const ps::MatGeom &mg = geom_of(g, mat);
    const bool paired = mat == PS_MAT_GATE || mat == PS_MAT_UP;
    const uint32_t parity = mat == PS_MAT_UP ? 1 : 0;
    const uint32_t step = paired ? 2 : 1;
    const uint64_t pitch = mg.tile_bytes * step;

    if (st->multi) {
        // the whole matrix goes into its host image; what the installed tier pinned of it is copied
        // from there to the arena and noted as that stretch's content
        auto im = st->image.find(std::make_tuple(layer, kind, kind == PS_SHARD_EXPERT ? expert : ps::kNoExpert));
        if (im == st->image.end()) { ps::set_error("internal: no image for this matrix"); return PS_E_STATE; }
        const bool ex = kind == PS_SHARD_EXPERT;
        const uint32_t nt_all = ex ? (mat == PS_MAT_DOWN ? g.down.ntiles : g.gate_up.ntiles) : mg.ntiles;
        const uint64_t base_off = ex && mat == PS_MAT_DOWN ? g.gate_up.bytes : 0;
        uint8_t *img = im->second + base_off;
        const uint32_t count_all = (nt_all + step - 1 - parity) / step;
        parallel_for(count_all, [&](uint32_t j) {
            const uint32_t pt = parity + j * step;
            ps::pack_tile(mg, scales, codes, paired ? pt / 2 : pt, img + (uint64_t)pt * mg.tile_bytes);
        });
        for (uint32_t si : it->second) {
            const ps::Shard &s = p.shards[si];
            if (s.resident != 1) continue;
            const uint32_t t0 = ex ? 0 : s.tile0, nt = ex ? nt_all : s.ntiles;
            const uint32_t n = (nt + step - 1 - parity) / step;
            PS_HIP(hipMemcpy2D(st->arena + s.offset + base_off + (uint64_t)parity * mg.tile_bytes, pitch,
                               img + (uint64_t)(t0 + parity) * mg.tile_bytes, pitch, mg.tile_bytes, n, hipMemcpyHostToDevice));
            note_content(st, s);
        }
    } else
    for (uint32_t si : it->second) {
        const ps::Shard &s = p.shards[si];
        uint32_t t0 = s.tile0, nt = s.ntiles;
        uint64_t base_off = 0;
        if (kind == PS_SHARD_EXPERT) {
            t0 = 0;
            nt = mat == PS_MAT_DOWN ? g.down.ntiles : g.gate_up.ntiles;
            base_off = mat == PS_MAT_DOWN ? g.gate_up.bytes : 0;
        }
        // physical tiles t0 + parity, t0 + parity + step, ... (t0 is even for paired matrices)
        const uint32_t count = (nt + step - 1 - parity) / step;
        if (s.resident != 1) {
            uint8_t *dst = st->shard_host[si] + base_off;
            parallel_for(count, [&](uint32_t j) {
                const uint32_t pt = t0 + parity + j * step;
                ps::pack_tile(mg, scales, codes, paired ? pt / 2 : pt, dst + (uint64_t)(pt - t0) * mg.tile_bytes);
            });
        } else {
            uint8_t *dst = st->arena + s.offset + base_off;
            const uint32_t per = (uint32_t)(st->stage_bytes / mg.tile_bytes);
            for (uint32_t j0 = 0; j0 < count; j0 += per) {
                const uint32_t n = std::min(per, count - j0);
                uint8_t *stg = static_cast<uint8_t *>(st->stage);
                parallel_for(n, [&](uint32_t j) {
                    const uint32_t pt = t0 + parity + (j0 + j) * step;
                    ps::pack_tile(mg, scales, codes, paired ? pt / 2 : pt, stg + (uint64_t)j * mg.tile_bytes);
                });
                uint8_t *d = dst + (uint64_t)(parity + j0 * step) * mg.tile_bytes;
                PS_HIP(hipMemcpy2D(d, pitch, stg, mg.tile_bytes, mg.tile_bytes, n, hipMemcpyHostToDevice));
            }
        }
    }
    const uint32_t per_layer = (g.has_attn ? 2 : 0) + 3 * (g.moe ? m.n_experts : 1);
    uint32_t slot;
    if (is_head) slot = 0;   // the one entry after the last layer's
    else if (is_attn) slot = mat == PS_MAT_QKV ? 0 : 1;
    else slot = (g.has_attn ? 2 : 0) + 3 * (g.moe ? expert : 0) + (mat - PS_MAT_GATE);
    uint8_t &flag = st->loaded[(size_t)layer * per_layer + slot];
    if (!flag) { flag = 1; st->n_loaded++; }
    return PS_OK;
}

int32_t ps_stack_load_kv(ps_stack *st, uint32_t layer, uint32_t kv_head, const uint16_t *k_rows,
                         const uint16_t *v_rows, uint32_t n_pos) {
    if (!st || (n_pos && (!k_rows || !v_rows))) { ps::set_error("NULL argument"); return PS_E_ARG; }
    const ps_plan &p = st->plan;
    const auto &m = p.g.m;
    if (!p.g.kv) { ps::set_error("this stack has no KV cache (kv_context is 0)"); return PS_E_STATE; }
    if (layer >= m.n_layers || kv_head >= m.n_kv_heads || n_pos > m.kv_context) {
        ps::set_error("KV load out of range (layer %u, head %u, %u positions)", layer, kv_head, n_pos);
        return PS_E_ARG;
    }
    auto it = st->cover.find(std::make_tuple(layer, (uint32_t)PS_SHARD_KV, kv_head));
    if (it == st->cover.end() || it->second.size() != 1) { ps::set_error("internal: no cache shard"); return PS_E_STATE; }
    const uint32_t si = it->second[0];
    const ps::Shard &s = p.shards[si];
    const size_t row_bytes = (size_t)m.head_dim * 2, vbase = (size_t)m.kv_context * row_bytes;
    if (n_pos == 0) return PS_OK;
    st->kv_rows = std::max(st->kv_rows, n_pos);
    PS_HIP(hipStreamSynchronize(st->compute));
    if (st->copy) PS_HIP(hipStreamSynchronize(st->copy));
    if (s.resident) {
        PS_HIP(hipMemcpy(st->arena + s.offset, k_rows, n_pos * row_bytes, hipMemcpyHostToDevice));
        PS_HIP(hipMemcpy(st->arena + s.offset + vbase, v_rows, n_pos * row_bytes, hipMemcpyHostToDevice));
    } else {
        std::memcpy(st->shard_host[si], k_rows, n_pos * row_bytes);
        std::memcpy(st->shard_host[si] + vbase, v_rows, n_pos * row_bytes);
    }
    return PS_OK;
}

int32_t ps_stack_set_context(ps_stack *st, uint32_t context) {
    if (!st) { ps::set_error("NULL argument"); return PS_E_ARG; }
    if (!st->plan.g.kv) { ps::set_error("this stack has no KV cache (kv_context is 0)"); return PS_E_STATE; }
    if (context >= st->plan.g.m.kv_context) {
        ps::set_error("context %u needs a cache of at least %u positions (kv_context is %u)", context, context + 1,
                      st->plan.g.m.kv_context);
        return PS_E_ARG;
    }
    st->ctx = context;
    return PS_OK;
}

int32_t ps_stack_set_logits_out(ps_stack *st, void *logits_dev, uint32_t first_token, uint32_t rows) {
    if (!st) { ps::set_error("NULL argument"); return PS_E_ARG; }
    const ps_plan &p = st->plan;
    if (!p.g.m.vocab) { ps::set_error("this stack has no output head (vocab is 0)"); return PS_E_STATE; }
    if (rows != 0 && rows != 1 && rows != p.M) {
        ps::set_error("logits rows must be 0, 1 or the plan's %u tokens (got %u)", p.M, rows); return PS_E_ARG;
    }
    if (rows && (first_token >= p.M || (rows == p.M && first_token != 0))) {
        ps::set_error("logits of tokens %u..%u asked from a plan of %u tokens", first_token, first_token + rows - 1, p.M);
        return PS_E_ARG;
    }
    if (rows && !logits_dev) { ps::set_error("logits buffer is NULL"); return PS_E_ARG; }
    if (rows && (uintptr_t)logits_dev % 16) { ps::set_error("logits buffer must be 16-byte aligned"); return PS_E_ARG; }
    st->logits = rows ? static_cast<__half *>(logits_dev) : nullptr;
    st->head_rows = rows;
    st->head_row0 = rows ? first_token : 0;
    return PS_OK;
}

int32_t ps_stack_set_cpu_threads(ps_stack *st, uint32_t threads) {
    if (!st || threads == 0 || threads > 64) { ps::set_error("threads must be 1..64"); return PS_E_ARG; }
    if (!st->plan.cpu_bytes) { ps::set_error("this plan has no CPU shard"); return PS_E_STATE; }
    st->pool.reset(new ps::CpuPool(threads));
    return PS_OK;
}

// One trip through the plan's schedule over the first n_valid of its M token rows.
// router_logits (host) / logits_dev (device, optional): token t of layer l at [l * layer_stride + t * n_experts].
static int32_t forward_impl(ps_stack *st, const void *x_in, void *x_out, const float *router_logits,
                            const float *logits_dev, uint64_t layer_stride, uint32_t n_valid) {
    const ps_plan &p = st->plan;
    st->n_valid = n_valid;
    if (p.g.kv) {
        if ((uint64_t)st->ctx + n_valid > p.g.m.kv_context) {
            ps::set_error("context %u and %u new token(s) leave no room in a cache of %u positions", st->ctx, n_valid, p.g.m.kv_context);
            return PS_E_STATE;
        }
        // this step's cache copies read rows the previous step appended from the compute stream
        if (st->kv_copied && st->step_pending) PS_HIP(hipStreamWaitEvent(st->copy, st->ev_step, 0));
    }
    if (p.g.kv) st->kv_rows = std::max(st->kv_rows, st->ctx + n_valid);   // rows this forward appends
    if (!p.g.moe) {
        const int32_t rc = run_schedule(st, st->dense_sched, static_cast<const __half *>(x_in), static_cast<__half *>(x_out));
        if (rc == PS_OK && st->kv_copied) { PS_HIP(hipEventRecord(st->ev_step, st->compute)); st->step_pending = true; }
        return rc;
    }

    if (!router_logits) { ps::set_error("MoE forward needs host router logits"); return PS_E_ARG; }
    const uint32_t E = p.g.m.n_experts, L = p.g.m.n_layers;
    ps_schedule sc;
    int32_t rc = ps::build_schedule(&st->plan, router_logits, &sc, layer_stride, n_valid);
    if (rc) return rc;
    // device tables: logits | tasks | pairs, staged in pinned memory and uploaded on the compute stream
    // two table buffers alternate, so the host can prepare a forward while the previous one runs
    st->table_idx ^= 1;
    const uint32_t tb = st->table_idx;
    if (st->upload_pending[tb]) { PS_HIP(hipEventSynchronize(st->ev_upload[tb])); st->upload_pending[tb] = false; }
    st->n_descs = 0;
    uint8_t *th = static_cast<uint8_t *>(st->tables_host[tb]);
    ps::DeviceTask *dt = reinterpret_cast<ps::DeviceTask *>(th + p.ws.logits_bytes);
    if (sc.tasks.size() * sizeof(ps::DeviceTask) > p.ws.tasks_bytes || sc.pairs.size() * 4 > p.ws.pairs_bytes) {
        ps::set_error("internal: routing tables exceed the workspace"); return PS_E_STATE;
    }
    for (size_t t = 0; t < sc.tasks.size(); ++t) {
        const ps::TaskHost &h = sc.tasks[t];
        const ps::Shard &s = p.shards[h.shard];
        // (experts run by the CPU are never launched on the GPU: their entries only keep the table dense)
        const uint8_t *w = s.resident == 1 ? st->arena + s.offset : s.resident == 2 ? st->arena : slot_ptr(st, h.slot) + h.slot_offset;
        dt[t].w_gate_up = (uint64_t)(uintptr_t)w;
        dt[t].w_down = (uint64_t)(uintptr_t)(w + p.g.gate_up.bytes);
        dt[t].pair0 = h.pair0; dt[t].npairs = h.npairs; dt[t].expert = h.expert; dt[t].pad = 0;
    }
    std::memcpy(th + p.ws.logits_bytes + p.ws.tasks_bytes, sc.pairs.data(), sc.pairs.size() * 4);
    if (logits_dev) {   // the routing kernel reads the caller's device copy in place: nothing to upload
        st->route_logits = logits_dev;
        st->route_layer_stride = layer_stride;
    } else {            // the workspace copy: [layer][M][E], the first n_valid rows of each layer filled
        float *lh = reinterpret_cast<float *>(th);
        for (uint32_t l = 0; l < L; ++l)
            std::memcpy(lh + (size_t)l * p.M * E, router_logits + (size_t)l * layer_stride, (size_t)n_valid * E * 4);
        PS_HIP(hipMemcpyAsync(st->ws_base + p.ws.logits, th, p.ws.logits_bytes, hipMemcpyHostToDevice, st->compute));
        st->route_logits = reinterpret_cast<const float *>(st->ws_base + p.ws.logits);
        st->route_layer_stride = (uint64_t)p.M * E;
    }
    if (!sc.tasks.empty())
        PS_HIP(hipMemcpyAsync(st->ws_base + p.ws.tasks, dt, sc.tasks.size() * sizeof(ps::DeviceTask), hipMemcpyHostToDevice, st->compute));
    if (!sc.pairs.empty())
        PS_HIP(hipMemcpyAsync(st->ws_base + p.ws.pairs, th + p.ws.logits_bytes + p.ws.tasks_bytes, sc.pairs.size() * 4,
                              hipMemcpyHostToDevice, st->compute));
    rc = run_schedule(st, sc, static_cast<const __half *>(x_in), static_cast<__half *>(x_out));
    // the buffer is free again once the uploads (compute stream) and the gathers (copy stream) are done
    PS_HIP(hipStreamWaitEvent(st->compute, st->ev_ready[0], 0));
    PS_HIP(hipStreamWaitEvent(st->compute, st->ev_ready[1], 0));
    PS_HIP(hipEventRecord(st->ev_upload[tb], st->compute));
    st->upload_pending[tb] = true;
    return rc;
}

static int32_t forward_checks(ps_stack *st, const void *x_in, void *x_out) {
    if (!st || !x_in || !x_out) { ps::set_error("NULL argument"); return PS_E_ARG; }
    if (x_in == x_out) { ps::set_error("x_in and x_out may not alias"); return PS_E_ARG; }
    if (st->n_loaded != st->n_expected) {
        ps::set_error("forward before all matrices were loaded (%llu of %llu)", (unsigned long long)st->n_loaded,
                      (unsigned long long)st->n_expected);
        return PS_E_STATE;
    }
    return PS_OK;
}

int32_t ps_stack_forward(ps_stack *st, const void *x_in, void *x_out, const float *router_logits,
                         const float *router_logits_dev) {
    const int32_t rc = forward_checks(st, x_in, x_out);
    if (rc) return rc;
    const ps_plan &p = st->plan;
    return forward_impl(st, x_in, x_out, router_logits, router_logits_dev, (uint64_t)p.M * p.g.m.n_experts, p.M);
}

int32_t ps_stack_forward_noalloc(ps_stack *st, const void *x_in, void *x_out) {
    const int32_t rc0 = forward_checks(st, x_in, x_out);
    if (rc0) return rc0;
    const ps_plan &p = st->plan;
    if (p.g.moe || p.g.kv || p.cpu_bytes) {
        ps::set_error("ps_stack_forward_noalloc takes dense GPU-only stacks without a KV cache"); return PS_E_STATE;
    }
    if (st->profiling) { ps::set_error("ps_stack_forward_noalloc does not record profiling events: switch profiling off"); return PS_E_STATE; }
    if (p.ws.total > kStaticWsBytes) {
        ps::set_error("workspace of %llu B for %u tokens exceeds the static scratch of %llu B", (unsigned long long)p.ws.total,
                      p.M, (unsigned long long)kStaticWsBytes);
        return PS_E_ARG;
    }
    // every kernel of this forward takes its workspace pointers from ws_base: the static array's
    // address on this device.  Launch per shard (a graph would have to be instantiated).
    const bool graph = st->use_graph;
    st->use_graph = false;
    st->ws_base = st->static_ws;
    const int32_t rc = forward_impl(st, x_in, x_out, nullptr, nullptr, 0, p.M);
    st->ws_base = st->arena + p.ws_off;
    st->use_graph = graph;
    return rc;
}

int32_t ps_stack_forward_chunked(ps_stack *st, const void *x_in, void *x_out, uint32_t n_tokens,
                                 const float *router_logits, const float *router_logits_dev, void *last_logits_dev,
                                 uint32_t *trips) {
    int32_t rc = forward_checks(st, x_in, x_out);
    if (rc) return rc;
    if (n_tokens == 0) { ps::set_error("n_tokens is 0"); return PS_E_ARG; }
    const ps_plan &p = st->plan;
    if (last_logits_dev && !p.g.m.vocab) { ps::set_error("this stack has no output head (vocab is 0)"); return PS_E_STATE; }
    if (last_logits_dev && (uintptr_t)last_logits_dev % 16) { ps::set_error("logits buffer must be 16-byte aligned"); return PS_E_ARG; }
    const uint32_t T = p.M, H = p.g.m.hidden, E = p.g.m.n_experts;
    // the head setting of plain forwards is put back afterwards
    __half *const saved_logits = st->logits;
    const uint32_t saved_rows = st->head_rows, saved_row0 = st->head_row0;
    uint32_t n_trips = 0;
    const uint32_t ctx0 = st->ctx;
    if (p.g.kv && (uint64_t)ctx0 + n_tokens > p.g.m.kv_context) {
        ps::set_error("context %u and %u new tokens do not fit a cache of %u positions", ctx0, n_tokens, p.g.m.kv_context);
        return PS_E_ARG;
    }
    for (uint32_t r0 = 0; r0 < n_tokens && rc == PS_OK; r0 += T, ++n_trips) {
        const uint32_t nv = std::min(T, n_tokens - r0);
        const bool last = r0 + nv == n_tokens;
        // the head runs on the last trip only, for the prompt's last token
        st->logits = last && last_logits_dev ? static_cast<__half *>(last_logits_dev) : nullptr;
        st->head_rows = st->logits ? 1 : 0;
        st->head_row0 = st->logits ? nv - 1 : 0;
        if (p.g.kv) st->ctx = ctx0 + r0;      // each trip attends over the cache and the rows the earlier trips appended
        rc = forward_impl(st, static_cast<const __half *>(x_in) + (size_t)r0 * H, static_cast<__half *>(x_out) + (size_t)r0 * H,
                          router_logits ? router_logits + (size_t)r0 * E : nullptr,
                          router_logits_dev ? router_logits_dev + (size_t)r0 * E : nullptr, (uint64_t)n_tokens * E, nv);
    }
    st->logits = saved_logits; st->head_rows = saved_rows; st->head_row0 = saved_row0;
    if (p.g.kv && rc == PS_OK) st->ctx = ctx0 + n_tokens;   // the prompt's rows are in the cache now
    if (trips) *trips = n_trips;
    return rc;
}

int32_t ps_stack_set_decode_mode(ps_stack *st, int32_t mode) {
    if (!st) { ps::set_error("NULL argument"); return PS_E_ARG; }
    if (mode < 0 || mode > 2) { ps::set_error("decode mode must be 0, 1 or 2"); return PS_E_ARG; }
    const ps_plan &p = st->plan;
    // eligible: dense, one token, every shard resident (nothing to wait for but the previous kernel)
    st->decode_mode = mode;
    st->use_graph = mode == 1 && graph_eligible(p) && st->have_dense_sched;
    st->own_rinv_launch = mode == 2;
    return PS_OK;
}

int32_t ps_stack_set_copy_mode(ps_stack *st, int32_t gather) {
    if (!st) { ps::set_error("NULL argument"); return PS_E_ARG; }
    if (gather < 0 || gather > 2) { ps::set_error("copy mode must be 0, 1 or 2"); return PS_E_ARG; }
    st->copy_mode = gather;
    st->gather_copy = gather != 0;
    st->inline_fill = gather == 1;
    st->gather_dense = st->have_dense_sched && dense_gather_pays(st->plan, gather);
    return PS_OK;
}

int32_t ps_stack_sync_check(ps_stack *st) {
    if (!st) { ps::set_error("NULL argument"); return PS_E_ARG; }
    PS_HIP(hipStreamSynchronize(st->copy));
    PS_HIP(hipStreamSynchronize(st->compute));
    return PS_OK;
}

int32_t ps_stack_set_profiling(ps_stack *st, int32_t on) {
    if (!st) { ps::set_error("NULL argument"); return PS_E_ARG; }
    st->profiling = on != 0;
    return PS_OK;
}

int32_t ps_stack_stats(ps_stack *st, ps_stats *out) {
    if (!st || !out) { ps::set_error("NULL argument"); return PS_E_ARG; }
    if (st->prof_valid) {
        PS_HIP(hipStreamSynchronize(st->copy));
        PS_HIP(hipStreamSynchronize(st->compute));
        const size_t n = st->prof_is_copy.size();
        st->prof_start.assign(n, 0.0); st->prof_dur.assign(n, 0.0);
        double copy_ms = 0, comp_ms = 0, t_min = 0, t_max = 0;
        bool first = true;
        for (size_t i = 0; i < n; ++i) {
            float dur = 0, t0 = 0;
            PS_HIP(hipEventElapsedTime(&dur, st->prof_ev[2 * i], st->prof_ev[2 * i + 1]));
            PS_HIP(hipEventElapsedTime(&t0, st->prof_ev[0], st->prof_ev[2 * i]));
            (st->prof_is_copy[i] ? copy_ms : comp_ms) += dur;
            st->prof_start[i] = t0; st->prof_dur[i] = dur;
            if (first || t0 < t_min) t_min = t0;
            if (first || t0 + dur > t_max) t_max = t0 + dur;
            first = false;
        }
        ps_stats &s = st->stats;
        s.copy_ms = copy_ms; s.compute_ms = comp_ms; s.wall_ms = t_max - t_min;
        const double mn = std::min(copy_ms, comp_ms);
        s.overlap = mn > 0 ? (copy_ms + comp_ms - s.wall_ms) / mn : 0.0;
        s.h2d_gbps = copy_ms > 0 ? (double)s.streamed_bytes_step / (copy_ms * 1e-3) / 1e9 : 0.0;
        st->prof_valid = false;
    }
    *out = st->stats;
    return PS_OK;
}

int32_t ps_stack_op_time(ps_stack *st, uint32_t i, double *start_ms, double *dur_ms) {
    if (!st || !start_ms || !dur_ms) { ps::set_error("NULL argument"); return PS_E_ARG; }
    if (st->prof_valid) { ps_stats tmp; int32_t rc = ps_stack_stats(st, &tmp); if (rc) return rc; }
    if (i >= st->prof_dur.size()) { ps::set_error("no profiled op %u", i); return PS_E_ARG; }
    *start_ms = st->prof_start[i]; *dur_ms = st->prof_dur[i];
    return PS_OK;
}

int32_t ps_stack_time_kernel(ps_stack *st, uint32_t kernel, uint32_t reps, double *avg_launch_ms, uint32_t *launches) {
    if (!st || !avg_launch_ms || !launches || reps == 0) { ps::set_error("bad argument"); return PS_E_ARG; }
    if (!st->have_dense_sched || st->n_loaded != st->n_expected) { ps::set_error("needs a loaded dense stack"); return PS_E_STATE; }
    if (kernel == PS_K_OUT && !st->head_rows) { ps::set_error("timing the output head needs a logits buffer"); return PS_E_STATE; }
    const ps_plan &p = st->plan;
    st->n_valid = p.M;
    // activations: the workspace ping-pong buffers stand in for the caller's tensors
    const __half *xin = reinterpret_cast<const __half *>(st->ws_base + p.ws.x0);
    __half *xout = reinterpret_cast<__half *>(st->ws_base + p.ws.x1);
    hipEvent_t e0, e1;
    PS_HIP(hipEventCreate(&e0));
    PS_HIP(hipEventCreate(&e1));
    uint32_t n = 0;
    int32_t rc = PS_OK;
    for (uint32_t r = 0; r <= reps && rc == PS_OK; ++r) {   // pass 0 warms up
        if (r == 1) { if (hipEventRecord(e0, st->compute) != hipSuccess) rc = PS_E_HIP; n = 0; }
        for (const ps::Op &op : st->dense_sched.ops) {
            if (op.info.type != PS_OP_KERNEL || op.info.kernel != kernel || op.info.slot >= 0) continue;
            st->rinv_of = nullptr;   // timed in isolation: every launch is issued
            rc = issue_kernel(st, st->dense_sched, op, xin, xout);
            if (rc) break;
            ++n;
        }
    }
    st->rinv_of = nullptr;
    float ms = 0;
    if (rc == PS_OK && (hipEventRecord(e1, st->compute) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                        hipEventElapsedTime(&ms, e0, e1) != hipSuccess)) {
        ps::set_error("event timing failed");
        rc = PS_E_HIP;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    if (n == 0) { ps::set_error("no resident op of kernel kind %u", kernel); return PS_E_ARG; }
    *avg_launch_ms = (double)ms / n;
    *launches = n / reps;
    return PS_OK;
}

int32_t ps_stack_debug_buffer(ps_stack *st, uint32_t which, void **dev_ptr, uint64_t *bytes) {
    if (!st || !dev_ptr || !bytes) { ps::set_error("NULL argument"); return PS_E_ARG; }
    const ps_plan &p = st->plan;
    const uint64_t P = (uint64_t)p.M * std::max(1u, p.g.m.top_k);
    switch (which) {
        case 0: *dev_ptr = st->ws_base + p.ws.qkv; *bytes = p.ws.qkv_bytes; return PS_OK;
        case 1: *dev_ptr = st->ws_base + p.ws.h; *bytes = p.ws.h_bytes; return PS_OK;
        case 2: *dev_ptr = st->ws_base + p.ws.s; *bytes = p.ws.s_bytes; return PS_OK;
        case 3: if (!p.g.moe) break; *dev_ptr = st->ws_base + p.ws.ridx; *bytes = P * 4; return PS_OK;
        case 4: if (!p.g.moe) break; *dev_ptr = st->ws_base + p.ws.rw; *bytes = P * 4; return PS_OK;
    }
    ps::set_error("no such debug buffer");
    return PS_E_ARG;
}

void ps_stack_destroy(ps_stack *st) {
    if (!st) return;
    if (st->compute || st->copy) {
        if (st->copy) (void)hipStreamSynchronize(st->copy);
        if (st->compute) (void)hipStreamSynchronize(st->compute);
    }
    for (void *c : st->host_chunks) (void)hipHostFree(c);
    if (st->stage) (void)hipHostFree(st->stage);
    for (uint16_t *b : {st->host_h, st->host_s, st->host_x, st->host_out}) if (b) (void)hipHostFree(b);
    for (int b = 0; b < 2; ++b) if (st->tables_host[b]) (void)hipHostFree(st->tables_host[b]);
    if (st->dense_descs) (void)hipHostFree(st->dense_descs);
    for (int s = 0; s < 2; ++s) {
        if (st->ev_ready[s]) (void)hipEventDestroy(st->ev_ready[s]);
        if (st->ev_free[s]) (void)hipEventDestroy(st->ev_free[s]);
    }
    for (auto e : st->ev_router) if (e) (void)hipEventDestroy(e);
    if (st->ev_step) (void)hipEventDestroy(st->ev_step);
    for (int b = 0; b < 2; ++b) if (st->ev_upload[b]) (void)hipEventDestroy(st->ev_upload[b]);
    for (auto e : st->prof_ev) (void)hipEventDestroy(e);
    for (auto &g : st->graphs) (void)hipGraphExecDestroy(g.second);
    delete st;
}

int32_t ps_lds_tr_probe(const uint32_t *addr_dev, uint16_t *out_dev, void *stream) {
    if (!addr_dev || !out_dev) { ps::set_error("probe buffers missing"); return PS_E_ARG; }
    PS_HIP(ps::launch_lds_tr_probe(addr_dev, out_dev, static_cast<hipStream_t>(stream)));
    return PS_OK;
}

int32_t ps_mfma_probe(int32_t pi, int32_t pk, int32_t pj, float *out_dev, void *stream) {
    if (pi < 0 || pi > 15 || pj < 0 || pj > 15 || pk < 0 || pk > 31 || !out_dev) { ps::set_error("probe index out of range"); return PS_E_ARG; }
    PS_HIP(ps::launch_mfma_probe(pi, pk, pj, out_dev, static_cast<hipStream_t>(stream)));
    return PS_OK;
}

}  // extern "C"
