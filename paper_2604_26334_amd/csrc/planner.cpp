// Planning phase of pipelined sharding for the GPU-only plan (paper Section 3:
// Algorithm 1 procedures PlanningPhase and PinShardsToGPU, "Plan One", and the
// profile-based timing estimate).  Host code only; no HIP calls.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <numeric>

#include "ps_internal.h"

namespace ps {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

static const uint32_t kTiers[PS_NTIERS] = {1, 4, 16, 32, 64, 512, 1024, 2048, 4096, 8192, 16384};

MatGeom make_geom(uint32_t rows, uint32_t K, bool paired) {
    MatGeom g;
    g.K = K;
    g.rows = rows;
    g.ntiles = rows / kTileRows;
    g.nsb = K / kSuperK;
    g.ngroups = (g.nsb + kGroupSb - 1) / kGroupSb;
    g.tile_bytes = (uint64_t)(g.nsb + g.ngroups) * kSbBytes;
    g.bytes = g.tile_bytes * g.ntiles;
    // slabs are cut at multiples of 16 tiles (256 rows) when the matrix allows it, else
    // at 2 tiles (one gate tile + its up tile) or 1
    g.quantum_tiles = (g.ntiles % 16 == 0) ? 16 : (paired ? 2 : 1);
    return g;
}

int32_t make_model_geom(const ps_model_desc *m, ModelGeom *out) {
    if (!m) { set_error("model is NULL"); return PS_E_ARG; }
    ModelGeom g;
    g.m = *m;
    g.has_attn = !(m->flags & PS_FLAG_NO_ATTN);
    g.moe = m->n_experts > 0;
    auto bad_k = [](uint32_t K) { return K == 0 || K % kSuperK != 0 || K > 16384; };
    if (m->n_layers == 0 || bad_k(m->hidden)) {
        set_error("hidden=%u must be a multiple of 128, <= 16384; n_layers=%u must be > 0", m->hidden, m->n_layers);
        return PS_E_ARG;
    }
    if (m->hidden % kTileRows) { set_error("hidden must be a multiple of 16"); return PS_E_ARG; }
    if (g.has_attn) {
        if (m->head_dim != 128 || m->n_kv_heads == 0 || m->n_q_heads == 0 || m->n_q_heads % m->n_kv_heads) {
            set_error("attention needs head_dim 128 and n_q_heads a multiple of n_kv_heads (got %u, %u, %u)",
                      m->head_dim, m->n_q_heads, m->n_kv_heads);
            return PS_E_ARG;
        }
        g.qkv_w = (m->n_q_heads + 2 * m->n_kv_heads) * m->head_dim;
        g.attn_w = m->n_q_heads * m->head_dim;
        if (bad_k(g.attn_w)) { set_error("n_q_heads*head_dim=%u unsupported", g.attn_w); return PS_E_ARG; }
        g.qkv = make_geom(g.qkv_w, m->hidden, false);
        g.o = make_geom(m->hidden, g.attn_w, false);
        g.kv = m->kv_context > 0;
        if (m->kv_context > (1u << 20)) { set_error("kv_context=%u too large", m->kv_context); return PS_E_ARG; }
        g.kv_shard_bytes = (uint64_t)m->kv_context * m->head_dim * 2 * 2;   // K rows then V rows, fp16
    } else if (m->kv_context) {
        set_error("kv_context needs attention layers");
        return PS_E_ARG;
    }
    if (g.moe) {
        if (m->ffn_inter != 0 || m->top_k == 0 || m->top_k > m->n_experts || m->top_k > 32 || m->n_experts > 1024) {
            set_error("MoE needs ffn_inter 0, 0 < top_k <= min(n_experts, 32), n_experts <= 1024");
            return PS_E_ARG;
        }
        if (m->flags & PS_FLAG_NO_RESIDUAL) {
            // the flag describes the bare dense FFN block (RMSNorm -> gate/up -> SwiGLU -> down); an MoE layer's
            // combine is defined with its residual
            set_error("PS_FLAG_NO_RESIDUAL applies to dense FFN layers only");
            return PS_E_ARG;
        }
        g.ffn_i = m->expert_inter;
    } else {
        g.ffn_i = m->ffn_inter;
    }
    if (bad_k(g.ffn_i) || g.ffn_i % kTileRows) {
        set_error("FFN width %u must be a multiple of 128 and <= 16384", g.ffn_i);
        return PS_E_ARG;
    }
    g.gate_up = make_geom(2 * g.ffn_i, m->hidden, true);
    g.down = make_geom(m->hidden, g.ffn_i, false);
    g.expert_bytes = g.moe ? g.gate_up.bytes + g.down.bytes : 0;
    if (m->vocab) {
        if (m->vocab % kTileRows || m->vocab > (1u << 20)) { set_error("vocab=%u must be a multiple of 16, <= 2^20", m->vocab); return PS_E_ARG; }
        g.head = make_geom(m->vocab, m->hidden, false);
        if (g.head.bytes > 0xFFFFFFFFull) { set_error("output head too large"); return PS_E_ARG; }
    }
    *out = g;
    return PS_OK;
}

uint32_t gemm_sb_per_part(const MatGeom &mg, uint32_t M) {
    if (M < 2 || M > 64) return 0;
    // batched decode: with few tokens a matrix has too few 8-tile workgroups to fill 256 CUs, so K is
    // split into at most 8 parts.  Measured on the 8B shapes at 4, 16 and 64 tokens: a matrix whose
    // workgroups already fill 7/8 of the CUs is faster unsplit (gate/up, 224 workgroups: one launch
    // instead of GEMM + plane sum); the others take as many parts as still give at most one
    // workgroup per CU, and parts of equal length win over one part more (QKV, 48 workgroups x 32
    // super-blocks: 4 x 8 beats 5 parts of 7,7,7,7,4 and 6 of 6,..,2; O and down: 8 even parts)
    const uint32_t wgs = (mg.ntiles + 7) / 8;
    if (wgs * 8 >= 256 * 7) return 0;
    const uint32_t pmax = std::min(std::min(mg.nsb, 8u), std::max(1u, 256u / wgs));
    uint32_t parts = pmax;
    for (uint32_t d = pmax; 2 * d > pmax; --d)
        if (mg.nsb % d == 0) { parts = d; break; }
    if (parts <= 1) return 0;
    return (mg.nsb + parts - 1) / parts;
}

Workspace make_workspace(const ModelGeom &g, uint32_t M, bool cpu_experts) {
    Workspace w;
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) { uint64_t o = off; off = align_up(off + bytes, kAlign); return o; };
    const uint64_t H = g.m.hidden;
    w.h_bytes = (uint64_t)M * H * 2;
    w.x0 = take(w.h_bytes);
    w.x1 = take(w.h_bytes);
    w.h = take(w.h_bytes);
    w.qkv_bytes = (uint64_t)M * g.qkv_w * 2;
    w.qkv = take(w.qkv_bytes);
    w.rinv = take((uint64_t)M * 4);
    if (g.moe) {
        const uint64_t P = (uint64_t)M * g.m.top_k;  // (token, rank) pairs
        w.s_bytes = P * g.ffn_i * 2;
        w.s = take(w.s_bytes);
        w.y = take(P * H * 4);
        w.ridx = take(P * 4);
        w.rw = take(P * 4);
        w.logits_bytes = (uint64_t)g.m.n_layers * M * g.m.n_experts * 4;
        w.logits = take(w.logits_bytes);
        const uint64_t tasks_per_layer = std::min<uint64_t>(g.m.n_experts, P);
        w.tasks_bytes = (uint64_t)g.m.n_layers * tasks_per_layer * sizeof(DeviceTask);
        w.tasks = take(w.tasks_bytes);
        w.pairs_bytes = (uint64_t)g.m.n_layers * P * 4;
        w.pairs = take(w.pairs_bytes);
        // landing area of the experts computed on the CPU: fp32 rows [P][H], then their pair indices
        if (cpu_experts) w.cpu_y = take(P * H * 4 + P * 4);
    } else {
        w.s_bytes = (uint64_t)M * g.ffn_i * 2;
        w.s = take(w.s_bytes);
    }
    uint64_t pb = 0;   // fp32 partial planes of the split-K batched-decode GEMMs (attention matrices; dense FFN)
    for (const MatGeom *mg : {&g.qkv, &g.o, &g.gate_up, &g.down, &g.head}) {
        if (!mg->ntiles || (g.moe && (mg == &g.gate_up || mg == &g.down))) continue;
        const uint32_t per = gemm_sb_per_part(*mg, M);
        if (per) pb = std::max<uint64_t>(pb, (uint64_t)((mg->nsb + per - 1) / per) * M * mg->rows * 4);
    }
    if (pb) w.partial = take(pb);
    if (g.kv) {
        w.attn = take((uint64_t)M * g.attn_w * 2);
        // per token, query head and position chunk: running maximum, sum of weights, 128 weighted sums;
        // a chunk of several tokens adds the chunks of its own rows behind the cache's
        // (chunks of kAttnOnePassTokens tokens and more keep running statistics in the kernel instead)
        const uint64_t chunks = (g.m.kv_context + kAttnChunk - 1) / kAttnChunk + (M > 1 ? (M + kAttnChunk - 1) / kAttnChunk : 0);
        w.apart = take(M >= kAttnOnePassTokens ? kAlign : (uint64_t)M * g.m.n_q_heads * chunks * (g.m.head_dim + 2) * 4);
        w.kvhome = take((uint64_t)g.m.n_layers * g.m.n_kv_heads * 8);
        w.ctx = take(4);   // context length as the kernels of a replayed graph read it
    }
    w.total = off;
    return w;
}

struct Cand {  // a whole matrix / expert before any split
    Shard s;
    uint32_t quantum_tiles;
    uint64_t tile_bytes;
    double freq;
};

// shards that a CPU plan may leave in system memory: FFN matrices, whole experts and the output
// head (the low end of the priority list); attention matrices and caches always run on the GPU
static bool cpu_eligible(const Shard &s) {
    return s.kind == PS_SHARD_GATE_UP || s.kind == PS_SHARD_DOWN || s.kind == PS_SHARD_OUT || s.kind == PS_SHARD_EXPERT;
}

static double shard_compute_ms(const ps_plan &p, uint64_t bytes, double tokens) {
    // memory-bound price vs compute-bound price (roofline rule of the paper's estimator)
    const double weights = (double)bytes / 0.5625;
    const double t_mem = p.prof.gemv_gbps > 0 ? (double)bytes / (p.prof.gemv_gbps * 1e9) : 0;
    const double tf = p.prof.gemm_tflops[p.tier];
    const double t_cmp = tf > 0 ? 2.0 * tokens * weights / (tf * 1e12) : 0;
    return (std::max(t_mem, t_cmp)) * 1e3 + p.prof.launch_us * 1e-3;
}

static void estimate(ps_plan &p, const float *freq) {
    // Each shard's time is the larger of its compute time and the concurrent H2D copy of
    // the next shard; shard times are summed (paper Section 3, timing estimation).  MoE
    // expert shards are weighted by the probability that a step touches them.  The CPU part of a
    // matrix runs beside the GPU's work on the same matrix: the matrix costs the larger of the two.
    // When both the CPU and PCIe pull on system memory, both are priced at their contended rates.
    const auto &m = p.g.m;
    const size_t n = p.shards.size();
    bool any_cpu = false, any_stream = false;
    for (const Shard &s : p.shards) { any_cpu |= s.resident == 2; any_stream |= s.resident == 0; }
    const bool contend = any_cpu && any_stream;
    const double h2d = contend && p.prof.h2d_gbps_busy > 0 ? p.prof.h2d_gbps_busy : p.prof.h2d_gbps;
    const double cpu = contend && p.prof.cpu_gbps_busy > 0 ? p.prof.cpu_gbps_busy : p.prof.cpu_gbps;
    std::vector<double> prob(n, 1.0), comp(n, 0.0), copy(n, 0.0);
    // With a profile database a shard's matmuls are looked up there (exact match, nearest neighbour
    // with a roofline, or skipped); a shard the database cannot price keeps the profile's rates.
    const ModelGeom &g = p.g;
    auto db_matmuls = [&](const Shard &s, double tokens, bool on_cpu, double *ms) -> bool {
        if (!p.db) return false;
        const uint64_t mt = (uint64_t)std::max(1.0, std::round(tokens));
        struct { uint64_t n, k; } mats[2];
        int nm = 1;
        switch (s.kind) {
            case PS_SHARD_QKV: mats[0] = {(uint64_t)s.ntiles * 16, m.hidden}; break;
            case PS_SHARD_O: mats[0] = {(uint64_t)s.ntiles * 16, g.attn_w}; break;
            case PS_SHARD_GATE_UP: mats[0] = {(uint64_t)s.ntiles * 16, m.hidden}; break;
            case PS_SHARD_DOWN: mats[0] = {(uint64_t)s.ntiles * 16, g.ffn_i}; break;
            case PS_SHARD_OUT: mats[0] = {(uint64_t)s.ntiles * 16, m.hidden}; break;
            case PS_SHARD_EXPERT: mats[0] = {2ull * g.ffn_i, m.hidden}; mats[1] = {m.hidden, g.ffn_i}; nm = 2; break;
            default: return false;
        }
        const uint32_t op = on_cpu ? PS_OPK_CPU : (mt == 1 ? PS_OPK_GEMV : PS_OPK_GEMM);
        const double bw = on_cpu ? p.prof.cpu_gbps : p.prof.gemv_gbps;
        if (!(bw > 0)) return false;
        double t = 0;
        for (int q = 0; q < nm; ++q) {
            ps_prof_estimate e;
            db_estimate(p.db.get(), bw, op, 4, on_cpu ? p.db_threads : 0, mats[q].n, mats[q].k, mt, &e);
            if (e.match == PS_MATCH_NONE) return false;
            t += e.ms;
        }
        if (on_cpu && contend && p.prof.cpu_gbps_busy > 0 && p.prof.cpu_gbps > 0) t *= p.prof.cpu_gbps / p.prof.cpu_gbps_busy;
        *ms = t;
        return true;
    };
    auto copy_ms = [&](uint64_t bytes) -> double {
        if (p.db) {
            ps_prof_estimate e;
            db_estimate(p.db.get(), 1.0, PS_OPK_H2D, 0, 0, bytes, 1, 1, &e);
            if (e.match != PS_MATCH_NONE) {
                const double scale = contend && p.prof.h2d_gbps_busy > 0 && p.prof.h2d_gbps > 0 ? p.prof.h2d_gbps / p.prof.h2d_gbps_busy : 1.0;
                return e.ms * scale;
            }
        }
        return h2d > 0 ? (double)bytes / (h2d * 1e9) * 1e3 : 0.0;
    };
    for (size_t i = 0; i < n; ++i) {
        const Shard &s = p.shards[i];
        double tokens = p.M;
        if (s.resident == 2 && s.kind != PS_SHARD_EXPERT) {
            const double slow = p.prof.cpu_tokens_free > 0 ? std::max(1.0, tokens / p.prof.cpu_tokens_free) : 1.0;
            double t;
            if (!db_matmuls(s, tokens, true, &t)) t = cpu > 0 ? (double)s.bytes / (cpu * 1e9) * 1e3 * slow : 0.0;
            comp[i] = t + p.prof.cpu_sync_us * 1e-3;
            continue;
        }
        if (s.kind == PS_SHARD_EXPERT) {
            double f = (double)m.top_k / m.n_experts;
            if (freq) f = freq[(size_t)s.layer * m.n_experts + s.expert];
            f = std::min(1.0, std::max(0.0, f));
            prob[i] = 1.0 - std::pow(1.0 - f, (double)p.M);
            tokens = prob[i] > 0 ? p.M * f / prob[i] : 0;
        }
        if (s.resident == 2) {   // an expert on the CPU: touched with probability prob, by `tokens` tokens
            const double slow = p.prof.cpu_tokens_free > 0 ? std::max(1.0, tokens / p.prof.cpu_tokens_free) : 1.0;
            double t;
            if (!db_matmuls(s, tokens, true, &t)) t = cpu > 0 ? (double)s.bytes / (cpu * 1e9) * 1e3 * slow : 0.0;
            comp[i] = t * prob[i];
            continue;
        }
        double t;
        if (!db_matmuls(s, tokens, false, &t)) t = shard_compute_ms(p, s.bytes, tokens);
        comp[i] = t * prob[i];
        if (!s.resident) copy[i] = copy_ms(s.bytes) * prob[i];
    }
    std::vector<size_t> gpu;   // the GPU's shards, in order
    for (size_t i = 0; i < n; ++i) if (p.shards[i].resident != 2) gpu.push_back(i);
    std::vector<double> tg(n, 0.0);
    for (size_t j = 0; j < gpu.size(); ++j) tg[gpu[j]] = std::max(comp[gpu[j]], j + 1 < gpu.size() ? copy[gpu[j + 1]] : 0.0);
    double t = gpu.empty() ? 0.0 : copy[gpu[0]], streamed = 0;
    for (size_t i = 0; i < n;) {   // one matrix (or expert, or cache head) at a time
        // the experts of a layer form one group: the CPU's run beside the GPU's, one hand-over per layer
        size_t j = i;
        double t_gpu = 0, t_cpu = 0;
        const bool experts = p.shards[i].kind == PS_SHARD_EXPERT;
        while (j < n && p.shards[j].layer == p.shards[i].layer && p.shards[j].kind == p.shards[i].kind &&
               (experts || p.shards[j].expert == p.shards[i].expert)) {
            if (p.shards[j].resident == 2) t_cpu += comp[j]; else t_gpu += tg[j];
            if (!p.shards[j].resident) streamed += (double)p.shards[j].bytes * prob[j];
            ++j;
        }
        if (experts && t_cpu > 0) t_cpu += p.prof.cpu_sync_us * 1e-3;
        t += std::max(t_gpu, t_cpu);
        i = j;
    }
    p.est_step_ms = t;
    p.est_streamed_per_step = streamed;
}

// One plan of the given kind.  cpu_frac: Plan Three's share of each unpinned CPU-eligible matrix
// that stays on the CPU (ignored otherwise).
// the database the plans of the current ps_plan_create_db call are estimated with
static thread_local std::shared_ptr<const ps_profile_db> t_db;

static int32_t build_plan(const ps_model_desc *model, uint64_t budget, const ps_profile *prof, uint32_t M,
                          const float *freq, uint32_t kind, double cpu_frac, ps_plan *p) {
    int32_t rc = make_model_geom(model, &p->g);
    if (rc) return rc;
    p->db = t_db;
    p->db_threads = 0;
    if (p->db) for (const ps_prof_entry &e : p->db->entries) if (e.op == PS_OPK_CPU) p->db_threads = std::max(p->db_threads, e.threads);
    if (M == 0 || M > kTiers[PS_NTIERS - 1]) { set_error("n_tokens=%u out of range 1..16384", M); return PS_E_ARG; }
    if (p->g.kv && M >= p->g.m.kv_context) { set_error("a chunk of %u tokens does not fit a cache of %u positions", M, p->g.m.kv_context); return PS_E_BUDGET; }
    if (p->g.kv && M > 1 && kind != PS_PLAN_GPU_ONLY) { set_error("chunks of several tokens over a KV cache take the GPU-only plan"); return PS_E_ARG; }
    if (prof) p->prof = *prof;
    if (kind != PS_PLAN_GPU_ONLY && !(p->prof.cpu_gbps > 0)) {
        set_error("plans with CPU shards need a profile with cpu_gbps > 0"); return PS_E_STATE;
    }
    if (kind != PS_PLAN_GPU_ONLY && M > 64) { set_error("the CPU back-end takes at most 64 tokens (got %u)", M); return PS_E_ARG; }
    p->budget = budget;
    p->M = M;
    p->kind = kind;
    p->cpu_frac = kind == PS_PLAN_DYNAMIC ? std::min(1.0, std::max(0.0, cpu_frac)) : (kind == PS_PLAN_STATIC ? 1.0 : 0.0);
    p->tier = ps_tier_for_tokens(M);
    p->ws = make_workspace(p->g, M, kind != PS_PLAN_GPU_ONLY);
    p->shards.clear();
    const ModelGeom &g = p->g;
    const auto &m = g.m;

    // ShardIntoSubLayers: one candidate per weight matrix (dense) or per expert (MoE)
    std::vector<Cand> cands;
    for (uint32_t l = 0; l < m.n_layers; ++l) {
        auto add = [&](uint32_t kind, uint32_t cls, const MatGeom &mg) {
            Cand c{};
            c.s.layer = l; c.s.kind = kind; c.s.cls = cls; c.s.ntiles = mg.ntiles; c.s.bytes = mg.bytes;
            c.quantum_tiles = mg.quantum_tiles; c.tile_bytes = mg.tile_bytes; c.freq = 0;
            cands.push_back(c);
        };
        if (g.has_attn) {
            add(PS_SHARD_QKV, PS_CLASS_ATTN, g.qkv);
            if (g.kv) for (uint32_t h = 0; h < m.n_kv_heads; ++h) {   // one whole shard per kv head
                Cand c{};
                c.s.layer = l; c.s.kind = PS_SHARD_KV; c.s.cls = PS_CLASS_KVCACHE; c.s.expert = h;
                c.s.ntiles = 0; c.s.bytes = g.kv_shard_bytes;
                c.quantum_tiles = 0; c.tile_bytes = 0; c.freq = 0;
                cands.push_back(c);
            }
            add(PS_SHARD_O, PS_CLASS_ATTN, g.o);
        }
        if (!g.moe) { add(PS_SHARD_GATE_UP, PS_CLASS_FFN, g.gate_up); add(PS_SHARD_DOWN, PS_CLASS_FFN, g.down); }
        else for (uint32_t e = 0; e < m.n_experts; ++e) {
            Cand c{};
            c.s.layer = l; c.s.kind = PS_SHARD_EXPERT; c.s.cls = PS_CLASS_FFN; c.s.expert = e;
            c.s.ntiles = g.gate_up.ntiles + g.down.ntiles; c.s.bytes = g.expert_bytes;
            c.quantum_tiles = 0; c.tile_bytes = 0;  // experts are never split
            c.freq = freq ? freq[(size_t)l * m.n_experts + e] : 0.0;
            cands.push_back(c);
        }
    }
    if (m.vocab) {   // the output head, after the last layer, lowest priority class
        Cand c{};
        c.s.layer = m.n_layers; c.s.kind = PS_SHARD_OUT; c.s.cls = PS_CLASS_OUTS; c.s.ntiles = g.head.ntiles;
        c.s.bytes = g.head.bytes; c.quantum_tiles = g.head.quantum_tiles; c.tile_bytes = g.head.tile_bytes; c.freq = 0;
        cands.push_back(c);
    }
    p->weight_bytes = 0;
    uint64_t max_unit = 0;  // smallest thing a slot must be able to hold
    for (auto &c : cands) {
        p->weight_bytes += c.s.bytes;
        max_unit = std::max(max_unit, c.quantum_tiles ? c.tile_bytes * c.quantum_tiles : c.s.bytes);
    }
    if (p->ws.total > budget) {
        set_error("budget %llu B < workspace %llu B for %u tokens", (unsigned long long)budget,
                  (unsigned long long)p->ws.total, M);
        return PS_E_BUDGET;
    }

    // SortByPriority: class first; experts by descending frequency; then the layer's place in a
    // spread walk over the stack (bit-reversed layer index: 0, L/2, L/4, 3L/4, ...), then matrix
    // order / expert id.  The paper fixes the order of the classes only.  With the spread walk the
    // layers a budget pins whole lie evenly between the streamed ones, so a pinned layer's kernels
    // run while the next streamed layer's first slot fills cross PCIe (in the timing estimate: a
    // shard costs the larger of its compute and the next shard's copy), where pinning the first
    // layers of the stack leaves nothing beside the copies of the rest.  The walk does not
    // depend on the token count, so every tier of a budget ranks the shards alike.
    uint32_t lbits = 0;
    while ((1u << lbits) < m.n_layers) ++lbits;
    auto spread = [&](uint32_t layer) {
        uint32_t r = 0;
        for (uint32_t b = 0; b < lbits; ++b) r |= ((layer >> b) & 1u) << (lbits - 1 - b);
        return r;
    };
    std::vector<uint32_t> order(cands.size());
    std::iota(order.begin(), order.end(), 0u);
    std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        const Cand &x = cands[a], &y = cands[b];
        if (x.s.cls != y.s.cls) return x.s.cls < y.s.cls;
        if (x.s.kind == PS_SHARD_EXPERT && y.s.kind == PS_SHARD_EXPERT && x.freq != y.freq) return x.freq > y.freq;
        if (x.s.layer != y.s.layer) return spread(x.s.layer) < spread(y.s.layer);
        return a < b;  // enumeration order inside a layer = matrix order / expert id
    });
    for (uint32_t r = 0; r < order.size(); ++r) cands[order[r]].s.rank = r;

    // PinShardsToGPU: first fit in priority order; the first shard that does not fit
    // is split at slab granularity and its head pinned; scanning continues
    std::vector<uint32_t> head_tiles(cands.size(), 0);  // tiles pinned per candidate (whole shards: 0 or 1)
    auto pin = [&](uint64_t remaining) {
        std::fill(head_tiles.begin(), head_tiles.end(), 0u);
        bool split_done = false;
        for (uint32_t r = 0; r < order.size(); ++r) {
            Cand &c = cands[order[r]];
            if (c.s.bytes <= remaining) { head_tiles[order[r]] = c.quantum_tiles ? c.s.ntiles : 1; remaining -= c.s.bytes; continue; }
            if (!split_done && c.quantum_tiles) {
                split_done = true;
                uint64_t q = remaining / (c.tile_bytes * c.quantum_tiles);
                head_tiles[order[r]] = (uint32_t)q * c.quantum_tiles;
                remaining -= (uint64_t)head_tiles[order[r]] * c.tile_bytes;
            }
        }
    };
    auto fully_pinned = [&](size_t i) { return head_tiles[i] == (cands[i].quantum_tiles ? cands[i].s.ntiles : 1u); };

    // DecideScratchVRAMBudget: none if everything fits, else a double buffer.  Plan Two gives the
    // scratch to the pinned region when every shard that must run on the GPU can be pinned.
    // the workspace ends the arena, the two slots lie in front of it, the pinned region starts at 0
    p->ws_off = (budget - p->ws.total) / kAlign * kAlign;
    bool need_slots = p->weight_bytes > p->ws_off;
    if (need_slots && kind == PS_PLAN_STATIC) {
        pin(p->ws_off);
        need_slots = false;
        for (size_t i = 0; i < cands.size(); ++i) need_slots |= !fully_pinned(i) && !cpu_eligible(cands[i].s);
    }
    if (!need_slots) {
        p->n_slots = 0; p->slot_bytes = 0;
        p->scratch_off = p->ws_off;
        pin(p->scratch_off);
    } else {
        uint64_t lo = std::min<uint64_t>(1ull << 20, budget / 8), hi = 64ull << 20;
        uint64_t slot = std::min(std::max(budget / 16, lo), hi) / kAlign * kAlign;
        if (slot < max_unit) slot = align_up(max_unit, kAlign);
        p->slot_bytes = slot; p->n_slots = 2;
        if (p->ws.total + 2 * slot > budget || p->ws_off < 2 * slot) {
            set_error("budget %llu B < workspace %llu B + 2 scratch slots of %llu B",
                      (unsigned long long)budget, (unsigned long long)p->ws.total, (unsigned long long)slot);
            return PS_E_BUDGET;
        }
        p->scratch_off = p->ws_off - 2 * slot;
        pin(p->scratch_off);
    }
    p->pinned_off = 0;

    // Emit shards in execution order; streamed remainders are cut into slabs that fit a slot; the
    // CPU's part of a matrix is its tail, one shard.  Arena offsets of resident shards follow
    // priority rank so the pinned region is dense.
    std::vector<uint64_t> res_off(cands.size(), 0);
    {
        uint64_t off = p->pinned_off;
        for (uint32_t r = 0; r < order.size(); ++r) {
            const Cand &c = cands[order[r]];
            uint64_t b = c.quantum_tiles ? (uint64_t)head_tiles[order[r]] * c.tile_bytes
                                         : (head_tiles[order[r]] ? c.s.bytes : 0);
            res_off[order[r]] = off;
            off += b;
        }
        if (off > p->scratch_off) { set_error("internal: pinned region overflows the budget"); return PS_E_STATE; }
    }
    // unpinned experts: the share cpu_frac at the cold end of the priority order stays on the CPU
    std::vector<char> expert_on_cpu(cands.size(), 0);
    if (p->cpu_frac > 0 && g.moe) {
        std::vector<uint32_t> un;
        for (uint32_t r = 0; r < order.size(); ++r)
            if (cands[order[r]].s.kind == PS_SHARD_EXPERT && !head_tiles[order[r]]) un.push_back(order[r]);
        const size_t n_cpu = p->n_slots ? std::min(un.size(), (size_t)std::lround(p->cpu_frac * un.size())) : un.size();
        for (size_t k = un.size() - n_cpu; k < un.size(); ++k) expert_on_cpu[un[k]] = 1;
    }
    uint64_t host_off = 0;
    p->resident_bytes = p->streamed_bytes = p->cpu_bytes = 0;
    for (size_t i = 0; i < cands.size(); ++i) {
        const Cand &c = cands[i];
        if (!c.quantum_tiles) {  // expert or cache head: whole
            Shard s = c.s;
            s.resident = head_tiles[i] ? 1 : (expert_on_cpu[i] ? 2 : 0);
            s.offset = s.resident == 1 ? res_off[i] : host_off;
            if (s.resident != 1) host_off += s.bytes;
            (s.resident == 1 ? p->resident_bytes : s.resident == 2 ? p->cpu_bytes : p->streamed_bytes) += s.bytes;
            if (!s.resident && !p->n_slots) { set_error("internal: streamed shard without scratch"); return PS_E_STATE; }
            p->shards.push_back(s);
            continue;
        }
        if (head_tiles[i]) {
            Shard s = c.s;
            s.tile0 = 0; s.ntiles = head_tiles[i]; s.bytes = (uint64_t)s.ntiles * c.tile_bytes;
            s.resident = 1; s.offset = res_off[i];
            p->resident_bytes += s.bytes;
            p->shards.push_back(s);
        }
        uint32_t t = head_tiles[i];
        uint32_t cpu_tiles = 0;   // tail of the unpinned remainder that stays on the CPU, in slab quanta
        if (t < c.s.ntiles && p->cpu_frac > 0 && cpu_eligible(c.s)) {
            const uint32_t quanta = (c.s.ntiles - t) / c.quantum_tiles;
            cpu_tiles = std::min(quanta, (uint32_t)std::lround(p->cpu_frac * quanta)) * c.quantum_tiles;
            if (!p->n_slots) cpu_tiles = c.s.ntiles - t;   // nowhere to stream to
        }
        const uint32_t t_end = c.s.ntiles - cpu_tiles;
        if (t < t_end) {
            if (!p->n_slots) { set_error("internal: streamed shard without scratch"); return PS_E_STATE; }
            uint32_t per = (uint32_t)(p->slot_bytes / (c.tile_bytes * c.quantum_tiles)) * c.quantum_tiles;
            if (per == 0) { set_error("internal: slot smaller than a slab quantum"); return PS_E_STATE; }
            while (t < t_end) {
                Shard s = c.s;
                s.tile0 = t; s.ntiles = std::min(per, t_end - t); s.bytes = (uint64_t)s.ntiles * c.tile_bytes;
                s.resident = 0; s.offset = host_off;
                host_off += s.bytes;
                p->streamed_bytes += s.bytes;
                p->shards.push_back(s);
                t += s.ntiles;
            }
        }
        if (cpu_tiles) {
            Shard s = c.s;
            s.tile0 = t_end; s.ntiles = cpu_tiles; s.bytes = (uint64_t)cpu_tiles * c.tile_bytes;
            s.resident = 2; s.offset = host_off;
            host_off += s.bytes;
            p->cpu_bytes += s.bytes;
            p->shards.push_back(s);
        }
    }
    estimate(*p, freq);
    for (double &e : p->est_kind) e = -1.0;
    p->est_kind[kind] = p->est_step_ms;
    return PS_OK;
}

// Plan Three: one CPU share for the whole plan, the best of a grid by the estimate
static int32_t build_dynamic(const ps_model_desc *model, uint64_t budget, const ps_profile *prof, uint32_t M,
                             const float *freq, ps_plan *p) {
    double best_f = -1, best_ms = 0;
    for (int k = 1; k <= 19; ++k) {
        ps_plan trial;
        const int32_t rc = build_plan(model, budget, prof, M, freq, PS_PLAN_DYNAMIC, k * 0.05, &trial);
        if (rc) return rc;
        if (best_f < 0 || trial.est_step_ms < best_ms) { best_f = k * 0.05; best_ms = trial.est_step_ms; }
    }
    return build_plan(model, budget, prof, M, freq, PS_PLAN_DYNAMIC, best_f, p);
}

static int32_t plan_impl(const ps_model_desc *model, uint64_t budget, const ps_profile *prof, uint32_t M,
                         const float *freq, uint32_t kind, ps_plan *p) {
    if (kind == PS_PLAN_GPU_ONLY || kind == PS_PLAN_STATIC) return build_plan(model, budget, prof, M, freq, kind, 0.0, p);
    if (kind == PS_PLAN_DYNAMIC) return build_dynamic(model, budget, prof, M, freq, p);
    if (kind != PS_PLAN_AUTO) { set_error("unknown plan kind %u", kind); return PS_E_ARG; }
    // HeuristicSplit: all three, the lowest estimate wins; a plan that cannot be built drops out
    int32_t rc = build_plan(model, budget, prof, M, freq, PS_PLAN_GPU_ONLY, 0.0, p);
    if (rc) return rc;
    double est[3] = {p->est_step_ms, -1.0, -1.0};
    const bool cpu_ok = prof && prof->cpu_gbps > 0 && M <= 64;
    if (cpu_ok) {
        ps_plan st, dy;
        if (build_plan(model, budget, prof, M, freq, PS_PLAN_STATIC, 0.0, &st) == PS_OK) {
            est[1] = st.est_step_ms;
            if (st.est_step_ms < p->est_step_ms) *p = st;
        }
        if (build_dynamic(model, budget, prof, M, freq, &dy) == PS_OK) {
            est[2] = dy.est_step_ms;
            if (dy.est_step_ms < p->est_step_ms) *p = dy;
        }
    }
    for (int k = 0; k < 3; ++k) p->est_kind[k] = est[k];
    return PS_OK;
}

}  // namespace ps

extern "C" {

const char *ps_last_error(void) { return ps::g_err; }

uint32_t ps_tier_tokens(uint32_t t) { return t < PS_NTIERS ? ps::kTiers[t] : 0; }

uint32_t ps_tier_for_tokens(uint32_t n) {
    for (uint32_t t = 0; t < PS_NTIERS; ++t)
        if (n <= ps::kTiers[t]) return t;
    return PS_NTIERS - 1;
}

uint64_t ps_packed_bytes(uint32_t rows, uint32_t K) {
    if (K == 0 || K % ps::kSuperK || rows % ps::kTileRows) return 0;
    return ps::make_geom(rows, K, false).bytes;
}

int32_t ps_plan_create(const ps_model_desc *model, uint64_t budget, const ps_profile *prof,
                       uint32_t n_tokens, const float *expert_freq, ps_plan **out) {
    if (!out) { ps::set_error("out is NULL"); return PS_E_ARG; }
    *out = nullptr;
    ps_plan *p = new (std::nothrow) ps_plan();
    if (!p) { ps::set_error("out of host memory"); return PS_E_NOMEM; }
    int32_t rc = ps::plan_impl(model, budget, prof, n_tokens, expert_freq, PS_PLAN_GPU_ONLY, p);
    if (rc) { delete p; return rc; }
    *out = p;
    return PS_OK;
}

int32_t ps_plan_create_kind(const ps_model_desc *model, uint64_t budget, const ps_profile *prof,
                            uint32_t n_tokens, const float *expert_freq, uint32_t kind, ps_plan **out) {
    if (!out) { ps::set_error("out is NULL"); return PS_E_ARG; }
    *out = nullptr;
    ps_plan *p = new (std::nothrow) ps_plan();
    if (!p) { ps::set_error("out of host memory"); return PS_E_NOMEM; }
    int32_t rc = ps::plan_impl(model, budget, prof, n_tokens, expert_freq, kind, p);
    if (rc) { delete p; return rc; }
    *out = p;
    return PS_OK;
}

int32_t ps_plan_create_db(const ps_model_desc *model, uint64_t budget, const ps_profile *prof, const ps_profile_db *db,
                          uint32_t n_tokens, const float *expert_freq, uint32_t kind, ps_plan **out) {
    if (!db) { ps::set_error("profile database is NULL"); return PS_E_ARG; }
    ps::t_db = std::make_shared<const ps_profile_db>(*db);
    const int32_t rc = ps_plan_create_kind(model, budget, prof, n_tokens, expert_freq, kind, out);
    ps::t_db.reset();
    return rc;
}

int32_t ps_plan_summary(const ps_plan *p, ps_plan_summary_t *o) {
    if (!p || !o) { ps::set_error("NULL argument"); return PS_E_ARG; }
    o->budget_bytes = p->budget;
    o->weight_bytes = p->weight_bytes;
    o->resident_bytes = p->resident_bytes;
    o->streamed_bytes = p->streamed_bytes;
    o->scratch_bytes = (uint64_t)p->n_slots * p->slot_bytes;
    o->workspace_bytes = p->ws.total;
    o->slot_bytes = p->slot_bytes;
    o->n_slots = p->n_slots;
    o->n_shards = (uint32_t)p->shards.size();
    o->n_tokens = p->M;
    o->tier = p->tier;
    o->est_step_ms = p->est_step_ms;
    o->est_streamed_bytes_per_step = p->est_streamed_per_step;
    o->cpu_bytes = p->cpu_bytes;
    o->plan_kind = p->kind;
    o->pad = 0;
    o->cpu_fraction = p->cpu_frac;
    for (int k = 0; k < 3; ++k) o->est_kind_ms[k] = p->est_kind[k];
    return PS_OK;
}

int32_t ps_plan_num_shards(const ps_plan *p, uint32_t *n) {
    if (!p || !n) { ps::set_error("NULL argument"); return PS_E_ARG; }
    *n = (uint32_t)p->shards.size();
    return PS_OK;
}

int32_t ps_plan_get_shard(const ps_plan *p, uint32_t i, ps_shard_info *o) {
    if (!p || !o || i >= p->shards.size()) { ps::set_error("shard index out of range"); return PS_E_ARG; }
    const ps::Shard &s = p->shards[i];
    o->layer = s.layer; o->kind = s.kind; o->expert = s.expert; o->cls = s.cls;
    o->tile0 = s.tile0; o->ntiles = s.ntiles; o->resident = s.resident; o->priority_rank = s.rank;
    o->bytes = s.bytes; o->offset = s.offset;
    return PS_OK;
}

void ps_plan_destroy(ps_plan *p) { delete p; }

int32_t ps_tier_table_create(const ps_model_desc *model, uint64_t budget, const ps_profile *prof,
                             const float *expert_freq, ps_tier_table **out) {
    return ps_tier_table_create_kind(model, budget, prof, expert_freq, PS_PLAN_GPU_ONLY, out);
}

int32_t ps_tier_table_create_kind(const ps_model_desc *model, uint64_t budget, const ps_profile *prof,
                                  const float *expert_freq, uint32_t kind, ps_tier_table **out) {
    if (!out) { ps::set_error("out is NULL"); return PS_E_ARG; }
    if (kind > PS_PLAN_AUTO) { ps::set_error("unknown plan kind %u", kind); return PS_E_ARG; }
    *out = nullptr;
    ps_tier_table *tb = new (std::nothrow) ps_tier_table();
    if (!tb) { ps::set_error("out of host memory"); return PS_E_NOMEM; }
    for (uint32_t t = 0; t < PS_NTIERS; ++t) {
        ps_plan *p = new (std::nothrow) ps_plan();
        if (!p) { delete tb; ps::set_error("out of host memory"); return PS_E_NOMEM; }
        // the CPU back-end takes at most 64 tokens, and one token per step over a KV cache: other tiers
        // keep Plan One whatever was asked for
        const uint32_t k = (ps::kTiers[t] > 64 || (model && model->kv_context && t > 0)) ? (uint32_t)PS_PLAN_GPU_ONLY : kind;
        const int32_t rc = ps::plan_impl(model, budget, prof, ps::kTiers[t], expert_freq, k, p);
        if (rc == PS_OK) { tb->plans[t] = p; continue; }
        delete p;
        if (rc != PS_E_BUDGET) { delete tb; return rc; }   // a bad model or profile fails every tier
    }
    *out = tb;
    return PS_OK;
}

int32_t ps_tier_table_create_db(const ps_model_desc *model, uint64_t budget, const ps_profile *prof,
                                const ps_profile_db *db, const float *expert_freq, uint32_t kind,
                                ps_tier_table **out) {
    if (!db) { ps::set_error("profile database is NULL"); return PS_E_ARG; }
    ps::t_db = std::make_shared<const ps_profile_db>(*db);
    const int32_t rc = ps_tier_table_create_kind(model, budget, prof, expert_freq, kind, out);
    ps::t_db.reset();
    return rc;
}

int32_t ps_tier_table_entry(const ps_tier_table *tb, uint32_t tier, ps_tier_entry *o) {
    if (!tb || !o || tier >= PS_NTIERS) { ps::set_error("bad tier table argument"); return PS_E_ARG; }
    std::memset(o, 0, sizeof *o);
    o->tier = tier;
    o->tier_tokens = ps::kTiers[tier];
    o->feasible = tb->plans[tier] ? 1 : 0;
    return o->feasible ? ps_plan_summary(tb->plans[tier], &o->summary) : PS_OK;
}

int32_t ps_tier_table_plan(const ps_tier_table *tb, uint32_t tier, const ps_plan **out) {
    if (!tb || !out || tier >= PS_NTIERS) { ps::set_error("bad tier table argument"); return PS_E_ARG; }
    if (!tb->plans[tier]) { ps::set_error("tier %u (%u tokens) does not fit the budget", tier, ps::kTiers[tier]); return PS_E_ARG; }
    *out = tb->plans[tier];
    return PS_OK;
}

int32_t ps_tier_pick(const ps_tier_table *tb, uint32_t new_tokens, ps_tier_choice *o) {
    if (!tb || !o) { ps::set_error("NULL argument"); return PS_E_ARG; }
    if (new_tokens == 0) { ps::set_error("new_tokens is 0"); return PS_E_ARG; }
    bool found = false;
    double best = 0;
    for (uint32_t t = 0; t < PS_NTIERS; ++t) {
        if (!tb->plans[t]) continue;
        const uint32_t iters = (new_tokens + ps::kTiers[t] - 1) / ps::kTiers[t];
        const double total = (double)iters * tb->plans[t]->est_step_ms;
        if (found && !(total < best)) continue;   // ties keep the lower tier
        found = true;
        best = total;
        o->tier = t; o->tier_tokens = ps::kTiers[t]; o->iterations = iters; o->pad = 0;
        o->est_iter_ms = tb->plans[t]->est_step_ms; o->est_total_ms = total;
    }
    if (!found) { ps::set_error("no token tier fits the budget"); return PS_E_BUDGET; }
    return PS_OK;
}

void ps_tier_table_destroy(ps_tier_table *tb) { delete tb; }

}  // extern "C"
