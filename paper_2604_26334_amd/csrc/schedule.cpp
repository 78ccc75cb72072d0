// Executor schedule as plain data, and its checker.  The schedule is the host issue
// order of copy-stream and compute-stream operations for one forward pass of the
// GPU-only plan (paper Section 3, "Plan One": unpinned sub-layers are copied before
// each use into a VRAM-scratch double buffer while the GPU computes on the other half).
// Host code only; no HIP calls.
#include <algorithm>
#include <cstring>
#include <map>

#include "ps_internal.h"

namespace ps {

void route_host(const float *logits, uint32_t M, uint32_t E, uint32_t k, int32_t *idx) {
    std::vector<char> taken(E);
    for (uint32_t m = 0; m < M; ++m) {
        const float *l = logits + (size_t)m * E;
        std::fill(taken.begin(), taken.end(), 0);
        for (uint32_t j = 0; j < k; ++j) {
            int best = -1;
            for (uint32_t e = 0; e < E; ++e)
                if (!taken[e] && (best < 0 || l[e] > l[best])) best = (int)e;
            taken[best] = 1;
            idx[(size_t)m * k + j] = best;
        }
    }
}

namespace {

struct KernelItem {   // one compute-stream op before copies are interleaved
    Op op;
    int batch = -1;   // slot batch it reads from, -1 if resident only
    bool last_of_batch = false;
};

struct Batch {
    std::vector<Op> copies;
    uint32_t layer = 0;
    bool expert = false;
    uint64_t used = 0;
};

struct Builder {
    const ps_plan *p;
    ps_schedule *out;
    std::vector<KernelItem> kernels;
    std::vector<Batch> batches;
    bool batch_open = false;
    bool host_has_h = false;   // the host copy of the FFN input is current (same layer, fetched once)

    static Op kernel_op(uint32_t kernel, uint32_t layer) {
        Op o;
        o.info.type = PS_OP_KERNEL; o.info.kernel = kernel; o.info.layer = layer;
        o.info.slot = -1; o.info.nshards = 1;
        return o;
    }

    // place shard si into the current batch (opening a new one if needed); returns offset
    uint64_t stage(uint32_t si, uint32_t layer, bool expert, int *batch_out) {
        const Shard &s = p->shards[si];
        if (!batch_open || batches.back().layer != layer || batches.back().expert != expert ||
            batches.back().used + s.bytes > p->slot_bytes) {
            batches.emplace_back();
            batches.back().layer = layer;
            batches.back().expert = expert;
            batch_open = true;
        }
        Batch &b = batches.back();
        const int bi = (int)batches.size() - 1;
        Op c;
        c.info.type = PS_OP_COPY; c.info.layer = layer; c.info.slot = bi % 2;
        c.info.shard0 = si; c.info.nshards = 1; c.info.slot_offset = b.used; c.info.bytes = s.bytes;
        if (expert) c.info.flags |= PS_OPF_WAIT_ROUTER;
        b.copies.push_back(c);
        uint64_t off = b.used;
        b.used += s.bytes;
        *batch_out = bi;
        return off;
    }

    // activation buffers the CPU back-end reads for a sub-layer
    uint32_t cpu_inputs(uint32_t kernel) const {
        const bool resid = !(p->g.m.flags & PS_FLAG_NO_RESIDUAL);
        switch (kernel) {
            case PS_K_GATE_UP: return PS_BUF_H;
            case PS_K_DOWN: return PS_BUF_S | (resid ? PS_BUF_H : 0u);
            case PS_K_OUT: return PS_BUF_X;
        }
        return 0;
    }

    // One matrix: its GPU shards (pinned head, streamed slabs), then its CPU shard if the plan left
    // one in system memory.  The activations the CPU needs are fetched before the GPU kernels are
    // launched, so the GPU works through its slabs while the host computes its rows.
    void add_matrix_kernels(uint32_t kernel, uint32_t layer, uint32_t kind, size_t &si) {
        size_t end = si;
        bool any_cpu = false;
        while (end < p->shards.size() && p->shards[end].layer == layer && p->shards[end].kind == kind) {
            any_cpu |= p->shards[end].resident == 2;
            ++end;
        }
        if (any_cpu) {
            uint32_t need = cpu_inputs(kernel);
            if (host_has_h) need &= ~PS_BUF_H;
            if (need) {
                KernelItem f;
                f.op = kernel_op(kernel, layer);
                f.op.info.type = PS_OP_FETCH; f.op.info.nshards = 0; f.op.info.buffers = need;
                kernels.push_back(f);
            }
            if (cpu_inputs(kernel) & PS_BUF_H) host_has_h = true;
        }
        for (int pass = 0; pass < 2; ++pass)
            for (size_t i = si; i < end; ++i) {
                const Shard &s = p->shards[i];
                if ((s.resident == 2) != (pass == 1)) continue;
                KernelItem k;
                k.op = kernel_op(kernel, layer);
                k.op.info.shard0 = (uint32_t)i;
                k.op.info.bytes = s.bytes;
                if (s.resident == 2) {
                    k.op.info.type = PS_OP_CPU;
                    k.op.info.buffers = cpu_inputs(kernel);
                } else if (!s.resident) {
                    k.op.info.slot_offset = stage((uint32_t)i, layer, false, &k.batch);
                    k.op.info.slot = k.batch % 2;
                }
                kernels.push_back(k);
            }
        si = end;
    }

    // KV-cache shards of a layer (one per kv head, consecutive): one attention launch per run of
    // shards that sit next to each other -- pinned neighbours in the arena, or one slot fill
    void add_kv_kernels(uint32_t layer, size_t &si) {
        KernelItem cur;
        bool open = false;
        uint64_t next_off = 0;   // where the next shard must start to extend the open launch
        while (si < p->shards.size() && p->shards[si].layer == layer && p->shards[si].kind == PS_SHARD_KV) {
            const Shard &s = p->shards[si];
            int batch = -1;
            uint64_t off = s.offset;
            if (!s.resident) off = stage((uint32_t)si, layer, false, &batch);
            if (open && cur.batch == batch && off == next_off) {
                cur.op.info.nshards++;
                cur.op.info.bytes += s.bytes;
            } else {
                if (open) kernels.push_back(cur);
                cur = KernelItem();
                cur.op = kernel_op(PS_K_ATTN, layer);
                cur.op.info.shard0 = (uint32_t)si;
                cur.op.info.bytes = s.bytes;
                cur.batch = batch;
                if (batch >= 0) { cur.op.info.slot = batch % 2; cur.op.info.slot_offset = off; }
                open = true;
            }
            next_off = off + s.bytes;
            ++si;
        }
        if (open) kernels.push_back(cur);
    }

    // sub: which half of the layer a RINV op serves (0 = attention input, 1 = FFN input)
    void add_plain(uint32_t kernel, uint32_t layer, uint32_t flags = 0, uint32_t sub = 0) {
        KernelItem k;
        k.op = kernel_op(kernel, layer);
        k.op.info.flags = flags;
        k.op.info.nshards = 0;
        k.op.info.shard0 = sub;
        kernels.push_back(k);
    }

    void add_expert_launch(uint32_t layer, const std::vector<TaskHost> &tasks, int batch) {
        if (tasks.empty()) return;
        uint64_t bytes = 0;
        for (auto &t : tasks) bytes += p->shards[t.shard].bytes;
        const uint32_t t0 = (uint32_t)out->tasks.size();
        out->tasks.insert(out->tasks.end(), tasks.begin(), tasks.end());
        for (uint32_t kern : {(uint32_t)PS_K_EXPERT_GATE_UP, (uint32_t)PS_K_EXPERT_DOWN}) {
            KernelItem k;
            k.op = kernel_op(kern, layer);
            k.op.info.shard0 = tasks[0].shard; k.op.info.nshards = (uint32_t)tasks.size();
            k.op.info.slot = batch >= 0 ? batch % 2 : -1;
            k.op.info.bytes = kern == PS_K_EXPERT_GATE_UP ? bytes : 0;  // counted once per expert
            k.op.task0 = t0; k.op.ntasks = (uint32_t)tasks.size();
            k.batch = batch;
            kernels.push_back(k);
        }
    }

    // logits: token t of layer l at logits[l * layer_stride + t * n_experts]; only the first n_valid of
    // the plan's M token rows are routed (a last prefill chunk shorter than the tier): the op list keeps
    // the plan's shape, the expert task lists hold the valid tokens' pairs only
    int32_t run(const float *logits, uint64_t layer_stride, uint32_t n_valid) {
        const ModelGeom &g = p->g;
        const auto &m = g.m;
        const uint32_t M = p->M;
        if (g.moe && !logits) { set_error("MoE schedule needs host router logits"); return PS_E_ARG; }
        if (n_valid == 0 || n_valid > M) { set_error("%u valid token rows in a plan of %u", n_valid, M); return PS_E_ARG; }
        std::vector<int32_t> idx((size_t)n_valid * std::max(1u, m.top_k));
        size_t si = 0;
        for (uint32_t l = 0; l < m.n_layers; ++l) {
            host_has_h = false;
            if (g.has_attn) {
                if (M > 1) add_plain(PS_K_RINV, l);
                add_matrix_kernels(PS_K_QKV, l, PS_SHARD_QKV, si);
                if (g.kv) {
                    add_kv_kernels(l, si);
                    add_plain(PS_K_ATTN_COMBINE, l);
                }
                add_matrix_kernels(PS_K_O, l, PS_SHARD_O, si);
            }
            if (M > 1) add_plain(PS_K_RINV, l, 0, 1);
            if (!g.moe) {
                add_matrix_kernels(PS_K_GATE_UP, l, PS_SHARD_GATE_UP, si);
                add_matrix_kernels(PS_K_DOWN, l, PS_SHARD_DOWN, si);
                continue;
            }
            add_plain(PS_K_ROUTE, l, PS_OPF_RECORD_ROUTER);
            batch_open = false;  // expert batches never share a slot fill with other layers
            route_host(logits + (size_t)l * layer_stride, n_valid, m.n_experts, m.top_k, idx.data());
            // shards of this layer's experts are consecutive: si + e
            const size_t e0 = si;
            si += m.n_experts;
            std::vector<TaskHost> resident, streamed, on_cpu;
            for (uint32_t e = 0; e < m.n_experts; ++e) {
                TaskHost t;
                t.shard = (uint32_t)(e0 + e); t.expert = e; t.pair0 = (uint32_t)out->pairs.size();
                for (uint32_t q = 0; q < n_valid * m.top_k; ++q)
                    if (idx[q] == (int32_t)e) out->pairs.push_back((int32_t)q);
                t.npairs = (uint32_t)out->pairs.size() - t.pair0;
                if (!t.npairs) continue;
                const uint32_t where = p->shards[t.shard].resident;
                (where == 1 ? resident : where == 2 ? on_cpu : streamed).push_back(t);
            }
            if (!on_cpu.empty()) {   // the FFN input goes to the host before the GPU's experts are launched
                KernelItem f;
                f.op = kernel_op(PS_K_EXPERT_GATE_UP, l);
                f.op.info.type = PS_OP_FETCH; f.op.info.nshards = 0; f.op.info.buffers = PS_BUF_H;
                kernels.push_back(f);
            }
            add_expert_launch(l, resident, -1);
            std::vector<TaskHost> cur;
            int cur_batch = -1;
            for (auto &t : streamed) {
                int b;
                uint64_t off = stage(t.shard, l, true, &b);
                if (b != cur_batch && !cur.empty()) { add_expert_launch(l, cur, cur_batch); cur.clear(); }
                cur_batch = b;
                t.slot = b % 2; t.slot_offset = off;
                cur.push_back(t);
            }
            add_expert_launch(l, cur, cur_batch);
            batch_open = false;
            if (!on_cpu.empty()) {   // one host step for all of the layer's CPU experts, beside the GPU's launches
                KernelItem k;
                k.op = kernel_op(PS_K_EXPERT_GATE_UP, l);
                k.op.info.type = PS_OP_CPU; k.op.info.buffers = PS_BUF_H;
                k.op.info.shard0 = on_cpu[0].shard; k.op.info.nshards = (uint32_t)on_cpu.size();
                k.op.task0 = (uint32_t)out->tasks.size(); k.op.ntasks = (uint32_t)on_cpu.size();
                for (auto &t : on_cpu) k.op.info.bytes += p->shards[t.shard].bytes;
                out->tasks.insert(out->tasks.end(), on_cpu.begin(), on_cpu.end());
                kernels.push_back(k);
            }
            add_plain(PS_K_COMBINE, l);
        }
        if (m.vocab) {   // output head on the final hidden state (its own RMS factor when several tokens)
            if (M > 1) add_plain(PS_K_RINV, m.n_layers, 0, 2);
            add_matrix_kernels(PS_K_OUT, m.n_layers, PS_SHARD_OUT, si);
        }
        if (si != p->shards.size()) { set_error("internal: schedule did not consume every shard"); return PS_E_STATE; }

        // wait/record flags on kernels, batch boundaries
        std::vector<int> last_kernel(batches.size(), -1), first_kernel(batches.size(), -1);
        for (size_t i = 0; i < kernels.size(); ++i)
            if (kernels[i].batch >= 0) {
                if (first_kernel[kernels[i].batch] < 0) first_kernel[kernels[i].batch] = (int)i;
                last_kernel[kernels[i].batch] = (int)i;
            }
        for (size_t b = 0; b < batches.size(); ++b) {
            kernels[first_kernel[b]].op.info.flags |= PS_OPF_WAIT_READY;
            kernels[last_kernel[b]].op.info.flags |= PS_OPF_RECORD_FREE;
            kernels[last_kernel[b]].last_of_batch = true;
            batches[b].copies.front().info.flags |= PS_OPF_WAIT_SLOT_FREE;
            batches[b].copies.back().info.flags |= PS_OPF_RECORD_READY;
        }

        // host issue order: a batch's copies are issued as soon as (a) the batch two before
        // it has had its last kernel issued (its slot_free record exists) and (b) for expert
        // batches, the layer's routing kernel has been issued (its router_done record exists)
        size_t next_batch = 0;
        std::vector<char> router_issued(m.n_layers, 0);
        std::vector<char> batch_done(batches.size(), 0);
        auto try_issue = [&]() {
            while (next_batch < batches.size()) {
                const Batch &b = batches[next_batch];
                if (next_batch >= 2 && !batch_done[next_batch - 2]) break;
                if (b.expert && !router_issued[b.layer]) break;
                for (auto &c : b.copies) out->ops.push_back(c);
                ++next_batch;
            }
        };
        try_issue();
        for (auto &k : kernels) {
            if (k.batch >= 0 && (size_t)k.batch >= next_batch) {
                set_error("internal: kernel issued before its copies"); return PS_E_STATE;
            }
            out->ops.push_back(k.op);
            if (k.op.info.kernel == PS_K_ROUTE) router_issued[k.op.info.layer] = 1;
            if (k.last_of_batch) batch_done[k.batch] = 1;
            try_issue();
        }
        if (next_batch != batches.size()) { set_error("internal: copies left unissued"); return PS_E_STATE; }
        out->n_slots = p->n_slots; out->slot_bytes = p->slot_bytes; out->n_layers = m.n_layers;
        out->shard_bytes.resize(p->shards.size());
        for (size_t i = 0; i < p->shards.size(); ++i) out->shard_bytes[i] = p->shards[i].bytes;
        if (!batches.empty() && p->n_slots < 2) { set_error("internal: streamed shards but no scratch"); return PS_E_STATE; }
        return PS_OK;
    }
};

}  // namespace

int32_t build_schedule(const ps_plan *plan, const float *router_logits, ps_schedule *out, uint64_t layer_stride,
                       uint32_t n_valid) {
    Builder b{};
    b.p = plan;
    b.out = out;
    return b.run(router_logits, layer_stride ? layer_stride : (uint64_t)plan->M * plan->g.m.n_experts,
                 n_valid ? n_valid : plan->M);
}

// Vector-clock check over the two in-order streams.  An event wait refers to the latest
// record of that event issued earlier in host order (HIP semantics); a wait with no
// earlier record is a no-op.  clock = (copy ops known complete, kernel ops known complete).
int32_t validate_schedule(const ps_schedule *s) {
    struct Clock { int64_t copy = 0, comp = 0; };
    auto join = [](Clock a, Clock b) { return Clock{std::max(a.copy, b.copy), std::max(a.comp, b.comp)}; };
    const size_t n = s->ops.size();
    std::vector<Clock> start(n), end(n);
    std::vector<Clock> ev_ready(2), ev_free(2), ev_router(s->n_layers);
    std::vector<char> has_ready(2, 0);
    Clock copy_tail, comp_tail;
    int64_t ncopy = 0, ncomp = 0;
    struct Region { uint32_t shard; uint64_t off, bytes; int64_t copy_pos; };
    std::vector<std::vector<Region>> content(2);            // what each slot holds, by region
    struct Read { uint64_t off, bytes; int64_t comp_pos; };
    std::vector<std::vector<Read>> reads(2);                // kernel reads since the region was written
    auto overlap = [](uint64_t a0, uint64_t ab, uint64_t b0, uint64_t bb) { return a0 < b0 + bb && b0 < a0 + ab; };
    uint32_t host_valid = 0;      // activation buffers whose host copy is current (PS_BUF_*)
    uint32_t host_layer = ~0u;

    for (size_t i = 0; i < n; ++i) {
        const Op &op = s->ops[i];
        const ps_op_info &o = op.info;
        if (o.type == PS_OP_COPY) {
            if (o.slot < 0 || o.slot >= (int)s->n_slots || o.slot_offset + o.bytes > s->slot_bytes) {
                set_error("op %zu: copy outside slot bounds", i); return PS_E_STATE;
            }
            Clock c = copy_tail;
            if (o.flags & PS_OPF_WAIT_SLOT_FREE) c = join(c, ev_free[o.slot]);
            if (o.flags & PS_OPF_WAIT_ROUTER) c = join(c, ev_router[o.layer]);
            start[i] = c;
            // WAR: every kernel that read an overlapping region of this slot must be complete
            for (const Read &r : reads[o.slot])
                if (overlap(o.slot_offset, o.bytes, r.off, r.bytes) && c.comp < r.comp_pos) {
                    set_error("op %zu: copy into slot %d overwrites data still being read (kernel #%lld)", i,
                              o.slot, (long long)r.comp_pos);
                    return PS_E_STATE;
                }
            auto &rd = reads[o.slot];
            rd.erase(std::remove_if(rd.begin(), rd.end(), [&](const Read &r) {
                         return overlap(o.slot_offset, o.bytes, r.off, r.bytes); }), rd.end());
            auto &ct = content[o.slot];
            ct.erase(std::remove_if(ct.begin(), ct.end(), [&](const Region &r) {
                         return overlap(o.slot_offset, o.bytes, r.off, r.bytes); }), ct.end());
            ++ncopy;
            ct.push_back(Region{o.shard0, o.slot_offset, o.bytes, ncopy});
            c.copy = ncopy;
            end[i] = c; copy_tail = c;
            if (o.flags & PS_OPF_RECORD_READY) { ev_ready[o.slot] = c; has_ready[o.slot] = 1; }
        } else {
            // host copies of activations: fetched on the compute stream (the host waits), stale once
            // the layer moves on or a later op rewrites the buffer; a CPU shard reads only current ones
            if (o.layer != host_layer) { host_valid = 0; host_layer = o.layer; }
            if (o.type == PS_OP_FETCH) {
                if (!o.buffers || o.slot >= 0) { set_error("op %zu: malformed fetch", i); return PS_E_STATE; }
                host_valid |= o.buffers;
            } else if (o.type == PS_OP_CPU) {
                if (o.slot >= 0 || (o.flags & (PS_OPF_WAIT_READY | PS_OPF_RECORD_FREE))) {
                    set_error("op %zu: a CPU shard does not touch the scratch slots", i); return PS_E_STATE;
                }
                if (o.buffers & ~host_valid) {
                    set_error("op %zu: CPU shard reads activations (mask %u) that were not fetched (have %u)", i, o.buffers, host_valid);
                    return PS_E_STATE;
                }
            }
            if (o.type != PS_OP_FETCH) {
                if (o.kernel == PS_K_O || o.kernel == PS_K_COMBINE) host_valid &= ~PS_BUF_H;
                if (o.kernel == PS_K_GATE_UP || o.kernel == PS_K_EXPERT_GATE_UP) host_valid &= ~PS_BUF_S;
                if (o.kernel == PS_K_DOWN || o.kernel == PS_K_COMBINE) host_valid &= ~PS_BUF_X;
            }
            Clock c = comp_tail;
            if (o.flags & PS_OPF_WAIT_READY) {
                if (o.slot < 0 || !has_ready[o.slot]) { set_error("op %zu: waits for a slot never filled", i); return PS_E_STATE; }
                c = join(c, ev_ready[o.slot]);
            }
            start[i] = c;
            // RAW: each streamed shard this kernel reads must be in its slot, copy complete
            auto check_read = [&](uint32_t shard, int slot, uint64_t off) -> bool {
                const uint64_t bytes = s->shard_bytes[shard];
                for (const Region &r : content[slot])
                    if (r.shard == shard && r.off == off && r.bytes == bytes) {
                        if (c.copy < r.copy_pos) return false;
                        reads[slot].push_back(Read{off, bytes, ncomp + 1});
                        return true;
                    }
                return false;
            };
            if (op.ntasks) {
                for (uint32_t t = op.task0; t < op.task0 + op.ntasks; ++t)
                    if (s->tasks[t].slot >= 0 && !check_read(s->tasks[t].shard, s->tasks[t].slot, s->tasks[t].slot_offset)) {
                        set_error("op %zu: expert kernel reads shard %u before its copy completed", i, s->tasks[t].shard);
                        return PS_E_STATE;
                    }
            } else if (o.slot >= 0 && o.nshards) {
                uint64_t off = o.slot_offset;   // a run of shards lies back to back in the slot
                for (uint32_t k = 0; k < o.nshards; ++k) {
                    if (!check_read(o.shard0 + k, o.slot, off)) {
                        set_error("op %zu: kernel reads shard %u before its copy completed", i, o.shard0 + k);
                        return PS_E_STATE;
                    }
                    off += s->shard_bytes[o.shard0 + k];
                }
            }
            ++ncomp;
            c.comp = ncomp;
            end[i] = c; comp_tail = c;
            if (o.flags & PS_OPF_RECORD_FREE) ev_free[o.slot] = c;
            if (o.flags & PS_OPF_RECORD_ROUTER) ev_router[o.layer] = c;
        }
    }
    return PS_OK;
}

}  // namespace ps

extern "C" {

int32_t ps_schedule_create(const ps_plan *plan, const float *router_logits, ps_schedule **out) {
    if (!plan || !out) { ps::set_error("NULL argument"); return PS_E_ARG; }
    *out = nullptr;
    ps_schedule *s = new (std::nothrow) ps_schedule();
    if (!s) { ps::set_error("out of host memory"); return PS_E_NOMEM; }
    int32_t rc = ps::build_schedule(plan, router_logits, s);
    if (rc) { delete s; return rc; }
    *out = s;
    return PS_OK;
}

int32_t ps_schedule_num_ops(const ps_schedule *s, uint32_t *n) {
    if (!s || !n) { ps::set_error("NULL argument"); return PS_E_ARG; }
    *n = (uint32_t)s->ops.size();
    return PS_OK;
}

int32_t ps_schedule_get_op(const ps_schedule *s, uint32_t i, ps_op_info *out) {
    if (!s || !out || i >= s->ops.size()) { ps::set_error("op index out of range"); return PS_E_ARG; }
    *out = s->ops[i].info;
    return PS_OK;
}

int32_t ps_schedule_validate(const ps_schedule *s) {
    if (!s) { ps::set_error("NULL argument"); return PS_E_ARG; }
    return ps::validate_schedule(s);
}

void ps_schedule_destroy(ps_schedule *s) { delete s; }

int32_t ps_route_host(const float *logits, uint32_t M, uint32_t E, uint32_t k, int32_t *idx) {
    if (!logits || !idx || k == 0 || k > E) { ps::set_error("bad routing arguments"); return PS_E_ARG; }
    ps::route_host(logits, M, E, k, idx);
    return PS_OK;
}

}  // extern "C"
