// Profile database and the time estimate drawn from it (paper Section 3, profiler-based timing
// estimation): benchmarked kernels keyed by operation, quantisation level, CPU thread count and
// dimensions; a kernel to be priced takes the rate of its exact match, else the nearest entry of
// the same operation / quantisation / thread count gives the FLOPS roof of a roofline whose memory
// roof is the machine's bandwidth for that device, else it is skipped.  Host code only.
#include <cmath>
#include <cstdio>
#include <cstring>

#include "ps_internal.h"

namespace ps {

void op_work(uint32_t op, uint32_t quant, uint64_t n, uint64_t k, uint64_t m, double *flops, double *bytes) {
    if (op == PS_OPK_H2D) { *flops = 0.0; *bytes = (double)n; return; }
    *flops = 2.0 * (double)n * (double)k * (double)m;
    *bytes = (double)n * (double)k * (quant / 8.0 + 2.0 / 32.0) + 2.0 * (double)m * (double)(k + n);
}

int32_t db_estimate(const ps_profile_db *db, double bandwidth_gbps, uint32_t op, uint32_t quant, uint32_t threads,
                    uint64_t n, uint64_t k, uint64_t m, ps_prof_estimate *out) {
    ps_prof_estimate r{};
    r.neighbour = -1;
    op_work(op, quant, n, k, m, &r.flops, &r.bytes);
    int best = -1;
    double best_d = 0;
    for (size_t i = 0; i < db->entries.size(); ++i) {
        const ps_prof_entry &e = db->entries[i];
        if (e.op != op || e.quant != quant || e.threads != threads) continue;
        if (e.n == n && e.k == k && e.m == m) {
            r.ms = e.ms; r.match = PS_MATCH_EXACT; r.neighbour = (int32_t)i;
            *out = r;
            return PS_OK;
        }
        const double dn = std::log2((double)e.n) - std::log2((double)n), dk = std::log2((double)e.k) - std::log2((double)k),
                     dm = std::log2((double)e.m) - std::log2((double)m);
        const double d = std::sqrt(dn * dn + dk * dk + dm * dm);
        if (best < 0 || d < best_d) { best = (int)i; best_d = d; }   // equal distances keep the earlier entry
    }
    if (best < 0) { r.match = PS_MATCH_NONE; *out = r; return PS_OK; }
    const ps_prof_entry &e = db->entries[best];
    double e_flops, e_bytes;
    op_work(e.op, e.quant, e.n, e.k, e.m, &e_flops, &e_bytes);
    r.match = PS_MATCH_NEIGHBOUR;
    r.neighbour = best;
    if (op == PS_OPK_H2D) {          // a copy has no FLOPS: its byte rate takes that place
        r.ms = r.bytes / (e_bytes / e.ms);
        r.compute_bound = 0;
    } else {
        const double roof_flops = e_flops / (e.ms * 1e-3), roof_bw = bandwidth_gbps * 1e9;
        r.compute_bound = r.flops / r.bytes >= roof_flops / roof_bw;
        r.ms = r.compute_bound ? r.flops / roof_flops * 1e3 : r.bytes / roof_bw * 1e3;
    }
    *out = r;
    return PS_OK;
}

}  // namespace ps

extern "C" {

int32_t ps_profile_db_create(ps_profile_db **out) {
    if (!out) { ps::set_error("out is NULL"); return PS_E_ARG; }
    *out = new (std::nothrow) ps_profile_db();
    if (!*out) { ps::set_error("out of host memory"); return PS_E_NOMEM; }
    return PS_OK;
}

void ps_profile_db_destroy(ps_profile_db *db) { delete db; }

int32_t ps_profile_db_add(ps_profile_db *db, const ps_prof_entry *e) {
    if (!db || !e) { ps::set_error("NULL argument"); return PS_E_ARG; }
    if (e->op > PS_OPK_H2D || e->n == 0 || e->k == 0 || e->m == 0 || !(e->ms > 0)) {
        ps::set_error("profile entry needs a known op, non-zero dimensions and a positive time"); return PS_E_ARG;
    }
    for (ps_prof_entry &o : db->entries)   // one entry per key: a new measurement replaces the old one
        if (o.op == e->op && o.quant == e->quant && o.threads == e->threads && o.n == e->n && o.k == e->k && o.m == e->m) {
            o.ms = e->ms;
            return PS_OK;
        }
    db->entries.push_back(*e);
    return PS_OK;
}

int32_t ps_profile_db_count(const ps_profile_db *db, uint32_t *n) {
    if (!db || !n) { ps::set_error("NULL argument"); return PS_E_ARG; }
    *n = (uint32_t)db->entries.size();
    return PS_OK;
}

int32_t ps_profile_db_get(const ps_profile_db *db, uint32_t i, ps_prof_entry *out) {
    if (!db || !out || i >= db->entries.size()) { ps::set_error("profile entry index out of range"); return PS_E_ARG; }
    *out = db->entries[i];
    return PS_OK;
}

int32_t ps_profile_db_estimate(const ps_profile_db *db, double bandwidth_gbps, uint32_t op, uint32_t quant, uint32_t threads,
                               uint64_t n, uint64_t k, uint64_t m, ps_prof_estimate *out) {
    if (!db || !out || n == 0 || k == 0 || m == 0 || op > PS_OPK_H2D || (op != PS_OPK_H2D && !(bandwidth_gbps > 0))) {
        ps::set_error("bad profile look-up argument"); return PS_E_ARG;
    }
    return ps::db_estimate(db, bandwidth_gbps, op, quant, threads, n, k, m, out);
}

int32_t ps_profile_db_save(const ps_profile_db *db, const char *path) {
    if (!db || !path) { ps::set_error("NULL argument"); return PS_E_ARG; }
    FILE *f = std::fopen(path, "w");
    if (!f) { ps::set_error("cannot write %s", path); return PS_E_ARG; }
    std::fprintf(f, "# op quant threads n k m ms\n");
    for (const ps_prof_entry &e : db->entries)
        std::fprintf(f, "%u %u %u %llu %llu %llu %.9g\n", e.op, e.quant, e.threads, (unsigned long long)e.n,
                     (unsigned long long)e.k, (unsigned long long)e.m, e.ms);
    const bool ok = std::fclose(f) == 0;
    if (!ok) { ps::set_error("write to %s failed", path); return PS_E_ARG; }
    return PS_OK;
}

int32_t ps_profile_db_load(ps_profile_db *db, const char *path) {
    if (!db || !path) { ps::set_error("NULL argument"); return PS_E_ARG; }
    FILE *f = std::fopen(path, "r");
    if (!f) { ps::set_error("cannot read %s", path); return PS_E_ARG; }
    char line[256];
    int32_t rc = PS_OK;
    while (rc == PS_OK && std::fgets(line, sizeof line, f)) {
        if (line[0] == '#' || line[0] == '\n') continue;
        ps_prof_entry e{};
        unsigned long long n, k, m;
        if (std::sscanf(line, "%u %u %u %llu %llu %llu %lf", &e.op, &e.quant, &e.threads, &n, &k, &m, &e.ms) != 7) {
            ps::set_error("malformed profile line: %.60s", line);
            rc = PS_E_ARG;
            break;
        }
        e.n = n; e.k = k; e.m = m;
        rc = ps_profile_db_add(db, &e);
    }
    std::fclose(f);
    return rc;
}

}  // extern "C"
