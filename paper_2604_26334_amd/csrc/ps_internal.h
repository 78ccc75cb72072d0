// Internal host-side structures shared by the planner, the schedule builder,
// the packer and the executor.  Nothing here is part of the C ABI.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <memory>
#include <string>
#include <vector>

#include "pshard.h"

namespace ps {

constexpr uint32_t kNoExpert = 0xFFFFFFFFu;
constexpr uint32_t kTileRows = 16;       // rows of one physical row-tile
constexpr uint32_t kSuperK = 128;        // k extent of one super-block (4 blocks of 32)
constexpr uint32_t kGroupSb = 8;         // super-blocks per scale group
constexpr uint64_t kSbBytes = 1024;      // 16 rows x 128 k x 4 bit
constexpr uint64_t kAlign = 256;
constexpr uint32_t kAttnChunk = 128;    // granule the attention partials are sized by (multiple of 64)
constexpr uint32_t kAttnOnePassTokens = 256;   // plans of this many tokens and more: attention without partial records
constexpr uint32_t kAttnPosPerWg = 256; // positions one attention workgroup covers (a multiple of kAttnChunk)

void set_error(const char *fmt, ...);

inline uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

// Geometry of one packed matrix.  A row-tile (16 physical rows, full K) is a
// contiguous run of scale groups; group g holds min(8, nsb - 8g) super-blocks
// of nibbles (1024 B each, lane-ordered) followed by 1024 B of scales.
struct MatGeom {
    uint32_t K = 0, rows = 0, ntiles = 0, nsb = 0, ngroups = 0, quantum_tiles = 0;
    uint64_t tile_bytes = 0, bytes = 0;
};
MatGeom make_geom(uint32_t rows, uint32_t K, bool paired);

struct ModelGeom {
    ps_model_desc m{};
    bool has_attn = false, moe = false, kv = false;   // kv: real attention over a KV cache
    uint64_t kv_shard_bytes = 0;                      // K + V of one kv head at full capacity
    uint32_t qkv_w = 0, attn_w = 0, ffn_i = 0;
    MatGeom qkv, o, gate_up, down, head;  // gate_up/down are per expert for MoE; head: output projection
    uint64_t expert_bytes = 0;
};
int32_t make_model_geom(const ps_model_desc *m, ModelGeom *out);

// Activation / table workspace at the head of the arena, sized for M tokens.
struct Workspace {
    uint64_t x0 = 0, x1 = 0, h = 0, qkv = 0, s = 0, y = 0, rinv = 0, ridx = 0, rw = 0,
             logits = 0, tasks = 0, pairs = 0, partial = 0,
             attn = 0, apart = 0, kvhome = 0, ctx = 0, cpu_y = 0, total = 0;   // attention output, chunk partials, cache home table, CPU experts' results
    uint64_t qkv_bytes = 0, h_bytes = 0, s_bytes = 0, tasks_bytes = 0, pairs_bytes = 0, logits_bytes = 0;
};
Workspace make_workspace(const ModelGeom &g, uint32_t M, bool cpu_experts = false);
// split-K of the batched-decode GEMM (2..64 tokens): super-blocks per part, 0 = no split.  A
// function of the matrix and the token count only, so every placement sums the same partials.
uint32_t gemm_sb_per_part(const MatGeom &mg, uint32_t M);

struct Shard {
    uint32_t layer = 0, kind = 0, expert = kNoExpert, cls = 0, tile0 = 0, ntiles = 0;
    uint32_t resident = 0, rank = 0;   // resident: 1 pinned in VRAM, 0 streamed, 2 run on the CPU
    uint64_t bytes = 0, offset = 0;
};

struct DeviceTask {       // one expert of a grouped launch (device-visible, 32 bytes)
    uint64_t w_gate_up;   // device address of the expert's gate/up tiles
    uint64_t w_down;      // device address of its down tiles
    uint32_t pair0;       // first entry in the pair list
    uint32_t npairs;      // (token, rank) pairs routed to this expert
    uint32_t expert, pad;
};

struct Op {
    ps_op_info info{};
    uint32_t task0 = 0, ntasks = 0;  // expert kernels: range in Schedule::tasks
};

struct TaskHost {
    uint32_t shard = 0;      // plan shard index of the expert
    int32_t slot = -1;       // -1 resident
    uint64_t slot_offset = 0;
    uint32_t pair0 = 0, npairs = 0, expert = 0;
};

}  // namespace ps

struct ps_plan {
    ps::ModelGeom g;
    ps_profile prof{};
    uint64_t budget = 0;
    uint32_t M = 0, tier = 0;
    ps::Workspace ws;
    // arena layout: [pinned shards in priority order from 0 | (free) | slot 0 | slot 1 | workspace]:
    // the workspace and the slots sit at the END, so that a shard pinned in two token tiers' plans
    // under one budget has the same arena offset in both (the tiers differ in workspace size only)
    uint64_t slot_bytes = 0, scratch_off = 0, pinned_off = 0, ws_off = 0;
    uint32_t n_slots = 0;
    std::vector<ps::Shard> shards;  // execution order
    uint64_t weight_bytes = 0, resident_bytes = 0, streamed_bytes = 0, cpu_bytes = 0;
    double est_step_ms = 0, est_streamed_per_step = 0;
    uint32_t kind = PS_PLAN_GPU_ONLY;   // which of the three schedule plans this is
    double cpu_frac = 0;                // Plan Three: CPU share of each unpinned eligible matrix
    double est_kind[3] = {-1, -1, -1};  // estimates per plan kind (all three after HeuristicSplit)
    std::shared_ptr<const ps_profile_db> db;   // optional: shard times come from here
    uint32_t db_threads = 0;                   // thread count of the database's CPU entries
};

struct ps_profile_db {
    std::vector<ps_prof_entry> entries;
};

struct ps_tier_table {
    ps_plan *plans[PS_NTIERS] = {};   // null: infeasible under this budget
    ~ps_tier_table() { for (ps_plan *p : plans) delete p; }
};

struct ps_schedule {
    std::vector<ps::Op> ops;
    std::vector<ps::TaskHost> tasks;
    std::vector<int32_t> pairs;  // token*top_k + rank, grouped by task
    uint32_t n_slots = 0, n_layers = 0;
    uint64_t slot_bytes = 0;
    std::vector<uint64_t> shard_bytes;
};

namespace ps {
void op_work(uint32_t op, uint32_t quant, uint64_t n, uint64_t k, uint64_t m, double *flops, double *bytes);
int32_t db_estimate(const ps_profile_db *db, double bandwidth_gbps, uint32_t op, uint32_t quant, uint32_t threads,
                    uint64_t n, uint64_t k, uint64_t m, ps_prof_estimate *out);
// router_logits: token t of layer l at [l * layer_stride + t * n_experts] (layer_stride 0: the plan's
// M * n_experts); n_valid: token rows that carry data, 1..M (0: all M)
int32_t build_schedule(const ps_plan *plan, const float *router_logits, ps_schedule *out, uint64_t layer_stride = 0,
                       uint32_t n_valid = 0);
int32_t validate_schedule(const ps_schedule *s);
void route_host(const float *logits, uint32_t M, uint32_t E, uint32_t k, int32_t *idx);
// pack logical rows [16*logical_tile, +16) of a [N][K] matrix (scales fp16 [N][K/32],
// codes u8 [N][K]) into one physical row-tile image of g.tile_bytes bytes at dst.
void pack_tile(const MatGeom &g, const uint16_t *scales, const uint8_t *codes,
               uint32_t logical_tile, uint8_t *dst);
}  // namespace ps
