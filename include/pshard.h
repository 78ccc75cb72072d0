/*
 * pshard -- C ABI of the pipelined-sharding hot path for one MI355X (gfx950).
 *
 * What the library does (paper Section 3, "Pipelined Sharding", Algorithm 1 and
 * the GPU-only plan, "Plan One"): a decoder weight stack in a 4-bit block
 * format is cut at sub-layer granularity into shards; a planner pins shards
 * into a fixed VRAM budget by priority (attention before FFN) and leaves the
 * rest in pinned host memory; at run time host shards are copied on a copy
 * stream into a double-buffered VRAM scratch while the compute stream runs the
 * dequantising matmul kernels on the previous shard.  The method is lossless:
 * outputs do not depend on the budget or on where a shard lives.
 * Around that core: the token-tier table with PickTier, the KV cache as a shard
 * class with decode attention, the output head as the lowest priority class,
 * the two plans that run unpinned low-priority shards on the CPU ("Plan Two",
 * "Plan Three") with HeuristicSplit choosing among the three, and the profile
 * database the time estimates can be drawn from.  Plan One is what every entry
 * point does unless a plan kind is asked for; nothing falls back to the CPU.
 *
 * Conventions
 *  - every function returns 0 (PS_OK) or a negative PS_E_* code; nothing throws
 *    or exits across the boundary; ps_last_error() gives a thread-local text.
 *  - "host" / "device" is stated for every pointer.  The library never
 *    allocates device memory: the caller hands one VRAM arena whose size is the
 *    budget.  Pinned host memory for streamed shards is allocated and owned by
 *    the library (hipHostMalloc).
 *  - streams are hipStream_t handles passed as void*, owned by the caller,
 *    default priority.  One ps_stack is used from one host thread at a time.
 *
 * Logical weight format (benchmark definition; the paper only says "q4"):
 *  blocks of 32 weights along K, one fp16 scale d per block, one 4-bit code q
 *  per weight, w = d * (q - 8).  At the boundary a matrix [N outputs][K inputs]
 *  is two host arrays: scales, fp16 bits, [N][K/32]; codes, one code per byte,
 *  [N][K].  The physical layout in VRAM / pinned memory is private.
 *  Constraints: K % 128 == 0, K <= 16384, output rows % 16 == 0, head_dim == 128.
 */
#ifndef PSHARD_H
#define PSHARD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PS_OK 0
#define PS_E_ARG (-1)    /* bad argument / unsupported shape                      */
#define PS_E_BUDGET (-2) /* budget < workspace + two minimum scratch slots        */
#define PS_E_HIP (-3)    /* a HIP runtime call failed (text in ps_last_error)     */
#define PS_E_STATE (-4)  /* call order violated (e.g. forward before all loads)   */
#define PS_E_NOMEM (-5)  /* host allocation failed                                */

/* logical matrices handed to ps_stack_load_matrix */
#define PS_MAT_QKV 0
#define PS_MAT_O 1
#define PS_MAT_GATE 2
#define PS_MAT_UP 3
#define PS_MAT_DOWN 4
#define PS_MAT_OUT 5 /* output head [vocab][hidden], loaded with layer = n_layers */

/* shard kinds in a plan.  GATE_UP is gate and up interleaved in 16-row tiles so
 * that one slab yields finished SwiGLU outputs; EXPERT is one whole MoE expert
 * (its gate/up tiles followed by its down tiles), never split. */
#define PS_SHARD_QKV 0
#define PS_SHARD_O 1
#define PS_SHARD_GATE_UP 2
#define PS_SHARD_DOWN 3
#define PS_SHARD_EXPERT 4
#define PS_SHARD_KV 5 /* K and V cache of one kv head of one layer (field `expert` = kv head) */
#define PS_SHARD_OUT 6 /* N-slab of the output head (class "outputs"); layer field = n_layers */

/* priority classes, in the paper's order (Section 3, planning phase):
 * attention, KV cache, FFN, outputs. */
#define PS_CLASS_ATTN 0
#define PS_CLASS_KVCACHE 1
#define PS_CLASS_FFN 2
#define PS_CLASS_OUTS 3

/* where the shards that are not pinned run (Section 3, the three schedule plans) */
#define PS_PLAN_GPU_ONLY 0 /* Plan One: all on the GPU, streamed through the VRAM scratch double buffer */
#define PS_PLAN_STATIC 1   /* Plan Two: unpinned FFN / output shards stay in system memory and run on
                              the CPU; only activations cross PCIe; no scratch unless an attention or
                              cache shard is unpinned                                                 */
#define PS_PLAN_DYNAMIC 2  /* Plan Three: each unpinned FFN / output matrix is split, part streamed to
                              the GPU and part run on the CPU at the same time                        */
#define PS_PLAN_AUTO 3     /* HeuristicSplit: build all three, keep the one with the lowest estimate  */

#define PS_FLAG_NO_ATTN 1u     /* layers have no attention sub-layer (FFN block only) */
#define PS_FLAG_NO_RESIDUAL 2u /* dense FFN output is not added to its input (the bare FFN block of
                                  benchmark config 1); PS_E_ARG together with MoE layers */

/* token tiers of the paper's tier table (Section 3, inference phase) */
#define PS_NTIERS 11
/* {1, 4, 16, 32, 64, 512, 1024, 2048, 4096, 8192, 16384} -- see ps_tier_tokens */

typedef struct ps_model_desc {
    uint32_t n_layers;
    uint32_t hidden;       /* H                                                  */
    uint32_t n_q_heads;    /* 0 with PS_FLAG_NO_ATTN                             */
    uint32_t n_kv_heads;
    uint32_t head_dim;     /* must be 128 when attention is present              */
    uint32_t ffn_inter;    /* dense FFN width I, 0 for MoE                       */
    uint32_t n_experts;    /* 0 for dense                                        */
    uint32_t top_k;
    uint32_t expert_inter; /* per-expert FFN width                               */
    uint32_t flags;        /* PS_FLAG_*                                          */
    float rms_eps;
    uint32_t kv_context;   /* 0: attention is the identity on V (no cache).  > 0: causal softmax attention over
                              a KV cache with room for kv_context positions per kv head; a forward takes
                              one new token, or a chunk of new tokens (a plan's token count must be below
                              kv_context; chunks take the GPU-only plan)                             */
    uint32_t vocab;        /* 0: no output head.  > 0 (multiple of 16): after the last layer the final
                              hidden state is RMS-normalised and projected to `vocab` logits by one
                              more 4-bit matrix, whose shards form the lowest priority class
                              ("outputs", Section 3 planning phase)                                  */
} ps_model_desc;

/* measured (ps_profile_measure) or caller-supplied machine profile; the
 * planner's time estimate uses nothing else (paper Section 3, timing
 * estimation: a kernel is priced compute-bound or memory-bound). */
typedef struct ps_profile {
    double h2d_gbps;               /* pinned host -> device copy rate, GB/s      */
    double gemv_gbps;              /* weight bytes/s the decode kernels sustain  */
    double gemm_tflops[PS_NTIERS]; /* dequant-GEMM rate at each token tier       */
    double launch_us;              /* fixed cost per kernel launch               */
    /* CPU back-end (plans Two and Three); cpu_gbps == 0 means "no CPU back-end": such plans are
     * rejected and PS_PLAN_AUTO keeps Plan One */
    double cpu_gbps;               /* packed weight bytes/s of the CPU kernel, one token, alone     */
    double cpu_gbps_busy;          /* the same while H2D weight copies run (shared memory controller;
                                      Section 3, Plan Three); 0: use cpu_gbps                        */
    double h2d_gbps_busy;          /* H2D copy rate while the CPU kernel runs; 0: use h2d_gbps      */
    double cpu_tokens_free;        /* tokens up to which the CPU kernel stays memory-bound: its time
                                      is priced bytes / rate * max(1, n_tokens / cpu_tokens_free)    */
    double cpu_sync_us;            /* fixed cost of one CPU shard: activations to the host, wake-up,
                                      result back                                                    */
} ps_profile;

typedef struct ps_shard_info {
    uint32_t layer;
    uint32_t kind;          /* PS_SHARD_*                                        */
    uint32_t expert;        /* expert id, 0xFFFFFFFF if none                     */
    uint32_t cls;           /* PS_CLASS_*                                        */
    uint32_t tile0;         /* first 16-row tile of the slab within its matrix   */
    uint32_t ntiles;        /* number of 16-row tiles (EXPERT: gate/up + down)   */
    uint32_t resident;      /* 1 = pinned in VRAM; 0 = in pinned host memory, streamed to the
                               scratch before each use; 2 = in pinned host memory, run on the CPU */
    uint32_t priority_rank; /* position in the priority order (0 = first)        */
    uint64_t bytes;         /* packed bytes of this shard                        */
    uint64_t offset;        /* resident: byte offset in the arena (pinned shards fill it from 0 in
                               priority order; scratch slots and workspace end it); streamed:
                               byte offset in the library's host shard pool      */
} ps_shard_info;

typedef struct ps_plan_summary_t {
    uint64_t budget_bytes;
    uint64_t weight_bytes;    /* all shards                                      */
    uint64_t resident_bytes;  /* pinned in VRAM                                  */
    uint64_t streamed_bytes;  /* left in host memory (whole stack)               */
    uint64_t scratch_bytes;   /* n_slots * slot_bytes                            */
    uint64_t workspace_bytes; /* activations and tables for n_tokens             */
    uint64_t slot_bytes;
    uint32_t n_slots;         /* 0 or 2                                          */
    uint32_t n_shards;
    uint32_t n_tokens;
    uint32_t tier;            /* index into the tier table used for the estimate */
    double est_step_ms;       /* sum over shards of max(compute, next copy)      */
    double est_streamed_bytes_per_step; /* expected bytes crossing PCIe per step */
    uint64_t cpu_bytes;       /* shards run on the CPU (subset of streamed_bytes' complement: counted
                                 in neither resident_bytes nor streamed_bytes)                       */
    uint32_t plan_kind;       /* PS_PLAN_GPU_ONLY / STATIC / DYNAMIC: what this plan is              */
    uint32_t pad;
    double cpu_fraction;      /* Plan Three: share of each unpinned FFN / output matrix on the CPU   */
    double est_kind_ms[3];    /* PS_PLAN_AUTO: the estimate of each of the three plans, < 0 where a
                                 plan could not be built; otherwise only [plan_kind] is filled       */
} ps_plan_summary_t;

typedef struct ps_stats {
    uint64_t resident_bytes_step; /* weight bytes read in place in the last forward */
    uint64_t streamed_bytes_step; /* weight bytes copied H2D in the last forward    */
    uint32_t n_copies, n_kernels;
    /* the rest is valid only after a forward with profiling on, once complete   */
    double copy_ms;     /* sum of copy durations on the copy stream              */
    double compute_ms;  /* sum of kernel durations on the compute stream         */
    double wall_ms;     /* first op start to last op end                         */
    double overlap;     /* (copy + compute - wall) / min(copy, compute), 0 if either is 0 */
    double h2d_gbps;    /* streamed_bytes_step / copy_ms                         */
    uint64_t cpu_bytes_step; /* weight bytes read by the CPU back-end in the last forward           */
    double cpu_ms;      /* host time inside the CPU kernel in the last forward (always valid)       */
    double cpu_wait_ms; /* host time waiting for activations to arrive from the GPU (always valid)  */
    uint32_t graph_replay; /* 1 if the last forward was one HIP-graph launch (decode mode 1), else 0  */
    uint32_t reserved;
} ps_stats;

/* one operation of an executor schedule, as plain data (see ps_schedule_*) */
#define PS_OP_COPY 0
#define PS_OP_KERNEL 1
#define PS_OP_CPU 2   /* one shard computed by the CPU back-end (kernel = the sub-layer, PS_K_*), its
                         result uploaded on the compute stream; the host blocks while it computes   */
#define PS_OP_FETCH 3 /* compute stream copies the activation buffers in `buffers` to the host and the
                         host waits for them: issued before the GPU kernels of a matrix that also has
                         a CPU shard, so both sides then work on the matrix at the same time        */
#define PS_BUF_H 1u   /* FFN input (the attention half's output)     */
#define PS_BUF_S 2u   /* SwiGLU output (the down projection's input) */
#define PS_BUF_X 4u   /* final hidden state (the output head's input) */
#define PS_K_RINV 0
#define PS_K_QKV 1
#define PS_K_O 2
#define PS_K_GATE_UP 3
#define PS_K_DOWN 4
#define PS_K_ROUTE 5
#define PS_K_EXPERT_GATE_UP 6
#define PS_K_EXPERT_DOWN 7
#define PS_K_COMBINE 8
#define PS_K_ATTN 9          /* decode attention over a run of kv-head cache shards          */
#define PS_K_ATTN_COMBINE 10 /* merge the position chunks, add the new token, append its rows */
#define PS_K_OUT 11          /* output head: logits = W_out RMSNorm(x_final)                   */
#define PS_OPF_WAIT_SLOT_FREE 1u  /* copy stream waits for slot_free[slot]        */
#define PS_OPF_WAIT_ROUTER 2u     /* copy stream waits for router_done[layer]     */
#define PS_OPF_RECORD_READY 4u    /* copy stream records slot_ready[slot] after   */
#define PS_OPF_WAIT_READY 8u      /* compute stream waits for slot_ready[slot]    */
#define PS_OPF_RECORD_FREE 16u    /* compute stream records slot_free[slot] after */
#define PS_OPF_RECORD_ROUTER 32u  /* compute stream records router_done[layer]    */

typedef struct ps_op_info {
    uint32_t type;   /* PS_OP_*                                                  */
    uint32_t kernel; /* PS_K_* for kernels                                       */
    uint32_t layer;
    uint32_t flags;  /* PS_OPF_*                                                 */
    int32_t slot;    /* scratch slot touched, -1 if none                         */
    uint32_t shard0; /* first plan shard this op copies / reads                  */
    uint32_t nshards;/* number of consecutive task entries (expert batches) or 1 */
    uint32_t buffers;/* PS_BUF_*: FETCH copies these to the host, CPU reads these there */
    uint64_t slot_offset; /* byte offset inside the slot (copy destination / kernel source) */
    uint64_t bytes;  /* weight bytes copied or read                              */
} ps_op_info;

typedef struct ps_plan ps_plan;
typedef struct ps_schedule ps_schedule;
typedef struct ps_stack ps_stack;

/* thread-local description of the last error on this thread (never NULL) */
const char *ps_last_error(void);

/* token count of tier t (t < PS_NTIERS), and the smallest tier holding n_tokens */
uint32_t ps_tier_tokens(uint32_t t);
uint32_t ps_tier_for_tokens(uint32_t n_tokens);

/* packed bytes of a [rows][K] matrix in the private device layout (host only) */
uint64_t ps_packed_bytes(uint32_t rows, uint32_t K);

/* Planning phase for one token count (Algorithm 1, PlanningPhase and
 * PinShardsToGPU; GPU-only plan).  Host only, no GPU needed.
 *  model, profile: host, copied.  expert_freq: host [n_layers*n_experts]
 *  selection frequencies used to rank experts (NULL: rank by layer, expert).
 *  *out is owned by the caller until ps_plan_destroy.
 *  PS_E_BUDGET when the budget cannot hold the workspace plus two slots. */
int32_t ps_plan_create(const ps_model_desc *model, uint64_t vram_budget_bytes,
                       const ps_profile *profile, uint32_t n_tokens,
                       const float *expert_freq, ps_plan **out);
/* The same for one of the three schedule plans of Section 3 (kind = PS_PLAN_*), or, with
 * PS_PLAN_AUTO, HeuristicSplit: all three are built and the one with the lowest estimated time
 * is returned (its summary lists the three estimates).  Plans Two and Three place the unpinned
 * parts of dense FFN matrices and of the output head, and unpinned MoE experts (whole), on the CPU
 * back-end; attention matrices and KV caches always run on the GPU.  Plan Three chooses the CPU
 * share (of each such matrix, and of the unpinned experts counted from the cold end of the priority
 * order), one value for the whole plan, that minimises the estimate.  They need a profile with
 * cpu_gbps > 0 and a host CPU the back-end supports (PS_E_STATE otherwise; PS_PLAN_AUTO then
 * returns Plan One). */
int32_t ps_plan_create_kind(const ps_model_desc *model, uint64_t vram_budget_bytes,
                            const ps_profile *profile, uint32_t n_tokens,
                            const float *expert_freq, uint32_t kind, ps_plan **out);
/* What the planning phase decided (Algorithm 1, PlanningPhase: the split of the budget into pinned
 * region and scratch, DecideScratchVRAMBudget; and Section 3, timing estimation: est_step_ms). */
int32_t ps_plan_summary(const ps_plan *plan, ps_plan_summary_t *out);
/* The schedule's shards with their residency marks (Algorithm 1: every sub-layer is added to the
 * schedule marked Residency = VRAM or SysMem), in execution (topological) order: *n of them,
 * i < *n. */
int32_t ps_plan_num_shards(const ps_plan *plan, uint32_t *n);
int32_t ps_plan_get_shard(const ps_plan *plan, uint32_t i, ps_shard_info *out);
void ps_plan_destroy(ps_plan *plan);

/* Token-tier table (Algorithm 1, the loop over tiers, and Section 3, inference phase).
 * ps_tier_table_create runs the planning phase once per tier of the set J =
 * {1, 4, 16, 32, 64, 512, 1K, 2K, 4K, 8K, 16K} under one budget: a lower tier has a smaller
 * workspace, so it pins more shards.  A tier whose workspace plus two minimum slots does not fit
 * the budget is recorded as infeasible (it is not an error).  Host only, no GPU needed.
 * Arguments as for ps_plan_create; *out is owned by the caller until ps_tier_table_destroy. */
typedef struct ps_tier_table ps_tier_table;
/* (ps_tier_table_create_kind, below, lets every tier of at most 64 tokens be planned as one of
 * the CPU plans or by HeuristicSplit, as Algorithm 1 does per tier; larger tiers keep Plan One) */
typedef struct ps_tier_entry {
    uint32_t tier;             /* index into J                                            */
    uint32_t tier_tokens;      /* tokens one trip through this tier's schedule processes  */
    int32_t feasible;          /* 0: the budget cannot hold this tier's workspace + slots */
    uint32_t pad;
    ps_plan_summary_t summary; /* valid when feasible                                     */
} ps_tier_entry;
/* PickTier: the feasible tier t minimising ceil(new_tokens / tier_tokens[t]) * est_step_ms[t];
 * among equal products the lowest tier wins.  The chosen tier's token count is also the chunk
 * size of a chunked prefill: `iterations` trips through its schedule, the last one padded. */
typedef struct ps_tier_choice {
    uint32_t tier;
    uint32_t tier_tokens;
    uint32_t iterations;       /* ceil(new_tokens / tier_tokens)                          */
    uint32_t pad;
    double est_iter_ms;        /* the tier's est_step_ms                                  */
    double est_total_ms;       /* iterations * est_iter_ms                                */
} ps_tier_choice;
int32_t ps_tier_table_create(const ps_model_desc *model, uint64_t vram_budget_bytes,
                             const ps_profile *profile, const float *expert_freq,
                             ps_tier_table **out);
int32_t ps_tier_table_create_kind(const ps_model_desc *model, uint64_t vram_budget_bytes,
                                  const ps_profile *profile, const float *expert_freq,
                                  uint32_t kind, ps_tier_table **out);
int32_t ps_tier_table_entry(const ps_tier_table *table, uint32_t tier, ps_tier_entry *out);
/* the plan of a feasible tier, owned by the table (valid until ps_tier_table_destroy);
 * ps_stack_create copies it.  PS_E_ARG for an infeasible tier. */
int32_t ps_tier_table_plan(const ps_tier_table *table, uint32_t tier, const ps_plan **out);
/* PS_E_ARG when new_tokens is 0; PS_E_BUDGET when no tier is feasible. */
int32_t ps_tier_pick(const ps_tier_table *table, uint32_t new_tokens, ps_tier_choice *out);
void ps_tier_table_destroy(ps_tier_table *table);

/* The executor's op list for one forward, as plain data (host only, no GPU).
 * router_logits: host fp32 [n_layers][n_tokens][n_experts], NULL for dense.
 * ps_schedule_validate proves with vector clocks over the two streams that no
 * kernel reads a slot before its copy completed and no copy overwrites a slot
 * before its last reader finished; returns PS_E_STATE with a text otherwise. */
int32_t ps_schedule_create(const ps_plan *plan, const float *router_logits, ps_schedule **out);
int32_t ps_schedule_num_ops(const ps_schedule *s, uint32_t *n);
int32_t ps_schedule_get_op(const ps_schedule *s, uint32_t i, ps_op_info *out);
int32_t ps_schedule_validate(const ps_schedule *s);
void ps_schedule_destroy(ps_schedule *s);

/* MoE routing on the host with the same rule as the device kernel: the top_k
 * largest fp32 logits, ties to the lower index, in descending order.
 * logits host [n_tokens][n_experts] -> idx host [n_tokens][top_k]. */
int32_t ps_route_host(const float *logits, uint32_t n_tokens, uint32_t n_experts,
                      uint32_t top_k, int32_t *idx);

/* Measure the machine profile on the current device (Section 3, install phase:
 * several asynchronous launches timed together).  scratch: device, at least
 * 256 MiB, contents destroyed.  Streams as for ps_stack_create. */
int32_t ps_profile_measure(void *scratch_dev, uint64_t scratch_bytes,
                           void *compute_stream, void *copy_stream, ps_profile *out);

/* Profile database (Section 3, profiler-based timing estimation).  One entry per benchmarked
 * kernel: operation, quantisation level (bits per weight, 0 for copies), CPU thread count (0 for
 * GPU operations), dimensions (n output rows, k reduction length, m tokens; a copy: n = bytes,
 * k = m = 1) and the measured time of one call.  ps_profile_db_estimate prices a kernel the way the
 * paper does: an entry with the same operation, quantisation, thread count and dimensions gives
 * its own time (PS_MATCH_EXACT); otherwise the entry of the same operation, quantisation and thread
 * count nearest in the space of dimensions (Euclidean in log2 n, log2 k, log2 m; the earlier entry
 * on a tie) gives the FLOPS roof of a roofline whose memory roof is bandwidth_gbps, and the kernel
 * costs flops / roof if its arithmetic intensity lies right of the ridge, bytes / bandwidth if left
 * (PS_MATCH_NEIGHBOUR; for a copy the neighbour's byte rate is used); with no such entry the kernel
 * is skipped (PS_MATCH_NONE, 0 ms).  flops = 2 n k m; bytes = n k (quant / 8 + 1 / 16) + 2 m (k + n).
 * Host only.  A database handed to ps_plan_create_db is copied. */
#define PS_OPK_GEMV 0 /* GPU dequant GEMV, one token            */
#define PS_OPK_GEMM 1 /* GPU dequant MFMA GEMM, several tokens  */
#define PS_OPK_CPU 2  /* CPU back-end matmul                    */
#define PS_OPK_H2D 3  /* pinned host -> device copy             */
#define PS_MATCH_NONE 0
#define PS_MATCH_EXACT 1
#define PS_MATCH_NEIGHBOUR 2
typedef struct ps_profile_db ps_profile_db;
typedef struct ps_prof_entry {
    uint32_t op, quant, threads, pad;
    uint64_t n, k, m;
    double ms;
} ps_prof_entry;
typedef struct ps_prof_estimate {
    double ms;             /* estimated time of one call, 0 if skipped                     */
    double flops, bytes;   /* work of the priced kernel                                    */
    uint32_t match;        /* PS_MATCH_*                                                   */
    uint32_t compute_bound;/* neighbour match: which side of the ridge                     */
    int32_t neighbour;     /* index of the entry used, -1 if none                          */
    uint32_t pad;
} ps_prof_estimate;
int32_t ps_profile_db_create(ps_profile_db **out);
void ps_profile_db_destroy(ps_profile_db *db);
/* add one entry (an entry with the same key is replaced) */
int32_t ps_profile_db_add(ps_profile_db *db, const ps_prof_entry *entry);
int32_t ps_profile_db_count(const ps_profile_db *db, uint32_t *n);
int32_t ps_profile_db_get(const ps_profile_db *db, uint32_t i, ps_prof_entry *out);
int32_t ps_profile_db_estimate(const ps_profile_db *db, double bandwidth_gbps, uint32_t op, uint32_t quant,
                               uint32_t threads, uint64_t n, uint64_t k, uint64_t m, ps_prof_estimate *out);
/* text file, one entry per line: op quant threads n k m ms */
int32_t ps_profile_db_save(const ps_profile_db *db, const char *path);
int32_t ps_profile_db_load(ps_profile_db *db, const char *path);
/* Install phase: run the benchmark suite for a model on the current device and add its entries:
 * every weight matrix of the model (QKV, O, gate/up, down or the expert pair, output head) as a
 * GEMV at one token and as a GEMM at the tiers up to 2048 tokens, each timed as ten asynchronous
 * launches together; pinned H2D copies of 1 to 64 MiB; and, where the CPU back-end is supported,
 * the FFN / expert / head matrices on it at 1, 2, 4, 8, 16 and 64 tokens (matrices under 8 MB, i.e.
 * experts, eight at a time in one pass over the worker pool, as the executor runs them; threads = the worker count
 * used, min(hardware threads, 16)).  scratch, streams: as for ps_profile_measure, scratch at least
 * 768 MiB. */
int32_t ps_profile_db_measure(ps_profile_db *db, const ps_model_desc *model, void *scratch_dev,
                              uint64_t scratch_bytes, void *compute_stream, void *copy_stream);
/* ps_plan_create_kind with shard times taken from a profile database: each shard's matmul is
 * priced by ps_profile_db_estimate (memory roof: the profile's gemv_gbps for GPU kernels, cpu_gbps
 * for the CPU back-end), copies by the H2D entries; what the database skips falls back to the
 * profile's rates.  The profile still supplies the contention factors (the ratio of its busy to
 * alone rates scales the database's CPU and copy times) and the fixed cost per CPU shard. */
int32_t ps_plan_create_db(const ps_model_desc *model, uint64_t vram_budget_bytes, const ps_profile *profile,
                          const ps_profile_db *db, uint32_t n_tokens, const float *expert_freq, uint32_t kind,
                          ps_plan **out);
/* ps_tier_table_create_kind with every tier's plan priced from a profile database as in
 * ps_plan_create_db (the paper's overview: the install-time database feeds the timing estimator
 * that fills the (token tier, best schedule) table of the planning phase).  PickTier then compares
 * tiers by times measured on the model's own matrices at each tier's token count.  The database is
 * copied. */
int32_t ps_tier_table_create_db(const ps_model_desc *model, uint64_t vram_budget_bytes,
                                const ps_profile *profile, const ps_profile_db *db,
                                const float *expert_freq, uint32_t kind, ps_tier_table **out);

/* Algorithm 1, SetupForSched: install one schedule.  Binds a plan to a VRAM arena (device, 256-byte
 * aligned, arena_bytes >= the plan's budget: the arena IS the VRAM budget of Section 3, nothing else
 * is allocated on the device) and two streams.  Allocates pinned host memory for the shards the plan
 * left in system memory.  The plan is copied; the arena and streams must outlive the stack. */
int32_t ps_stack_create(const ps_plan *plan, void *vram_arena, uint64_t arena_bytes,
                        void *compute_stream, void *copy_stream, ps_stack **out);
/* One stack for every token tier of a budget (Algorithm 1: the planning phase leaves one schedule
 * per tier; at inference PickTier chooses one, SetupForSched installs it, and the schedule runs).
 * ps_stack_create_tiers binds all feasible tiers of a table (any plan kind per tier: a table from
 * ps_tier_table_create_kind may stream everything through the GPU in its many-token tiers and leave
 * unpinned shards to the CPU in its low ones; the CPU reads the same host images) to one
 * arena of the table's budget and installs the lowest feasible tier (it pins the most).  Every
 * tier's arena is laid out [pinned shards in priority order | scratch slots | workspace], so a shard
 * that two tiers pin lies at the same place in both, and the library keeps a packed image of every
 * matrix in pinned host memory (the whole model, host side).  ps_stack_set_tier installs another
 * tier's schedule without reloading or repacking anything: shards the new tier pins and whose bytes
 * are still in place stay; those that the previous tier's larger workspace or slots overwrote are
 * copied from the host images again (*uploaded_bytes, may be NULL, receives how much).  KV caches
 * are state, not copies: a cache shard that the two tiers place differently (pinned in one, in the
 * host pool in the other) moves with the rows written so far (counted in *uploaded_bytes).  It waits
 * for both streams first; PS_E_STATE before every matrix is loaded or on a single-plan stack,
 * PS_E_ARG for an infeasible tier.  Outputs do not depend on which tiers ran before.
 * ps_stack_tier reports the installed tier and its token count (for a single-plan stack: the plan's). */
int32_t ps_stack_create_tiers(const ps_tier_table *table, void *vram_arena, uint64_t arena_bytes,
                              void *compute_stream, void *copy_stream, ps_stack **out);
int32_t ps_stack_set_tier(ps_stack *st, uint32_t tier, uint64_t *uploaded_bytes);
int32_t ps_stack_tier(const ps_stack *st, uint32_t *tier, uint32_t *n_tokens);
/* Put one logical matrix where the plan placed it (Algorithm 1, PinShardsToGPU: Residency = VRAM
 * for pinned shards, SysMem for the rest): host scales fp16 [N][K/32] and host codes u8 [N][K] are
 * packed into every shard that covers the matrix; resident slabs are copied to the arena
 * (synchronous), the others into the pinned host pool.  expert: id or 0xFFFFFFFF. */
int32_t ps_stack_load_matrix(ps_stack *st, uint32_t layer, uint32_t mat, uint32_t expert,
                             const uint16_t *scales, const uint8_t *codes);
/* KV cache (priority class "KV cache", Section 3 planning phase; only with kv_context > 0).
 * ps_stack_load_kv fills positions [0, n_pos) of one kv head of one layer from host fp16
 * K, V [n_pos][head_dim] (copied; synchronous) into that shard's home: the arena if the plan pinned
 * it, the pinned host pool otherwise.  ps_stack_set_context sets how many cached positions the next
 * forward attends over; that forward appends its tokens' K and V rows at positions context,
 * context + 1, ... of every head's home (context + tokens <= kv_context), so consecutive decode
 * steps pass context, context + 1, ... (ps_stack_forward_chunked advances the context by itself).
 * Attention (no positional encoding): the token at position p attends over positions 0 .. p -- the
 * cached ones and, in a chunk of several new tokens, the chunk's earlier tokens and itself: scores
 * q.K_j / sqrt(head_dim), softmax, weighted sum of V; query head h uses kv head h / (n_q / n_kv).
 * A streamed cache shard crosses PCIe with its `context` valid rows only. */
int32_t ps_stack_load_kv(ps_stack *st, uint32_t layer, uint32_t kv_head, const uint16_t *k_rows,
                         const uint16_t *v_rows, uint32_t n_pos);
int32_t ps_stack_set_context(ps_stack *st, uint32_t context);
/* Output head (models with vocab > 0; Section 3 planning phase lists the outputs as the last
 * priority class).  Chooses what the following ps_stack_forward calls compute after the last layer:
 *   rows == 0         nothing: the head's kernels and the copies of its streamed shards are left
 *                     out (the state after ps_stack_create; e.g. all but the last prefill chunk);
 *   rows == 1         logits of token `first_token` only (0 <= first_token < n_tokens), written to
 *                     logits_dev[0 .. vocab): fused RMSNorm + GEMV, whatever the plan's n_tokens;
 *   rows == n_tokens  logits of every token, logits_dev[n_tokens][vocab] (first_token must be 0).
 * logits = W_out * RMSNorm(x_out row), fp32 accumulation, stored fp16.  logits_dev: device memory,
 * caller-owned, 16-byte aligned, must stay valid for every forward until changed, and must not
 * overlap the arena, x_in or x_out.  PS_E_STATE if the model has no head, PS_E_ARG for any other
 * rows / first_token. */
int32_t ps_stack_set_logits_out(ps_stack *st, void *logits_dev, uint32_t first_token, uint32_t rows);
/* The CPU back-end's matrix kernel on its own (host pointers only; for tests and for measuring
 * the CPU rate): `packed` is the image ps_pack_matrix (pshard_test.h) makes of a [rows][K] matrix; x fp16 [n_tokens][K];
 * out fp16 [n_tokens][rows] (mode 2: [n_tokens][rows / 2]).  mode 0: out = W RMSNorm(x);
 * mode 1: out = W x + res (res fp16 [n_tokens][rows] or NULL); mode 2: the matrix holds gate and
 * up row-tiles alternately (16 gate rows, 16 up rows, ...) and out = SiLU(g) * u of
 * g, u = W RMSNorm(x).  fp32 accumulation, n_tokens <= 64, 1 <= threads <= 64.
 * PS_E_STATE if the CPU lacks AVX-512 / F16C. */
int32_t ps_cpu_matmul(const uint8_t *packed, uint32_t rows, uint32_t K, int32_t mode, const uint16_t *x,
                      uint32_t n_tokens, float eps, const uint16_t *res, uint16_t *out, uint32_t threads);
/* Worker threads of the CPU back-end (plans with CPU shards), 1..64; default min(hardware
 * threads, 16).  PS_E_STATE if the plan has no CPU shard. */
int32_t ps_stack_set_cpu_threads(ps_stack *st, uint32_t threads);
/* One pass over the whole stack (Algorithm 1, RunInTopologicalOrder).
 *  x_in, x_out: device fp16 [n_tokens][hidden] (n_tokens = the plan's), caller-owned, may not alias.
 *  router_logits: host fp32 [n_layers][n_tokens][n_experts] (MoE: required, the host routes with the
 *  device's rule to know which experts to copy and to build the per-expert token lists), NULL for dense.
 *  router_logits_dev: NULL, or a device copy of the same array: the routing kernel then reads it in
 *  place and nothing is uploaded (the two copies must hold the same values; the device copy must stay
 *  unchanged until the forward has completed).
 * Asynchronous: returns after enqueueing; x_out is complete when compute_stream is. */
int32_t ps_stack_forward(ps_stack *st, const void *x_in, void *x_out, const float *router_logits,
                         const float *router_logits_dev);
/* For callers that cannot allocate device memory or hand over a workspace at the time of the call:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same pass
 * as ps_stack_forward over a dense GPU-only stack without a KV cache, except that every buffer the
 * kernels use between them (activations of the sub-layers, RMS factors, split-K partial sums: the
 * plan's workspace) lies in a 32 MiB array inside the library's device image instead of the head
 * of the arena; inputs, outputs, pinned shards and scratch slots are where they always are.  The
 * call allocates nothing on the device and calls no allocating routine; one launch per shard
 * whatever the decode mode.  PS_E_ARG if the plan's workspace exceeds 33554432 bytes (e.g. 64 tokens
 * of the 8B-shaped stack need 13 MB, 2048 tokens 134 MB); PS_E_STATE for MoE / KV-cache / CPU-shard
 * stacks and while profiling is on.  Every stack on a GPU shares that GPU's array (it keeps the last
 * call's contents; nothing in it needs clearing, every buffer is written before it is read): two
 * such forwards that overlap in time on one GPU race.  Bit-identical to ps_stack_forward. */
int32_t ps_stack_forward_noalloc(ps_stack *st, const void *x_in, void *x_out);
/* Chunked prefill (Section 3, inference phase: the picked tier's size is the chunk size): n_tokens
 * rows go through the plan's schedule in ceil(n_tokens / T) trips of T = the plan's token count.  A
 * last chunk shorter than T runs the same schedule with the same launch shapes over its rows only
 * (a row's result does not depend on how many rows share its trip; rows past the end are neither
 * read nor written), so each trip costs at most what the tier's estimate prices.
 *  x_in, x_out: device fp16 [n_tokens][hidden].  router_logits / router_logits_dev: as for
 *  ps_stack_forward with [n_layers][n_tokens][n_experts].  last_logits_dev: NULL, or device fp16
 *  [vocab], 16-byte aligned: the output head runs on the last trip only, for the prompt's last token
 *  (its copies and kernels are left out of the other trips); the setting of ps_stack_set_logits_out
 *  is not used and is left as it was.  *trips (may be NULL) receives the number of trips.
 *  With a KV cache every trip attends over the cache and the rows the earlier trips appended, starting
 *  at the context set by ps_stack_set_context; afterwards the context stands at that value + n_tokens
 *  (PS_E_ARG if that exceeds kv_context), so decode steps can follow without setting it.
 *  Asynchronous like ps_stack_forward. */
int32_t ps_stack_forward_chunked(ps_stack *st, const void *x_in, void *x_out, uint32_t n_tokens,
                                 const float *router_logits, const float *router_logits_dev,
                                 void *last_logits_dev, uint32_t *trips);
/* Decode execution mode.  0 (default): one launch per shard.  1: applies when the plan is dense with
 * every shard (KV-cache shards included) resident and no CPU share, for one token or, without a KV
 * cache, for a batched-decode step of up to 64 tokens (otherwise mode 0 runs): the launch-per-shard
 * kernel sequence is captured once per (x_in, x_out, logits, valid rows) into a HIP graph (kernel
 * nodes only) and replayed; with a KV cache the context length then travels in a
 * device word set before each replay, and the attention launch covers every chunk the cache can
 * hold (workgroups past the context leave at once).  Order and arithmetic are unchanged
 * (Algorithm 1's RunInTopologicalOrder); both modes give bit-identical results.  (A third value
 * exists for tests only, see pshard_test.h.)  Not to be called while a forward is in flight. */
int32_t ps_stack_set_decode_mode(ps_stack *st, int32_t mode);
/* How streamed shards cross PCIe (Section 3: the copy of the next shard runs beside the compute of
 * the current one).  gather = 1 (default): the streamed experts of one slot fill are pulled from
 * the pinned pool by one kernel on the copy stream (one launch per slot fill), and so are the
 * dense slabs of a plan whose step is copy time almost alone (copy estimate at least ten times the
 * kernel estimate, from the plan's profile: the kernel keeps the link busier than back-to-back
 * hipMemcpyAsync calls but slows kernels that run beside it); other dense slabs and all KV rows
 * use hipMemcpyAsync.  In this mode, in one-token steps, an expert fill that is its layer's only one
 * is launched on the compute stream, between the router and the experts that wait for it (two
 * cross-stream hand-overs per layer are saved, which at one token outweigh running the resident
 * experts beside the copy); modes 0 and 2 keep every copy on the copy stream.  gather = 0: hipMemcpyAsync for everything, one per expert.  gather = 2:
 * the kernel for every expert and dense slab.  The bytes that arrive are the same in every mode.
 * PS_E_ARG for another value.  Not to be called while a forward is in flight. */
int32_t ps_stack_set_copy_mode(ps_stack *st, int32_t gather);
/* Block until both streams are idle, i.e. until the schedule's last shard has run (Algorithm 1,
 * RunInTopologicalOrder, seen from the caller); PS_E_HIP if either stream reports an error. */
int32_t ps_stack_sync_check(ps_stack *st);
/* record per-op timing events in the next forwards (adds event overhead) */
int32_t ps_stack_set_profiling(ps_stack *st, int32_t on);
/* Counters of the last forward: bytes read in place, bytes copied H2D, bytes read by the CPU, and,
 * with profiling on, copy time, compute time and their overlap -- the quantities Section 3's timing
 * estimation models (a shard's time is the larger of its compute and the concurrent PCIe copy), so
 * that an estimate can be set beside a measurement.  Blocks until both streams are idle when
 * profiling is on. */
int32_t ps_stack_stats(ps_stack *st, ps_stats *out);
/* start (relative to the first op) and duration in ms of op i of the last profiled forward;
 * ops are numbered as in the schedule of the same plan.  Blocks like ps_stack_stats. */
int32_t ps_stack_op_time(ps_stack *st, uint32_t i, double *start_ms, double *dur_ms);
void ps_stack_destroy(ps_stack *st);

#ifdef __cplusplus
}
#endif
#endif /* PSHARD_H */
