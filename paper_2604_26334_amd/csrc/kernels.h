// Launch interface between the executor (stack.hip) and the device kernels (kernels.hip).
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "ps_internal.h"

namespace ps {

enum { GEMV_PLAIN = 0, GEMV_RESID = 1, GEMV_GATE_UP = 2, GEMV_F32 = 3 };
enum { GEMM_PLAIN = 0, GEMM_RESID = 1, GEMM_GATE_UP = 2, GEMM_F32 = 3 };

// One token.  PLAIN: out = rinv * (W x) with rinv from x's RMS; RESID: out = res + W x;
// GATE_UP: out = silu(rinv * gate) * (rinv * up); F32: out_f32 = W x.
struct GemvArgs {
    const uint4 *W;       // first tile of the slab (ignored when tasks != null)
    uint32_t nunits;      // row-tiles (GATE_UP: tile pairs) in this launch
    uint32_t tile_u4;     // tile stride in 16-byte units
    uint32_t nsb, ngroups, K;
    const __half *x;      // input row
    uint32_t x_off, x_group;   // input column map (identity: 0, 1)
    uint32_t x_stride;    // grouped launches: elements between input rows
    float eps;
    const __half *res;    // RESID: residual row or null
    __half *out;
    float *out_f32;
    uint32_t out_row0;    // first output element of the slab
    uint32_t out_stride;  // grouped launches: elements between output rows
    uint32_t top_k;
    const DeviceTask *tasks;  // grouped (MoE) launch: one expert per blockIdx.y
    const int32_t *pairs;
};

// M tokens on the matrix cores.  Same modes; rinv comes from a buffer.
struct GemmArgs {
    const uint4 *W;
    uint32_t ntiles;      // row-tiles in this launch
    uint32_t total_tiles; // row-tiles of the whole matrix (picks the tile shape)
    uint32_t tile_u4, nsb;
    uint32_t M;
    const __half *x;
    uint32_t x_stride, x_off, x_group;
    const float *rinv;
    const __half *res;
    __half *out;
    float *out_f32;
    uint32_t out_stride, out_row0, top_k;
    uint32_t sb_per_part;  // split-K: super-blocks per blockIdx.z part (0 = whole K in one part)
    uint32_t part_stride;  // split-K: elements between the fp32 partial planes
    const DeviceTask *tasks;
    const int32_t *pairs;
};

// one host->device copy of a gathered batch: n16 16-byte units from pinned host memory to VRAM
struct CopyDesc {
    uint64_t src, dst;
    uint32_t n16, pad0, pad1, pad2;
};
// one launch copies `n` shards (descs may live in pinned host memory): the GPU pulls them over
// PCIe itself, which avoids the per-call cost of many small hipMemcpyAsync
hipError_t launch_h2d_gather(const CopyDesc *descs, uint32_t n, hipStream_t st);

uint32_t gemv_ksplit(uint32_t ngroups, uint32_t total_units);
hipError_t launch_gemv(int mode, uint32_t ksplit, const GemvArgs &a, uint32_t ntasks, hipStream_t st);
hipError_t launch_gemm(int mode, const GemmArgs &a, uint32_t ntasks, uint32_t max_tok, hipStream_t st);
// Two to kGemvMtTokens tokens of a dense sub-layer whose K is a multiple of 1024 (rows of x x_stride
// elements apart, rows of out and res out_stride apart): the one-token kernel's launch shape with the dot
// products on the matrix cores; PLAIN, RESID and GATE_UP, the RMS factors computed from the activations
constexpr int kGemvMtTokens = 4;
hipError_t launch_gemv_mt(int mode, uint32_t ksplit, const GemvArgs &a, uint32_t ntok, hipStream_t st);
// sums `parts` fp32 partial planes [M][ncols_phys] in ascending order and applies the mode's epilogue
hipError_t launch_splitk_epilogue(int mode, const float *partial, uint32_t parts, uint32_t part_stride, uint32_t M,
                                  uint32_t ncols_phys, const float *rinv, const __half *res, __half *out,
                                  uint32_t out_stride, uint32_t out_row0, hipStream_t st);
hipError_t launch_rinv(const __half *x, uint32_t M, uint32_t H, float eps, float *rinv, hipStream_t st);
// residual epilogue over whole rows of the hidden state (ncols == out_stride == H, first column 0,
// at most 8 planes) that also writes the RMS factor of each row it stores, bit-identical to
// launch_splitk_epilogue(GEMM_RESID, ...) followed by launch_rinv(out, ...)
hipError_t launch_splitk_epilogue_resid_rinv(const float *partial, uint32_t parts, uint32_t part_stride, uint32_t M,
                                             uint32_t H, const __half *res, __half *out, float eps, float *rinv,
                                             hipStream_t st);
hipError_t launch_route(const float *logits, uint32_t M, uint32_t E, uint32_t top_k, int32_t *idx, float *w,
                        hipStream_t st);
// Decode attention over a KV cache, one new token.  A cache shard of one kv head is K rows
// [cap][128] followed by V rows [cap][128], fp16; `nheads` shards lie head_stride bytes apart from
// kv (kv heads head0 .. head0 + nheads - 1).  Each workgroup covers one kv head x one chunk of 256
// cached positions for the head's `group` query heads and writes, per query head and chunk, the
// chunk's score maximum, sum of weights and 128 weighted value sums (fp32) to
// part[(q_head * chunk_cap + chunk) * 130].  ctx = cached positions (nothing is launched for 0).
struct AttnArgs {
    const __half *kv;
    uint64_t head_stride;
    uint32_t cap, ctx, head0, nheads, group, chunk_cap;
    const __half *q;      // the token's QKV row: query head h at [h * 128]
    float *part;
    const uint32_t *ctx_dev;   // not null: the context length is read from here (device) instead of ctx, and
                               // the launch covers every chunk the cache can hold (a captured graph is
                               // replayed at any context); workgroups past the context leave at once
};
// Attention of a chunk of `ntok` new tokens (rows of q, q_stride elements apart) over one kind of rows:
//  causal == 0: the cache shards of kv heads head0 .. head0 + nheads - 1 (k_base = first shard; shards
//   head_stride bytes apart, K rows [cap][128] then V rows; row_stride = 128); every token sees the ctx
//   cached positions;
//  causal == 1: the chunk's own K / V rows, read in place from the tokens' QKV rows (k_base / v_base =
//   kv head 0 of token 0, row_stride = the QKV row width; head0 .. as above): token t sees rows 0 .. t.
// Partials go to part[((t * n_q + q_head) * chunk_cap + chunk0 + chunk) * 130] (maximum, weight sum, 128 sums).
struct AttnChunkArgs {
    const __half *k_base, *v_base;
    uint64_t head_stride;
    uint32_t cap, ctx, head0, nheads, group, n_q;
    uint32_t row_stride, causal, ntok, q_stride, chunk0, chunk_cap;
    uint32_t tok_per_wg;   // set by the launch: tokens one workgroup serves
    // the one-pass form only (launch_attn_chunk_onepass): it walks the cache shards at k_base (row_stride 128,
    // ctx positions) AND the chunk's own rows in one launch, and writes finished attention rows
    const __half *k_own, *v_own;   // kv head 0 of token 0 in the QKV rows
    uint32_t own_stride;           // elements between two tokens' QKV rows
    __half *out;                   // attention rows [ntok][n_q * 128], out_stride elements apart
    uint32_t out_stride;
    const __half *q;
    float *part;
};
hipError_t launch_attn_chunk(const AttnChunkArgs &a, hipStream_t st);
// Chunks of many tokens: one launch per run of cache shards walks the cached positions and then the chunk's own
// rows with running softmax statistics and writes out[t][q_head * 128 ..] directly (no partial records)
hipError_t launch_attn_chunk_onepass(const AttnChunkArgs &a, hipStream_t st);
// appends ntok tokens' K / V rows (from their QKV rows) at positions ctx .. of every kv head's cache home
hipError_t launch_kv_append_rows(uint32_t ctx, uint32_t cap, const __half *qkv, uint32_t qkv_w, uint32_t n_q, uint32_t n_kv, uint32_t ntok,
                                 const uint64_t *home, hipStream_t st);
// merges every token's chunks (cache chunks below ctx, then the chunk's own) in ascending order, writes the
// attention rows out[t][n_q * 128] (out_stride elements apart) and appends the tokens' K / V rows at
// positions ctx .. ctx + ntok - 1 of each kv head's cache home
hipError_t launch_attn_combine_chunk(const float *part, uint32_t chunk_cap, uint32_t ctx, uint32_t cap, const __half *qkv,
                                     uint32_t qkv_w, uint32_t n_q, uint32_t n_kv, uint32_t ntok, const uint64_t *home, __half *out,
                                     uint32_t out_stride, hipStream_t st);
// *dst = v (device word), in stream order
hipError_t launch_set_u32(uint32_t *dst, uint32_t v, hipStream_t st);
// dst[idx[r]][0..H) = src[r][0..H) for r < n (fp32 rows; H a multiple of 4; idx values are row numbers of dst)
hipError_t launch_scatter_rows(const float *src, const int32_t *idx, uint32_t n, uint32_t H, float *dst, hipStream_t st);
hipError_t launch_attn_decode(const AttnArgs &a, hipStream_t st);
// Merge the chunks of every query head in ascending order with the token's own position (score
// q.k_new / sqrt(128), value v_new), write the attention output (fp16 [n_q * 128]) and append the
// token's K and V rows at position ctx of each kv head's cache home (home[g] = address of that
// head's K row 0, device memory or device-visible pinned host memory).
hipError_t launch_attn_combine(const float *part, uint32_t chunk_cap, uint32_t ctx, const uint32_t *ctx_dev, uint32_t cap,
                               const __half *qkv, uint32_t n_q, uint32_t n_kv, const uint64_t *home, __half *out, hipStream_t st);
hipError_t launch_combine(const __half *h, const float *y, const float *w, uint32_t M, uint32_t H, uint32_t top_k,
                          int residual, __half *out, hipStream_t st);
hipError_t launch_mfma_probe(int pi, int pk, int pj, float *out, hipStream_t st);
hipError_t launch_lds_tr_probe(const uint32_t *addr, uint16_t *out, hipStream_t st);

}  // namespace ps
