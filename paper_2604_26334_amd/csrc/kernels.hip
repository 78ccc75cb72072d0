// CDNA4 (gfx950) kernels of the pipelined-sharding hot path: the dequantising matmuls of
// the decoder sub-layers with their fused RMSNorm / SwiGLU / residual steps, MoE routing and
// the expert combine, and attention over the KV cache.  Weight layout: see pack.cpp.  wave64 only.
//   matmuls by token count:  1 -> gemv_w4_kernel,  2..4 -> gemv_mt_kernel (whole scale groups),
//                            otherwise gemm_w4_kernel (+ splitk_epilogue* when K is split)
//   attention:  one query token -> attn_decode_kernel + attn_combine_kernel,
//               a long chunk of query tokens -> attn_chunk_onepass_kernel (one walk over the cache and
//               the chunk's own rows);  a short chunk -> attn_chunk_mfma_kernel over 256-position
//               pieces of the cache (attn_chunk_kernel when there are fewer than 16 score rows), the
//               pieces merged by attn_combine_chunk_kernel
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>
#include <cstdlib>

#include "kernels.h"

namespace ps {

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef float f4_t __attribute__((ext_vector_type(4)));

typedef uint32_t u4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ h2_t as_h2(uint32_t v) { return __builtin_bit_cast(h2_t, v); }

// streaming 16-byte load: weights are read once per step, keep them out of the way of the caches
__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
    const u4_t v = __builtin_nontemporal_load(reinterpret_cast<const u4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// 8 codes of one dword -> four fp16 pairs holding (q - 8), exact.  Codes sit in the
// mantissa of 1024 + q (low nibbles) or 1024 + 16 q (next nibbles).
// (v & mask) | magic in one VALU op: the mask rides the scalar operand slot, the magic a VGPR
__device__ __forceinline__ uint32_t and_or(uint32_t v, uint32_t mask, uint32_t magic) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "s"(mask), "v"(magic));
    return r;
}

__device__ __forceinline__ void dequant8(uint32_t v, h2_t w[4]) {
    const h2_t k1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
    const h2_t k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const h2_t k72 = {(_Float16)72.0f, (_Float16)72.0f};
    const uint32_t v8 = v >> 8;
    w[0] = as_h2(and_or(v, 0x000F000Fu, 0x64006400u)) - k1032;
    w[1] = __builtin_elementwise_fma(as_h2(and_or(v, 0x00F000F0u, 0x64006400u)), k16th, -k72);
    w[2] = as_h2(and_or(v8, 0x000F000Fu, 0x64006400u)) - k1032;
    w[3] = __builtin_elementwise_fma(as_h2(and_or(v8, 0x00F000F0u, 0x64006400u)), k16th, -k72);
}

// Decode dot product of 8 codes with 8 activations WITHOUT removing the code offsets: the fp16
// patterns 1024 + q (codes 0, 1, 4, 5 of the dword) and 1024 + 16 q (codes 2, 3, 6, 7) go straight
// into the fp32 dot-product accumulators lo / hi.  With S_lo, S_hi the sums of the activations at
// those positions, sum((q - 8) x) = lo + hi / 16 - 1032 S_lo - 72 S_hi; the two S terms depend on
// the activations only and are shared by every row (see gemv_item).  Saves the four packed
// subtract / multiply-add operations per dword; the fp32 accumulators carry terms near 1024 |x|,
// which costs about 1e-4 of a block's sum in relative accuracy.
__device__ __forceinline__ void dot8_raw(uint32_t v, uint4 x, float &lo, float &hi) {
    const uint32_t v8 = v >> 8;
    lo = __builtin_amdgcn_fdot2(as_h2(and_or(v, 0x000F000Fu, 0x64006400u)), as_h2(x.x), lo, false);
    hi = __builtin_amdgcn_fdot2(as_h2(and_or(v, 0x00F000F0u, 0x64006400u)), as_h2(x.y), hi, false);
    lo = __builtin_amdgcn_fdot2(as_h2(and_or(v8, 0x000F000Fu, 0x64006400u)), as_h2(x.z), lo, false);
    hi = __builtin_amdgcn_fdot2(as_h2(and_or(v8, 0x00F000F0u, 0x64006400u)), as_h2(x.w), hi, false);
}

__device__ __forceinline__ float half_of(uint4 v, int s) {  // s-th fp16 of a 16-byte vector
    const uint32_t d = (s < 2) ? v.x : (s < 4) ? v.y : (s < 6) ? v.z : v.w;
    const uint16_t h = (s & 1) ? (uint16_t)(d >> 16) : (uint16_t)(d & 0xFFFFu);
    return (float)__builtin_bit_cast(_Float16, h);
}

__device__ __forceinline__ float sumsq8(uint4 v) {
    float s = 0.f;
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const h2_t p = as_h2(d[i]);
        s += (float)p.x * (float)p.x;
        s += (float)p.y * (float)p.y;
    }
    return s;
}

// sum over the wave, the same value in every lane: the 16 lanes of a row meet through DPP row
// operations, the four rows through four lane reads (no LDS permutes, whose six dependent round
// trips cost a wave several hundred cycles)
__device__ __forceinline__ float wave_sum(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false));   // quad_perm 1,0,3,2
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, false));   // quad_perm 2,3,0,1
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, false));  // row_half_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, false));  // row_mirror
    const int b = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0)), r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32)), r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return (r0 + r1) + (r2 + r3);
}

// Lanes l, l ^ 16, l ^ 32, l ^ 48 (one column of the wave's four rows) meet, the result in all four:
// (row 0 + row 1) + (row 2 + row 3), by the row-swap instructions of gfx950 (vector ALU, no LDS
// permute).  v_permlane16_swap exchanges the odd rows of its first operand with the even rows of its
// second, v_permlane32_swap the upper half of the first with the lower half of the second; with both
// operands the same value, the two results are the two partners of every lane (lane layout checked
// on the hardware with lane numbers as data).
template <bool MAX = false>
__device__ __forceinline__ float rows4_meet(float v) {
#if defined(__HIP_DEVICE_COMPILE__)
    // written as instructions: the two operands are exchanged in place, so they are two registers
    // holding the same value (this compiler's builtin for the swap loses its second result when
    // the two results are combined, checked on the hardware); s_nop covers the write-to-swap
    // hazard the compiler would otherwise pad
    float a = v, b = v;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    float y = MAX ? fmaxf(a, b) : a + b, z = y;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(y), "+v"(z));
    return MAX ? fmaxf(y, z) : y + z;
#else
    return v;
#endif
}

// fp32 -> fp16 with the rounding kept as its own step: the value passes through an opaque
// register so the compiler cannot merge the producing multiply/add into a mixed-precision
// convert in one kernel and not in another (the decode paths must agree bit for bit)
__device__ __forceinline__ __half to_half(float v) {
    asm volatile("" : "+v"(v));
    return __float2half(v);
}

__device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }

// raw buffer descriptor over the whole 32-bit offset range from `base` (offsets are validated on the
// host); loads through it take a 32-bit lane offset plus a scalar offset
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)0xFFFFFFFFu, 0x00020000);
}
typedef __attribute__((address_space(3))) void lds_void;
// 16 bytes per lane from global memory straight into LDS: lane l of the wave lands at dst + 16 l
// (dst is wave-uniform), without passing through registers.  The host pass has no such builtin and
// only needs the kernel's signature.
__device__ __forceinline__ void load_to_lds16(__amdgpu_buffer_rsrc_t rsrc, lds_void *dst, uint32_t voff, uint32_t soff) {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst, 16, voff, soff, 0, 0);
#endif
}
constexpr int kAuxNt = 2;   // non-temporal: streamed weights are not worth keeping in cache

// source column of logical input column k: identity, or the identity-on-V attention
// stand-in where query head h reads kv head h / group (head_dim 128)
__device__ __forceinline__ uint32_t gather_col(uint32_t k, uint32_t x_off, uint32_t group) {
    return x_off + ((k >> 7) / group) * 128u + (k & 127u);
}

// ------------------------------------------------------------------------------------
// Decode kernel, one token: fused 4-bit dequant GEMV.  A "unit" is one row-tile (16 outputs)
// or, for GATE_UP, a gate tile plus its up tile.  KSPLIT waves share a unit, wave kpart taking
// scale groups kpart, kpart + KSPLIT, ... of K; a workgroup holds NW / KSPLIT units.
// Each wave first issues all weight loads of its group (they do not depend on the
// activations), then fetches only the 1024 activations of that group and spreads them to its
// lanes through a wave-private LDS window (LDS operations of one wave execute in order, so no
// barrier is needed).  The RMSNorm sum of squares is accumulated from the same fetch.
// Partial sums of the KSPLIT waves meet in LDS in a fixed order behind the only barrier, so
// a row's result does not depend on which slab or slot it came from.
// ------------------------------------------------------------------------------------
template <int NT>
struct GemvBuf {
    uint4 sc[NT];
    uint4 wq[NT][8];
    uint4 xa, xb;
};

// weights of scale group g of a unit's NT tiles (independent of the activations).  unit, g and
// nsb_g are the same for the whole wave, so their share of the address is kept in scalar registers
// and the loads take (descriptor, lane offset, scalar offset): no per-lane address arithmetic.
template <int NT, bool FULLG = false>
__device__ __forceinline__ void gemv_issue_w(GemvBuf<NT> &b, const uint4 *W, uint32_t unit, uint32_t tile_u4,
                                             uint32_t g, uint32_t nsb_g, int lane) {
    const __amdgpu_buffer_rsrc_t wb = make_rsrc(W);
    const uint32_t tile_b = tile_u4 * 16u;
    const uint32_t base = __builtin_amdgcn_readfirstlane(unit * NT * tile_b + g * (9u * 1024u));
    // FULLG: every scale group has its 8 super-blocks, so the number of loads in flight is a
    // compile-time fact and the compiler can wait for exactly the load a dot product needs
    const uint32_t nsb_u = FULLG ? 8u : __builtin_amdgcn_readfirstlane(nsb_g);
    const uint32_t voff = (uint32_t)lane * 16u;
    // issue order = consumption order (loads return in order): scales, then super-block by
    // super-block across the tiles, so the dot products of a super-block can start while the later
    // ones are still in flight
#pragma unroll
    for (int t = 0; t < NT; ++t)
        b.sc[t] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(wb, voff, base + t * tile_b + nsb_u * 1024u, kAuxNt));
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if (FULLG || (uint32_t)s < nsb_u) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
                b.wq[t][s] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(wb, voff, base + t * tile_b + s * 1024u, kAuxNt));
        }
    }
}

// activations of scale group g: 128 chunks of 8, lane takes chunks lane and lane + 64
template <int NT>
__device__ __forceinline__ void gemv_issue_x(GemvBuf<NT> &b, uint32_t g, uint32_t K, const __half *x,
                                             uint32_t x_off, uint32_t x_group, int lane) {
    const uint32_t k0 = g * 1024u + (uint32_t)lane * 8u, k1 = k0 + 512u;
    b.xa = make_uint4(0, 0, 0, 0);
    b.xb = make_uint4(0, 0, 0, 0);
    if (k0 < K) b.xa = *reinterpret_cast<const uint4 *>(x + gather_col(k0, x_off, x_group));
    if (k1 < K) b.xb = *reinterpret_cast<const uint4 *>(x + gather_col(k1, x_off, x_group));
}

// chunk q (0..127) of a group -> slot in the wave's LDS window: block b = q / 4, part p = q % 4,
// super-block sb = b / 4, c = b % 4; the four lanes groups c read distinct banks for a given p
__device__ __forceinline__ uint32_t xslot(uint32_t q) {
    const uint32_t b = q >> 2, p = q & 3u;
    return (b >> 2) * 16u + p * 4u + (b & 3u);
}

// LDS of one decode workgroup of NW waves: a 2 KB activation window per wave and the reduction
// scratch.  The scratch holds one
// partial sum per (unit, scale group): a row's result is the sum of its scale-group partials in
// ascending group order, whichever wave produced which partial -- so it depends neither on the
// K split nor on the workgroup shape, let alone on the slab or slot the weights came from.
constexpr int kMaxGroups = 16;   // K <= 16384
template <int NW>
struct GemvLds {
    uint4 x[NW][128];
    float red[(NW / 2) * kMaxGroups][2][16];   // K split >= 2: at most NW / 2 units per workgroup
    float red_ss[(NW / 2) * kMaxGroups];
    float corr[NW][32];   // per wave: code-offset corrections of the current scale group
};

// One work item of the decode GEMV: the NW waves of the workgroup cover NW / ks units, ks
// waves per unit.
// DBUF: a wave with several scale groups issues the next group's loads before computing the
// current one (costs a second register buffer; the one-tile modes can afford it).
template <int MODE, int NW, bool DBUF = false, bool FULLG = false>
__device__ __forceinline__ void gemv_item(const GemvArgs &a, const uint4 *W, const __half *x, __half *out,
                                          float *out_f32, uint32_t item, uint32_t ks, GemvLds<NW> &lds) {
    constexpr int NT = (MODE == GEMV_GATE_UP) ? 2 : 1;
    constexpr bool NORM = (MODE == GEMV_PLAIN || MODE == GEMV_GATE_UP);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, c = lane >> 4;
    const uint32_t units = NW / ks;
    const uint32_t unit = item * units + wave / ks;
    const uint32_t kpart = wave % ks;
    const bool active = unit < a.nunits;
    float acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = 0.f;
    float ss = 0.f;
    uint4 *win = lds.x[wave];
    const uint32_t row = a.out_row0 + unit * 16 + i;
    float resv = 0.f;   // residual of this lane's output row, fetched early (it only waits on the previous phase)
    const bool writer = active && kpart == 0 && c == 0;

    if (active && kpart < a.ngroups) {
        GemvBuf<NT> cur, nxt;
        uint32_t g = kpart;
        // activations first: they are ready (and cached), and nothing can be computed before them
        gemv_issue_x<NT>(cur, g, a.K, x, a.x_off, a.x_group, lane);
        gemv_issue_w<NT, FULLG>(cur, W, unit, a.tile_u4, g, min(8u, a.nsb - g * 8u), lane);
        if (MODE == GEMV_RESID && writer && a.res) resv = __half2float(a.res[row]);
        while (true) {
            const uint32_t nsb_g = FULLG ? 8u : min(8u, a.nsb - g * 8u);
            const uint32_t gn = g + ks;
            const bool more = gn < a.ngroups;
            if (DBUF && more) {
                gemv_issue_x<NT>(nxt, gn, a.K, x, a.x_off, a.x_group, lane);
                gemv_issue_w<NT, FULLG>(nxt, W, unit, a.tile_u4, gn, min(8u, a.nsb - gn * 8u), lane);
            }
            win[xslot(lane)] = cur.xa;
            win[xslot(lane + 64)] = cur.xb;
            // code-offset corrections (see dot8_raw): lane (c, i) sums the activations of super-block
            // i % 8, lane group c, that meet low-pattern and high-pattern codes; 1032 S_lo + 72 S_hi
            // goes through LDS and each lane picks up the term of its c per super-block
            {
                const uint32_t *wp = reinterpret_cast<const uint32_t *>(win) + ((i & 7) * 16 + c) * 4;
                const h2_t one = {(_Float16)1.0f, (_Float16)1.0f};
                float sl = 0.f, sh = 0.f;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const uint4 xq = *reinterpret_cast<const uint4 *>(wp + p * 16);
                    sl = __builtin_amdgcn_fdot2(as_h2(xq.x), one, sl, false);
                    sh = __builtin_amdgcn_fdot2(as_h2(xq.y), one, sh, false);
                    sl = __builtin_amdgcn_fdot2(as_h2(xq.z), one, sl, false);
                    sh = __builtin_amdgcn_fdot2(as_h2(xq.w), one, sh, false);
                }
                if (i < 8) lds.corr[wave][c * 8 + i] = fmaf(72.0f, sh, 1032.0f * sl);
            }
            const float *corr = &lds.corr[wave][c * 8];
            float gacc[NT];   // this scale group's partial sums
#pragma unroll
            for (int t = 0; t < NT; ++t) gacc[t] = 0.f;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                if (FULLG || (uint32_t)s < nsb_g) {
                    uint4 xv[4];
#pragma unroll
                    for (int p = 0; p < 4; ++p) xv[p] = win[s * 16 + p * 4 + c];
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        float lo = 0.f, hi = 0.f;
                        dot8_raw(cur.wq[t][s].x, xv[0], lo, hi);
                        dot8_raw(cur.wq[t][s].y, xv[1], lo, hi);
                        dot8_raw(cur.wq[t][s].z, xv[2], lo, hi);
                        dot8_raw(cur.wq[t][s].w, xv[3], lo, hi);
                        const float part = fmaf(hi, 0.0625f, lo) - corr[s];
                        gacc[t] = fmaf(half_of(cur.sc[t], s), part, gacc[t]);
                    }
                }
            }
            // the 4 lanes of a row (c = 0..3) meet; then the group partial joins the others in group order
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                gacc[t] = rows4_meet<false>(gacc[t]);
            }
            float gss = 0.f;
            if (NORM) gss = wave_sum(sumsq8(cur.xa) + sumsq8(cur.xb));
            if (ks == 1) {   // this wave sees the groups in ascending order: add as it goes
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[t] += gacc[t];
                ss += gss;
            } else {
                const uint32_t slot = (wave / ks) * kMaxGroups + g;
                if (c == 0) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) lds.red[slot][t][i] = gacc[t];
                }
                if (NORM && lane == 0) lds.red_ss[slot] = gss;
            }
            if (!more) break;
            if (DBUF) {
                cur = nxt;
            } else {
                gemv_issue_x<NT>(cur, gn, a.K, x, a.x_off, a.x_group, lane);
                gemv_issue_w<NT, FULLG>(cur, W, unit, a.tile_u4, gn, min(8u, a.nsb - gn * 8u), lane);
            }
            g = gn;
        }
    }
    if (ks > 1) {
        __syncthreads();
        if (writer) {
            const uint32_t slot0 = (wave / ks) * kMaxGroups;
            for (uint32_t g = 0; g < a.ngroups; ++g) {
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[t] += lds.red[slot0 + g][t][i];
                if (NORM) ss += lds.red_ss[slot0 + g];
            }
        }
    }
    if (!writer) return;
    const float rinv = NORM ? rsqrtf(ss / (float)a.K + a.eps) : 1.f;
    if (MODE == GEMV_F32) {
        out_f32[row] = acc[0];
        return;
    }
    float v;
    if (MODE == GEMV_PLAIN) v = rinv * acc[0];
    else if (MODE == GEMV_RESID) v = resv + acc[0];
    else v = silu(rinv * acc[0]) * (rinv * acc[NT - 1]);
    out[row] = to_half(v);
}

template <int MODE, int NW, bool FULLG>
__global__ __launch_bounds__(NW * 64, 4) void gemv_w4_kernel(GemvArgs a, uint32_t ks) {   // 4 waves per SIMD: at most 128 VGPRs
    __shared__ GemvLds<NW> lds;
    const uint4 *W = a.W;
    const __half *x = a.x;
    __half *out = a.out;
    float *out_f32 = a.out_f32;
    if (a.tasks) {  // grouped launch: blockIdx.y selects the expert
        const DeviceTask t = a.tasks[blockIdx.y];
        const uint32_t pair = (uint32_t)a.pairs[t.pair0];
        if (MODE == GEMV_GATE_UP) {
            W = reinterpret_cast<const uint4 *>(t.w_gate_up);
            x = a.x + (size_t)(pair / a.top_k) * a.x_stride;
            out = a.out + (size_t)pair * a.out_stride;
        } else {
            W = reinterpret_cast<const uint4 *>(t.w_down);
            x = a.x + (size_t)pair * a.x_stride;
            out_f32 = a.out_f32 + (size_t)pair * a.out_stride;
        }
    }
    // second register buffer for the one-tile modes (the residual mode with ragged scale groups would
    // spill a register with it)
    constexpr bool DBUF = (MODE == GEMV_F32 || (MODE == GEMV_RESID && FULLG)) && NW < 16;
    gemv_item<MODE, NW, DBUF, FULLG>(a, W, x, out, out_f32, blockIdx.x, ks, lds);
}

template <int MODE, bool FULLG>
static hipError_t launch_gemv_f(const GemvArgs &a, uint32_t ks, uint32_t ntasks, hipStream_t st) {
    // waves per workgroup: at least the K split; two units per workgroup (8 waves) when that still
    // leaves about one workgroup per CU -- fewer, larger workgroups start sooner (measured on the
    // 8B shapes: QKV 6.6 -> 5.4 us, gate/up 13.4 -> 13.0 us; O, with 256 units, is best left at one
    // unit per workgroup).  The result does not depend on the shape.
    uint32_t nw = ks > 8 ? 16 : ks > 4 ? 8 : 4;
    if (ks == 4 && (a.nunits + 1) / 2 >= 192) nw = 8;   // (with one wave per unit, ks < 4, the larger workgroup measured slower)
    const uint32_t units = nw / ks;
    dim3 grid((a.nunits + units - 1) / units, ntasks ? ntasks : 1);
    if (nw == 16) hipLaunchKernelGGL((gemv_w4_kernel<MODE, 16, FULLG>), grid, dim3(1024), 0, st, a, ks);
    else if (nw == 8) hipLaunchKernelGGL((gemv_w4_kernel<MODE, 8, FULLG>), grid, dim3(512), 0, st, a, ks);
    else hipLaunchKernelGGL((gemv_w4_kernel<MODE, 4, FULLG>), grid, dim3(256), 0, st, a, ks);
    return hipGetLastError();
}

template <int MODE>
static hipError_t launch_gemv_t(const GemvArgs &a, uint32_t ks, uint32_t ntasks, hipStream_t st) {
    return (a.nsb % 8 == 0) ? launch_gemv_f<MODE, true>(a, ks, ntasks, st) : launch_gemv_f<MODE, false>(a, ks, ntasks, st);
}

// The K split is a pure performance choice (results do not depend on it): it grows until the
// launch has about four waves per SIMD or every wave is down to one scale group.
uint32_t gemv_ksplit(uint32_t ngroups, uint32_t total_units) {
    uint32_t ks = 1;
    while (ks < 16 && ks < ngroups && total_units * ks < 4096) ks *= 2;
    return ks;
}

hipError_t launch_gemv(int mode, uint32_t ksplit, const GemvArgs &a, uint32_t ntasks, hipStream_t st) {
    if (ksplit != 1 && ksplit != 2 && ksplit != 4 && ksplit != 8 && ksplit != 16) return hipErrorInvalidValue;
    // weights are addressed as a uniform base plus 32-bit byte offsets
    if ((uint64_t)a.nunits * (mode == GEMV_GATE_UP ? 2u : 1u) * a.tile_u4 * 16u > 0xFFFFFFFFull) return hipErrorInvalidValue;
    switch (mode) {
        case GEMV_PLAIN: return launch_gemv_t<GEMV_PLAIN>(a, ksplit, ntasks, st);
        case GEMV_RESID: return launch_gemv_t<GEMV_RESID>(a, ksplit, ntasks, st);
        case GEMV_GATE_UP: return launch_gemv_t<GEMV_GATE_UP>(a, ksplit, ntasks, st);
        case GEMV_F32: return launch_gemv_t<GEMV_F32>(a, ksplit, ntasks, st);
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------
// Two to kGemvMtTokens tokens: the decode kernel's structure -- units, K split over the waves of a
// unit, a whole scale group of weights requested at once, wave-private activation windows, no
// barrier before the last reduction -- with the dot products on the matrix cores.  A wave's lanes
// hold a row-tile's weights exactly as the GEMM's do (lane (i, c): block 4 sb + c of row i, dword kk
// the A operand of MFMA step kk, the scale folded in); the B operand of a step is one 16-byte chunk
// of a token's window, MFMA column j serving token j % kGemvMtTokens.  Against the one-token kernel
// the weight stream is the same and the vector ALU does a third more per weight (the exact
// (q - 8) d instead of the raw patterns), whatever the token count; against the MFMA GEMM at these
// token counts there are no partial planes, no plane-sum launches and no separate RMS-factor
// launch (four launches per layer instead of seven).  K must be a multiple of 1024.
// The windows are filled from global memory straight into LDS; chunk q of token t sits in slot
// q ^ t, so the 16 lanes x 4 lane groups of an operand read touch 16 different slots.
// A row's result is the sum of its scale-group partials in ascending group order, as in the
// one-token kernel: it depends neither on the K split nor on the workgroup shape.
// ------------------------------------------------------------------------------------
template <int MODE, int NW>
__global__ __launch_bounds__(NW * 64, 4) void gemv_mt_kernel(GemvArgs a, uint32_t ks, uint32_t ntok) {
    extern __shared__ uint4 mt_lds[];
    // a wave holds ONE row-tile's weights of a scale group at a time (two tiles' do not fit the registers beside
    // the operands): of a gate/up unit it takes the gate tile first and, super-block by super-block as the gate
    // tile's registers are used up, requests the up tile's into them, so one window serves both tiles
    constexpr int NT = (MODE == GEMV_GATE_UP) ? 2 : 1;
    constexpr int TK = kGemvMtTokens;
    constexpr bool NORM = (MODE == GEMV_PLAIN || MODE == GEMV_GATE_UP);
    static_assert(MODE != GEMV_F32, "dense sub-layers only");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, c = lane >> 4;
    const uint32_t wpu = ks;                    // waves per unit
    const uint32_t units = NW / wpu;
    const uint32_t unit = blockIdx.x * units + wave / wpu;
    const uint32_t kpart = wave % ks;
    const bool active = unit < a.nunits;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    uint4 *win = mt_lds + wave_u * (TK * 128);                                   // [token][128 chunks of 8]
    float *red = reinterpret_cast<float *>(mt_lds + NW * (TK * 128));            // [(unit, group)][tile][token][16 rows]
    float *red_ss = red + units * a.ngroups * (NT * TK * 16);                    // [(unit, group)][token]
    const uint32_t tb = j & (TK - 1);                                            // the token this lane's MFMA column serves
    const __amdgpu_buffer_rsrc_t xbuf = make_rsrc(a.x);

    if (active && kpart < a.ngroups) {
        for (uint32_t g = kpart; g < a.ngroups; g += ks) {
            // activations of the group for every token first (they are needed first), then the weights
            // slot r * 64 + lane of token t's window holds chunk (r * 64 + lane) ^ t: the same 128-column
            // stretch (one input head) for every t, so the column map is worked out once per r
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const uint32_t col0 = gather_col(g * 1024u + (uint32_t)(r * 64 + (lane & 48)) * 8u, a.x_off, a.x_group);
#pragma unroll
                for (int t = 0; t < TK; ++t) {
                    const uint32_t tokc = min((uint32_t)t, ntok - 1);   // windows past the last token repeat it (never stored)
                    const uint32_t voff = (tokc * a.x_stride + col0 + (((uint32_t)lane & 15u) ^ (uint32_t)t) * 8u) * (uint32_t)sizeof(__half);
                    load_to_lds16(xbuf, (lds_void *)(win + t * 128 + r * 64), voff, 0);
                }
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            GemvBuf<1> cur;
            gemv_issue_w<1, true>(cur, a.W, unit * NT, a.tile_u4, g, 8u, lane);
            const __amdgpu_buffer_rsrc_t wrs = make_rsrc(a.W);
            const uint32_t up_base = __builtin_amdgcn_readfirstlane((unit * NT + 1) * a.tile_u4 * 16u + g * (9u * 1024u));
            uint4 sc_up = make_uint4(0, 0, 0, 0);
            if (NT == 2) sc_up = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(wrs, (uint32_t)lane * 16u, up_base + 8u * 1024u, kAuxNt));
            // the window fills are the oldest loads in flight: all but the weight loads behind them
            // (the compiler does not know of loads into LDS; later loads only make this wait stricter)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(9 + (NT - 1)) : "memory");
            const uint32_t slot = (wave / wpu) * a.ngroups + g;
            if (NORM) {
#pragma unroll
                for (int t = 0; t < TK; ++t) {
                    const uint4 xa = win[t * 128 + lane], xb = win[t * 128 + 64 + lane];
                    float sq = 0.f;
                    sq = __builtin_amdgcn_fdot2(as_h2(xa.x), as_h2(xa.x), sq, false);
                    sq = __builtin_amdgcn_fdot2(as_h2(xa.y), as_h2(xa.y), sq, false);
                    sq = __builtin_amdgcn_fdot2(as_h2(xa.z), as_h2(xa.z), sq, false);
                    sq = __builtin_amdgcn_fdot2(as_h2(xa.w), as_h2(xa.w), sq, false);
                    sq = __builtin_amdgcn_fdot2(as_h2(xb.x), as_h2(xb.x), sq, false);
                    sq = __builtin_amdgcn_fdot2(as_h2(xb.y), as_h2(xb.y), sq, false);
                    sq = __builtin_amdgcn_fdot2(as_h2(xb.z), as_h2(xb.z), sq, false);
                    sq = __builtin_amdgcn_fdot2(as_h2(xb.w), as_h2(xb.w), sq, false);
                    const float gss = wave_sum(sq);
                    if (lane == 0) red_ss[slot * TK + t] = gss;
                }
            }
            const uint4 *wb = win + tb * 128;
#pragma unroll
            for (int tile = 0; tile < NT; ++tile) {
                const uint4 sc = tile == 0 ? cur.sc[0] : sc_up;
                f4_t gacc = f4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const uint4 wq = cur.wq[0][s];
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        const h8_t B = __builtin_bit_cast(h8_t, wb[(uint32_t)(s * 16 + c * 4 + kk) ^ tb]);
                        const uint32_t q = kk == 0 ? wq.x : kk == 1 ? wq.y : kk == 2 ? wq.z : wq.w;
                        const uint32_t dw = (s < 2) ? sc.x : (s < 4) ? sc.y : (s < 6) ? sc.z : sc.w;
                        const _Float16 d = __builtin_bit_cast(_Float16, (uint16_t)((s & 1) ? (dw >> 16) : (dw & 0xFFFFu)));
                        const h2_t dd = {d, d};
                        h2_t w[4];
                        dequant8(q, w);
                        w[0] *= dd; w[1] *= dd; w[2] *= dd; w[3] *= dd;
                        const h8_t A = h8_t{w[0].x, w[0].y, w[1].x, w[1].y, w[2].x, w[2].y, w[3].x, w[3].y};
                        gacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, B, gacc, 0, 0, 0);
                    }
                    // this super-block's registers are free: the next tile's super-block sets out into them
                    if (tile + 1 < NT)
                        cur.wq[0][s] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(wrs, (uint32_t)lane * 16u, up_base + (uint32_t)s * 1024u, kAuxNt));
                }
                // lane (j, c) holds rows 4c .. 4c + 3 of token column j
                if (j < TK)
                    *reinterpret_cast<float4 *>(red + ((slot * NT + tile) * TK + j) * 16 + c * 4) = make_float4(gacc[0], gacc[1], gacc[2], gacc[3]);
            }
            asm volatile("" ::: "memory");   // the window's reads are behind us before the next group's fills are issued
        }
    }
    __syncthreads();
    if (!(active && kpart == 0 && (uint32_t)j < ntok)) return;
    const uint32_t slot0 = (wave / wpu) * a.ngroups;
    float acc[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] = 0.f;
    float ss = 0.f;
    for (uint32_t g = 0; g < a.ngroups; ++g) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const float4 v = *reinterpret_cast<const float4 *>(red + (((slot0 + g) * NT + t) * TK + j) * 16 + c * 4);
            acc[t][0] += v.x; acc[t][1] += v.y; acc[t][2] += v.z; acc[t][3] += v.w;
        }
        if (NORM) ss += red_ss[(slot0 + g) * TK + j];
    }
    const float rinv = NORM ? rsqrtf(ss / (float)a.K + a.eps) : 1.f;
    const size_t o = (size_t)j * a.out_stride + a.out_row0 + unit * 16 + c * 4;
    float v[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        if (MODE == GEMV_PLAIN) v[r] = rinv * acc[0][r];
        else if (MODE == GEMV_RESID) v[r] = (a.res ? __half2float(a.res[o + r]) : 0.f) + acc[0][r];
        else v[r] = silu(rinv * acc[0][r]) * (rinv * acc[NT - 1][r]);
    }
    __half2 *dst = reinterpret_cast<__half2 *>(a.out + o);
    dst[0] = __halves2half2(to_half(v[0]), to_half(v[1]));
    dst[1] = __halves2half2(to_half(v[2]), to_half(v[3]));
}

size_t gemv_mt_lds_bytes(uint32_t nw, uint32_t units, uint32_t ngroups, uint32_t nt) {
    return (size_t)nw * kGemvMtTokens * 2048 + (size_t)units * ngroups * (nt * kGemvMtTokens * 64 + kGemvMtTokens * 4);
}

template <int MODE>
static hipError_t launch_gemv_mt_t(const GemvArgs &a, uint32_t ks, uint32_t ntok, hipStream_t st) {   // ks by value: adjusted below
    constexpr uint32_t NT = (MODE == GEMV_GATE_UP) ? 2 : 1;
    // workgroup shapes as for one token (launch_gemv_f)
    const uint32_t wpu = ks;
    uint32_t nw = wpu > 8 ? 16 : wpu > 4 ? 8 : 4;
    if (wpu == 4 && (a.nunits + 1) / 2 >= 192) nw = 8;
    const uint32_t units = nw / wpu;
    const size_t lds = gemv_mt_lds_bytes(nw, units, a.ngroups, NT);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    dim3 grid((a.nunits + units - 1) / units);
    static const hipError_t attr16 = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemv_mt_kernel<MODE, 16>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    static const hipError_t attr8 = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemv_mt_kernel<MODE, 8>),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr16 != hipSuccess) return attr16;
    if (attr8 != hipSuccess) return attr8;
    if (nw == 16) hipLaunchKernelGGL((gemv_mt_kernel<MODE, 16>), grid, dim3(1024), lds, st, a, ks, ntok);
    else if (nw == 8) hipLaunchKernelGGL((gemv_mt_kernel<MODE, 8>), grid, dim3(512), lds, st, a, ks, ntok);
    else hipLaunchKernelGGL((gemv_mt_kernel<MODE, 4>), grid, dim3(256), lds, st, a, ks, ntok);
    return hipGetLastError();
}

hipError_t launch_gemv_mt(int mode, uint32_t ksplit, const GemvArgs &a, uint32_t ntok, hipStream_t st) {
    if (ksplit != 1 && ksplit != 2 && ksplit != 4 && ksplit != 8 && ksplit != 16) return hipErrorInvalidValue;
    if (ntok < 1 || ntok > (uint32_t)kGemvMtTokens || a.nsb % 8 != 0 || a.tasks) return hipErrorInvalidValue;
    // weights and activations are addressed as a uniform base plus 32-bit byte offsets
    if ((uint64_t)a.nunits * (mode == GEMV_GATE_UP ? 2u : 1u) * a.tile_u4 * 16u > 0xFFFFFFFFull) return hipErrorInvalidValue;
    if ((uint64_t)ntok * a.x_stride * 2u > 0xFFFFFFFFull) return hipErrorInvalidValue;
    switch (mode) {
        case GEMV_PLAIN: return launch_gemv_mt_t<GEMV_PLAIN>(a, ksplit, ntok, st);
        case GEMV_RESID: return launch_gemv_mt_t<GEMV_RESID>(a, ksplit, ntok, st);
        case GEMV_GATE_UP: return launch_gemv_mt_t<GEMV_GATE_UP>(a, ksplit, ntok, st);
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------
// rinv[m] = 1 / sqrt(mean(x[m]^2) + eps), one workgroup per token (used when M > 1): thread t adds
// the 8-column chunks t, t + 256, ... in that order, the 64 lanes of a wave are summed by the
// butterfly, the four waves in order.  All of a thread's loads (up to four per round) are issued
// before the first is used; chunks past the row's end count as zeros.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rinv_kernel(const __half *x, uint32_t M, uint32_t H, float eps, float *rinv) {
    __shared__ float part[4];
    const uint32_t m = blockIdx.x;
    const uint4 *row = reinterpret_cast<const uint4 *>(x + (size_t)m * H);
    const uint32_t nq = H / 8;
    float ss = 0.f;
    for (uint32_t q0 = 0; q0 < nq; q0 += 1024) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            // (a chunk past the row's end re-reads the last one and counts as zeros: no branch around the load,
            // so the four requests go out together)
            const uint32_t q = q0 + u * 256 + threadIdx.x;
            const uint4 w = row[min(q, nq - 1)];
            v[u] = q < nq ? w : uint4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) ss += sumsq8(v[u]);
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) rinv[m] = rsqrtf((((part[0] + part[1]) + part[2]) + part[3]) / (float)H + eps);
}

hipError_t launch_rinv(const __half *x, uint32_t M, uint32_t H, float eps, float *rinv, hipStream_t st) {
    hipLaunchKernelGGL(rinv_kernel, dim3(M), dim3(256), 0, st, x, M, H, eps, rinv);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// MoE routing: per token the top_k largest fp32 logits (ties to the lower index, listed
// in descending order) and the softmax over the selected logits.  One wave per token.
// ------------------------------------------------------------------------------------
// Wave-wide maximum / minimum, the same value in every lane: the 16 lanes of a row meet through DPP
// row operations (no LDS traffic), the four rows through four lane reads.
__device__ __forceinline__ int dpp_i(int v, int ctrl) {
    switch (ctrl) {
        case 0: return __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);    // quad_perm 1,0,3,2
        case 1: return __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);    // quad_perm 2,3,0,1
        case 2: return __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false);   // row_half_mirror
        default: return __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, false);  // row_mirror
    }
}
__device__ __forceinline__ float wave_max_all(float v) {
#pragma unroll
    for (int c = 0; c < 4; ++c) v = fmaxf(v, __builtin_bit_cast(float, dpp_i(__builtin_bit_cast(int, v), c)));
    const int b = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0)), r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32)), r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ __forceinline__ uint32_t wave_min_all(uint32_t v) {
#pragma unroll
    for (int c = 0; c < 4; ++c) v = min(v, (uint32_t)dpp_i((int)v, c));
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    return min(min(r0, r1), min(r2, r3));
}

template <int NR>   // 64 * NR >= E
__global__ __launch_bounds__(256) void route_kernel(const float *logits, uint32_t M, uint32_t E, uint32_t top_k,
                                                    int32_t *idx, float *w) {
    const uint32_t m = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (m >= M) return;
    const float *l = logits + (size_t)m * E;
    float v[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const uint32_t e = r * 64 + lane;
        v[r] = e < E ? l[e] : -INFINITY;
    }
    uint32_t taken = 0;  // bit r: this lane's entry r already selected
    float sel = 0.f, lmax = 0.f;
    for (uint32_t j = 0; j < top_k; ++j) {
        float best = -INFINITY;
        uint32_t be = 0xFFFFFFFFu;
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const uint32_t e = r * 64 + lane;
            if (e < E && !((taken >> r) & 1u) && (be == 0xFFFFFFFFu || v[r] > best)) { best = v[r]; be = e; }
        }
        // the largest value in the wave, then the lowest index among the lanes that hold it
        // (a lane with nothing left holds -inf and the index 0xFFFFFFFF, which never wins)
        const float top = wave_max_all(best);
        be = wave_min_all(best == top ? be : 0xFFFFFFFFu);
        best = top;
        if ((be & 63u) == (uint32_t)lane) taken |= 1u << (be >> 6);
        if (j == 0) lmax = best;
        if ((uint32_t)lane == j) sel = best;
        if (lane == 0) idx[(size_t)m * top_k + j] = (int32_t)be;
    }
    const float ex = (uint32_t)lane < top_k ? __expf(sel - lmax) : 0.f;
    const float den = wave_sum(ex);
    if ((uint32_t)lane < top_k) w[(size_t)m * top_k + lane] = ex / den;
}

hipError_t launch_route(const float *logits, uint32_t M, uint32_t E, uint32_t top_k, int32_t *idx, float *w,
                        hipStream_t st) {
    if (E > 1024 || top_k == 0 || top_k > 64 || top_k > E) return hipErrorInvalidValue;
    if (E <= 128) hipLaunchKernelGGL(route_kernel<2>, dim3((M + 3) / 4), dim3(256), 0, st, logits, M, E, top_k, idx, w);
    else if (E <= 256) hipLaunchKernelGGL(route_kernel<4>, dim3((M + 3) / 4), dim3(256), 0, st, logits, M, E, top_k, idx, w);
    else hipLaunchKernelGGL(route_kernel<16>, dim3((M + 3) / 4), dim3(256), 0, st, logits, M, E, top_k, idx, w);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Decode attention over a KV cache (one new token; softmax(q.K / sqrt(d)) V, no positional
// encoding).  HBM-bound on the cache bytes: a workgroup streams 256 positions of one kv head
// (64 KB of K, then 64 KB of V) once for all G query heads that share it.
// 16 lanes hold one position (8 dims each), so a wave load covers 4 whole rows (1 KB contiguous).
// Pass 1: scores of the chunk -> LDS; chunk maximum per query head.  Pass 2: p = exp(s - max),
// sum of p and p-weighted V sums.  Chunks are merged by attn_combine_kernel in chunk order, so the
// result does not depend on where the cache shard lives.
// ------------------------------------------------------------------------------------
constexpr int kAttnWaves = 8;             // waves per workgroup (measured at a 16K context: 4 -> 1.716, 8 -> 1.680, 16 -> 1.744 ms per token)
constexpr int kAttnIts = 8;               // steps of 4 positions per wave
constexpr int kAttnPos = kAttnWaves * kAttnIts * 4;   // positions per workgroup (a multiple of kAttnChunk, which sizes the partials)
static_assert(kAttnPos % kAttnChunk == 0, "the workspace is sized for one partial per kAttnChunk positions");
constexpr uint32_t kKRowBytes = 272;   // LDS pitch of a staged K row: the 16 rows of an operand read lie 4 banks apart
constexpr uint32_t kVRowBytes = 288;   // LDS pitch of a staged V row: 256 + 32, so that the four rows of a transpose read lie 8 banks apart
// A operand of O^T += V^T P^T for MFMA step s of a staged chunk and dim tile dt: lane (i, c) needs dim
// 16 dt + i of the 8 positions 32 s + 8 c .. + 7, i.e. a COLUMN of the staged rows.  The LDS transpose read
// of gfx950 (ds_read_b64_tr_b16) does that within each group of 16 lanes: lane L of a group names 8 bytes
// (4 numbers), lane m receives number m % 4 of lanes m / 4, m / 4 + 4, m / 4 + 8, m / 4 + 12 (checked on the
// hardware with index numbers as data).  With lane L naming row L / 4, dims 4 (L % 4) .. + 3 of the tile,
// lane i receives dim i of four consecutive positions; two reads make the operand.
// lane_base = staged rows + (8 c + i / 4) * kVRowBytes + (i % 4) * 8.
__device__ __forceinline__ h8_t v_operand(const unsigned char *lane_base, int s, int dt) {
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((__vector_size__(4 * sizeof(__fp16)))) __fp16 fp16x4_t;
    typedef __attribute__((address_space(3))) fp16x4_t lds_fp16x4_t;
    const unsigned char *p = lane_base + (32 * s) * kVRowBytes + dt * 32;
    const fp16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4f16((lds_fp16x4_t *)(p));
    const fp16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4f16((lds_fp16x4_t *)(p + 4 * kVRowBytes));
    const uint2 a = __builtin_bit_cast(uint2, lo), b = __builtin_bit_cast(uint2, hi);
    return __builtin_bit_cast(h8_t, make_uint4(a.x, a.y, b.x, b.y));
#else
    return h8_t{};
#endif
}
static_assert(kAttnPos == kAttnPosPerWg, "the executor numbers the chunk's own partials behind ceil(ctx / kAttnPosPerWg) cache chunks");

// sum over each row of 16 lanes, result in every lane of the row (DPP: no LDS traffic)
__device__ __forceinline__ float row16_sum(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false));   // quad_perm 1,0,3,2
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, false));   // quad_perm 2,3,0,1
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, false));  // row_half_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, false));  // row_mirror
    return v;
}

template <int G>
__global__ __launch_bounds__(kAttnWaves * 64, 16 / kAttnWaves) void attn_decode_kernel(AttnArgs a) {
    __shared__ float red[kAttnWaves][G][128];
    __shared__ float redm[kAttnWaves][G], redl[kAttnWaves][G];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int dl = lane & 15, pg = lane >> 4;
    const uint32_t chunk = blockIdx.x, hk = blockIdx.y;               // kv head within this launch
    const uint32_t ctx = a.ctx_dev ? *a.ctx_dev : a.ctx;              // the same for the whole grid
    if (chunk * kAttnPos >= ctx) return;                              // (launches sized for the whole cache)
    const __half *K = reinterpret_cast<const __half *>(reinterpret_cast<const char *>(a.kv) + (size_t)hk * a.head_stride);
    const __half *V = K + (size_t)a.cap * 128;
    const uint32_t q0 = (a.head0 + hk) * G;                           // first query head of this kv head
    const float scale = 0.08838834764831845f;                         // 1 / sqrt(128)

    // the queries first (loads return in order: issued last they would arrive last, and the scores
    // could not start before every cache row had arrived)
    uint4 qv[G];
#pragma unroll
    for (int h = 0; h < G; ++h) qv[h] = *reinterpret_cast<const uint4 *>(a.q + (size_t)(q0 + h) * 128 + dl * 8);
    // all of the wave's cache rows are requested up front (K chunks, then V chunks):
    // the V rows stream in while the scores are computed
    // Buffer loads bounded to the ctx valid rows: a row past the end reads as zeros, so the loads
    // need no branch (a branch per load would also make the compiler wait for each load at once)
    const uint32_t base = chunk * kAttnPos + wave * (kAttnPos / kAttnWaves);
    const __amdgpu_buffer_rsrc_t kb = __builtin_amdgcn_make_buffer_rsrc(const_cast<__half *>(K), 0, (int)(ctx * 256u), 0x00020000);
    const __amdgpu_buffer_rsrc_t vb = __builtin_amdgcn_make_buffer_rsrc(const_cast<__half *>(V), 0, (int)(ctx * 256u), 0x00020000);
    const uint32_t voff = (uint32_t)pg * 256u + (uint32_t)dl * 16u;
    const uint32_t soff = __builtin_amdgcn_readfirstlane(base * 256u);
    uint4 kq[kAttnIts], vq[kAttnIts];
#pragma unroll
    for (int it = 0; it < kAttnIts; ++it)
        kq[it] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(kb, voff, soff + it * 1024, kAuxNt));
#pragma unroll
    for (int it = 0; it < kAttnIts; ++it)
        vq[it] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(vb, voff, soff + it * 1024, kAuxNt));
    // A wave works alone until the very end (no workgroup barrier between the passes): scores of its
    // positions stay in registers (the 16 lanes of a position meet through DPP row operations and
    // all hold the score), its own maximum, its own weights and sums.
    float sc[kAttnIts][G], mx[G];
#pragma unroll
    for (int h = 0; h < G; ++h) mx[h] = -INFINITY;
#pragma unroll
    for (int it = 0; it < kAttnIts; ++it) {
        const uint32_t j = base + it * 4 + pg;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float d = 0.f;
            d = __builtin_amdgcn_fdot2(as_h2(qv[h].x), as_h2(kq[it].x), d, false);
            d = __builtin_amdgcn_fdot2(as_h2(qv[h].y), as_h2(kq[it].y), d, false);
            d = __builtin_amdgcn_fdot2(as_h2(qv[h].z), as_h2(kq[it].z), d, false);
            d = __builtin_amdgcn_fdot2(as_h2(qv[h].w), as_h2(kq[it].w), d, false);
            const float r = row16_sum(d) * scale;      // outside any branch: every lane takes part
            sc[it][h] = j < ctx ? r : -INFINITY;
            mx[h] = fmaxf(mx[h], sc[it][h]);
        }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {   // the wave's 4 position groups
        mx[h] = fmaxf(mx[h], __shfl_xor(mx[h], 16, 64));
        mx[h] = fmaxf(mx[h], __shfl_xor(mx[h], 32, 64));
    }
    // a wave whose positions all lie past the end has maximum -inf: its weights must be 0, not NaN
    float l[G], o[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[h][e] = 0.f;
    }
#pragma unroll
    for (int it = 0; it < kAttnIts; ++it) {
        float vf[8];
        const uint32_t vd[4] = {vq[it].x, vq[it].y, vq[it].z, vq[it].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const h2_t pr = as_h2(vd[e]);
            vf[2 * e] = (float)pr.x;
            vf[2 * e + 1] = (float)pr.y;
        }
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float p = sc[it][h] == -INFINITY ? 0.f : __expf(sc[it][h] - mx[h]);
            l[h] += p;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[h][e] = fmaf(p, vf[e], o[h][e]);
        }
    }
    // the 4 position groups of a wave meet (36 independent values: LDS permutes, which pipeline, measured
    // faster here than the in-register row swaps the one-token GEMV uses for its one or two values);
    // then the workgroup's waves through LDS, rescaled to the chunk maximum, in fixed order
#pragma unroll
    for (int h = 0; h < G; ++h) {
        l[h] += __shfl_xor(l[h], 16, 64);
        l[h] += __shfl_xor(l[h], 32, 64);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            o[h][e] += __shfl_xor(o[h][e], 16, 64);
            o[h][e] += __shfl_xor(o[h][e], 32, 64);
        }
        if (pg == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) red[wave][h][dl * 8 + e] = o[h][e];
            if (dl == 0) { redl[wave][h] = l[h]; redm[wave][h] = mx[h]; }
        }
    }
    __syncthreads();
    for (int t = tid; t < G * 128; t += kAttnWaves * 64) {
        const int h = t >> 7, d = t & 127;
        // wave 0's first position is always valid in a launched chunk, so the chunk maximum is finite
        float m = redm[0][h];
#pragma unroll
        for (int k = 1; k < kAttnWaves; ++k) m = fmaxf(m, redm[k][h]);
        float od = 0.f, ld = 0.f;   // waves in ascending order
#pragma unroll
        for (int k = 0; k < kAttnWaves; ++k) {
            const float w = redm[k][h] == -INFINITY ? 0.f : __expf(redm[k][h] - m);
            od = fmaf(w, red[k][h][d], od);
            ld = fmaf(w, redl[k][h], ld);
        }
        float *dst = a.part + ((size_t)(q0 + h) * a.chunk_cap + chunk) * 130;
        dst[2 + d] = od;
        if (d == 0) {
            dst[0] = m;
            dst[1] = ld;
        }
    }
}

// ------------------------------------------------------------------------------------
// Attention for a CHUNK of new tokens (chunked prefill over the cache): the same streaming scheme with
// a loop over the chunk's tokens.  A workgroup holds 256 positions of one kv head in registers (cache
// rows, or the chunk's own K / V rows read in place from the QKV buffer: row stride and base differ,
// nothing else) and serves every token of the chunk in turn: token t sees positions below limit(t) =
// ctx for cache rows, t + 1 for the chunk's rows (causal).  Per (token, query head, position chunk) it
// writes the chunk maximum, weight sum and 128 weighted sums; attn_combine_chunk_kernel merges a
// token's chunks in ascending order, so the result does not depend on where a cache shard lives.
// ------------------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(kAttnWaves * 64, 16 / kAttnWaves) void attn_chunk_kernel(AttnChunkArgs a) {
    __shared__ float red[kAttnWaves][G][128];
    __shared__ float redm[kAttnWaves][G], redl[kAttnWaves][G];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int dl = lane & 15, pg = lane >> 4;
    const uint32_t chunk = blockIdx.x, hk = blockIdx.y;
    const uint32_t kv_head = a.head0 + hk;
    const __half *K = a.causal ? a.k_base + (size_t)kv_head * 128 : reinterpret_cast<const __half *>(reinterpret_cast<const char *>(a.k_base) + (size_t)hk * a.head_stride);
    const __half *V = a.causal ? a.v_base + (size_t)kv_head * 128 : K + (size_t)a.cap * 128;
    const uint32_t q0 = kv_head * G;
    const float scale = 0.08838834764831845f;   // 1 / sqrt(128)
    const uint32_t row_b = a.row_stride * 2u;   // bytes between two positions' rows
    const uint32_t npos = a.causal ? a.ntok : a.ctx;                        // rows that exist
    const uint32_t range = npos ? (npos - 1) * row_b + 256u : 0u;          // a row past the end reads as zeros
    const uint32_t base = chunk * kAttnPos + wave * (kAttnPos / kAttnWaves);
    const __amdgpu_buffer_rsrc_t kb = __builtin_amdgcn_make_buffer_rsrc(const_cast<__half *>(K), 0, (int)range, 0x00020000);
    const __amdgpu_buffer_rsrc_t vb = __builtin_amdgcn_make_buffer_rsrc(const_cast<__half *>(V), 0, (int)range, 0x00020000);
    const uint32_t voff = (uint32_t)pg * row_b + (uint32_t)dl * 16u;
    const uint32_t soff = __builtin_amdgcn_readfirstlane(base * row_b);
    uint4 kq[kAttnIts], vq[kAttnIts];
#pragma unroll
    for (int it = 0; it < kAttnIts; ++it)
        kq[it] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(kb, voff, soff + it * 4 * row_b, 0));
#pragma unroll
    for (int it = 0; it < kAttnIts; ++it)
        vq[it] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(vb, voff, soff + it * 4 * row_b, 0));
    float vf[kAttnIts][8];
#pragma unroll
    for (int it = 0; it < kAttnIts; ++it) {
        const uint32_t vd[4] = {vq[it].x, vq[it].y, vq[it].z, vq[it].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const h2_t pr = as_h2(vd[e]);
            vf[it][2 * e] = (float)pr.x;
            vf[it][2 * e + 1] = (float)pr.y;
        }
    }
    // this workgroup's share of the tokens (blockIdx.z), from the first token that sees any position of
    // this chunk (causal: token chunk * kAttnPos)
    const uint32_t t_lo = blockIdx.z * a.tok_per_wg, t_hi = min(a.ntok, t_lo + a.tok_per_wg);
    const uint32_t t_first = max(t_lo, a.causal ? chunk * kAttnPos : 0u);
#pragma unroll 1
    for (uint32_t t = t_first; t < t_hi; ++t) {
        const uint32_t limit = a.causal ? t + 1 : a.ctx;
        uint4 qv[G];
#pragma unroll
        for (int h = 0; h < G; ++h) qv[h] = *reinterpret_cast<const uint4 *>(a.q + (size_t)t * a.q_stride + (size_t)(q0 + h) * 128 + dl * 8);
        float sc[kAttnIts][G], mx[G];
#pragma unroll
        for (int h = 0; h < G; ++h) mx[h] = -INFINITY;
#pragma unroll
        for (int it = 0; it < kAttnIts; ++it) {
            const uint32_t j = base + it * 4 + pg;
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float d = 0.f;
                d = __builtin_amdgcn_fdot2(as_h2(qv[h].x), as_h2(kq[it].x), d, false);
                d = __builtin_amdgcn_fdot2(as_h2(qv[h].y), as_h2(kq[it].y), d, false);
                d = __builtin_amdgcn_fdot2(as_h2(qv[h].z), as_h2(kq[it].z), d, false);
                d = __builtin_amdgcn_fdot2(as_h2(qv[h].w), as_h2(kq[it].w), d, false);
                const float r = row16_sum(d) * scale;
                sc[it][h] = j < limit ? r : -INFINITY;
                mx[h] = fmaxf(mx[h], sc[it][h]);
            }
        }
#pragma unroll
        for (int h = 0; h < G; ++h) {
            mx[h] = fmaxf(mx[h], __shfl_xor(mx[h], 16, 64));
            mx[h] = fmaxf(mx[h], __shfl_xor(mx[h], 32, 64));
        }
        float l[G], o[G][8];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            l[h] = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[h][e] = 0.f;
        }
#pragma unroll
        for (int it = 0; it < kAttnIts; ++it) {
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float p = sc[it][h] == -INFINITY ? 0.f : __expf(sc[it][h] - mx[h]);
                l[h] += p;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[h][e] = fmaf(p, vf[it][e], o[h][e]);
            }
        }
#pragma unroll
        for (int h = 0; h < G; ++h) {
            l[h] += __shfl_xor(l[h], 16, 64);
            l[h] += __shfl_xor(l[h], 32, 64);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                o[h][e] += __shfl_xor(o[h][e], 16, 64);
                o[h][e] += __shfl_xor(o[h][e], 32, 64);
            }
            if (pg == 0) {
#pragma unroll
                for (int e = 0; e < 8; ++e) red[wave][h][dl * 8 + e] = o[h][e];
                if (dl == 0) { redl[wave][h] = l[h]; redm[wave][h] = mx[h]; }
            }
        }
        __syncthreads();
        for (int u = tid; u < G * 128; u += kAttnWaves * 64) {
            const int h = u >> 7, d = u & 127;
            // the chunk's first position is below the limit (t >= t_first), so wave 0's maximum is finite
            float m = redm[0][h];
#pragma unroll
            for (int k = 1; k < kAttnWaves; ++k) m = fmaxf(m, redm[k][h]);
            float od = 0.f, ld = 0.f;   // waves in ascending order
#pragma unroll
            for (int k = 0; k < kAttnWaves; ++k) {
                const float w = redm[k][h] == -INFINITY ? 0.f : __expf(redm[k][h] - m);
                od = fmaf(w, red[k][h][d], od);
                ld = fmaf(w, redl[k][h], ld);
            }
            float *dst = a.part + (((size_t)t * a.n_q + q0 + h) * a.chunk_cap + a.chunk0 + chunk) * 130;
            dst[2 + d] = od;
            if (d == 0) {
                dst[0] = m;
                dst[1] = ld;
            }
        }
        __syncthreads();   // the next token reuses the reduction buffers
    }
}

// ------------------------------------------------------------------------------------
// The same partials on the matrix cores.  Rows of the score matrix are (token, query head of the
// kv group) pairs, 16 per wave, 64 per workgroup; a workgroup covers 256 positions of one kv head in
// 8 steps of 32.
//  scores, transposed: S^T = K Q^T by v_mfma_f32_16x16x32_f16 with A = 16 positions x 32 dims of K
//   (lane (p, c) loads 16 bytes of a K row straight from memory) and B = the wave's 16 query rows
//   (registers, loaded once): the accumulator then holds, in lane (row j, rg), four positions of row j;
//  weights x values, transposed: O^T = V^T P^T with B = the weights exactly as the score
//   accumulators hold them (the two 16-position tiles of a step are numbered so that lane group c
//   owns 8 consecutive positions: 4 from each tile) and A = 16 dims x 32 positions of V, read
//   column-wise (8 two-byte reads) from the chunk's V rows staged in LDS once per workgroup.
// Two passes over the chunk's 8 steps: all scores (64 registers) and the row maximum, then weights,
// weight sum and O^T; per (row, chunk) the same (maximum, weight sum, 128 weighted sums) record as
// the vector-ALU kernel writes, merged by attn_combine_chunk_kernel in chunk order.
// ------------------------------------------------------------------------------------

// Score pass of the chunk kernels: S^T = K Q^T for the 16 position tiles of a 256-position chunk (tile t: step
// t / 2, tile t % 2 of the step: positions P0 + 32 (t / 2) + 8 (p / 4) + 4 (t % 2) + p % 4, p = 0 .. 15).  The K
// rows are A operands straight from memory, so their loads have to be under way well before the MFMAs that
// take them: kKAhead tiles (4 loads each) stay in flight, a tile's registers refilled as soon as its MFMAs have
// read them.  (Left to the scheduler, every load sat right in front of its MFMA: 64 exposed round trips to
// the L2 per chunk.)
constexpr int kKAhead = 4;
struct KTiles { h8_t k[kKAhead][4]; };
__device__ __forceinline__ void k_tile_load(__amdgpu_buffer_rsrc_t kb, uint32_t P0, uint32_t row_b, int t, int i, int c, h8_t (&dst)[4]) {
    const uint32_t pos = P0 + 32 * (t >> 1) + 8 * (i >> 2) + 4 * (t & 1) + (i & 3);        // the K row this lane supplies
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        dst[kk] = __builtin_bit_cast(h8_t, __builtin_amdgcn_raw_buffer_load_b128(kb, pos * row_b + kk * 64 + c * 16, 0, 0));
}
__device__ __forceinline__ void k_tiles_open(__amdgpu_buffer_rsrc_t kb, uint32_t P0, uint32_t row_b, int i, int c, KTiles &kt) {
#pragma unroll
    for (int t = 0; t < kKAhead; ++t) k_tile_load(kb, P0, row_b, t, i, c, kt.k[t]);
}
// scores (scaled, -inf where the lane's row does not see the position) and their maximum over the lane's registers
__device__ __forceinline__ void attn_scores(__amdgpu_buffer_rsrc_t kb, uint32_t P0, uint32_t row_b, int i, int c, KTiles &kt,
                                            const h8_t (&qreg)[4], float scale, uint32_t limit, f4_t (&S)[8][2], float &mx) {
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        __builtin_amdgcn_sched_barrier(0);
        f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kt.k[t % kKAhead][kk], qreg[kk], acc, 0, 0, 0);
        if (t + kKAhead < 16) k_tile_load(kb, P0, row_b, t + kKAhead, i, c, kt.k[t % kKAhead]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t pj = P0 + 32 * (t >> 1) + 8 * c + 4 * (t & 1) + r;
            acc[r] = pj < limit ? acc[r] * scale : -INFINITY;
            mx = fmaxf(mx, acc[r]);
        }
        S[t >> 1][t & 1] = acc;
    }
}

__global__ __launch_bounds__(256, 2) void attn_chunk_mfma_kernel(AttnChunkArgs a) {
    extern __shared__ uint4 lds_v4[];
    unsigned char *ldsv = reinterpret_cast<unsigned char *>(lds_v4);   // [256 positions][kVRowBytes]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, c = lane >> 4;
    const uint32_t chunk = blockIdx.x, hk = blockIdx.y, G = a.group;
    const uint32_t kv_head = a.head0 + hk;
    const __half *K = a.causal ? a.k_base + (size_t)kv_head * 128 : reinterpret_cast<const __half *>(reinterpret_cast<const char *>(a.k_base) + (size_t)hk * a.head_stride);
    const __half *V = a.causal ? a.v_base + (size_t)kv_head * 128 : K + (size_t)a.cap * 128;
    const uint32_t q0 = kv_head * G;
    const uint32_t row_b = a.row_stride * 2u;
    const uint32_t npos = a.causal ? a.ntok : a.ctx;
    const uint32_t range = npos ? (npos - 1) * row_b + 256u : 0u;   // a row past the end reads as zeros
    const uint32_t P0 = chunk * kAttnPos;
    const uint32_t R = a.ntok * G;                                   // score rows of this kv head
    const uint32_t row0 = blockIdx.z * 64;
    if (row0 >= R) return;
    // causal: the workgroup's last token sees nothing of this chunk -> nothing to write (uniform)
    if (a.causal && min(a.ntok - 1, (row0 + 63) / G) < P0) return;
    const __amdgpu_buffer_rsrc_t kb = __builtin_amdgcn_make_buffer_rsrc(const_cast<__half *>(K), 0, (int)range, 0x00020000);
    const __amdgpu_buffer_rsrc_t vb = __builtin_amdgcn_make_buffer_rsrc(const_cast<__half *>(V), 0, (int)range, 0x00020000);

    KTiles kt;
    k_tiles_open(kb, P0, row_b, i, c, kt);      // the first K tiles set out ahead of everything else
    __builtin_amdgcn_sched_barrier(0);
    // V rows of the chunk -> LDS (all 256 threads; 16 bytes each, 16 rounds): every piece is requested before
    // the first is written (written one by one, each load was waited for before the next was issued)
    {
        uint4 vq[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const uint32_t idx = r * 256 + tid, pos = idx >> 4, seg = idx & 15;
            vq[r] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(vb, (P0 + pos) * row_b + seg * 16, 0, 0));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const uint32_t idx = r * 256 + tid, pos = idx >> 4, seg = idx & 15;
            uint2 *dst = reinterpret_cast<uint2 *>(ldsv + pos * kVRowBytes + seg * 16);
            dst[0] = make_uint2(vq[r].x, vq[r].y);
            dst[1] = make_uint2(vq[r].z, vq[r].w);
        }
    }
    // this wave's 16 query rows (B operand of the score MFMAs): row rho = (token, head of the group)
    const uint32_t rho = min(row0 + wave * 16 + i, R - 1);
    const uint32_t tok = rho / G, hq = rho % G;
    const bool row_ok = row0 + wave * 16 + i < R;
    const uint32_t limit = a.causal ? tok + 1 : a.ctx;               // positions below it are visible to this lane's row
    h8_t qreg[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        qreg[kk] = __builtin_bit_cast(h8_t, *reinterpret_cast<const uint4 *>(a.q + (size_t)tok * a.q_stride + (size_t)(q0 + hq) * 128 + kk * 32 + c * 8));

    const float scale = 0.08838834764831845f;   // 1 / sqrt(128)
    // pass 1: scores of the 8 steps.  Tile T of a step holds positions base + 8 (p >> 2) + 4 T + (p & 3), p = 0..15
    f4_t S[8][2];
    float mx = -INFINITY;
    attn_scores(kb, P0, row_b, i, c, kt, qreg, scale, limit, S, mx);
    mx = rows4_meet<true>(mx);      // the row's four lanes (one per lane group) meet
    __syncthreads();                // the staged V rows are complete

    // pass 2: weights, their sum, and O^T += V^T P^T
    f4_t O[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) O[dt] = f4_t{0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        float pv[8];
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float sc = S[s][T][r];
                pv[4 * T + r] = sc == -INFINITY ? 0.f : __expf(sc - mx);
                l += pv[4 * T + r];
            }
        const h8_t Bp = {(_Float16)pv[0], (_Float16)pv[1], (_Float16)pv[2], (_Float16)pv[3],
                         (_Float16)pv[4], (_Float16)pv[5], (_Float16)pv[6], (_Float16)pv[7]};
        // A operand: dim 16 dt + i of the 8 positions 32 s + 8 c .. + 7 (a column of the staged rows)
        const unsigned char *vbase = ldsv + (8 * c + (i >> 2)) * kVRowBytes + (i & 3) * 8;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(v_operand(vbase, s, dt), Bp, O[dt], 0, 0, 0);
    }
    l = rows4_meet<false>(l);
    // lane (row i, group c) holds dims 16 dt + 4 c + r of its row
    if (!row_ok || mx == -INFINITY) return;      // no such row, or a row that sees nothing of this chunk
    float *dst = a.part + (((size_t)tok * a.n_q + q0 + hq) * a.chunk_cap + a.chunk0 + chunk) * 130;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
        float2 *d2 = reinterpret_cast<float2 *>(dst + 2 + 16 * dt + 4 * c);
        d2[0] = make_float2(O[dt][0], O[dt][1]);
        d2[1] = make_float2(O[dt][2], O[dt][3]);
    }
    if (c == 0) {
        dst[0] = mx;
        dst[1] = l;
    }
}

// ------------------------------------------------------------------------------------
// Many-token chunks (plans of kAttnOnePassTokens tokens and more): the same two products, but one
// workgroup walks ALL positions of its 64 score rows -- the cache's chunks, then the chunk's own rows up
// to its last token -- keeping a running maximum, weight sum and O^T per row and rescaling them when a
// chunk raises the maximum, and writes the finished attention rows.  No partial records: their size
// (tokens x heads x chunks) is what makes the record form unusable for long chunks over long contexts.
// The order of the chunks is fixed, so the result does not depend on where a cache shard lives.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 1) void attn_chunk_onepass_kernel(AttnChunkArgs a) {
    extern __shared__ uint4 lds_v4[];
    unsigned char *ldsv = reinterpret_cast<unsigned char *>(lds_v4);   // V rows [256 positions][kVRowBytes]
    unsigned char *ldsk = ldsv + kAttnPos * kVRowBytes;                 // K rows [256 positions][kKRowBytes]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, c = lane >> 4;
    const uint32_t hk = blockIdx.x, G = a.group;
    const uint32_t kv_head = a.head0 + hk;
    const uint32_t q0 = kv_head * G;
    const uint32_t R = a.ntok * G;
    const uint32_t row0 = blockIdx.y * 64;
    if (row0 >= R) return;
    const uint32_t rho = min(row0 + wave * 16 + i, R - 1);
    const uint32_t tok = rho / G, hq = rho % G;
    const bool row_ok = row0 + wave * 16 + i < R;
    const uint32_t last_tok = min(a.ntok - 1, (row0 + 63) / G);      // the workgroup's last token
    h8_t qreg[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        qreg[kk] = __builtin_bit_cast(h8_t, *reinterpret_cast<const uint4 *>(a.q + (size_t)tok * a.q_stride + (size_t)(q0 + hq) * 128 + kk * 32 + c * 8));
    const float scale = 0.08838834764831845f;   // 1 / sqrt(128)
    float m_run = -INFINITY, l_run = 0.f;
    f4_t O[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) O[dt] = f4_t{0.f, 0.f, 0.f, 0.f};

    const uint32_t nc_cache = (a.ctx + kAttnPos - 1) / kAttnPos, nc_own = last_tok / kAttnPos + 1;
#pragma unroll 1
    for (uint32_t cc = 0; cc < nc_cache + nc_own; ++cc) {
        const bool own = cc >= nc_cache;                  // the same for the whole workgroup
        const uint32_t chunk = own ? cc - nc_cache : cc;
        const __half *K = own ? a.k_own + (size_t)kv_head * 128 : reinterpret_cast<const __half *>(reinterpret_cast<const char *>(a.k_base) + (size_t)hk * a.head_stride);
        const __half *V = own ? a.v_own + (size_t)kv_head * 128 : K + (size_t)a.cap * 128;
        const uint32_t row_b = (own ? a.own_stride : 128u) * 2u;
        const uint32_t npos = own ? a.ntok : a.ctx;
        const uint32_t range = (npos - 1) * row_b + 256u;
        const uint32_t limit = own ? tok + 1 : a.ctx;
        const uint32_t P0 = chunk * kAttnPos;
        const __amdgpu_buffer_rsrc_t kb = __builtin_amdgcn_make_buffer_rsrc(const_cast<__half *>(K), 0, (int)range, 0x00020000);
        const __amdgpu_buffer_rsrc_t vb = __builtin_amdgcn_make_buffer_rsrc(const_cast<__half *>(V), 0, (int)range, 0x00020000);
        // the chunk's K and V rows -> LDS: every thread requests its 32 pieces (16 bytes each) at once, so the
        // whole 128 KB is under way together (the four waves share the K rows instead of each reading them all)
        {
            uint4 kq[16], vq[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const uint32_t idx = r * 256 + tid, pos = idx >> 4, seg = idx & 15;
                kq[r] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(kb, (P0 + pos) * row_b + seg * 16, 0, 0));
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const uint32_t idx = r * 256 + tid, pos = idx >> 4, seg = idx & 15;
                vq[r] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(vb, (P0 + pos) * row_b + seg * 16, 0, 0));
            }
            __syncthreads();     // every wave has left the previous chunk's staged rows
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const uint32_t idx = r * 256 + tid, pos = idx >> 4, seg = idx & 15;
                *reinterpret_cast<uint4 *>(ldsk + pos * kKRowBytes + seg * 16) = kq[r];
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const uint32_t idx = r * 256 + tid, pos = idx >> 4, seg = idx & 15;
                uint2 *dst = reinterpret_cast<uint2 *>(ldsv + pos * kVRowBytes + seg * 16);
                dst[0] = make_uint2(vq[r].x, vq[r].y);
                dst[1] = make_uint2(vq[r].z, vq[r].w);
            }
        }
        __syncthreads();     // the staged rows are complete
        f4_t S[8][2];
        float mx = -INFINITY;
        {
            // S^T = K Q^T, the K rows as A operands from LDS: lane (i, c) supplies row 8 (i / 4) + i % 4 (+ 4 for
            // the second tile of a step), bytes 64 kk + 16 c
            const unsigned char *kbase = ldsk + (8 * (i >> 2) + (i & 3)) * kKRowBytes + c * 16;
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const h8_t kreg = __builtin_bit_cast(h8_t, *reinterpret_cast<const uint4 *>(kbase + (32 * (t >> 1) + 4 * (t & 1)) * kKRowBytes + kk * 64));
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kreg, qreg[kk], acc, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint32_t pj = P0 + 32 * (t >> 1) + 8 * c + 4 * (t & 1) + r;
                    acc[r] = pj < limit ? acc[r] * scale : -INFINITY;
                    mx = fmaxf(mx, acc[r]);
                }
                S[t >> 1][t & 1] = acc;
            }
        }
        mx = rows4_meet<true>(mx);
        const float m_new = fmaxf(m_run, mx);
        // a row that has seen nothing yet keeps zeros (the difference of two -inf is not a number)
        const float resc = m_run == -INFINITY ? 0.f : __expf(m_run - m_new);
        m_run = m_new;
        l_run *= resc;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) O[dt] = O[dt] * resc;
        float l = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            float pv[8];
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float sc = S[s][T][r];
                    pv[4 * T + r] = sc == -INFINITY ? 0.f : __expf(sc - m_new);
                    l += pv[4 * T + r];
                }
            const h8_t Bp = {(_Float16)pv[0], (_Float16)pv[1], (_Float16)pv[2], (_Float16)pv[3],
                             (_Float16)pv[4], (_Float16)pv[5], (_Float16)pv[6], (_Float16)pv[7]};
            const unsigned char *vbase = ldsv + (8 * c + (i >> 2)) * kVRowBytes + (i & 3) * 8;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(v_operand(vbase, s, dt), Bp, O[dt], 0, 0, 0);
        }
        l_run += rows4_meet<false>(l);
    }
    if (!row_ok) return;
    // every row sees at least its own token, so l_run > 0; lane (row i, group c) holds dims 16 dt + 4 c + r
    const float inv = 1.0f / l_run;
    __half *dst = a.out + (size_t)tok * a.out_stride + (size_t)(q0 + hq) * 128;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
        __half2 *d2 = reinterpret_cast<__half2 *>(dst + 16 * dt + 4 * c);
        d2[0] = __half2{to_half(O[dt][0] * inv), to_half(O[dt][1] * inv)};
        d2[1] = __half2{to_half(O[dt][2] * inv), to_half(O[dt][3] * inv)};
    }
}

hipError_t launch_attn_chunk_onepass(const AttnChunkArgs &a, hipStream_t st) {
    if (a.nheads == 0 || a.ntok == 0) return hipSuccess;
    if (a.group == 0 || a.group > 16 || !a.out || !a.k_own || !a.v_own) return hipErrorInvalidValue;
    if (((uint64_t)a.ctx + kAttnPos) * 256u > 0x7FFFFFFFull || ((uint64_t)a.ntok + kAttnPos) * a.own_stride * 2u > 0x7FFFFFFFull) return hipErrorInvalidValue;
    dim3 grid(a.nheads, (a.ntok * a.group + 63) / 64);
    const size_t ldsb = (size_t)kAttnPos * (kVRowBytes + kKRowBytes);
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_chunk_onepass_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldsb);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(attn_chunk_onepass_kernel, grid, dim3(256), ldsb, st, a);
    return hipGetLastError();
}

// the tokens' K and V rows go to positions ctx .. ctx + ntok - 1 of each kv head's cache home
__global__ __launch_bounds__(128) void kv_append_rows_kernel(uint32_t ctx, uint32_t cap, const __half *qkv, uint32_t qkv_w, uint32_t n_q,
                                                             uint32_t n_kv, const uint64_t *home) {
    const uint32_t g = blockIdx.x, t = blockIdx.y, d = threadIdx.x;
    __half *Kh = reinterpret_cast<__half *>(home[g]);
    Kh[((size_t)ctx + t) * 128 + d] = qkv[(size_t)t * qkv_w + (size_t)(n_q + g) * 128 + d];
    Kh[((size_t)cap + ctx + t) * 128 + d] = qkv[(size_t)t * qkv_w + (size_t)(n_q + n_kv + g) * 128 + d];
}

hipError_t launch_kv_append_rows(uint32_t ctx, uint32_t cap, const __half *qkv, uint32_t qkv_w, uint32_t n_q, uint32_t n_kv, uint32_t ntok,
                                 const uint64_t *home, hipStream_t st) {
    if (ntok == 0) return hipSuccess;
    if (n_kv == 0 || (uint64_t)ctx + ntok > cap || ntok > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kv_append_rows_kernel, dim3(n_kv, ntok), dim3(128), 0, st, ctx, cap, qkv, qkv_w, n_q, n_kv, home);
    return hipGetLastError();
}

hipError_t launch_attn_chunk(const AttnChunkArgs &a_in, hipStream_t st) {
    AttnChunkArgs a = a_in;
    const uint32_t npos = a.causal ? a.ntok : a.ctx;
    if (npos == 0 || a.nheads == 0 || a.ntok == 0) return hipSuccess;
    if (a.group == 0 || a.group > 16) return hipErrorInvalidValue;
    if (a.ntok * a.group < 16) {
        // fewer score rows than one MFMA tile (a last chunk of one or two tokens): the vector-ALU form,
        // the tokens shared out over blockIdx.z.  Same records; which form runs depends on the token
        // count only, never on the placement.
        const uint32_t wg_xy = (npos + kAttnPos - 1) / kAttnPos * a.nheads;
        a.tok_per_wg = std::max(1u, (a.ntok + std::max(1u, 1024u / wg_xy) - 1) / std::max(1u, 1024u / wg_xy));
        dim3 gv((npos + kAttnPos - 1) / kAttnPos, a.nheads, (a.ntok + a.tok_per_wg - 1) / a.tok_per_wg);
        if (a.chunk0 + gv.x > a.chunk_cap || (uint64_t)npos * a.row_stride * 2u > 0x7FFFFFFFull) return hipErrorInvalidValue;
        switch (a.group) {
            case 1: hipLaunchKernelGGL(attn_chunk_kernel<1>, gv, dim3(kAttnWaves * 64), 0, st, a); break;
            case 2: hipLaunchKernelGGL(attn_chunk_kernel<2>, gv, dim3(kAttnWaves * 64), 0, st, a); break;
            case 4: hipLaunchKernelGGL(attn_chunk_kernel<4>, gv, dim3(kAttnWaves * 64), 0, st, a); break;
            case 8: hipLaunchKernelGGL(attn_chunk_kernel<8>, gv, dim3(kAttnWaves * 64), 0, st, a); break;
            default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    dim3 grid((npos + kAttnPos - 1) / kAttnPos, a.nheads, (a.ntok * a.group + 63) / 64);
    if (a.chunk0 + grid.x > a.chunk_cap) return hipErrorInvalidValue;
    if (((uint64_t)npos + kAttnPos) * a.row_stride * 2u > 0x7FFFFFFFull) return hipErrorInvalidValue;   // 32-bit buffer offsets
    const size_t ldsb = (size_t)kAttnPos * kVRowBytes;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_chunk_mfma_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldsb);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(attn_chunk_mfma_kernel, grid, dim3(256), ldsb, st, a);
    return hipGetLastError();
}

// One workgroup of 128 threads per (query head, token): thread d merges dimension d over the token's
// chunks in ascending order -- the cache's chunks below ctx, then the chunk's own rows up to the token
// itself -- writes the attention output row (the O projection's input) and, for the first query head
// of each kv group, appends the token's K and V rows at position ctx + t of that head's cache home.
__global__ __launch_bounds__(128) void attn_combine_chunk_kernel(const float *part, uint32_t chunk_cap, uint32_t ctx, uint32_t cap,
                                                                 const __half *qkv, uint32_t qkv_w, uint32_t n_q, uint32_t n_kv,
                                                                 const uint64_t *home, __half *out, uint32_t out_stride) {
    const uint32_t h = blockIdx.x, t = blockIdx.y, d = threadIdx.x;
    const uint32_t group = n_q / n_kv, g = h / group;
    const uint32_t nc_cache = (ctx + kAttnPos - 1) / kAttnPos, nc_own = t / kAttnPos + 1;
    const float *ph = part + ((size_t)t * n_q + h) * chunk_cap * 130;
    // the records are read eight (then four) chunks at a time, every load of a round requested before the first
    // is used (a chunk past the last re-reads the last one and is left out); the sums stay in chunk order
    const uint32_t nct = nc_cache + nc_own;
    float mx = -INFINITY;
    for (uint32_t c0 = 0; c0 < nct; c0 += 8) {
        float mv[8];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) mv[u] = ph[(size_t)min(c0 + u, nct - 1) * 130];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) mx = fmaxf(mx, mv[u]);
    }
    float L = 0.f, o = 0.f;
    for (uint32_t c0 = 0; c0 < nct; c0 += 4) {
        float mv[4], lv[4], ov[4];
#pragma unroll
        for (uint32_t u = 0; u < 4; ++u) {
            const float *pc = ph + (size_t)min(c0 + u, nct - 1) * 130;
            mv[u] = pc[0]; lv[u] = pc[1]; ov[u] = pc[2 + d];
        }
#pragma unroll
        for (uint32_t u = 0; u < 4; ++u) {
            if (c0 + u < nct) {
                const float w = __expf(mv[u] - mx);
                L = fmaf(w, lv[u], L);
                o = fmaf(w, ov[u], o);
            }
        }
    }
    out[(size_t)t * out_stride + (size_t)h * 128 + d] = to_half(o / L);
    if (h % group == 0) {
        __half *Kh = reinterpret_cast<__half *>(home[g]);
        Kh[((size_t)ctx + t) * 128 + d] = qkv[(size_t)t * qkv_w + (size_t)(n_q + g) * 128 + d];
        Kh[((size_t)cap + ctx + t) * 128 + d] = qkv[(size_t)t * qkv_w + (size_t)(n_q + n_kv + g) * 128 + d];
    }
}

hipError_t launch_attn_combine_chunk(const float *part, uint32_t chunk_cap, uint32_t ctx, uint32_t cap, const __half *qkv,
                                     uint32_t qkv_w, uint32_t n_q, uint32_t n_kv, uint32_t ntok, const uint64_t *home, __half *out,
                                     uint32_t out_stride, hipStream_t st) {
    if (ntok == 0) return hipSuccess;
    if (n_kv == 0 || n_q % n_kv || (uint64_t)ctx + ntok > cap || ntok > 65535) return hipErrorInvalidValue;
    if ((ctx + kAttnPos - 1) / kAttnPos + (ntok + kAttnPos - 1) / kAttnPos > chunk_cap) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_combine_chunk_kernel, dim3(n_q, ntok), dim3(128), 0, st, part, chunk_cap, ctx, cap, qkv, qkv_w, n_q, n_kv, home,
                       out, out_stride);
    return hipGetLastError();
}

__global__ void set_u32_kernel(uint32_t *dst, uint32_t v) { *dst = v; }

hipError_t launch_set_u32(uint32_t *dst, uint32_t v, hipStream_t st) {
    hipLaunchKernelGGL(set_u32_kernel, dim3(1), dim3(1), 0, st, dst, v);
    return hipGetLastError();
}

hipError_t launch_attn_decode(const AttnArgs &a, hipStream_t st) {
    if ((!a.ctx_dev && a.ctx == 0) || a.nheads == 0) return hipSuccess;
    // context read on the device: cover every chunk a cache of cap positions can hold (ctx < cap)
    const uint32_t span = a.ctx_dev ? a.cap - 1 : a.ctx;
    if (span == 0) return hipSuccess;
    dim3 grid((span + kAttnPos - 1) / kAttnPos, a.nheads);
    if (grid.x > a.chunk_cap) return hipErrorInvalidValue;
    switch (a.group) {
        case 1: hipLaunchKernelGGL(attn_decode_kernel<1>, grid, dim3(kAttnWaves * 64), 0, st, a); break;
        case 2: hipLaunchKernelGGL(attn_decode_kernel<2>, grid, dim3(kAttnWaves * 64), 0, st, a); break;
        case 4: hipLaunchKernelGGL(attn_decode_kernel<4>, grid, dim3(kAttnWaves * 64), 0, st, a); break;
        case 8: hipLaunchKernelGGL(attn_decode_kernel<8>, grid, dim3(kAttnWaves * 64), 0, st, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// one workgroup of 512 threads per query head.  The chunk maxima and weights are handled chunk-
// parallel (thread t takes chunks t, t + 512, ...); then four groups of 128 threads each sum one
// quarter of the chunks (thread d of a group owns dimension d, loads 16 at a time so none waits for
// an earlier one) and the four quarter sums meet in fixed order.
constexpr uint32_t kAttnMaxChunks = 8192;   // 1M positions

__device__ __forceinline__ float block512_reduce(float v, float *scratch, bool is_max) {
    v = is_max ? wave_max_all(v) : wave_sum(v);
    __syncthreads();                       // scratch may still be read from the previous reduction
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = scratch[0];
#pragma unroll
    for (int w = 1; w < 8; ++w) r = is_max ? fmaxf(r, scratch[w]) : r + scratch[w];
    return r;
}

__global__ __launch_bounds__(512) void attn_combine_kernel(const float *part, uint32_t chunk_cap, uint32_t ctx_arg,
                                                           const uint32_t *ctx_dev, uint32_t cap, const __half *qkv,
                                                           uint32_t n_q, uint32_t n_kv, const uint64_t *home, __half *out) {
    const uint32_t ctx = ctx_dev ? *ctx_dev : ctx_arg;
    __shared__ float scratch[8];
    __shared__ float wbuf[kAttnMaxChunks];
    __shared__ float osum[4][128];
    const uint32_t h = blockIdx.x, tid = threadIdx.x, d = tid & 127, grp = tid >> 7;
    const uint32_t group = n_q / n_kv, g = h / group;
    const uint32_t nchunks = (ctx + kAttnPos - 1) / kAttnPos;
    const float *ph = part + (size_t)h * chunk_cap * 130;
    // quarter q of the chunks: [q * per, min((q + 1) * per, nchunks))
    const uint32_t per = (nchunks + 3) / 4, c1 = min(nchunks, (grp + 1) * per);
    uint32_t c = min(nchunks, grp * per);
    // Everything that does not depend on a reduction is requested now, in one round trip: the
    // token's own rows, this thread's first chunk maximum and weight sum, and the first 16 partial
    // sums of its quarter (the partials were written by other XCDs a moment ago, so each dependent
    // read is a trip to the memory-side cache; the order of the arithmetic below is unchanged).
    const float kn = __half2float(qkv[(size_t)(n_q + g) * 128 + d]);
    const float vn = __half2float(qkv[(size_t)(n_q + n_kv + g) * 128 + d]);
    const float qd = grp == 0 ? __half2float(qkv[(size_t)h * 128 + d]) : 0.f;
    const bool mine = tid < nchunks, first16 = c + 16 <= c1;
    float m0 = 0.f, l0 = 0.f, v0[16];
    if (mine) { m0 = ph[(size_t)tid * 130]; l0 = ph[(size_t)tid * 130 + 1]; }
#pragma unroll
    for (int u = 0; u < 16; ++u) v0[u] = first16 ? ph[(size_t)(c + u) * 130 + 2 + d] : 0.f;
    // the token's own score (every group of 128 threads holds the 128 products once)
    const float s_self = block512_reduce(grp == 0 ? qd * kn : 0.f, scratch, false) * 0.08838834764831845f;
    float mloc = s_self;
    if (mine) mloc = fmaxf(mloc, m0);
    for (uint32_t cc = tid + 512; cc < nchunks; cc += 512) mloc = fmaxf(mloc, ph[(size_t)cc * 130]);
    const float mx = block512_reduce(mloc, scratch, true);
    float lloc = 0.f;
    if (mine) {
        const float w = __expf(m0 - mx);
        wbuf[tid] = w;
        lloc = fmaf(w, l0, lloc);
    }
    for (uint32_t cc = tid + 512; cc < nchunks; cc += 512) {
        const float w = __expf(ph[(size_t)cc * 130] - mx);
        wbuf[cc] = w;
        lloc = fmaf(w, ph[(size_t)cc * 130 + 1], lloc);
    }
    const float w_self = __expf(s_self - mx);
    const float L = block512_reduce(lloc, scratch, false) + w_self;   // also publishes wbuf
    float o = 0.f;
    if (first16) {
#pragma unroll
        for (int u = 0; u < 16; ++u) o = fmaf(wbuf[c + u], v0[u], o);
        c += 16;
    }
    for (; c + 16 <= c1; c += 16) {
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = ph[(size_t)(c + u) * 130 + 2 + d];
#pragma unroll
        for (int u = 0; u < 16; ++u) o = fmaf(wbuf[c + u], v[u], o);
    }
    for (; c < c1; ++c) o = fmaf(wbuf[c], ph[(size_t)c * 130 + 2 + d], o);
    osum[grp][d] = o;
    __syncthreads();
    if (grp != 0) return;
    o = fmaf(w_self, vn, ((osum[0][d] + osum[1][d]) + osum[2][d]) + osum[3][d]);
    out[(size_t)h * 128 + d] = to_half(o / L);
    if (h % group == 0) {   // append the token's rows to the cache home of kv head g
        __half *Kh = reinterpret_cast<__half *>(home[g]);
        Kh[(size_t)ctx * 128 + d] = qkv[(size_t)(n_q + g) * 128 + d];
        Kh[((size_t)cap + ctx) * 128 + d] = qkv[(size_t)(n_q + n_kv + g) * 128 + d];
    }
}

hipError_t launch_attn_combine(const float *part, uint32_t chunk_cap, uint32_t ctx, const uint32_t *ctx_dev, uint32_t cap,
                               const __half *qkv, uint32_t n_q, uint32_t n_kv, const uint64_t *home, __half *out, hipStream_t st) {
    // (with the context on the device the caller has checked it against cap; the chunk bound then goes by cap)
    const uint32_t span = ctx_dev ? cap - 1 : ctx;
    if (ctx >= cap || n_kv == 0 || n_q % n_kv || (span + kAttnPos - 1) / kAttnPos > kAttnMaxChunks) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_combine_kernel, dim3(n_q), dim3(512), 0, st, part, chunk_cap, ctx, ctx_dev, cap, qkv, n_q, n_kv, home, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// MoE combine: out[m] = h[m] + sum_j w[m][j] * y[m*top_k + j], j in rank order
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(const __half *h, const float *y, const float *w, uint32_t M,
                                                      uint32_t H, uint32_t top_k, int residual, __half *out) {
    const size_t n = (size_t)M * H;
    for (size_t q = (size_t)blockIdx.x * 256 + threadIdx.x; q < n; q += (size_t)gridDim.x * 256) {
        const uint32_t m = (uint32_t)(q / H), col = (uint32_t)(q % H);
        float s = 0.f;
        // eight experts' rows and weights are requested before the first is added (a rank past the last re-reads
        // the last one and is left out); the sum stays in rank order
        for (uint32_t j0 = 0; j0 < top_k; j0 += 8) {
            float wv[8], yv[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                const size_t pr = (size_t)m * top_k + min(j0 + u, top_k - 1);
                wv[u] = w[pr];
                yv[u] = y[pr * H + col];
            }
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u)
                if (j0 + u < top_k) s += wv[u] * yv[u];
        }
        out[q] = __float2half((residual ? __half2float(h[q]) : 0.f) + s);
    }
}

hipError_t launch_combine(const __half *h, const float *y, const float *w, uint32_t M, uint32_t H, uint32_t top_k,
                          int residual, __half *out, hipStream_t st) {
    const size_t n = (size_t)M * H;
    const size_t want = (n + 255) / 256;
    const uint32_t blocks = (uint32_t)(want < 4096 ? want : 4096);
    hipLaunchKernelGGL(combine_kernel, dim3(blocks), dim3(256), 0, st, h, y, w, M, H, top_k, residual, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Prefill / batched-decode kernel: 4-bit dequant GEMM on the matrix cores.
// v_mfma_f32_16x16x32_f16: A = weights (16 rows x 32 k), B = activations (32 k x 16 tokens).
// A lane's 16 weight bytes are four A operands as they sit in memory: lane (i, c) holds
// block 4*sb + c of row i, dword kk supplies k-slots c*8 .. c*8+7 of MFMA step kk, which
// this kernel maps to k = 32*(4*sb + c) + 8*kk + t; the B operand follows the same map.
// Scales are folded into the fp16 A operand ((q - 8) * d rounded to fp16).
// NW waves (4, or 8 for the many-token shape), each wave owns AT row-tiles and all MT tokens of
// the workgroup; the activation tile of one super-block (MT x 128 k) is staged in LDS, 16-byte
// chunks XOR-swizzled by token so that operand reads are conflict-free.
// ------------------------------------------------------------------------------------
// LDS column of activation chunk u (k = 8u .. 8u+7 of a super-block) within its token's 16-chunk
// row, before the XOR with the token index: MFMA step kk of lane group c consumes chunk 4c + kk,
// kept at column c + 4kk so that the four lane groups of one read touch adjacent columns (measured:
// the 4c + kk order costs 1.5x the LDS cycles of this one)
__device__ __forceinline__ uint32_t lds_col(uint32_t u) { return ((u & 3) << 2) | (u >> 2); }

// super-blocks of lookahead of the GEMM's prefetch ring (see the kernel): 2 for the few-token tiles;
// the 8-wave workgroup (one per CU, its activation stages shared by twice the row-tiles) has the
// LDS for 3
constexpr int gemm_depth(int MT, int NW = 4) { return NW == 8 ? 3 : MT <= 64 ? 2 : 1; }
// LDS of a workgroup: the activation stages, then per wave two scale buffers of 1 KB per row-tile
constexpr size_t gemm_lds_bytes(int MT, int AT, int NW) { return (size_t)MT * 256 * (gemm_depth(MT, NW) + 1) + (size_t)NW * 2 * AT * 1024; }

template <int MODE, int AT, int MT, bool GROUPED, int NW = 4>
__global__ __launch_bounds__(NW * 64, NW == 8 ? 1 : 2) void gemm_w4_kernel(GemmArgs a) {
    extern __shared__ uint4 lds[];                 // gemm_depth(MT, NW) + 1 stages of MT x 16 chunks, then 2 AT KB of scales per wave
    constexpr int NMT = MT / 16;
    constexpr int NFILL = MT / (4 * NW);           // 16-byte chunks each thread moves per stage
    static_assert(MT % (4 * NW) == 0, "a fill round covers 4 * NW tokens");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, c = lane >> 4;

    const uint4 *W = a.W;
    uint32_t ntok = a.M;           // tokens this workgroup column may touch
    const int32_t *pairs = nullptr;
    if (GROUPED) {
        const DeviceTask t = a.tasks[blockIdx.z];
        W = reinterpret_cast<const uint4 *>(MODE == GEMM_GATE_UP ? t.w_gate_up : t.w_down);
        ntok = t.npairs;
        pairs = a.pairs + t.pair0;
    }
    const uint32_t m0 = blockIdx.y * MT;
    if (m0 >= ntok) return;
    const uint32_t tile_base = (blockIdx.x * NW + wave) * AT;

    // activation fill, global memory straight into LDS (buffer_load ... lds): round r of a wave
    // writes 64 consecutive 16-byte slots, i.e. thread tid fills slot tid & 15 of token
    // tok0 + 4 NW r, tok0 = tid >> 4, and therefore fetches the chunk that belongs there,
    // u = lds_col(slot ^ (tok0 & 15)) (lds_col is its own inverse).
    // xoff: byte offset of that chunk in the token's row (grouped launches look the row up);
    // tokens past the end re-read the last valid row: their MFMA columns are never stored, and the
    // fill needs neither a branch nor zeros.  Addresses are a uniform base plus these 32-bit
    // offsets, so the loop does no 64-bit vector arithmetic.
    const uint32_t tok0 = tid >> 4, u = lds_col((tid & 15) ^ (tok0 & 15));
    uint32_t xoff[NFILL];
#pragma unroll
    for (int r = 0; r < NFILL; ++r) {
        const uint32_t tok = min(m0 + tok0 + r * (4 * NW), ntok - 1);
        size_t rowi = tok;
        if (GROUPED) rowi = (MODE == GEMM_GATE_UP) ? (size_t)(pairs[tok] / (int32_t)a.top_k) : (size_t)pairs[tok];
        xoff[r] = (uint32_t)((rowi * a.x_stride + u * 8) * sizeof(__half));
    }
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    // weights: 32-bit byte offset of the lane's 16 bytes in its tiles' first super-block; tiles past
    // the slab read tile 0 (discarded)
    uint32_t woff[AT];
#pragma unroll
    for (int t = 0; t < AT; ++t) {
        const uint32_t tile = tile_base + t < a.ntiles ? tile_base + t : 0;
        woff[t] = (tile * a.tile_u4 + lane) * 16u;
    }
    // buffer addressing: uniform part of an address in a scalar offset, lane part in xoff / woff
    const __amdgpu_buffer_rsrc_t xbuf = make_rsrc(a.x), wbuf = make_rsrc(W);

    f4_t acc[AT][NMT];
#pragma unroll
    for (int t = 0; t < AT; ++t)
#pragma unroll
        for (int n = 0; n < NMT; ++n) acc[t][n] = f4_t{0.f, 0.f, 0.f, 0.f};

    // Prefetch ring: DEPTH super-blocks are in flight ahead of the one being multiplied, in R =
    // DEPTH + 1 weight register sets and LDS stages.  With few tokens an iteration is shorter than
    // the memory latency, so one super-block of lookahead leaves the loop waiting on its loads.
    constexpr int DEPTH = gemm_depth(MT, NW), R = DEPTH + 1;
    static_assert(AT <= 2, "the dequantisation is pipelined one MFMA step ahead; more tiles per wave do not fit the registers");
    constexpr int LPI = NFILL + AT;              // loads every prefetch issues per lane (scale fills, when it has them: AT more)
    // one super-block of weights of the wave's tiles: the lane's 16 code bytes
    struct Wset { uint4 q[AT]; };
    Wset wr[R];
    // The fp16 scales come once per scale group (8 super-blocks), not once per super-block: a lane's
    // 16 bytes of a group's scale area hold the scales of its block column for all 8 super-blocks,
    // and they go from global memory straight into a wave-private LDS window (two buffers per tile,
    // by group parity), from where each step picks the two bytes it needs.  (One 4-byte load per
    // super-block instead touched the same eight cache lines eight times over, between which the
    // activation fills had pushed them out of the vector cache: a timing probe without scale loads
    // ran the 64-token gate/up launch 14 % faster.)  Like the activation fills these loads are not
    // register writes the compiler could wait for; the counted waits below cover them.
    uint4 *const sc_lds = lds + R * (MT * 16) + __builtin_amdgcn_readfirstlane(wave) * (2 * AT * 64);
    auto fill_x = [&](uint32_t sb, uint32_t stage) {
        // (wave-uniform; said so explicitly, or the fill's scalar offset is taken in a lane loop)
        const uint32_t xs = __builtin_amdgcn_readfirstlane(gather_col(sb * 128, a.x_off, a.x_group) * (uint32_t)sizeof(__half));
#pragma unroll
        for (int r = 0; r < NFILL; ++r)
            load_to_lds16(xbuf, (lds_void *)(lds + stage * (MT * 16) + r * (NW * 64) + wave_u * 64), xoff[r], xs);
    };

    // scale group / slot of super-block sb, clamped to the last one (a prefetch past the end
    // re-reads the last super-block instead of branching; nothing consumes it)
    auto load_w = [&](uint32_t sbn, Wset &w) {
        sbn = min(sbn, a.nsb - 1);
        const uint32_t gn = sbn >> 3, sn = sbn & 7;
        const uint32_t gb = gn * (9 * 1024);
#pragma unroll
        for (int t = 0; t < AT; ++t)
            w.q[t] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(wbuf, woff[t], gb + sn * 1024, kAuxNt));
    };
    // scale area of group g of the wave's tiles -> the window's buffer of parity g & 1
    auto fill_scales = [&](uint32_t g) {
        const uint32_t so = g * (9 * 1024) + min(8u, a.nsb - g * 8u) * 1024;
#pragma unroll
        for (int t = 0; t < AT; ++t) load_to_lds16(wbuf, (lds_void *)(sc_lds + ((g & 1) * AT + t) * 64), woff[t], so);
    };
    // the scales the next dequantisation uses (dsc): the lane's fp16 number sbx & 7 of its group
    uint32_t dsc[AT];
    auto scales_of = [&](uint32_t sbx) {
        const uint32_t g = sbx >> 3, sn = sbx & 7;
#pragma unroll
        for (int t = 0; t < AT; ++t)
            dsc[t] = *reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(sc_lds + ((g & 1) * AT + t) * 64) + lane * 16 + sn * 2);
    };
    // prefetched weights become visible to the compiler only where this is called, so nothing
    // derived from them is scheduled (and waited for) earlier
    auto arrive_w = [&](Wset &w) {
#pragma unroll
        for (int t = 0; t < AT; ++t) {
            // (an empty statement the compiler cannot see through: no instruction is issued)
            asm volatile("" : "+v"(w.q[t].x), "+v"(w.q[t].y), "+v"(w.q[t].z), "+v"(w.q[t].w));
        }
    };
    // A operands of MFMA step kk from raw dwords + scale: (q - 8) * d rounded to fp16
    auto dequant_a = [&](h8_t (&A)[AT], const Wset &ws, int kk) {
#pragma unroll
        for (int t = 0; t < AT; ++t) {
            const uint32_t q = kk == 0 ? ws.q[t].x : kk == 1 ? ws.q[t].y : kk == 2 ? ws.q[t].z : ws.q[t].w;
            const _Float16 d = __builtin_bit_cast(_Float16, (uint16_t)dsc[t]);
            const h2_t dd = {d, d};
            h2_t w[4];
            dequant8(q, w);
            w[0] *= dd; w[1] *= dd; w[2] *= dd; w[3] *= dd;
            A[t] = h8_t{w[0].x, w[0].y, w[1].x, w[1].y, w[2].x, w[2].y, w[3].x, w[3].y};
        }
    };

    // One prefetch = the stage's NFILL LDS fills, THEN the 2 AT weight loads, in that order in the
    // instruction stream: the hand-counted waits below rely on it (loads complete in issue order, so
    // "all but the newest n" is a statement about which loads have landed).  The fence keeps the
    // compiler from moving the weight loads, which depend on nothing, above fills whose addresses do
    // (in grouped launches the fill offsets come from a load of the pair list).
    // Scale fills come first of all.  A group's scales travel with the prefetch of the super-block
    // BEFORE the group (the dequantisation of a step's first operands runs at the end of the step
    // before, ahead of the wait that covers the step's own prefetch), and with the walk's opening
    // prefetch (FIRST) for the group it starts in.  The buffer they overwrite was last read nine
    // steps earlier.
    auto prefetch = [&](uint32_t sb_fill, uint32_t stage, uint32_t sb_w, Wset &w, auto FIRST) {
        const uint32_t sbc = min(sb_w, a.nsb - 1);
        if constexpr (decltype(FIRST)::value) fill_scales(sbc >> 3);
        if ((sbc & 7) == 7 && sbc + 1 < a.nsb) fill_scales((sbc >> 3) + 1);
        fill_x(sb_fill, stage);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        load_w(sb_w, w);
    };

    // split-K: this workgroup covers super-blocks [sb_begin, sb_end) and writes an fp32 partial plane
    uint32_t sb_begin = 0, sb_end = a.nsb;
    if (!GROUPED && a.sb_per_part) {
        sb_begin = blockIdx.z * a.sb_per_part;
        sb_end = min(a.nsb, sb_begin + a.sb_per_part);
    }
    prefetch(sb_begin, 0, sb_begin, wr[0], std::true_type{});
#pragma unroll
    for (int d = 1; d < DEPTH; ++d) prefetch(min(sb_begin + d, sb_end - 1), d, sb_begin + d, wr[d], std::false_type{});
    // the A operands of the next MFMA step are dequantised while this step's MFMAs run
    h8_t Acur[AT], Anxt[AT];
    arrive_w(wr[0]);
    // EARLY (three or more super-blocks of lookahead): a stage is required one step before it is
    // multiplied, so the barrier that ends step sb already covers the fills of stage sb + 2.  A wave
    // can then fetch the first B operands of step sb + 1 while step sb's last MFMAs run, instead
    // of every wave of the workgroup meeting the LDS latency together right after the barrier.
    constexpr bool EARLY = DEPTH >= 3;
    constexpr int kLand = EARLY ? DEPTH - 2 : DEPTH - 1;   // prefetches that may still be in flight at a barrier
    // a prefetch issues its LDS fills before its weight loads and loads return in order, so the
    // barrier of the EARLY shape needs only the fills of the stage it covers: that stage's weight
    // loads (from HBM, the slow ones; consumed a step later) may stay in flight as well
    // (counted without the scale fills that one prefetch in eight carries: with one of those among
    // the newest the wait asks for a little more than it needs, never for less)
    constexpr int kInFlight = kLand * LPI + (EARLY ? AT : 0);
    // Before the first step: everything issued so far has landed.  No count is assumed here, because
    // nothing orders the DEPTH opening prefetches among themselves: the compiler hoists the weight
    // loads of all of them above fills that wait for the pair list, and merges the scale loads of two
    // super-blocks that share a dword, so "all but the newest kInFlight" would not name the fills of
    // stage 0 (a build in which it happened not to gave wrong results now and then).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    scales_of(sb_begin);
    dequant_a(Acur, wr[0], 0);
    h8_t Bc[NMT], Bn[NMT];
    if (EARLY) {
#pragma unroll
        for (int n = 0; n < NMT; ++n) Bc[n] = __builtin_bit_cast(h8_t, lds[i * 16 + n * 256 + (c ^ i)]);
    }

    // one super-block: U = its position in the ring (compile-time, so every register set and LDS
    // stage below is addressed statically and nothing is copied when the ring turns)
    // TAIL: one of the at most R - 1 steps after the last whole turn of the ring.  What they would
    // prefetch lies past the end of the walk, so they issue nothing and wait for everything.
    auto step = [&](uint32_t sb, auto U, auto TAIL) {
        constexpr int u = decltype(U)::value;
        constexpr bool tail = decltype(TAIL)::value;
        constexpr int un = (u + 1) % R, up = (u + DEPTH) % R;   // next super-block's slot, the slot to refill
        // prefetch super-block sb + DEPTH: activations into the stage every wave left at the
        // barrier that ended the previous step, weights into the register set used then
        if (!tail) prefetch(min(sb + DEPTH, sb_end - 1), up, sb + DEPTH, wr[up], std::false_type{});
        __builtin_amdgcn_sched_barrier(0);   // keep the prefetch up here: its latency hides behind the MFMAs
        const uint4 *ls = lds + u * (MT * 16) + i * 16;   // + n * 256: token n*16 + i
        const uint4 *lsn = lds + un * (MT * 16) + i * 16;  // the next super-block's stage
        // B operands are read one MFMA step ahead, so the LDS latency hides behind a step's MFMAs
        if (!EARLY) {
#pragma unroll
            for (int n = 0; n < NMT; ++n) Bc[n] = __builtin_bit_cast(h8_t, ls[n * 256 + (c ^ i)]);
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk < 3) {
#pragma unroll
                for (int n = 0; n < NMT; ++n) Bn[n] = __builtin_bit_cast(h8_t, ls[n * 256 + ((c + (kk + 1) * 4) ^ i)]);
                __builtin_amdgcn_sched_barrier(0);   // or the scheduler sinks each read next to its MFMA
            } else if (EARLY) {
#pragma unroll
                for (int n = 0; n < NMT; ++n) Bn[n] = __builtin_bit_cast(h8_t, lsn[n * 256 + (c ^ i)]);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kk < 3) dequant_a(Anxt, wr[u], kk + 1);
            else {
                arrive_w(wr[un]);
                scales_of(sb + 1);
                dequant_a(Anxt, wr[un], 0);
            }
#pragma unroll
            for (int n = 0; n < NMT; ++n) {
#pragma unroll
                for (int t = 0; t < AT; ++t)
                    acc[t][n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(Acur[t], Bc[n], acc[t][n], 0, 0, 0);
            }
#pragma unroll
            for (int t = 0; t < AT; ++t) Acur[t] = Anxt[t];
            if (kk < 3 || EARLY) {
#pragma unroll
                for (int n = 0; n < NMT; ++n) Bc[n] = Bn[n];
            }
        }
        // super-block sb + 1's activations have landed once all but the later prefetches are done.
        // A bare barrier: __syncthreads() carries a fence that makes the compiler wait for EVERY
        // LDS-direct load in flight, i.e. also for the deeper prefetches.  What must be ordered
        // here is ordered by hand: this wave's fill of the next stage is complete (vmcnt), and
        // its LDS reads of the current stage, which the next step's fill overwrites, have
        // returned (lgkmcnt).
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(tail ? 0 : kInFlight) : "memory");
        __builtin_amdgcn_s_barrier();
    };
    // whole turns of the ring, then the remaining steps (no exit from inside a turn: the ring is back
    // in phase at the loop's back edge, so no register set is live across it in another slot)
    uint32_t sb = sb_begin;
    for (; sb + R <= sb_end; sb += R) {
        step(sb, std::integral_constant<int, 0>{}, std::false_type{});
        step(sb + 1, std::integral_constant<int, 1>{}, std::false_type{});
        if constexpr (R > 2) step(sb + 2, std::integral_constant<int, 2>{}, std::false_type{});
        if constexpr (R > 3) step(sb + 3, std::integral_constant<int, 3>{}, std::false_type{});
    }
    if (sb < sb_end) step(sb, std::integral_constant<int, 0>{}, std::true_type{});
    if constexpr (R > 2) {
        if (sb + 1 < sb_end) step(sb + 1, std::integral_constant<int, 1>{}, std::true_type{});
    }
    if constexpr (R > 3) {
        if (sb + 2 < sb_end) step(sb + 2, std::integral_constant<int, 2>{}, std::true_type{});
    }

    // epilogue: lane holds token j = lane & 15 of each token tile and rows 4*(lane >> 4) + r
    const int j = lane & 15, rg = lane >> 4;
#pragma unroll
    for (int n = 0; n < NMT; ++n) {
        const uint32_t tok = m0 + n * 16 + j;
        if (tok >= ntok) continue;
        size_t orow = tok;           // output row
        size_t xrow = tok;           // row of rinv / residual
        if (pairs) { orow = (size_t)pairs[tok]; xrow = orow / a.top_k; }
        if (MODE == GEMM_GATE_UP) {
            const float rinv = a.rinv[xrow];
#pragma unroll
            for (int t = 0; t < AT; t += 2) {
                if (tile_base + t >= a.ntiles) continue;
                const uint32_t col = a.out_row0 + ((tile_base + t) >> 1) * 16 + rg * 4;
                __half2 o01 = __floats2half2_rn(silu(rinv * acc[t][n][0]) * (rinv * acc[t + 1][n][0]),
                                               silu(rinv * acc[t][n][1]) * (rinv * acc[t + 1][n][1]));
                __half2 o23 = __floats2half2_rn(silu(rinv * acc[t][n][2]) * (rinv * acc[t + 1][n][2]),
                                               silu(rinv * acc[t][n][3]) * (rinv * acc[t + 1][n][3]));
                __half2 *dst = reinterpret_cast<__half2 *>(a.out + orow * a.out_stride + col);
                dst[0] = o01; dst[1] = o23;
            }
        } else {
#pragma unroll
            for (int t = 0; t < AT; ++t) {
                if (tile_base + t >= a.ntiles) continue;
                const uint32_t col = a.out_row0 + (tile_base + t) * 16 + rg * 4;
                if (MODE == GEMM_F32) {
                    float *plane = a.out_f32 + ((!GROUPED && a.sb_per_part) ? (size_t)blockIdx.z * a.part_stride : 0);
                    float4 *dst = reinterpret_cast<float4 *>(plane + orow * a.out_stride + col);
                    *dst = make_float4(acc[t][n][0], acc[t][n][1], acc[t][n][2], acc[t][n][3]);
                } else {
                    float v[4];
                    if (MODE == GEMM_PLAIN) {
                        const float rinv = a.rinv[xrow];
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = rinv * acc[t][n][r];
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = acc[t][n][r];
                        if (a.res) {
                            const __half2 *rs = reinterpret_cast<const __half2 *>(a.res + orow * a.out_stride + col);
                            const float2 r01 = __half22float2(rs[0]), r23 = __half22float2(rs[1]);
                            v[0] += r01.x; v[1] += r01.y; v[2] += r23.x; v[3] += r23.y;
                        }
                    }
                    __half2 *dst = reinterpret_cast<__half2 *>(a.out + orow * a.out_stride + col);
                    dst[0] = __floats2half2_rn(v[0], v[1]);
                    dst[1] = __floats2half2_rn(v[2], v[3]);
                }
            }
        }
    }
}

template <int MODE, int AT, int MT>
static hipError_t launch_gemm_t(const GemmArgs &a, uint32_t ntasks, uint32_t max_tok, hipStream_t st) {
    const uint32_t parts = (!ntasks && a.sb_per_part) ? (a.nsb + a.sb_per_part - 1) / a.sb_per_part : 1;
    if constexpr (MT == 128) {
        // Many-token launches of a whole matrix or slab: 8 waves per workgroup, one workgroup per CU.
        // Its activation stages serve twice the row-tiles, which leaves LDS for three super-blocks of
        // lookahead instead of one (measured: gate/up and down +10 %, O +6 %).  Both shapes multiply
        // in the same order, so the choice never changes a result; it goes by how evenly each
        // shape's workgroups fill the 256 CUs (a 6144-row QKV fills 1.5 rounds either way and runs
        // 8 % slower in the wide shape).
        const uint32_t ty = (max_tok + MT - 1) / MT;
        const uint32_t wg8 = (a.ntiles + 8 * AT - 1) / (8 * AT) * ty, wg4 = (a.ntiles + 4 * AT - 1) / (4 * AT) * ty;
        const double eff8 = (double)wg8 / ((wg8 + 255) / 256 * 256), eff4 = (double)wg4 / ((wg4 + 511) / 512 * 512);
        if (!ntasks && parts == 1 && (eff8 >= 0.9 || eff8 > eff4 + 0.05)) {
            dim3 grid8((a.ntiles + 8 * AT - 1) / (8 * AT), ty, 1);
            const size_t lds8 = gemm_lds_bytes(MT, AT, 8);
            static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_w4_kernel<MODE, AT, MT, false, 8>),
                                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds8);
            if (attr != hipSuccess) return attr;
            hipLaunchKernelGGL((gemm_w4_kernel<MODE, AT, MT, false, 8>), grid8, dim3(512), lds8, st, a);
            return hipGetLastError();
        }
    }
    dim3 grid((a.ntiles + 4 * AT - 1) / (4 * AT), (max_tok + MT - 1) / MT, ntasks ? ntasks : parts);
    const size_t lds = gemm_lds_bytes(MT, AT, 4);
    if (lds > 64 * 1024) {
        static const hipError_t attr_g = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_w4_kernel<MODE, AT, MT, true>),
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        static const hipError_t attr_u = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_w4_kernel<MODE, AT, MT, false>),
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (attr_g != hipSuccess) return attr_g;
        if (attr_u != hipSuccess) return attr_u;
    }
    if (ntasks) hipLaunchKernelGGL((gemm_w4_kernel<MODE, AT, MT, true>), grid, dim3(256), lds, st, a);
    else hipLaunchKernelGGL((gemm_w4_kernel<MODE, AT, MT, false>), grid, dim3(256), lds, st, a);
    return hipGetLastError();
}

template <int MODE>
static hipError_t launch_gemm_m(const GemmArgs &a, uint32_t ntasks, uint32_t max_tok, hipStream_t st) {
    if (max_tok <= 16) return launch_gemm_t<MODE, 2, 16>(a, ntasks, max_tok, st);
    if (max_tok <= 32) return launch_gemm_t<MODE, 2, 32>(a, ntasks, max_tok, st);
    if (max_tok <= 64) return launch_gemm_t<MODE, 2, 64>(a, ntasks, max_tok, st);
    // A few hundred tokens on a narrow matrix (O and down at 512 tokens: 32 eight-tile workgroups x 4 token
    // tiles) leave half the CUs without a workgroup in 128-token tiles: 64-token tiles double the workgroups.
    // The tile shape goes by the whole matrix and the plan's token count, never by the slab, and every shape
    // adds a row's super-blocks in the same order, so the choice does not change a bit of the result.
    // (measured on the 8B shapes over a 4K cache, per layer: 256 tokens 387 -> 296 us, 512 tokens 462 -> 409 us,
    // 1024 tokens 714 -> 697 us; from 1.5 workgroups per CU on, the 128-token tile is the faster one)
    if (!ntasks && (a.total_tiles + 7) / 8 * ((max_tok + 127) / 128) < 384) return launch_gemm_t<MODE, 2, 64>(a, ntasks, max_tok, st);
    // 2 row-tiles per wave leave room for the pipelined dequant at two workgroups per CU; the
    // 4-tile shape (half the LDS operand traffic) does not fit that register budget
    return launch_gemm_t<MODE, 2, 128>(a, ntasks, max_tok, st);
}

hipError_t launch_gemm(int mode, const GemmArgs &a, uint32_t ntasks, uint32_t max_tok, hipStream_t st) {
    // the kernel addresses weights and activations as a uniform base plus 32-bit byte offsets
    if ((uint64_t)a.ntiles * a.tile_u4 * 16u > 0xFFFFFFFFull || (uint64_t)a.M * (a.top_k ? a.top_k : 1u) * a.x_stride * 2u > 0xFFFFFFFFull)
        return hipErrorInvalidValue;
    switch (mode) {
        case GEMM_PLAIN: return launch_gemm_m<GEMM_PLAIN>(a, ntasks, max_tok, st);
        case GEMM_RESID: return launch_gemm_m<GEMM_RESID>(a, ntasks, max_tok, st);
        case GEMM_GATE_UP: return launch_gemm_m<GEMM_GATE_UP>(a, ntasks, max_tok, st);
        case GEMM_F32: return launch_gemm_m<GEMM_F32>(a, ntasks, max_tok, st);
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------
// Gathered host->device copy.  A fixed, small number of workgroups walks every shard of the list in
// turn, each taking its share of every shard in 16-byte units (a wave moves 1 KB contiguous per
// load), eight loads per thread in flight.
// ------------------------------------------------------------------------------------
constexpr uint32_t kGatherDescs = 128;   // descriptors staged in LDS at a time
constexpr uint32_t kGatherWgs = 16;
constexpr uint32_t kLdsPerCu = 160 * 1024;   // gfx950
__global__ __launch_bounds__(256) void h2d_gather_kernel(const CopyDesc *descs, uint32_t n) {
    __shared__ CopyDesc sd[kGatherDescs];
    // The rest of the CU's LDS is claimed and left unused: no workgroup that needs LDS (every
    // matmul and attention kernel does) can then be placed on this CU, where its loads would
    // queue behind half a megabyte of PCIe reads on the CU's one vector-memory path (a one-token
    // matmul beside a gather: 45 us without the claim, 25 us with it, 13 us alone).
    __shared__ uint8_t rest[kLdsPerCu - sizeof(CopyDesc) * kGatherDescs];
    asm volatile("" ::"v"(&rest[threadIdx.x]));
    const uint32_t stride = gridDim.x * 256;
    for (uint32_t base = 0; base < n; base += kGatherDescs) {
        const uint32_t m = min(kGatherDescs, n - base);
        __syncthreads();
        // the list may sit in pinned host memory: one round trip over PCIe for the whole chunk
        if (threadIdx.x < m) sd[threadIdx.x] = descs[base + threadIdx.x];
        __syncthreads();
        for (uint32_t e = 0; e < m; ++e) {
            const u4_t *src = reinterpret_cast<const u4_t *>(sd[e].src);
            u4_t *dst = reinterpret_cast<u4_t *>(sd[e].dst);
            const uint32_t n16 = sd[e].n16;
            if (n16 == 0) continue;
            // past the end a load re-reads the last unit and its store is skipped, so the last pass
            // keeps eight loads in flight like the others
            for (uint32_t idx = blockIdx.x * 256 + threadIdx.x; idx < n16; idx += 8 * stride) {
                u4_t v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + min(idx + u * stride, n16 - 1));
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (idx + u * stride < n16) dst[idx + u * stride] = v[u];
            }
        }
    }
}

hipError_t launch_h2d_gather(const CopyDesc *descs, uint32_t n, hipStream_t st) {
    if (n == 0) return hipSuccess;
    // 16 workgroups keep 512 KB of reads in flight, which fills the PCIe link; more only queue up
    // ahead of the compute stream's reads from HBM
    hipLaunchKernelGGL(h2d_gather_kernel, dim3(kGatherWgs), dim3(256), 0, st, descs, n);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Rows computed on the host (experts run by the CPU back-end) land in one contiguous upload;
// this puts each where the combine step expects it: dst row idx[r] = src row r.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void scatter_rows_kernel(const float *src, const int32_t *idx, uint32_t H, float *dst) {
    const float4 *s4 = reinterpret_cast<const float4 *>(src + (size_t)blockIdx.x * H);
    float4 *d4 = reinterpret_cast<float4 *>(dst + (size_t)idx[blockIdx.x] * H);
    for (uint32_t j = threadIdx.x; j < H / 4; j += 256) d4[j] = s4[j];
}

hipError_t launch_scatter_rows(const float *src, const int32_t *idx, uint32_t n, uint32_t H, float *dst, hipStream_t st) {
    if (n == 0) return hipSuccess;
    if (H % 4) return hipErrorInvalidValue;
    hipLaunchKernelGGL(scatter_rows_kernel, dim3(n), dim3(256), 0, st, src, idx, H, dst);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Split-K epilogue (batched decode): out = epilogue(sum over parts, ascending, of the fp32
// partial planes).  One thread per output element; GATE_UP pairs a gate column with the up
// column 16 physical columns further on.
// ------------------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void splitk_epilogue_kernel(const float *partial, uint32_t parts, uint32_t part_stride,
                                                              uint32_t M, uint32_t ncols_phys, const float *rinv,
                                                              const __half *res, __half *out, uint32_t out_stride,
                                                              uint32_t out_row0) {
    // one thread per four adjacent output columns (a 16-column tile is never straddled)
    const uint32_t ncols = MODE == GEMM_GATE_UP ? ncols_phys / 2 : ncols_phys;
    const uint32_t nq = ncols / 4;
    const size_t n = (size_t)M * nq;
    for (size_t q = (size_t)blockIdx.x * 256 + threadIdx.x; q < n; q += (size_t)gridDim.x * 256) {
        const uint32_t m = (uint32_t)(q / nq), j = (uint32_t)(q % nq) * 4;
        const uint32_t c0 = MODE == GEMM_GATE_UP ? (j >> 4) * 32 + (j & 15) : j;
        const float *p0 = partial + (size_t)m * ncols_phys + c0;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f), u = v;
        // all planes are requested before the first is added (a plane past the last re-reads the last one and
        // is left out of the sum): one round trip to memory instead of one per plane; the sum stays in plane order
        float4 pa[8], pb[8];
#pragma unroll
        for (uint32_t p = 0; p < 8; ++p) {
            const size_t off = (size_t)min(p, parts - 1) * part_stride;
            pa[p] = *reinterpret_cast<const float4 *>(p0 + off);
            if (MODE == GEMM_GATE_UP) pb[p] = *reinterpret_cast<const float4 *>(p0 + off + 16);
        }
#pragma unroll
        for (uint32_t p = 0; p < 8; ++p) {
            if (p < parts) {
                v.x += pa[p].x; v.y += pa[p].y; v.z += pa[p].z; v.w += pa[p].w;
                if (MODE == GEMM_GATE_UP) { u.x += pb[p].x; u.y += pb[p].y; u.z += pb[p].z; u.w += pb[p].w; }
            }
        }
        float r[4] = {v.x, v.y, v.z, v.w};
        if (MODE == GEMM_PLAIN) {
            const float ri = rinv[m];
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = ri * r[e];
        } else if (MODE == GEMM_RESID) {
            if (res) {
                const __half2 *rs = reinterpret_cast<const __half2 *>(res + (size_t)m * out_stride + out_row0 + j);
                const float2 r01 = __half22float2(rs[0]), r23 = __half22float2(rs[1]);
                r[0] = r01.x + r[0]; r[1] = r01.y + r[1]; r[2] = r23.x + r[2]; r[3] = r23.y + r[3];
            }
        } else {
            const float ri = rinv[m];
            const float g[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = silu(ri * r[e]) * (ri * g[e]);
        }
        __half2 *d2 = reinterpret_cast<__half2 *>(out + (size_t)m * out_stride + out_row0 + j);
        d2[0] = __half2{to_half(r[0]), to_half(r[1])};
        d2[1] = __half2{to_half(r[2]), to_half(r[3])};
    }
}

hipError_t launch_splitk_epilogue(int mode, const float *partial, uint32_t parts, uint32_t part_stride, uint32_t M,
                                  uint32_t ncols_phys, const float *rinv, const __half *res, __half *out,
                                  uint32_t out_stride, uint32_t out_row0, hipStream_t st) {
    // four columns per thread: 16-byte plane reads, 8-byte stores (columns come in tiles of 16 and
    // out_row0 / out_stride are multiples of 16, so both stay aligned)
    if (ncols_phys % 16 || out_row0 % 4 || out_stride % 4 || part_stride % 4 || parts < 1 || parts > 8) return hipErrorInvalidValue;
    const size_t n = (size_t)M * (ncols_phys / 4);
    const uint32_t blocks = (uint32_t)std::min<size_t>((n + 255) / 256, 2048);
    switch (mode) {
        case GEMM_PLAIN:
            hipLaunchKernelGGL(splitk_epilogue_kernel<GEMM_PLAIN>, dim3(blocks), dim3(256), 0, st, partial, parts, part_stride, M, ncols_phys, rinv, res, out, out_stride, out_row0);
            break;
        case GEMM_RESID:
            hipLaunchKernelGGL(splitk_epilogue_kernel<GEMM_RESID>, dim3(blocks), dim3(256), 0, st, partial, parts, part_stride, M, ncols_phys, rinv, res, out, out_stride, out_row0);
            break;
        case GEMM_GATE_UP:
            hipLaunchKernelGGL(splitk_epilogue_kernel<GEMM_GATE_UP>, dim3(blocks), dim3(256), 0, st, partial, parts, part_stride, M, ncols_phys, rinv, res, out, out_stride, out_row0);
            break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Split-K epilogue of a residual matrix whose launch covers whole rows of the hidden state
// (out = res + sum of the planes), with the RMS factor of the row it has just written: one
// workgroup per token.  Thread t owns the 8-column chunks t, t + 256, ... exactly as in
// rinv_kernel, squares the fp16 values it stores and reduces in the same order, so rinv[m] has the
// bits rinv_kernel would give on the stored row, and the separate launch can be left out.
// Planes past `parts` are not read (the load is redirected to the last plane and discarded by a
// select, so the loads carry no branch).
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void splitk_epilogue_resid_rinv_kernel(const float *partial, uint32_t parts,
                                                                         uint32_t part_stride, uint32_t H,
                                                                         const __half *res, __half *out, float eps,
                                                                         float *rinv) {
    __shared__ float part[4];
    const uint32_t m = blockIdx.x, nq = H / 8;
    const float *prow = partial + (size_t)m * H;
    float ss = 0.f;
    for (uint32_t q = threadIdx.x; q < nq; q += 256) {
        float4 a[8][2];
#pragma unroll
        for (uint32_t p = 0; p < 8; ++p) {
            const float *src = prow + (size_t)(p < parts ? p : parts - 1) * part_stride + q * 8;
            a[p][0] = *reinterpret_cast<const float4 *>(src);
            a[p][1] = *reinterpret_cast<const float4 *>(src + 4);
        }
        uint4 rv = uint4{0u, 0u, 0u, 0u};
        if (res) rv = *reinterpret_cast<const uint4 *>(res + (size_t)m * H + q * 8);
        float r[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (uint32_t p = 0; p < 8; ++p) {
            const bool on = p < parts;   // adding +0 leaves a sum that started at +0 unchanged
            r[0] += on ? a[p][0].x : 0.f; r[1] += on ? a[p][0].y : 0.f;
            r[2] += on ? a[p][0].z : 0.f; r[3] += on ? a[p][0].w : 0.f;
            r[4] += on ? a[p][1].x : 0.f; r[5] += on ? a[p][1].y : 0.f;
            r[6] += on ? a[p][1].z : 0.f; r[7] += on ? a[p][1].w : 0.f;
        }
        if (res) {
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = half_of(rv, e) + r[e];
        }
        uint32_t d[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint16_t lo = __builtin_bit_cast(uint16_t, to_half(r[2 * e]));
            const uint16_t hi = __builtin_bit_cast(uint16_t, to_half(r[2 * e + 1]));
            d[e] = (uint32_t)lo | ((uint32_t)hi << 16);
        }
        const uint4 o = uint4{d[0], d[1], d[2], d[3]};
        *reinterpret_cast<uint4 *>(out + (size_t)m * H + q * 8) = o;
        ss += sumsq8(o);
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) rinv[m] = rsqrtf((((part[0] + part[1]) + part[2]) + part[3]) / (float)H + eps);
}

hipError_t launch_splitk_epilogue_resid_rinv(const float *partial, uint32_t parts, uint32_t part_stride, uint32_t M,
                                             uint32_t H, const __half *res, __half *out, float eps, float *rinv,
                                             hipStream_t st) {
    if (M == 0) return hipSuccess;
    if (parts == 0 || parts > 8 || H % 8 || part_stride % 4 || !partial || !out || !rinv) return hipErrorInvalidValue;
    hipLaunchKernelGGL(splitk_epilogue_resid_rinv_kernel, dim3(M), dim3(256), 0, st, partial, parts, part_stride, H, res,
                       out, eps, rinv);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Lane-layout probe for v_mfma_f32_16x16x32_f16 (in-bounds, integer-valued inputs):
// A[i][k] = 1 if (i, k) == (pi, pk) else 0, B[k][j] = 1 if (k, j) == (pk, pj): the single
// non-zero of C tells which lane/register holds C[pi][pj] under the layout assumed above.
// ------------------------------------------------------------------------------------
__global__ void mfma_probe_kernel(int pi, int pk, int pj, float *out /*[64][4]*/) {
    const int lane = threadIdx.x & 63, i = lane & 15, c = lane >> 4;
    h8_t A = {0, 0, 0, 0, 0, 0, 0, 0}, B = {0, 0, 0, 0, 0, 0, 0, 0};
    if (i == pi && c == pk / 8) A[pk % 8] = (_Float16)1.0f;
    if (i == pj && c == pk / 8) B[pk % 8] = (_Float16)1.0f;
    f4_t C = {0.f, 0.f, 0.f, 0.f};
    C = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, B, C, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 4; ++r) out[lane * 4 + r] = C[r];
}

// LDS transpose read (ds_read_b64_tr_b16): LDS holds the 16-bit numbers 0 .. 2047 at their own index; lane l
// reads at byte address addr[l] (forced to a multiple of 8 inside the table) and stores its four results.
__global__ void lds_tr_probe_kernel(const uint32_t *addr, uint16_t *out /*[64][4]*/) {
    __shared__ __attribute__((aligned(16))) uint16_t tab[2048];
    const int lane = threadIdx.x & 63;
    for (int k = lane; k < 2048; k += 64) tab[k] = (uint16_t)k;
    __syncthreads();
    const uint32_t off = min(addr[lane] & ~7u, 4088u);
    typedef __attribute__((__vector_size__(4 * sizeof(__fp16)))) __fp16 fp16x4_t;
    typedef __attribute__((address_space(3))) fp16x4_t lds_fp16x4_t;
#if defined(__HIP_DEVICE_COMPILE__)
    const fp16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4f16((lds_fp16x4_t *)(reinterpret_cast<unsigned char *>(tab) + off));
    const uint2 bits = __builtin_bit_cast(uint2, v);
    out[lane * 4 + 0] = (uint16_t)(bits.x & 0xFFFFu);
    out[lane * 4 + 1] = (uint16_t)(bits.x >> 16);
    out[lane * 4 + 2] = (uint16_t)(bits.y & 0xFFFFu);
    out[lane * 4 + 3] = (uint16_t)(bits.y >> 16);
#endif
}

hipError_t launch_lds_tr_probe(const uint32_t *addr, uint16_t *out, hipStream_t st) {
    hipLaunchKernelGGL(lds_tr_probe_kernel, dim3(1), dim3(64), 0, st, addr, out);
    return hipGetLastError();
}

hipError_t launch_mfma_probe(int pi, int pk, int pj, float *out, hipStream_t st) {
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(1), dim3(64), 0, st, pi, pk, pj, out);
    return hipGetLastError();
}

}  // namespace ps
