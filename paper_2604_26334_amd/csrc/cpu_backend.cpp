// CPU back-end for weight shards that a plan leaves in system memory (paper Section 3, Plans Two
// and Three): 4-bit block-format matrix times a few fp16 activation rows, AVX-512, fp32
// accumulation, with the same fused steps as the GPU kernels (RMSNorm in front, SwiGLU or residual
// behind).  Reads the packed tile layout of the GPU kernels: a 16-row tile is a run of scale groups;
// a group is up to 8 super-blocks of 1024 B (64 chunks of 16 B, chunk c*16 + i = block 4 sb + c of
// row i, 32 codes) followed by 64 x 8 fp16 scales (chunk-major).
#include "cpu_backend.h"

#include "ps_internal.h"

#include <immintrin.h>

#include <algorithm>
#include <cmath>
#include <cstring>

#define PS_AVX512 __attribute__((target("avx512f,avx512bw,avx512vl,avx512dq,f16c,fma")))

namespace ps {

// ---------------------------------------------------------------------------- thread pool

CpuPool::CpuPool(unsigned threads) {
    for (unsigned t = 1; t < std::max(1u, threads); ++t) workers_.emplace_back([this] { worker(); });
}

CpuPool::~CpuPool() {
    {
        std::lock_guard<std::mutex> lk(mu_);
        stop_.store(true);
        gen_.fetch_add(1);
    }
    cv_.notify_all();
    for (auto &t : workers_) t.join();
}

// next_ carries the job's generation in its high half, so a worker that woke up late for an
// earlier job can never take an index of the current one with the earlier job's function.
bool CpuPool::take(uint64_t gen, uint32_t n, uint32_t *i) {
    uint64_t cur = next_.load(std::memory_order_acquire);
    for (;;) {
        if ((cur >> 32) != (gen & 0xFFFFFFFFu) || (uint32_t)cur >= n) return false;
        if (next_.compare_exchange_weak(cur, cur + 1, std::memory_order_acq_rel)) { *i = (uint32_t)cur; return true; }
    }
}

void CpuPool::worker() {
    uint64_t seen = 0;
    for (;;) {
        // short spin (jobs of one forward follow each other within microseconds), then sleep
        uint64_t g = gen_.load(std::memory_order_acquire);
        for (int spin = 0; g == seen && spin < 20000; ++spin) {
            _mm_pause();
            g = gen_.load(std::memory_order_acquire);
        }
        const std::function<void(uint32_t)> *fn;
        uint32_t n;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_.wait(lk, [&] { return gen_.load(std::memory_order_acquire) != seen; });
            g = gen_.load(std::memory_order_acquire);
            fn = fn_;
            n = n_;
        }
        seen = g;
        if (stop_.load()) return;
        for (uint32_t i; take(g, n, &i);) {
            (*fn)(i);
            done_.fetch_add(1, std::memory_order_acq_rel);
        }
    }
}

void CpuPool::run(uint32_t n, const std::function<void(uint32_t)> &fn) {
    if (n == 0) return;
    if (workers_.empty() || n == 1) {
        for (uint32_t i = 0; i < n; ++i) fn(i);
        return;
    }
    uint64_t g;
    {
        std::lock_guard<std::mutex> lk(mu_);
        fn_ = &fn;
        n_ = n;
        done_.store(0, std::memory_order_release);
        g = gen_.load(std::memory_order_relaxed) + 1;
        next_.store((g & 0xFFFFFFFFu) << 32, std::memory_order_release);
        gen_.store(g, std::memory_order_release);
    }
    cv_.notify_all();
    for (uint32_t i; take(g, n, &i);) {
        fn(i);
        done_.fetch_add(1, std::memory_order_acq_rel);
    }
    // every index was handed out under this generation's tag; wait for the ones still running
    while (done_.load(std::memory_order_acquire) < n) _mm_pause();
}

bool cpu_backend_supported() {
    return __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512bw") &&
           __builtin_cpu_supports("avx512vl") && __builtin_cpu_supports("avx512dq") && __builtin_cpu_supports("f16c");
}

// ---------------------------------------------------------------------------- kernel

namespace {

// Position j (0..31) of a block's dequantised order -> k offset inside the block.  A chunk's byte
// 4 kk + b holds, low nibble first, codes 8 kk + {0,4,1,5}[b] and 8 kk + {2,6,3,7}[b]; the kernel
// takes the 16 low nibbles, then the 16 high nibbles.
inline uint32_t block_k(uint32_t j) {
    static const uint8_t lo[4] = {0, 4, 1, 5}, hi[4] = {2, 6, 3, 7};
    const uint32_t jj = j & 15u, kk = jj >> 2, b = jj & 3u;
    return 8u * kk + (j < 16 ? lo[b] : hi[b]);
}

PS_AVX512 inline float half_to_float(uint16_t h) { return _cvtsh_ss(h); }
PS_AVX512 inline uint16_t float_to_half(float f) { return _cvtss_sh(f, _MM_FROUND_TO_NEAREST_INT); }

// dot products of one tile (16 rows) with TOK permuted activation rows: acc_out[row][tok]
template <int TOK>
PS_AVX512 void tile_dot(const uint8_t *tile, uint32_t nsb, uint32_t ngroups, const float *xp, size_t xp_stride,
                        float *acc_out /* [16][TOK] */) {
    // code q sits in the low (or high) nibble of a zero-extended byte: OR-ing it into the mantissa of
    // 2^23 gives the float 2^23 + q (or 2^23 + 16 q), and subtracting 2^23 + 8 (2^23 + 128) leaves
    // q - 8 (16 (q - 8)) exactly; the factor 16 is taken out of the activations it meets
    const __m512i nib_lo = _mm512_set1_epi32(0x0F), nib_hi = _mm512_set1_epi32(0xF0);
    const __m512i magic = _mm512_set1_epi32(0x4B000000);             // 2^23 as float bits
    const __m512 bias_lo = _mm512_set1_ps(8388608.0f + 8.0f), bias_hi = _mm512_set1_ps(8388608.0f + 128.0f);
    alignas(64) float scf[64 * 8];
    for (int rc = 0; rc < 4; ++rc) {                                 // rows 4 rc .. 4 rc + 3: one cache line per (sb, c)
        __m512 acc[4][TOK];
        for (int r = 0; r < 4; ++r)
            for (int m = 0; m < TOK; ++m) acc[r][m] = _mm512_setzero_ps();
        for (uint32_t g = 0; g < ngroups; ++g) {
            const uint32_t nsb_g = std::min(8u, nsb - g * 8u);
            const uint8_t *gbase = tile + (size_t)g * 9u * 1024u;
            const uint16_t *sc = reinterpret_cast<const uint16_t *>(gbase + (size_t)nsb_g * 1024u);
            // this row chunk's scales as fp32: chunks c*16 + 4 rc + r, 8 scales each
            for (int c = 0; c < 4; ++c)
                for (int r2 = 0; r2 < 4; r2 += 2) {
                    const int lane = c * 16 + 4 * rc + r2;
                    _mm512_store_ps(scf + lane * 8, _mm512_cvtph_ps(_mm256_loadu_si256(reinterpret_cast<const __m256i *>(sc + lane * 8))));
                }
            for (uint32_t s = 0; s < nsb_g; ++s) {
                const uint8_t *sbp = gbase + (size_t)s * 1024u;
                for (int c = 0; c < 4; ++c) {
                    const float *xk = xp + ((size_t)(g * 8u + s) * 4u + c) * 32u;
                    __m512 xlo[TOK], xhi[TOK];
                    for (int m = 0; m < TOK; ++m) {
                        xlo[m] = _mm512_loadu_ps(xk + m * xp_stride);
                        xhi[m] = _mm512_loadu_ps(xk + m * xp_stride + 16);
                    }
                    for (int r = 0; r < 4; ++r) {
                        const int lane = c * 16 + 4 * rc + r;
                        const __m512i v = _mm512_cvtepu8_epi32(_mm_loadu_si128(reinterpret_cast<const __m128i *>(sbp + lane * 16)));
                        const __m512 wl = _mm512_sub_ps(_mm512_castsi512_ps(_mm512_ternarylogic_epi32(v, nib_lo, magic, 0xEA)), bias_lo);
                        const __m512 wh = _mm512_sub_ps(_mm512_castsi512_ps(_mm512_ternarylogic_epi32(v, nib_hi, magic, 0xEA)), bias_hi);
                        const __m512 d = _mm512_set1_ps(scf[lane * 8 + s]);
                        if (TOK <= 2) {   // scale the block's dot product
                            for (int m = 0; m < TOK; ++m)
                                acc[r][m] = _mm512_fmadd_ps(_mm512_fmadd_ps(wh, xhi[m], _mm512_mul_ps(wl, xlo[m])), d, acc[r][m]);
                        } else {          // scale the weights once, reuse them for every token
                            const __m512 dl = _mm512_mul_ps(wl, d), dh = _mm512_mul_ps(wh, d);
                            for (int m = 0; m < TOK; ++m)
                                acc[r][m] = _mm512_fmadd_ps(dh, xhi[m], _mm512_fmadd_ps(dl, xlo[m], acc[r][m]));
                        }
                    }
                }
            }
        }
        for (int r = 0; r < 4; ++r)
            for (int m = 0; m < TOK; ++m) acc_out[(4 * rc + r) * TOK + m] = _mm512_reduce_add_ps(acc[r][m]);
    }
}

// One token, short rows: all 16 rows of the tile in a single pass, so the tile is read front to
// back (the four-pass form above touches every fourth cache line per pass).  Per row the blocks are
// added in the same order as there, so both forms give the same bits.
PS_AVX512 void tile_dot_one(const uint8_t *tile, uint32_t nsb, uint32_t ngroups, const float *xp, float *acc_out /* [16] */) {
    const __m512i nib_lo = _mm512_set1_epi32(0x0F), nib_hi = _mm512_set1_epi32(0xF0);
    const __m512i magic = _mm512_set1_epi32(0x4B000000);
    const __m512 bias_lo = _mm512_set1_ps(8388608.0f + 8.0f), bias_hi = _mm512_set1_ps(8388608.0f + 128.0f);
    alignas(64) float scf[64 * 8];
    __m512 acc[16];
    for (int i = 0; i < 16; ++i) acc[i] = _mm512_setzero_ps();
    for (uint32_t g = 0; g < ngroups; ++g) {
        const uint32_t nsb_g = std::min(8u, nsb - g * 8u);
        const uint8_t *gbase = tile + (size_t)g * 9u * 1024u;
        const uint16_t *sc = reinterpret_cast<const uint16_t *>(gbase + (size_t)nsb_g * 1024u);
        for (int q = 0; q < 32; ++q)
            _mm512_store_ps(scf + q * 16, _mm512_cvtph_ps(_mm256_loadu_si256(reinterpret_cast<const __m256i *>(sc + q * 16))));
        for (uint32_t s = 0; s < nsb_g; ++s) {
            const uint8_t *sbp = gbase + (size_t)s * 1024u;
            for (int c = 0; c < 4; ++c) {
                const float *xk = xp + ((size_t)(g * 8u + s) * 4u + c) * 32u;
                const __m512 xlo = _mm512_loadu_ps(xk), xhi = _mm512_loadu_ps(xk + 16);
#pragma GCC unroll 16
                for (int i = 0; i < 16; ++i) {
                    const int lane = c * 16 + i;
                    const __m512i v = _mm512_cvtepu8_epi32(_mm_loadu_si128(reinterpret_cast<const __m128i *>(sbp + lane * 16)));
                    const __m512 wl = _mm512_sub_ps(_mm512_castsi512_ps(_mm512_ternarylogic_epi32(v, nib_lo, magic, 0xEA)), bias_lo);
                    const __m512 wh = _mm512_sub_ps(_mm512_castsi512_ps(_mm512_ternarylogic_epi32(v, nib_hi, magic, 0xEA)), bias_hi);
                    const __m512 d = _mm512_set1_ps(scf[lane * 8 + s]);
                    acc[i] = _mm512_fmadd_ps(_mm512_fmadd_ps(wh, xhi, _mm512_mul_ps(wl, xlo)), d, acc[i]);
                }
            }
        }
    }
    for (int i = 0; i < 16; ++i) acc_out[i] = _mm512_reduce_add_ps(acc[i]);
}

template <int TOK>
PS_AVX512 inline void tile_dot_any(const uint8_t *tile, uint32_t nsb, uint32_t ngroups, const float *xp, size_t xp_stride, float *acc_out) {
    // measured on a 16-thread host, one token: K = 2048 tiles (MoE experts) 96 -> 113 GB/s in the
    // single pass, K = 4096 and 14336 tiles (dense FFN) 180 -> 158 GB/s; K = 768 the same either way
    if (TOK == 1 && nsb <= 16) tile_dot_one(tile, nsb, ngroups, xp, acc_out);
    else tile_dot<TOK>(tile, nsb, ngroups, xp, xp_stride, acc_out);
}

inline float silu(float v) { return v / (1.0f + std::exp(-v)); }

template <int TOK>
PS_AVX512 void run_unit(const CpuMatArgs &a, uint32_t u, uint32_t m0, const float *xp, const float *rinv) {
    const bool gu = a.mode == CPU_GATE_UP;
    float g[16 * TOK], up[16 * TOK];
    const uint8_t *t0 = a.W + (size_t)u * (gu ? 2 : 1) * a.tile_bytes;
    tile_dot_any<TOK>(t0, a.nsb, a.ngroups, xp + (size_t)m0 * a.K, a.K, g);
    if (gu) tile_dot_any<TOK>(t0 + a.tile_bytes, a.nsb, a.ngroups, xp + (size_t)m0 * a.K, a.K, up);
    for (int m = 0; m < TOK; ++m) {
        const size_t row = (size_t)(m0 + m) * a.out_stride + a.out_col0 + (size_t)u * 16u;
        for (int i = 0; i < 16; ++i) {
            float v = g[i * TOK + m];
            if (a.mode == CPU_F32) { a.out_f32[row + i] = v; continue; }
            if (a.mode == CPU_PLAIN) v = rinv[m0 + m] * v;
            else if (gu) v = silu(rinv[m0 + m] * v) * (rinv[m0 + m] * up[i * TOK + m]);
            else if (a.res) v += half_to_float(a.res[row + i]);
            a.out[row + i] = float_to_half(v);
        }
    }
}

}  // namespace

size_t cpu_scratch_floats(uint32_t M, uint32_t K) { return (size_t)M * K + M + 64; }

uint32_t cpu_units(const CpuMatArgs &a) { return a.mode == CPU_GATE_UP ? a.ntiles / 2 : a.ntiles; }

// activations once per call: fp32, in the order the kernel dequantises a block; RMS factors.
// A block of 32 fp16 values is converted and permuted in registers (small expert matrices are
// prepared once per expert and token, which a scalar loop made a visible share of their time);
// the squares are summed in double precision, eight partial sums per half block.
PS_AVX512 void cpu_prepare(const CpuMatArgs &a, float *scratch) {
    float *xp = scratch, *rinv = scratch + (size_t)a.M * a.K;
    const bool norm = a.mode == CPU_PLAIN || a.mode == CPU_GATE_UP;
    alignas(64) int32_t il[16], ih[16];
    for (uint32_t j = 0; j < 16; ++j) { il[j] = (int32_t)block_k(j); ih[j] = (int32_t)block_k(16 + j); }
    const __m512i idx_lo = _mm512_load_si512(il), idx_hi = _mm512_load_si512(ih);
    const __m512 sixteenth = _mm512_set1_ps(0.0625f);   // high-nibble weights come out as 16 (q - 8)
    for (uint32_t m = 0; m < a.M; ++m) {
        const uint16_t *x = a.x + (size_t)m * a.x_stride;
        float *o = xp + (size_t)m * a.K;
        __m512d s0 = _mm512_setzero_pd(), s1 = _mm512_setzero_pd();
        for (uint32_t b = 0; b < a.K / 32; ++b) {
            const __m512 v0 = _mm512_cvtph_ps(_mm256_loadu_si256(reinterpret_cast<const __m256i *>(x + b * 32)));
            const __m512 v1 = _mm512_cvtph_ps(_mm256_loadu_si256(reinterpret_cast<const __m256i *>(x + b * 32 + 16)));
            _mm512_storeu_ps(o + b * 32, _mm512_permutex2var_ps(v0, idx_lo, v1));
            _mm512_storeu_ps(o + b * 32 + 16, _mm512_mul_ps(_mm512_permutex2var_ps(v0, idx_hi, v1), sixteenth));
            if (norm) {
                const __m512d a0 = _mm512_cvtps_pd(_mm512_castps512_ps256(v0)), a1 = _mm512_cvtps_pd(_mm512_extractf32x8_ps(v0, 1));
                const __m512d b0 = _mm512_cvtps_pd(_mm512_castps512_ps256(v1)), b1 = _mm512_cvtps_pd(_mm512_extractf32x8_ps(v1, 1));
                s0 = _mm512_fmadd_pd(a0, a0, s0); s1 = _mm512_fmadd_pd(a1, a1, s1);
                s0 = _mm512_fmadd_pd(b0, b0, s0); s1 = _mm512_fmadd_pd(b1, b1, s1);
            }
        }
        const double ss = _mm512_reduce_add_pd(_mm512_add_pd(s0, s1));
        rinv[m] = norm ? 1.0f / std::sqrt((float)(ss / a.K) + a.eps) : 1.0f;
    }
}

// units [u0, u1) for every token: a tile is read from memory once and stays in cache for the
// token passes over it
PS_AVX512 void cpu_run_units(const CpuMatArgs &a, uint32_t u0, uint32_t u1, const float *scratch) {
    const float *xp = scratch, *rinv = scratch + (size_t)a.M * a.K;
    for (uint32_t u = u0; u < u1; ++u) {
        uint32_t m = 0;
        for (; m + 4 <= a.M; m += 4) run_unit<4>(a, u, m, xp, rinv);
        for (; m + 2 <= a.M; m += 2) run_unit<2>(a, u, m, xp, rinv);
        for (; m < a.M; ++m) run_unit<1>(a, u, m, xp, rinv);
    }
}

void cpu_matmul_w4(const CpuMatArgs &a, CpuPool &pool, float *scratch) {
    const uint32_t units = cpu_units(a);
    if (!units || !a.M) return;
    cpu_prepare(a, scratch);
    const uint32_t jobs = std::min(units, pool.size() * 2u);   // two ranges per thread evens out stragglers
    pool.run(jobs, [&](uint32_t j) {
        cpu_run_units(a, (uint32_t)((uint64_t)units * j / jobs), (uint32_t)((uint64_t)units * (j + 1) / jobs), scratch);
    });
}

void cpu_matmul_many(const std::vector<CpuMatArgs> &mats, CpuPool &pool, float *scratch, const std::vector<size_t> &scr) {
    uint32_t total = 0;
    for (size_t k = 0; k < mats.size(); ++k) { cpu_prepare(mats[k], scratch + scr[k]); total += cpu_units(mats[k]); }
    if (!total) return;
    const uint32_t per = std::max(1u, total / (pool.size() * 4u));
    struct Job { uint32_t mat, u0, u1; };
    std::vector<Job> jobs;
    for (uint32_t k = 0; k < mats.size(); ++k)
        for (uint32_t u = 0, n = cpu_units(mats[k]); u < n; u += per) jobs.push_back(Job{k, u, std::min(n, u + per)});
    pool.run((uint32_t)jobs.size(), [&](uint32_t j) {
        cpu_run_units(mats[jobs[j].mat], jobs[j].u0, jobs[j].u1, scratch + scr[jobs[j].mat]);
    });
}

}  // namespace ps

extern "C" int32_t ps_cpu_matmul(const uint8_t *packed, uint32_t rows, uint32_t K, int32_t mode, const uint16_t *x,
                                 uint32_t n_tokens, float eps, const uint16_t *res, uint16_t *out, uint32_t threads) {
    if (!packed || !x || !out || K == 0 || K % ps::kSuperK || K > 16384 || rows == 0 || rows % ps::kTileRows ||
        mode < ps::CPU_PLAIN || mode > ps::CPU_GATE_UP || n_tokens == 0 || n_tokens > 64 || threads == 0 || threads > 64 ||
        (mode == ps::CPU_GATE_UP && rows % (2 * ps::kTileRows))) {
        ps::set_error("ps_cpu_matmul: bad argument");
        return PS_E_ARG;
    }
    if (!ps::cpu_backend_supported()) { ps::set_error("the CPU back-end needs AVX-512 (F, BW, VL, DQ) and F16C"); return PS_E_STATE; }
    const ps::MatGeom g = ps::make_geom(rows, K, mode == ps::CPU_GATE_UP);
    ps::CpuMatArgs a;
    a.W = packed; a.ntiles = g.ntiles; a.tile_bytes = g.tile_bytes; a.nsb = g.nsb; a.ngroups = g.ngroups; a.K = K;
    a.M = n_tokens; a.x = x; a.x_stride = K; a.mode = mode; a.eps = eps; a.res = res; a.out = out;
    a.out_stride = mode == ps::CPU_GATE_UP ? rows / 2 : rows; a.out_col0 = 0;
    ps::CpuPool pool(threads);
    std::vector<float> scratch(ps::cpu_scratch_floats(n_tokens, K));
    ps::cpu_matmul_w4(a, pool, scratch.data());
    return PS_OK;
}
