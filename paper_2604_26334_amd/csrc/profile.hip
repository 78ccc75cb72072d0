// Machine profile for the planner's time estimate (paper Section 3, install phase: kernels
// are timed as a batch of asynchronous launches so that the rate reflects the concurrency
// the GPU offers).  Three kinds of numbers: pinned H2D copy rate, decode-kernel weight
// bandwidth, dequant-GEMM rate per token tier, plus the fixed cost of a launch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstring>
#include <memory>
#include <thread>
#include <vector>

#include "cpu_backend.h"
#include "kernels.h"
#include "ps_internal.h"

#define PS_HIP(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            ps::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
            rc = PS_E_HIP;                                                             \
            goto done;                                                                 \
        }                                                                              \
    } while (0)

extern "C" int32_t ps_profile_measure(void *scratch_dev, uint64_t scratch_bytes, void *compute_stream,
                                      void *copy_stream, ps_profile *out) {
    using namespace ps;
    constexpr uint64_t kHead = 64ull << 20;   // activations / outputs live here
    constexpr int kLaunches = 10;
    if (!scratch_dev || !out || scratch_bytes < (256ull << 20) || (uintptr_t)scratch_dev % kAlign) {
        set_error("profile scratch must be device memory, 256-byte aligned, >= 256 MiB");
        return PS_E_ARG;
    }
    int32_t rc = PS_OK;
    hipStream_t cs = static_cast<hipStream_t>(compute_stream), ps_copy = static_cast<hipStream_t>(copy_stream);
    uint8_t *base = static_cast<uint8_t *>(scratch_dev);
    void *host = nullptr, *cpu_img = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    float ms = 0;
    const MatGeom mg = make_geom(8192, 4096, false);  // an 8192 x 4096 matrix, 512 tiles
    __half *x = reinterpret_cast<__half *>(base);                         // [2048][4096] fp16 = 16 MiB
    __half *y = reinterpret_cast<__half *>(base + (16ull << 20));         // [2048][8192] fp16 = 32 MiB
    float *rinv = reinterpret_cast<float *>(base + (56ull << 20));
    uint8_t *wts = base + kHead;
    const uint64_t wbytes = scratch_bytes - kHead;
    *out = ps_profile{};

    PS_HIP(hipEventCreate(&e0));
    PS_HIP(hipEventCreate(&e1));
    PS_HIP(hipHostMalloc(&host, kHead, hipHostMallocDefault));
    std::memset(host, 0x11, kHead);
    // well-defined contents: activations 0x1111 (a small positive fp16), weights / scales likewise
    PS_HIP(hipMemsetAsync(base, 0x11, scratch_bytes, cs));
    PS_HIP(hipStreamSynchronize(cs));

    // pinned H2D rate: 64 MiB copies back to back on the copy stream
    PS_HIP(hipMemcpyAsync(wts, host, kHead, hipMemcpyHostToDevice, ps_copy));
    PS_HIP(hipEventRecord(e0, ps_copy));
    for (int i = 0; i < 8; ++i) PS_HIP(hipMemcpyAsync(wts, host, kHead, hipMemcpyHostToDevice, ps_copy));
    PS_HIP(hipEventRecord(e1, ps_copy));
    PS_HIP(hipEventSynchronize(e1));
    PS_HIP(hipEventElapsedTime(&ms, e0, e1));
    out->h2d_gbps = 8.0 * (double)kHead / (ms * 1e-3) / 1e9;

    // fixed launch cost: a trivial kernel, many launches
    PS_HIP(launch_rinv(x, 4, 4096, 1e-6f, rinv, cs));
    PS_HIP(hipEventRecord(e0, cs));
    for (int i = 0; i < 50; ++i) PS_HIP(launch_rinv(x, 4, 4096, 1e-6f, rinv, cs));
    PS_HIP(hipEventRecord(e1, cs));
    PS_HIP(hipEventSynchronize(e1));
    PS_HIP(hipEventElapsedTime(&ms, e0, e1));
    out->launch_us = ms * 1e3 / 50.0;

    {   // decode kernel bandwidth: ten launches over ten different weight regions
        const uint32_t tiles_total = (uint32_t)std::min<uint64_t>(wbytes / mg.tile_bytes, 1u << 20);
        const uint32_t per = tiles_total / kLaunches;
        GemvArgs a{};
        a.tile_u4 = (uint32_t)(mg.tile_bytes / 16); a.nsb = mg.nsb; a.ngroups = mg.ngroups; a.K = mg.K;
        a.x = x; a.x_group = 1; a.eps = 1e-6f; a.out = y; a.nunits = per; a.top_k = 1;
        for (int rep = 0; rep < 2; ++rep) {
            PS_HIP(hipEventRecord(e0, cs));
            for (int i = 0; i < kLaunches; ++i) {
                a.W = reinterpret_cast<const uint4 *>(wts + (uint64_t)i * per * mg.tile_bytes);
                PS_HIP(launch_gemv(GEMV_PLAIN, 1, a, 0, cs));
            }
            PS_HIP(hipEventRecord(e1, cs));
            PS_HIP(hipEventSynchronize(e1));
        }
        PS_HIP(hipEventElapsedTime(&ms, e0, e1));
        const double bytes = (double)kLaunches * per * mg.tile_bytes;
        out->gemv_gbps = bytes / (ms * 1e-3) / 1e9;
        out->gemm_tflops[0] = 2.0 * bytes / 0.5625 / (ms * 1e-3) / 1e12;
    }
    for (uint32_t t = 1; t < PS_NTIERS; ++t) {  // dequant GEMM at each token tier (capped at 2048 tokens)
        const uint32_t T = std::min(ps_tier_tokens(t), 2048u);
        if (ps_tier_tokens(t) > 2048) { out->gemm_tflops[t] = out->gemm_tflops[t - 1]; continue; }
        GemmArgs a{};
        a.W = reinterpret_cast<const uint4 *>(wts); a.ntiles = mg.ntiles; a.total_tiles = mg.ntiles; a.tile_u4 = (uint32_t)(mg.tile_bytes / 16);
        a.nsb = mg.nsb; a.M = T; a.x = x; a.x_stride = 4096; a.x_group = 1; a.rinv = rinv; a.out = y;
        a.out_stride = 8192; a.top_k = 1;
        PS_HIP(launch_rinv(x, T, 4096, 1e-6f, rinv, cs));
        // the executor runs two to kGemvMtTokens tokens in the few-token form of the decode kernel
        const bool few = T <= (uint32_t)kGemvMtTokens && mg.nsb % 8 == 0;
        GemvArgs fa{};
        fa.W = a.W; fa.nunits = mg.ntiles; fa.tile_u4 = a.tile_u4; fa.nsb = mg.nsb; fa.ngroups = mg.ngroups; fa.K = mg.K;
        fa.x = x; fa.x_group = 1; fa.x_stride = 4096; fa.eps = 1e-6f; fa.out = y; fa.out_stride = 8192; fa.top_k = 1;
        for (int rep = 0; rep < 2; ++rep) {
            PS_HIP(hipEventRecord(e0, cs));
            for (int i = 0; i < kLaunches; ++i) {
                if (few) PS_HIP(launch_gemv_mt(GEMV_PLAIN, gemv_ksplit(mg.ngroups, mg.ntiles), fa, T, cs));
                else PS_HIP(launch_gemm(GEMM_PLAIN, a, 0, T, cs));
            }
            PS_HIP(hipEventRecord(e1, cs));
            PS_HIP(hipEventSynchronize(e1));
        }
        PS_HIP(hipEventElapsedTime(&ms, e0, e1));
        out->gemm_tflops[t] = 2.0 * T * 8192.0 * 4096.0 * kLaunches / (ms * 1e-3) / 1e12;
    }
    if (cpu_backend_supported()) {
        // CPU back-end (plans Two and Three): its rate over a packed image far larger than the
        // caches, alone and while H2D copies pull on the same memory, the copy rate meanwhile, the
        // token count up to which it stays memory-bound, and the fixed cost of one CPU shard
        constexpr uint64_t kImage = 512ull << 20;
        auto now = [] { return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count(); };
        PS_HIP(hipHostMalloc(&cpu_img, kImage, hipHostMallocDefault));
        std::memset(cpu_img, 0x11, kImage);
        const unsigned hw = std::thread::hardware_concurrency();
        std::unique_ptr<CpuPool> pool(new CpuPool(std::min(hw ? hw : 4u, 16u)));
        std::vector<float> scratch(cpu_scratch_floats(16, 4096));
        std::vector<uint16_t> xh(16 * 4096, 0x1111), yh((size_t)16 * (kImage / mg.tile_bytes) * 16);
        CpuMatArgs a;
        a.W = static_cast<const uint8_t *>(cpu_img); a.ntiles = (uint32_t)(kImage / mg.tile_bytes); a.tile_bytes = mg.tile_bytes;
        a.nsb = mg.nsb; a.ngroups = mg.ngroups; a.K = mg.K; a.M = 1; a.x = xh.data(); a.x_stride = 4096;
        a.mode = CPU_PLAIN; a.eps = 1e-6f; a.out = yh.data(); a.out_stride = a.ntiles * 16; a.out_col0 = 0;
        const double image_bytes = (double)a.ntiles * mg.tile_bytes;
        for (int r = 0; r < 3; ++r) cpu_matmul_w4(a, *pool, scratch.data());   // warm-up: pages touched, workers awake, cores clocked up
        double t0 = now();
        for (int r = 0; r < 6; ++r) cpu_matmul_w4(a, *pool, scratch.data());
        out->cpu_gbps = 6.0 * image_bytes / (now() - t0) / 1e9;
        {   // tokens the kernel takes before it turns compute-bound: 16 tokens against 1 on 1/8 of the image
            CpuMatArgs b = a;
            b.ntiles = a.ntiles / 8; b.out_stride = b.ntiles * 16;
            t0 = now();
            cpu_matmul_w4(b, *pool, scratch.data());
            const double t1 = now() - t0;
            b.M = 16;
            t0 = now();
            cpu_matmul_w4(b, *pool, scratch.data());
            const double t16 = now() - t0;
            out->cpu_tokens_free = t16 > t1 ? std::max(1.0, 16.0 * t1 / t16) : 64.0;
        }
        {   // both at once: 24 copies of 64 MiB on the copy stream, the CPU kernel looping until they end
            PS_HIP(hipEventRecord(e0, ps_copy));
            for (int i = 0; i < 24; ++i) PS_HIP(hipMemcpyAsync(wts, host, kHead, hipMemcpyHostToDevice, ps_copy));
            PS_HIP(hipEventRecord(e1, ps_copy));
            t0 = now();
            int passes = 0;
            double t_in = 0;   // CPU time that ended while the copies were still running
            while (hipEventQuery(e1) == hipErrorNotReady) {
                cpu_matmul_w4(a, *pool, scratch.data());
                ++passes;
                if (hipEventQuery(e1) == hipErrorNotReady) t_in = now() - t0; else if (passes > 1) --passes;
            }
            PS_HIP(hipEventSynchronize(e1));
            PS_HIP(hipEventElapsedTime(&ms, e0, e1));
            out->h2d_gbps_busy = 24.0 * (double)kHead / (ms * 1e-3) / 1e9;
            out->cpu_gbps_busy = (passes > 0 && t_in > 0) ? passes * image_bytes / t_in / 1e9 : out->cpu_gbps;
        }
        {   // one CPU shard's fixed cost: 8 KB down, wait, a 16-tile job, 8 KB up
            CpuMatArgs b = a;
            b.ntiles = 16; b.out_stride = 256;
            const int n = 20;
            PS_HIP(hipStreamSynchronize(cs));
            t0 = now();
            for (int i = 0; i < n; ++i) {
                PS_HIP(hipMemcpyAsync(host, x, 8192, hipMemcpyDeviceToHost, cs));
                PS_HIP(hipStreamSynchronize(cs));
                cpu_matmul_w4(b, *pool, scratch.data());
                PS_HIP(hipMemcpy2DAsync(y, 8192, host, 8192, 512, 1, hipMemcpyHostToDevice, cs));
            }
            PS_HIP(hipStreamSynchronize(cs));
            out->cpu_sync_us = (now() - t0) / n * 1e6;
        }
    }
done:
    if (cpu_img) (void)hipHostFree(cpu_img);
    if (host) (void)hipHostFree(host);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    return rc;
}

extern "C" int32_t ps_profile_db_measure(ps_profile_db *db, const ps_model_desc *model, void *scratch_dev,
                                         uint64_t scratch_bytes, void *compute_stream, void *copy_stream) {
    using namespace ps;
    constexpr uint64_t kX = 64ull << 20, kY = 64ull << 20, kHeadRoom = 132ull << 20;   // activations, outputs, rinv
    constexpr uint32_t kMaxRows = 16384, kMaxTok = 2048;
    constexpr int kLaunches = 10;
    if (!db || !model || !scratch_dev || scratch_bytes < (768ull << 20) || (uintptr_t)scratch_dev % kAlign) {
        set_error("profile database scratch must be device memory, 256-byte aligned, >= 768 MiB");
        return PS_E_ARG;
    }
    ModelGeom g;
    int32_t rc = make_model_geom(model, &g);
    if (rc) return rc;
    hipStream_t cs = static_cast<hipStream_t>(compute_stream), cp = static_cast<hipStream_t>(copy_stream);
    uint8_t *base = static_cast<uint8_t *>(scratch_dev);
    __half *x = reinterpret_cast<__half *>(base);
    __half *y = reinterpret_cast<__half *>(base + kX);
    float *rinv = reinterpret_cast<float *>(base + kX + kY);
    uint8_t *wts = base + kHeadRoom;
    const uint64_t wbytes = scratch_bytes - kHeadRoom;
    void *host = nullptr, *cpu_img = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    float ms = 0;
    auto add = [&](uint32_t op, uint32_t threads, uint64_t n, uint64_t k, uint64_t m, double t_ms) {
        ps_prof_entry e{};
        e.op = op; e.quant = op == PS_OPK_H2D ? 0 : 4; e.threads = threads; e.n = n; e.k = k; e.m = m; e.ms = t_ms;
        return ps_profile_db_add(db, &e);
    };
    // the model's distinct weight matrices (rows capped: a larger one is priced from its nearest entry)
    struct Mat { uint32_t rows, K; bool cpu; };
    std::vector<Mat> mats;
    auto push = [&](const MatGeom &mg, bool cpu) {
        if (!mg.ntiles) return;
        const uint32_t rows = std::min(mg.rows, kMaxRows);
        for (const Mat &o : mats) if (o.rows == rows && o.K == mg.K) return;
        mats.push_back(Mat{rows, mg.K, cpu});
    };
    push(g.qkv, false); push(g.o, false); push(g.gate_up, true); push(g.down, true); push(g.head, true);

    PS_HIP(hipEventCreate(&e0));
    PS_HIP(hipEventCreate(&e1));
    PS_HIP(hipHostMalloc(&host, 64ull << 20, hipHostMallocDefault));
    std::memset(host, 0x11, 64ull << 20);
    PS_HIP(hipMemsetAsync(base, 0x11, scratch_bytes, cs));
    PS_HIP(hipStreamSynchronize(cs));

    for (uint64_t mib : {1ull, 4ull, 16ull, 64ull}) {   // pinned H2D copies, eight timed together
        const uint64_t bytes = mib << 20;
        PS_HIP(hipMemcpyAsync(wts, host, bytes, hipMemcpyHostToDevice, cp));
        PS_HIP(hipEventRecord(e0, cp));
        for (int i = 0; i < 8; ++i) PS_HIP(hipMemcpyAsync(wts + (uint64_t)i * bytes, host, bytes, hipMemcpyHostToDevice, cp));
        PS_HIP(hipEventRecord(e1, cp));
        PS_HIP(hipEventSynchronize(e1));
        PS_HIP(hipEventElapsedTime(&ms, e0, e1));
        rc = add(PS_OPK_H2D, 0, bytes, 1, 1, ms / 8.0);
        if (rc) goto done;
    }
    PS_HIP(hipMemsetAsync(wts, 0x11, wbytes, cs));
    for (const Mat &mt : mats) {
        const MatGeom mg = make_geom(mt.rows, mt.K, false);
        const uint32_t fit = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(kLaunches, wbytes / mg.bytes));
        {   // one token: ten launches over different copies of the matrix
            GemvArgs a{};
            a.tile_u4 = (uint32_t)(mg.tile_bytes / 16); a.nsb = mg.nsb; a.ngroups = mg.ngroups; a.K = mg.K;
            a.x = x; a.x_group = 1; a.eps = 1e-6f; a.out = y; a.nunits = mg.ntiles; a.top_k = 1;
            const uint32_t ks = gemv_ksplit(mg.ngroups, mg.ntiles);
            for (int rep = 0; rep < 2; ++rep) {
                PS_HIP(hipEventRecord(e0, cs));
                for (int i = 0; i < kLaunches; ++i) {
                    a.W = reinterpret_cast<const uint4 *>(wts + (uint64_t)(i % fit) * mg.bytes);
                    PS_HIP(launch_gemv(GEMV_PLAIN, ks, a, 0, cs));
                }
                PS_HIP(hipEventRecord(e1, cs));
                PS_HIP(hipEventSynchronize(e1));
            }
            PS_HIP(hipEventElapsedTime(&ms, e0, e1));
            rc = add(PS_OPK_GEMV, 0, mt.rows, mt.K, 1, ms / kLaunches);
            if (rc) goto done;
        }
        for (uint32_t t = 1; t < PS_NTIERS && ps_tier_tokens(t) <= kMaxTok; ++t) {
            const uint32_t T = ps_tier_tokens(t);
            GemmArgs a{};
            a.ntiles = mg.ntiles; a.total_tiles = mg.ntiles; a.tile_u4 = (uint32_t)(mg.tile_bytes / 16);
            a.nsb = mg.nsb; a.M = T; a.x = x; a.x_stride = mt.K; a.x_group = 1; a.rinv = rinv; a.out = y;
            a.out_stride = mt.rows; a.top_k = 1;
            PS_HIP(launch_rinv(x, T, mt.K, 1e-6f, rinv, cs));
            // (two to kGemvMtTokens tokens: the few-token form of the decode kernel, as in the executor)
            const bool few = T <= (uint32_t)kGemvMtTokens && mg.nsb % 8 == 0;
            GemvArgs fa{};
            fa.nunits = mg.ntiles; fa.tile_u4 = a.tile_u4; fa.nsb = mg.nsb; fa.ngroups = mg.ngroups; fa.K = mg.K;
            fa.x = x; fa.x_group = 1; fa.x_stride = mt.K; fa.eps = 1e-6f; fa.out = y; fa.out_stride = mt.rows; fa.top_k = 1;
            for (int rep = 0; rep < 2; ++rep) {
                PS_HIP(hipEventRecord(e0, cs));
                for (int i = 0; i < kLaunches; ++i) {
                    a.W = reinterpret_cast<const uint4 *>(wts + (uint64_t)(i % fit) * mg.bytes);
                    fa.W = a.W;
                    if (few) PS_HIP(launch_gemv_mt(GEMV_PLAIN, gemv_ksplit(mg.ngroups, mg.ntiles), fa, T, cs));
                    else PS_HIP(launch_gemm(GEMM_PLAIN, a, 0, T, cs));
                }
                PS_HIP(hipEventRecord(e1, cs));
                PS_HIP(hipEventSynchronize(e1));
            }
            PS_HIP(hipEventElapsedTime(&ms, e0, e1));
            rc = add(PS_OPK_GEMM, 0, mt.rows, mt.K, T, ms / kLaunches);
            if (rc) goto done;
        }
    }
    if (cpu_backend_supported()) {
        constexpr uint64_t kImage = 512ull << 20;
        auto now = [] { return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count(); };
        PS_HIP(hipHostMalloc(&cpu_img, kImage, hipHostMallocDefault));
        std::memset(cpu_img, 0x11, kImage);
        const unsigned hw = std::thread::hardware_concurrency();
        std::unique_ptr<CpuPool> pool(new CpuPool(std::min(hw ? hw : 4u, 16u)));
        std::vector<float> scratch(cpu_scratch_floats(64, 16384));
        std::vector<uint16_t> xh((size_t)64 * 16384, 0x1111), yh((size_t)8 * 64 * kMaxRows);   // an output block per batched matrix
        for (const Mat &mt : mats) {
            if (!mt.cpu) continue;
            const MatGeom mg = make_geom(mt.rows, mt.K, false);
            const uint32_t fit = (uint32_t)std::max<uint64_t>(1, kImage / mg.bytes);
            for (uint32_t T : {1u, 2u, 4u, 8u, 16u, 64u}) {
                CpuMatArgs a;
                a.ntiles = mg.ntiles; a.tile_bytes = mg.tile_bytes; a.nsb = mg.nsb; a.ngroups = mg.ngroups; a.K = mg.K;
                a.M = T; a.x = xh.data(); a.x_stride = mt.K; a.mode = CPU_PLAIN; a.eps = 1e-6f; a.out = yh.data();
                a.out_stride = mt.rows; a.out_col0 = 0;
                const int reps = T <= 4 ? 4 : 2;
                // a matrix too small to keep the threads busy on its own (an expert) is run the way the
                // executor runs such matrices: several of them in one pass over the pool
                const uint32_t batch = mg.bytes < (8ull << 20) ? std::min(fit, 8u) : 1u;
                std::vector<CpuMatArgs> many(batch, a);
                std::vector<size_t> scr(batch);
                if (scratch.size() < batch * cpu_scratch_floats(T, mt.K)) scratch.resize(batch * cpu_scratch_floats(T, mt.K));
                for (uint32_t b = 0; b < batch; ++b) {
                    scr[b] = b * cpu_scratch_floats(T, mt.K);
                    many[b].out = yh.data() + (size_t)b * 64 * kMaxRows;
                }
                double t0 = 0;
                for (int r = -1; r < reps; ++r) {          // pass -1 warms up; each pass reads other copies of the matrix
                    if (r == 0) t0 = now();
                    for (uint32_t b = 0; b < batch; ++b)
                        many[b].W = static_cast<const uint8_t *>(cpu_img) + (uint64_t)(((r + 1) * batch + b) % fit) * mg.bytes;
                    if (batch == 1) cpu_matmul_w4(many[0], *pool, scratch.data());
                    else cpu_matmul_many(many, *pool, scratch.data(), scr);
                }
                rc = add(PS_OPK_CPU, pool->size(), mt.rows, mt.K, T, (now() - t0) / reps / batch);
                if (rc) goto done;
            }
        }
    }
done:
    if (cpu_img) (void)hipHostFree(cpu_img);
    if (host) (void)hipHostFree(host);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    return rc;
}
