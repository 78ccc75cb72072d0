// CPU execution of weight shards (paper Section 3, "Plan Two" and "Plan Three": sub-layers that
// stay in system memory and run on the CPU, so that only activations cross PCIe).  The CPU reads the
// same packed tile images the GPU kernels read, straight from the pinned host pool.
// Host code only; nothing here is part of the C ABI.
#pragma once
#include <atomic>
#include <condition_variable>
#include <cstdint>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

namespace ps {

enum { CPU_PLAIN = 0, CPU_RESID = 1, CPU_GATE_UP = 2, CPU_F32 = 3 };   // epilogues, as the GPU kernels' modes

// Worker threads that run one indexed job at a time.  run(n, fn) calls fn(0..n-1) once each,
// the caller taking part, and returns when all are done.  Workers spin briefly between jobs of one
// forward and sleep on a condition variable otherwise.
class CpuPool {
public:
    explicit CpuPool(unsigned threads);
    ~CpuPool();
    unsigned size() const { return (unsigned)workers_.size() + 1; }
    void run(uint32_t n, const std::function<void(uint32_t)> &fn);

private:
    void worker();
    bool take(uint64_t gen, uint32_t n, uint32_t *i);
    std::vector<std::thread> workers_;
    std::mutex mu_;
    std::condition_variable cv_;
    std::atomic<uint64_t> gen_{0};
    std::atomic<uint64_t> next_{0};   // generation << 32 | next index
    std::atomic<uint32_t> done_{0};
    uint32_t n_ = 0;
    const std::function<void(uint32_t)> *fn_ = nullptr;
    std::atomic<bool> stop_{false};
};

struct CpuMatArgs {
    const uint8_t *W = nullptr;     // first physical tile of the shard (host memory, packed layout)
    uint32_t ntiles = 0;            // physical tiles in the shard (GATE_UP: even, gate/up interleaved)
    uint64_t tile_bytes = 0;
    uint32_t nsb = 0, ngroups = 0, K = 0;
    uint32_t M = 0;                 // tokens
    const uint16_t *x = nullptr;    // fp16 input rows [M][x_stride] (host)
    uint32_t x_stride = 0;
    int mode = CPU_PLAIN;           // PLAIN and GATE_UP apply RMSNorm(x) (unit gain) first
    float eps = 0.f;
    const uint16_t *res = nullptr;  // RESID: fp16 [M][out_stride] added to the result (may be null)
    uint16_t *out = nullptr;        // fp16 [M][out_stride]; this shard writes columns out_col0 ..
    float *out_f32 = nullptr;       // CPU_F32: raw fp32 sums instead (expert down projection)
    uint32_t out_stride = 0, out_col0 = 0;
};

// true if this CPU can run cpu_matmul_w4 (AVX-512 F/BW/VL + F16C)
bool cpu_backend_supported();
// out[m][out_col0 + j] = epilogue(sum_k W[j][k] x[m][k]) for the shard's rows j, fp32 accumulation.
// scratch: at least cpu_scratch_floats(M, K) floats, reused between calls.
size_t cpu_scratch_floats(uint32_t M, uint32_t K);
void cpu_matmul_w4(const CpuMatArgs &a, CpuPool &pool, float *scratch);
// The same in two steps, for callers that spread several small matrices over one pool.run:
// cpu_prepare once per matrix (its own scratch), then cpu_run_units over any split of
// [0, cpu_units(a)) from any thread.
uint32_t cpu_units(const CpuMatArgs &a);
void cpu_prepare(const CpuMatArgs &a, float *scratch);
void cpu_run_units(const CpuMatArgs &a, uint32_t u0, uint32_t u1, const float *scratch);
// Several (small) matrices in one pass over the pool: the units of all of them form one job list,
// about four jobs per thread.  Matrix k uses scratch + scr[k] (cpu_scratch_floats of its own).
void cpu_matmul_many(const std::vector<CpuMatArgs> &mats, CpuPool &pool, float *scratch, const std::vector<size_t> &scr);

}  // namespace ps
