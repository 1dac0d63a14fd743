// Optional per-kernel timing with HIP events on the launch stream, plus the algorithmic
// byte / flop counts of every launch.  Off by default; when a kernel's bit is set in the
// mask each of its launches is bracketed by two events, which are resolved lazily when the
// statistics are read.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <vector>

namespace hch {

enum KernelId : int {
    K_NEIGHBOUR = 0, K_CHILD,
    K_HASH2COL_VEC, K_HASH2COL_ELEM,
    K_COL2HASH,
    K_GEMM_ROWS, K_GEMM_ROWS_BT, K_GEMM_COLS, K_GEMM_GATHER, K_GEMM_GATHER_T, K_FLIP_WEIGHTS,
    K_SPLITK_REDUCE,
    K_POOL_FWD, K_POOL_BWD, K_RELU_FWD, K_RELU_BWD,
    K_COUNT
};

inline const char *kernel_name(int id)
{
    static const char *names[K_COUNT] = {
        "neighbour_kernel", "child_kernel", "hash2col_kernel<uint4>", "hash2col_kernel<elem>", "col2hash_kernel",
        "gemm_f32_kernel<A_ROWS,B_KC=0>", "gemm_f32_kernel<A_ROWS,B_KC=1>", "gemm_f32_kernel<A_COLS>",
        "gemm_f32_kernel<A_GATHER>", "gemm_f32_kernel<A_GATHER_T>", "flip_transpose_weights_kernel",
        "splitk_reduce_kernel", "pool_fwd_kernel", "pool_bwd_kernel", "relu_fwd_kernel",
        "relu_bwd_kernel"};
    return (id >= 0 && id < K_COUNT) ? names[id] : "";
}

struct KernelStats {
    int64_t launches = 0;
    double ms = 0.0;       // sum of event-measured durations
    double bytes = 0.0;    // algorithmic bytes of those launches
    double flops = 0.0;    // algorithmic flops of those launches
};

class Profiler {
public:
    static Profiler &get() { static Profiler p; return p; }

    void set_mask(uint64_t m) { std::lock_guard<std::mutex> g(mu_); mask_ = m; }
    bool on(int id) const { return (mask_ >> id) & 1u; }

    // called right before / after a launch of kernel `id` on stream s
    void before(int id, hipStream_t s, double bytes, double flops)
    {
        std::lock_guard<std::mutex> g(mu_);
        Pending p;
        p.id = id; p.bytes = bytes; p.flops = flops;
        p.a = take(); p.b = take();
        if (!p.a || !p.b) return;
        (void)hipEventRecord(p.a, s);
        pending_.push_back(p);
    }
    void after(hipStream_t s)
    {
        std::lock_guard<std::mutex> g(mu_);
        if (!pending_.empty()) (void)hipEventRecord(pending_.back().b, s);
    }

    // resolve all pending event pairs (blocks until those launches finished)
    void collect()
    {
        std::lock_guard<std::mutex> g(mu_);
        for (Pending &p : pending_) {
            float ms = 0.f;
            if (hipEventSynchronize(p.b) == hipSuccess && hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
                KernelStats &st = stats_[p.id];
                st.launches += 1; st.ms += ms; st.bytes += p.bytes; st.flops += p.flops;
            }
            free_.push_back(p.a); free_.push_back(p.b);
        }
        pending_.clear();
    }
    KernelStats read(int id) { std::lock_guard<std::mutex> g(mu_); return stats_[id]; }
    void reset() { std::lock_guard<std::mutex> g(mu_); for (auto &s : stats_) s = KernelStats(); }

private:
    struct Pending { int id; hipEvent_t a, b; double bytes, flops; };
    hipEvent_t take()
    {
        if (!free_.empty()) { hipEvent_t e = free_.back(); free_.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
    std::mutex mu_;
    uint64_t mask_ = 0;
    std::vector<Pending> pending_;
    std::vector<hipEvent_t> free_;
    KernelStats stats_[K_COUNT];
};

// RAII bracket around one launch
struct LaunchTimer {
    hipStream_t s; bool active;
    LaunchTimer(int id, hipStream_t stream, double bytes, double flops) : s(stream), active(Profiler::get().on(id))
    {
        if (active) Profiler::get().before(id, s, bytes, flops);
    }
    ~LaunchTimer() { if (active) Profiler::get().after(s); }
};

}  // namespace hch
