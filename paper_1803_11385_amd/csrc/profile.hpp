// Optional per-kernel timing with HIP events on the launch stream, plus the algorithmic
// byte / flop counts of every launch.  Off by default.  Kernels are registered by the name of
// their __global__ function (template arguments included, spelled as a profiler prints them)
// the first time they are launched; while timing is on for a kernel each of its launches
// carries two events that take the start and the end of the dispatch itself (the launch goes
// through hipExtLaunchKernelGGL, which attaches them to the kernel: no command-processor time
// between an event and the kernel is counted); they are resolved lazily when the statistics
// are read.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <string>
#include <vector>

namespace hch {

// the events the next launch on this thread carries (null: none); set by LaunchTimer, taken by
// the launch macro
inline thread_local hipEvent_t tls_start_event = nullptr, tls_stop_event = nullptr;

struct KernelStats {
    int64_t launches = 0;
    double ms = 0.0;       // sum of event-measured durations
    double bytes = 0.0;    // algorithmic bytes of those launches
    double flops = 0.0;    // algorithmic flops of those launches
};

class Profiler {
public:
    static Profiler &get() { static Profiler p; return p; }

    // id of a kernel name, registering it on first sight
    int id_for(const std::string &name)
    {
        std::lock_guard<std::mutex> g(mu_);
        for (size_t i = 0; i < names_.size(); ++i) if (names_[i] == name) return (int)i;
        names_.push_back(name);
        stats_.push_back(KernelStats());
        on_.push_back(all_on_);
        return (int)names_.size() - 1;
    }
    int count() { std::lock_guard<std::mutex> g(mu_); return (int)names_.size(); }
    std::string name(int id) { std::lock_guard<std::mutex> g(mu_); return id >= 0 && id < (int)names_.size() ? names_[id] : std::string(); }

    // id < 0: every kernel, including ones not launched yet
    void enable(int id, bool on)
    {
        std::lock_guard<std::mutex> g(mu_);
        if (id < 0) { all_on_ = on; for (size_t i = 0; i < on_.size(); ++i) on_[i] = on; }
        else if (id < (int)on_.size()) on_[id] = on;
    }
    bool on(int id) { std::lock_guard<std::mutex> g(mu_); return id >= 0 && id < (int)on_.size() && on_[id]; }

    // called right before / after a launch of kernel `id` on stream s
    void before(int id, hipStream_t s, double bytes, double flops)
    {
        std::lock_guard<std::mutex> g(mu_);
        Pending p;
        p.id = id; p.bytes = bytes; p.flops = flops;
        p.a = take(); p.b = take();
        if (!p.a || !p.b) return;
        (void)s;
        tls_start_event = p.a; tls_stop_event = p.b;
        pending_.push_back(p);
    }
    void after(hipStream_t)
    {
        tls_start_event = tls_stop_event = nullptr;     // a scope without a launch times nothing
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
    KernelStats read(int id) { std::lock_guard<std::mutex> g(mu_); return id >= 0 && id < (int)stats_.size() ? stats_[id] : KernelStats(); }
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
    bool all_on_ = false;
    std::vector<std::string> names_;
    std::vector<KernelStats> stats_;
    std::vector<bool> on_;
    std::vector<Pending> pending_;
    std::vector<hipEvent_t> free_;
};

// RAII bracket around one launch.  `id` comes from Profiler::id_for, cached by the call site.
struct LaunchTimer {
    hipStream_t s; bool active;
    LaunchTimer(int id, hipStream_t stream, double bytes, double flops) : s(stream), active(Profiler::get().on(id))
    {
        if (active) Profiler::get().before(id, s, bytes, flops);
    }
    ~LaunchTimer() { if (active) Profiler::get().after(s); }
};

}  // namespace hch

// id of a kernel whose name is a literal, looked up once per call site
#define HCH_KERNEL_ID(name_literal) ([]() { static const int id_ = hch::Profiler::get().id_for(name_literal); return id_; }())
