// Optional per-launch timing: when enabled, every kernel launcher brackets its launch with a HIP
// event pair on the launch stream; lga_profile_end() aggregates them per kernel name.
#pragma once

#include <hip/hip_runtime.h>

#include <cstring>
#include <string>
#include <vector>

namespace lga {

struct LaunchRecord {
    std::string name;
    double flops, bytes;
    hipEvent_t start, stop;
};

struct LaunchProfiler {
    bool enabled = false;
    std::string only;       // not empty: bracket only the launches whose kernel name starts with this
    std::vector<LaunchRecord> records;
};

LaunchProfiler &profiler();

// RAII bracket around one launch.  flops / bytes are the algorithmic work of that launch.
class ProfScope {
  public:
    // timed = false: never bracket this launch (for callers that must not create events)
    ProfScope(const char *name, double flops, double bytes, hipStream_t s, bool timed = true)
        : stream_(s), active_(timed && profiler().enabled) {
        if (active_ && !profiler().only.empty() && std::strncmp(name, profiler().only.c_str(), profiler().only.size()) != 0)
            active_ = false;
        if (!active_) return;
        LaunchRecord r{name, flops, bytes, nullptr, nullptr};
        if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) {
            active_ = false;
            return;
        }
        (void)hipEventRecord(r.start, stream_);
        profiler().records.push_back(r);
    }
    ~ProfScope() {
        if (active_) (void)hipEventRecord(profiler().records.back().stop, stream_);
    }

  private:
    hipStream_t stream_;
    bool active_;
};

}  // namespace lga
