// Worker streams of the library: a small per-device pool, created on first use and kept until the
// process ends.  Stages (weight-gradient side stream) and schedules (per-stage forward / backward
// streams) borrow from it instead of creating and destroying streams of their own, so the number of
// streams a process holds stays bounded however many stages and schedules come and go.  Two borrowers
// that share a stream only gain extra ordering between their work; the enqueue order of a schedule is a
// topological order of its dependency graph, so shared streams cannot dead-lock it.
#include "lpm_internal.h"

#include <map>
#include <mutex>

namespace lpm {

namespace {
std::mutex g_mu;
std::map<int, std::vector<hipStream_t>> g_pool;   // device -> streams
int g_next_side = 0;
}  // namespace

hipError_t pooled_stream(int index, hipStream_t* out) {
    if (index < 0 || index >= LPM_POOL_STREAMS) return hipErrorInvalidValue;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(g_mu);
    std::vector<hipStream_t>& v = g_pool[dev];
    if (v.empty()) v.assign(LPM_POOL_STREAMS, nullptr);
    if (!v[(size_t)index]) {
        e = hipStreamCreateWithFlags(&v[(size_t)index], hipStreamNonBlocking);
        if (e != hipSuccess) { v[(size_t)index] = nullptr; return e; }
    }
    *out = v[(size_t)index];
    return hipSuccess;
}

int next_side_stream_index() {
    std::lock_guard<std::mutex> lock(g_mu);
    const int i = LPM_POOL_SCHEDULE_STREAMS + g_next_side;
    g_next_side = (g_next_side + 1) % (LPM_POOL_STREAMS - LPM_POOL_SCHEDULE_STREAMS);
    return i;
}

}  // namespace lpm
