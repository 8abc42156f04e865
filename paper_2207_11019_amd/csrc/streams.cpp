// Worker streams of the library: a small per-device pool, created on first use and kept until the
// process ends.  Stages (weight-gradient side stream) and schedules (per-stage forward / backward
// streams) borrow from it instead of creating and destroying streams of their own, so the number of
// streams a process holds stays bounded however many stages and schedules come and go.  Two borrowers
// that share a stream only gain extra ordering between their work; the enqueue order of a schedule is a
// topological order of its dependency graph, so shared streams cannot dead-lock it.
#include "lpm_internal.h"

#include <algorithm>
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

// One probe: the longer of the two time spans (ms) from the common start to the end of each stream's spin kernel.
static hipError_t probe_pair(hipStream_t a, hipStream_t b, hipEvent_t e0, hipEvent_t ea, hipEvent_t eb, long long ticks, float* span) {
    // b's kernel may start once a's stream has reached the probe, so both time spans start at e0
    hipError_t e = hipEventRecord(e0, a);
    if (e == hipSuccess) e = launch_spin(ticks, a);
    if (e == hipSuccess) e = hipStreamWaitEvent(b, e0, 0);
    if (e == hipSuccess) e = launch_spin(ticks, b);
    if (e == hipSuccess) e = hipEventRecord(eb, b);
    if (e == hipSuccess) e = hipEventRecord(ea, a);
    if (e == hipSuccess) e = hipEventSynchronize(ea);
    if (e == hipSuccess) e = hipEventSynchronize(eb);
    float ta = 0.f, tb = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ta, e0, ea);
    if (e == hipSuccess) e = hipEventElapsedTime(&tb, e0, eb);
    *span = std::max(ta, tb);
    return e;
}

hipError_t streams_share_queue(hipStream_t a, hipStream_t b, bool* shared) {
    *shared = true;
    if (a == b) return hipSuccess;
    constexpr long long SPIN_TICKS = 5000;               // 50 us of the 100 MHz clock
    hipEvent_t e0 = nullptr, ea = nullptr, eb = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&ea);
    if (e == hipSuccess) e = hipEventCreate(&eb);
    // the first launch on a stream can take far longer than any later one (the runtime sets the stream up): not timed
    if (e == hipSuccess) e = launch_spin(1, a);
    if (e == hipSuccess) e = launch_spin(1, b);
    if (e == hipSuccess) e = hipStreamSynchronize(a);
    if (e == hipSuccess) e = hipStreamSynchronize(b);
    // three probes, the median decides: other work on the GPU can stretch one probe, rarely two
    float t[3] = {0.f, 0.f, 0.f};
    for (int k = 0; k < 3 && e == hipSuccess; ++k) e = probe_pair(a, b, e0, ea, eb, SPIN_TICKS, &t[k]);
    if (e0) (void)hipEventDestroy(e0);
    if (ea) (void)hipEventDestroy(ea);
    if (eb) (void)hipEventDestroy(eb);
    if (e != hipSuccess) return e;
    std::sort(t, t + 3);
    // side by side both spans are one spin (0.05 ms) plus launch latency; back to back the later one is two spins
    *shared = t[1] > 0.08f;
    return hipSuccess;
}

hipError_t pick_concurrent_streams(const hipStream_t* taken, int n_taken, hipStream_t* out, int want, int* found) {
    std::vector<hipStream_t> have(taken, taken + n_taken);
    *found = 0;
    // the side streams first (they exist anyway), then the per-stage schedule streams
    for (int k = 0; k < LPM_POOL_STREAMS && *found < want; ++k) {
        const int index = (k + LPM_POOL_SCHEDULE_STREAMS) % LPM_POOL_STREAMS;
        hipStream_t c = nullptr;
        hipError_t e = pooled_stream(index, &c);
        if (e != hipSuccess) return e;
        bool clash = false;
        for (size_t i = 0; i < have.size() && !clash; ++i) {
            e = streams_share_queue(have[i], c, &clash);
            if (e != hipSuccess) return e;
        }
        if (clash) continue;
        have.push_back(c);
        out[(*found)++] = c;
    }
    return hipSuccess;
}

int next_side_stream_index() {
    std::lock_guard<std::mutex> lock(g_mu);
    const int i = LPM_POOL_SCHEDULE_STREAMS + g_next_side;
    g_next_side = (g_next_side + 1) % (LPM_POOL_STREAMS - LPM_POOL_SCHEDULE_STREAMS);
    return i;
}

}  // namespace lpm
