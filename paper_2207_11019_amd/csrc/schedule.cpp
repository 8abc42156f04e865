// One mini-batch step of the whole partitioned network on one GPU.
//
// Forward Pass and Backward Pass Parallelisation and Optimisation: the mini-batch is split into M
// micro-batches; F_{z,j} / B_{z,j} are the forward / backward operations of stage z on micro-batch j.
//   LOCKED      F_{0,j}..F_{Z-1,j}, B_{Z-1,j}..B_{0,j} one after the other (non-parallel schedule)
//   OVERLAPPED  the forward chain of micro-batch j+1 runs on one stream while the backward chain of
//               micro-batch j runs on another; a stage holds at most `window` micro-batches in
//               flight, i.e. F_{z,j+window} starts after B_{z,j} ("B_{0,0} finishes before F_{0,2}").
//   PIPELINED   the same dependency set, but every stage owns a forward and a backward stream (the
//               one-device-per-sub-module layout of the method's figure, with streams standing in for
//               devices): F_{z,j+1} also overlaps F_{z+1,j}, and B_{z,j} overlaps B_{z+1,j+1}.  Each stage
//               is enqueued by a host thread of its own (launching is what bounds small micro-batches).
// Every buffer that belongs to a micro-batch (stash, stage output, input gradient) lives in slot
// j % window.  In LOCKED and OVERLAPPED micro-batch j + window starts at stage 0 only after all of
// micro-batch j, so a slot is never rewritten while an operation of its previous owner is pending; in
// PIPELINED F_{z,j+window} waits for every reader of the slots it rewrites (B_{z,j} and the weight phase of
// B_{z+1,j}).
// Gradients are accumulated over the micro-batches in the fixed order j = 0..M-1 and every stage is
// updated once, right after its last backward, so both modes produce bit-identical results.
#include "stage.h"

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <thread>

using namespace lpm;



int32_t lpm_stage_prepare(lpm_stage* s);

namespace {
struct GraphEntry {
    std::vector<unsigned char> key;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};
}  // namespace

struct lpm_schedule {
    std::vector<lpm_stage*> st;
    int32_t Z = 0, M = 0, window = 2;
    std::vector<hipEvent_t> ev_f;   // [Z*M]  F_{z,j} done (index j*Z + z)
    std::vector<hipEvent_t> ev_b;   // [Z*M]  data phase of B_{z,j} done
    std::vector<hipEvent_t> ev_w;   // [Z*M]  all of B_{z,j} done (weight phase included)
    hipEvent_t ev_fork = nullptr;
    std::vector<hipStream_t> sf, sb;     // PIPELINED: per-stage forward / backward streams (borrowed from the pool)
    // OVERLAPPED: the weight phases' streams, picked from the pool so that forward, data phases, weight phases and
    // stage 0's weight phase each feed a hardware queue of their own; measured once per (sf, sb) pair
    hipStream_t ov_sf = nullptr, ov_sb = nullptr, ov_w = nullptr, ov_w0 = nullptr;
    std::vector<char> cut_fused;         // [Z] the ReLU backward of stage z-1's last layer runs inside stage z's backward kernel
    std::vector<GraphEntry> graphs;

    // PIPELINED: one enqueue thread per stage, started at the first such run.  An event may only be waited
    // on once its record has been enqueued, so each record is published to the other threads by storing the
    // run's epoch in rec_*[j*Z+z]; a thread spins on that before it enqueues the matching wait.
    int device = 0;
    std::vector<std::thread> workers;
    std::mutex mu;
    std::condition_variable cv_go, cv_done;
    uint64_t epoch = 0;
    int pending = 0;
    bool quit = false;
    const void* job = nullptr;             // RunArgs of the current run
    void* job_fn = nullptr;                // what every participating worker runs (RoleFn)
    int32_t job_roles = 0;                 // workers 0..job_roles-1 take part
    std::atomic<bool> abort{false};
    std::vector<int32_t> wrc;              // per worker: status and error text of the current run
    std::vector<std::string> werr;
    std::unique_ptr<std::atomic<uint64_t>[]> rec_f, rec_b, rec_w;
};

static void destroy_events(lpm_schedule* s) {
    for (hipEvent_t e : s->ev_f) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : s->ev_b) if (e) (void)hipEventDestroy(e);
    if (s->ev_fork) (void)hipEventDestroy(s->ev_fork);
    for (hipEvent_t e : s->ev_w) if (e) (void)hipEventDestroy(e);
    for (GraphEntry& g : s->graphs) {
        if (g.exec) (void)hipGraphExecDestroy(g.exec);
        if (g.graph) (void)hipGraphDestroy(g.graph);
    }
}

extern "C" int32_t lpm_schedule_create(lpm_stage* const* stages, int32_t Z, int32_t n_microbatch, int32_t window,
                                       lpm_schedule** out) {
    if (!out) return fail(LPM_EINVAL, "out is NULL");
    *out = nullptr;
    if (!stages || Z <= 0) return fail(LPM_EINVAL, "no stages");
    if (n_microbatch <= 0) return fail(LPM_EINVAL, "n_microbatch must be positive");
    if (window < 1 || window > LPM_MAX_WINDOW) return fail(LPM_EINVAL, "window must be in 1..%d", LPM_MAX_WINDOW);
    for (int32_t z = 0; z < Z; ++z) {
        if (!stages[z]) return fail(LPM_EINVAL, "stage %d is NULL", z);
        if (stages[z]->m != stages[0]->m || stages[z]->dtype != stages[0]->dtype || stages[z]->L != stages[0]->L)
            return fail(LPM_ESHAPE, "stage %d differs from stage 0 in micro-batch, element type or network", z);
        if (z == 0 ? stages[z]->first != 0 : stages[z]->first != stages[z - 1]->last)
            return fail(LPM_ESHAPE, "stage %d does not start where stage %d ends", z, z - 1);
        if (stages[z]->loss && z != Z - 1) return fail(LPM_ESHAPE, "only the last stage may hold the loss");
    }
    if (stages[Z - 1]->last != stages[0]->L) return fail(LPM_ESHAPE, "the stages do not cover the whole network");
    for (int32_t z = 0; z < Z; ++z) {      // side streams and events exist before any capture starts
        const int32_t rc = lpm_stage_prepare(stages[z]);
        if (rc) return rc;
    }
    lpm_schedule* s = new (std::nothrow) lpm_schedule();
    if (!s) return fail(LPM_ENOMEM, "out of host memory");
    s->st.assign(stages, stages + Z);
    s->Z = Z; s->M = n_microbatch; s->window = window;
    s->ev_f.assign((size_t)n_microbatch * Z, nullptr);
    s->ev_b.assign((size_t)n_microbatch * Z, nullptr);
    s->ev_w.assign((size_t)n_microbatch * Z, nullptr);
    s->sf.assign((size_t)Z, nullptr);
    s->sb.assign((size_t)Z, nullptr);
    s->cut_fused.assign((size_t)Z, 0);
    for (int32_t z = 1; z < Z; ++z) s->cut_fused[(size_t)z] = lpm_stage_takes_dz(stages[z - 1]) && lpm_stage_can_mask_dx(stages[z]);
    s->rec_f.reset(new std::atomic<uint64_t>[(size_t)n_microbatch * Z]);
    s->rec_b.reset(new std::atomic<uint64_t>[(size_t)n_microbatch * Z]);
    s->rec_w.reset(new std::atomic<uint64_t>[(size_t)n_microbatch * Z]);
    for (size_t i = 0; i < (size_t)n_microbatch * Z; ++i) { s->rec_f[i].store(0); s->rec_b[i].store(0); s->rec_w[i].store(0); }
    hipError_t e = hipGetDevice(&s->device);
    for (int32_t z = 0; z < Z; ++z) {
        if (e == hipSuccess) e = pooled_stream((2 * z) % LPM_POOL_SCHEDULE_STREAMS, &s->sf[(size_t)z]);
        if (e == hipSuccess) e = pooled_stream((2 * z + 1) % LPM_POOL_SCHEDULE_STREAMS, &s->sb[(size_t)z]);
    }
    for (hipEvent_t& ev : s->ev_w) if (e == hipSuccess) e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    for (hipEvent_t& ev : s->ev_f) if (e == hipSuccess) e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    for (hipEvent_t& ev : s->ev_b) if (e == hipSuccess) e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->ev_fork, hipEventDisableTiming);
    if (e != hipSuccess) {
        destroy_events(s);
        delete s;
        return hip_fail(e, "creating the schedule's streams and events");
    }
    *out = s;
    return LPM_OK;
}

extern "C" int32_t lpm_schedule_cut_fused(const lpm_schedule* s, int32_t z) {
    if (!s || z < 0 || z >= s->Z) return fail(LPM_EINVAL, "bad schedule or stage index");
    return s->cut_fused[(size_t)z] ? 1 : 0;
}

extern "C" int32_t lpm_schedule_destroy(lpm_schedule* s) {
    if (!s) return LPM_OK;
    if (!s->workers.empty()) {
        {
            std::lock_guard<std::mutex> lk(s->mu);
            s->quit = true;
        }
        s->cv_go.notify_all();
        for (std::thread& t : s->workers) t.join();
    }
    destroy_events(s);
    delete s;
    return LPM_OK;
}

namespace {

struct RunArgs {
    int32_t mode;
    const void* x_batch; const int32_t* labels; const void* dy_batch;
    const lpm_stage_buffers* bufs; int32_t dx_wanted; float lr, mu; float* loss_out;
    hipStream_t sf, sb;
};

// Weight version `ver` of a stage: -1 = the synchronous step (one version, in params / lowp); otherwise even
// versions live in params / lowp and odd ones in params_alt / lowp_alt (LPM_ASYNC_UPDATE).
inline float* ver_params(const lpm_stage_buffers& b, int32_t ver) { return (ver > 0 && (ver & 1)) ? b.params_alt : b.params; }
inline void* ver_lowp(const lpm_stage_buffers& b, int32_t ver) { return (ver > 0 && (ver & 1)) ? b.lowp_alt : b.lowp; }

int32_t fwd_op(lpm_schedule* s, const RunArgs& a, int32_t z, int32_t j, hipStream_t st, int32_t ver = -1) {
    lpm_stage* sg = s->st[(size_t)z];
    const int32_t slot = j % s->window;
    const lpm_stage_buffers& b = a.bufs[z];
    const void* in = z == 0 ? (const void*)((const char*)a.x_batch + (size_t)j * sg->T(sg->first - 1).bytes)
                            : (const void*)a.bufs[z - 1].act_out[slot];
    const int32_t* lab = sg->loss ? a.labels + (size_t)j * sg->m : nullptr;
    // synchronous step: the loss is the mean over the mini-batch; asynchronous update: over the micro-batch
    const float loss_scale = 1.0f / (float)(ver < 0 ? s->M * sg->m : sg->m);
    return lpm_stage_forward(sg, in, b.act_out[slot], lab, a.loss_out, ver_params(b, ver), ver_lowp(b, ver), b.stash[slot],
                             b.fwd_ws, loss_scale, st);
}

// wst: stream of the weight phase (see lpm_stage_backward_on)
// by_layer: the two phases come as separate calls and the weight phase follows the data phase layer by layer
int32_t bwd_op(lpm_schedule* s, const RunArgs& a, int32_t z, int32_t j, hipStream_t st, hipStream_t wst,
               int32_t phases = LPM_PHASE_DATA | LPM_PHASE_WEIGHTS, int32_t ver = -1, bool by_layer = false,
               hipStream_t wst2 = nullptr) {
    lpm_stage* sg = s->st[(size_t)z];
    const int32_t slot = j % s->window;
    const lpm_stage_buffers& b = a.bufs[z];
    const void* in = z == 0 ? (const void*)((const char*)a.x_batch + (size_t)j * sg->T(sg->first - 1).bytes)
                            : (const void*)a.bufs[z - 1].act_out[slot];
    const void* dy = nullptr;
    if (z < s->Z - 1) dy = a.bufs[z + 1].grad_in[slot];
    else if (!sg->loss) dy = (const char*)a.dy_batch + (size_t)j * sg->T(sg->t_out).bytes;
    void* dx = (z > 0 || a.dx_wanted) ? b.grad_in[slot] : nullptr;
    // synchronous step over few enough micro-batches: large fully connected layers file their operands per micro-batch and
    // contract the weight gradient once, at the last one (the weight phases of a stage run in micro-batch order)
    const bool staged = ver < 0 && s->M <= LPM_FC_STAGE_SLOTS;
    return lpm_stage_backward_on(sg, in, b.act_out[slot], dy, dx, ver_params(b, ver), ver_lowp(b, ver), b.stash[slot], b.grads,
                                 ver < 0 ? j > 0 : 0, b.bwd_ws, st, wst, j & 1, phases, staged ? j : -1,
                                 staged ? s->M : 0, by_layer ? j % LPM_MAX_WINDOW : -1,
                                 (s->cut_fused[(size_t)z] ? LPM_MASK_DX : 0) | (z + 1 < s->Z && s->cut_fused[(size_t)z + 1] ? LPM_DY_IS_DZ : 0),
                                 wst2);
}

// ver < 0: the one update of the synchronous step; else U_{z,ver}: version ver -> version ver + 1
int32_t upd_op(lpm_schedule* s, const RunArgs& a, int32_t z, hipStream_t st, int32_t ver = -1) {
    const lpm_stage_buffers& b = a.bufs[z];
    if (ver < 0) return lpm_stage_update(s->st[(size_t)z], b.params, b.lowp, b.grads, b.momentum, a.lr, a.mu, 0, st);
    return lpm_stage_update_to(s->st[(size_t)z], ver_params(b, ver), ver_params(b, ver + 1), ver_lowp(b, ver + 1), b.grads,
                               b.momentum, a.lr, a.mu, 0, st);
}

// LPM_ASYNC_UPDATE with an odd number of micro-batches leaves the final version in the alternate buffers
int32_t copy_final_version(lpm_schedule* s, const RunArgs& a, int32_t z, hipStream_t st) {
    if (!(s->M & 1)) return LPM_OK;
    lpm_stage* sg = s->st[(size_t)z];
    const lpm_stage_buffers& b = a.bufs[z];
    if (sg->n_trainable == 0) return LPM_OK;
    LPM_HIP(hipMemcpyAsync(b.params, b.params_alt, sg->n_trainable * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (sg->dtype == LPM_BF16 && sg->lowp_bytes)
        LPM_HIP(hipMemcpyAsync(b.lowp, b.lowp_alt, sg->lowp_bytes, hipMemcpyDeviceToDevice, st));
    return LPM_OK;
}

// version F_{z,j} reads under LPM_ASYNC_UPDATE: one update behind when it overlaps B_{z,j-1}
inline int32_t forward_version(int32_t j, int32_t overlap_window) { return std::max(0, j - (overlap_window - 1)); }

// ---- enqueue threads.  Launching, not the GPU, bounds a step of small micro-batches, so the decoupled
// schedules are enqueued by several host threads, each feeding streams of its own.  An event may only be
// waited on once its record has been enqueued: every record another thread waits for is published by storing
// the run's epoch in a rec_* slot, and the waiting thread spins on that slot before it enqueues the wait.
// Each thread's sequence is the restriction of one topological order of the dependency graph to its
// streams, so no thread waits for a record that can never be enqueued.

int32_t await_record(lpm_schedule* s, const std::atomic<uint64_t>& rec, uint64_t epoch) {
    unsigned spins = 0;
    while (rec.load(std::memory_order_acquire) != epoch) {
        if (s->abort.load(std::memory_order_relaxed)) return fail(LPM_EHIP, "another enqueue thread failed");
        if (++spins > 2000) std::this_thread::yield();
    }
    return LPM_OK;
}
inline void publish(std::atomic<uint64_t>& rec, uint64_t epoch) { rec.store(epoch, std::memory_order_release); }

// PIPELINED, worker z: stage z on sf[z] (forward), sb[z] (data phase of backward) and the stage's side stream
// (weight phase, update).  ev_f / ev_b: F_{z,j} / data phase of B_{z,j} done; ev_w: all of B_{z,j} done.
// Order: F_{z,0..W-1}, then B_{z,j}, F_{z,j+W} for j = 0..M-1 -- the restriction to stage z of
// "B_{Z-1,j}..B_{0,j}, F_{0,j+W}..F_{Z-1,j+W}".
int32_t pipelined_role(lpm_schedule* s, const RunArgs& a, int32_t z, uint64_t epoch) {
    const int32_t Z = s->Z, M = s->M, W = s->window;
    hipStream_t f = s->sf[(size_t)z], b = s->sb[(size_t)z], w = s->st[(size_t)z]->side;
    int32_t rc;
    LPM_HIP(hipStreamWaitEvent(f, s->ev_fork, 0));
    LPM_HIP(hipStreamWaitEvent(b, s->ev_fork, 0));
    auto F = [&](int32_t j) -> int32_t {
        if (j >= W) {
            // the slot's previous owner is done: this stage's B_{z,j-W}, and the weight phase of B_{z+1,j-W},
            // which reads this stage's output (the input of stage z+1's first layer)
            LPM_HIP(hipStreamWaitEvent(f, s->ev_w[(size_t)(j - W) * Z + z], 0));
            if (z < Z - 1) {
                const size_t i = (size_t)(j - W) * Z + z + 1;
                if ((rc = await_record(s, s->rec_w[i], epoch))) return rc;
                LPM_HIP(hipStreamWaitEvent(f, s->ev_w[i], 0));
            }
        }
        if (z > 0) {
            const size_t i = (size_t)j * Z + z - 1;
            if ((rc = await_record(s, s->rec_f[i], epoch))) return rc;
            LPM_HIP(hipStreamWaitEvent(f, s->ev_f[i], 0));
        }
        if ((rc = fwd_op(s, a, z, j, f))) return rc;
        LPM_HIP(hipEventRecord(s->ev_f[(size_t)j * Z + z], f));
        publish(s->rec_f[(size_t)j * Z + z], epoch);
        return LPM_OK;
    };
    auto B = [&](int32_t j) -> int32_t {
        const size_t me = (size_t)j * Z + z;
        // B_{z,j} follows F_{z,j}: directly for the last stage, through B_{z+1,j} for the others
        if (z == Z - 1) {
            LPM_HIP(hipStreamWaitEvent(b, s->ev_f[me], 0));
        } else {
            if ((rc = await_record(s, s->rec_b[me + 1], epoch))) return rc;
            LPM_HIP(hipStreamWaitEvent(b, s->ev_b[me + 1], 0));
        }
        if (W > 2 && j >= 2) LPM_HIP(hipStreamWaitEvent(b, s->ev_w[(size_t)(j - 2) * Z + z], 0));
        if ((rc = bwd_op(s, a, z, j, b, w, LPM_PHASE_DATA))) return rc;
        LPM_HIP(hipEventRecord(s->ev_b[me], b));
        publish(s->rec_b[me], epoch);
        LPM_HIP(hipStreamWaitEvent(w, s->ev_b[me], 0));
        if ((rc = bwd_op(s, a, z, j, b, w, LPM_PHASE_WEIGHTS))) return rc;
        if (j == M - 1 && (rc = upd_op(s, a, z, w))) return rc;
        LPM_HIP(hipEventRecord(s->ev_w[me], w));
        publish(s->rec_w[me], epoch);
        return LPM_OK;
    };
    for (int32_t j = 0; j < W && j < M; ++j) if ((rc = F(j))) return rc;
    for (int32_t j = 0; j < M; ++j) {
        if ((rc = B(j))) return rc;
        if (j + W < M && (rc = F(j + W))) return rc;
    }
    return LPM_OK;
}

// Streams of the weight phases for an OVERLAPPED run on (sf, sb): two pooled streams that share a hardware queue
// neither with sf or sb nor with each other; failing that one such stream for both, failing that stage 0's side
// stream.  The choice only affects how much overlaps, never the result.
int32_t pick_weight_streams(lpm_schedule* s, hipStream_t sf, hipStream_t sb) {
    if (s->ov_w && s->ov_sf == sf && s->ov_sb == sb) return LPM_OK;
    const hipStream_t taken[2] = {sf, sb};
    hipStream_t got[2] = {nullptr, nullptr};
    int found = 0;
    LPM_HIP(pick_concurrent_streams(taken, 2, got, 2, &found));
    s->ov_w = found > 0 ? got[0] : s->st[0]->side;
    s->ov_w0 = found > 1 ? got[1] : s->ov_w;
    s->ov_sf = sf;
    s->ov_sb = sb;
    return LPM_OK;
}

// OVERLAPPED, three workers: 0 enqueues the forward chains on sf, 1 the data phases of the backward chains
// on sb, 2 the weight phases and the updates on the weight streams (ov_w, and ov_w0 for stage 0; see pick_weight_streams).
// ev_f[j*Z+Z-1]: forward chain j done; ev_b[j*Z+z]: data phase of B_{z,j} done; ev_w[j*Z]: micro-batch j done.
int32_t overlapped_role(lpm_schedule* s, const RunArgs& a, int32_t role, uint64_t epoch) {
    const int32_t Z = s->Z, M = s->M, W = s->window;
    const bool async = (a.mode & LPM_ASYNC_UPDATE) != 0;
    hipStream_t sw = s->ov_w;
    int32_t rc;
    if (role == 0) {
        for (int32_t j = 0; j < M; ++j) {
            // F_{0,j} after B_{0,j-W}, the last operation of micro-batch j-W; the other stages follow in stream order
            if (j >= W) {
                const size_t i = (size_t)(j - W) * Z;
                if ((rc = await_record(s, s->rec_w[i], epoch))) return rc;
                LPM_HIP(hipStreamWaitEvent(a.sf, s->ev_w[i], 0));
            }
            for (int32_t z = 0; z < Z; ++z) if ((rc = fwd_op(s, a, z, j, a.sf, async ? forward_version(j, W) : -1))) return rc;
            LPM_HIP(hipEventRecord(s->ev_f[(size_t)j * Z + Z - 1], a.sf));
            publish(s->rec_f[(size_t)j * Z + Z - 1], epoch);
        }
    } else if (role == 1) {
        LPM_HIP(hipStreamWaitEvent(a.sb, s->ev_fork, 0));
        for (int32_t j = 0; j < M; ++j) {
            const size_t i = (size_t)j * Z + Z - 1;
            if ((rc = await_record(s, s->rec_f[i], epoch))) return rc;
            LPM_HIP(hipStreamWaitEvent(a.sb, s->ev_f[i], 0));
            if (W > 2 && j >= 2) {
                if ((rc = await_record(s, s->rec_w[(size_t)(j - 2) * Z], epoch))) return rc;
                LPM_HIP(hipStreamWaitEvent(a.sb, s->ev_w[(size_t)(j - 2) * Z], 0));
            }
            for (int32_t z = Z - 1; z >= 0; --z) {
                if (async && j > 0) {      // B_{z,j} reads version j: after U_{z,j-1} (which has also consumed the bias gradients)
                    const size_t u = (size_t)(j - 1) * Z + z;
                    if ((rc = await_record(s, s->rec_w[u], epoch))) return rc;
                    LPM_HIP(hipStreamWaitEvent(a.sb, s->ev_w[u], 0));
                }
                if ((rc = bwd_op(s, a, z, j, a.sb, sw, LPM_PHASE_DATA, async ? j : -1, z == 0 && !async))) return rc;
                LPM_HIP(hipEventRecord(s->ev_b[(size_t)j * Z + z], a.sb));
                publish(s->rec_b[(size_t)j * Z + z], epoch);
            }
        }
    } else {
        // Stage 0's weight phase closes every micro-batch, and the next forward chain but one waits for it: with a
        // hardware queue to itself it follows stage 0's data phase from the start instead of queueing behind the other
        // stages' weight phases.  ev_w[j*Z+1] then marks the end of those on the common weight stream.
        const bool own0 = !async && Z > 1 && s->ov_w0 != s->ov_w;
        // Asynchronous update: B_{z,j+1} waits for U_{z,j}, so the weight phases and updates are a chain per stage; odd
        // stages take the second stream (each stage keeps its stream, which orders its updates).
        const bool async2 = async && Z > 1 && s->ov_w0 != s->ov_w;
        // A single stage has the second stream to spare: its weight gradients alternate between the two (ResNet-50
        // conv4_x: 2.43 -> 2.34 ms per step; the weight phases are the longest of the three chains there).
        hipStream_t sw_pair = (!async && Z == 1 && s->ov_w0 != s->ov_w) ? s->ov_w0 : nullptr;
        hipStream_t sw_all = sw, sw_0 = s->ov_w0;
        for (int32_t j = 0; j < M; ++j) {
            for (int32_t z = Z - 1; z >= 0; --z) {
                sw = ((own0 && z == 0) || (async2 && (z & 1))) ? sw_0 : sw_all;
                const size_t i = (size_t)j * Z + z;
                if ((rc = await_record(s, s->rec_b[i], epoch))) return rc;
                // Stage 0 closes the micro-batch, and the next forward chain but one waits for it: there the weight
                // gradients follow the data phase layer by layer (the events were recorded before rec_b was published)
                const bool by_layer = z == 0 && !async;
                if (!by_layer) LPM_HIP(hipStreamWaitEvent(sw, s->ev_b[i], 0));
                if ((rc = bwd_op(s, a, z, j, a.sb, sw, LPM_PHASE_WEIGHTS, async ? j : -1, by_layer, sw_pair))) return rc;
                // whatever follows on this stream (the update, the record that closes the micro-batch) is still ordered
                // after the whole data phase
                if (by_layer) LPM_HIP(hipStreamWaitEvent(sw, s->ev_b[i], 0));
                if (async) {
                    if ((rc = upd_op(s, a, z, sw, j))) return rc;
                    if (j == M - 1 && (rc = copy_final_version(s, a, z, sw))) return rc;
                    if (z > 0) {           // ev_w[j*Z+z], z > 0: U_{z,j} done (the entry of stage 0 closes the micro-batch below)
                        LPM_HIP(hipEventRecord(s->ev_w[i], sw));
                        publish(s->rec_w[i], epoch);
                    }
                } else if (j == M - 1 && (rc = upd_op(s, a, z, sw))) return rc;
            }
            if (own0) {        // sw is stage 0's stream here: the micro-batch is done when the other stream is, too
                LPM_HIP(hipEventRecord(s->ev_w[(size_t)j * Z + 1], sw_all));
                LPM_HIP(hipStreamWaitEvent(sw, s->ev_w[(size_t)j * Z + 1], 0));
            }
            // (asynchronous update on two streams: U_{1,j}, recorded above, is the last operation of the odd stages)
            if (async2) LPM_HIP(hipStreamWaitEvent(sw, s->ev_w[(size_t)j * Z + 1], 0));
            LPM_HIP(hipEventRecord(s->ev_w[(size_t)j * Z], sw));
            publish(s->rec_w[(size_t)j * Z], epoch);
        }
    }
    return LPM_OK;
}

typedef int32_t (*RoleFn)(lpm_schedule*, const RunArgs&, int32_t, uint64_t);

void enqueue_worker(lpm_schedule* s, int32_t idx) {
    (void)hipSetDevice(s->device);
    uint64_t seen = 0;
    for (;;) {
        RunArgs a;
        RoleFn fn;
        bool mine;
        {
            std::unique_lock<std::mutex> lk(s->mu);
            s->cv_go.wait(lk, [&] { return s->quit || s->epoch != seen; });
            if (s->quit) return;
            seen = s->epoch;
            a = *(const RunArgs*)s->job;
            fn = (RoleFn)s->job_fn;
            mine = idx < s->job_roles;
        }
        if (!mine) continue;
        const int32_t rc = fn(s, a, idx, seen);
        if (rc) {
            s->abort.store(true);
            s->wrc[(size_t)idx] = rc;
            s->werr[(size_t)idx] = lpm_last_error();
        }
        {
            std::lock_guard<std::mutex> lk(s->mu);
            if (--s->pending == 0) s->cv_done.notify_one();
        }
    }
}

// Runs fn(s, a, role, epoch) for role = 0..roles-1 on the schedule's enqueue threads and waits for all of them.
int32_t run_roles(lpm_schedule* s, const RunArgs& a, RoleFn fn, int32_t roles) {
    const int32_t want = std::max(s->Z, 3);
    if (s->workers.empty()) {
        s->wrc.assign((size_t)want, LPM_OK);
        s->werr.assign((size_t)want, std::string());
        try {
            for (int32_t i = 0; i < want; ++i) s->workers.emplace_back(enqueue_worker, s, i);
        } catch (...) {
            return fail(LPM_ENOMEM, "cannot start the enqueue threads");
        }
    }
    if ((int32_t)s->workers.size() < roles) return fail(LPM_ENOMEM, "enqueue threads are missing");
    {
        std::lock_guard<std::mutex> lk(s->mu);
        s->abort.store(false);
        for (int32_t& r : s->wrc) r = LPM_OK;
        s->job = &a;
        s->job_fn = (void*)fn;
        s->job_roles = roles;
        s->pending = roles;
        ++s->epoch;
    }
    s->cv_go.notify_all();
    {
        std::unique_lock<std::mutex> lk(s->mu);
        s->cv_done.wait(lk, [&] { return s->pending == 0; });
    }
    for (int32_t i = 0; i < roles; ++i)
        if (s->wrc[(size_t)i]) return fail(s->wrc[(size_t)i], "enqueue thread %d: %s", i, s->werr[(size_t)i].c_str());
    return LPM_OK;
}

// The dz area of a stage's backward scratch has two copies (micro-batch parity), so the weight phase of
// micro-batch j may still run while the data phase of j + 1 writes; the data phase of j + 2 follows the
// forward pass of j + 2, which the window rule places after micro-batch j when window <= 2.  A wider
// window needs the explicit wait below.
int32_t enqueue(lpm_schedule* s, const RunArgs& a) {
    const int32_t Z = s->Z, M = s->M, W = s->window;
    const bool capturing = (a.mode & LPM_GRAPH) != 0;
    int32_t rc;
    if (s->st[(size_t)Z - 1]->loss) LPM_HIP(launch_fill_f32(a.loss_out, 1, 0.f, a.sf));
    if ((a.mode & 15) == LPM_LOCKED && (a.mode & LPM_ASYNC_UPDATE)) {      // plain per-micro-batch SGD
        for (int32_t j = 0; j < M; ++j) {
            for (int32_t z = 0; z < Z; ++z) if ((rc = fwd_op(s, a, z, j, a.sf, j))) return rc;
            for (int32_t z = Z - 1; z >= 0; --z) {
                if ((rc = bwd_op(s, a, z, j, a.sf, a.sf, LPM_PHASE_DATA | LPM_PHASE_WEIGHTS, j))) return rc;
                if ((rc = upd_op(s, a, z, a.sf, j))) return rc;
                if (j == M - 1 && (rc = copy_final_version(s, a, z, a.sf))) return rc;
            }
        }
        return LPM_OK;
    }
    if ((a.mode & 15) == LPM_LOCKED) {
        for (int32_t j = 0; j < M; ++j) {
            for (int32_t z = 0; z < Z; ++z) if ((rc = fwd_op(s, a, z, j, a.sf))) return rc;
            for (int32_t z = Z - 1; z >= 0; --z) if ((rc = bwd_op(s, a, z, j, a.sf, a.sf))) return rc;
        }
        for (int32_t z = 0; z < Z; ++z) if ((rc = upd_op(s, a, z, a.sf))) return rc;
        return LPM_OK;
    }
    LPM_HIP(hipEventRecord(s->ev_fork, a.sf));
    if ((a.mode & 15) == LPM_PIPELINED) {
        if ((rc = run_roles(s, a, pipelined_role, Z))) return rc;
        for (int32_t z = 0; z < Z; ++z)      // the weight stream's last event is ordered after all work of its stage
            LPM_HIP(hipStreamWaitEvent(a.sf, s->ev_w[(size_t)(M - 1) * Z + z], 0));
        return LPM_OK;
    }
    if (!capturing) {
        if ((rc = pick_weight_streams(s, a.sf, a.sb))) return rc;
        if ((rc = run_roles(s, a, overlapped_role, 3))) return rc;
        LPM_HIP(hipStreamWaitEvent(a.sf, s->ev_w[(size_t)(M - 1) * Z], 0));
        return LPM_OK;
    }
    // OVERLAPPED while a graph is captured: one thread, forward chains on sf, backward chains on sb (the weight
    // gradients are branches of the graph, see lpm_stage_backward_on).  ev_w[j*Z]: micro-batch j done.
    LPM_HIP(hipStreamWaitEvent(a.sb, s->ev_fork, 0));
    for (int32_t j = 0; j < M; ++j) {
        if (j >= W) LPM_HIP(hipStreamWaitEvent(a.sf, s->ev_w[(size_t)(j - W) * Z], 0));
        for (int32_t z = 0; z < Z; ++z) if ((rc = fwd_op(s, a, z, j, a.sf))) return rc;
        LPM_HIP(hipEventRecord(s->ev_f[(size_t)j * Z + Z - 1], a.sf));
        LPM_HIP(hipStreamWaitEvent(a.sb, s->ev_f[(size_t)j * Z + Z - 1], 0));
        for (int32_t z = Z - 1; z >= 0; --z) {
            if ((rc = bwd_op(s, a, z, j, a.sb, nullptr))) return rc;
            if (j == M - 1 && (rc = upd_op(s, a, z, a.sb))) return rc;
        }
        if (j + W < M || j == M - 1) LPM_HIP(hipEventRecord(s->ev_w[(size_t)j * Z], a.sb));
    }
    LPM_HIP(hipStreamWaitEvent(a.sf, s->ev_w[(size_t)(M - 1) * Z], 0));
    return LPM_OK;
}

}  // namespace

extern "C" int32_t lpm_schedule_run(lpm_schedule* s, int32_t mode, const void* x_batch, const int32_t* labels,
                                    const void* dy_batch, const lpm_stage_buffers* per_stage, int32_t dx_wanted,
                                    float lr, float mu, float* loss_out, void* stream_fwd, void* stream_bwd) {
    if (!s || !x_batch || !per_stage) return fail(LPM_EINVAL, "NULL argument");
    const int32_t base = mode & 15;
    if ((base != LPM_LOCKED && base != LPM_OVERLAPPED && base != LPM_PIPELINED) || (mode & ~(15 | LPM_GRAPH | LPM_ASYNC_UPDATE)))
        return fail(LPM_EINVAL, "unknown mode %d", mode);
    if (mode & LPM_ASYNC_UPDATE) {
        if (base == LPM_PIPELINED || (mode & LPM_GRAPH)) return fail(LPM_EINVAL, "LPM_ASYNC_UPDATE goes with LPM_LOCKED or LPM_OVERLAPPED, without LPM_GRAPH");
        if (s->window > 2) return fail(LPM_EINVAL, "LPM_ASYNC_UPDATE keeps two weight versions: window must be 1 or 2");
        for (int32_t z = 0; z < s->Z; ++z) {
            const lpm_stage_buffers& b = per_stage[z];
            if (!b.params_alt || (s->st[(size_t)z]->dtype == LPM_BF16 && !b.lowp_alt) || ((uintptr_t)b.params_alt & 255u) || ((uintptr_t)b.lowp_alt & 255u))
                return fail(LPM_EINVAL, "stage %d: LPM_ASYNC_UPDATE needs 256-byte aligned params_alt (and lowp_alt for bf16)", z);
        }
    }
    // Capturing the per-stage streams (many streams forked from and cross-joined inside one capture, plus the
    // backward pass's edits of the capture frontier) ended in a crash inside the runtime's capture code; the
    // combination is refused.  Replay is no faster than enqueueing for a multi-branch graph anyway.
    if (base == LPM_PIPELINED && (mode & LPM_GRAPH)) return fail(LPM_EINVAL, "LPM_PIPELINED cannot be combined with LPM_GRAPH");
    const bool loss = s->st[(size_t)s->Z - 1]->loss;
    if (loss && (!labels || !loss_out)) return fail(LPM_EINVAL, "the last stage holds the loss: labels and loss_out are required");
    if (!loss && !dy_batch) return fail(LPM_EINVAL, "the last stage is not a loss stage: dy_batch is required");
    if (base == LPM_OVERLAPPED && stream_fwd == stream_bwd) return fail(LPM_EINVAL, "LPM_OVERLAPPED needs two distinct streams");
    if (((uintptr_t)x_batch & 255u) || (dy_batch && ((uintptr_t)dy_batch & 255u))) return fail(LPM_EALIGN, "x_batch / dy_batch must be 256-byte aligned");
    for (int32_t z = 0; z < s->Z; ++z) {
        const lpm_stage_buffers& b = per_stage[z];
        if (!b.params || !b.grads || !b.momentum || !b.fwd_ws || !b.bwd_ws) return fail(LPM_EINVAL, "stage %d: NULL buffer", z);
        for (int32_t w = 0; w < s->window; ++w)
            if (!b.stash[w] || !b.act_out[w] || ((z > 0 || dx_wanted) && !b.grad_in[w]))
                return fail(LPM_EINVAL, "stage %d: stash / act_out / grad_in slot %d is NULL", z, w);
    }
    RunArgs a{mode, x_batch, labels, dy_batch, per_stage, dx_wanted, lr, mu, loss_out, (hipStream_t)stream_fwd,
              (hipStream_t)stream_bwd};
    if (!(mode & LPM_GRAPH)) return enqueue(s, a);

    // Captured replay: the graph is keyed by every argument value (pointers included).
    std::vector<unsigned char> key;
    auto put = [&](const void* p, size_t n) { key.insert(key.end(), (const unsigned char*)p, (const unsigned char*)p + n); };
    put(&mode, sizeof mode); put(&x_batch, sizeof x_batch); put(&labels, sizeof labels); put(&dy_batch, sizeof dy_batch);
    put(per_stage, sizeof(lpm_stage_buffers) * (size_t)s->Z); put(&dx_wanted, sizeof dx_wanted);
    put(&lr, sizeof lr); put(&mu, sizeof mu); put(&loss_out, sizeof loss_out); put(&stream_bwd, sizeof stream_bwd);
    for (GraphEntry& g : s->graphs)
        if (g.key == key) {
            LPM_HIP(hipGraphLaunch(g.exec, a.sf));
            return LPM_OK;
        }
    LPM_HIP(hipStreamBeginCapture(a.sf, hipStreamCaptureModeRelaxed));
    const int32_t rc = enqueue(s, a);
    hipGraph_t graph = nullptr;
    const hipError_t e = hipStreamEndCapture(a.sf, &graph);
    if (rc) {
        if (graph) (void)hipGraphDestroy(graph);
        return rc;
    }
    if (e != hipSuccess) return hip_fail(e, "hipStreamEndCapture");
    GraphEntry ge;
    ge.key = key;
    ge.graph = graph;
    const hipError_t ei = hipGraphInstantiate(&ge.exec, graph, nullptr, nullptr, 0);
    if (ei != hipSuccess) {
        (void)hipGraphDestroy(graph);
        return hip_fail(ei, "hipGraphInstantiate");
    }
    if (s->graphs.size() >= 8) {      // bounded cache: drop the oldest
        (void)hipGraphExecDestroy(s->graphs.front().exec);
        (void)hipGraphDestroy(s->graphs.front().graph);
        s->graphs.erase(s->graphs.begin());
    }
    s->graphs.push_back(ge);
    LPM_HIP(hipGraphLaunch(ge.exec, a.sf));
    return LPM_OK;
}
