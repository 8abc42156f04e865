// Layer-wise partitioning of one layer ("Layer-wise Partitioning and Merging" section, fig. 1a): the layer's output
// channels are split into n equal sub-layers, each sub-layer is computed on its own (own weights slice, own launch,
// own stream -- the stand-in for the paper's n devices), and the sub-layer outputs are concatenated before the next
// layer.  Backward, the incoming gradient is re-partitioned by channel, every sub-layer produces its slice of the
// weight gradient and a full-size partial input gradient, and the partials are summed in a fixed order.  The results
// equal those of the merged layer; what differs is the extra traffic (concatenate, re-partition, sum) and the smaller
// contractions -- the overhead that the paper's merging operation removes, which lpm_layerwise_time measures.
#include "lpm_internal.h"
#include <algorithm>
#include <initializer_list>
#include <new>

using namespace lpm;

struct lpm_layerwise {
    ConvGeom g;         // the merged layer
    ConvGeom gs;        // one sub-layer (Cout / n output channels)
    int32_t dtype, n;
    size_t es;          // bytes per activation element
    size_t y_bytes, dz_bytes, dx_bytes, fwd_ws, bwd_ws;      // per sub-layer, each a multiple of 256
    hipEvent_t fork, join[8];
    hipStream_t probed_for;   // the caller stream sub[] was chosen for (NULL: not yet)
    hipStream_t sub[8];       // stream of sub-layer i
};

namespace {

size_t up256(size_t b) { return (b + 255) & ~(size_t)255; }

// SPLIT = false: merged[r][part * cn + c] = parts[part][r][c] (concatenation along the channel axis);
// SPLIT = true: the inverse (re-partition of a merged tensor).  Moves 16-byte chunks; cn * es is a multiple of 16.
template <bool SPLIT>
__global__ void __launch_bounds__(256) layerwise_regroup(const uint4* __restrict__ merged_in, uint4* __restrict__ merged_out,
                                                         const uint4* __restrict__ parts_in, uint4* __restrict__ parts_out,
                                                         int64_t rows, int chunks_per_part, int n, int64_t part_stride_chunks) {
    const int64_t total = rows * chunks_per_part * n;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / ((int64_t)chunks_per_part * n);
        const int q = (int)(i - r * chunks_per_part * n);
        const int part = q / chunks_per_part, c = q - part * chunks_per_part;
        const int64_t pi = (int64_t)part * part_stride_chunks + r * chunks_per_part + c;
        if (SPLIT) parts_out[pi] = merged_in[i];
        else merged_out[i] = parts_in[pi];
    }
}

__device__ inline float bf16_to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ inline uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// dx[i] = sum over parts (in part order) of partial[part][i]; fp32 sum, one rounding for bf16
template <bool BF16>
__global__ void __launch_bounds__(256) layerwise_sum(const void* __restrict__ partial, void* __restrict__ dx, int64_t count, int n,
                                                     int64_t part_stride_elems) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) {
        float s = 0.f;
        for (int p = 0; p < n; ++p) {
            if (BF16) s += bf16_to_f32(((const uint16_t*)partial)[p * part_stride_elems + i]);
            else s += ((const float*)partial)[p * part_stride_elems + i];
        }
        if (BF16) ((uint16_t*)dx)[i] = f32_to_bf16(s);
        else ((float*)dx)[i] = s;
    }
}

// Streams of the n sub-layers for a caller stream st: the runtime maps streams onto four hardware queues that each run
// their kernels one after the other, so "n devices" are best imitated by st itself plus up to three pooled streams
// measured to sit on other queues (streams_share_queue); further sub-layers share them round-robin.
int32_t choose_streams(lpm_layerwise* L, hipStream_t st) {
    if (L->probed_for == st && L->sub[0]) return LPM_OK;
    hipStream_t got[3] = {nullptr, nullptr, nullptr};
    int found = 0;
    const hipStream_t taken[1] = {st};
    LPM_HIP(pick_concurrent_streams(taken, 1, got, std::min(3, L->n - 1), &found));
    hipStream_t set[4] = {st, got[0], got[1], got[2]};
    const int have = 1 + found;
    for (int i = 0; i < L->n; ++i) L->sub[i] = set[(i + 1) % have];      // the caller's stream takes the last of every round
    L->probed_for = st;
    return LPM_OK;
}

unsigned blocks_for(int64_t work) { return (unsigned)std::min<int64_t>((work + 255) / 256, 256 * 8); }

bool misaligned(std::initializer_list<const void*> ps) {
    for (const void* p : ps) if (p && ((uintptr_t)p & 255u)) return true;
    return false;
}

}  // namespace

extern "C" int32_t lpm_layerwise_create(const lpm_conv_geom* g, int32_t dtype, int32_t n, lpm_layerwise** out) {
    if (!g || !out) return fail(LPM_EINVAL, "NULL argument");
    if (dtype != LPM_F32 && dtype != LPM_BF16) return fail(LPM_EINVAL, "dtype must be LPM_F32 or LPM_BF16");
    if (n < 2 || n > 8) return fail(LPM_EINVAL, "n must be 2..8");
    if (g->m <= 0 || g->h <= 0 || g->w <= 0 || g->cin <= 0 || g->cout <= 0 || g->kh <= 0 || g->kw <= 0 || g->stride <= 0 ||
        g->pad < 0 || g->pad >= g->kh || g->pad >= g->kw || g->h + 2 * g->pad < g->kh || g->w + 2 * g->pad < g->kw)
        return fail(LPM_ESHAPE, "bad convolution geometry");
    if (g->cout % n || (g->cout / n) % 8) return fail(LPM_ESHAPE, "cout / n must be a whole multiple of 8 channels");
    if (g->d > 1 || g->kd > 1) return fail(LPM_ESHAPE, "layer-wise partitioning takes two-dimensional layers");
    lpm_layerwise* L = new (std::nothrow) lpm_layerwise{};
    if (!L) return fail(LPM_ENOMEM, "out of host memory");
    const int32_t ho = (g->h + 2 * g->pad - g->kh) / g->stride + 1, wo = (g->w + 2 * g->pad - g->kw) / g->stride + 1;
    L->g = ConvGeom{g->m, g->h, g->w, g->cin, ho, wo, g->cout, g->kh, g->kw, g->stride, g->pad};
    L->gs = L->g;
    L->gs.Cout = g->cout / n;
    L->dtype = dtype;
    L->n = n;
    L->es = dtype == LPM_BF16 ? 2 : 4;
    L->y_bytes = up256((size_t)L->gs.rows_out() * L->gs.Cout * L->es);
    L->dz_bytes = L->y_bytes;
    L->dx_bytes = up256((size_t)L->g.rows_in() * L->g.Cin * L->es);
    L->fwd_ws = up256(fwd_ws_bytes(dtype, L->gs));
    L->bwd_ws = up256(std::max(dgrad_ws_bytes(dtype, L->gs), wgrad_ws_bytes(dtype, L->gs)));
    hipError_t e = hipEventCreateWithFlags(&L->fork, hipEventDisableTiming);
    for (int i = 0; i < n && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&L->join[i], hipEventDisableTiming);
    if (e != hipSuccess) {
        lpm_layerwise_destroy(L);
        return hip_fail(e, "hipEventCreateWithFlags");
    }
    *out = L;
    return LPM_OK;
}

extern "C" int32_t lpm_layerwise_destroy(lpm_layerwise* L) {
    if (!L) return LPM_OK;
    if (L->fork) (void)hipEventDestroy(L->fork);
    for (int i = 0; i < 8; ++i) if (L->join[i]) (void)hipEventDestroy(L->join[i]);
    delete L;
    return LPM_OK;
}

extern "C" int32_t lpm_layerwise_ws_bytes(const lpm_layerwise* L, size_t* forward, size_t* backward) {
    if (!L) return fail(LPM_EINVAL, "NULL handle");
    if (forward) *forward = (size_t)L->n * (L->y_bytes + L->fwd_ws);
    if (backward) *backward = (size_t)L->n * (L->dz_bytes + L->dx_bytes + L->bwd_ws);
    return LPM_OK;
}

extern "C" int32_t lpm_layerwise_forward(lpm_layerwise* L, const void* x, const void* w, const float* scale, const float* bias,
                                         int32_t relu, void* y, void* ws, void* stream) {
    if (!L || !x || !w || !y || !ws) return fail(LPM_EINVAL, "NULL argument");
    if (misaligned({x, w, scale, bias, y, ws})) return fail(LPM_EALIGN, "device buffers must be 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    int32_t src = choose_streams(L, st);
    if (src) return src;
    hipStream_t* sub = L->sub;
    const int cn = L->gs.Cout;
    const size_t w_slice = (size_t)cn * L->g.K() * L->es;
    char* yparts = (char*)ws;
    char* scratch = yparts + (size_t)L->n * L->y_bytes;
    LPM_HIP(hipEventRecord(L->fork, st));
    for (int i = 0; i < L->n; ++i) {
        LPM_HIP(hipStreamWaitEvent(sub[i], L->fork, 0));
        LPM_HIP(launch_conv_fwd(L->dtype, L->gs, x, (const char*)w + i * w_slice, scale ? scale + i * cn : nullptr,
                                bias ? bias + i * cn : nullptr, nullptr, relu != 0, yparts + i * L->y_bytes,
                                scratch + i * L->fwd_ws, sub[i]));
        LPM_HIP(hipEventRecord(L->join[i], sub[i]));
    }
    for (int i = 0; i < L->n; ++i) LPM_HIP(hipStreamWaitEvent(st, L->join[i], 0));
    // concatenation of the sub-layer outputs along the channel axis
    const int chunks = (int)((size_t)cn * L->es / 16);
    const int64_t rows = L->g.rows_out();
    hipLaunchKernelGGL(layerwise_regroup<false>, dim3(blocks_for(rows * chunks * L->n)), dim3(256), 0, st, nullptr, (uint4*)y,
                       (const uint4*)yparts, nullptr, rows, chunks, L->n, (int64_t)(L->y_bytes / 16));
    LPM_HIP(hipGetLastError());
    return LPM_OK;
}

extern "C" int32_t lpm_layerwise_backward(lpm_layerwise* L, const void* x, const void* dz, const void* w, const void* wt,
                                          void* dx, float* dw, int32_t accumulate, void* ws, void* stream) {
    if (!L || !x || !dz || !w || !dw || !ws) return fail(LPM_EINVAL, "NULL argument");
    if (misaligned({x, dz, w, wt, dx, dw, ws})) return fail(LPM_EALIGN, "device buffers must be 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    int32_t src = choose_streams(L, st);
    if (src) return src;
    hipStream_t* sub = L->sub;
    const int cn = L->gs.Cout;
    const size_t w_slice = (size_t)cn * L->g.K() * L->es;          // also the size of one sub-layer's transposed weights
    const size_t dw_slice = (size_t)cn * L->g.K();
    char* dzparts = (char*)ws;
    char* dxparts = dzparts + (size_t)L->n * L->dz_bytes;
    char* scratch = dxparts + (size_t)L->n * L->dx_bytes;
    // the incoming gradient, re-partitioned by output channel
    const int chunks = (int)((size_t)cn * L->es / 16);
    const int64_t rows = L->g.rows_out();
    hipLaunchKernelGGL(layerwise_regroup<true>, dim3(blocks_for(rows * chunks * L->n)), dim3(256), 0, st, (const uint4*)dz, nullptr,
                       nullptr, (uint4*)dzparts, rows, chunks, L->n, (int64_t)(L->dz_bytes / 16));
    LPM_HIP(hipGetLastError());
    LPM_HIP(hipEventRecord(L->fork, st));
    for (int i = 0; i < L->n; ++i) {
        LPM_HIP(hipStreamWaitEvent(sub[i], L->fork, 0));
        const char* dzi = dzparts + i * L->dz_bytes;
        if (dx)
            LPM_HIP(launch_conv_dgrad(L->dtype, L->gs, dzi, (const char*)w + i * w_slice, wt ? (const char*)wt + i * w_slice : nullptr,
                                      dxparts + i * L->dx_bytes, 0, nullptr, nullptr, scratch + i * L->bwd_ws, sub[i]));
        LPM_HIP(launch_conv_wgrad(L->dtype, L->gs, x, dzi, dw + i * dw_slice, nullptr, nullptr, accumulate != 0,
                                  scratch + i * L->bwd_ws, sub[i]));
        LPM_HIP(hipEventRecord(L->join[i], sub[i]));
    }
    for (int i = 0; i < L->n; ++i) LPM_HIP(hipStreamWaitEvent(st, L->join[i], 0));
    if (dx) {
        const int64_t count = L->g.rows_in() * L->g.Cin;
        if (L->dtype == LPM_BF16)
            hipLaunchKernelGGL(layerwise_sum<true>, dim3(blocks_for(count)), dim3(256), 0, st, dxparts, dx, count, L->n,
                               (int64_t)(L->dx_bytes / 2));
        else
            hipLaunchKernelGGL(layerwise_sum<false>, dim3(blocks_for(count)), dim3(256), 0, st, dxparts, dx, count, L->n,
                               (int64_t)(L->dx_bytes / 4));
        LPM_HIP(hipGetLastError());
    }
    return LPM_OK;
}

extern "C" int32_t lpm_layerwise_time(lpm_layerwise* L, int32_t op, const void* x, const void* w, const void* wt, void* y, void* dx,
                                      float* dw, void* ws, int32_t warmup, int32_t iters, void* stream, float* avg_us) {
    if (!L || op < 0 || op > 1 || iters <= 0 || warmup < 0 || !avg_us) return fail(LPM_EINVAL, "bad op / iteration count");
    hipEvent_t e0 = nullptr, e1 = nullptr;
    LPM_HIP(hipEventCreate(&e0));
    hipError_t he = hipEventCreate(&e1);
    if (he != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(he, "hipEventCreate"); }
    int32_t rc = LPM_OK;
    for (int32_t i = 0; i < warmup + iters && rc == LPM_OK; ++i) {
        if (i == warmup) he = hipEventRecord(e0, (hipStream_t)stream);
        if (op == 0) rc = lpm_layerwise_forward(L, x, w, nullptr, nullptr, 1, y, ws, stream);
        else rc = lpm_layerwise_backward(L, x, y, w, wt, dx, dw, 1, ws, stream);
    }
    if (rc == LPM_OK && he == hipSuccess) he = hipEventRecord(e1, (hipStream_t)stream);
    if (rc == LPM_OK && he == hipSuccess) he = hipEventSynchronize(e1);
    float ms = 0.f;
    if (rc == LPM_OK && he == hipSuccess) he = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != LPM_OK) return rc;
    if (he != hipSuccess) return hip_fail(he, "event timing");
    *avg_us = ms * 1000.f / (float)iters;
    return LPM_OK;
}
