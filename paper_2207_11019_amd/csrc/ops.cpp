// Single-layer entry points: the contractions of eq. 1 (forward), eq. 9 (data gradient) and eq. 8
// (weight gradient) on their own, for layer-level tests and per-kernel measurement.
#include "lpm_internal.h"
#include <mutex>

using namespace lpm;

static int32_t to_geom(const lpm_conv_geom* g, int32_t dtype, ConvGeom& out) {
    if (!g) return fail(LPM_EINVAL, "geometry is NULL");
    if (dtype != LPM_F32 && dtype != LPM_BF16) return fail(LPM_EINVAL, "dtype must be LPM_F32 or LPM_BF16");
    if (g->m <= 0 || g->h <= 0 || g->w <= 0 || g->cin <= 0 || g->cout <= 0 || g->kh <= 0 || g->kw <= 0 || g->stride <= 0 ||
        g->pad < 0 || g->pad >= g->kh || g->pad >= g->kw)
        return fail(LPM_ESHAPE, "bad convolution geometry");
    const int32_t ho = g->h + 2 * g->pad - g->kh, wo = g->w + 2 * g->pad - g->kw;
    if (ho < 0 || wo < 0) return fail(LPM_ESHAPE, "kernel larger than padded input");
    out = ConvGeom{g->m, g->h, g->w, g->cin, ho / g->stride + 1, wo / g->stride + 1, g->cout, g->kh, g->kw, g->stride, g->pad};
    // volumetric form (0 in d / kd means 1)
    const int32_t d = g->d > 0 ? g->d : 1, kd = g->kd > 0 ? g->kd : 1;
    if (g->d < 0 || g->kd < 0 || g->pad_d < 0 || g->pad_d >= kd || d + 2 * g->pad_d - kd < 0) return fail(LPM_ESHAPE, "bad depth geometry");
    out.D = d; out.Kd = kd; out.pad_d = g->pad_d; out.Do = (d + 2 * g->pad_d - kd) / g->stride + 1;
    return LPM_OK;
}

static bool bad_align(std::initializer_list<const void*> ps) {
    for (const void* p : ps) if (p && ((uintptr_t)p & 255u)) return true;
    return false;
}

extern "C" int32_t lpm_conv_ws_bytes(const lpm_conv_geom* g, int32_t dtype, size_t* fwd, size_t* dgrad, size_t* wgrad) {
    ConvGeom cg;
    int32_t rc = to_geom(g, dtype, cg);
    if (rc) return rc;
    if (fwd) *fwd = fwd_ws_bytes(dtype, cg);
    if (dgrad) *dgrad = dgrad_ws_bytes(dtype, cg);
    if (wgrad) *wgrad = wgrad_ws_bytes(dtype, cg);
    return LPM_OK;
}

extern "C" int32_t lpm_conv_forward(const lpm_conv_geom* g, int32_t dtype, const void* x, const void* w, const float* scale,
                                    const float* bias, const void* add, int32_t relu, void* y, void* ws, void* stream) {
    ConvGeom cg;
    int32_t rc = to_geom(g, dtype, cg);
    if (rc) return rc;
    if (!x || !w || !y) return fail(LPM_EINVAL, "NULL argument");
    if (fwd_ws_bytes(dtype, cg) && !ws) return fail(LPM_EINVAL, "scratch required");
    if (bad_align({x, w, scale, bias, add, y, ws})) return fail(LPM_EALIGN, "device buffers must be 256-byte aligned");
    LPM_HIP(launch_conv_fwd(dtype, cg, x, w, scale, bias, add, relu != 0, y, ws, (hipStream_t)stream));
    return LPM_OK;
}

extern "C" int32_t lpm_conv_dgrad(const lpm_conv_geom* g, int32_t dtype, const void* dz, const void* w, const void* wt,
                                  void* dx, int32_t accumulate, void* ws, void* stream) {
    ConvGeom cg;
    int32_t rc = to_geom(g, dtype, cg);
    if (rc) return rc;
    if (!dz || !w || !dx) return fail(LPM_EINVAL, "NULL argument");
    if (dgrad_ws_bytes(dtype, cg) && !ws) return fail(LPM_EINVAL, "scratch required");
    if (bad_align({dz, w, wt, dx, ws})) return fail(LPM_EALIGN, "device buffers must be 256-byte aligned");
    LPM_HIP(launch_conv_dgrad(dtype, cg, dz, w, wt, dx, accumulate != 0, nullptr, nullptr, ws, (hipStream_t)stream));
    return LPM_OK;
}

extern "C" int32_t lpm_conv_wgrad(const lpm_conv_geom* g, int32_t dtype, const void* x, const void* dz, float* dw,
                                  int32_t accumulate, void* ws, void* stream) {
    ConvGeom cg;
    int32_t rc = to_geom(g, dtype, cg);
    if (rc) return rc;
    if (!x || !dz || !dw) return fail(LPM_EINVAL, "NULL argument");
    if (wgrad_ws_bytes(dtype, cg) && !ws) return fail(LPM_EINVAL, "scratch required");
    if (bad_align({x, dz, dw, ws})) return fail(LPM_EALIGN, "device buffers must be 256-byte aligned");
    LPM_HIP(launch_conv_wgrad(dtype, cg, x, dz, dw, nullptr, nullptr, accumulate != 0, ws, (hipStream_t)stream));
    return LPM_OK;
}

// ---- the weight gradient for callers that cannot allocate -----------------------------------------------------------
// Scratch of lpm_conv_wgrad_static: a fixed area in the library's own device image (every GPU the library runs on holds
// its copy until the process ends).  In host code the array's name is only a handle for hipGetSymbolAddress; the
// device address it yields is what the kernels get.
static __device__ __align__(256) unsigned char scratch[LPM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES];      // per device: address of that device's copy of `scratch`, NULL until asked for
}  // namespace

// Address of the current device's copy (looked up once per device, with that device current).
static int32_t static_scratch(void** out) {
    int dev = 0;
    LPM_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(LPM_EINVAL, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        LPM_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(LPM_EHIP, "hipGetSymbolAddress returned NULL");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LPM_OK;
}

extern "C" int32_t lpm_conv_wgrad_static(const lpm_conv_geom* g, int32_t dtype, const void* x, const void* dz, float* dw,
                                         int32_t accumulate, void* stream) {
    ConvGeom cg;
    int32_t rc = to_geom(g, dtype, cg);
    if (rc) return rc;
    if (!x || !dz || !dw) return fail(LPM_EINVAL, "NULL argument");
    if (bad_align({x, dz, dw})) return fail(LPM_EALIGN, "device buffers must be 256-byte aligned");
    const size_t need = wgrad_ws_bytes(dtype, cg);
    if (need > (size_t)LPM_STATIC_SCRATCH_BYTES)
        return fail(LPM_EINVAL, "this geometry needs %zu bytes of scratch, the built-in area holds %zu: use lpm_conv_wgrad",
                    need, (size_t)LPM_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    if ((rc = static_scratch(&ws))) return rc;
    // (every partial sum a reduction reads is written by the contraction of the same call: nothing has to start at zero)
    LPM_HIP(launch_conv_wgrad(dtype, cg, x, dz, dw, nullptr, nullptr, accumulate != 0, ws, (hipStream_t)stream));
    return LPM_OK;
}

extern "C" int32_t lpm_conv_time(int32_t op, const lpm_conv_geom* g, int32_t dtype, void* x, const void* w, const void* wt,
                                 void* y, float* dw, void* ws, int32_t warmup, int32_t iters, void* stream, float* avg_us) {
    if (op < 0 || op > 2 || iters <= 0 || warmup < 0 || !avg_us) return fail(LPM_EINVAL, "bad op / iteration count");
    hipEvent_t e0 = nullptr, e1 = nullptr;
    LPM_HIP(hipEventCreate(&e0));
    hipError_t he = hipEventCreate(&e1);
    if (he != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(he, "hipEventCreate"); }
    int32_t rc = LPM_OK;
    for (int32_t i = 0; i < warmup + iters && rc == LPM_OK; ++i) {
        if (i == warmup) he = hipEventRecord(e0, (hipStream_t)stream);
        if (op == 0) rc = lpm_conv_forward(g, dtype, x, w, nullptr, nullptr, nullptr, 1, y, ws, stream);
        else if (op == 1) rc = lpm_conv_dgrad(g, dtype, y, w, wt, x, 0, ws, stream);
        else rc = lpm_conv_wgrad(g, dtype, x, y, dw, 1, ws, stream);
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
