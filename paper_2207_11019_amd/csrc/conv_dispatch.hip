// Chooses the contraction kernel for a convolution / FC shape: bf16 MFMA implicit GEMM where the
// channel counts allow 16-byte K chunks, the shape-generic kernels otherwise (float element type,
// 3-channel first layer, 10-class head).
#include "lpm_internal.h"
#include <algorithm>

namespace lpm {

hipError_t conv_fwd_generic_launch(int dtype, const ConvGeom& g, const void* x, const void* w, const float* scale,
                                   const float* bias, const void* add, int relu, void* y, hipStream_t s);
hipError_t conv_dgrad_generic_launch(int dtype, const ConvGeom& g, const void* dz, const float* dzscale, const void* w, void* dx,
                                     int accumulate, const void* mask, const float* mscale, hipStream_t s);
hipError_t conv_wgrad_generic_launch(int dtype, const ConvGeom& g, const void* x, const void* dz, float* dw,
                                     int accumulate, void* ws, hipStream_t s);
size_t wgrad_generic_ws_bytes(const ConvGeom& g);

bool mfma_fwd_ok(const ConvGeom& g);
bool mfma_dgrad_ok(const ConvGeom& g);
bool mfma_wgrad_ok(const ConvGeom& g);
size_t mfma_fwd_ws_bytes(const ConvGeom& g);
size_t mfma_dgrad_ws_bytes(const ConvGeom& g);
size_t mfma_wgrad_ws_bytes(const ConvGeom& g);
bool mfma_fwd_pools(const ConvGeom& g);
hipError_t mfma_conv_fwd(const ConvGeom& g, const void* x, const void* w, const float* scale, const float* bias,
                         const void* add, int relu, void* y, void* ws, hipStream_t st, void* pool_y);
hipError_t mfma_conv_dgrad(const ConvGeom& g, const void* dz, const void* wt, void* dx, int accumulate, const void* mask,
                           const float* mscale, void* ws, hipStream_t st, const UnpoolDesc* unpool, const DgradSide* side);
hipError_t mfma_conv_wgrad(const ConvGeom& g, const void* x, const void* dz, float* dw, float* dbias, const float* rscale,
                           int accumulate, void* ws, hipStream_t st, ReduceDesc* deferred);

bool wgrad_tr_ok(const ConvGeom& g);
size_t wgrad_tr_ws_bytes(const ConvGeom& g);
hipError_t wgrad_tr(const ConvGeom& g, const void* x, const void* dz, float* dw, float* dbias, const float* rscale,
                    int accumulate, void* ws, hipStream_t st, ReduceDesc* deferred);

bool fc_skinny_ok(const ConvGeom& g);
size_t fc_dgrad_ws_bytes(const ConvGeom& g);
hipError_t fc_dgrad(const ConvGeom& g, const void* dz, const float* dzscale, const void* w, void* dx, int accumulate, const void* mask,
                    const float* mscale, void* ws, hipStream_t st);
hipError_t fc_wgrad(const ConvGeom& g, const void* x, const void* dz, float* dw, float* dbias, const float* rscale,
                    int accumulate, hipStream_t st);

bool fc_staged_ok(const ConvGeom& g);
hipError_t fc_wgrad_staged(const ConvGeom& g, const void* xs, const void* dzs, int slots, float* dw, float* dbias,
                           const float* rscale, int accumulate, hipStream_t st);

bool mfma_wgrad_flat_ok(const ConvGeom& g);
size_t mfma_wgrad_flat_ws_bytes(const ConvGeom& g);
hipError_t mfma_conv_wgrad_flat(const ConvGeom& g, const void* x, const void* dz, float* dw, float* dbias,
                                const float* rscale, int accumulate, void* ws, hipStream_t st);

bool smallk_ok(const ConvGeom& g);
hipError_t smallk_conv_fwd(const ConvGeom& g, const void* x, const void* w, const float* scale, const float* bias,
                           const void* add, int relu, void* y, hipStream_t st);

size_t fwd_ws_bytes(int dtype, const ConvGeom& g) { return (dtype == LPM_BF16 && mfma_fwd_ok(g)) ? mfma_fwd_ws_bytes(g) : 0; }
size_t dgrad_ws_bytes(int dtype, const ConvGeom& g) {
    if (dtype == LPM_BF16 && fc_skinny_ok(g)) return std::max(fc_dgrad_ws_bytes(g), mfma_dgrad_ok(g) ? mfma_dgrad_ws_bytes(g) : 0);
    return (dtype == LPM_BF16 && mfma_dgrad_ok(g)) ? mfma_dgrad_ws_bytes(g) : 0;
}
size_t wgrad_ws_bytes(int dtype, const ConvGeom& g) {
    if (dtype == LPM_BF16 && fc_skinny_ok(g)) return 0;
    if (dtype == LPM_BF16 && wgrad_tr_ok(g)) return wgrad_tr_ws_bytes(g);
    if (dtype == LPM_BF16 && mfma_wgrad_ok(g)) return mfma_wgrad_ws_bytes(g);
    if (dtype == LPM_BF16 && mfma_wgrad_flat_ok(g)) return mfma_wgrad_flat_ws_bytes(g);
    return wgrad_generic_ws_bytes(g);
}

bool fwd_can_pool(int dtype, const ConvGeom& g) { return dtype == LPM_BF16 && mfma_fwd_pools(g); }

hipError_t launch_conv_fwd(int dtype, const ConvGeom& g, const void* x, const void* w, const float* scale,
                           const float* bias, const void* add, int relu, void* y, void* ws, hipStream_t st, void* pool_y) {
    if (pool_y && !fwd_can_pool(dtype, g)) return hipErrorInvalidValue;      // callers ask fwd_can_pool first
    if (dtype == LPM_BF16 && mfma_fwd_ok(g)) return mfma_conv_fwd(g, x, w, scale, bias, add, relu, y, ws, st, pool_y);
    if (dtype == LPM_BF16 && smallk_ok(g)) return smallk_conv_fwd(g, x, w, scale, bias, add, relu, y, st);
    return conv_fwd_generic_launch(dtype, g, x, w, scale, bias, add, relu, y, st);
}

bool wgrad_fuses_bias(int dtype, const ConvGeom& g) { return dtype == LPM_BF16 && (fc_skinny_ok(g) || mfma_wgrad_ok(g) || mfma_wgrad_flat_ok(g)); }

// whether the data gradient wants the [Cin][Kh][Kw][Cout] copy of the weights
bool dgrad_uses_wt(int dtype, const ConvGeom& g) { return dtype == LPM_BF16 && !fc_skinny_ok(g) && mfma_dgrad_ok(g); }

// the stride-1 MFMA data gradient can route its result through a following (in forward order: preceding) max-pooling
// (worth it while the kernel is bound by its launch: measured on the 224x224 VGG layers the scattered 2-byte stores
// in the contraction's epilogue cost more than the separate pooling kernel, so large gradients keep that kernel)
bool dgrad_can_unpool(int dtype, const ConvGeom& g) {
    return dtype == LPM_BF16 && !g.is3d() && !fc_skinny_ok(g) && mfma_dgrad_ok(g) && g.stride == 1 &&
           (int64_t)g.rows_in() * g.Cin <= ((int64_t)1 << 20);
}

// the MFMA data gradient can take over the epilogue backward of a layer with a shortcut (DgradSide)
bool dgrad_has_side(int dtype, const ConvGeom& g) { return dgrad_uses_wt(dtype, g); }

hipError_t launch_conv_dgrad(int dtype, const ConvGeom& g, const void* dz, const void* w, const void* wt, void* dx,
                             int accumulate, const void* mask, const float* mscale, void* ws, hipStream_t st,
                             const UnpoolDesc* unpool, const DgradSide* side, const float* dzscale) {
    if (unpool && !(dgrad_can_unpool(dtype, g) && wt)) return hipErrorInvalidValue;      // callers ask dgrad_can_unpool first
    if (side && !(dgrad_has_side(dtype, g) && wt)) return hipErrorInvalidValue;          // ... and dgrad_has_side
    if (dtype == LPM_BF16 && fc_skinny_ok(g)) return fc_dgrad(g, dz, dzscale, w, dx, accumulate, mask, mscale, ws, st);
    if (dtype == LPM_BF16 && wt && mfma_dgrad_ok(g)) return mfma_conv_dgrad(g, dz, wt, dx, accumulate, mask, mscale, ws, st, unpool, side);
    return conv_dgrad_generic_launch(dtype, g, dz, dzscale, w, dx, accumulate, mask, mscale, st);
}

hipError_t launch_conv_wgrad(int dtype, const ConvGeom& g, const void* x, const void* dz, float* dw, float* dbias,
                             const float* rscale, int accumulate, void* ws, hipStream_t st, ReduceDesc* deferred) {
    if (deferred) deferred->splits = 0;
    if (dtype == LPM_BF16 && fc_skinny_ok(g)) return fc_wgrad(g, x, dz, dw, dbias, rscale, accumulate, st);
    if (dtype == LPM_BF16 && wgrad_tr_ok(g)) return wgrad_tr(g, x, dz, dw, dbias, rscale, accumulate, ws, st, deferred);
    if (dtype == LPM_BF16 && mfma_wgrad_ok(g)) return mfma_conv_wgrad(g, x, dz, dw, dbias, rscale, accumulate, ws, st, deferred);
    if (dtype == LPM_BF16 && mfma_wgrad_flat_ok(g)) return mfma_conv_wgrad_flat(g, x, dz, dw, dbias, rscale, accumulate, ws, st);
    if (dbias || rscale) return hipErrorInvalidValue;      // callers ask wgrad_fuses_bias first
    return conv_wgrad_generic_launch(dtype, g, x, dz, dw, accumulate, ws, st);
}

// Staging pays when one read-modify-write pass over dW moves several times the bytes of the staged operands.
bool wgrad_staged_ok(int dtype, const ConvGeom& g) {
    if (dtype != LPM_BF16) return false;
    if (fc_staged_ok(g)) return true;
    if (fc_skinny_ok(g) || !mfma_wgrad_ok(g)) return false;
    const int64_t dw_rmw = (int64_t)g.Cout * g.K() * 8, staged = (g.rows_in() * g.Cin + g.rows_out() * g.Cout) * 2;
    return (int64_t)g.Cout * g.K() >= 32768 && dw_rmw >= 6 * staged;
}

static ConvGeom staged_geom(const ConvGeom& g, int slots) { ConvGeom b = g; b.m = g.m * slots; return b; }

size_t wgrad_staged_ws_bytes(int dtype, const ConvGeom& g) {
    if (!wgrad_staged_ok(dtype, g) || fc_staged_ok(g)) return 0;
    size_t b = 0;
    for (int s = 1; s <= LPM_FC_STAGE_SLOTS; ++s) b = std::max(b, wgrad_ws_bytes(dtype, staged_geom(g, s)));
    return b;
}

hipError_t launch_wgrad_staged(int dtype, const ConvGeom& g, const void* xs, const void* dzs, int slots, float* dw, float* dbias,
                               const float* rscale, int accumulate, void* ws, hipStream_t st, ReduceDesc* deferred) {
    if (deferred) deferred->splits = 0;
    if (fc_staged_ok(g)) return fc_wgrad_staged(g, xs, dzs, slots, dw, dbias, rscale, accumulate, st);
    // the staged micro-batches are one larger batch in the same layout
    return launch_conv_wgrad(dtype, staged_geom(g, slots), xs, dzs, dw, dbias, rscale, accumulate, ws, st, deferred);
}

}  // namespace lpm
