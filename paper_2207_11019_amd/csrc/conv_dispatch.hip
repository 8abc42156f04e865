// Chooses the contraction kernel for a convolution / FC shape.
#include "lpm_internal.h"

namespace lpm {

hipError_t conv_fwd_generic_launch(int dtype, const ConvGeom& g, const void* x, const void* w, const float* scale,
                                   const float* bias, const void* add, int relu, void* y, hipStream_t s);
hipError_t conv_dgrad_generic_launch(int dtype, const ConvGeom& g, const void* dz, const void* w, void* dx,
                                     int accumulate, hipStream_t s);
hipError_t conv_wgrad_generic_launch(int dtype, const ConvGeom& g, const void* x, const void* dz, float* dw,
                                     int accumulate, void* ws, hipStream_t s);
size_t wgrad_generic_ws_bytes(const ConvGeom& g);

size_t fwd_ws_bytes(int, const ConvGeom&) { return 0; }
size_t dgrad_ws_bytes(int, const ConvGeom&) { return 0; }
size_t wgrad_ws_bytes(int, const ConvGeom& g) { return wgrad_generic_ws_bytes(g); }

hipError_t launch_conv_fwd(int dtype, const ConvGeom& g, const void* x, const void* w, const float* scale,
                           const float* bias, const void* add, int relu, void* y, void*, hipStream_t st) {
    return conv_fwd_generic_launch(dtype, g, x, w, scale, bias, add, relu, y, st);
}

hipError_t launch_conv_dgrad(int dtype, const ConvGeom& g, const void* dz, const void* w, const void*, void* dx,
                             int accumulate, void*, hipStream_t st) {
    return conv_dgrad_generic_launch(dtype, g, dz, w, dx, accumulate, st);
}

hipError_t launch_conv_wgrad(int dtype, const ConvGeom& g, const void* x, const void* dz, float* dw, int accumulate,
                             void* ws, hipStream_t st) {
    return conv_wgrad_generic_launch(dtype, g, x, dz, dw, accumulate, ws, st);
}

}  // namespace lpm
