// Convolutions whose whole reduction fits a few dozen terms (an image-input first layer: Cin*Kh*Kw <= 32,
// e.g. 3 channels x 3x3): too short for MFMA K tiles, and bound by activation traffic (about 26 flop/B).
// Forward (eq. 1) on the vector ALU with the filter bank in LDS.  bf16 activations, fp32 accumulation.
// (The weight gradient has a long reduction over the pixels and runs on the matrix cores; no data gradient:
// such a layer reads the network input.)
#include "lpm_internal.h"
#include "elem.h"

namespace lpm {

constexpr int SK_MAXK = 32;       // Cin*Kh*Kw
constexpr int SK_MAXCO = 128;

bool smallk_ok(const ConvGeom& g) {
    return g.K() <= SK_MAXK && g.Cout <= SK_MAXCO && g.Cout % 8 == 0 && g.rows_out() < (1ll << 31) / SK_MAXCO;
}

// one thread = one output pixel x 8 output channels
__global__ void __launch_bounds__(256) conv_fwd_smallk(ConvGeom g, const uint16_t* __restrict__ x,
                                                       const uint16_t* __restrict__ w, const float* __restrict__ scale,
                                                       const float* __restrict__ bias, const uint16_t* __restrict__ add,
                                                       int relu, uint16_t* __restrict__ y) {
    __shared__ float ws[SK_MAXK][SK_MAXCO + 1];
    const int K = g.K(), C8 = g.Cout / 8;
    for (int i = threadIdx.x; i < g.Cout * K; i += 256) ws[i % K][i / K] = bf2f(w[i]);
    __syncthreads();
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = idx / C8;
    if (row >= g.rows_out()) return;
    const int c0 = (int)(idx % C8) * 8;
    const int wo = (int)(row % g.Wo), ho = (int)((row / g.Wo) % g.Ho), n = (int)(row / ((int64_t)g.Wo * g.Ho));
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int k = 0;
    for (int kh = 0; kh < g.Kh; ++kh) {
        const int h = ho * g.stride + kh - g.pad;
        for (int kw = 0; kw < g.Kw; ++kw) {
            const int ww = wo * g.stride + kw - g.pad;
            const bool ok = (unsigned)h < (unsigned)g.H && (unsigned)ww < (unsigned)g.W;
            const uint16_t* xp = x + (((int64_t)n * g.H + h) * g.W + ww) * g.Cin;
            for (int ci = 0; ci < g.Cin; ++ci, ++k) {
                const float xv = ok ? bf2f(xp[ci]) : 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = fmaf(xv, ws[k][c0 + j], acc[j]);
            }
        }
    }
    uint32_t out[4];
    const int64_t o = row * g.Cout + c0;
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
        float v0 = acc[j], v1 = acc[j + 1];
        if (scale) { v0 *= scale[c0 + j]; v1 *= scale[c0 + j + 1]; }
        if (bias) { v0 += bias[c0 + j]; v1 += bias[c0 + j + 1]; }
        if (add) { v0 += bf2f(add[o + j]); v1 += bf2f(add[o + j + 1]); }
        if (relu) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); }
        out[j / 2] = pack_bf16x2(v0, v1);
    }
    *reinterpret_cast<uint4*>(y + o) = make_uint4(out[0], out[1], out[2], out[3]);
}

hipError_t smallk_conv_fwd(const ConvGeom& g, const void* x, const void* w, const float* scale, const float* bias,
                           const void* add, int relu, void* y, hipStream_t st) {
    const int64_t total = g.rows_out() * (g.Cout / 8);
    hipLaunchKernelGGL(conv_fwd_smallk, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g, (const uint16_t*)x,
                       (const uint16_t*)w, scale, bias, (const uint16_t*)add, relu, (uint16_t*)y);
    return hipGetLastError();
}

}  // namespace lpm
