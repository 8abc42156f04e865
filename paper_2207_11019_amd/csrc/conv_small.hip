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
    return !g.is3d() && g.K() <= SK_MAXK && g.Cout <= SK_MAXCO && g.Cout % 8 == 0 && g.rows_out() < (1ll << 31) / SK_MAXCO;
}

// one thread = PX output pixels (consecutive rows of the flattened output) x 8 output channels: the filter values
// read from LDS serve all PX pixels.  PX = 1 for small launches (more threads, bound by latency), 4 for large ones
// (bound by the LDS reads: 216 per thread for a 3x3x3 filter, whatever PX).
template <int PX>
__global__ void __launch_bounds__(256) conv_fwd_smallk(ConvGeom g, const uint16_t* __restrict__ x,
                                                       const uint16_t* __restrict__ w, const float* __restrict__ scale,
                                                       const float* __restrict__ bias, const uint16_t* __restrict__ add,
                                                       int relu, uint16_t* __restrict__ y) {
    __shared__ float ws[SK_MAXK][SK_MAXCO + 1];
    const int K = g.K(), C8 = g.Cout / 8;
    for (int i = threadIdx.x; i < g.Cout * K; i += 256) ws[i % K][i / K] = bf2f(w[i]);
    __syncthreads();
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row0 = (idx / C8) * PX;
    if (row0 >= g.rows_out()) return;
    const int c0 = (int)(idx % C8) * 8;
    float acc[PX][8];
    int ho[PX], wo[PX], n[PX];
    bool live[PX];
#pragma unroll
    for (int q = 0; q < PX; ++q) {
        const int64_t row = row0 + q;
        live[q] = row < g.rows_out();
        const int64_t r = live[q] ? row : row0;
        wo[q] = (int)(r % g.Wo); ho[q] = (int)((r / g.Wo) % g.Ho); n[q] = (int)(r / ((int64_t)g.Wo * g.Ho));
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[q][j] = 0.f;
    }
    int k = 0;
    for (int kh = 0; kh < g.Kh; ++kh) {
        for (int kw = 0; kw < g.Kw; ++kw) {
            const uint16_t* xp[PX];
            bool ok[PX];
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                const int h = ho[q] * g.stride + kh - g.pad, ww = wo[q] * g.stride + kw - g.pad;
                ok[q] = (unsigned)h < (unsigned)g.H && (unsigned)ww < (unsigned)g.W;
                xp[q] = x + (((int64_t)n[q] * g.H + h) * g.W + ww) * g.Cin;
            }
            for (int ci = 0; ci < g.Cin; ++ci, ++k) {
                float xv[PX];
#pragma unroll
                for (int q = 0; q < PX; ++q) xv[q] = ok[q] ? bf2f(xp[q][ci]) : 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float wv = ws[k][c0 + j];
#pragma unroll
                    for (int q = 0; q < PX; ++q) acc[q][j] = fmaf(xv[q], wv, acc[q][j]);
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < PX; ++q) {
        if (!live[q]) continue;
        uint32_t out[4];
        const int64_t o = (row0 + q) * g.Cout + c0;
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
            float v0 = acc[q][j], v1 = acc[q][j + 1];
            if (scale) { v0 *= scale[c0 + j]; v1 *= scale[c0 + j + 1]; }
            if (bias) { v0 += bias[c0 + j]; v1 += bias[c0 + j + 1]; }
            if (add) { v0 += bf2f(add[o + j]); v1 += bf2f(add[o + j + 1]); }
            if (relu) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); }
            out[j / 2] = pack_bf16x2(v0, v1);
        }
        *reinterpret_cast<uint4*>(y + o) = make_uint4(out[0], out[1], out[2], out[3]);
    }
}

hipError_t smallk_conv_fwd(const ConvGeom& g, const void* x, const void* w, const float* scale, const float* bias,
                           const void* add, int relu, void* y, hipStream_t st) {
    if (g.rows_out() >= 131072) {
        const int64_t total = ((g.rows_out() + 3) / 4) * (g.Cout / 8);
        hipLaunchKernelGGL(conv_fwd_smallk<4>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g, (const uint16_t*)x,
                           (const uint16_t*)w, scale, bias, (const uint16_t*)add, relu, (uint16_t*)y);
        return hipGetLastError();
    }
    const int64_t total = g.rows_out() * (g.Cout / 8);
    hipLaunchKernelGGL(conv_fwd_smallk<1>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g, (const uint16_t*)x,
                       (const uint16_t*)w, scale, bias, (const uint16_t*)add, relu, (uint16_t*)y);
    return hipGetLastError();
}

}  // namespace lpm
