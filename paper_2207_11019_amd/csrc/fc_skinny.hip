// Fully connected layers at a micro-batch of a few samples: one row of K = Kh*Kw*Cin inputs per sample, so the
// three contractions do a handful of multiply-adds per weight and are bound by streaming the weight matrix
// (or its fp32 gradient) once.  Data gradient (eq. 9) and weight gradient (eq. 8) on the vector ALU with
// 16-byte accesses along K; the forward pass (eq. 1) already streams K-contiguous rows through the MFMA kernel.
//   x  [m][K] bf16      w  [Cout][K] bf16      dz [m][Cout] bf16      dW [Cout][K] fp32
#include "lpm_internal.h"
#include "elem.h"
#include <algorithm>

namespace lpm {

hipError_t launch_splitk_epilogue(const float* part, int splits, int64_t MN, int N, const float* scale, const float* bias,
                                  const void* add, int relu, int accumulate, const void* mask, const float* mscale,
                                  void* C, hipStream_t st);

constexpr int FC_MAX_M = 8;       // beyond this the per-lane accumulators no longer fit the register file

bool fc_skinny_ok(const ConvGeom& g) {
    return !g.is3d() && g.Ho == 1 && g.Wo == 1 && g.Kh == g.H && g.Kw == g.W && g.pad == 0 && g.m <= FC_MAX_M && g.K() % 8 == 0 &&
           (int64_t)g.m * g.K() < ((int64_t)1 << 31);
}

__device__ __forceinline__ void unpack8(const uint4 v, float (&f)[8]) {
    f[0] = bf2f((uint16_t)(v.x & 0xffffu)); f[1] = bf2f((uint16_t)(v.x >> 16));
    f[2] = bf2f((uint16_t)(v.y & 0xffffu)); f[3] = bf2f((uint16_t)(v.y >> 16));
    f[4] = bf2f((uint16_t)(v.z & 0xffffu)); f[5] = bf2f((uint16_t)(v.z >> 16));
    f[6] = bf2f((uint16_t)(v.w & 0xffffu)); f[7] = bf2f((uint16_t)(v.w >> 16));
}

// ---- data gradient: part[split][r][k] = sum over the split's output channels of dz[r][co] * w[co][k] ------
// Block = 4 wavefronts over the same 512 columns of K (a lane owns 8), each on every fourth channel of the
// block's range; the four partial sums are added through LDS in wavefront order.
constexpr int FCD_COLS = 512, FCD_MAX_CPS = 256;

template <int MB>
__global__ void __launch_bounds__(256) fc_dgrad_skinny(const uint16_t* __restrict__ dz, const float* __restrict__ dzscale,
                                                       const uint16_t* __restrict__ w, float* __restrict__ part, int m, int Cout,
                                                       int K, int cps) {
    __shared__ float dzs[MB][FCD_MAX_CPS];
    __shared__ float red[MB][FCD_COLS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int k0 = blockIdx.x * FCD_COLS + lane * 8;
    const bool kok = k0 < K;
    const int c0 = blockIdx.y * cps, cn = min(cps, Cout - c0);
    for (int i = tid; i < MB * cn; i += 256) {
        const int r = i / cn, c = i - r * cn;
        dzs[r][c] = r < m ? bf2f(dz[(size_t)r * Cout + c0 + c]) * (dzscale ? dzscale[c0 + c] : 1.f) : 0.f;
    }
    __syncthreads();
    float acc[MB][8];
#pragma unroll
    for (int r = 0; r < MB; ++r)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[r][j] = 0.f;
    if (kok) {
        const uint16_t* wp = w + (size_t)c0 * K + k0;
        int c = wave;
        // four channels per step: the loads are issued together
        for (; c + 12 < cn; c += 16) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const uint4*>(wp + (size_t)(c + 4 * u) * K);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float f[8];
                unpack8(v[u], f);
#pragma unroll
                for (int r = 0; r < MB; ++r) {
                    const float d = dzs[r][c + 4 * u];
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[r][j] = fmaf(d, f[j], acc[r][j]);
                }
            }
        }
        for (; c < cn; c += 4) {
            float f[8];
            unpack8(*reinterpret_cast<const uint4*>(wp + (size_t)c * K), f);
#pragma unroll
            for (int r = 0; r < MB; ++r) {
                const float d = dzs[r][c];
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[r][j] = fmaf(d, f[j], acc[r][j]);
            }
        }
    }
    // wavefronts 1..3 hand their sums to wavefront 0, one after the other
    for (int src = 1; src < 4; ++src) {
        __syncthreads();
        if (wave == src) {
#pragma unroll
            for (int r = 0; r < MB; ++r)
#pragma unroll
                for (int j = 0; j < 8; ++j) red[r][lane * 8 + j] = acc[r][j];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int r = 0; r < MB; ++r)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[r][j] += red[r][lane * 8 + j];
        }
    }
    if (wave == 0 && kok) {
#pragma unroll
        for (int r = 0; r < MB; ++r) {
            if (r >= m) break;
            float4* o = reinterpret_cast<float4*>(part + ((size_t)blockIdx.y * m + r) * K + k0);
            o[0] = make_float4(acc[r][0], acc[r][1], acc[r][2], acc[r][3]);
            o[1] = make_float4(acc[r][4], acc[r][5], acc[r][6], acc[r][7]);
        }
    }
}

struct FcDgradPlan { int colblocks, splits, cps; };

static FcDgradPlan plan_fc_dgrad(const ConvGeom& g) {
    FcDgradPlan p{};
    p.colblocks = (g.K() + FCD_COLS - 1) / FCD_COLS;
    int s = (1536 + p.colblocks - 1) / p.colblocks;          // enough blocks to cover the memory latency
    s = std::min(s, std::max(1, g.Cout / 32));                // at least 32 channels per block
    s = std::min(s, 32);                                      // the reduction kernel adds the partials one after the other
    s = std::max(s, (g.Cout + FCD_MAX_CPS - 1) / FCD_MAX_CPS);
    p.cps = (g.Cout + s - 1) / s;
    p.splits = (g.Cout + p.cps - 1) / p.cps;
    return p;
}

size_t fc_dgrad_ws_bytes(const ConvGeom& g) { return (size_t)plan_fc_dgrad(g).splits * g.m * g.K() * sizeof(float); }

// dzscale (may be NULL): dz is the gradient before the layer's per-channel scale; channel co is multiplied by dzscale[co]
hipError_t fc_dgrad(const ConvGeom& g, const void* dz, const float* dzscale, const void* w, void* dx, int accumulate, const void* mask,
                    const float* mscale, void* ws, hipStream_t st) {
    const FcDgradPlan p = plan_fc_dgrad(g);
    const dim3 grid((unsigned)p.colblocks, (unsigned)p.splits);
    const int K = g.K();
#define LPM_FCD(MB) hipLaunchKernelGGL((fc_dgrad_skinny<MB>), grid, dim3(256), 0, st, (const uint16_t*)dz, dzscale, (const uint16_t*)w, \
                                       (float*)ws, g.m, g.Cout, K, p.cps)
    if (g.m <= 4) LPM_FCD(4);
    else LPM_FCD(8);
#undef LPM_FCD
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // the epilogue's channel index is (element index) % Cin: K is a multiple of Cin
    return launch_splitk_epilogue((const float*)ws, p.splits, (int64_t)g.m * K, g.Cin, nullptr, nullptr, nullptr, 0, accumulate,
                                  mask, mscale, dx, st);
}

// ---- weight gradient: dW[co][k] (+)= rscale[co] * sum_r dz[r][co] * x[r][k];  db[co] (+)= sum_r dz[r][co] ----
// (rscale, may be NULL: the layer's per-channel scale; dz is the gradient before that scale)
// A thread keeps its 8 columns of every sample in registers and walks the block's output channels, reading
// (when accumulating) and writing 32 bytes of dW per channel: one pass over the gradient matrix.
constexpr int FCW_CPB = 16;

template <int MB>
__global__ void __launch_bounds__(256) fc_wgrad_skinny(const uint16_t* __restrict__ x, const uint16_t* __restrict__ dz,
                                                       float* __restrict__ dw, float* __restrict__ db,
                                                       const float* __restrict__ rscale, int m, int Cout, int K,
                                                       int accumulate) {
    __shared__ float dzs[MB][FCW_CPB];
    const int tid = threadIdx.x;
    const int k0 = (blockIdx.x * blockDim.x + tid) * 8;
    const int c0 = blockIdx.y * FCW_CPB, cn = min(FCW_CPB, Cout - c0);
    for (int i = tid; i < MB * FCW_CPB; i += blockDim.x) {
        const int r = i / FCW_CPB, c = i % FCW_CPB;
        dzs[r][c] = (r < m && c < cn) ? bf2f(dz[(size_t)r * Cout + c0 + c]) : 0.f;
    }
    __syncthreads();
    if (db && blockIdx.x == 0 && tid < cn) {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < MB; ++r) s += dzs[r][tid];
        const int co = c0 + tid;
        db[co] = accumulate ? db[co] + s : s;
    }
    if (rscale) {                                   // from here on the block's dz values carry the layer's scale
        __syncthreads();
        for (int i = tid; i < MB * FCW_CPB; i += blockDim.x) {
            const int c = i % FCW_CPB;
            if (c < cn) dzs[i / FCW_CPB][c] *= rscale[c0 + c];
        }
        __syncthreads();
    }
    if (k0 >= K) return;
    float xr[MB][8];
#pragma unroll
    for (int r = 0; r < MB; ++r) {
        if (r < m) unpack8(*reinterpret_cast<const uint4*>(x + (size_t)r * K + k0), xr[r]);
        else {
#pragma unroll
            for (int j = 0; j < 8; ++j) xr[r][j] = 0.f;
        }
    }
    float4* row = reinterpret_cast<float4*>(dw + (size_t)c0 * K + k0);
    const size_t rs = (size_t)K / 4;      // float4 per row
    for (int c = 0; c < cn; c += 4) {
        float4 a[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a[u][0] = make_float4(0.f, 0.f, 0.f, 0.f);
            a[u][1] = a[u][0];
            if (accumulate && c + u < cn) { a[u][0] = row[(size_t)(c + u) * rs]; a[u][1] = row[(size_t)(c + u) * rs + 1]; }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (c + u >= cn) break;
            float g8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < MB; ++r) {
                const float d = dzs[r][c + u];
#pragma unroll
                for (int j = 0; j < 8; ++j) g8[j] = fmaf(d, xr[r][j], g8[j]);
            }
            row[(size_t)(c + u) * rs] = make_float4(a[u][0].x + g8[0], a[u][0].y + g8[1], a[u][0].z + g8[2], a[u][0].w + g8[3]);
            row[(size_t)(c + u) * rs + 1] = make_float4(a[u][1].x + g8[4], a[u][1].y + g8[5], a[u][1].z + g8[6], a[u][1].w + g8[7]);
        }
    }
}

hipError_t fc_wgrad(const ConvGeom& g, const void* x, const void* dz, float* dw, float* dbias, const float* rscale,
                    int accumulate, hipStream_t st) {
    const int K = g.K();
    const int threads = std::min(256, ((K / 8 + 63) / 64) * 64);
    const dim3 grid((unsigned)((K / 8 + threads - 1) / threads), (unsigned)((g.Cout + FCW_CPB - 1) / FCW_CPB));
#define LPM_FCW(MB) hipLaunchKernelGGL((fc_wgrad_skinny<MB>), grid, dim3(threads), 0, st, (const uint16_t*)x, (const uint16_t*)dz, \
                                       dw, dbias, rscale, g.m, g.Cout, K, accumulate)
    if (g.m <= 4) LPM_FCW(4);
    else LPM_FCW(8);
#undef LPM_FCW
    return hipGetLastError();
}

// ---- the same weight gradient contracted once per mini-batch ----------------------------------------------
// Accumulating dW micro-batch by micro-batch reads and writes the whole fp32 gradient matrix every time (822 MB
// per micro-batch for a 25088 x 4096 layer).  A schedule that knows all M micro-batches of the mini-batch can
// instead keep the layer's inputs and output gradients -- a few rows each -- and contract over all M*m rows at
// the last one: dW is written once.  (The sum over the rows is the same; only its rounding order differs.)
bool fc_staged_ok(const ConvGeom& g) {
    return fc_skinny_ok(g) && ((int64_t)g.m * g.Cout) % 8 == 0 && (int64_t)g.Cout * g.K() >= 32768;
}

__global__ void __launch_bounds__(256) fc_stage_copy(const uint4* __restrict__ x, uint4* __restrict__ xs, int nx,
                                                     const uint4* __restrict__ dz, uint4* __restrict__ dzs, int nd) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < nx) xs[i] = x[i];
    else if (i - nx < nd) dzs[i - nx] = dz[i - nx];
}

// a layer's input and output gradient of micro-batch `slot` into the staging areas (xs [slots][m][H][W][Cin],
// dzs [slots][m][Ho][Wo][Cout], bf16; both sizes are multiples of 16 bytes)
hipError_t stage_operands(const ConvGeom& g, const void* x, const void* dz, void* xs, void* dzs, int slot, hipStream_t st) {
    const int nx = (int)((size_t)g.rows_in() * g.Cin * 2 / 16), nd = (int)((size_t)g.rows_out() * g.Cout * 2 / 16);
    hipLaunchKernelGGL(fc_stage_copy, dim3((unsigned)((nx + nd + 255) / 256)), dim3(256), 0, st, (const uint4*)x,
                       (uint4*)xs + (size_t)slot * nx, nx, (const uint4*)dz, (uint4*)dzs + (size_t)slot * nd, nd);
    return hipGetLastError();
}

// dW[co][k] (+)= sum over R rows of dz[r][co] * x[r][k]: a thread owns 8 columns of 16 output channels and walks the
// rows 8 at a time (dz of the block's channels sits in LDS as floats, read as broadcasts).
constexpr int FCR_CPB = 16;
__global__ void __launch_bounds__(256) fc_wgrad_rows(const uint16_t* __restrict__ x, const uint16_t* __restrict__ dz,
                                                     float* __restrict__ dw, float* __restrict__ db,
                                                     const float* __restrict__ rscale, int R, int Cout, int K, int accumulate) {
    extern __shared__ float dzr[];               // [R rounded up to 8][FCR_CPB]
    const int tid = threadIdx.x;
    const int k0 = (blockIdx.x * blockDim.x + tid) * 8;
    const int c0 = blockIdx.y * FCR_CPB, cn = min(FCR_CPB, Cout - c0);
    const int R8 = (R + 7) & ~7;
    for (int i = tid; i < R8 * FCR_CPB; i += blockDim.x) {
        const int r = i / FCR_CPB, c = i % FCR_CPB;
        dzr[i] = (r < R && c < cn) ? bf2f(dz[(size_t)r * Cout + c0 + c]) : 0.f;
    }
    __syncthreads();
    if (db && blockIdx.x == 0 && tid < cn) {
        float sum = 0.f;
        for (int r = 0; r < R; ++r) sum += dzr[r * FCR_CPB + tid];
        const int co = c0 + tid;
        db[co] = accumulate ? db[co] + sum : sum;
    }
    if (rscale) {
        __syncthreads();
        for (int i = tid; i < R8 * FCR_CPB; i += blockDim.x) {
            const int c = i % FCR_CPB;
            if (c < cn) dzr[i] *= rscale[c0 + c];
        }
        __syncthreads();
    }
    if (k0 >= K) return;
    float acc[FCR_CPB][8];
#pragma unroll
    for (int c = 0; c < FCR_CPB; ++c)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[c][j] = 0.f;
    for (int rg = 0; rg < R8; rg += 8) {
        float xr[8][8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (rg + r < R) unpack8(*reinterpret_cast<const uint4*>(x + (size_t)(rg + r) * K + k0), xr[r]);
            else {
#pragma unroll
                for (int j = 0; j < 8; ++j) xr[r][j] = 0.f;
            }
        }
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int c = 0; c < FCR_CPB; ++c) {
                const float d = dzr[(rg + r) * FCR_CPB + c];
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[c][j] = fmaf(d, xr[r][j], acc[c][j]);
            }
    }
    const size_t rs = (size_t)K / 4;
    float4* row = reinterpret_cast<float4*>(dw + (size_t)c0 * K + k0);
#pragma unroll
    for (int c = 0; c < FCR_CPB; ++c) {
        if (c < cn) {        // (no early exit: the unrolled loop keeps the accumulators in registers)
            float4 a0 = make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
            float4 a1 = make_float4(acc[c][4], acc[c][5], acc[c][6], acc[c][7]);
            if (accumulate) {
                const float4 o0 = row[(size_t)c * rs], o1 = row[(size_t)c * rs + 1];
                a0.x += o0.x; a0.y += o0.y; a0.z += o0.z; a0.w += o0.w;
                a1.x += o1.x; a1.y += o1.y; a1.z += o1.z; a1.w += o1.w;
            }
            row[(size_t)c * rs] = a0;
            row[(size_t)c * rs + 1] = a1;
        }
    }
}

// contraction over the first `slots` staged micro-batches
hipError_t fc_wgrad_staged(const ConvGeom& g, const void* xs, const void* dzs, int slots, float* dw, float* dbias,
                           const float* rscale, int accumulate, hipStream_t st) {
    const int K = g.K(), R = slots * g.m;
    const int threads = std::min(256, ((K / 8 + 63) / 64) * 64);
    const dim3 grid((unsigned)((K / 8 + threads - 1) / threads), (unsigned)((g.Cout + FCR_CPB - 1) / FCR_CPB));
    const size_t lds = (size_t)((R + 7) & ~7) * FCR_CPB * sizeof(float);
    hipLaunchKernelGGL(fc_wgrad_rows, grid, dim3(threads), lds, st, (const uint16_t*)xs, (const uint16_t*)dzs, dw, dbias,
                       rscale, R, g.Cout, K, accumulate);
    return hipGetLastError();
}

}  // namespace lpm
