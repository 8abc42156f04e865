// One-head self-attention over the positions of a sample -- the "self-attention layer" of the residual self-attention
// block in the method's first use case (3D-ResAttNet), read as scaled dot-product attention:
//   x [m][P][3C] holds queries | keys | values per position (made by the 1x1 convolution in front of the layer)
//   S[i][j] = q_i . k_j / sqrt(C);   A = softmax over j;   y_i = sum_j A[i][j] v_j                    (forward, eq. 1)
//   dv_j = sum_i A[i][j] dy_i;  dA[i][j] = dy_i . v_j;  dS = A (dA - rowsum(A dA));
//   dq_i = sum_j dS[i][j] k_j / sqrt(C);  dk_j = sum_i dS[i][j] q_i / sqrt(C)                        (backward, eq. 9)
// Sizes here are small (P up to a few hundred positions after the last down-sampling stage, C up to a few hundred
// channels: well under a GFLOP per sample), so the kernels are plain fp32 vector-ALU code with the row being worked on
// in LDS; float or bf16 storage.  No atomics: every output element is one thread's sequential sum, so results do not
// depend on scheduling.  The backward pass recomputes the scores (nothing but the layer input is kept from the forward
// pass) in two kernels: one per block of queries (dq, and the row statistics max, sum, rowsum(A dA)), one per block
// of keys (dk, dv), which needs those statistics.
#include "lpm_internal.h"
#include "elem.h"

namespace lpm {

constexpr int ATT_QB = 8;        // queries (keys) per block
constexpr int ATT_LIMIT = 1000;  // C + P: the key-block kernel keeps 8 x (2C + 2P) floats in LDS (under 64 KiB)

bool attn_ok(int32_t P, int32_t C) { return P > 0 && C > 0 && P + C <= ATT_LIMIT; }
size_t attn_bwd_ws_bytes(int32_t m, int32_t P) { return (size_t)m * P * 3 * sizeof(float); }

__device__ inline float att_wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline float att_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// eight consecutive elements of a row (the caller has checked that rows start at multiples of eight elements)
__device__ __forceinline__ void att_ld8(const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void att_ld8(const bf16_t* p, float (&v)[8]) {
    const uint4 w = *reinterpret_cast<const uint4*>(p);
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) { v[2 * k] = bf2f((uint16_t)(ww[k] & 0xffffu)); v[2 * k + 1] = bf2f((uint16_t)(ww[k] >> 16)); }
}

// acc[i] += sum_c row[c] * mat[i][c] for the ATT_QB rows of mat (LDS, [ATT_QB][C]); the row is read 8 channels at a
// time where C allows (a thread walking its row two bytes at a time was the slowest part of these kernels)
template <typename T>
__device__ __forceinline__ void att_row_dots(const T* __restrict__ row, int C, const float* mat, float (&acc)[ATT_QB]) {
    int c = 0;
    if ((C & 7) == 0) {
        for (; c < C; c += 8) {
            float v[8];
            att_ld8(row + c, v);
#pragma unroll
            for (int i = 0; i < ATT_QB; ++i) {
                const float4 m0 = *reinterpret_cast<const float4*>(mat + i * C + c), m1 = *reinterpret_cast<const float4*>(mat + i * C + c + 4);
                acc[i] = fmaf(v[0], m0.x, acc[i]); acc[i] = fmaf(v[1], m0.y, acc[i]); acc[i] = fmaf(v[2], m0.z, acc[i]); acc[i] = fmaf(v[3], m0.w, acc[i]);
                acc[i] = fmaf(v[4], m1.x, acc[i]); acc[i] = fmaf(v[5], m1.y, acc[i]); acc[i] = fmaf(v[6], m1.z, acc[i]); acc[i] = fmaf(v[7], m1.w, acc[i]);
            }
        }
        return;
    }
    for (; c < C; ++c) {
        const float v = ld(row, c);
#pragma unroll
        for (int i = 0; i < ATT_QB; ++i) acc[i] = fmaf(v, mat[i * C + c], acc[i]);
    }
}

// The per-block score tiles live in LDS position-major: tile[j * ATT_QB + i] for position j and the block's row i, so the
// eight values of one position are one 32-byte read.

// scores of the block's queries against every key, into sc[P][QB]; qs[QB][C] holds the queries times 1/sqrt(C)
template <typename T>
__device__ __forceinline__ void att_scores(const T* __restrict__ xs, int P, int C, const float* qs, float* sc) {
    for (int j = threadIdx.x; j < P; j += blockDim.x) {
        float acc[ATT_QB];
#pragma unroll
        for (int i = 0; i < ATT_QB; ++i) acc[i] = 0.f;
        att_row_dots(xs + (int64_t)j * 3 * C + C, C, qs, acc);
#pragma unroll
        for (int i = 0; i < ATT_QB; ++i) sc[j * ATT_QB + i] = acc[i];
    }
}

// per query row of the block: maximum and sum of exp (one wavefront per row at a time); sc becomes the softmax
__device__ __forceinline__ void att_softmax_rows(int P, int nq, float* sc, float* rmax, float* rsum) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    for (int i = wave; i < nq; i += nw) {
        float mx = -INFINITY;
        for (int j = lane; j < P; j += 64) mx = fmaxf(mx, sc[j * ATT_QB + i]);
        mx = att_wave_max(mx);
        float se = 0.f;
        for (int j = lane; j < P; j += 64) { const float e = expf(sc[j * ATT_QB + i] - mx); sc[j * ATT_QB + i] = e; se += e; }
        se = att_wave_sum(se);
        const float inv = 1.f / se;
        for (int j = lane; j < P; j += 64) sc[j * ATT_QB + i] *= inv;
        if (lane == 0) { rmax[i] = mx; rsum[i] = se; }
    }
}

// out[i][c] = sum_j tile[j][i] * rows[j][c] over all positions j, for the block's rows i < n_rows and all channels c:
// a thread owns a channel and ATT_QB / NP of the rows (NP parts of the block share a channel when C is small), so one
// element of rows[j] feeds that many multiply-adds.  f(i, c, value) stores.
template <int NP, typename T, typename F>
__device__ __forceinline__ void att_mix(const float* tile, const T* __restrict__ rows, int64_t row_stride, int P, int C, int n_rows, F&& f) {
    constexpr int QPP = ATT_QB / NP;
    const int cols = blockDim.x / NP, part = threadIdx.x / cols, i0 = part * QPP;
    for (int c = threadIdx.x - part * cols; c < C; c += cols) {
        float acc[QPP];
#pragma unroll
        for (int i = 0; i < QPP; ++i) acc[i] = 0.f;
        // Sixteen positions per trip, their loads issued together before the first is used: one memory latency per sixteen
        // positions (left to itself the compiler keeps four loads in flight; asked to unroll further it chains the
        // 2-byte loads through one register and waits for each).
        int j = 0;
        for (; j + 16 <= P; j += 16) {
            T raw[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) raw[k] = rows[(int64_t)(j + k) * row_stride + c];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const float v = ld(raw, k);
#pragma unroll
                for (int i = 0; i < QPP; ++i) acc[i] = fmaf(tile[(j + k) * ATT_QB + i0 + i], v, acc[i]);
            }
        }
        for (; j < P; ++j) {
            const float v = ld(rows, (int64_t)j * row_stride + c);
#pragma unroll
            for (int i = 0; i < QPP; ++i) acc[i] = fmaf(tile[j * ATT_QB + i0 + i], v, acc[i]);
        }
#pragma unroll
        for (int i = 0; i < QPP; ++i) if (i0 + i < n_rows) f(i0 + i, c, acc[i]);
    }
}

template <typename T, int NP>
__global__ void __launch_bounds__(256) attn_fwd_kernel(int P, int C, const T* __restrict__ x, T* __restrict__ y) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float* qs = lds;                    // [QB][C]
    float* sc = lds + ATT_QB * C;       // [P][QB]
    __shared__ float rmax[ATT_QB], rsum[ATT_QB];
    const int n = blockIdx.y, i0 = blockIdx.x * ATT_QB, nq = min(ATT_QB, P - i0);
    const T* xs = x + (int64_t)n * P * 3 * C;
    const float scale = rsqrtf((float)C);
    for (int e = threadIdx.x; e < ATT_QB * C; e += blockDim.x) {
        const int i = e / C, c = e - i * C;
        qs[e] = i < nq ? ld(xs, (int64_t)(i0 + i) * 3 * C + c) * scale : 0.f;
    }
    __syncthreads();
    att_scores(xs, P, C, qs, sc);
    __syncthreads();
    att_softmax_rows(P, nq, sc, rmax, rsum);
    __syncthreads();
    att_mix<NP>(sc, xs + 2 * C, 3 * C, P, C, nq, [&](int i, int c, float v) { st(y, ((int64_t)n * P + i0 + i) * C + c, v); });
}

// per block of queries: dq, and per query row (max, sum of exp, sum_j A dA) into stats [m][P][3]
template <typename T, int NP>
__global__ void __launch_bounds__(256) attn_bwd_q_kernel(int P, int C, const T* __restrict__ x, const T* __restrict__ dy,
                                                         T* __restrict__ dx, int accumulate, float* __restrict__ stats) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float* qs = lds;                           // [QB][C] queries / sqrt(C)
    float* gs = qs + ATT_QB * C;               // [QB][C] dy rows
    float* sc = gs + ATT_QB * C;               // [P][QB] A, then dS
    float* da = sc + ATT_QB * P;               // [P][QB] dA
    __shared__ float rmax[ATT_QB], rsum[ATT_QB];
    const int n = blockIdx.y, i0 = blockIdx.x * ATT_QB, nq = min(ATT_QB, P - i0);
    const T* xs = x + (int64_t)n * P * 3 * C;
    const T* gy = dy + (int64_t)n * P * C;
    const float scale = rsqrtf((float)C);
    for (int e = threadIdx.x; e < ATT_QB * C; e += blockDim.x) {
        const int i = e / C, c = e - i * C;
        qs[e] = i < nq ? ld(xs, (int64_t)(i0 + i) * 3 * C + c) * scale : 0.f;
        gs[e] = i < nq ? ld(gy, (int64_t)(i0 + i) * C + c) : 0.f;
    }
    __syncthreads();
    att_scores(xs, P, C, qs, sc);
    // dA[i][j] = dy_i . v_j
    for (int j = threadIdx.x; j < P; j += blockDim.x) {
        float acc[ATT_QB];
#pragma unroll
        for (int i = 0; i < ATT_QB; ++i) acc[i] = 0.f;
        att_row_dots(xs + (int64_t)j * 3 * C + 2 * C, C, gs, acc);
#pragma unroll
        for (int i = 0; i < ATT_QB; ++i) da[j * ATT_QB + i] = acc[i];
    }
    __syncthreads();
    att_softmax_rows(P, nq, sc, rmax, rsum);
    __syncthreads();
    {   // rowsum(A dA), then dS = A (dA - rowsum) in place of A
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
        for (int i = wave; i < nq; i += nw) {
            float r = 0.f;
            for (int j = lane; j < P; j += 64) r = fmaf(sc[j * ATT_QB + i], da[j * ATT_QB + i], r);
            r = att_wave_sum(r);
            for (int j = lane; j < P; j += 64) sc[j * ATT_QB + i] *= (da[j * ATT_QB + i] - r);
            if (lane == 0) {
                float* s3 = stats + ((int64_t)n * P + i0 + i) * 3;
                s3[0] = rmax[i]; s3[1] = rsum[i]; s3[2] = r;
            }
        }
    }
    __syncthreads();
    att_mix<NP>(sc, xs + C, 3 * C, P, C, nq, [&](int i, int c, float v) {
        const int64_t o = ((int64_t)n * P + i0 + i) * 3 * C + c;
        v *= scale;
        st(dx, o, accumulate ? v + ld(dx, o) : v);
    });
}

// per block of keys: dk and dv
template <typename T, int NP>
__global__ void __launch_bounds__(256) attn_bwd_kv_kernel(int P, int C, const T* __restrict__ x, const T* __restrict__ dy,
                                                          T* __restrict__ dx, int accumulate, const float* __restrict__ stats) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float* ks = lds;                           // [QB][C] keys / sqrt(C)
    float* vs = ks + ATT_QB * C;               // [QB][C] values
    float* aa = vs + ATT_QB * C;               // [P][QB] A[i][j] for the block's keys j, all queries i
    float* ds = aa + ATT_QB * P;               // [P][QB] dS[i][j]
    const int n = blockIdx.y, j0 = blockIdx.x * ATT_QB, nk = min(ATT_QB, P - j0);
    const T* xs = x + (int64_t)n * P * 3 * C;
    const T* gy = dy + (int64_t)n * P * C;
    const float scale = rsqrtf((float)C);
    for (int e = threadIdx.x; e < ATT_QB * C; e += blockDim.x) {
        const int j = e / C, c = e - j * C;
        ks[e] = j < nk ? ld(xs, (int64_t)(j0 + j) * 3 * C + C + c) * scale : 0.f;
        vs[e] = j < nk ? ld(xs, (int64_t)(j0 + j) * 3 * C + 2 * C + c) : 0.f;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < P; i += blockDim.x) {
        float s[ATT_QB], d[ATT_QB];
#pragma unroll
        for (int j = 0; j < ATT_QB; ++j) { s[j] = 0.f; d[j] = 0.f; }
        att_row_dots(xs + (int64_t)i * 3 * C, C, ks, s);
        att_row_dots(gy + (int64_t)i * C, C, vs, d);
        const float* s3 = stats + ((int64_t)n * P + i) * 3;
        const float mx = s3[0], inv = 1.f / s3[1], r = s3[2];
#pragma unroll
        for (int j = 0; j < ATT_QB; ++j) {
            const float a = expf(s[j] - mx) * inv;
            aa[i * ATT_QB + j] = a;
            ds[i * ATT_QB + j] = a * (d[j] - r);
        }
    }
    __syncthreads();
    att_mix<NP>(aa, gy, C, P, C, nk, [&](int j, int c, float v) {
        const int64_t o = ((int64_t)n * P + j0 + j) * 3 * C + 2 * C + c;
        st(dx, o, accumulate ? v + ld(dx, o) : v);
    });
    att_mix<NP>(ds, xs, 3 * C, P, C, nk, [&](int j, int c, float v) {
        const int64_t o = ((int64_t)n * P + j0 + j) * 3 * C + C + c;
        v *= scale;
        st(dx, o, accumulate ? v + ld(dx, o) : v);
    });
}

// parts of a block that share a channel in att_mix: as many as leave every thread a channel
static int att_parts(int C) { return C <= 32 ? 8 : C <= 64 ? 4 : C <= 128 ? 2 : 1; }
#define LPM_ATT_NP(NP_, ...)                                       \
    do {                                                           \
        if ((NP_) == 8) { constexpr int NP = 8; __VA_ARGS__; }     \
        else if ((NP_) == 4) { constexpr int NP = 4; __VA_ARGS__; } \
        else if ((NP_) == 2) { constexpr int NP = 2; __VA_ARGS__; } \
        else { constexpr int NP = 1; __VA_ARGS__; }                \
    } while (0)

hipError_t launch_attn_fwd(int dtype, int32_t m, int32_t P, int32_t C, const void* x, void* y, hipStream_t st) {
    if (!attn_ok(P, C)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((P + ATT_QB - 1) / ATT_QB), (unsigned)m);
    const size_t lds = (size_t)ATT_QB * (C + P) * sizeof(float);
    const int np = att_parts(C);
    if (dtype == LPM_BF16) LPM_ATT_NP(np, hipLaunchKernelGGL((attn_fwd_kernel<bf16_t, NP>), grid, dim3(256), lds, st, P, C, (const bf16_t*)x, (bf16_t*)y));
    else LPM_ATT_NP(np, hipLaunchKernelGGL((attn_fwd_kernel<float, NP>), grid, dim3(256), lds, st, P, C, (const float*)x, (float*)y));
    return hipGetLastError();
}

hipError_t launch_attn_bwd(int dtype, int32_t m, int32_t P, int32_t C, const void* x, const void* dy, void* dx, int accumulate,
                           void* ws, hipStream_t st) {
    if (!attn_ok(P, C) || !ws) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((P + ATT_QB - 1) / ATT_QB), (unsigned)m);
    const size_t lds = (size_t)ATT_QB * (2 * C + 2 * P) * sizeof(float);
    const int np = att_parts(C);
    if (dtype == LPM_BF16) {
        LPM_ATT_NP(np, hipLaunchKernelGGL((attn_bwd_q_kernel<bf16_t, NP>), grid, dim3(256), lds, st, P, C, (const bf16_t*)x, (const bf16_t*)dy,
                                          (bf16_t*)dx, accumulate, (float*)ws));
        LPM_ATT_NP(np, hipLaunchKernelGGL((attn_bwd_kv_kernel<bf16_t, NP>), grid, dim3(256), lds, st, P, C, (const bf16_t*)x, (const bf16_t*)dy,
                                          (bf16_t*)dx, accumulate, (const float*)ws));
    } else {
        LPM_ATT_NP(np, hipLaunchKernelGGL((attn_bwd_q_kernel<float, NP>), grid, dim3(256), lds, st, P, C, (const float*)x, (const float*)dy,
                                          (float*)dx, accumulate, (float*)ws));
        LPM_ATT_NP(np, hipLaunchKernelGGL((attn_bwd_kv_kernel<float, NP>), grid, dim3(256), lds, st, P, C, (const float*)x, (const float*)dy,
                                          (float*)dx, accumulate, (const float*)ws));
    }
    return hipGetLastError();
}

}  // namespace lpm
