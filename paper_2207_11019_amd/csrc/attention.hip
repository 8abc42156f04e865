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

// scores of the block's queries against every key, into sc[QB][P] (LDS); qs[QB][C] holds the queries times 1/sqrt(C)
template <typename T>
__device__ __forceinline__ void att_scores(const T* __restrict__ xs, int P, int C, int nq, const float* qs, float* sc) {
    for (int j = threadIdx.x; j < P; j += blockDim.x) {
        const T* kj = xs + (int64_t)j * 3 * C + C;
        float acc[ATT_QB];
#pragma unroll
        for (int i = 0; i < ATT_QB; ++i) acc[i] = 0.f;
        for (int c = 0; c < C; ++c) {
            const float kv = ld(kj, c);
#pragma unroll
            for (int i = 0; i < ATT_QB; ++i) acc[i] = fmaf(qs[i * C + c], kv, acc[i]);
        }
#pragma unroll
        for (int i = 0; i < ATT_QB; ++i) if (i < nq) sc[i * P + j] = acc[i];
    }
}

// per query row of the block: maximum and sum of exp (one wavefront per row at a time); sc becomes the softmax
__device__ __forceinline__ void att_softmax_rows(int P, int nq, float* sc, float* rmax, float* rsum) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    for (int i = wave; i < nq; i += nw) {
        float mx = -INFINITY;
        for (int j = lane; j < P; j += 64) mx = fmaxf(mx, sc[i * P + j]);
        mx = att_wave_max(mx);
        float se = 0.f;
        for (int j = lane; j < P; j += 64) { const float e = expf(sc[i * P + j] - mx); sc[i * P + j] = e; se += e; }
        se = att_wave_sum(se);
        const float inv = 1.f / se;
        for (int j = lane; j < P; j += 64) sc[i * P + j] *= inv;
        if (lane == 0) { rmax[i] = mx; rsum[i] = se; }
    }
}

template <typename T>
__global__ void __launch_bounds__(256) attn_fwd_kernel(int P, int C, const T* __restrict__ x, T* __restrict__ y) {
    extern __shared__ float lds[];
    float* qs = lds;                    // [QB][C]
    float* sc = lds + ATT_QB * C;       // [QB][P]
    __shared__ float rmax[ATT_QB], rsum[ATT_QB];
    const int n = blockIdx.y, i0 = blockIdx.x * ATT_QB, nq = min(ATT_QB, P - i0);
    const T* xs = x + (int64_t)n * P * 3 * C;
    const float scale = rsqrtf((float)C);
    for (int e = threadIdx.x; e < ATT_QB * C; e += blockDim.x) {
        const int i = e / C, c = e - i * C;
        qs[e] = i < nq ? ld(xs, (int64_t)(i0 + i) * 3 * C + c) * scale : 0.f;
    }
    __syncthreads();
    att_scores(xs, P, C, nq, qs, sc);
    __syncthreads();
    att_softmax_rows(P, nq, sc, rmax, rsum);
    __syncthreads();
    for (int e = threadIdx.x; e < nq * C; e += blockDim.x) {
        const int i = e / C, c = e - i * C;
        float acc = 0.f;
        for (int j = 0; j < P; ++j) acc = fmaf(sc[i * P + j], ld(xs, (int64_t)j * 3 * C + 2 * C + c), acc);
        st(y, ((int64_t)n * P + i0 + i) * C + c, acc);
    }
}

// per block of queries: dq, and per query row (max, sum of exp, sum_j A dA) into stats [m][P][3]
template <typename T>
__global__ void __launch_bounds__(256) attn_bwd_q_kernel(int P, int C, const T* __restrict__ x, const T* __restrict__ dy,
                                                         T* __restrict__ dx, int accumulate, float* __restrict__ stats) {
    extern __shared__ float lds[];
    float* qs = lds;                           // [QB][C] queries / sqrt(C)
    float* gs = qs + ATT_QB * C;               // [QB][C] dy rows
    float* sc = gs + ATT_QB * C;               // [QB][P] A, then dS
    float* da = sc + ATT_QB * P;               // [QB][P] dA
    __shared__ float rmax[ATT_QB], rsum[ATT_QB], rdot[ATT_QB];
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
    att_scores(xs, P, C, nq, qs, sc);
    // dA[i][j] = dy_i . v_j
    for (int j = threadIdx.x; j < P; j += blockDim.x) {
        const T* vj = xs + (int64_t)j * 3 * C + 2 * C;
        float acc[ATT_QB];
#pragma unroll
        for (int i = 0; i < ATT_QB; ++i) acc[i] = 0.f;
        for (int c = 0; c < C; ++c) {
            const float vv = ld(vj, c);
#pragma unroll
            for (int i = 0; i < ATT_QB; ++i) acc[i] = fmaf(gs[i * C + c], vv, acc[i]);
        }
#pragma unroll
        for (int i = 0; i < ATT_QB; ++i) if (i < nq) da[i * P + j] = acc[i];
    }
    __syncthreads();
    att_softmax_rows(P, nq, sc, rmax, rsum);
    __syncthreads();
    {   // rowsum(A dA), then dS = A (dA - rowsum) in place of A
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
        for (int i = wave; i < nq; i += nw) {
            float r = 0.f;
            for (int j = lane; j < P; j += 64) r = fmaf(sc[i * P + j], da[i * P + j], r);
            r = att_wave_sum(r);
            for (int j = lane; j < P; j += 64) sc[i * P + j] *= (da[i * P + j] - r);
            if (lane == 0) {
                rdot[i] = r;
                float* s3 = stats + ((int64_t)n * P + i0 + i) * 3;
                s3[0] = rmax[i]; s3[1] = rsum[i]; s3[2] = r;
            }
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < nq * C; e += blockDim.x) {
        const int i = e / C, c = e - i * C;
        float acc = 0.f;
        for (int j = 0; j < P; ++j) acc = fmaf(sc[i * P + j], ld(xs, (int64_t)j * 3 * C + C + c), acc);
        const int64_t o = ((int64_t)n * P + i0 + i) * 3 * C + c;
        acc *= scale;
        st(dx, o, accumulate ? acc + ld(dx, o) : acc);
    }
}

// per block of keys: dk and dv
template <typename T>
__global__ void __launch_bounds__(256) attn_bwd_kv_kernel(int P, int C, const T* __restrict__ x, const T* __restrict__ dy,
                                                          T* __restrict__ dx, int accumulate, const float* __restrict__ stats) {
    extern __shared__ float lds[];
    float* ks = lds;                           // [QB][C] keys / sqrt(C)
    float* vs = ks + ATT_QB * C;               // [QB][C] values
    float* aa = vs + ATT_QB * C;               // [QB][P] A[i][j] for the block's keys j, all queries i
    float* ds = aa + ATT_QB * P;               // [QB][P] dS[i][j]
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
        const T* qi = xs + (int64_t)i * 3 * C;
        const T* gi = gy + (int64_t)i * C;
        float s[ATT_QB], d[ATT_QB];
#pragma unroll
        for (int j = 0; j < ATT_QB; ++j) { s[j] = 0.f; d[j] = 0.f; }
        for (int c = 0; c < C; ++c) {
            const float qv = ld(qi, c), gv = ld(gi, c);
#pragma unroll
            for (int j = 0; j < ATT_QB; ++j) { s[j] = fmaf(qv, ks[j * C + c], s[j]); d[j] = fmaf(gv, vs[j * C + c], d[j]); }
        }
        const float* s3 = stats + ((int64_t)n * P + i) * 3;
        const float mx = s3[0], inv = 1.f / s3[1], r = s3[2];
#pragma unroll
        for (int j = 0; j < ATT_QB; ++j) {
            const float a = expf(s[j] - mx) * inv;
            aa[j * P + i] = a;
            ds[j * P + i] = a * (d[j] - r);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < nk * C; e += blockDim.x) {
        const int j = e / C, c = e - j * C;
        float dv = 0.f, dk = 0.f;
        for (int i = 0; i < P; ++i) {
            dv = fmaf(aa[j * P + i], ld(gy, (int64_t)i * C + c), dv);
            dk = fmaf(ds[j * P + i], ld(xs, (int64_t)i * 3 * C + c), dk);
        }
        dk *= scale;
        const int64_t ok = ((int64_t)n * P + j0 + j) * 3 * C + C + c, ov = ok + C;
        st(dx, ok, accumulate ? dk + ld(dx, ok) : dk);
        st(dx, ov, accumulate ? dv + ld(dx, ov) : dv);
    }
}

hipError_t launch_attn_fwd(int dtype, int32_t m, int32_t P, int32_t C, const void* x, void* y, hipStream_t st) {
    if (!attn_ok(P, C)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((P + ATT_QB - 1) / ATT_QB), (unsigned)m);
    const size_t lds = (size_t)ATT_QB * (C + P) * sizeof(float);
    if (dtype == LPM_BF16) hipLaunchKernelGGL(attn_fwd_kernel<bf16_t>, grid, dim3(256), lds, st, P, C, (const bf16_t*)x, (bf16_t*)y);
    else hipLaunchKernelGGL(attn_fwd_kernel<float>, grid, dim3(256), lds, st, P, C, (const float*)x, (float*)y);
    return hipGetLastError();
}

hipError_t launch_attn_bwd(int dtype, int32_t m, int32_t P, int32_t C, const void* x, const void* dy, void* dx, int accumulate,
                           void* ws, hipStream_t st) {
    if (!attn_ok(P, C) || !ws) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((P + ATT_QB - 1) / ATT_QB), (unsigned)m);
    const size_t lds = (size_t)ATT_QB * (2 * C + 2 * P) * sizeof(float);
    if (dtype == LPM_BF16) {
        hipLaunchKernelGGL(attn_bwd_q_kernel<bf16_t>, grid, dim3(256), lds, st, P, C, (const bf16_t*)x, (const bf16_t*)dy, (bf16_t*)dx,
                           accumulate, (float*)ws);
        hipLaunchKernelGGL(attn_bwd_kv_kernel<bf16_t>, grid, dim3(256), lds, st, P, C, (const bf16_t*)x, (const bf16_t*)dy, (bf16_t*)dx,
                           accumulate, (const float*)ws);
    } else {
        hipLaunchKernelGGL(attn_bwd_q_kernel<float>, grid, dim3(256), lds, st, P, C, (const float*)x, (const float*)dy, (float*)dx,
                           accumulate, (float*)ws);
        hipLaunchKernelGGL(attn_bwd_kv_kernel<float>, grid, dim3(256), lds, st, P, C, (const float*)x, (const float*)dy, (float*)dx,
                           accumulate, (const float*)ws);
    }
    return hipGetLastError();
}

}  // namespace lpm
