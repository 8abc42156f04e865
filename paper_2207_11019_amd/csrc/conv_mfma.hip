// bf16 MFMA implicit-GEMM contractions for gfx950: convolution forward (eq. 1), data gradient (eq. 9)
// and weight gradient (eq. 8), fp32 accumulation, LDS-staged K tiles of 32..128, 4 wavefronts per block.
//
// Forward / data gradient:  C[M][N] = A[M][K] * B[N][K]^T
//   forward  rows = output pixels, A gathered from x [m][H][W][Cin],  B = w  [Cout][Kh][Kw][Cin]
//   dgrad    rows = input pixels,  A gathered from dz [m][Ho][Wo][Cout], B = wt [Cin][Kh][Kw][Cout]
//   K runs over (kh, kw, channel); a K tile lies inside one filter tap (channels % tile depth == 0).
// Weight gradient:  dW[co][tap][ci] = sum_rows dz[row][co] * x[pixel(row,tap)][ci]
//   both operands are stored with the reduction index (the pixel) outermost, so the loader transposes
//   4 pixels x 8 channels in registers before writing K-contiguous rows to LDS.
// The matrix instruction is v_mfma_f32_32x32x16_bf16: each lane supplies 8 consecutive K values of row
// (lane % 32); lane holds D[(i/4)*8 + (lane/32)*4 + i%4][lane % 32] in accumulator element i.
#include "lpm_internal.h"
#include "elem.h"
#include "lds_dma.h"
#include <algorithm>

namespace lpm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Global operands are read through buffer resources: a 16-byte load whose byte offset lies outside the
// buffer returns zeros, so padding taps, ragged tiles and strided gaps need no branch and no select --
// the loader just hands such chunks the offset OOB.  (Buffers are below 4 GiB; the host checks.)
constexpr unsigned OOB = 0xffffffffu;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, unsigned off) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ unsigned short buf_load2(__amdgpu_buffer_rsrc_t r, unsigned off) {
    return (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, off, 0, 0);
}

// A K tile of depth BK is stored in LDS as rows of BK + 8 elements (16-byte aligned, staggers banks).
// Small-M shapes are bound by the latency of one global load per K tile, so they take deep tiles.

enum { MODE_FWD = 0, MODE_DGRAD = 1 /* stride 1 */, MODE_DGRAD_S = 2 /* stride 2..4, by residue class */ };

struct IgemmArgs {
    const uint16_t* A;
    const uint16_t* B;
    uint16_t* C;          // bf16 output [M][N]
    float* part;          // split-K: fp32 partials [split][M][N]; NULL otherwise
    const float* scale;
    const float* bias;
    const uint16_t* add;
    const uint16_t* mask;   // data gradient: zero the result where this tensor (the producer's output) is <= 0
    const float* mscale;    // data gradient: then multiply by the producer's per-channel scale
    int relu, accumulate;
    uint16_t* C2;           // data gradient: the masked, not yet scaled result also goes here (the producer's shortcut), or NULL
    int acc2;               // ... added to what C2 holds
    const float* c2scale;   // ... times this per-channel factor (NULL: 1)
    int M, N, Ktot;
    int Hi, Wi, Ci;       // extent of the gathered tensor
    int Hr, Wr;           // extent of the row space
    int Kw, stride, pad;
    int kt_total, kt_per_split;
    unsigned a_bytes, b_bytes;   // extents of A and B for the buffer resources
    // strided data gradient: the input pixels are processed by residue class (h % stride, w % stride); a class
    // only meets the filter taps of matching parity.  cls_tile0[c] = first row tile of class c (c = ph*stride+pw).
    int Kh;
    int cls_tile0[17];
    int wshift, hshift;          // log2 of Wr, Hr when both are powers of two, else -1 (set by run_igemm)
    int m_tiles;                 // host only: row tiles to launch (0: ceil(M / 64)); K the plan is made for (0: Ktot)
    int plan_K;
    // stride-1 data gradient routed through a 2x2 max-pooling (see UnpoolDesc): the rows are pooled pixels
    // volumetric layers (forward and stride-1 data gradient): depth of the gathered tensor and of the row space, filter
    // depth and depth padding; a row space image index is then sample * Dr + slice.  2-D layers: 1, 1, 1, 0.
    int Di, Dr, Kd, pad_d;
    const uint16_t* pool_x;      // pooling input [m][2*Hr][2*Wr][N], NULL: plain output
    uint16_t* pool_dst;
    int pool_acc, pool_mask;     // (the per-channel factor is mscale)
    uint16_t* fwd_pool;          // forward with split K only: also store the 2x2 max-pooling of C, [m][Hr/2][Wr/2][N]
};

// One element v of the gradient of a 2x2 max-pooling output at pooled pixel `row`, channel `col`: goes to the first
// maximum of the window (row-major), times the ReLU derivative at the maximum and a per-channel factor when asked.
__device__ __forceinline__ void unpool_store(float v, int row, int col, int Hr, int Wr, int N, const uint16_t* __restrict__ pool_x,
                                             uint16_t* __restrict__ dst, int acc, int mask, const float* __restrict__ mscale) {
    const int wq = row % Wr, t = row / Wr, hq = t % Hr, n = t / Hr;
    const size_t base = ((size_t)(n * 2 * Hr + 2 * hq) * (2 * Wr) + 2 * wq) * N + col;
    const size_t off[4] = {0, (size_t)N, (size_t)2 * Wr * N, (size_t)2 * Wr * N + N};
    float a[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) a[k] = bf2f(pool_x[base + off[k]]);
    const float mx = fmaxf(fmaxf(a[0], a[1]), fmaxf(a[2], a[3]));
    float g = bf2f(f2bf(v));             // the value a stored bf16 gradient of the pooling output would have had
    if (mask && !(mx > 0.f)) g = 0.f;
    if (mscale) g *= mscale[col];
    bool found = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const bool hit = !found && (a[k] == mx);
        found = found || hit;
        float o = hit ? g : 0.f;
        if (acc) o += bf2f(dst[base + off[k]]);
        dst[base + off[k]] = f2bf(o);
    }
}

template <int BM, int BN, int WGM, int WGN>
struct TileCfg {
    static constexpr int WTM = BM / WGM, WTN = BN / WGN, MI = WTM / 32, NI = WTN / 32;
    static_assert(WGM * WGN == 4 && WTM % 32 == 0 && WTN % 32 == 0, "4 wavefronts, 32x32 MFMA tiles");
};

// acc[mi][ni] += A-tile(wave rows) * B-tile(wave cols) over one BK-deep K tile held in LDS (rows of LDK elements).
// HALF: the rows are only 8-byte aligned, fetch each operand as two 8-byte reads.
template <int MI, int NI, int BK, int LDK, bool HALF>
__device__ __forceinline__ void mma_tile(const uint16_t* As, const uint16_t* Bs, int arow0, int brow0, int lane,
                                         f32x16 (&acc)[MI][NI]) {
    const int r = lane & 31, kq = (lane >> 5) * 8;
    auto fetch = [&](const uint16_t* ptr) __attribute__((always_inline)) -> bf16x8 {
        if (HALF) {
            const uint2 lo = *reinterpret_cast<const uint2*>(ptr), hi = *reinterpret_cast<const uint2*>(ptr + 4);
            return __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
        }
        return *reinterpret_cast<const bf16x8*>(ptr);
    };
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8 a[MI], b[NI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) a[mi] = fetch(As + (arow0 + mi * 32 + r) * LDK + ks * 16 + kq);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) b[ni] = fetch(Bs + (brow0 + ni * 32 + r) * LDK + ks * 16 + kq);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
    }
}

// Strided data gradient: pixel index (in the full tensor) of row `row` of the residue class (pd, ph, pw), whose rows run over
// (sample, slice of the class, row of the class, column of the class); Dc = 1 and pd = 0 for two-dimensional layers.
__device__ __forceinline__ int class_pixel(const IgemmArgs& p, int row, int Hc, int Wc, int ph, int pw, int Dc, int pd) {
    const int wq = row % Wc, t = row / Wc, hq = t % Hc;
    int n = t / Hc, img = n;
    if (p.Dr > 1) { const int dq = n % Dc; n /= Dc; img = n * p.Dr + dq * p.stride + pd; }
    return (img * p.Hr + hq * p.stride + ph) * p.Wr + wq * p.stride + pw;
}

// Writes a block's accumulators: split-K partials, the max-pooling route of a data gradient, or the fused epilogue.
// The optional terms of the epilogue (shortcut, accumulation, mask) are the same for the whole launch; each of the
// eight combinations gets its own straight-line copy of the store loop instead of three branches per element.
template <int MI, int NI, int WTM, int WTN, int MODE, bool ADD, bool ACC, bool MASK>
__device__ __forceinline__ void igemm_store(const IgemmArgs& p, const f32x16 (&acc)[MI][NI], int ni, int col, int m0, int wm, int rq,
                                            int rows, int Hc, int Wc, int ph, int pw, int Dc, int pd) {
    const float sc = p.scale ? p.scale[col] : 1.f, bi = p.bias ? p.bias[col] : 0.f, ms = p.mscale ? p.mscale[col] : 1.f;
    const bool relu = p.relu != 0;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = m0 + wm * WTM + mi * 32 + (i >> 2) * 8 + rq + (i & 3);
            if (row >= rows) continue;
            size_t o = (size_t)(unsigned)(row * p.N + col);            // (the host checked that the output has fewer than 2^31 elements)
            if (MODE == MODE_DGRAD_S) {      // class row -> pixel of the full image
                o = (size_t)(unsigned)(class_pixel(p, row, Hc, Wc, ph, pw, Dc, pd) * p.N + col);
            }
            float v = acc[mi][ni][i] * sc + bi;
            if (ADD) v += bf2f(p.add[o]);
            if (ACC) v += bf2f(p.C[o]);
            const float r = fmaxf(v, 0.f);
            v = relu ? r : v;
            if (MASK) v = bf2f(p.mask[o]) > 0.f ? v : 0.f;
            if (p.C2) {
                const float u = p.c2scale ? v * p.c2scale[col] : v;
                p.C2[o] = f2bf(p.acc2 ? u + bf2f(p.C2[o]) : u);
            }
            p.C[o] = f2bf(v * ms);
        }
}

// The same epilogue with 16-byte accesses.  A 32x32 accumulator tile has a column per lane (2-byte stores, 64 bytes
// per row and instruction; the masked / shortcut forms add as many 2-byte loads); the wavefront passes the tile through
// a private LDS area and every lane then owns 8 consecutive channels of a row.  tile: 32 rows of 36 floats.
// (PART: the fp32 split-K partials instead of the epilogue; strided data gradient: a row is a pixel of the block's
// residue class, Hc x Wc of them per image)
template <int MODE, bool PART, bool ADD, bool ACC, bool MASK>
__device__ __forceinline__ void igemm_store_vec(const IgemmArgs& p, const f32x16& acc, float* tile, int row0, int col0, int rows, int lane,
                                                int Hc, int Wc, int ph, int pw, int Dc, int pd) {
    const int col_l = lane & 31, rq = (lane >> 5) * 4;
    asm volatile("" ::: "memory");
#pragma unroll
    for (int i = 0; i < 16; ++i) tile[((i >> 2) * 8 + rq + (i & 3)) * 36 + col_l] = acc[i];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const bool relu = p.relu != 0;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int idx = lane + 64 * c, r = idx >> 2, ch = (idx & 3) * 8;
        const int row = row0 + r, col = col0 + ch;
        if (row >= rows || col >= p.N) continue;
        const float4 lo = *reinterpret_cast<const float4*>(tile + r * 36 + ch), hi = *reinterpret_cast<const float4*>(tile + r * 36 + ch + 4);
        float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        size_t o = (size_t)(unsigned)(row * p.N + col);
        if (MODE == MODE_DGRAD_S) {      // class row -> pixel of the full image
            o = (size_t)(unsigned)(class_pixel(p, row, Hc, Wc, ph, pw, Dc, pd) * p.N + col);
        }
        if (PART) {
            float* q = p.part + (size_t)blockIdx.z * p.M * p.N + o;
            *reinterpret_cast<float4*>(q) = lo;
            *reinterpret_cast<float4*>(q + 4) = hi;
            continue;
        }
        auto vec8 = [&](const float* q, float (&d)[8]) __attribute__((always_inline)) {
            const float4 a = *reinterpret_cast<const float4*>(q + col), b = *reinterpret_cast<const float4*>(q + col + 4);
            d[0] = a.x; d[1] = a.y; d[2] = a.z; d[3] = a.w; d[4] = b.x; d[5] = b.y; d[6] = b.z; d[7] = b.w;
        };
        auto bf8 = [&](const uint16_t* q, float (&d)[8]) __attribute__((always_inline)) {
            const uint4 w = *reinterpret_cast<const uint4*>(q + o);
            const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) { d[2 * k] = bf2f((uint16_t)(ww[k] & 0xffffu)); d[2 * k + 1] = bf2f((uint16_t)(ww[k] >> 16)); }
        };
        auto st8 = [&](uint16_t* q, const float (&d)[8]) __attribute__((always_inline)) {
            *reinterpret_cast<uint4*>(q + o) = make_uint4(pack_bf16x2(d[0], d[1]), pack_bf16x2(d[2], d[3]), pack_bf16x2(d[4], d[5]),
                                                          pack_bf16x2(d[6], d[7]));
        };
        float t[8];
        if (p.scale) { vec8(p.scale, t);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] *= t[k]; }
        if (p.bias) { vec8(p.bias, t);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] += t[k]; }
        if (ADD) { bf8(p.add, t);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] += t[k]; }
        if (ACC) { bf8(p.C, t);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] += t[k]; }
        if (relu) {
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = fmaxf(v[k], 0.f); }
        if (MASK) { bf8(p.mask, t);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = t[k] > 0.f ? v[k] : 0.f; }
        if (p.C2) {
            float u[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) u[k] = v[k];
            if (p.c2scale) { vec8(p.c2scale, t);
#pragma unroll
                for (int k = 0; k < 8; ++k) u[k] *= t[k]; }
            if (p.acc2) { bf8(p.C2, t);
#pragma unroll
                for (int k = 0; k < 8; ++k) u[k] += t[k]; }
            st8(p.C2, u);
        }
        if (p.mscale) { vec8(p.mscale, t);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] *= t[k]; }
        st8(p.C, v);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();        // the area is written again for the wavefront's next tile
}

// tile: this wavefront's private LDS area of 32 x 36 floats (NULL: none -- element-wise stores)
template <int MI, int NI, int WTM, int WTN, int MODE>
__device__ __forceinline__ void igemm_epilogue(const IgemmArgs& p, f32x16 (&acc)[MI][NI], int m0, int n0, int wm, int wn, int lane,
                                               int rows, int Hc, int Wc, int ph, int pw, int Dc, int pd, float* tile = nullptr) {
    const int col_l = lane & 31, rq = (lane >> 5) * 4;
    const int variant = (p.add ? 1 : 0) | (p.accumulate ? 2 : 0) | (p.mask ? 4 : 0);
    if (tile && (p.part || !(MODE == MODE_DGRAD && p.pool_x)) && (p.N & 7) == 0) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int row0 = m0 + wm * WTM + mi * 32, col0 = n0 + wn * WTN + ni * 32;
                if (p.part) {
                    igemm_store_vec<MODE, true, false, false, false>(p, acc[mi][ni], tile, row0, col0, rows, lane, Hc, Wc, ph, pw, Dc, pd);
                    continue;
                }
#define LPM_STORE_VEC(A, B, C) igemm_store_vec<MODE, false, A, B, C>(p, acc[mi][ni], tile, row0, col0, rows, lane, Hc, Wc, ph, pw, Dc, pd)
                switch (variant) {
                    case 0: LPM_STORE_VEC(false, false, false); break;
                    case 1: LPM_STORE_VEC(true, false, false); break;
                    case 2: LPM_STORE_VEC(false, true, false); break;
                    case 3: LPM_STORE_VEC(true, true, false); break;
                    case 4: LPM_STORE_VEC(false, false, true); break;
                    case 5: LPM_STORE_VEC(true, false, true); break;
                    case 6: LPM_STORE_VEC(false, true, true); break;
                    default: LPM_STORE_VEC(true, true, true); break;
                }
#undef LPM_STORE_VEC
            }
        return;
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int col = n0 + wn * WTN + ni * 32 + col_l;
        if (col >= p.N) continue;
        if (p.part || (MODE == MODE_DGRAD && p.pool_x)) {
            float* part = p.part ? p.part + (size_t)blockIdx.z * p.M * p.N : nullptr;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = m0 + wm * WTM + mi * 32 + (i >> 2) * 8 + rq + (i & 3);
                    if (row >= rows) continue;
                    size_t o = (size_t)(unsigned)(row * p.N + col);
                    if (MODE == MODE_DGRAD_S) {
                        o = (size_t)(unsigned)(class_pixel(p, row, Hc, Wc, ph, pw, Dc, pd) * p.N + col);
                    }
                    if (part) part[o] = acc[mi][ni][i];
                    else unpool_store(acc[mi][ni][i], row, col, p.Hr, p.Wr, p.N, p.pool_x, p.pool_dst, p.pool_acc, p.pool_mask, p.mscale);
                }
            continue;
        }
#define LPM_STORE(A, B, C) igemm_store<MI, NI, WTM, WTN, MODE, A, B, C>(p, acc, ni, col, m0, wm, rq, rows, Hc, Wc, ph, pw, Dc, pd)
        switch (variant) {
            case 0: LPM_STORE(false, false, false); break;
            case 1: LPM_STORE(true, false, false); break;
            case 2: LPM_STORE(false, true, false); break;
            case 3: LPM_STORE(true, true, false); break;
            case 4: LPM_STORE(false, false, true); break;
            case 5: LPM_STORE(true, false, true); break;
            case 6: LPM_STORE(false, true, true); break;
            default: LPM_STORE(true, true, true); break;
        }
#undef LPM_STORE
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, int MODE>
__global__ void __launch_bounds__(256, 2) igemm_kernel(IgemmArgs p) {
    typedef TileCfg<BM, BN, WGM, WGN> Cfg;
    constexpr int LDK = BK + 8, CPR = BK / 8;                 // chunks (16 bytes) per row
    constexpr int A_CH = (BM * CPR + 255) / 256, B_CH = (BN * CPR + 255) / 256;
    __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * LDK];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nt = (p.N + BN - 1) / BN;
    // (strided data gradient: the residue classes differ in work -- 1, 2, 2 and 4 taps of a 3x3 filter, one
    // class in four for a 1x1 filter -- so their tiles stay in launch order, which deals them round-robin to the XCDs)
    const int tile = MODE == MODE_DGRAD_S ? (int)blockIdx.x : xcd_remap(blockIdx.x, gridDim.x);
    int m0 = (tile / nt) * BM;
    const int n0 = (tile % nt) * BN;
    int kt0 = blockIdx.z * p.kt_per_split;
    int kt1 = min(p.kt_total, kt0 + p.kt_per_split);
    // filter taps visited: all of them in steps of 1, or (strided data gradient) those of the block's residue class
    int kstep = 1, kh_first = 0, kw_first = 0, kd_first = 0;
    int ph = 0, pw = 0, pd = 0, Hc = p.Hr, Wc = p.Wr, Dc = p.Dr, rows = p.M;     // residue class of the block's rows and its extent
    int nkh_c = 1, nkw_c = 1;                                                     // filter taps of the class per axis
    if (MODE == MODE_DGRAD_S) {
        // class c = (pd * s + ph) * s + pw; a two-dimensional layer (Dr = 1) has the s * s classes with pd = 0
        const int s_ = p.stride, mt = tile / nt, ncls = (p.Dr > 1 ? s_ : 1) * s_ * s_;
        int c = 0;
        while (c + 1 < ncls && mt >= p.cls_tile0[c + 1]) ++c;
        pd = c / (s_ * s_);
        ph = (c - pd * s_ * s_) / s_; pw = c - (pd * s_ + ph) * s_;
        Hc = (p.Hr - ph + s_ - 1) / s_; Wc = (p.Wr - pw + s_ - 1) / s_;
        Dc = p.Dr > 1 ? (p.Dr - pd + s_ - 1) / s_ : 1;
        rows = (p.M / (p.Dr * p.Hr * p.Wr)) * Dc * Hc * Wc;
        m0 = (mt - p.cls_tile0[c]) * BM;
        kstep = s_;
        kh_first = (ph + p.pad) % s_; kw_first = (pw + p.pad) % s_;
        kd_first = p.Dr > 1 ? (pd + p.pad_d) % s_ : 0;
        const int nkh = kh_first < p.Kh ? (p.Kh - kh_first + s_ - 1) / s_ : 0;
        const int nkw = kw_first < p.Kw ? (p.Kw - kw_first + s_ - 1) / s_ : 0;
        const int nkd = p.Dr > 1 ? (kd_first < p.Kd ? (p.Kd - kd_first + s_ - 1) / s_ : 0) : 1;
        nkh_c = max(nkh, 1); nkw_c = max(nkw, 1);
        const int kt_cls = nkd * nkh * nkw * (p.Ci / BK);
        const int per = (kt_cls + (int)gridDim.z - 1) / (int)gridDim.z;
        kt0 = blockIdx.z * per;
        kt1 = min(kt_cls, kt0 + per);
    }

    // per-thread gather state of its A chunks (a chunk = 8 channels of one row = 16 bytes)
    const __amdgpu_buffer_rsrc_t rsA = make_rsrc(p.A, p.a_bytes), rsB = make_rsrc(p.B, p.b_bytes);
    // Per chunk: the byte offset of its row's pixel at filter tap (0,0) (a_base, may wrap below zero for rows
    // that start in the padding; it is only used when the tap lands inside the image) and the pixel's
    // coordinates at tap (0,0).  Per K tile only a wave-uniform tap offset is added.
    // (Strided data gradient: the row's coordinates inside its residue class and the image's base offset.)
    int a_h0[A_CH], a_w0[A_CH], a_d0[A_CH];
    unsigned a_base[A_CH];
    bool a_ok[A_CH];
    unsigned b_off[B_CH];
#pragma unroll
    for (int c = 0; c < A_CH; ++c) {
        const int id = tid + c * 256, row = m0 + id / CPR, kc = id % CPR;
        a_ok[c] = (id < BM * CPR) & (row < rows);
        const int rr = a_ok[c] ? row : 0;
        int wq, hq, n;
        if (MODE != MODE_DGRAD_S && p.wshift >= 0) {       // power-of-two image extents (same for the whole launch): no division
            wq = rr & (Wc - 1);
            const int t = rr >> p.wshift;
            hq = t & (Hc - 1);
            n = t >> p.hshift;
        } else {
            wq = rr % Wc;
            const int t = rr / Wc;
            hq = t % Hc;
            n = t / Hc;
        }
        int dq = 0;
        if (MODE != MODE_DGRAD_S && p.Dr > 1) { const int ns = n / p.Dr; dq = n - ns * p.Dr; n = ns; }      // sample, slice
        if (MODE == MODE_DGRAD_S && p.Dr > 1) { const int ns = n / Dc; dq = n - ns * Dc; n = ns; }           // sample, slice of the class
        if (MODE == MODE_FWD) { a_h0[c] = hq * p.stride - p.pad; a_w0[c] = wq * p.stride - p.pad; a_d0[c] = dq * p.stride - p.pad_d; }
        else if (MODE == MODE_DGRAD) { a_h0[c] = hq + p.pad; a_w0[c] = wq + p.pad; a_d0[c] = dq + p.pad_d; }
        else { a_h0[c] = hq; a_w0[c] = wq; a_d0[c] = dq; }
        if (MODE == MODE_DGRAD_S) a_base[c] = (unsigned)(n * p.Di * p.Hi * p.Wi * p.Ci + kc * 8) * 2u;
        else a_base[c] = (unsigned)((((n * p.Di + a_d0[c]) * p.Hi + a_h0[c]) * p.Wi + a_w0[c]) * p.Ci + kc * 8) * 2u;
    }
#pragma unroll
    for (int c = 0; c < B_CH; ++c) {
        const int id = tid + c * 256, n = n0 + id / CPR;
        b_off[c] = ((id < BN * CPR) & (n < p.N)) ? (unsigned)(((size_t)n * p.Ktot + (id % CPR) * 8) * 2) : OOB;
    }
    // cursor of the next K tile to load (tiles are loaded strictly in order): filter tap and channel offset
    int cur_kt = kt0, cur_c0, cur_kh, cur_kw, cur_kd = 0;
    {
        const int k0 = kt0 * BK, tap = k0 / p.Ci;
        cur_c0 = k0 - tap * p.Ci;
        if (MODE == MODE_DGRAD_S) {
            const int td = tap / (nkh_c * nkw_c), r = tap - td * (nkh_c * nkw_c);
            cur_kd = kd_first + td * kstep;
            cur_kh = kh_first + (r / nkw_c) * kstep; cur_kw = kw_first + (r % nkw_c) * kstep;
        } else {
            const int hw = p.Kh * p.Kw;
            cur_kd = tap / hw;
            const int r = tap - cur_kd * hw;
            cur_kh = r / p.Kw; cur_kw = r - cur_kh * p.Kw;
        }
    }
    // two K tiles in flight in registers
    uint4 ra0[A_CH], rb0[B_CH], ra1[A_CH], rb1[B_CH];

#define LPM_LOAD_TILE(RA, RB)                                                                                \
    {                                                                                                        \
        const bool live_ = cur_kt < kt1;                                                                     \
        const int kh_ = cur_kh, kw_ = cur_kw, kd_ = cur_kd;                                                  \
        const unsigned tapoff_ = (MODE == MODE_FWD)                                                          \
                                     ? (unsigned)(((kd_ * p.Hi + kh_) * p.Wi + kw_) * p.Ci + cur_c0) * 2u    \
                                     : (unsigned)(cur_c0 - ((kd_ * p.Hi + kh_) * p.Wi + kw_) * p.Ci) * 2u;   \
        /* strided data gradient: output pixel = class coordinate + (ph + pad - kh) / stride, an exact quotient */ \
        const int dh_ = (MODE == MODE_DGRAD_S) ? (ph + p.pad - kh_) / kstep : 0;                             \
        const int dw_ = (MODE == MODE_DGRAD_S) ? (pw + p.pad - kw_) / kstep : 0;                             \
        const int dd_ = (MODE == MODE_DGRAD_S && p.Dr > 1) ? (pd + p.pad_d - kd_) / kstep : 0;               \
        _Pragma("unroll") for (int c = 0; c < A_CH; ++c) {                                                   \
            int h_, w_;                                                                                      \
            bool ok_ = a_ok[c] & live_;                                                                      \
            unsigned off_;                                                                                   \
            if (MODE == MODE_FWD) {                                                                          \
                h_ = a_h0[c] + kh_; w_ = a_w0[c] + kw_; off_ = a_base[c] + tapoff_;                          \
                ok_ = ok_ & ((unsigned)(a_d0[c] + kd_) < (unsigned)p.Di);                                    \
            } else if (MODE == MODE_DGRAD) {                                                                 \
                h_ = a_h0[c] - kh_; w_ = a_w0[c] - kw_; off_ = a_base[c] + tapoff_;                          \
                ok_ = ok_ & ((unsigned)(a_d0[c] - kd_) < (unsigned)p.Di);                                    \
            }                                                                                                \
            else {                                                                                           \
                h_ = a_h0[c] + dh_; w_ = a_w0[c] + dw_;                                                      \
                const int d_ = a_d0[c] + dd_;                                                                \
                ok_ = ok_ & ((unsigned)d_ < (unsigned)p.Di);                                                 \
                off_ = a_base[c] + (unsigned)(((d_ * p.Hi + h_) * p.Wi + w_) * p.Ci + cur_c0) * 2u;          \
            }                                                                                                \
            ok_ = ok_ & ((unsigned)h_ < (unsigned)p.Hi) & ((unsigned)w_ < (unsigned)p.Wi);                   \
            RA[c] = buf_load16(rsA, ok_ ? off_ : OOB);                                                       \
        }                                                                                                    \
        const unsigned k0b_ = (unsigned)(((kd_ * p.Kh + kh_) * p.Kw + kw_) * p.Ci + cur_c0) * 2u;            \
        _Pragma("unroll") for (int c = 0; c < B_CH; ++c)                                                     \
            RB[c] = buf_load16(rsB, ((b_off[c] == OOB) | !live_) ? OOB : b_off[c] + k0b_);                   \
        ++cur_kt;                                                                                            \
        cur_c0 += BK;                                                                                        \
        if (cur_c0 >= p.Ci) {                                                                                \
            cur_c0 = 0;                                                                                      \
            cur_kw += kstep;                                                                                 \
            if (cur_kw >= p.Kw) {                                                                            \
                cur_kw = kw_first; cur_kh += kstep;                                                          \
                if (cur_kh >= p.Kh) { cur_kh = kh_first; cur_kd += kstep; }                                  \
            }                                                                                                \
        }                                                                                                    \
    }
#define LPM_STORE_TILE(BUF, RA, RB)                                                                          \
    {                                                                                                        \
        _Pragma("unroll") for (int c = 0; c < A_CH; ++c) {                                                   \
            const int id_ = tid + c * 256;                                                                   \
            if (A_CH * 256 == BM * CPR || id_ < BM * CPR)                                                    \
                *reinterpret_cast<uint4*>(&As[BUF][(id_ / CPR) * LDK + (id_ % CPR) * 8]) = RA[c];            \
        }                                                                                                    \
        _Pragma("unroll") for (int c = 0; c < B_CH; ++c) {                                                   \
            const int id_ = tid + c * 256;                                                                   \
            if (B_CH * 256 == BN * CPR || id_ < BN * CPR)                                                    \
                *reinterpret_cast<uint4*>(&Bs[BUF][(id_ / CPR) * LDK + (id_ % CPR) * 8]) = RB[c];            \
        }                                                                                                    \
    }

    f32x16 acc[Cfg::MI][Cfg::NI];
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    const int wm = wave / WGN, wn = wave % WGN;
    // Pipeline: LDS holds tile i (being multiplied) and receives tile i+1; registers hold tiles i+1 and i+2,
    // so every global load has two iterations to arrive.
    const int nk = kt1 - kt0;
    if (nk > 0) {
        // Loads are issued unconditionally (a tile index past the end loads zeros that are never stored), so the
        // wait before an LDS store counts exactly the younger tile's loads and lets them stay in flight.
        LPM_LOAD_TILE(ra0, rb0);
        LPM_LOAD_TILE(ra1, rb1);
        LPM_STORE_TILE(0, ra0, rb0);
        __syncthreads();
        // Tiles are processed in pairs with no exit in between; an odd count is padded by one all-zero tile.
        const int npair = (nk + 1) >> 1;
        for (int it = 0; it < npair; ++it) {
            LPM_LOAD_TILE(ra0, rb0);
            mma_tile<Cfg::MI, Cfg::NI, BK, LDK, false>(As[0], Bs[0], wm * Cfg::WTM, wn * Cfg::WTN, lane, acc);
            LPM_STORE_TILE(1, ra1, rb1);
            __syncthreads();
            LPM_LOAD_TILE(ra1, rb1);
            mma_tile<Cfg::MI, Cfg::NI, BK, LDK, false>(As[1], Bs[1], wm * Cfg::WTM, wn * Cfg::WTN, lane, acc);
            LPM_STORE_TILE(0, ra0, rb0);
            __syncthreads();
        }
    }
#undef LPM_LOAD_TILE
#undef LPM_STORE_TILE

    // (every wavefront is past the loop's last barrier: the A tiles are dead and take the epilogue's staging areas)
    constexpr bool STAGE_FITS = sizeof(As) >= 4 * 32 * 36 * sizeof(float);
    float* stage = STAGE_FITS ? reinterpret_cast<float*>(&As[0][0]) + wave * (32 * 36) : nullptr;
    igemm_epilogue<Cfg::MI, Cfg::NI, Cfg::WTM, Cfg::WTN, MODE>(p, acc, m0, n0, wm, wn, lane, rows, Hc, Wc, ph, pw, Dc, pd, stage);
}


// Sum of one element's split-K partials in split order.  The loads are issued eight at a time before the first add (a
// plain loop over a run-time split count waits for every load in turn); the additions keep the order.
__device__ __forceinline__ float sum_partials(const float* __restrict__ part, int splits, int64_t stride, int64_t i) {
    float v = 0.f;
    for (int s0 = 0; s0 < splits; s0 += 8) {
        float t[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) t[k] = s0 + k < splits ? part[(int64_t)(s0 + k) * stride + i] : 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) if (s0 + k < splits) v = (s0 + k == 0) ? t[k] : v + t[k];
    }
    return v;
}

// sums split-K partials in split order and applies the epilogue
__global__ void __launch_bounds__(256) splitk_epilogue(const float* __restrict__ part, int splits, int64_t MN, int N,
                                                       const float* __restrict__ scale, const float* __restrict__ bias,
                                                       const uint16_t* __restrict__ add, int relu, int accumulate,
                                                       const uint16_t* __restrict__ mask, const float* __restrict__ mscale,
                                                       uint16_t* __restrict__ C, uint16_t* __restrict__ C2, int acc2,
                                                       const float* __restrict__ c2scale) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= MN) return;
    float v = sum_partials(part, splits, MN, i);
    const int col = (int)((unsigned)i % (unsigned)N);      // (the output has fewer than 2^31 elements)
    if (scale) v *= scale[col];
    if (bias) v += bias[col];
    if (add) v += bf2f(add[i]);
    if (accumulate) v += bf2f(C[i]);
    if (relu) v = fmaxf(v, 0.f);
    if (mask && !(bf2f(mask[i]) > 0.f)) v = 0.f;
    if (C2) {
        const float u = c2scale ? v * c2scale[col] : v;
        C2[i] = f2bf(acc2 ? u + bf2f(C2[i]) : u);
    }
    if (mscale) v *= mscale[col];
    C[i] = f2bf(v);
}

// The same for four consecutive channels per thread (N a multiple of 4): 16-byte partial loads, 8-byte tensor accesses.
__global__ void __launch_bounds__(256) splitk_epilogue_x4(const float* __restrict__ part, int splits, int64_t MN, int N,
                                                          const float* __restrict__ scale, const float* __restrict__ bias,
                                                          const uint16_t* __restrict__ add, int relu, int accumulate,
                                                          const uint16_t* __restrict__ mask, const float* __restrict__ mscale,
                                                          uint16_t* __restrict__ C, uint16_t* __restrict__ C2, int acc2,
                                                          const float* __restrict__ c2scale) {
    const unsigned i = (blockIdx.x * 256u + threadIdx.x) * 4u;
    if (i >= (unsigned)MN) return;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < splits; s0 += 8) {          // eight splits' loads before the first add; the adds keep the split order
        float4 t[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            t[k] = s0 + k < splits ? *reinterpret_cast<const float4*>(part + (size_t)(s0 + k) * MN + i) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (s0 + k < splits) {
                if (s0 + k == 0) { v[0] = t[k].x; v[1] = t[k].y; v[2] = t[k].z; v[3] = t[k].w; }
                else { v[0] += t[k].x; v[1] += t[k].y; v[2] += t[k].z; v[3] += t[k].w; }
            }
    }
    const unsigned col = i % (unsigned)N;
    auto f4 = [&](const float* q, float (&d)[4]) __attribute__((always_inline)) {
        const float4 a = *reinterpret_cast<const float4*>(q + col);
        d[0] = a.x; d[1] = a.y; d[2] = a.z; d[3] = a.w;
    };
    auto b4 = [&](const uint16_t* q, float (&d)[4]) __attribute__((always_inline)) {
        const uint2 w = *reinterpret_cast<const uint2*>(q + i);
        d[0] = bf2f((uint16_t)(w.x & 0xffffu)); d[1] = bf2f((uint16_t)(w.x >> 16));
        d[2] = bf2f((uint16_t)(w.y & 0xffffu)); d[3] = bf2f((uint16_t)(w.y >> 16));
    };
    float t[4];
    if (scale) { f4(scale, t);
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] *= t[k]; }
    if (bias) { f4(bias, t);
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] += t[k]; }
    if (add) { b4(add, t);
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] += t[k]; }
    if (accumulate) { b4(C, t);
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] += t[k]; }
    if (relu) {
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = fmaxf(v[k], 0.f); }
    if (mask) { b4(mask, t);
#pragma unroll
        for (int k = 0; k < 4; ++k) if (!(t[k] > 0.f)) v[k] = 0.f; }
    if (C2) {
        float u[4] = {v[0], v[1], v[2], v[3]};
        if (c2scale) { f4(c2scale, t);
#pragma unroll
            for (int k = 0; k < 4; ++k) u[k] *= t[k]; }
        if (acc2) { b4(C2, t);
#pragma unroll
            for (int k = 0; k < 4; ++k) u[k] += t[k]; }
        *reinterpret_cast<uint2*>(C2 + i) = make_uint2(pack_bf16x2(u[0], u[1]), pack_bf16x2(u[2], u[3]));
    }
    if (mscale) { f4(mscale, t);
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] *= t[k]; }
    *reinterpret_cast<uint2*>(C + i) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}

// the same sum routed through a 2x2 max-pooling (see unpool_store)
__global__ void __launch_bounds__(256) splitk_epilogue_unpool(const float* __restrict__ part, int splits, int64_t MN, int N,
                                                              int Hr, int Wr, const uint16_t* __restrict__ pool_x,
                                                              uint16_t* __restrict__ dst, int acc, int mask,
                                                              const float* __restrict__ mscale) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= MN) return;
    float v = sum_partials(part, splits, MN, i);
    unpool_store(v, (int)((unsigned)i / (unsigned)N), (int)((unsigned)i % (unsigned)N), Hr, Wr, N, pool_x, dst, acc, mask, mscale);
}

// forward: the same sum and epilogue, and the 2x2 max-pooling of the result as well (of the rounded values, as the
// pooling kernel would see them): P[m][Hr/2][Wr/2][N].  A block takes one pooling window x 64 channels; wavefront k
// takes window position k, so every thread sums one element as in splitk_epilogue and the maximum goes through LDS.
__global__ void __launch_bounds__(256) splitk_epilogue_pool(const float* __restrict__ part, int splits, int64_t MN, int N, int Hr,
                                                            int Wr, const float* __restrict__ scale,
                                                            const float* __restrict__ bias, int relu,
                                                            uint16_t* __restrict__ C, uint16_t* __restrict__ P) {
    __shared__ float win[4][64];
    const int lane = threadIdx.x & 63, k = threadIdx.x >> 6;
    const int cgroups = (N + 63) >> 6;
    const int col = (int)(blockIdx.x % cgroups) * 64 + lane;
    int64_t q = blockIdx.x / cgroups;        // pooled pixel (n, py, px)
    const int64_t pooled = q;
    const int Wp = Wr >> 1, Hp = Hr >> 1;
    const int px = (int)(q % Wp); q /= Wp;
    const int py = (int)(q % Hp);
    const int64_t n = q / Hp;
    float r = 0.f;
    if (col < N) {
        const int64_t e = ((n * Hr + 2 * py + (k >> 1)) * Wr + 2 * px + (k & 1)) * N + col;
        float v = sum_partials(part, splits, MN, e);
        if (scale) v *= scale[col];
        if (bias) v += bias[col];
        if (relu) v = fmaxf(v, 0.f);
        const uint16_t h = f2bf(v);
        C[e] = h;
        r = bf2f(h);
    }
    win[k][lane] = r;
    __syncthreads();
    if (k == 0 && col < N) P[pooled * N + col] = f2bf(fmaxf(fmaxf(win[0][lane], win[1][lane]), fmaxf(win[2][lane], win[3][lane])));
}

hipError_t launch_splitk_epilogue(const float* part, int splits, int64_t MN, int N, const float* scale, const float* bias,
                                  const void* add, int relu, int accumulate, const void* mask, const float* mscale,
                                  void* C, hipStream_t st) {
    hipLaunchKernelGGL(splitk_epilogue, dim3((unsigned)((MN + 255) / 256)), dim3(256), 0, st, part, splits, MN, N, scale, bias,
                       (const uint16_t*)add, relu, accumulate, (const uint16_t*)mask, mscale, (uint16_t*)C, (uint16_t*)nullptr, 0, (const float*)nullptr);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------------------------
struct IgemmPlan { int big; int bk; int splits; int kt_total; int kt_per; };

// ci: channel count of the gathered tensor (a K tile must not straddle a filter tap).
// Measured on MI355X over the layer shapes of the CIFAR, ResNet and 224x224 VGG workloads: 64x64 tiles with
// 64-deep K tiles (four blocks per CU) are never behind the other variants by more than a few per cent, and
// splitting K pays only while the tiles alone leave CUs idle and the K loop is long -- every split costs a
// second kernel that sums fp32 partials.
static IgemmPlan plan_igemm(int64_t M, int N, int Ktot, int ci) {
    IgemmPlan pl{};
    pl.big = 0;
    pl.bk = (ci % 64 == 0) ? 64 : 32;
    pl.kt_total = Ktot / pl.bk;
    const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64);
    const int kt64 = Ktot / 64;                                   // K depth in units of 64
    // about 8 K tiles per block: timed alone a contraction is fastest at about 14, but inside a step, where two or
    // three kernels share the GPU and a K tile takes longer, shorter loops win (VGG-16/CIFAR: -5 % locked, -2 % overlapped)
    int kpb = 8;
    int s = std::max(1, (kt64 + kpb / 2) / kpb);
    // no more blocks than fill the chip once -- except for a single row of tiles (a small-batch FC layer), which
    // only streams weights and needs many blocks in flight to cover the memory latency
    int64_t cap_blocks = 320;
    const int64_t cap = (M <= 64 ? 1024 : cap_blocks) / tiles;
    s = (int)std::min<int64_t>(s, std::max<int64_t>(1, cap));
    s = std::min(s, pl.kt_total);
    pl.splits = std::max(1, s);
    pl.kt_per = (pl.kt_total + pl.splits - 1) / pl.splits;
    pl.splits = (pl.kt_total + pl.kt_per - 1) / pl.kt_per;
    return pl;
}


template <int MODE>
static void launch_igemm_cfg(const IgemmPlan& pl, const IgemmArgs& a, hipStream_t st) {
    const int mt = a.m_tiles ? a.m_tiles : (a.M + 63) / 64;
    const dim3 grid((unsigned)(mt * ((a.N + 63) / 64)), 1, pl.splits);
    if (pl.bk == 64) hipLaunchKernelGGL((igemm_kernel<64, 64, 64, 2, 2, MODE>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((igemm_kernel<64, 64, 32, 2, 2, MODE>), grid, dim3(256), 0, st, a);
}

static hipError_t run_igemm(int mode, IgemmArgs a, void* ws, hipStream_t st) {
    a.wshift = a.hshift = -1;
    if (a.Di < 1) a.Di = 1;
    if (a.Dr < 1) a.Dr = 1;
    if (a.Kd < 1) a.Kd = 1;
    if (a.Wr > 0 && a.Hr > 0 && !(a.Wr & (a.Wr - 1)) && !(a.Hr & (a.Hr - 1))) {
        a.wshift = __builtin_ctz((unsigned)a.Wr);
        a.hshift = __builtin_ctz((unsigned)a.Hr);
    }
    const IgemmPlan pl = plan_igemm(a.M, a.N, a.plan_K ? a.plan_K : a.Ktot, a.Ci);
    a.kt_total = pl.kt_total;
    a.kt_per_split = pl.kt_per;
    a.part = pl.splits > 1 ? (float*)ws : nullptr;
    if (mode == MODE_FWD) launch_igemm_cfg<MODE_FWD>(pl, a, st);
    else if (a.stride == 1) launch_igemm_cfg<MODE_DGRAD>(pl, a, st);
    else launch_igemm_cfg<MODE_DGRAD_S>(pl, a, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.splits == 1) return e;
    const int64_t MN = (int64_t)a.M * a.N;
    if (a.fwd_pool)
        hipLaunchKernelGGL(splitk_epilogue_pool, dim3((unsigned)((a.M / 4) * ((a.N + 63) / 64))), dim3(256), 0, st, (const float*)ws, pl.splits,
                           MN, a.N, a.Hr, a.Wr, a.scale, a.bias, a.relu, a.C, a.fwd_pool);
    else if (a.pool_x)
        hipLaunchKernelGGL(splitk_epilogue_unpool, dim3((unsigned)((MN + 255) / 256)), dim3(256), 0, st, (const float*)ws,
                           pl.splits, MN, a.N, a.Hr, a.Wr, a.pool_x, a.pool_dst, a.pool_acc, a.pool_mask, a.mscale);
    else if ((a.N & 3) == 0)
        hipLaunchKernelGGL(splitk_epilogue_x4, dim3((unsigned)((MN / 4 + 255) / 256)), dim3(256), 0, st, (const float*)ws, pl.splits,
                           MN, a.N, a.scale, a.bias, a.add, a.relu, a.accumulate, a.mask, a.mscale, a.C, a.C2, a.acc2, a.c2scale);
    else
        hipLaunchKernelGGL(splitk_epilogue, dim3((unsigned)((MN + 255) / 256)), dim3(256), 0, st, (const float*)ws, pl.splits,
                           MN, a.N, a.scale, a.bias, a.add, a.relu, a.accumulate, a.mask, a.mscale, a.C, a.C2, a.acc2, a.c2scale);
    return hipGetLastError();
}

// 32-bit byte offsets into every operand, 32-bit element counts of the output
static bool fits32(const ConvGeom& g) {
    const int64_t lim = (int64_t)1 << 31;
    return g.rows_in() * g.Cin < lim && g.rows_out() * g.Cout < lim && (int64_t)g.Cout * g.K() < lim;
}
bool mfma_fwd_ok(const ConvGeom& g) { return g.Cin % 32 == 0 && fits32(g); }
// (a strided data gradient goes by residue classes of the image axes: stride^2 classes, stride^3 for a volume -- at most 16)
bool mfma_dgrad_ok(const ConvGeom& g) { return g.Cout % 32 == 0 && g.stride <= 4 && (g.stride <= 2 || !g.is3d()) && fits32(g); }

size_t mfma_fwd_ws_bytes(const ConvGeom& g) {
    const IgemmPlan pl = plan_igemm(g.rows_out(), g.Cout, g.K(), g.Cin);
    return pl.splits > 1 ? (size_t)pl.splits * g.rows_out() * g.Cout * sizeof(float) : 0;
}
// K a residue class of a strided data gradient runs over at most: the taps of matching parity
static int dgrad_plan_K(const ConvGeom& g) {
    const int s = g.stride;
    return ((g.Kd + s - 1) / s) * ((g.Kh + s - 1) / s) * ((g.Kw + s - 1) / s) * g.Cout;
}

size_t mfma_dgrad_ws_bytes(const ConvGeom& g) {
    const IgemmPlan pl = plan_igemm(g.rows_in(), g.Cin, dgrad_plan_K(g), g.Cout);
    return pl.splits > 1 ? (size_t)pl.splits * g.rows_in() * g.Cin * sizeof(float) : 0;
}

// whether the forward contraction of this layer can also store the 2x2 max-pooling of its output (pool_y below):
// the split-K form, whose second kernel sees whole pooling windows
bool mfma_fwd_pools(const ConvGeom& g) {
    return mfma_fwd_ok(g) && !g.is3d() && !(g.Ho & 1) && !(g.Wo & 1) && plan_igemm(g.rows_out(), g.Cout, g.K(), g.Cin).splits > 1;
}

hipError_t mfma_conv_fwd(const ConvGeom& g, const void* x, const void* w, const float* scale, const float* bias,
                         const void* add, int relu, void* y, void* ws, hipStream_t st, void* pool_y) {
    if (pool_y && (add || !mfma_fwd_pools(g))) return hipErrorInvalidValue;
    IgemmArgs a{};
    a.fwd_pool = (uint16_t*)pool_y;
    a.A = (const uint16_t*)x; a.B = (const uint16_t*)w; a.C = (uint16_t*)y;
    a.scale = scale; a.bias = bias; a.add = (const uint16_t*)add; a.relu = relu; a.accumulate = 0;
    a.M = (int)g.rows_out(); a.N = g.Cout; a.Ktot = g.K();
    a.Hi = g.H; a.Wi = g.W; a.Ci = g.Cin; a.Hr = g.Ho; a.Wr = g.Wo; a.Kw = g.Kw; a.stride = g.stride; a.pad = g.pad;
    a.Kh = g.Kh;
    a.Di = g.D; a.Dr = g.Do; a.Kd = g.Kd; a.pad_d = g.pad_d;
    a.a_bytes = (unsigned)(g.rows_in() * g.Cin * 2); a.b_bytes = (unsigned)((int64_t)g.Cout * g.K() * 2);
    return run_igemm(MODE_FWD, a, ws, st);
}

// wt: weights laid out [Cin][Kh][Kw][Cout]
// side (may be NULL): the gradient is the last contribution to a tensor whose producer's epilogue backward this kernel
// performs -- see DgradSide
hipError_t mfma_conv_dgrad(const ConvGeom& g, const void* dz, const void* wt, void* dx, int accumulate, const void* mask,
                           const float* mscale, void* ws, hipStream_t st, const UnpoolDesc* unpool, const DgradSide* side) {
    if (side && unpool) return hipErrorInvalidValue;
    IgemmArgs a{};
    a.A = (const uint16_t*)dz; a.B = (const uint16_t*)wt; a.C = (uint16_t*)dx;
    a.accumulate = accumulate; a.mask = (const uint16_t*)mask; a.mscale = mscale;
    if (side) { a.add = (const uint16_t*)side->earlier; a.C2 = (uint16_t*)side->shortcut; a.acc2 = side->shortcut_acc; a.c2scale = side->shortcut_scale; }
    if (unpool) {
        a.C = nullptr; a.accumulate = 0; a.mask = nullptr;
        a.pool_x = (const uint16_t*)unpool->pool_x; a.pool_dst = (uint16_t*)unpool->dst;
        a.pool_acc = unpool->accumulate; a.pool_mask = unpool->mask; a.mscale = unpool->mscale;
    }
    a.M = (int)g.rows_in(); a.N = g.Cin; a.Ktot = g.taps() * g.Cout;
    a.Di = g.Do; a.Dr = g.D; a.Kd = g.Kd; a.pad_d = g.pad_d;
    a.Hi = g.Ho; a.Wi = g.Wo; a.Ci = g.Cout; a.Hr = g.H; a.Wr = g.W; a.Kw = g.Kw; a.stride = g.stride; a.pad = g.pad;
    a.a_bytes = (unsigned)(g.rows_out() * g.Cout * 2); a.b_bytes = (unsigned)((int64_t)g.Cout * g.K() * 2);
    a.Kh = g.Kh;
    a.plan_K = dgrad_plan_K(g);
    if (g.stride > 1) {          // row tiles per residue class (d % stride, h % stride, w % stride)
        const int s = g.stride, ncls = (g.D > 1 ? s : 1) * s * s;
        int t = 0;
        for (int c = 0; c < ncls; ++c) {
            a.cls_tile0[c] = t;
            const int pd = c / (s * s), ph = (c / s) % s, pw = c % s;
            const int64_t Dc = g.D > 1 ? (g.D - pd + s - 1) / s : 1, Hc = (g.H - ph + s - 1) / s, Wc = (g.W - pw + s - 1) / s;
            t += (int)(((int64_t)g.m * Dc * Hc * Wc + 63) / 64);
        }
        for (int c = ncls; c <= 16; ++c) a.cls_tile0[c] = t;
        a.m_tiles = t;
    }
    return run_igemm(MODE_DGRAD, a, ws, st);
}

// --------------------------------------------------------------------------------------------------
// weight gradient
struct WgradArgs {
    const uint16_t* X;
    const uint16_t* DZ;
    float* out;            // dW, or the partials base when splits > 1
    float* db;             // bias gradient (column sums of dz), or NULL
    const float* rscale;   // the layer's per-channel scale, or NULL: dz is the gradient before that scale, so row co of dW is multiplied by it
    size_t part_stride;    // floats between the partials of consecutive splits (>= Cout*K + Cout)
    unsigned dz_bytes, x_bytes;   // extents of DZ and X for the buffer resources
    int Cout, Cin, KhKw, Kw;
    int H, W, Ho, Wo, stride, pad;
    int R;                 // reduction length m*Ho*Wo
    int rt_total, rt_per_split, splits;
    int accumulate;
    int co_tiles, ci_tiles;
    int x_cin, x_taps;     // flattened mode (see wgrad_kernel): channels and filter taps of the real input
    int Kh, D, Do, pad_d;  // volumetric layers: filter height (KhKw then counts Kd*Kh*Kw taps), slices in / out, depth padding
};

template <int LDK>
__device__ __forceinline__ void transpose4x8_store(const uint4 (&q)[4], uint16_t* dst /* row 0 of the 8 channels */) {
    const uint32_t d[4][4] = {{q[0].x, q[0].y, q[0].z, q[0].w}, {q[1].x, q[1].y, q[1].z, q[1].w},
                              {q[2].x, q[2].y, q[2].z, q[2].w}, {q[3].x, q[3].y, q[3].z, q[3].w}};
#pragma unroll
    for (int pr = 0; pr < 4; ++pr) {
        // channel 2*pr: low halves; channel 2*pr+1: high halves; 4 pixels -> 8 bytes, K-contiguous
        const uint32_t lo0 = __builtin_amdgcn_perm(d[1][pr], d[0][pr], 0x05040100u);
        const uint32_t lo1 = __builtin_amdgcn_perm(d[3][pr], d[2][pr], 0x05040100u);
        const uint32_t hi0 = __builtin_amdgcn_perm(d[1][pr], d[0][pr], 0x07060302u);
        const uint32_t hi1 = __builtin_amdgcn_perm(d[3][pr], d[2][pr], 0x07060302u);
        *reinterpret_cast<uint2*>(dst + (2 * pr) * LDK) = make_uint2(lo0, lo1);
        *reinterpret_cast<uint2*>(dst + (2 * pr + 1) * LDK) = make_uint2(hi0, hi1);
    }
}

// FLAT: for an input of very few channels (an image: Cin*Kh*Kw <= BN) the N dimension of the tile is the
// flattened (tap, channel) index instead of the channels of one tap; its operand is gathered 2 bytes at a time.
// There p.Cin holds Cin*Kh*Kw and p.KhKw is 1, so the output index is the same expression in both modes.
template <int BM, int BN, int BK, bool FLAT>
__global__ void __launch_bounds__(256, 2) wgrad_kernel(WgradArgs p) {
    typedef TileCfg<BM, BN, 2, 2> Cfg;
    // LDS rows of BK + 12 elements: 8 rows apart is 192 bytes apart modulo the 256-byte bank period, so the 4
    // channel chunks x 8 pixel groups a half-wavefront writes per step fall on distinct banks (an item mapping
    // with all 16 chunks in one wavefront put 88 % of the LDS cycles into bank conflicts).
    constexpr int LDK = BK + 12;
    constexpr int RGS = BK / 4;       // pixel groups per tile
    constexpr int A_ITEMS = (BM / 8) * (BK / 4), B_ITEMS = (BN / 8) * (BK / 4);   // item = 4 pixels x 8 channels
    constexpr int A_PT = (A_ITEMS + 255) / 256, B_PT = (B_ITEMS + 255) / 256;
    __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * LDK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // Workgroups go to the 8 XCDs round-robin in launch order (x fastest, then z).  All tiles of one pixel range
    // read the same dz and x rows (each filter tap a shifted copy), so they are given to one XCD, whose L2 then
    // serves the repeats: virtual index = position in the XCD's contiguous share, pixel range outermost.
    const int v_id = xcd_remap((int)(blockIdx.z * gridDim.x + blockIdx.x), (int)(gridDim.x * gridDim.z));
    const int split = v_id / (int)gridDim.x;
    int tile = v_id - split * (int)gridDim.x;
    const int ci_t = tile % p.ci_tiles; tile /= p.ci_tiles;
    const int tap = tile % p.KhKw;
    const int co_t = tile / p.KhKw;
    const int co0 = co_t * BM, ci0 = ci_t * BN;
    const int kd = tap / (p.Kh * p.Kw), tap2 = tap - kd * (p.Kh * p.Kw);
    const int kh = tap2 / p.Kw, kw = tap2 - kh * p.Kw;
    const int rt0 = split * p.rt_per_split, rt1 = min(p.rt_total, rt0 + p.rt_per_split);

    // Two pixel tiles in flight in registers; out-of-range items (ragged channels, pixels past the end, taps
    // in the padding) load zeros through the buffer resources.
    const __amdgpu_buffer_rsrc_t rsD = make_rsrc(p.DZ, p.dz_bytes), rsX = make_rsrc(p.X, p.x_bytes);
    uint4 qa0[A_PT][4], qb0[B_PT][4], qa1[A_PT][4], qb1[B_PT][4];
    unsigned short qs0[B_PT][4][8], qs1[B_PT][4][8];      // FLAT: the raw 2-byte gathers of the B items

    // Cursors of the next pixel tile to load (tiles are loaded strictly in order).  Per item: the first of its
    // 4 pixels as (row index, wo, ho, image); a tile step adds BK pixels with carries, pixels 1..3 follow by +1.
    const int step_wo = BK % p.Wo, step_q = BK / p.Wo, step_ho = step_q % p.Ho, step_n = step_q / p.Ho;
    int cur_rt = rt0;
    int a_r[A_PT];
    unsigned a_off[A_PT];
    bool a_chok[A_PT];
    int b_r[B_PT], b_wo[B_PT], b_ho[B_PT], b_n[B_PT];
    unsigned b_choff[B_PT];
    bool b_chok[B_PT];
#pragma unroll
    for (int t = 0; t < A_PT; ++t) {
        const int item = tid + t * 256, rg = (item >> 2) % RGS, cc = (item & 3) + 4 * (item / (4 * RGS));
        const int ch = co0 + cc * 8;
        a_chok[t] = (item < A_ITEMS) & (ch < p.Cout);
        a_r[t] = rt0 * BK + rg * 4;
        a_off[t] = (unsigned)(a_r[t] * p.Cout + ch) * 2u;
    }
#pragma unroll
    for (int t = 0; t < B_PT; ++t) {
        const int item = tid + t * 256, rg = (item >> 2) % RGS, cc = (item & 3) + 4 * (item / (4 * RGS));
        const int ch = ci0 + cc * 8;
        b_chok[t] = (item < B_ITEMS) & (ch < p.Cin);
        b_choff[t] = (unsigned)ch * 2u;
        b_r[t] = rt0 * BK + rg * 4;
        const int q = b_r[t] / p.Wo;
        b_wo[t] = b_r[t] - q * p.Wo; b_ho[t] = q % p.Ho; b_n[t] = q / p.Ho;
    }
    // FLAT: the 8 (tap, channel) indices of an item -- element offset from the pixel at tap (0,0), and the tap
    int f_off[B_PT][8], f_hw[B_PT][8];        // f_hw = kd << 24 | kh << 12 | kw, or -1 when the index is past Cin*Kd*Kh*Kw
    if (FLAT) {
#pragma unroll
        for (int t = 0; t < B_PT; ++t) {
            const int item = tid + t * 256, cc = (item & 3) + 4 * (item / (4 * RGS));
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = ci0 + cc * 8 + e;
                const int tp = k / p.x_cin, ci = k - tp * p.x_cin, td = tp / (p.Kh * p.Kw), tr = tp - td * (p.Kh * p.Kw);
                const int th = tr / p.Kw, tw = tr - th * p.Kw;
                const bool ok = (item < B_ITEMS) & (k < p.Cin);
                f_off[t][e] = ((td * p.H + th) * p.W + tw) * p.x_cin + ci;      // (a volume's slices are consecutive images)
                f_hw[t][e] = ok ? ((td << 24) | (th << 12) | tw) : -1;
            }
        }
    }

#define LPM_LOAD_TILE(QA, QB, QS)                                                                            \
    {                                                                                                        \
        const bool live_ = cur_rt < rt1;                                                                     \
        _Pragma("unroll") for (int t = 0; t < A_PT; ++t) {                                                   \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                  \
                const bool ok_ = a_chok[t] & live_ & (a_r[t] + j < p.R);                                     \
                QA[t][j] = buf_load16(rsD, ok_ ? a_off[t] + (unsigned)(j * p.Cout) * 2u : OOB);              \
            }                                                                                                \
            a_r[t] += BK; a_off[t] += (unsigned)(BK * p.Cout) * 2u;                                          \
        }                                                                                                    \
        _Pragma("unroll") for (int t = 0; t < B_PT; ++t) {                                                   \
            int wo_ = b_wo[t], ho_ = b_ho[t], n_ = b_n[t];                                                   \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                  \
                if (FLAT) {                                                                                  \
                    const int h0_ = ho_ * p.stride - p.pad, w0_ = wo_ * p.stride - p.pad;                    \
                    int img0_ = n_, d0_ = 0;      /* n_ counts (sample, output slice) pairs */                   \
                    if (p.Do > 1 || p.D > 1) { const int ns_ = n_ / p.Do; d0_ = (n_ - ns_ * p.Do) * p.stride - p.pad_d; img0_ = ns_ * p.D + d0_; } \
                    const int base_ = ((img0_ * p.H + h0_) * p.W + w0_) * p.x_cin;                           \
                    const bool pix_ = live_ & (b_r[t] + j < p.R);                                            \
                    _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                          \
                        const int hw_ = f_hw[t][e];                                                          \
                        const bool ok_ = pix_ & (hw_ >= 0) & ((unsigned)(h0_ + ((hw_ >> 12) & 0xfff)) < (unsigned)p.H) & \
                                         ((unsigned)(w0_ + (hw_ & 0xfff)) < (unsigned)p.W) &                 \
                                         ((unsigned)(d0_ + (hw_ >> 24)) < (unsigned)p.D);                    \
                        QS[t][j][e] = buf_load2(rsX, ok_ ? (unsigned)(base_ + f_off[t][e]) * 2u : OOB);      \
                    }                                                                                        \
                } else {                                                                                     \
                    const int h_ = ho_ * p.stride + kh - p.pad, w_ = wo_ * p.stride + kw - p.pad;            \
                    int img_ = n_, d_ = 0;        /* n_ counts (sample, output slice) pairs */                   \
                    if (p.Do > 1 || p.D > 1) { const int ns_ = n_ / p.Do; d_ = (n_ - ns_ * p.Do) * p.stride + kd - p.pad_d; img_ = ns_ * p.D + d_; } \
                    const bool ok_ = b_chok[t] & live_ & (b_r[t] + j < p.R) & ((unsigned)h_ < (unsigned)p.H) & \
                                     ((unsigned)w_ < (unsigned)p.W) & ((unsigned)d_ < (unsigned)p.D);        \
                    QB[t][j] = buf_load16(rsX, ok_ ? (unsigned)(((img_ * p.H + h_) * p.W + w_) * p.Cin) * 2u + b_choff[t] : OOB); \
                }                                                                                            \
                ++wo_;                                                                                       \
                if (wo_ == p.Wo) { wo_ = 0; ++ho_; if (ho_ == p.Ho) { ho_ = 0; ++n_; } }                     \
            }                                                                                                \
            b_r[t] += BK;                                                                                    \
            b_wo[t] += step_wo; b_ho[t] += step_ho; b_n[t] += step_n;                                        \
            if (b_wo[t] >= p.Wo) { b_wo[t] -= p.Wo; ++b_ho[t]; }                                             \
            if (b_ho[t] >= p.Ho) { b_ho[t] -= p.Ho; ++b_n[t]; }                                              \
        }                                                                                                    \
        ++cur_rt;                                                                                            \
    }
#define LPM_STORE_TILE(BUF, QA, QB, QS)                                                                      \
    {                                                                                                        \
        _Pragma("unroll") for (int t = 0; t < A_PT; ++t) {                                                   \
            const int item_ = tid + t * 256, rg_ = (item_ >> 2) % RGS, cc_ = (item_ & 3) + 4 * (item_ / (4 * RGS)); \
            if (item_ < A_ITEMS) transpose4x8_store<LDK>(QA[t], &As[BUF][(cc_ * 8) * LDK + rg_ * 4]);        \
        }                                                                                                    \
        _Pragma("unroll") for (int t = 0; t < B_PT; ++t) {                                                   \
            const int item_ = tid + t * 256, rg_ = (item_ >> 2) % RGS, cc_ = (item_ & 3) + 4 * (item_ / (4 * RGS)); \
            if (FLAT) {                                                                                      \
                _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                \
                    QB[t][j] = make_uint4(QS[t][j][0] | ((uint32_t)QS[t][j][1] << 16), QS[t][j][2] | ((uint32_t)QS[t][j][3] << 16), \
                                          QS[t][j][4] | ((uint32_t)QS[t][j][5] << 16), QS[t][j][6] | ((uint32_t)QS[t][j][7] << 16)); \
            }                                                                                                \
            if (item_ < B_ITEMS) transpose4x8_store<LDK>(QB[t], &Bs[BUF][(cc_ * 8) * LDK + rg_ * 4]);        \
        }                                                                                                    \
    }

    f32x16 acc[Cfg::MI][Cfg::NI];
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    // the blocks of filter tap 0 / Cin tile 0 also sum their dz tile over the pixels: the bias gradient
    const bool do_bias = p.db != nullptr && tap == 0 && ci_t == 0;
    float bsum = 0.f;

    const int wm = wave >> 1, wn = wave & 1;
    auto bias_tile = [&](int buf) __attribute__((always_inline)) {
        if (do_bias && tid < BM) {
            const uint2* rowp = reinterpret_cast<const uint2*>(&As[buf][tid * LDK]);
#pragma unroll
            for (int k = 0; k < BK / 4; ++k) {
                const uint2 v = rowp[k];
                bsum += (bf2f((uint16_t)(v.x & 0xffffu)) + bf2f((uint16_t)(v.x >> 16))) +
                        (bf2f((uint16_t)(v.y & 0xffffu)) + bf2f((uint16_t)(v.y >> 16)));
            }
        }
    };
    const int nk = rt1 - rt0;
    if (nk > 0) {
        LPM_LOAD_TILE(qa0, qb0, qs0);
        LPM_LOAD_TILE(qa1, qb1, qs1);
        LPM_STORE_TILE(0, qa0, qb0, qs0);
        __syncthreads();
        // pixel tiles in pairs with no exit in between; an odd count is padded by one all-zero tile
        const int npair = (nk + 1) >> 1;
        for (int it = 0; it < npair; ++it) {
            LPM_LOAD_TILE(qa0, qb0, qs0);
            bias_tile(0);
            mma_tile<Cfg::MI, Cfg::NI, BK, LDK, true>(As[0], Bs[0], wm * Cfg::WTM, wn * Cfg::WTN, lane, acc);
            LPM_STORE_TILE(1, qa1, qb1, qs1);
            __syncthreads();
            LPM_LOAD_TILE(qa1, qb1, qs1);
            bias_tile(1);
            mma_tile<Cfg::MI, Cfg::NI, BK, LDK, true>(As[1], Bs[1], wm * Cfg::WTM, wn * Cfg::WTN, lane, acc);
            LPM_STORE_TILE(0, qa0, qb0, qs0);
            __syncthreads();
        }
    }
#undef LPM_LOAD_TILE
#undef LPM_STORE_TILE

    const size_t total = (size_t)p.Cout * p.KhKw * p.Cin;
    float* out = p.out + (p.splits > 1 ? (size_t)split * p.part_stride : 0);
    if (do_bias && tid < BM && co0 + tid < p.Cout) {
        const int co = co0 + tid;
        if (p.splits > 1) out[total + co] = bsum;
        else {
            p.db[co] = p.accumulate ? p.db[co] + bsum : bsum;
        }
    }
    const int col_l = lane & 31, rq = (lane >> 5) * 4;
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni) {
        const int ci = ci0 + wn * Cfg::WTN + ni * 32 + col_l;
        if (ci >= p.Cin) continue;
#pragma unroll
        for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int co = co0 + wm * Cfg::WTM + mi * 32 + (i >> 2) * 8 + rq + (i & 3);
                if (co >= p.Cout) continue;
                const size_t o = ((size_t)co * p.KhKw + tap) * p.Cin + ci;
                float v = acc[mi][ni][i];
                if (p.splits == 1 && p.rscale) v *= p.rscale[co];
                if (p.splits == 1 && p.accumulate) v += out[o];
                out[o] = v;
            }
    }
}

struct WgradPlan { int big; int bk; int splits; int rt_total; int rt_per; int co_tiles, ci_tiles; };

// Measured on the same shapes: 128x128 tiles win once the contraction is large (about 6e9 multiply-adds), the
// 64x64 tile otherwise, with 128-pixel tiles when there are at least 1024 pixels; the pixel range is split
// until one wave of blocks (two per CU) is full, keeping at least four pixel tiles per block.
static WgradPlan plan_wgrad(const ConvGeom& g) {
    WgradPlan pl{};
    const int64_t R = g.rows_out();
    const double macs = (double)R * g.Cout * g.K();
    pl.big = (g.Cout >= 128 && g.Cin >= 128 && macs >= 6e9);
    pl.bk = pl.big ? 64 : (R >= 1024 ? 128 : 64);
    pl.rt_total = (int)((R + pl.bk - 1) / pl.bk);
    const int t = pl.big ? 128 : 64;
    pl.co_tiles = (g.Cout + t - 1) / t;
    pl.ci_tiles = (g.Cin + t - 1) / t;
    const int64_t tiles = (int64_t)pl.co_tiles * pl.ci_tiles * g.taps();
    int s = (int)std::min<int64_t>(512 / std::max<int64_t>(tiles, 1), std::max(1, pl.rt_total / 4));
    if (s > 24) s = 24;          // beyond this the partial sums cost more than the shorter pixel loops save
    // the partials must stay modest for very large weight tensors
    const int64_t wbytes = (int64_t)g.Cout * g.K() * 4;
    while (s > 1 && wbytes * s > (256ll << 20)) --s;
    if (s < 1) s = 1;
    pl.rt_per = (pl.rt_total + s - 1) / s;
    pl.splits = (pl.rt_total + pl.rt_per - 1) / pl.rt_per;
    return pl;
}

bool mfma_wgrad_ok(const ConvGeom& g) { return g.Cin % 8 == 0 && g.Cout % 8 == 0 && fits32(g); }

size_t mfma_wgrad_ws_bytes(const ConvGeom& g) {
    const WgradPlan pl = plan_wgrad(g);
    return pl.splits > 1 ? (size_t)pl.splits * ((size_t)g.Cout * g.K() + g.Cout) * sizeof(float) : 0;
}

// dbias (may be NULL): also produce the bias gradient, the per-channel sum of dz; rscale (may be NULL): per-row factor of dW
struct ReduceBatchArgs {
    ReduceDesc d[LPM_REDUCE_BATCH];
    int64_t first[LPM_REDUCE_BATCH + 1];     // first thread of every reduction (a thread sums four outputs)
    int count;
};

// A thread sums four consecutive outputs over the splits with 16-byte loads, four splits in flight (split s goes to
// chain s % 4, the chains are added pairwise at the end: a fixed order); the bias part and ragged ends go one by one.
__global__ void __launch_bounds__(256) wgrad_reduce_batch(ReduceBatchArgs a) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= a.first[a.count]) return;
    int k = 0;
    while (k + 1 < a.count && t >= a.first[k + 1]) ++k;
    const ReduceDesc& d = a.d[k];
    const int64_t i = (t - a.first[k]) * 4;
    if (i >= d.n + d.nb) return;              // padding up to a whole block
    if (i + 4 <= d.n && (d.stride & 3) == 0 && (d.row_len & 3) == 0) {
        float4 c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) c[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        const float* p = d.part + i;
        int s = 0;
        for (; s + 4 <= d.splits; s += 4) {
            float4 v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = *reinterpret_cast<const float4*>(p + (size_t)(s + j) * d.stride);
#pragma unroll
            for (int j = 0; j < 4; ++j) { c[j].x += v[j].x; c[j].y += v[j].y; c[j].z += v[j].z; c[j].w += v[j].w; }
        }
#pragma unroll
        for (int j = 0; j < 3; ++j) {             // the last one to three splits (static chain index: registers)
            if (s + j < d.splits) {
                const float4 v = *reinterpret_cast<const float4*>(p + (size_t)(s + j) * d.stride);
                c[j].x += v.x; c[j].y += v.y; c[j].z += v.z; c[j].w += v.w;
            }
        }
        float4 r = make_float4((c[0].x + c[1].x) + (c[2].x + c[3].x), (c[0].y + c[1].y) + (c[2].y + c[3].y),
                               (c[0].z + c[1].z) + (c[2].z + c[3].z), (c[0].w + c[1].w) + (c[2].w + c[3].w));
        if (d.rscale) {                           // (row_len is a multiple of 4 on this path: the four outputs share a row)
            const float f = d.rscale[i / d.row_len];
            r.x *= f; r.y *= f; r.z *= f; r.w *= f;
        }
        float4* o = reinterpret_cast<float4*>(d.dst + i);
        if (d.accumulate) { const float4 q = *o; r.x += q.x; r.y += q.y; r.z += q.z; r.w += q.w; }
        *o = r;
        return;
    }
    for (int64_t e = i; e < i + 4 && e < d.n + d.nb; ++e) {
        float acc = d.part[e];
        for (int s = 1; s < d.splits; ++s) acc += d.part[(size_t)s * d.stride + e];
        if (e < d.n) {
            if (d.rscale) acc *= d.rscale[e / d.row_len];
            d.dst[e] = d.accumulate ? d.dst[e] + acc : acc;
        } else {
            const int c = (int)(e - d.n);
            d.db[c] = d.accumulate ? d.db[c] + acc : acc;
        }
    }
}

hipError_t launch_reduce_batch(const ReduceDesc* d, int count, hipStream_t st) {
    for (int done = 0; done < count;) {
        ReduceBatchArgs a{};
        int64_t tot = 0;
        int k = 0;
        for (; k < LPM_REDUCE_BATCH && done + k < count; ++k) {
            a.d[k] = d[done + k];
            a.first[k] = tot;
            // a thread per four outputs, whole blocks per reduction: a block never straddles two of them
            tot += (((a.d[k].n + a.d[k].nb + 3) / 4 + 255) / 256) * 256;
        }
        a.first[k] = tot;
        a.count = k;
        done += k;
        if (tot == 0) continue;
        hipLaunchKernelGGL(wgrad_reduce_batch, dim3((unsigned)(tot / 256)), dim3(256), 0, st, a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t mfma_conv_wgrad(const ConvGeom& g, const void* x, const void* dz, float* dw, float* dbias, const float* rscale,
                           int accumulate, void* ws, hipStream_t st, ReduceDesc* deferred) {
    const WgradPlan pl = plan_wgrad(g);
    WgradArgs a{};
    a.X = (const uint16_t*)x; a.DZ = (const uint16_t*)dz;
    a.out = pl.splits > 1 ? (float*)ws : dw;
    a.Cout = g.Cout; a.Cin = g.Cin; a.KhKw = g.taps(); a.Kw = g.Kw;
    a.Kh = g.Kh; a.D = g.D; a.Do = g.Do; a.pad_d = g.pad_d;
    a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo; a.stride = g.stride; a.pad = g.pad;
    a.R = (int)g.rows_out();
    a.db = dbias; a.rscale = rscale;
    a.part_stride = (size_t)g.Cout * g.K() + g.Cout;
    a.dz_bytes = (unsigned)(g.rows_out() * g.Cout * 2); a.x_bytes = (unsigned)(g.rows_in() * g.Cin * 2);
    a.rt_total = pl.rt_total; a.rt_per_split = pl.rt_per; a.splits = pl.splits;
    a.accumulate = accumulate;
    a.co_tiles = pl.co_tiles; a.ci_tiles = pl.ci_tiles;
    const dim3 grid((unsigned)(pl.co_tiles * pl.ci_tiles * a.KhKw), 1, pl.splits);
    if (pl.big) hipLaunchKernelGGL((wgrad_kernel<128, 128, 64, false>), grid, dim3(256), 0, st, a);
    else if (pl.bk == 128) hipLaunchKernelGGL((wgrad_kernel<64, 64, 128, false>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((wgrad_kernel<64, 64, 64, false>), grid, dim3(256), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.splits == 1) return e;
    const int64_t n = (int64_t)g.Cout * g.K();
    const int nb = dbias ? g.Cout : 0;
    // one reduction kernel whether it runs now or batched with the stage's other layers: the same summation order
    const ReduceDesc d{(const float*)ws, a.part_stride, pl.splits, dw, n, dbias, nb, rscale, g.K(), accumulate};
    if (deferred) { *deferred = d; return hipSuccess; }
    return launch_reduce_batch(&d, 1, st);
}

// The same reduction for a short output vector (a first layer's few thousand weights) and many partials:
// 8 lanes share one output, each adds a contiguous eighth of the partials in order, and the eight sums are
// added in lane order -- a fixed order, with 8 loads in flight per output instead of one.
__global__ void __launch_bounds__(256) wgrad_reduce_short(const float* __restrict__ part, size_t stride, int splits,
                                                          float* __restrict__ dst, int64_t n, float* __restrict__ db, int nb,
                                                          const float* __restrict__ rscale, int row_len, int accumulate) {
    __shared__ float red[8][32];
    const int o = threadIdx.x & 31, l = threadIdx.x >> 5;
    const int64_t i = (int64_t)blockIdx.x * 32 + o;
    float acc = 0.f;
    if (i < n + nb) {
        const int per = (splits + 7) / 8;
        const int s1 = min(splits, (l + 1) * per);
        for (int s = l * per; s < s1; ++s) acc += part[(size_t)s * stride + i];
    }
    red[l][o] = acc;
    __syncthreads();
    if (l != 0 || i >= n + nb) return;
    float v = red[0][o];
#pragma unroll
    for (int k = 1; k < 8; ++k) v += red[k][o];
    if (i < n) {
        if (rscale) v *= rscale[i / row_len];
        dst[i] = accumulate ? dst[i] + v : v;
    } else {
        const int c = (int)(i - n);
        db[c] = accumulate ? db[c] + v : v;
    }
}

// Weight gradient of an image-input layer (Cin*Kh*Kw <= 64): one N tile holds every (tap, channel) index.
bool mfma_wgrad_flat_ok(const ConvGeom& g) { return g.K() <= 64 && g.Cout % 8 == 0 && fits32(g); }

static WgradPlan plan_wgrad_flat(const ConvGeom& g) {
    WgradPlan pl{};
    const int64_t R = g.rows_out();
    pl.bk = R >= 1024 ? 128 : 64;
    pl.rt_total = (int)((R + pl.bk - 1) / pl.bk);
    pl.co_tiles = (g.Cout + 63) / 64;
    pl.ci_tiles = 1;
    // the 2-byte gathers make a pixel tile slow (about 2 us), so blocks take as few as two of them
    int s = std::min(std::min(512 / pl.co_tiles, std::max(1, pl.rt_total / 2)), 256);
    pl.rt_per = (pl.rt_total + s - 1) / s;
    pl.splits = (pl.rt_total + pl.rt_per - 1) / pl.rt_per;
    return pl;
}

size_t mfma_wgrad_flat_ws_bytes(const ConvGeom& g) {
    const WgradPlan pl = plan_wgrad_flat(g);
    return pl.splits > 1 ? (size_t)pl.splits * ((size_t)g.Cout * g.K() + g.Cout) * sizeof(float) : 0;
}

hipError_t mfma_conv_wgrad_flat(const ConvGeom& g, const void* x, const void* dz, float* dw, float* dbias,
                                const float* rscale, int accumulate, void* ws, hipStream_t st) {
    const WgradPlan pl = plan_wgrad_flat(g);
    WgradArgs a{};
    a.X = (const uint16_t*)x; a.DZ = (const uint16_t*)dz;
    a.out = pl.splits > 1 ? (float*)ws : dw;
    a.Cout = g.Cout; a.Cin = g.K(); a.KhKw = 1; a.Kw = g.Kw;
    a.Kh = g.Kh; a.D = g.D; a.Do = g.Do; a.pad_d = g.pad_d;
    a.x_cin = g.Cin; a.x_taps = g.taps();
    a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo; a.stride = g.stride; a.pad = g.pad;
    a.R = (int)g.rows_out();
    a.db = dbias; a.rscale = rscale;
    a.part_stride = (size_t)g.Cout * g.K() + g.Cout;
    a.dz_bytes = (unsigned)(g.rows_out() * g.Cout * 2); a.x_bytes = (unsigned)(g.rows_in() * g.Cin * 2);
    a.rt_total = pl.rt_total; a.rt_per_split = pl.rt_per; a.splits = pl.splits;
    a.accumulate = accumulate;
    a.co_tiles = pl.co_tiles; a.ci_tiles = 1;
    const dim3 grid((unsigned)pl.co_tiles, 1, pl.splits);
    if (pl.bk == 128) hipLaunchKernelGGL((wgrad_kernel<64, 64, 128, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((wgrad_kernel<64, 64, 64, true>), grid, dim3(256), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.splits == 1) return e;
    const int64_t n = (int64_t)g.Cout * g.K();
    const int nb = dbias ? g.Cout : 0;
    hipLaunchKernelGGL(wgrad_reduce_short, dim3((unsigned)((n + nb + 31) / 32)), dim3(256), 0, st, (const float*)ws,
                       a.part_stride, pl.splits, dw, n, dbias, nb, rscale, g.K(), accumulate);
    return hipGetLastError();
}

}  // namespace lpm
