// Weight gradient (eq. 8) of convolutions whose output images are at least 7x7 pixels: bf16 MFMA, fp32 accumulation.
//
//   dW[co][kh][kw][ci] = sum over output pixels q of dz[q][co] * x[pixel(q, kh, kw)][ci]
//
// The reduction index is the output pixel, and both operands are stored with the pixel outermost
// (dz [m][Ho][Wo][Cout], x [m][H][W][Cin]).  Instead of transposing them on the way into LDS, the tiles are
// copied as they are -- rows of 64 channels, written by loads that go straight from global memory to LDS -- and
// the matrix-instruction operands are fetched with the LDS transpose read of gfx950 (16-bit elements, 64 bits per
// lane): in every group of 16 lanes, lane i supplies the address of 4 consecutive elements of a row, and
// receives element (i % 4) of the rows supplied by lanes 4j + i/4, j = 0..3 -- a column of 4 rows.
//
// A reduction tile is an 8x8 patch of output pixels of one image.  The input pixels that the patch meets under
// a group of filter taps form a small halo tile, loaded once and shared by the taps of the group: the operand
// of tap (kh, kw) is the same LDS tile read at a row offset.  A block owns 64 output x 64 input channels and
// one tap group (all 9 taps of a 3x3 filter, the 3 taps of one filter row, or a single tap), over a range of
// patches; ranges are summed afterwards like the splits of the other weight-gradient kernel.
#include "lpm_internal.h"
#include "elem.h"
#include "lds_dma.h"
#include <algorithm>

namespace lpm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef short short4_ __attribute__((ext_vector_type(4)));
typedef short short8_ __attribute__((ext_vector_type(8)));

struct WgradTrArgs {
    const uint16_t* X;
    const uint16_t* DZ;
    float* out;            // dW, or the partials base when splits > 1
    float* db;             // bias gradient (sum of dz over the pixels), or NULL
    const float* rscale;   // the layer's per-channel scale, or NULL: row co of dW is multiplied by it (dz is the gradient before the scale)
    size_t part_stride;    // floats between the partials of consecutive splits (>= Cout*K + Cout)
    unsigned dz_bytes, x_bytes;
    int Cout, Cin, Kh, Kw, H, W, Ho, Wo, stride, pad;
    int TY, TX;            // patches per image
    int kt_total, kt_per_split, splits;
    int accumulate;
    int co_tiles, ci_tiles, tap_groups;
    int Kd, D, Do, pad_d;  // volumetric layers: filter depth, slices in / out, depth padding (1, 1, 1, 0 otherwise); an "image"
                           // of the patch cursor is one output slice, and a block's taps all lie in one filter slice kd
};

template <int TAPS>
struct TrCfg {
    static constexpr int KH_G = TAPS == 9 ? 3 : 1, KW_G = TAPS == 1 ? 1 : 3;     // taps of a group along h and w
    static constexpr int HH = 8 + KH_G - 1, HW = 8 + KW_G - 1;                  // halo tile (stride 1 when TAPS > 1)
    static constexpr int NB = (HH * HW + 7) / 8;                                 // 1 KiB loads of the halo tile
    static constexpr int BMAX = (NB + 3) / 4;                                    // ... per wavefront, at most
    static constexpr int A_BYTES = 64 * 128, B_BYTES = NB * 1024, STAGE = A_BYTES + B_BYTES;
};

constexpr unsigned TR_OOB = 0xffffffffu;
// 8 reduction values of column `col`: rows r..r+3 and r+4..r+7 of a tile with 128-byte rows
__device__ __forceinline__ bf16x8 tr_fetch(const unsigned char* p) {
    const short4_ lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_*)(p));
    const short4_ hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_*)(p + 4 * 128));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

typedef unsigned int u32x2_ __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x2_ tr_words(const unsigned char* p) {
    return __builtin_bit_cast(u32x2_, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_*)(p)));
}

// NST: stages of the LDS ring; the loads run NST - 1 patches ahead.  Four stages leave room for two blocks per CU;
// a ring of eight for a block alone on its CU measured no faster.
template <int TAPS, int NST>
__global__ void __launch_bounds__(256, 2) wgrad_tr_kernel(WgradTrArgs p) {
    typedef TrCfg<TAPS> C;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];      // NST stages of C::STAGE bytes + 256 (a filter row's third fetch reaches 2 pixels past its halo tile)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // all blocks of one patch range go to one XCD (they read the same dz and x rows)
    const int v_id = xcd_remap((int)(blockIdx.z * gridDim.x + blockIdx.x), (int)(gridDim.x * gridDim.z));
    const int split = v_id / (int)gridDim.x;
    int tile = v_id - split * (int)gridDim.x;
    const int ci_t = tile % p.ci_tiles; tile /= p.ci_tiles;
    const int grp = tile % p.tap_groups;
    const int co_t = tile / p.tap_groups;
    const int co0 = co_t * 64, ci0 = ci_t * 64;
    const int g2d = p.tap_groups / p.Kd, kd = grp / g2d, grp2 = grp - kd * g2d;      // filter slice, tap group inside it
    const int kh0 = TAPS == 9 ? 0 : (TAPS == 3 ? grp2 : grp2 / p.Kw), kw0 = TAPS == 1 ? grp2 % p.Kw : 0;
    const int kt0 = split * p.kt_per_split, nk = min(p.kt_total, kt0 + p.kt_per_split) - kt0;

    const u32x4_ rsD = buffer_words(p.DZ, p.dz_bytes), rsX = buffer_words(p.X, p.x_bytes);

    // ---- loader state: one load writes 1 KiB = 8 tile rows (pixels) x 8 chunks of 8 channels; lane = row * 8 + chunk
    const int l_row = lane >> 3, l_chunk = lane & 7;
    // dz tile: load wl (0..7) is patch row wl; this wavefront takes wl = wave, wave + 4
    const bool a_cok = co0 + l_chunk * 8 < p.Cout;
    unsigned a_loc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) a_loc[i] = (unsigned)(((wave + 4 * i) * p.Wo + l_row) * p.Cout + co0 + l_chunk * 8) * 2u;
    // halo tile: load wl holds halo pixels wl*8 .. wl*8+7 (row-major over HH x HW); this wavefront takes wl = wave + 4i
    const bool b_cok = ci0 + l_chunk * 8 < p.Cin;
    unsigned b_loc[C::BMAX];
    int b_dy[C::BMAX], b_dx[C::BMAX];
    bool b_ok[C::BMAX];
#pragma unroll
    for (int i = 0; i < C::BMAX; ++i) {
        const int hp = (wave + 4 * i) * 8 + l_row, hy = hp / C::HW, hx = hp - hy * C::HW;
        b_ok[i] = b_cok & (hp < C::HH * C::HW);
        b_dy[i] = hy * p.stride; b_dx[i] = hx * p.stride;
        b_loc[i] = (unsigned)((b_dy[i] * p.W + b_dx[i]) * p.Cin + ci0 + l_chunk * 8) * 2u;
    }
    const int nbw = (C::NB - wave + 3) / 4;                 // halo loads of this wavefront: BMAX or BMAX - 1
    // cursor of the next patch to load: image and patch coordinates
    int c_n, c_ty, c_tx;
    {
        const int per = p.TY * p.TX;
        c_n = kt0 / per;
        const int r = kt0 - c_n * per;
        c_ty = r / p.TX; c_tx = r - c_ty * p.TX;
    }

#define LPM_ISSUE(ST)                                                                                         \
    {                                                                                                         \
        unsigned char* st_ = lds + (ST) * C::STAGE;                                                           \
        const int y0_ = c_ty * 8, x0_ = c_tx * 8;                                                             \
        const unsigned baseA_ = (unsigned)(((c_n * p.Ho + y0_) * p.Wo + x0_) * p.Cout) * 2u;                  \
        _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                       \
            const bool ok_ = a_cok & (y0_ + wave + 4 * i < p.Ho) & (x0_ + l_row < p.Wo);                      \
            load_to_lds16(rsD, st_ + (wave + 4 * i) * 1024, ok_ ? baseA_ + a_loc[i] : TR_OOB);                \
        }                                                                                                     \
        const int by_ = y0_ * p.stride + kh0 - p.pad, bx_ = x0_ * p.stride + kw0 - p.pad;                     \
        int imgB_ = c_n;                                                                                      \
        bool dok_ = true;                                                                                     \
        if (p.D > 1 || p.Do > 1) {          /* c_n counts (sample, output slice) pairs */                        \
            const int ns_ = c_n / p.Do, d_ = (c_n - ns_ * p.Do) * p.stride + kd - p.pad_d;                    \
            dok_ = (unsigned)d_ < (unsigned)p.D;                                                              \
            imgB_ = ns_ * p.D + d_;                                                                           \
        }                                                                                                     \
        const unsigned baseB_ = (unsigned)(((imgB_ * p.H + by_) * p.W + bx_) * p.Cin) * 2u;                   \
        _Pragma("unroll") for (int i = 0; i < C::BMAX; ++i) {                                                 \
            if (wave + 4 * i < C::NB) {                                                                       \
                const bool ok_ = b_ok[i] & dok_ & ((unsigned)(by_ + b_dy[i]) < (unsigned)p.H) &               \
                                 ((unsigned)(bx_ + b_dx[i]) < (unsigned)p.W);                                 \
                load_to_lds16(rsX, st_ + C::A_BYTES + (wave + 4 * i) * 1024, ok_ ? baseB_ + b_loc[i] : TR_OOB); \
            }                                                                                                 \
        }                                                                                                     \
        if (++c_tx == p.TX) { c_tx = 0; if (++c_ty == p.TY) { c_ty = 0; ++c_n; } }                            \
    }

    f32x16 acc[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
    // the blocks of tap group 0 / Cin tile 0 also sum dz over the pixels (the bias gradient): one more matrix
    // instruction per step against a tile of ones, on the wavefronts of the first column
    const int wm = wave >> 1, wn = wave & 1;
    const bool do_bias = p.db != nullptr && grp == 0 && ci_t == 0 && wn == 0;
    f32x16 accb;
#pragma unroll
    for (int i = 0; i < 16; ++i) accb[i] = 0.f;
    bf16x8 ones;
#pragma unroll
    for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;

    // operand addresses: reduction rows (lane / 32) * 8 + (lane % 16) / 4 (+ 4 for the second read), columns
    // (lane / 16 % 2) * 16 + (lane % 4) * 4 .. + 3 of the wavefront's 32 -- each lane ends up with column lane % 32
    const int col_b = (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
    const int a_base = ((lane >> 5) * 8 + ((lane & 15) >> 2)) * 128 + wm * 64 + col_b;
    const int b_base = ((lane >> 5) * C::HW + ((lane & 15) >> 2)) * 128 + wn * 64 + col_b + C::A_BYTES;

#pragma unroll
    for (int i = 0; i < NST - 1; ++i)
        if (i < nk) LPM_ISSUE(i);
    int st = 0;
    for (int it = 0; it < nk; ++it) {
        // patch `it` has landed once only the loads of the patches behind it (at most NST - 2) are outstanding
        if (nbw == C::BMAX) wait_tiles_behind<2 + C::BMAX, NST - 2>(nk - 1 - it);
        else wait_tiles_behind<1 + C::BMAX, NST - 2>(nk - 1 - it);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();      // every wavefront's part has landed, and all are done reading the stage loaded next
        asm volatile("" ::: "memory");
        if (it + NST - 1 < nk) {
            const int st2 = st == 0 ? NST - 1 : st - 1;          // (st + NST - 1) % NST
            LPM_ISSUE(st2);
        }
        const unsigned char* sp = lds + st * C::STAGE;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bf16x8 a = tr_fetch(sp + a_base + ks * 16 * 128);
#pragma unroll
            for (int dkh = 0; dkh < C::KH_G; ++dkh) {
                const unsigned char* bp = sp + b_base + ((ks * 2 + dkh) * C::HW) * 128;
                if (C::KW_G == 1) {
                    acc[dkh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, tr_fetch(bp), acc[dkh], 0, 0, 0);
                } else {
                    // the three taps of a filter row read halo pixels x .. x+7, x+1 .. x+8, x+2 .. x+9 of one halo row:
                    // fetch pixels x .. x+11 once (two per 32-bit word) and shift
                    const u32x2_ r0 = tr_words(bp), r1 = tr_words(bp + 4 * 128), r2 = tr_words(bp + 8 * 128);
                    const u32x4_ f0 = {r0.x, r0.y, r1.x, r1.y};
                    const u32x4_ f2 = {r0.y, r1.x, r1.y, r2.x};
                    const u32x4_ f1 = {__builtin_amdgcn_alignbit(r0.y, r0.x, 16), __builtin_amdgcn_alignbit(r1.x, r0.y, 16),
                                       __builtin_amdgcn_alignbit(r1.y, r1.x, 16), __builtin_amdgcn_alignbit(r2.x, r1.y, 16)};
                    acc[dkh * 3 + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, f0), acc[dkh * 3 + 0], 0, 0, 0);
                    acc[dkh * 3 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, f1), acc[dkh * 3 + 1], 0, 0, 0);
                    acc[dkh * 3 + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, f2), acc[dkh * 3 + 2], 0, 0, 0);
                }
            }
            if (do_bias) accb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, ones, accb, 0, 0, 0);
        }
        st = st == NST - 1 ? 0 : st + 1;
    }
#undef LPM_ISSUE

    // accumulator element i of a lane: row (i / 4) * 8 + (lane / 32) * 4 + i % 4, column lane % 32
    const int KhKw = p.Kd * p.Kh * p.Kw;             // all taps of the filter
    const size_t total = (size_t)p.Cout * KhKw * p.Cin;
    float* out = p.out + (p.splits > 1 ? (size_t)split * p.part_stride : 0);
    const int rq = (lane >> 5) * 4;
    if (do_bias && (lane & 31) == 0) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int co = co0 + wm * 32 + (i >> 2) * 8 + rq + (i & 3);
            if (co >= p.Cout) continue;
            if (p.splits > 1) out[total + co] = accb[i];
            else {
                p.db[co] = p.accumulate ? p.db[co] + accb[i] : accb[i];
            }
        }
    }
    const int ci = ci0 + wn * 32 + (lane & 31);
    if (ci < p.Cin) {
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            const int tap = kd * p.Kh * p.Kw + (TAPS == 9 ? t : (TAPS == 3 ? grp2 * 3 + t : grp2));
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int co = co0 + wm * 32 + (i >> 2) * 8 + rq + (i & 3);
                if (co >= p.Cout) continue;
                const size_t o = ((size_t)co * KhKw + tap) * p.Cin + ci;
                float v = acc[t][i];
                if (p.splits == 1 && p.rscale) v *= p.rscale[co];
                if (p.splits == 1 && p.accumulate) v += out[o];
                out[o] = v;
            }
        }
    }
}

// --------------------------------------------------------------------------------------------------
struct TrPlan { int taps, groups, co_tiles, ci_tiles, TY, TX, kt_total, kt_per, splits; };

static bool fits32_tr(const ConvGeom& g) {
    const int64_t lim = (int64_t)1 << 31;
    return g.rows_in() * g.Cin < lim && g.rows_out() * g.Cout < lim && (int64_t)g.Cout * g.K() < lim;
}

static bool tr_shape_ok(const ConvGeom& g) {
    if (g.Cin % 8 != 0 || g.Cout % 8 != 0 || !fits32_tr(g)) return false;
    if (g.Ho < 7 || g.Wo < 7) return false;
    // patches waste the part that hangs over the image edge: at least 3/4 of their pixels must be real
    const int TY = (g.Ho + 7) / 8, TX = (g.Wo + 7) / 8;
    return (int64_t)g.Ho * g.Wo * 4 >= (int64_t)TY * TX * 64 * 3;
}

// A 1x1 stride-1 filter without padding maps output pixel q to input pixel q, so the pixels of the whole micro-batch
// may be regrouped at will: as one image of (pixels / 8) x 8 every 8x8 patch is full (a 14x14 image cut into 2x2 patches
// fills them to 77 %), and small images still give long runs of whole patches.
static ConvGeom tr_view(const ConvGeom& g) {
    const int64_t total = g.rows_out();
    if (g.Kd != 1 || g.Kh != 1 || g.Kw != 1 || g.stride != 1 || g.pad != 0 || g.pad_d != 0 || (total & 7) || (total >> 3) >= ((int64_t)1 << 30))
        return g;
    ConvGeom v = g;
    v.m = 1;
    v.D = v.Do = 1;
    v.H = v.Ho = (int32_t)(total >> 3);
    v.W = v.Wo = 8;
    return v;
}

// Measured on MI355X against the kernel that tiles the flattened pixel index (which transposes in registers):
// this one wins clearly for 3x3 filters over large images (56x56 and up: 1.05x to 1.45x), where the halo tile and
// the untransposed copies save the most, and by 5-10 % on the CIFAR-size layers (15.8 against 17.1 us on
// m16 32x32x64->64), which adds up over a training step (ResNet-18/CIFAR: 5.34 -> 5.10 ms).  It takes every
// shape whose patches are mostly inside the image.
bool wgrad_tr_ok(const ConvGeom& g) {
    return tr_shape_ok(tr_view(g));
}

static TrPlan plan_wgrad_tr(const ConvGeom& g) {
    TrPlan pl{};
    pl.co_tiles = (g.Cout + 63) / 64;
    pl.ci_tiles = (g.Cin + 63) / 64;
    pl.TY = (g.Ho + 7) / 8; pl.TX = (g.Wo + 7) / 8;
    pl.kt_total = g.m * g.Do * pl.TY * pl.TX;
    const int KhKw = g.taps();
    const bool s33 = g.Kh == 3 && g.Kw == 3 && g.stride == 1;
    const int64_t out_bytes = ((int64_t)g.Cout * g.K() + g.Cout) * 4;
    // a filter row per block once both channel counts give several tiles (the shared halo tile then cuts the L2
    // traffic that bounds the single-tap blocks); the patch range is split to about one block per CU, keeping
    // at least eight patches per block and the partial sums (written and read once) below 64 MiB.  (Alone on the
    // GPU a weight gradient is 3-6 % faster at 1.5 blocks per CU; beside the forward and data-gradient kernels of
    // an overlapped step the smaller partial sums win: -1 to -2.6 % per step on the five workloads.)
    const int64_t macs = g.rows_out() * g.Cout * g.K();
    int taps = (s33 && g.Cin >= 128 && g.Cout >= 128 && macs >= (int64_t)1000000000) ? 3 : 1;
    const int64_t base = (int64_t)pl.co_tiles * pl.ci_tiles * (KhKw / taps);
    int64_t target = 256;
    int64_t sp = std::max<int64_t>(1, target / base);
    // (rounding down can leave a third of the CUs without a block -- 144 tile groups of a 3x3 stride-2 layer: the ranges
    //  then fill one wave of two blocks per CU minus a margin instead; measured on that layer 39 / 28 / 23 / 31 us at 1-4 ranges)
    if (base * sp < 192) sp = std::max<int64_t>(sp, 448 / base);
    sp = std::min<int64_t>(sp, std::max(1, pl.kt_total / 8));
    sp = std::min<int64_t>(sp, std::max<int64_t>(1, (64ll << 20) / out_bytes));
    int best_taps = taps, best_s = (int)sp;
    pl.taps = best_taps;
    pl.groups = KhKw / best_taps;
    pl.kt_per = (pl.kt_total + best_s - 1) / best_s;
    pl.splits = (pl.kt_total + pl.kt_per - 1) / pl.kt_per;
    return pl;
}

size_t wgrad_tr_ws_bytes(const ConvGeom& g_) {
    const ConvGeom g = tr_view(g_);
    const TrPlan pl = plan_wgrad_tr(g);
    return pl.splits > 1 ? (size_t)pl.splits * ((size_t)g.Cout * g.K() + g.Cout) * sizeof(float) : 0;
}

hipError_t wgrad_tr(const ConvGeom& g_, const void* x, const void* dz, float* dw, float* dbias, const float* rscale,
                    int accumulate, void* ws, hipStream_t st, ReduceDesc* deferred) {
    const ConvGeom g = tr_view(g_);
    const TrPlan pl = plan_wgrad_tr(g);
    WgradTrArgs a{};
    a.X = (const uint16_t*)x; a.DZ = (const uint16_t*)dz;
    a.out = pl.splits > 1 ? (float*)ws : dw;
    a.db = dbias; a.rscale = rscale;
    a.part_stride = (size_t)g.Cout * g.K() + g.Cout;
    a.dz_bytes = (unsigned)(g.rows_out() * g.Cout * 2); a.x_bytes = (unsigned)(g.rows_in() * g.Cin * 2);
    a.Cout = g.Cout; a.Cin = g.Cin; a.Kh = g.Kh; a.Kw = g.Kw;
    a.Kd = g.Kd; a.D = g.D; a.Do = g.Do; a.pad_d = g.pad_d;
    a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo; a.stride = g.stride; a.pad = g.pad;
    a.TY = pl.TY; a.TX = pl.TX;
    a.kt_total = pl.kt_total; a.kt_per_split = pl.kt_per; a.splits = pl.splits;
    a.accumulate = accumulate;
    a.co_tiles = pl.co_tiles; a.ci_tiles = pl.ci_tiles; a.tap_groups = pl.groups;
    const dim3 grid((unsigned)(pl.co_tiles * pl.ci_tiles * pl.groups), 1, pl.splits);
    hipError_t e = hipSuccess;
#define LPM_TR_LAUNCH(TAPS, NST)                                                                              \
    {                                                                                                         \
        const int bytes = NST * TrCfg<TAPS>::STAGE + 256;                                                     \
        static const hipError_t attr = hipFuncSetAttribute((const void*)wgrad_tr_kernel<TAPS, NST>,           \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, bytes); \
        if (attr != hipSuccess) return attr;                                                                  \
        hipLaunchKernelGGL((wgrad_tr_kernel<TAPS, NST>), grid, dim3(256), bytes, st, a);                      \
    }
    if (pl.taps == 3) LPM_TR_LAUNCH(3, 4)
    else LPM_TR_LAUNCH(1, 4)
#undef LPM_TR_LAUNCH
    e = hipGetLastError();
    if (e != hipSuccess || pl.splits == 1) return e;
    const int64_t n = (int64_t)g.Cout * g.K();
    const int nb = dbias ? g.Cout : 0;
    const ReduceDesc d{(const float*)ws, a.part_stride, pl.splits, dw, n, dbias, nb, rscale, g.K(), accumulate};
    if (deferred) { *deferred = d; return hipSuccess; }
    return launch_reduce_batch(&d, 1, st);
}

}  // namespace lpm
