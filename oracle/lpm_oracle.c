/*
 * fp64 CPU oracle for the layer arithmetic of a partition's training step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct checker the
 * GPU library is compared against; nothing on the product path may call it.
 * It shares no code with the HIP sources.
 *
 * Every routine is the textbook definition written as direct loops in double
 * precision.  Tensors are dense, row-major, in the logical layout
 *   activations  [N][C][H][W]
 *   conv weights [Cout][Cin][Kh][Kw]
 * A fully connected layer is the special case Kh=H, Kw=W, pad 0 (one output
 * pixel), so it needs no routine of its own.
 *
 * Paper passages followed:
 *   layer evaluation a^{l+1} = g_l(a^l, p^l)          -- Problem Statement, eq. (1)
 *   chain rule for parameter / activation gradients   -- Problem Statement, eqs. (8), (9)
 * The paper fixes no layer formulas beyond naming convolution, pooling, ReLU and
 * fully connected layers (Use-case 2 description), so the definitions here are the
 * standard ones: cross-correlation (no kernel flip) with zero padding, 2x2/2 max
 * pooling whose gradient goes to the first maximum in row-major window order.
 *
 * Parallelism: OpenMP over (image x channel) only; each output element is still
 * one sequential fp64 sum.
 */
#include <stddef.h>
#include <stdint.h>

#define IDX4(n, c, h, w, C, H, W) ((((size_t)(n) * (C) + (c)) * (H) + (h)) * (W) + (w))

/* z[n,co,ho,wo] = sum_{ci,kh,kw} Wt[co,ci,kh,kw] * x[n,ci,ho*s+kh-p,wo*s+kw-p], zero outside. */
void orc_conv_fwd(const double *x, const double *wt, double *z, int N, int Cin, int H, int W,
                  int Cout, int Kh, int Kw, int stride, int pad)
{
    const int Ho = (H + 2 * pad - Kh) / stride + 1, Wo = (W + 2 * pad - Kw) / stride + 1;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Cout; ++co) {
            double *zp = z + IDX4(n, co, 0, 0, Cout, Ho, Wo);
            for (int i = 0; i < Ho * Wo; ++i) zp[i] = 0.0;
            for (int ci = 0; ci < Cin; ++ci)
                for (int kh = 0; kh < Kh; ++kh)
                    for (int kw = 0; kw < Kw; ++kw) {
                        const double wv = wt[IDX4(co, ci, kh, kw, Cin, Kh, Kw)];
                        for (int ho = 0; ho < Ho; ++ho) {
                            const int h = ho * stride + kh - pad;
                            if (h < 0 || h >= H) continue;
                            const double *xr = x + IDX4(n, ci, h, 0, Cin, H, W);
                            for (int wo = 0; wo < Wo; ++wo) {
                                const int w = wo * stride + kw - pad;
                                if (w < 0 || w >= W) continue;
                                zp[ho * Wo + wo] += wv * xr[w];
                            }
                        }
                    }
        }
}

/* dx[n,ci,h,w] = sum over (co,kh,kw,ho,wo) with h=ho*s+kh-p, w=wo*s+kw-p of dz[n,co,ho,wo]*Wt[co,ci,kh,kw]. */
void orc_conv_bwd_data(const double *dz, const double *wt, double *dx, int N, int Cin, int H, int W,
                       int Cout, int Kh, int Kw, int stride, int pad)
{
    const int Ho = (H + 2 * pad - Kh) / stride + 1, Wo = (W + 2 * pad - Kw) / stride + 1;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int n = 0; n < N; ++n)
        for (int ci = 0; ci < Cin; ++ci) {
            double *dxp = dx + IDX4(n, ci, 0, 0, Cin, H, W);
            for (int i = 0; i < H * W; ++i) dxp[i] = 0.0;
            for (int co = 0; co < Cout; ++co) {
                const double *dzp = dz + IDX4(n, co, 0, 0, Cout, Ho, Wo);
                for (int kh = 0; kh < Kh; ++kh)
                    for (int kw = 0; kw < Kw; ++kw) {
                        const double wv = wt[IDX4(co, ci, kh, kw, Cin, Kh, Kw)];
                        for (int ho = 0; ho < Ho; ++ho) {
                            const int h = ho * stride + kh - pad;
                            if (h < 0 || h >= H) continue;
                            for (int wo = 0; wo < Wo; ++wo) {
                                const int w = wo * stride + kw - pad;
                                if (w < 0 || w >= W) continue;
                                dxp[h * W + w] += wv * dzp[ho * Wo + wo];
                            }
                        }
                    }
            }
        }
}

/* dW[co,ci,kh,kw] = sum_{n,ho,wo} dz[n,co,ho,wo] * x[n,ci,ho*s+kh-p,wo*s+kw-p]. */
void orc_conv_bwd_weight(const double *x, const double *dz, double *dwt, int N, int Cin, int H, int W,
                         int Cout, int Kh, int Kw, int stride, int pad)
{
    const int Ho = (H + 2 * pad - Kh) / stride + 1, Wo = (W + 2 * pad - Kw) / stride + 1;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int co = 0; co < Cout; ++co)
        for (int ci = 0; ci < Cin; ++ci)
            for (int kh = 0; kh < Kh; ++kh)
                for (int kw = 0; kw < Kw; ++kw) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n) {
                        const double *dzp = dz + IDX4(n, co, 0, 0, Cout, Ho, Wo);
                        for (int ho = 0; ho < Ho; ++ho) {
                            const int h = ho * stride + kh - pad;
                            if (h < 0 || h >= H) continue;
                            const double *xr = x + IDX4(n, ci, h, 0, Cin, H, W);
                            for (int wo = 0; wo < Wo; ++wo) {
                                const int w = wo * stride + kw - pad;
                                if (w < 0 || w >= W) continue;
                                acc += dzp[ho * Wo + wo] * xr[w];
                            }
                        }
                    }
                    dwt[IDX4(co, ci, kh, kw, Cin, Kh, Kw)] = acc;
                }
}

/* 2x2 window, stride 2, H and W even.  y = max of the window. */
void orc_maxpool2_fwd(const double *x, double *y, int N, int C, int H, int W)
{
    const int Ho = H / 2, Wo = W / 2;
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < N * C; ++nc) {
        const double *xp = x + (size_t)nc * H * W;
        double *yp = y + (size_t)nc * Ho * Wo;
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                double m = xp[(2 * ho) * W + 2 * wo];
                for (int a = 0; a < 2; ++a)
                    for (int b = 0; b < 2; ++b) {
                        const double v = xp[(2 * ho + a) * W + 2 * wo + b];
                        if (v > m) m = v;
                    }
                yp[ho * Wo + wo] = m;
            }
    }
}

/* dx gets dy at the first maximum of each window (row-major order inside the window), 0 elsewhere. */
void orc_maxpool2_bwd(const double *x, const double *dy, double *dx, int N, int C, int H, int W)
{
    const int Ho = H / 2, Wo = W / 2;
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < N * C; ++nc) {
        const double *xp = x + (size_t)nc * H * W;
        const double *dyp = dy + (size_t)nc * Ho * Wo;
        double *dxp = dx + (size_t)nc * H * W;
        for (int i = 0; i < H * W; ++i) dxp[i] = 0.0;
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                int ba = 0, bb = 0;
                double m = xp[(2 * ho) * W + 2 * wo];
                for (int a = 0; a < 2; ++a)
                    for (int b = 0; b < 2; ++b) {
                        const double v = xp[(2 * ho + a) * W + 2 * wo + b];
                        if (v > m) { m = v; ba = a; bb = b; }   /* strict: first maximum wins */
                    }
                dxp[(2 * ho + ba) * W + 2 * wo + bb] = dyp[ho * Wo + wo];
            }
    }
}
