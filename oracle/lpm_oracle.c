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

/* ---- three-dimensional convolution (the 3x3x3 layers of the volumetric use case) ------------------------------
 * Same definition with one more spatial index: activations [N][C][D][H][W], weights [Cout][Cin][Kd][Kh][Kw],
 * one stride for all three axes, padding pd along the depth and p along height and width.
 *   z[n,co,do,ho,wo] = sum_{ci,kd,kh,kw} Wt[co,ci,kd,kh,kw] * x[n,ci,do*s+kd-pd,ho*s+kh-p,wo*s+kw-p], zero outside. */
#define IDX5(n, c, d, h, w, C, D, H, W) (((((size_t)(n) * (C) + (c)) * (D) + (d)) * (H) + (h)) * (W) + (w))

void orc_conv3d_fwd(const double *x, const double *wt, double *z, int N, int Cin, int D, int H, int W,
                    int Cout, int Kd, int Kh, int Kw, int stride, int pad_d, int pad)
{
    const int Do = (D + 2 * pad_d - Kd) / stride + 1, Ho = (H + 2 * pad - Kh) / stride + 1, Wo = (W + 2 * pad - Kw) / stride + 1;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Cout; ++co)
            for (int dq = 0; dq < Do; ++dq)
                for (int ho = 0; ho < Ho; ++ho)
                    for (int wo = 0; wo < Wo; ++wo) {
                        double acc = 0.0;
                        for (int ci = 0; ci < Cin; ++ci)
                            for (int kd = 0; kd < Kd; ++kd) {
                                const int d = dq * stride + kd - pad_d;
                                if (d < 0 || d >= D) continue;
                                for (int kh = 0; kh < Kh; ++kh) {
                                    const int h = ho * stride + kh - pad;
                                    if (h < 0 || h >= H) continue;
                                    for (int kw = 0; kw < Kw; ++kw) {
                                        const int w = wo * stride + kw - pad;
                                        if (w < 0 || w >= W) continue;
                                        acc += wt[IDX5(co, ci, kd, kh, kw, Cin, Kd, Kh, Kw)] * x[IDX5(n, ci, d, h, w, Cin, D, H, W)];
                                    }
                                }
                            }
                        z[IDX5(n, co, dq, ho, wo, Cout, Do, Ho, Wo)] = acc;
                    }
}

/* dx[n,ci,d,h,w] = sum over (co,kd,kh,kw) and the output positions (do,ho,wo) that read (d,h,w) through that tap. */
void orc_conv3d_bwd_data(const double *dz, const double *wt, double *dx, int N, int Cin, int D, int H, int W,
                         int Cout, int Kd, int Kh, int Kw, int stride, int pad_d, int pad)
{
    const int Do = (D + 2 * pad_d - Kd) / stride + 1, Ho = (H + 2 * pad - Kh) / stride + 1, Wo = (W + 2 * pad - Kw) / stride + 1;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int n = 0; n < N; ++n)
        for (int ci = 0; ci < Cin; ++ci)
            for (int d = 0; d < D; ++d)
                for (int h = 0; h < H; ++h)
                    for (int w = 0; w < W; ++w) {
                        double acc = 0.0;
                        for (int co = 0; co < Cout; ++co)
                            for (int kd = 0; kd < Kd; ++kd) {
                                const int td = d + pad_d - kd;
                                if (td < 0 || td % stride || td / stride >= Do) continue;
                                for (int kh = 0; kh < Kh; ++kh) {
                                    const int th = h + pad - kh;
                                    if (th < 0 || th % stride || th / stride >= Ho) continue;
                                    for (int kw = 0; kw < Kw; ++kw) {
                                        const int tw = w + pad - kw;
                                        if (tw < 0 || tw % stride || tw / stride >= Wo) continue;
                                        acc += wt[IDX5(co, ci, kd, kh, kw, Cin, Kd, Kh, Kw)] *
                                               dz[IDX5(n, co, td / stride, th / stride, tw / stride, Cout, Do, Ho, Wo)];
                                    }
                                }
                            }
                        dx[IDX5(n, ci, d, h, w, Cin, D, H, W)] = acc;
                    }
}

/* dW[co,ci,kd,kh,kw] = sum_{n,do,ho,wo} dz[n,co,do,ho,wo] * x[n,ci,do*s+kd-pd,ho*s+kh-p,wo*s+kw-p]. */
void orc_conv3d_bwd_weight(const double *x, const double *dz, double *dwt, int N, int Cin, int D, int H, int W,
                           int Cout, int Kd, int Kh, int Kw, int stride, int pad_d, int pad)
{
    const int Do = (D + 2 * pad_d - Kd) / stride + 1, Ho = (H + 2 * pad - Kh) / stride + 1, Wo = (W + 2 * pad - Kw) / stride + 1;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int co = 0; co < Cout; ++co)
        for (int ci = 0; ci < Cin; ++ci)
            for (int kd = 0; kd < Kd; ++kd)
                for (int kh = 0; kh < Kh; ++kh)
                    for (int kw = 0; kw < Kw; ++kw) {
                        double acc = 0.0;
                        for (int n = 0; n < N; ++n)
                            for (int dq = 0; dq < Do; ++dq) {
                                const int d = dq * stride + kd - pad_d;
                                if (d < 0 || d >= D) continue;
                                for (int ho = 0; ho < Ho; ++ho) {
                                    const int h = ho * stride + kh - pad;
                                    if (h < 0 || h >= H) continue;
                                    for (int wo = 0; wo < Wo; ++wo) {
                                        const int w = wo * stride + kw - pad;
                                        if (w < 0 || w >= W) continue;
                                        acc += dz[IDX5(n, co, dq, ho, wo, Cout, Do, Ho, Wo)] * x[IDX5(n, ci, d, h, w, Cin, D, H, W)];
                                    }
                                }
                            }
                        dwt[IDX5(co, ci, kd, kh, kw, Cin, Kd, Kh, Kw)] = acc;
                    }
}
