/*
 * CPU ORACLE -- test infrastructure only, never part of the product path.
 *
 * Direct-summation 2-D convolution over a batch of frames, in double
 * precision, written out from the textbook definition.  The paper builds its
 * video network from "pure 2D CNN" layers applied to each of the N*T frames
 * (section 2, "Temporal modeling unit"); this file is that per-frame 2-D
 * cross-correlation and its two adjoints.  The temporal shift is NOT here: the
 * Python side materialises the shifted tensor explicitly and then calls these.
 *
 * Layout of every tensor: dense row-major,
 *   x  [F][Cin][H][W]      dy, y [F][Cout][Ho][Wo]      w [Cout][Cin][KH][KW]
 * with Ho = (H + 2*pad - KH)/stride + 1 (floor), likewise Wo.
 *
 * No blocking, no im2col, no library calls.  OpenMP only distributes whole
 * output planes over threads; each output element is still one plain sum.
 */
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* y[f,co,oh,ow] = sum_{ci,kh,kw} w[co,ci,kh,kw] * x[f,ci,oh*s+kh-p,ow*s+kw-p],
 * taps that fall outside the frame contribute zero. */
void oracle_conv2d_fwd(const double* x, const double* w, double* y,
                       int F, int Cin, int H, int W, int Cout, int KH, int KW,
                       int stride, int pad) {
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
    const long planes = (long)F * Cout;
#pragma omp parallel for schedule(static)
    for (long fc = 0; fc < planes; ++fc) {
        const int f = (int)(fc / Cout), co = (int)(fc % Cout);
        double* yp = y + (size_t)fc * Ho * Wo;
        memset(yp, 0, sizeof(double) * (size_t)Ho * Wo);
        for (int ci = 0; ci < Cin; ++ci) {
            const double* xp = x + ((size_t)f * Cin + ci) * H * W;
            for (int kh = 0; kh < KH; ++kh)
                for (int kw = 0; kw < KW; ++kw) {
                    const double wv = w[(((size_t)co * Cin + ci) * KH + kh) * KW + kw];
                    for (int oh = 0; oh < Ho; ++oh) {
                        const int ih = oh * stride + kh - pad;
                        if (ih < 0 || ih >= H) continue;
                        for (int ow = 0; ow < Wo; ++ow) {
                            const int iw = ow * stride + kw - pad;
                            if (iw < 0 || iw >= W) continue;
                            yp[oh * Wo + ow] += wv * xp[ih * W + iw];
                        }
                    }
                }
        }
    }
}

/* dx[f,ci,ih,iw] = sum over (co,kh,kw,oh,ow) with oh*s+kh-p == ih and
 * ow*s+kw-p == iw of w[co,ci,kh,kw] * dy[f,co,oh,ow]. */
void oracle_conv2d_dgrad(const double* dy, const double* w, double* dx,
                         int F, int Cin, int H, int W, int Cout, int KH, int KW,
                         int stride, int pad) {
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
    const long planes = (long)F * Cin;
#pragma omp parallel for schedule(static)
    for (long fc = 0; fc < planes; ++fc) {
        const int f = (int)(fc / Cin), ci = (int)(fc % Cin);
        double* dxp = dx + (size_t)fc * H * W;
        memset(dxp, 0, sizeof(double) * (size_t)H * W);
        for (int co = 0; co < Cout; ++co) {
            const double* dyp = dy + ((size_t)f * Cout + co) * Ho * Wo;
            for (int kh = 0; kh < KH; ++kh)
                for (int kw = 0; kw < KW; ++kw) {
                    const double wv = w[(((size_t)co * Cin + ci) * KH + kh) * KW + kw];
                    for (int oh = 0; oh < Ho; ++oh) {
                        const int ih = oh * stride + kh - pad;
                        if (ih < 0 || ih >= H) continue;
                        for (int ow = 0; ow < Wo; ++ow) {
                            const int iw = ow * stride + kw - pad;
                            if (iw < 0 || iw >= W) continue;
                            dxp[ih * W + iw] += wv * dyp[oh * Wo + ow];
                        }
                    }
                }
        }
    }
}

/* dw[co,ci,kh,kw] = sum_{f,oh,ow} dy[f,co,oh,ow] * x[f,ci,oh*s+kh-p,ow*s+kw-p]. */
void oracle_conv2d_wgrad(const double* x, const double* dy, double* dw,
                         int F, int Cin, int H, int W, int Cout, int KH, int KW,
                         int stride, int pad) {
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
    const long pairs = (long)Cout * Cin;
#pragma omp parallel for schedule(static)
    for (long cc = 0; cc < pairs; ++cc) {
        const int co = (int)(cc / Cin), ci = (int)(cc % Cin);
        for (int kh = 0; kh < KH; ++kh)
            for (int kw = 0; kw < KW; ++kw) {
                double acc = 0.0;
                for (int f = 0; f < F; ++f) {
                    const double* xp = x + ((size_t)f * Cin + ci) * H * W;
                    const double* dyp = dy + ((size_t)f * Cout + co) * Ho * Wo;
                    for (int oh = 0; oh < Ho; ++oh) {
                        const int ih = oh * stride + kh - pad;
                        if (ih < 0 || ih >= H) continue;
                        for (int ow = 0; ow < Wo; ++ow) {
                            const int iw = ow * stride + kw - pad;
                            if (iw < 0 || iw >= W) continue;
                            acc += dyp[oh * Wo + ow] * xp[ih * W + iw];
                        }
                    }
                }
                dw[(((size_t)co * Cin + ci) * KH + kh) * KW + kw] = acc;
            }
    }
}
