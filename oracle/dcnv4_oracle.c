/*
 * DCNv4 spatial aggregation -- CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision loop nest that writes out the operator's
 * definition (paper Sec. 3.1, Eq. 1-2, with the softmax over the K taps removed
 * as Sec. 3.1 "Enhancing dynamic property" prescribes).  Nothing here is blocked,
 * fused or reordered; a reader can check each line against the equation.  The
 * GPU library shares no code, header or table with this file, and nothing in the
 * product path may call it: only the tests, the smoke check and the benchmark's
 * CPU-baseline leg do.
 *
 * Tensors are dense, row-major, double:
 *   x      [N, H,  W,  G*Cg]      channel-last input (Sec. 3.2, footnote)
 *   offset [N, Ho, Wo, G, K, 2]   last axis: [0] = displacement along the width,
 *                                 [1] = displacement along the height
 *   mask   [N, Ho, Wo, G, K]      unnormalised aggregation weights m_gk
 *   y      [N, Ho, Wo, G*Cg]      group outputs concatenated on channels (Eq. 2)
 * K = kernel_h * kernel_w taps; tap k = j*kernel_h + i samples the window cell
 * with width index j (slow) and height index i (fast) -- the order in which the
 * grid {(-1,-1), (-1,0), ..., (+1,+1)} of Sec. 3.1 is listed when each tuple is
 * read as (width, height).
 *
 * Readings where the paper is silent (all stated in the design notes):
 *   - sampling position: height = oh*stride_h - pad_h + i*dil_h + offset_scale*dY,
 *     width likewise; with pad 1, dilation 1 this is p0 + p_k + dp_gk of Eq. 1;
 *   - integer coordinates are pixel centres, the four neighbours are floor and
 *     floor+1, and a neighbour outside the image contributes zero (per corner);
 *   - at an integer coordinate the derivative is the right-hand one (floor rule).
 * The backward pass is the chain rule applied to those formulas (the paper gives
 * no backward); gradients are accumulated in double, in plain loop order.
 */
#include <math.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int dcnv4_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int dcnv4_oracle_output_hw(int H, int W, int kh, int kw, int sh, int sw, int ph, int pw,
                           int dh, int dw, int *Ho, int *Wo)
{
    if (H < 1 || W < 1 || kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw < 1)
        return 1;
    long eh = (long)H + 2L * ph - (long)dh * (kh - 1) - 1;
    long ew = (long)W + 2L * pw - (long)dw * (kw - 1) - 1;
    if (eh < 0 || ew < 0)
        return 1;
    *Ho = (int)(eh / sh + 1);
    *Wo = (int)(ew / sw + 1);
    return 0;
}

/* x_g at integer pixel (r, q), channel ch of image n; zero outside the image. */
static double pixel(const double *x, int H, int W, int C, int n, double r, double q, int ch)
{
    if (!(r >= 0.0 && r <= (double)(H - 1) && q >= 0.0 && q <= (double)(W - 1)))
        return 0.0;
    return x[(((size_t)n * H + (size_t)r) * W + (size_t)q) * C + ch];
}

static int inside(int H, int W, double r, double q)
{
    return r >= 0.0 && r <= (double)(H - 1) && q >= 0.0 && q <= (double)(W - 1);
}

/* Forward: Eq. 1 per group, Eq. 2 by channel indexing. */
int dcnv4_oracle_forward(const double *x, const double *offset, const double *mask, double *y,
                         int N, int H, int W, int G, int Cg,
                         int kh, int kw, int sh, int sw, int ph, int pw, int dh, int dw,
                         double offset_scale)
{
    int Ho, Wo;
    if (dcnv4_oracle_output_hw(H, W, kh, kw, sh, sw, ph, pw, dh, dw, &Ho, &Wo))
        return 1;
    const int K = kh * kw, C = G * Cg;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < Ho; ++oh)
            for (int ow = 0; ow < Wo; ++ow)
                for (int g = 0; g < G; ++g) {
                    const size_t pg = (((size_t)n * Ho + oh) * Wo + ow) * G + g;
                    for (int c = 0; c < Cg; ++c) {
                        const int ch = g * Cg + c;
                        double acc = 0.0;
                        for (int j = 0; j < kw; ++j)
                            for (int i = 0; i < kh; ++i) {
                                const int k = j * kh + i;
                                const double dX = offset[(pg * K + k) * 2 + 0];
                                const double dY = offset[(pg * K + k) * 2 + 1];
                                const double hy = (double)(oh * sh - ph + i * dh) + offset_scale * dY;
                                const double wx = (double)(ow * sw - pw + j * dw) + offset_scale * dX;
                                const double h0 = floor(hy), w0 = floor(wx);
                                const double lh = hy - h0, lw = wx - w0;
                                const double S =
                                    (1.0 - lh) * (1.0 - lw) * pixel(x, H, W, C, n, h0, w0, ch) +
                                    (1.0 - lh) * lw * pixel(x, H, W, C, n, h0, w0 + 1.0, ch) +
                                    lh * (1.0 - lw) * pixel(x, H, W, C, n, h0 + 1.0, w0, ch) +
                                    lh * lw * pixel(x, H, W, C, n, h0 + 1.0, w0 + 1.0, ch);
                                acc += mask[pg * K + k] * S;
                            }
                        y[(pg / G) * C + ch] = acc;
                    }
                }
    return 0;
}

/*
 * Backward: with S_k[c] the bilinear sample of tap k and channel c,
 *   y[c]           = sum_k m_k * S_k[c]
 *   grad_mask_k    = sum_c gy[c] * S_k[c]
 *   grad_dY_k      = offset_scale * m_k * sum_c gy[c] * dS_k[c]/dhy
 *   grad_dX_k      = offset_scale * m_k * sum_c gy[c] * dS_k[c]/dwx
 *   grad_x[corner] += m_k * (corner weight) * gy[c]      (corners inside the image)
 * where dS/dhy = (1-lw)(X10-X00) + lw(X11-X01), dS/dwx = (1-lh)(X01-X00) + lh(X11-X10),
 * Xab the neighbour at (h0+a, w0+b), zero outside the image.
 * All three outputs are overwritten.
 */
int dcnv4_oracle_backward(const double *x, const double *offset, const double *mask,
                          const double *grad_y, double *grad_x, double *grad_offset,
                          double *grad_mask,
                          int N, int H, int W, int G, int Cg,
                          int kh, int kw, int sh, int sw, int ph, int pw, int dh, int dw,
                          double offset_scale)
{
    int Ho, Wo;
    if (dcnv4_oracle_output_hw(H, W, kh, kw, sh, sw, ph, pw, dh, dw, &Ho, &Wo))
        return 1;
    const int K = kh * kw, C = G * Cg;
    const size_t nx = (size_t)N * H * W * C;
    for (size_t t = 0; t < nx; ++t)
        grad_x[t] = 0.0;
    /* images are independent, so each thread scatters into its own image only */
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < Ho; ++oh)
            for (int ow = 0; ow < Wo; ++ow)
                for (int g = 0; g < G; ++g) {
                    const size_t pg = (((size_t)n * Ho + oh) * Wo + ow) * G + g;
                    for (int j = 0; j < kw; ++j)
                        for (int i = 0; i < kh; ++i) {
                            const int k = j * kh + i;
                            const double dX = offset[(pg * K + k) * 2 + 0];
                            const double dY = offset[(pg * K + k) * 2 + 1];
                            const double m = mask[pg * K + k];
                            const double hy = (double)(oh * sh - ph + i * dh) + offset_scale * dY;
                            const double wx = (double)(ow * sw - pw + j * dw) + offset_scale * dX;
                            const double h0 = floor(hy), w0 = floor(wx);
                            const double lh = hy - h0, lw = wx - w0;
                            double gm = 0.0, gdy = 0.0, gdx = 0.0;
                            for (int c = 0; c < Cg; ++c) {
                                const int ch = g * Cg + c;
                                const double gy = grad_y[(pg / G) * C + ch];
                                const double X00 = pixel(x, H, W, C, n, h0, w0, ch);
                                const double X01 = pixel(x, H, W, C, n, h0, w0 + 1.0, ch);
                                const double X10 = pixel(x, H, W, C, n, h0 + 1.0, w0, ch);
                                const double X11 = pixel(x, H, W, C, n, h0 + 1.0, w0 + 1.0, ch);
                                const double S = (1.0 - lh) * (1.0 - lw) * X00 + (1.0 - lh) * lw * X01 +
                                                 lh * (1.0 - lw) * X10 + lh * lw * X11;
                                const double dS_dh = (1.0 - lw) * (X10 - X00) + lw * (X11 - X01);
                                const double dS_dw = (1.0 - lh) * (X01 - X00) + lh * (X11 - X10);
                                gm += gy * S;
                                gdy += gy * dS_dh;
                                gdx += gy * dS_dw;
                                for (int a = 0; a < 2; ++a)
                                    for (int b = 0; b < 2; ++b) {
                                        const double r = h0 + a, q = w0 + b;
                                        if (!inside(H, W, r, q))
                                            continue;
                                        const double wt = (a ? lh : 1.0 - lh) * (b ? lw : 1.0 - lw);
                                        grad_x[(((size_t)n * H + (size_t)r) * W + (size_t)q) * C + ch] +=
                                            m * wt * gy;
                                    }
                            }
                            grad_mask[pg * K + k] = gm;
                            grad_offset[(pg * K + k) * 2 + 0] = offset_scale * m * gdx;
                            grad_offset[(pg * K + k) * 2 + 1] = offset_scale * m * gdy;
                        }
                }
    return 0;
}
