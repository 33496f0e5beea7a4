/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, direct convolutions in double precision.  Nothing in the
 * product path may call this file; only tests, the smoke check and the
 * benchmark's cpu_baseline leg do.  It shares no code with the HIP library.
 *
 * What it computes.  The method (Section 3.1) replaces a layer's weights W by
 * W~ = W (.) M with a block-constant 0/1 mask M, and the sparse kernels
 * (Algorithm 1) only skip the blocks that are zero.  The exact result is
 * therefore the ordinary dense convolution evaluated on the masked weights.
 * This file is that definition written out: the caller passes weights that
 * are ALREADY masked; every weight, zero or not, is multiplied and added.
 *
 * Layouts follow Section 3.1 / Algorithm 1:
 *   activations  [n][ih][iw][ic]     (NHWC)
 *   weights      [oc][kh][kw][ic]    (OHWI)
 *   bias         [oc]
 * Accumulation is fp64 in (ky, kx, c) order, rounded once to fp32.
 * Out-of-range input positions (zero padding) contribute exactly nothing.
 * `bound` receives sum |x|*|w| per output element (fp64), the scale of the
 * acceptance test  |y_gpu - y| <= 1e-4 * bound.
 *
 * No blocking, no vector intrinsics, no zero skipping: one loop nest per
 * definition.  OpenMP splits the independent output pixels over threads.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_ACT_NONE 0
#define ORACLE_ACT_RELU 1

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static float finish(double acc, int act)
{
    float r = (float)acc;
    if (act == ORACLE_ACT_RELU && !(r > 0.0f)) r = 0.0f;
    return r;
}

/*
 * Dense direct convolution, y = act(bias + x (*) w).
 * oh = (ih + 2*pad - kh)/stride + 1, likewise ow.  y is [n][oh][ow][oc];
 * bound may be NULL.  Returns 0, or -1 on a bad argument.
 */
int oracle_conv_nhwc(const float *x, int n, int ih, int iw, int ic,
                     const float *w, int oc, int kh, int kw,
                     const float *bias, int stride, int pad, int act,
                     float *y, double *bound)
{
    if (!x || !w || !y || n < 0 || ih <= 0 || iw <= 0 || ic <= 0 || oc <= 0 ||
        kh <= 0 || kw <= 0 || stride <= 0 || pad < 0)
        return -1;
    const int oh = (ih + 2 * pad - kh) / stride + 1;
    const int ow = (iw + 2 * pad - kw) / stride + 1;
    if (oh <= 0 || ow <= 0) return -1;
    const long npix = (long)n * oh * ow;

#pragma omp parallel for schedule(static)
    for (long p = 0; p < npix; ++p) {
        const int ox = (int)(p % ow);
        const int oy = (int)((p / ow) % oh);
        const int b = (int)(p / ((long)ow * oh));
        for (int o = 0; o < oc; ++o) {
            double acc = bias ? (double)bias[o] : 0.0;
            double bnd = 0.0;
            for (int ky = 0; ky < kh; ++ky) {
                const int iy = oy * stride + ky - pad;
                if (iy < 0 || iy >= ih) continue;
                for (int kx = 0; kx < kw; ++kx) {
                    const int ix = ox * stride + kx - pad;
                    if (ix < 0 || ix >= iw) continue;
                    const float *xp = x + (((size_t)b * ih + iy) * iw + ix) * ic;
                    const float *wp = w + (((size_t)o * kh + ky) * kw + kx) * ic;
                    for (int c = 0; c < ic; ++c) {
                        acc += (double)xp[c] * (double)wp[c];
                        bnd += fabs((double)xp[c]) * fabs((double)wp[c]);
                    }
                }
            }
            y[(size_t)p * oc + o] = finish(acc, act);
            if (bound) bound[(size_t)p * oc + o] = bnd;
        }
    }
    return 0;
}

/*
 * Dense depthwise 3x3 convolution (one 3x3 kernel per channel), pad 1:
 * x [n][ih][iw][c], w [c][3][3], y [n][oh][ow][c], oh = (ih-1)/stride + 1.
 * Used only between pointwise layers when a whole network is chained.
 */
int oracle_dwconv3x3_nhwc(const float *x, int n, int ih, int iw, int c,
                          const float *w, const float *bias, int stride, int act,
                          float *y, double *bound)
{
    if (!x || !w || !y || n < 0 || ih <= 0 || iw <= 0 || c <= 0 || stride <= 0)
        return -1;
    const int oh = (ih + 2 - 3) / stride + 1;
    const int ow = (iw + 2 - 3) / stride + 1;
    const long npix = (long)n * oh * ow;

#pragma omp parallel for schedule(static)
    for (long p = 0; p < npix; ++p) {
        const int ox = (int)(p % ow);
        const int oy = (int)((p / ow) % oh);
        const int b = (int)(p / ((long)ow * oh));
        for (int ch = 0; ch < c; ++ch) {
            double acc = bias ? (double)bias[ch] : 0.0;
            double bnd = 0.0;
            for (int ky = 0; ky < 3; ++ky) {
                const int iy = oy * stride + ky - 1;
                if (iy < 0 || iy >= ih) continue;
                for (int kx = 0; kx < 3; ++kx) {
                    const int ix = ox * stride + kx - 1;
                    if (ix < 0 || ix >= iw) continue;
                    const double xv = x[(((size_t)b * ih + iy) * iw + ix) * c + ch];
                    const double wv = w[((size_t)ch * 3 + ky) * 3 + kx];
                    acc += xv * wv;
                    bnd += fabs(xv) * fabs(wv);
                }
            }
            y[(size_t)p * c + ch] = finish(acc, act);
            if (bound) bound[(size_t)p * c + ch] = bnd;
        }
    }
    return 0;
}

/*
 * Global average pool over the spatial positions: x [n][h][w][c] -> y [n][c],
 * fp64 sum in (h, w) order divided by h*w, rounded once.
 */
int oracle_avgpool_nhwc(const float *x, int n, int h, int w, int c, float *y)
{
    if (!x || !y || n < 0 || h <= 0 || w <= 0 || c <= 0) return -1;
    for (int b = 0; b < n; ++b)
        for (int ch = 0; ch < c; ++ch) {
            double acc = 0.0;
            for (int p = 0; p < h * w; ++p)
                acc += (double)x[((size_t)b * h * w + p) * c + ch];
            y[(size_t)b * c + ch] = (float)(acc / (double)(h * w));
        }
    return 0;
}
