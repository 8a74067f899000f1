/*
 * CPU oracle for multi-channel multi-kernel (MCMK) 2-D convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code with the GPU library and
 * must never be called from the product path: only the tests, the smoke check
 * and the benchmark's cpu_baseline leg use it.
 *
 * What it computes is the definition itself, because the kn2row method is an
 * exact re-association of the same products (section III-A): for every output
 * element the single-channel sum of Eq. 1, summed over the C channels (Eq. 2),
 * for each of the M kernels (Eq. 3), with one more outer loop over the images
 * of a batch.  Accumulation is in double precision; every float*float product
 * is exact in double, so the oracle's own error is far below any tolerance the
 * tests use.
 *
 * Readings of the paper taken here:
 *   - no kernel flip (Eq. 1 indexes I(x - floor(k/2) + i) * K(i): correlation);
 *   - the first spatial index is the row (Eq. 1: x in [0, output height));
 *   - "properly padded" (section II-A) means zero padding by `pad` on every
 *     side; contributions from outside the image are dropped, which is the
 *     same thing as the out-of-bounds discard of section III-A;
 *   - layouts: I[N][C][H][W], K[M][C][k][k] (row tap, then column tap),
 *     O[N][M][Q][P], Q = H + 2 pad - k + 1 rows, P = W + 2 pad - k + 1 columns;
 *   - strides: the paper leaves them out (section II-A treats unit stride only).
 *     The generalisation taken here is the usual one: output (q, p) of a
 *     stride-s convolution is output (s q, s p) of the unit-stride one, for
 *     Q = floor((H + 2 pad - k) / s) + 1 rows and likewise P columns.
 *
 * Pinned by tests/test_oracle_pins.py (hand-worked examples, delta kernels,
 * linearity, constant-input closed form, im2col and kn2row reformulations,
 * the k = 1 matrix product, and a library convolution in float64).
 */
#include "conv_oracle.h"

#include <math.h>
#include <stddef.h>

static int bad_shape(int n, int c, int h, int w, int m, int k, int pad, int stride)
{
    if (n < 1 || c < 1 || h < 1 || w < 1 || m < 1 || k < 1 || pad < 0 || stride < 1) return 1;
    if (h + 2 * pad - k + 1 < 1 || w + 2 * pad - k + 1 < 1) return 1;
    return 0;
}

static int out_size(int in, int k, int pad, int stride) { return (in + 2 * pad - k) / stride + 1; }

/* One output element: Eq. 1 inside Eq. 2.  Also returns sum |K||I| over the same terms. */
static void one_output(int c, int h, int w, int k, int pad, int stride,
                       const float *img /* [C][H][W] */, const float *ker /* [C][k][k] */,
                       int q, int p, double *value, double *absvalue)
{
    double acc = 0.0, aacc = 0.0;
    for (int ch = 0; ch < c; ++ch)
        for (int i = 0; i < k; ++i)
            for (int j = 0; j < k; ++j) {
                int y = q * stride - pad + i;
                int x = p * stride - pad + j;
                if (y < 0 || y >= h || x < 0 || x >= w) continue;
                double a = (double)img[((size_t)ch * h + y) * w + x];
                double b = (double)ker[((size_t)ch * k + i) * k + j];
                acc += a * b;
                aacc += fabs(a) * fabs(b);
            }
    *value = acc;
    *absvalue = aacc;
}

/* Whole output (Eq. 3 plus the loop over the images of a batch); see conv_oracle.h. */
int conv_mcmk_oracle_f64(const conv_oracle_desc *d, const float *I, const float *K, double *O, double *absO)
{
    if (!d) return 1;
    const int n = d->n, c = d->c, h = d->h, w = d->w, m = d->m, k = d->k, pad = d->pad, stride = d->stride;
    if (bad_shape(n, c, h, w, m, k, pad, stride) || !I || !K || !O) return 1;
    const int Q = out_size(h, k, pad, stride), P = out_size(w, k, pad, stride);
#pragma omp parallel for collapse(2) schedule(static)
    for (int in = 0; in < n; ++in)
        for (int im = 0; im < m; ++im)
            for (int q = 0; q < Q; ++q)
                for (int p = 0; p < P; ++p) {
                    double v, a;
                    one_output(c, h, w, k, pad, stride, I + (size_t)in * c * h * w,
                               K + (size_t)im * c * k * k, q, p, &v, &a);
                    size_t o = (((size_t)in * m + im) * Q + q) * P + p;
                    O[o] = v;
                    if (absO) absO[o] = a;
                }
    return 0;
}

/* Selected outputs only; see conv_oracle.h. */
int conv_mcmk_oracle_f64_at(const conv_oracle_desc *d, const float *I, const float *K,
                            int npts, const int *pts, double *O, double *absO)
{
    if (!d) return 1;
    const int n = d->n, c = d->c, h = d->h, w = d->w, m = d->m, k = d->k, pad = d->pad, stride = d->stride;
    if (bad_shape(n, c, h, w, m, k, pad, stride) || !I || !K || !O || !pts || npts < 0) return 1;
    const int Q = out_size(h, k, pad, stride), P = out_size(w, k, pad, stride);
    for (int t = 0; t < npts; ++t) {
        const int *pt = pts + 4 * t;
        if (pt[0] < 0 || pt[0] >= n || pt[1] < 0 || pt[1] >= m ||
            pt[2] < 0 || pt[2] >= Q || pt[3] < 0 || pt[3] >= P) return 2;
    }
#pragma omp parallel for schedule(dynamic, 16)
    for (int t = 0; t < npts; ++t) {
        const int *pt = pts + 4 * t;
        double v, a;
        one_output(c, h, w, k, pad, stride, I + (size_t)pt[0] * c * h * w,
                   K + (size_t)pt[1] * c * k * k, pt[2], pt[3], &v, &a);
        O[t] = v;
        if (absO) absO[t] = a;
    }
    return 0;
}
