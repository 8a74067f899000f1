/*
 * conv_oracle.h -- C boundary of the CPU oracle (libconv_oracle.so).
 *
 * TEST INFRASTRUCTURE ONLY: the plain double-precision evaluation of the
 * defining sum of multi-channel multi-kernel convolution (paper Eq. 1-3) that
 * the GPU library is checked against.  Host pointers only; no GPU header is
 * included and nothing here is shared with the GPU library.  Only tests, the
 * smoke check and the benchmark's cpu_baseline leg call it.
 *
 * Layouts: I[N][C][H][W] and K[M][C][k][k] (row tap, then column tap) in float,
 * O[N][M][Q][P] in double, all dense and row-major,
 * Q = floor((H + 2 pad - k) / stride) + 1, P likewise from W.
 */
#ifndef CONV_ORACLE_H
#define CONV_ORACLE_H

#ifdef __cplusplus
extern "C" {
#endif

/* One convolution problem; every field as in the paper's notation (section II-A), plus the batch size and
 * the stride, which the paper leaves at 1. */
typedef struct conv_oracle_desc {
    int n;      /* images, >= 1 */
    int c;      /* channels, >= 1 */
    int h, w;   /* input rows, columns, >= 1 */
    int m;      /* kernels, >= 1 */
    int k;      /* kernel side, >= 1 */
    int pad;    /* zero padding on every side, >= 0 */
    int stride; /* >= 1 */
} conv_oracle_desc;

/*
 * Whole output: O[n][m][q][p] = sum over c, i, j of I[n][c][stride q - pad + i][stride p - pad + j] * K[m][c][i][j],
 * terms outside the image dropped, accumulated in double.  absO (may be NULL) receives the sum of
 * |I| * |K| over the same terms, the norm the parity bounds are stated in.  The caller owns all buffers.
 * Returns 0, or 1 for a NULL pointer or a shape that is no valid convolution (nothing is written then).
 */
int conv_mcmk_oracle_f64(const conv_oracle_desc *desc, const float *I, const float *K, double *O, double *absO);

/*
 * Selected outputs: pts holds npts quadruples (n, m, q, p); O and absO (may be NULL) get npts doubles.
 * Returns 0, 1 as above, 2 when a point lies outside the output.
 */
int conv_mcmk_oracle_f64_at(const conv_oracle_desc *desc, const float *I, const float *K,
                            int npts, const int *pts, double *O, double *absO);

#ifdef __cplusplus
}
#endif
#endif /* CONV_ORACLE_H */
