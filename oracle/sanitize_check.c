/*
 * Driver that runs the CPU oracle as a plain host program, so that it can be built with
 * -fsanitize=address,undefined (python -m oracle.build --sanitize) and fed the same pinned cases the
 * Python tests use.  TEST INFRASTRUCTURE ONLY.
 *
 * stdin:  any number of cases, each
 *           n c h w m k pad stride npts
 *           n*c*h*w input values, m*c*k*k kernel values, npts quadruples (n m q p)
 * stdout: per case one line "rc <code> <count>" followed by count outputs and count |.|-sums of the whole
 *         output (one per line), then "at <code> <npts>" followed by the npts selected outputs and |.|-sums.
 * Buffers are allocated to their exact sizes, so any access of the oracle outside them is reported.
 */
#include "conv_oracle.h"

#include <stdio.h>
#include <stdlib.h>

int main(void)
{
    conv_oracle_desc d;
    int npts;
    while (scanf("%d %d %d %d %d %d %d %d %d", &d.n, &d.c, &d.h, &d.w, &d.m, &d.k, &d.pad, &d.stride, &npts) == 9) {
        /* sizes from the raw fields (the oracle itself must reject the invalid ones); clamp only the allocations */
        const long long in_count = (long long)d.n * d.c * d.h * d.w, k_count = (long long)d.m * d.c * d.k * d.k;
        if (in_count < 0 || k_count < 0 || in_count > (1LL << 26) || k_count > (1LL << 26) || npts < 0 || npts > (1 << 20)) return 2;
        float *I = malloc(sizeof(float) * (size_t)(in_count > 0 ? in_count : 1));
        float *K = malloc(sizeof(float) * (size_t)(k_count > 0 ? k_count : 1));
        int *pts = malloc(sizeof(int) * 4 * (size_t)(npts > 0 ? npts : 1));
        if (!I || !K || !pts) return 3;
        for (long long e = 0; e < in_count; ++e) if (scanf("%f", &I[e]) != 1) return 4;
        for (long long e = 0; e < k_count; ++e) if (scanf("%f", &K[e]) != 1) return 4;
        for (int e = 0; e < 4 * npts; ++e) if (scanf("%d", &pts[e]) != 1) return 4;
        long long out_count = 0;
        if (d.stride >= 1 && d.h + 2 * d.pad >= d.k && d.w + 2 * d.pad >= d.k && d.n > 0 && d.m > 0 && d.k > 0)
            out_count = (long long)d.n * d.m * ((d.h + 2 * d.pad - d.k) / d.stride + 1) * ((d.w + 2 * d.pad - d.k) / d.stride + 1);
        double *O = malloc(sizeof(double) * (size_t)(out_count > 0 ? out_count : 1));
        double *A = malloc(sizeof(double) * (size_t)(out_count > 0 ? out_count : 1));
        double *Op = malloc(sizeof(double) * (size_t)(npts > 0 ? npts : 1));
        double *Ap = malloc(sizeof(double) * (size_t)(npts > 0 ? npts : 1));
        if (!O || !A || !Op || !Ap) return 3;
        int rc = conv_mcmk_oracle_f64(&d, I, K, O, A);
        printf("rc %d %lld\n", rc, rc == 0 ? out_count : 0);
        if (rc == 0) {
            for (long long e = 0; e < out_count; ++e) printf("%.17g\n", O[e]);
            for (long long e = 0; e < out_count; ++e) printf("%.17g\n", A[e]);
        }
        rc = conv_mcmk_oracle_f64_at(&d, I, K, npts, pts, Op, Ap);
        printf("at %d %d\n", rc, rc == 0 ? npts : 0);
        if (rc == 0) {
            for (int e = 0; e < npts; ++e) printf("%.17g\n", Op[e]);
            for (int e = 0; e < npts; ++e) printf("%.17g\n", Ap[e]);
        }
        free(I); free(K); free(pts); free(O); free(A); free(Op); free(Ap);
    }
    return 0;
}
