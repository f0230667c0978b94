/* Test infrastructure: runs every function of the C oracle on small, odd-sized inputs held in heap buffers of exactly
 * the size the function may touch, for a build with -fsanitize=address,undefined (tests/test_sanitizers.py): an access
 * outside a tensor or undefined arithmetic aborts the run.  A few identities (delta kernel, constant input, one token)
 * make sure the calls did something. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "wmdec_oracle.c"

static double *rnd(size_t n, unsigned *s)
{
    double *p = (double *)malloc(n * sizeof(double));
    for (size_t i = 0; i < n; ++i) {
        *s = *s * 1664525u + 1013904223u;
        p[i] = (double)(*s >> 8) / (double)(1u << 24) - 0.5;
    }
    return p;
}

static int finite_all(const double *p, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        if (!isfinite(p[i])) return 0;
    return 1;
}

int main(void)
{
    unsigned seed = 20260208u;
    const int n = 2, c = 6, h = 5, w = 7, groups = 3, cout = 4;
    const size_t hw = (size_t)h * w;
    int bad = 0;

    double *x = rnd((size_t)n * c * hw, &seed);
    double *mean = (double *)malloc((size_t)n * groups * sizeof(double));
    double *rstd = (double *)malloc((size_t)n * groups * sizeof(double));
    orc_gn_stats(x, n, c, h, w, groups, 1e-6, mean, rstd);
    bad += !finite_all(mean, (size_t)n * groups) || !finite_all(rstd, (size_t)n * groups);

    double *gamma = rnd(c, &seed), *beta = rnd(c, &seed);
    double *y = (double *)malloc((size_t)n * c * hw * sizeof(double));
    orc_gn_apply(x, n, c, h, w, groups, mean, rstd, gamma, beta, 1, y);
    orc_gn_apply(x, n, c, h, w, groups, mean, rstd, gamma, beta, 0, y);
    bad += !finite_all(y, (size_t)n * c * hw);
    orc_silu(x, (size_t)n * c * hw, y);
    orc_silu(x, 0, y);

    /* 3x3 and 1x1 convolution; a centre-tap delta kernel reproduces the input channel */
    for (int k = 1; k <= 3; k += 2) {
        double *wt = (double *)calloc((size_t)cout * c * k * k, sizeof(double));
        double *bias = (double *)calloc(cout, sizeof(double));
        double *z = (double *)malloc((size_t)n * cout * hw * sizeof(double));
        for (int co = 0; co < cout; ++co) wt[((size_t)co * c + co) * k * k + (k * k) / 2] = 1.0;
        orc_conv2d(x, wt, bias, n, c, cout, h, w, k, z);
        for (int in = 0; in < n; ++in)
            for (int co = 0; co < cout; ++co)
                for (size_t i = 0; i < hw; ++i)
                    bad += z[((size_t)in * cout + co) * hw + i] != x[((size_t)in * c + co) * hw + i];
        orc_conv2d(x, wt, NULL, n, c, cout, h, w, k, z);
        free(wt); free(bias); free(z);
    }
    /* one row, one column */
    {
        double *wt = rnd((size_t)cout * c * 9, &seed);
        double *z = (double *)malloc((size_t)n * cout * w * sizeof(double));
        orc_conv2d(x, wt, NULL, n, c, cout, 1, w, 3, z);
        orc_conv2d(x, wt, NULL, n, c, cout, w, 1, 3, z);
        bad += !finite_all(z, (size_t)n * cout * w);
        free(wt); free(z);
    }

    double *u = (double *)malloc((size_t)n * c * hw * 4 * sizeof(double));
    orc_upsample2x(x, n, c, h, w, u);
    bad += u[0] != x[0] || u[(size_t)2 * w + 1] != x[0] || u[(size_t)n * c * hw * 4 - 1] != x[(size_t)n * c * hw - 1];

    /* attention: odd sizes, and one token (the output is v) */
    {
        const int t = 9, d = 5;
        double *q = rnd((size_t)t * d, &seed), *kk = rnd((size_t)t * d, &seed), *v = rnd((size_t)t * d, &seed);
        double *o = (double *)malloc((size_t)t * d * sizeof(double));
        orc_attention_core(q, kk, v, t, d, 0.4472, o);
        bad += !finite_all(o, (size_t)t * d);
        orc_attention_core(q, kk, v, 1, d, 0.4472, o);
        for (int i = 0; i < d; ++i) bad += fabs(o[i] - v[i]) > 1e-15;
        free(q); free(kk); free(v); free(o);
    }
    free(x); free(mean); free(rstd); free(gamma); free(beta); free(y); free(u);
    if (bad) { printf("sanitize_check: %d checks failed\n", bad); return 1; }
    printf("sanitize_check: ok\n");
    return 0;
}
