/*
 * fp64 CPU oracle for the latent -> frame convolutional decoder.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of every
 * operation of the decoder hot path.  It shares no code with the HIP library,
 * is never linked into it and must never be called by the product path; only
 * the tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What is computed follows the operator list of the paper's vertical fusion
 * (Sec. IV-B-1: Upsample, Conv2d, GroupNorm, SiLU) and its cost model
 * (Eq. 8 vs Eq. 9): fusion moves intermediates, it does not change values.  So
 * every function here is the textbook definition of its operator, in double
 * precision, with direct loops.  Tensors are dense row-major in logical
 * NCHW order.  OpenMP only distributes independent output rows over threads;
 * the order of summation inside one output element is the loop order shown.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

/* GroupNorm statistics, two passes (operator list of Sec. IV-B-1).
 * Group g of sample n holds the cpg = c/groups consecutive channels
 * [g*cpg, (g+1)*cpg) over all h*w pixels, M = cpg*h*w values.
 * pass 1: mean = sum(x)/M;  pass 2: var = sum((x-mean)^2)/M  (biased);
 * rstd = 1/sqrt(var + eps), eps inside the root. */
void orc_gn_stats(const double *x, int n, int c, int h, int w, int groups,
                  double eps, double *mean, double *rstd)
{
    const int cpg = c / groups;
    const size_t m = (size_t)cpg * h * w;
#pragma omp parallel for schedule(static)
    for (int ng = 0; ng < n * groups; ++ng) {
        const double *p = x + (size_t)ng * m; /* a group's channels are adjacent in NCHW */
        double s = 0.0;
        for (size_t i = 0; i < m; ++i) s += p[i];
        const double mu = s / (double)m;
        double q = 0.0;
        for (size_t i = 0; i < m; ++i) { const double d = p[i] - mu; q += d * d; }
        mean[ng] = mu;
        rstd[ng] = 1.0 / sqrt(q / (double)m + eps);
    }
}

/* SiLU(t) = t / (1 + exp(-t)). */
static double silu(double t) { return t / (1.0 + exp(-t)); }

void orc_silu(const double *x, size_t count, double *y)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < count; ++i) y[i] = silu(x[i]);
}

/* y = gamma_c * (x - mean_{n,g}) * rstd_{n,g} + beta_c, then SiLU if
 * apply_silu != 0.  mean/rstd as produced by orc_gn_stats. */
void orc_gn_apply(const double *x, int n, int c, int h, int w, int groups,
                  const double *mean, const double *rstd, const double *gamma,
                  const double *beta, int apply_silu, double *y)
{
    const int cpg = c / groups;
    const size_t hw = (size_t)h * w;
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < n * c; ++nc) {
        const int in = nc / c, ic = nc % c, g = ic / cpg;
        const double mu = mean[in * groups + g], rs = rstd[in * groups + g];
        const double *p = x + (size_t)nc * hw;
        double *o = y + (size_t)nc * hw;
        for (size_t i = 0; i < hw; ++i) {
            const double t = gamma[ic] * ((p[i] - mu) * rs) + beta[ic];
            o[i] = apply_silu ? silu(t) : t;
        }
    }
}

/* Direct k x k cross-correlation (no kernel flip), stride 1, zero padding
 * k/2 on every side (k = 1 or 3 in the decoder):
 *   y[n,co,oy,ox] = b[co] + sum_{ci,ky,kx} wt[co,ci,ky,kx] * x[n,ci,oy+ky-k/2,ox+kx-k/2]
 * with x taken as 0 outside the image.  bias may be NULL (= 0).
 * One thread owns one output row and accumulates it tap by tap. */
void orc_conv2d(const double *x, const double *wt, const double *bias, int n,
                int cin, int cout, int h, int w, int k, double *y)
{
    const int pad = k / 2;
    const size_t hw = (size_t)h * w;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
    for (int in = 0; in < n; ++in) {
        for (int oy = 0; oy < h; ++oy) {
            for (int co = 0; co < cout; ++co) {
                double *row = y + ((size_t)in * cout + co) * hw + (size_t)oy * w;
                const double b = bias ? bias[co] : 0.0;
                for (int ox = 0; ox < w; ++ox) row[ox] = b;
                for (int ci = 0; ci < cin; ++ci) {
                    for (int ky = 0; ky < k; ++ky) {
                        const int iy = oy + ky - pad;
                        if (iy < 0 || iy >= h) continue; /* zero padding */
                        const double *src = x + ((size_t)in * cin + ci) * hw + (size_t)iy * w;
                        for (int kx = 0; kx < k; ++kx) {
                            const double wv = wt[(((size_t)co * cin + ci) * k + ky) * k + kx];
                            const int lo = (pad - kx > 0) ? pad - kx : 0;           /* ox + kx - pad >= 0 */
                            const int hi = (w + pad - kx < w) ? w + pad - kx : w;   /* ox + kx - pad <  w */
                            for (int ox = lo; ox < hi; ++ox) row[ox] += wv * src[ox + kx - pad];
                        }
                    }
                }
            }
        }
    }
}

/* Nearest-neighbour 2x upsample: y[n,c,oy,ox] = x[n,c,oy/2,ox/2] (integer
 * division), output 2h x 2w. */
void orc_upsample2x(const double *x, int n, int c, int h, int w, double *y)
{
    const int oh = 2 * h, ow = 2 * w;
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < n * c; ++nc)
        for (int oy = 0; oy < oh; ++oy)
            for (int ox = 0; ox < ow; ++ox)
                y[((size_t)nc * oh + oy) * ow + ox] = x[((size_t)nc * h + oy / 2) * w + ox / 2];
}

/* Single-head attention core on token-major matrices q,k,v [t,d]:
 *   s_ij = (q_i . k_j) * scale;  p_i = softmax_j(s_ij) with the row maximum
 *   subtracted before exp;  o_i = sum_j p_ij v_j.
 * Each score row is materialised in full before the softmax. */
void orc_attention_core(const double *q, const double *k, const double *v,
                        int t, int d, double scale, double *o)
{
#pragma omp parallel
    {
        double *s = (double *)malloc((size_t)t * sizeof(double));
#pragma omp for schedule(dynamic, 8)
        for (int i = 0; i < t; ++i) {
            const double *qi = q + (size_t)i * d;
            double mx = -INFINITY;
            for (int j = 0; j < t; ++j) {
                const double *kj = k + (size_t)j * d;
                double acc = 0.0;
                for (int e = 0; e < d; ++e) acc += qi[e] * kj[e];
                s[j] = acc * scale;
                if (s[j] > mx) mx = s[j];
            }
            double den = 0.0;
            for (int j = 0; j < t; ++j) { s[j] = exp(s[j] - mx); den += s[j]; }
            double *oi = o + (size_t)i * d;
            for (int e = 0; e < d; ++e) oi[e] = 0.0;
            for (int j = 0; j < t; ++j) {
                const double pj = s[j] / den;
                const double *vj = v + (size_t)j * d;
                for (int e = 0; e < d; ++e) oi[e] += pj * vj[e];
            }
        }
        free(s);
    }
}
