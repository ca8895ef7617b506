/*
 * CPU oracle for the ROCKET random-convolutional-kernel transform.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  It shares no code with the library, and
 * only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.
 *
 * What it computes (paper section 3, items (1) and (2); section 3.2, Eq. 1-4):
 *
 *   kernel k: length len, dilation d, padding p, bias, a list of channels and
 *   one weight row per listed channel.
 *
 *   conv output      y[t] = bias + sum_c sum_j w[c][j] * x[ch[c]][t + j*d - p]
 *                    for t = 0 .. n-1,  n = L + 2p - (len-1)d,  x = 0 outside [0,L)
 *                    (cross-correlation: the weights are not flipped)
 *   max feature      max_t y[t]
 *   PPV   (Eq. 1-2)  (1/n) * #{t : y[t] > 0}            (strict inequality)
 *   softPPV (Eq.3-4) (1/n) * sum_t 1 / (1 + exp(-(lambda*y[t] + shift)))
 *                    The prose of section 3.2 fixes shift = -3 (negative inputs
 *                    land nearer 0 than positive inputs land near 1); the
 *                    printed formula corresponds to shift = +3.  shift is an
 *                    argument so both readings can be evaluated.
 *   backward         derivative of  sum_{b,k} g_soft[b,k]*softPPV[b,k]
 *                                 + sum_{b,k} g_max[b,k]*max[b,k]
 *                    with respect to the stored weights and biases (the
 *                    gradient flow the paper says softPPV allows).
 *
 * All arithmetic is fp64 on fp32 inputs; nothing is blocked, fused or
 * reordered.  OpenMP, when enabled, only distributes independent
 * (series, kernel) pairs over threads.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef long long i64;

/* number of output positions of one kernel */
static int out_len(int L, int len, int dil, int pad)
{
    return L + 2 * pad - (len - 1) * dil;
}

/* y[t] for one series x (C rows of L floats) and one kernel */
static double conv_at(const float *x, int L, int len, int dil, int pad,
                      double bias, int nch, const int *ch, const float *w, int t)
{
    double acc = 0.0;
    for (int c = 0; c < nch; ++c) {
        const float *row = x + (size_t)ch[c] * (size_t)L;
        for (int j = 0; j < len; ++j) {
            i64 idx = (i64)t + (i64)j * dil - pad;
            if (idx >= 0 && idx < L)
                acc += (double)w[c * len + j] * (double)row[idx];
        }
    }
    return acc + bias;
}

int rk_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void rk_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Full conv output of one kernel over one series; y must hold n doubles.
 * Returns n, or -1 if the kernel does not fit the series. */
int rk_oracle_conv(const float *x, int C, int L, int len, int dil, int pad,
                   double bias, int nch, const int *ch, const float *w, double *y)
{
    int n = out_len(L, len, dil, pad);
    if (n < 1) return -1;
    for (int c = 0; c < nch; ++c)
        if (ch[c] < 0 || ch[c] >= C) return -1;
    for (int t = 0; t < n; ++t)
        y[t] = conv_at(x, L, len, dil, pad, bias, nch, ch, w, t);
    return n;
}

/*
 * Pooled features of every series b in [0,B) for the kernels listed in
 * sel[0..nsel).  Outputs are B x nsel, row-major:
 *   omax   max_t y            ocnt  #{y > 0}        on  n (per selected kernel)
 *   oamb   #{|y| < amb_eps}   (positions whose sign a float32 evaluation may
 *                              legitimately get wrong; used by the tolerance rule)
 *   osoft  softPPV            oarg  first t attaining the max
 *   ogap   max minus the largest y at any other position (inf if n == 1)
 */
int rk_oracle_transform(const float *x, int B, int C, int L,
                        const int *length, const int *dilation, const int *padding,
                        const float *bias, const int *n_ch,
                        const i64 *ch_off, const int *channels,
                        const i64 *w_off, const float *weights,
                        int nsel, const int *sel,
                        double lambda, double shift, double amb_eps,
                        double *omax, i64 *ocnt, i64 *oamb, double *osoft,
                        int *on, i64 *oarg, double *ogap)
{
    for (int s = 0; s < nsel; ++s) {
        int k = sel[s];
        int n = out_len(L, length[k], dilation[k], padding[k]);
        if (n < 1) return -1;
        on[s] = n;
    }
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int s = 0; s < nsel; ++s) {
            int k = sel[s];
            const float *xb = x + (size_t)b * (size_t)C * (size_t)L;
            int len = length[k], dil = dilation[k], pad = padding[k];
            int n = on[s];
            const int *ch = channels + ch_off[k];
            const float *w = weights + w_off[k];
            double best = -INFINITY, second = -INFINITY, soft = 0.0;
            i64 cnt = 0, amb = 0, arg = 0;
            for (int t = 0; t < n; ++t) {
                double y = conv_at(xb, L, len, dil, pad, (double)bias[k], n_ch[k], ch, w, t);
                if (y > best) { second = best; best = y; arg = t; }
                else if (y > second) second = y;
                if (y > 0.0) ++cnt;
                if (fabs(y) < amb_eps) ++amb;
                soft += 1.0 / (1.0 + exp(-(lambda * y + shift)));
            }
            size_t o = (size_t)b * (size_t)nsel + (size_t)s;
            omax[o] = best;
            ocnt[o] = cnt;
            oamb[o] = amb;
            osoft[o] = soft / (double)n;
            oarg[o] = arg;
            ogap[o] = best - second;
        }
    }
    return 0;
}

/*
 * Backward pass.  g_soft and g_max are B x nsel (g_max may be NULL: the max
 * feature then contributes nothing).  grad_w has the layout of `weights`,
 * grad_b has K entries; both are overwritten, entries of kernels that are not
 * selected become 0, and contributions are summed over the batch.
 *
 *   s_t   = 1 / (1 + exp(-(lambda*y_t + shift)))
 *   q_t   = g_soft * (lambda / n) * s_t * (1 - s_t)          d softPPV / d y_t
 *   grad_b       += sum_t q_t
 *   grad_w[c][j] += sum_t q_t * x[ch[c]][t + j*d - p]
 * and, for the max feature, with t* the first position attaining the max:
 *   grad_b += g_max ;  grad_w[c][j] += g_max * x[ch[c]][t* + j*d - p]
 */
int rk_oracle_backward(const float *x, int B, int C, int L, int K,
                       const int *length, const int *dilation, const int *padding,
                       const float *bias, const int *n_ch,
                       const i64 *ch_off, const int *channels,
                       const i64 *w_off, const float *weights,
                       int nsel, const int *sel,
                       double lambda, double shift,
                       const double *g_soft, const double *g_max,
                       double *grad_w, double *grad_b)
{
    i64 total_w = w_off[K];
    for (i64 i = 0; i < total_w; ++i) grad_w[i] = 0.0;
    for (int k = 0; k < K; ++k) grad_b[k] = 0.0;
    for (int s = 0; s < nsel; ++s)
        if (out_len(L, length[sel[s]], dilation[sel[s]], padding[sel[s]]) < 1) return -1;

    /* kernels are independent of each other; the batch sum stays sequential
       inside one thread so the result does not depend on the thread count */
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < nsel; ++s) {
        int k = sel[s];
        int len = length[k], dil = dilation[k], pad = padding[k], nch = n_ch[k];
        int n = out_len(L, len, dil, pad);
        const int *ch = channels + ch_off[k];
        const float *w = weights + w_off[k];
        double *gw = grad_w + w_off[k];
        for (int b = 0; b < B; ++b) {
            const float *xb = x + (size_t)b * (size_t)C * (size_t)L;
            double gs = g_soft[(size_t)b * nsel + s];
            double best = -INFINITY;
            int arg = 0;
            for (int t = 0; t < n; ++t) {
                double y = conv_at(xb, L, len, dil, pad, (double)bias[k], nch, ch, w, t);
                if (y > best) { best = y; arg = t; }
                double sg = 1.0 / (1.0 + exp(-(lambda * y + shift)));
                double q = gs * (lambda / (double)n) * sg * (1.0 - sg);
                grad_b[k] += q;
                for (int c = 0; c < nch; ++c) {
                    const float *row = xb + (size_t)ch[c] * (size_t)L;
                    for (int j = 0; j < len; ++j) {
                        i64 idx = (i64)t + (i64)j * dil - pad;
                        if (idx >= 0 && idx < L) gw[c * len + j] += q * (double)row[idx];
                    }
                }
            }
            if (g_max) {
                double gm = g_max[(size_t)b * nsel + s];
                grad_b[k] += gm;
                for (int c = 0; c < nch; ++c) {
                    const float *row = xb + (size_t)ch[c] * (size_t)L;
                    for (int j = 0; j < len; ++j) {
                        i64 idx = (i64)arg + (i64)j * dil - pad;
                        if (idx >= 0 && idx < L) gw[c * len + j] += gm * (double)row[idx];
                    }
                }
            }
        }
    }
    return 0;
}
