/* Drives the C oracle (conv, pooled features, backward) on small cases that reach its edges (padding on
 * both sides, the largest dilation, one output position, several channels) so that it can run under
 * AddressSanitizer and UndefinedBehaviorSanitizer.  TEST INFRASTRUCTURE. */
#include <stdio.h>
#include <stdlib.h>

typedef long long i64;
int rk_oracle_conv(const float *x, int C, int L, int len, int dil, int pad, double bias, int nch, const int *ch,
                   const float *w, double *y);
int rk_oracle_transform(const float *x, int B, int C, int L, const int *length, const int *dilation, const int *padding,
                        const float *bias, const int *n_ch, const i64 *ch_off, const int *channels, const i64 *w_off,
                        const float *weights, int nsel, const int *sel, double lambda, double shift, double amb_eps,
                        double *omax, i64 *ocnt, i64 *oamb, double *osoft, int *on, i64 *oarg, double *ogap);
int rk_oracle_backward(const float *x, int B, int C, int L, int K, const int *length, const int *dilation,
                       const int *padding, const float *bias, const int *n_ch, const i64 *ch_off, const int *channels,
                       const i64 *w_off, const float *weights, int nsel, const int *sel, double lambda, double shift,
                       const double *g_soft, const double *g_max, double *grad_w, double *grad_b);

static unsigned state = 12345u;
static float rnd(void) { state = state * 1664525u + 1013904223u; return (float)((state >> 8) & 0xffff) / 32768.f - 1.f; }

int main(void)
{
    enum { B = 3, C = 4, L = 61, K = 6 };
    /* lengths, dilations, paddings: d = 1 unpadded; largest dilation with and without padding (one output
     * position without); mid dilation padded; three channels */
    const int length[K] = {7, 9, 11, 7, 9, 11};
    const int dilation[K] = {1, 7, 6, 10, 3, 2};
    const int padding[K] = {0, 28, 0, 30, 12, 0};
    const int n_ch[K] = {1, 2, 1, 4, 3, 2};
    i64 ch_off[K + 1], w_off[K + 1];
    int channels[16];
    float weights[200], bias[K];
    ch_off[0] = 0; w_off[0] = 0;
    for (int k = 0; k < K; ++k) {
        for (int c = 0; c < n_ch[k]; ++c) channels[ch_off[k] + c] = (k + c) % C;
        ch_off[k + 1] = ch_off[k] + n_ch[k];
        w_off[k + 1] = w_off[k] + (i64)n_ch[k] * length[k];
        bias[k] = rnd();
    }
    for (i64 i = 0; i < w_off[K]; ++i) weights[i] = rnd();
    float *x = malloc(sizeof(float) * B * C * L);
    for (int i = 0; i < B * C * L; ++i) x[i] = rnd();
    double *y = malloc(sizeof(double) * (L + 64));
    for (int k = 0; k < K; ++k) {
        int n = rk_oracle_conv(x, C, L, length[k], dilation[k], padding[k], bias[k], n_ch[k], channels + ch_off[k],
                               weights + w_off[k], y);
        if (n != L + 2 * padding[k] - (length[k] - 1) * dilation[k]) { fprintf(stderr, "conv length %d\n", k); return 1; }
    }
    int sel[K] = {5, 0, 3, 1, 2, 4};
    double omax[B * K], osoft[B * K], ogap[B * K];
    i64 ocnt[B * K], oamb[B * K], oarg[B * K];
    int on[K];
    if (rk_oracle_transform(x, B, C, L, length, dilation, padding, bias, n_ch, ch_off, channels, w_off, weights, K, sel,
                            10.0, -3.0, 1e-5, omax, ocnt, oamb, osoft, on, oarg, ogap)) return 1;
    double gs[B * K], gm[B * K], *gw = malloc(sizeof(double) * w_off[K]), gb[K];
    for (int i = 0; i < B * K; ++i) { gs[i] = rnd(); gm[i] = rnd(); }
    if (rk_oracle_backward(x, B, C, L, K, length, dilation, padding, bias, n_ch, ch_off, channels, w_off, weights, K, sel,
                           10.0, -3.0, gs, gm, gw, gb)) return 1;
    if (rk_oracle_backward(x, B, C, L, K, length, dilation, padding, bias, n_ch, ch_off, channels, w_off, weights, 2, sel,
                           3.0, 3.0, gs, NULL, gw, gb)) return 1;
    /* a kernel that does not fit is an error, not an out-of-bounds read */
    const int too_wide[K] = {1, 7, 7, 10, 3, 2};
    if (rk_oracle_transform(x, B, C, L, length, too_wide, padding, bias, n_ch, ch_off, channels, w_off, weights, K, sel,
                            10.0, -3.0, 1e-5, omax, ocnt, oamb, osoft, on, oarg, ogap) == 0) return 1;
    free(x); free(y); free(gw);
    puts("oracle driver: ok");
    return 0;
}
