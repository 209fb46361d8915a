/*
 * CPU oracle for the forward 2-D convolution.  TEST INFRASTRUCTURE ONLY: it is called by the
 * tests, by the smoke check and by the benchmark's CPU-baseline leg, never by the library.
 *
 * What it computes is the paper's convolution loop nest (figure "The 2-D Convolution code",
 * section "Convolutions") with the channel blocking removed:
 *
 *   out[n][k][p][q] = sum_{c, r, s} in[n][c][p*stride + r - pad][q*stride + s - pad] * wt[k][c][r][s]
 *
 * Readings where the paper is silent (it shows no padding, no bias and accumulates in place):
 * taps that fall outside the image contribute zero; the same stride and padding apply to both
 * axes; the filter is not flipped (the listing indexes ij+kj, ii+ki); out is overwritten;
 * P = floor((H + 2 pad - R)/stride) + 1.  The optional element-wise tail stands for the
 * operator fused into the last reduction iteration (section "Operator Fusion"): add bias[k],
 * then ReLU y = max(x,0) or ReLU6 y = min(max(x,0),6) (section "Evaluation of Operator Fusion").
 *
 * Every product and sum is IEEE double, summed in the fixed order c, r, s.  absum receives
 * |bias[k]| + sum |in * wt|, the scale against which a float32 result is judged.
 *
 * Pinned by tests/test_oracle_conv.py: hand-counted tap tables, one-hot filters (shifted copy),
 * 1x1 convolution == matrix product, linearity, exact small-integer sums against numpy int64.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2 };

static void conv_point(int C, int H, int W, int K, int R, int S, int stride, int pad,
                       const float *in, const float *wt, const float *bias, int act,
                       int64_t n, int64_t k, int64_t p, int64_t q, double *y, double *scale)
{
    double acc = 0.0, mag = 0.0;
    (void)K;
    for (int c = 0; c < C; ++c)
        for (int r = 0; r < R; ++r)
            for (int s = 0; s < S; ++s) {
                int64_t h = p * stride + r - pad;
                int64_t w = q * stride + s - pad;
                if (h < 0 || h >= H || w < 0 || w >= W)
                    continue; /* zero padding */
                double x = (double)in[((n * C + c) * H + h) * W + w];
                double f = (double)wt[((k * C + c) * R + r) * S + s];
                acc += x * f;
                mag += fabs(x * f);
            }
    if (bias) {
        acc += (double)bias[k];
        mag += fabs((double)bias[k]);
    }
    if (act == ACT_RELU || act == ACT_RELU6)
        acc = acc > 0.0 ? acc : 0.0;
    if (act == ACT_RELU6)
        acc = acc < 6.0 ? acc : 6.0;
    *y = acc;
    *scale = mag;
}

/* Whole output tensor, NKPQ.  Returns 0, or -1 on a shape that has no output. */
int oracle_conv2d_fwd(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                      const float *in, const float *wt, const float *bias, int act,
                      double *out, double *absum)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return -1;
    int64_t P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    if (H + 2 * pad < R || W + 2 * pad < S || P <= 0 || Q <= 0)
        return -1;
    int64_t rows = (int64_t)N * K;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t nk = 0; nk < rows; ++nk) {
        int64_t n = nk / K, k = nk % K;
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q) {
                int64_t o = (nk * P + p) * Q + q;
                conv_point(C, H, W, K, R, S, stride, pad, in, wt, bias, act, n, k, p, q,
                           &out[o], &absum[o]);
            }
    }
    return 0;
}

/* Only the outputs whose flat NKPQ indices are listed in idx[0..count). */
int oracle_conv2d_fwd_at(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                         const float *in, const float *wt, const float *bias, int act,
                         int64_t count, const int64_t *idx, double *out, double *absum)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return -1;
    int64_t P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    if (H + 2 * pad < R || W + 2 * pad < S || P <= 0 || Q <= 0)
        return -1;
    int64_t total = (int64_t)N * K * P * Q;
    for (int64_t i = 0; i < count; ++i)
        if (idx[i] < 0 || idx[i] >= total)
            return -2;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        int64_t o = idx[i];
        int64_t q = o % Q, p = (o / Q) % P, k = (o / (Q * P)) % K, n = o / (Q * P * K);
        conv_point(C, H, W, K, R, S, stride, pad, in, wt, bias, act, n, k, p, q, &out[i], &absum[i]);
    }
    return 0;
}
