/*
 * CPU reference convolutions — TEST INFRASTRUCTURE ONLY.
 *
 * Slow, plain, direct (no im2col, no tiling) implementations of the three
 * spatial operators a SubNet forward pass needs.  Only tests, the smoke check
 * and the CPU-baseline leg of the benchmark may call this; the GPU library
 * never does and shares no code with it.
 *
 * Layout: activations x[n][c][h][w], weights w[k][c][r][s], all float32.
 * Every output element is accumulated in double and rounded to float once.
 *
 * The operator is the textbook one the paper relies on for SubNet inference
 * (Section 2.1: a SubNet forward pass over conv layers selected from the
 * SuperNet; Section 4.2.1: 3x3 and 1x1 kernels):
 *   y[n,k,p,q] = sum_{c,r,s} w[k,c,r,s] * x[n,c,p*st+r-pad,q*st+s-pad]
 * with zero padding.
 */
#include <float.h>
#include <stdlib.h>
#include <string.h>

static int out_extent(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

/* Dense convolution. y has shape [N][K][P][Q], P,Q from out_extent(). Returns 0, or -1 on bad sizes. */
int ref_conv2d(const float *x, const float *w, float *y, int N, int C, int H, int W, int K, int R, int S,
               int stride, int pad)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return -1;
    const int P = out_extent(H, R, stride, pad), Q = out_extent(W, S, stride, pad);
    if (P <= 0 || Q <= 0) return -1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            double *acc = (double *)calloc((size_t)P * Q, sizeof(double));
            for (int c = 0; c < C; ++c)
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s) {
                        const double wv = w[(((size_t)k * C + c) * R + r) * S + s];
                        const float *xc = x + ((size_t)n * C + c) * H * W;
                        for (int p = 0; p < P; ++p) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int q = 0; q < Q; ++q) {
                                const int v = q * stride + s - pad;
                                if (v < 0 || v >= W) continue;
                                acc[(size_t)p * Q + q] += wv * (double)xc[(size_t)h * W + v];
                            }
                        }
                    }
            float *yo = y + ((size_t)n * K + k) * P * Q;
            for (int i = 0; i < P * Q; ++i) yo[i] = (float)acc[i];
            free(acc);
        }
    return 0;
}

/* Depthwise convolution: w[c][r][s], y[n][c][p][q] = sum_{r,s} w[c,r,s] * x[n,c,p*st+r-pad,q*st+s-pad]. */
int ref_dwconv2d(const float *x, const float *w, float *y, int N, int C, int H, int W, int R, int S, int stride,
                 int pad)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return -1;
    const int P = out_extent(H, R, stride, pad), Q = out_extent(W, S, stride, pad);
    if (P <= 0 || Q <= 0) return -1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            const float *xc = x + ((size_t)n * C + c) * H * W;
            float *yo = y + ((size_t)n * C + c) * P * Q;
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int r = 0; r < R; ++r) {
                        const int h = p * stride + r - pad;
                        if (h < 0 || h >= H) continue;
                        for (int s = 0; s < S; ++s) {
                            const int v = q * stride + s - pad;
                            if (v < 0 || v >= W) continue;
                            acc += (double)w[((size_t)c * R + r) * S + s] * (double)xc[(size_t)h * W + v];
                        }
                    }
                    yo[(size_t)p * Q + q] = (float)acc;
                }
        }
    return 0;
}

/* Max pooling, window k, padded cells never win (treated as -infinity). */
int ref_maxpool2d(const float *x, float *y, int N, int C, int H, int W, int k, int stride, int pad)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || k <= 0 || stride <= 0 || pad < 0) return -1;
    const int P = out_extent(H, k, stride, pad), Q = out_extent(W, k, stride, pad);
    if (P <= 0 || Q <= 0) return -1;
#pragma omp parallel for collapse(2)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            const float *xc = x + ((size_t)n * C + c) * H * W;
            float *yo = y + ((size_t)n * C + c) * P * Q;
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    float m = -FLT_MAX;
                    for (int r = 0; r < k; ++r) {
                        const int h = p * stride + r - pad;
                        if (h < 0 || h >= H) continue;
                        for (int s = 0; s < k; ++s) {
                            const int v = q * stride + s - pad;
                            if (v < 0 || v >= W) continue;
                            const float t = xc[(size_t)h * W + v];
                            if (t > m) m = t;
                        }
                    }
                    yo[(size_t)p * Q + q] = m;
                }
        }
    return 0;
}

/*
 * Integer operators of the int8 path (paper Section 5.1, footnote: int8 weights, activations and zero points):
 *   acc[n,k,p,q] = sum_{c,r,s} w[k,c,r,s] * (x[n,c,p*st+r-pad,q*st+s-pad] - zx)
 * over the taps that fall inside the image (a padded position holds the real value 0, i.e. the code zx, and adds
 * nothing).  int8 in, exact int32 out (|acc| <= C*R*S*127*255 must stay below 2^31: checked).
 */
#include <stdint.h>

int ref_conv2d_i8(const int8_t *x, const int8_t *w, int32_t *acc, int N, int C, int H, int W, int K, int R, int S,
                  int stride, int pad, int zx)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return -1;
    if ((double)C * R * S * 127.0 * 255.0 >= 2147483647.0) return -2;
    const int P = out_extent(H, R, stride, pad), Q = out_extent(W, S, stride, pad);
    if (P <= 0 || Q <= 0) return -1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            int32_t *a = acc + ((size_t)n * K + k) * P * Q;
            memset(a, 0, sizeof(int32_t) * (size_t)P * Q);
            for (int c = 0; c < C; ++c)
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s) {
                        const int32_t wv = w[(((size_t)k * C + c) * R + r) * S + s];
                        const int8_t *xc = x + ((size_t)n * C + c) * H * W;
                        for (int p = 0; p < P; ++p) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int q = 0; q < Q; ++q) {
                                const int v = q * stride + s - pad;
                                if (v < 0 || v >= W) continue;
                                a[(size_t)p * Q + q] += wv * ((int32_t)xc[(size_t)h * W + v] - zx);
                            }
                        }
                    }
        }
    return 0;
}

/* Max pooling on int8 codes (one scale, one zero point: the order of codes is the order of values); positions
 * outside the image take no part. */
int ref_maxpool2d_i8(const int8_t *x, int8_t *y, int N, int C, int H, int W, int R, int stride, int pad)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || R <= 0 || stride <= 0 || pad < 0) return -1;
    const int P = out_extent(H, R, stride, pad), Q = out_extent(W, R, stride, pad);
    if (P <= 0 || Q <= 0) return -1;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            const int8_t *xc = x + ((size_t)n * C + c) * H * W;
            int8_t *yc = y + ((size_t)n * C + c) * P * Q;
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    int best = -129;
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < R; ++s) {
                            const int h = p * stride + r - pad, v = q * stride + s - pad;
                            if (h < 0 || h >= H || v < 0 || v >= W) continue;
                            if (xc[(size_t)h * W + v] > best) best = xc[(size_t)h * W + v];
                        }
                    if (best < -128) return -3; /* an empty window */
                    yc[(size_t)p * Q + q] = (int8_t)best;
                }
        }
    return 0;
}
