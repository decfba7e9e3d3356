/*
 * CPU oracle for the EXEC step of an INFER action (paper section 5.2, "Actions":
 * EXEC runs the model's kernels on weights and inputs that are already present).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
 * hot path computes.  It shares no code, header, table or helper with the HIP
 * library, and only tests, the smoke check and the bench's cpu_baseline leg may
 * call it.  Nothing here is blocked, fused, vectorised by hand or reordered: each
 * function is the textbook formula written as nested loops so it can be checked
 * against the formula by eye.
 *
 * The paper treats a DNN inference as a fixed sequence of tensor operations on a
 * fixed-size input (section 2, "Predictable Performance" discussion; Table 1 gives
 * the fp32 input of 3*224*224*4 B and the 1000*4 B output).  The paper does not
 * define the layers of a ResNet; the operators below are the standard ones:
 * cross-correlation convolution with zero padding, ReLU, 3x3 max pooling with
 * padding ignored, global average pooling, a fully connected layer and softmax.
 *
 * Compiled twice: -DREAL=float (storage and accumulation in fp32, the precision of
 * the paper's own buffers in Table 1) and -DREAL=double (everything in fp64, used to
 * bound the fp32 build's own rounding).  Tensors are dense NCHW, row-major.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#ifndef REAL
#define REAL float
#endif

/* y[n][k][p][q] = b[k] + sum_{c,r,s} x[n][c][p*st-pad+r][q*st-pad+s] * w[k][c][r][s]
 * with x taken as 0 outside [0,H)x[0,W); Ho = floor((H+2*pad-kh)/st)+1 (same for W).
 * No kernel flip (cross-correlation).  b may be NULL (treated as zeros). */
void orc_conv2d(const REAL *x, const REAL *w, const REAL *b, REAL *y,
                int N, int C, int H, int W, int K, int kh, int kw, int st, int pad)
{
    int Ho = (H + 2 * pad - kh) / st + 1;
    int Wo = (W + 2 * pad - kw) / st + 1;
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    REAL acc = b ? b[k] : (REAL)0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < kh; ++r)
                            for (int s = 0; s < kw; ++s) {
                                int ih = p * st - pad + r;
                                int iw = q * st - pad + s;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W)
                                    continue;
                                acc += x[(((size_t)n * C + c) * H + ih) * W + iw] *
                                       w[(((size_t)k * C + c) * kh + r) * kw + s];
                            }
                    y[(((size_t)n * K + k) * Ho + p) * Wo + q] = acc;
                }
}

/* y[i] = max(x[i], 0) */
void orc_relu(const REAL *x, REAL *y, size_t count)
{
    for (size_t i = 0; i < count; ++i)
        y[i] = x[i] > (REAL)0 ? x[i] : (REAL)0;
}

/* y[i] = a[i] + b[i]  (the shortcut addition of a residual block) */
void orc_add(const REAL *a, const REAL *b, REAL *y, size_t count)
{
    for (size_t i = 0; i < count; ++i)
        y[i] = a[i] + b[i];
}

/* y[n][c][p][q] = max over the kh x kw window of in-range x; padded taps are ignored
 * (equivalent to padding with -infinity).  Output size uses floor, like the conv. */
void orc_maxpool2d(const REAL *x, REAL *y, int N, int C, int H, int W,
                   int kh, int kw, int st, int pad)
{
    int Ho = (H + 2 * pad - kh) / st + 1;
    int Wo = (W + 2 * pad - kw) / st + 1;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    REAL m = (REAL)(-INFINITY);
                    for (int r = 0; r < kh; ++r)
                        for (int s = 0; s < kw; ++s) {
                            int ih = p * st - pad + r;
                            int iw = q * st - pad + s;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W)
                                continue;
                            REAL v = x[(((size_t)n * C + c) * H + ih) * W + iw];
                            if (v > m)
                                m = v;
                        }
                    y[(((size_t)n * C + c) * Ho + p) * Wo + q] = m;
                }
}

/* y[n][c] = (1/(H*W)) * sum_{h,w} x[n][c][h][w] */
void orc_global_avgpool(const REAL *x, REAL *y, int N, int C, int H, int W)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            REAL acc = (REAL)0;
            for (int i = 0; i < H * W; ++i)
                acc += x[((size_t)n * C + c) * H * W + i];
            y[(size_t)n * C + c] = acc / (REAL)(H * W);
        }
}

/* z[n][j] = b[j] + sum_i f[n][i] * Wfc[j][i] */
void orc_fc(const REAL *f, const REAL *w, const REAL *b, REAL *z, int N, int In, int Out)
{
    for (int n = 0; n < N; ++n)
        for (int j = 0; j < Out; ++j) {
            REAL acc = b ? b[j] : (REAL)0;
            for (int i = 0; i < In; ++i)
                acc += f[(size_t)n * In + i] * w[(size_t)j * In + i];
            z[(size_t)n * Out + j] = acc;
        }
}

/* p[n][j] = exp(z[n][j] - max_j z[n][.]) / sum_j exp(z[n][j] - max_j z[n][.]) */
void orc_softmax(const REAL *z, REAL *p, int N, int D)
{
    for (int n = 0; n < N; ++n) {
        const REAL *row = z + (size_t)n * D;
        REAL m = row[0];
        for (int j = 1; j < D; ++j)
            if (row[j] > m)
                m = row[j];
        REAL sum = (REAL)0;
        for (int j = 0; j < D; ++j) {
            REAL e = (REAL)exp((double)(row[j] - m));
            p[(size_t)n * D + j] = e;
            sum += e;
        }
        for (int j = 0; j < D; ++j)
            p[(size_t)n * D + j] /= sum;
    }
}

/* top-1 of each row: the smallest index that attains the row maximum */
void orc_argmax(const REAL *z, int32_t *idx, int N, int D)
{
    for (int n = 0; n < N; ++n) {
        const REAL *row = z + (size_t)n * D;
        int best = 0;
        for (int j = 1; j < D; ++j)
            if (row[j] > row[best])
                best = j;
        idx[n] = best;
    }
}

/* ---- operators of the other model families the paper serves (Table 1: DenseNet, Inception v3,
 * a MobileNet-v3 pose model; Table 2 lists more).  The paper names the families only; these are
 * their standard operators, written out as definitions like the ones above. ---- */

/* Grouped cross-correlation with a rectangular filter and separate paddings.
 * Input channels are split into G equal groups and so are the output channels; output channel k
 * belongs to group g = k / (K/G) and sees only that group's C/G input channels:
 *   y[n][k][p][q] = b[k] + sum_{c' < C/G} sum_{r < kh} sum_{s < kw}
 *                   x[n][g*(C/G) + c'][p*st - ph + r][q*st - pw + s] * w[k][c'][r][s]
 * with x = 0 outside the image; Ho = floor((H + 2*ph - kh)/st) + 1, Wo likewise with pw, kw.
 * G = 1 is the dense convolution; G = C = K is a depthwise convolution (one filter per channel);
 * kh != kw gives the 1x7 / 7x1 filters of Inception.  w is [K][C/G][kh][kw]; b may be NULL. */
void orc_conv2d_grouped(const REAL *x, const REAL *w, const REAL *b, REAL *y,
                        int N, int C, int H, int W, int K, int kh, int kw, int st, int ph, int pw, int G)
{
    int Ho = (H + 2 * ph - kh) / st + 1;
    int Wo = (W + 2 * pw - kw) / st + 1;
    int Cg = C / G, Kg = K / G;
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            int g = k / Kg;
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    REAL acc = b ? b[k] : (REAL)0;
                    for (int c = 0; c < Cg; ++c)
                        for (int r = 0; r < kh; ++r)
                            for (int s = 0; s < kw; ++s) {
                                int ih = p * st - ph + r;
                                int iw = q * st - pw + s;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W)
                                    continue;
                                acc += x[(((size_t)n * C + g * Cg + c) * H + ih) * W + iw] *
                                       w[(((size_t)k * Cg + c) * kh + r) * kw + s];
                            }
                    y[(((size_t)n * K + k) * Ho + p) * Wo + q] = acc;
                }
        }
}

/* hard swish: y = x * min(max(x + 3, 0), 6) / 6  (0 for x <= -3, x for x >= 3) */
void orc_hswish(const REAL *x, REAL *y, size_t count)
{
    for (size_t i = 0; i < count; ++i) {
        REAL t = x[i] + (REAL)3;
        if (t < (REAL)0)
            t = (REAL)0;
        if (t > (REAL)6)
            t = (REAL)6;
        y[i] = x[i] * t / (REAL)6;
    }
}

/* channel concatenation: y[n][c] = a[n][c] for c < Ca, b[n][c - Ca] for Ca <= c < Ca + Cb;
 * HW = spatial positions per channel */
void orc_concat_channels(const REAL *a, const REAL *b, REAL *y, int N, int Ca, int Cb, int HW)
{
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < Ca; ++c)
            for (int i = 0; i < HW; ++i)
                y[((size_t)n * (Ca + Cb) + c) * HW + i] = a[((size_t)n * Ca + c) * HW + i];
        for (int c = 0; c < Cb; ++c)
            for (int i = 0; i < HW; ++i)
                y[((size_t)n * (Ca + Cb) + Ca + c) * HW + i] = b[((size_t)n * Cb + c) * HW + i];
    }
}
