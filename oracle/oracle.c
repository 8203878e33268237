/*
 * CPU oracle for the ResNet18 stage computation -- TEST INFRASTRUCTURE ONLY.
 *
 * The paper ("GPU Speedup Analysis" and "Simulation Results" sections) names
 * the operators of its benchmark task -- convolution, max pooling and the
 * "other operations" of ResNet18 (batch normalisation, ReLU, residual add,
 * global average pooling, fully connected layer) on a 224x224 input, split
 * into six stages -- but restates none of them.  Each function below is the
 * textbook definition of its operator written out as direct loops in fp64,
 * on logical NCHW tensors and OIHW weights.  There is no blocking, no
 * im2col, no GEMM and nothing shared with the HIP library: no header, no
 * table, no helper.  Only tests, the smoke check and the bench's CPU
 * baseline leg may call this file; the product path never does.
 *
 * Every function here is pinned by tests that do not go through this file's
 * own formulas: hand-worked small cases, delta-kernel / linearity / all-ones
 * closed forms, pooling monotonicity, folded-vs-unfolded BN, and agreement
 * with an independent library's fp64 operators.  Nothing is "parity unpinned".
 *
 * OpenMP splits the (image, output channel) planes across threads; each
 * output element is still one sequential sum in the order c, r, s.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#define IDX4(n, c, h, w, C, H, W) ((((size_t)(n) * (C) + (c)) * (H) + (h)) * (W) + (w))

int oracle_out_size(int in, int kernel, int stride, int pad)
{
    return (in + 2 * pad - kernel) / stride + 1;
}

/* y[n,k,p,q] = sum_{c,r,s} x[n,c,p*stride-pad+r,q*stride-pad+s] * w[k,c,r,s];
 * x outside the image counts as 0; cross-correlation (the kernel is not
 * flipped); no bias.  Output size floor((H+2*pad-R)/stride)+1. */
void oracle_conv2d(const double *x, const double *w, double *y, int N, int C, int H, int W,
                   int K, int R, int S, int stride, int pad)
{
    const int P = oracle_out_size(H, R, stride, pad);
    const int Q = oracle_out_size(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            double *yp = y + IDX4(n, k, 0, 0, K, P, Q);
            for (int i = 0; i < P * Q; ++i) yp[i] = 0.0;
            for (int c = 0; c < C; ++c)
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s) {
                        const double wv = w[IDX4(k, c, r, s, C, R, S)];
                        for (int p = 0; p < P; ++p) {
                            const int ih = p * stride - pad + r;
                            if (ih < 0 || ih >= H) continue;
                            const double *xr = x + IDX4(n, c, ih, 0, C, H, W);
                            for (int q = 0; q < Q; ++q) {
                                const int iw = q * stride - pad + s;
                                if (iw < 0 || iw >= W) continue;
                                yp[p * Q + q] += xr[iw] * wv;
                            }
                        }
                    }
        }
}

/* Inference batch normalisation, unfolded:
 * y = gamma * (x - mean) / sqrt(var + eps) + beta, per channel. */
void oracle_bn(const double *x, const double *gamma, const double *beta, const double *mean,
               const double *var, double eps, double *y, int N, int C, int HW)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            const double inv = 1.0 / sqrt(var[c] + eps);
            const size_t o = ((size_t)n * C + c) * HW;
            for (int i = 0; i < HW; ++i) y[o + i] = gamma[c] * ((x[o + i] - mean[c]) * inv) + beta[c];
        }
}

/* Folded form of the same: scale = gamma / sqrt(var + eps),
 * shift = beta - mean * scale. */
void oracle_bn_fold(const double *gamma, const double *beta, const double *mean,
                    const double *var, double eps, double *scale, double *shift, int C)
{
    for (int c = 0; c < C; ++c) {
        scale[c] = gamma[c] / sqrt(var[c] + eps);
        shift[c] = beta[c] - mean[c] * scale[c];
    }
}

/* y = scale_c * x + shift_c */
void oracle_scale_shift(const double *x, const double *scale, const double *shift, double *y,
                        int N, int C, int HW)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            const size_t o = ((size_t)n * C + c) * HW;
            for (int i = 0; i < HW; ++i) y[o + i] = scale[c] * x[o + i] + shift[c];
        }
}

void oracle_relu(const double *x, double *y, size_t n)
{
    for (size_t i = 0; i < n; ++i) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}

void oracle_add(const double *a, const double *b, double *y, size_t n)
{
    for (size_t i = 0; i < n; ++i) y[i] = a[i] + b[i];
}

/* Max pooling: maximum over the taps that fall inside the image (padding
 * never wins, i.e. it acts as -infinity); floor output size. */
void oracle_maxpool2d(const double *x, double *y, int N, int C, int H, int W, int kernel,
                      int stride, int pad)
{
    const int P = oracle_out_size(H, kernel, stride, pad);
    const int Q = oracle_out_size(W, kernel, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double m = -INFINITY;
                    for (int r = 0; r < kernel; ++r)
                        for (int s = 0; s < kernel; ++s) {
                            const int ih = p * stride - pad + r, iw = q * stride - pad + s;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            const double v = x[IDX4(n, c, ih, iw, C, H, W)];
                            if (v > m) m = v;
                        }
                    y[IDX4(n, c, p, q, C, P, Q)] = m;
                }
}

/* v[n,c] = arithmetic mean over the HW positions */
void oracle_global_avgpool(const double *x, double *v, int N, int C, int HW)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double s = 0.0;
            const size_t o = ((size_t)n * C + c) * HW;
            for (int i = 0; i < HW; ++i) s += x[o + i];
            v[(size_t)n * C + c] = s / (double)HW;
        }
}

/* y[n,o] = sum_c w[o,c] * v[n,c] + b[o]   (b may be NULL) */
void oracle_fc(const double *v, const double *w, const double *b, double *y, int N, int Cin,
               int Cout)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < Cout; ++o) {
            double s = 0.0;
            for (int c = 0; c < Cin; ++c) s += w[(size_t)o * Cin + c] * v[(size_t)n * Cin + c];
            y[(size_t)n * Cout + o] = s + (b ? b[o] : 0.0);
        }
}

/* ---- composition: conv + BN (+ReLU), BasicBlock, the six stages ---------- */

/* One convolution's parameters: OIHW weight and the four BN vectors. */
typedef struct {
    const double *w, *gamma, *beta, *mean, *var;
} conv_bn_t;

static double *alloc_d(size_t n)
{
    double *p = (double *)malloc(n * sizeof(double));
    if (!p) abort();
    return p;
}

/* y = BN(conv(x)), optionally followed by ReLU; BN in its unfolded form. */
static void conv_bn(const double *x, const conv_bn_t *p, double eps, double *y, int N, int C,
                    int H, int K, int R, int stride, int pad, int relu)
{
    const int P = oracle_out_size(H, R, stride, pad);
    oracle_conv2d(x, p->w, y, N, C, H, H, K, R, R, stride, pad);
    oracle_bn(y, p->gamma, p->beta, p->mean, p->var, eps, y, N, K, P * P);
    if (relu) oracle_relu(y, y, (size_t)N * K * P * P);
}

/* BasicBlock: y = ReLU( BN2(conv2( ReLU(BN1(conv1(x))) )) + shortcut(x) ),
 * the add coming before the last ReLU.  conv1 is 3x3 with the given stride,
 * conv2 is 3x3 stride 1; shortcut is x itself, or BN(conv1x1 stride s)(x)
 * without ReLU when `down` is given.  p points at {conv1, conv2[, down]}. */
void oracle_basic_block(const double *x, const double *const *params, int has_down, double eps,
                        double *y, int N, int C, int H, int K, int stride)
{
    conv_bn_t c1 = {params[0], params[1], params[2], params[3], params[4]};
    conv_bn_t c2 = {params[5], params[6], params[7], params[8], params[9]};
    const int P = oracle_out_size(H, 3, stride, 1);
    const size_t out_n = (size_t)N * K * P * P;
    double *t1 = alloc_d(out_n), *t2 = alloc_d(out_n), *sc = NULL;
    conv_bn(x, &c1, eps, t1, N, C, H, K, 3, stride, 1, 1);
    conv_bn(t1, &c2, eps, t2, N, K, P, K, 3, 1, 1, 0);
    if (has_down) {
        conv_bn_t cd = {params[10], params[11], params[12], params[13], params[14]};
        sc = alloc_d(out_n);
        conv_bn(x, &cd, eps, sc, N, C, H, K, 1, stride, 0, 0);
        oracle_add(t2, sc, t2, out_n);
    } else {
        oracle_add(t2, x, t2, out_n); /* identity: C == K, stride 1 */
    }
    oracle_relu(t2, y, out_n);
    free(t1); free(t2); free(sc);
}

/* Stage j of the six-stage ResNet18 task.  params = 102 pointers: for each of
 * the 20 convolutions in forward order {w, gamma, beta, mean, var}, then the
 * FC weight [1000][512] and bias [1000].
 *   0: conv7x7 s2 p3 3->64 + BN + ReLU, max-pool 3x3 s2 p1     3x224x224 -> 64x56x56
 *   1: layer1, two BasicBlocks 64->64                           -> 64x56x56
 *   2..4: layer2..4: block0 stride 2 with 1x1 projection shortcut, block1 identity
 *   5: global average pool + FC 512->1000                       -> 1000
 * in / out are NCHW fp64 (stage 5 out: [N][1000]).  Returns 0, or -1 for a bad j. */
int oracle_resnet18_stage(int j, const double *const *params, double eps, const double *in,
                          double *out, int N)
{
    if (j == 0) {
        conv_bn_t st = {params[0], params[1], params[2], params[3], params[4]};
        double *t = alloc_d((size_t)N * 64 * 112 * 112);
        conv_bn(in, &st, eps, t, N, 3, 224, 64, 7, 2, 3, 1);
        oracle_maxpool2d(t, out, N, 64, 112, 112, 3, 2, 1);
        free(t);
        return 0;
    }
    if (j == 1) {
        double *t = alloc_d((size_t)N * 64 * 56 * 56);
        oracle_basic_block(in, params + 5 * 1, 0, eps, t, N, 64, 56, 64, 1);
        oracle_basic_block(t, params + 5 * 3, 0, eps, out, N, 64, 56, 64, 1);
        free(t);
        return 0;
    }
    if (j >= 2 && j <= 4) {
        const int first = 5 + 5 * (j - 2);           /* index of layerJ.0.conv1 */
        const int C = 64 << (j - 2), K = 2 * C, H = 56 >> (j - 2);
        double *t = alloc_d((size_t)N * K * (H / 2) * (H / 2));
        oracle_basic_block(in, params + 5 * first, 1, eps, t, N, C, H, K, 2);
        oracle_basic_block(t, params + 5 * (first + 3), 0, eps, out, N, K, H / 2, K, 1);
        free(t);
        return 0;
    }
    if (j == 5) {
        double *v = alloc_d((size_t)N * 512);
        oracle_global_avgpool(in, v, N, 512, 49);
        oracle_fc(v, params[100], params[101], out, N, 512, 1000);
        free(v);
        return 0;
    }
    return -1;
}

/* Whole network: the six stages in order.  stage_out, if not NULL, holds six
 * caller buffers that receive each stage's output. */
int oracle_resnet18(const double *const *params, double eps, const double *in, double *logits,
                    int N, double *const *stage_out)
{
    static const size_t per_img[6] = {64 * 56 * 56, 64 * 56 * 56, 128 * 28 * 28,
                                      256 * 14 * 14, 512 * 7 * 7, 1000};
    const double *cur = in;
    double *owned = NULL;
    for (int j = 0; j < 6; ++j) {
        double *dst = (j == 5) ? logits : (stage_out ? stage_out[j] : alloc_d(N * per_img[j]));
        if (oracle_resnet18_stage(j, params, eps, cur, dst, N)) return -1;
        if (j == 5 && stage_out && stage_out[5] != logits)
            memcpy(stage_out[5], logits, N * per_img[5] * sizeof(double));
        free(owned);
        owned = (stage_out || j == 5) ? NULL : dst;
        cur = dst;
    }
    free(owned);
    return 0;
}
