/*
 * fp64 CPU oracle for the linked-operator-chain CNN path.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product path may call, link or load this file.
 *
 * The paper's linking (Section 4.1) and split (Section 4.2, Eq. 1) change where and
 * in which order data moves, never the values: the optimised model is stated to be
 * equivalent to the original one (Section 3).  So the oracle is the plain definition
 * of every operator of the operator library (Table 3), applied one operator at a
 * time on NCHW tensors in double precision, with no fusion, folding, tiling or
 * reordering.  The paper prints no formula for the operators themselves; the
 * standard deep-learning definitions are used (cross-correlation, zero padding,
 * floor output size, inference-form batch normalisation).
 *
 * Pins (tests/test_oracle_pins.py): delta / all-ones kernels, 1x1 conv == matrix
 * product, stride subsampling, depthwise == independent single-channel convs,
 * linearity, an independently written im2col+matmul formulation, torch's float64
 * conv2d / pooling as library special cases, BN folding identities, pooling
 * closed forms, flatten one-hot, and the K-split identity of Eq. 1.
 * The paper prints no worked numeric example, so nothing here is pinned to a
 * paper-printed value.
 *
 * All tensors are dense row-major doubles; sizes are passed as plain ints.
 * Loops over independent outputs carry an OpenMP pragma; each output element is
 * still computed by one thread, in the fixed order c, r, s.
 */
#include <math.h>
#include <stddef.h>
#include <omp.h>

#define IDX4(n, c, h, w, C, H, W) ((((size_t)(n) * (C) + (c)) * (H) + (h)) * (W) + (w))

int xo_threads(void) { return omp_get_max_threads(); }

/* x.conv (Table 3): y[n,k,oh,ow] = b[k] + sum_{c,r,s} x[n, g*Cg + c, oh*sh + r - ph, ow*sw + s - pw] * w[k,c,r,s]
 * with g = k / (K/groups), Cg = C/groups, out-of-range x taken as 0, OH = floor((H + 2ph - R)/sh) + 1.
 * w is [K][Cg][R][S]; bias may be NULL. */
void xo_conv2d(const double* x, int N, int C, int H, int W,
               const double* w, const double* bias, int K, int R, int S,
               int sh, int sw, int ph, int pw, int groups, double* y)
{
    const int Cg = C / groups, Kg = K / groups;
    const int OH = (H + 2 * ph - R) / sh + 1, OW = (W + 2 * pw - S) / sw + 1;
#pragma omp parallel for collapse(3) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int oh = 0; oh < OH; ++oh) {
                const int g = k / Kg;
                for (int ow = 0; ow < OW; ++ow) {
                    double acc = bias ? bias[k] : 0.0;
                    for (int c = 0; c < Cg; ++c)
                        for (int r = 0; r < R; ++r) {
                            const int ih = oh * sh + r - ph;
                            if (ih < 0 || ih >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                const int iw = ow * sw + s - pw;
                                if (iw < 0 || iw >= W) continue;
                                acc += x[IDX4(n, g * Cg + c, ih, iw, C, H, W)] *
                                       w[(((size_t)k * Cg + c) * R + r) * S + s];
                            }
                        }
                    y[IDX4(n, k, oh, ow, K, OH, OW)] = acc;
                }
            }
}

/* Bias node of the CBR group (Section 4.3): y = x + b[c]. */
void xo_bias(const double* x, int N, int C, int H, int W, const double* b, double* y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int i = 0; i < H * W; ++i)
                y[((size_t)n * C + c) * H * W + i] = x[((size_t)n * C + c) * H * W + i] + b[c];
}

/* Bn node of the CBR group, inference form: y = gamma * (x - mean) / sqrt(var + eps) + beta. */
void xo_bn(const double* x, int N, int C, int H, int W, const double* gamma, const double* beta,
           const double* mean, const double* var, double eps, double* y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int i = 0; i < H * W; ++i) {
                const size_t j = ((size_t)n * C + c) * H * W + i;
                y[j] = gamma[c] * (x[j] - mean[c]) / sqrt(var[c] + eps) + beta[c];
            }
}

/* Relu node of the CBR group. */
void xo_relu(const double* x, size_t count, double* y)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < count; ++i) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}

/* x.gampool, max or average over a k x k window (Table 3).  Padding never takes part in a
 * maximum.  For the average, the divisor is the number of in-range elements, or, with
 * count_include_pad, the number of window positions that lie in the padded map.
 * OH, OW are given by the caller (floor or ceil mode is a shape decision). */
void xo_pool(const double* x, int N, int C, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw,
             int OH, int OW, int is_avg, int count_include_pad, double* y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int oh = 0; oh < OH; ++oh)
                for (int ow = 0; ow < OW; ++ow) {
                    double m = -INFINITY, sum = 0.0;
                    int cnt = 0, cnt_pad = 0;
                    for (int r = 0; r < kh; ++r)
                        for (int s = 0; s < kw; ++s) {
                            const int ih = oh * sh + r - ph, iw = ow * sw + s - pw;
                            if (ih < H + ph && iw < W + pw) ++cnt_pad;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            const double v = x[IDX4(n, c, ih, iw, C, H, W)];
                            if (v > m) m = v;
                            sum += v;
                            ++cnt;
                        }
                    y[IDX4(n, c, oh, ow, C, OH, OW)] =
                        is_avg ? sum / (double)(count_include_pad ? cnt_pad : cnt) : m;
                }
}

/* Global average pooling: mean over H*W. */
void xo_gap(const double* x, int N, int C, int H, int W, double* y)
{
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < N * C; ++nc) {
        double sum = 0.0;
        for (int i = 0; i < H * W; ++i) sum += x[(size_t)nc * H * W + i];
        y[nc] = sum / (double)(H * W);
    }
}

/* x.add */
void xo_add(const double* a, const double* b, size_t count, double* y)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < count; ++i) y[i] = a[i] + b[i];
}

/* x.concat along channels: copies one input of Ci channels to channel offset c0 of y (Ct channels). */
void xo_concat_part(const double* x, int N, int Ci, int HW, int c0, int Ct, double* y)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < Ci; ++c)
            for (int i = 0; i < HW; ++i)
                y[((size_t)n * Ct + c0 + c) * HW + i] = x[((size_t)n * Ci + c) * HW + i];
}

/* x.matmul as FullyConnected (Table 4): y[n,o] = b[o] + sum_i x[n,i] * w[o,i], i running over the
 * NCHW flattening c*H*W + h*W + w of the input. */
void xo_fc(const double* x, int N, int I, const double* w, const double* bias, int O, double* y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < O; ++o) {
            double acc = bias ? bias[o] : 0.0;
            for (int i = 0; i < I; ++i) acc += x[(size_t)n * I + i] * w[(size_t)o * I + i];
            y[(size_t)n * O + o] = acc;
        }
}
