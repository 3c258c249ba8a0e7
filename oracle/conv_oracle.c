/*
 * CPU oracle for the fused conv2d / depthwise conv2d / max-pool path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against; it shares no code with the GPU library and
 * must never be called from the product path.
 *
 * What it follows (TVM paper, arXiv 1802.04799):
 *   - the operator itself is the conv2d / depthwise conv2d of the operator
 *     table (Table 2: H/W, IC, OC, kernel size K, stride S, channel multiplier
 *     1 for depthwise), written here as the textbook cross-correlation with
 *     symmetric zero padding;
 *   - the element-wise operators that follow the convolution are applied to
 *     its output in the same pass (Section 3, "Operator Fusion": conv2d is
 *     complex-out-fusable, element-wise maps fuse onto its output).
 *
 * Arithmetic: every product and sum in fp64, taken in the fixed order
 * ic -> r -> s for one output element; the result is NOT rounded.  Inputs are
 * float arrays holding exactly the values the GPU sees (bf16 inputs are
 * bf16-representable floats), so widening them to double is exact.
 *
 * Epilogue order (the paper is silent; this is the ResNet convention
 * relu(bn(conv) + identity)):
 *     t = acc + bias[oc]; t = t*scale[oc] + shift[oc]; t += residual; relu.
 *
 * Parallelism: OpenMP over (n, oc) only, so each output element is produced by
 * one thread in one order and results do not depend on the thread count.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static double epilogue(double acc, int oc, const float *scale, const float *shift,
                       const float *bias, const float *residual, int64_t out_index, int relu)
{
    double t = acc;
    if (bias) t += (double)bias[oc];
    t = t * (double)scale[oc] + (double)shift[oc];
    if (residual) t += (double)residual[out_index];
    if (relu && !(t > 0.0)) t = 0.0;
    return t;
}

static int out_extent(int in, int pad, int k, int stride)
{
    int span = in + 2 * pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

/* One output element of the dense convolution, before the epilogue. */
static double dense_point(const float *x, const float *w, int IC, int H, int W, int R, int S,
                          int sh, int sw, int ph, int pw, int n, int oc, int oh, int ow)
{
    double acc = 0.0;
    for (int ic = 0; ic < IC; ++ic)
        for (int r = 0; r < R; ++r)
            for (int s = 0; s < S; ++s) {
                int ih = oh * sh - ph + r;
                int iw = ow * sw - pw + s;
                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                double xv = (double)x[(((int64_t)n * IC + ic) * H + ih) * W + iw];
                double wv = (double)w[(((int64_t)oc * IC + ic) * R + r) * S + s];
                acc += xv * wv;
            }
    return acc;
}

/* One output element of the depthwise convolution (channel multiplier 1). */
static double depthwise_point(const float *x, const float *w, int C, int H, int W, int R, int S,
                              int sh, int sw, int ph, int pw, int n, int c, int oh, int ow)
{
    double acc = 0.0;
    for (int r = 0; r < R; ++r)
        for (int s = 0; s < S; ++s) {
            int ih = oh * sh - ph + r;
            int iw = ow * sw - pw + s;
            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
            double xv = (double)x[(((int64_t)n * C + c) * H + ih) * W + iw];
            double wv = (double)w[((int64_t)c * R + r) * S + s];
            acc += xv * wv;
        }
    return acc;
}

/*
 * Dense fused conv2d.  x [N][IC][H][W], w [OC][IC][R][S], scale/shift [OC],
 * bias [OC] or NULL, residual [N][OC][OH][OW] or NULL, y [N][OC][OH][OW] (fp64).
 * Returns 0, or -1 when the output would be empty.
 */
int oracle_conv2d_fused(const float *x, const float *w, const float *scale, const float *shift,
                        const float *bias, const float *residual, double *y,
                        int N, int IC, int H, int W, int OC, int R, int S,
                        int sh, int sw, int ph, int pw, int relu)
{
    int OH = out_extent(H, ph, R, sh), OW = out_extent(W, pw, S, sw);
    if (OH < 1 || OW < 1) return -1;
    int64_t planes = (int64_t)N * OC;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t plane = 0; plane < planes; ++plane) {
        int n = (int)(plane / OC), oc = (int)(plane % OC);
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow) {
                int64_t o = (plane * OH + oh) * OW + ow;
                double acc = dense_point(x, w, IC, H, W, R, S, sh, sw, ph, pw, n, oc, oh, ow);
                y[o] = epilogue(acc, oc, scale, shift, bias, residual, o, relu);
            }
    }
    return 0;
}

/* Same operator evaluated only at the flat output indices idx[0..count). */
int oracle_conv2d_fused_at(const float *x, const float *w, const float *scale, const float *shift,
                           const float *bias, const float *residual,
                           const int64_t *idx, int64_t count, double *out,
                           int N, int IC, int H, int W, int OC, int R, int S,
                           int sh, int sw, int ph, int pw, int relu)
{
    int OH = out_extent(H, ph, R, sh), OW = out_extent(W, pw, S, sw);
    if (OH < 1 || OW < 1) return -1;
    int64_t total = (int64_t)N * OC * OH * OW;
    for (int64_t i = 0; i < count; ++i)
        if (idx[i] < 0 || idx[i] >= total) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        int64_t o = idx[i];
        int ow = (int)(o % OW);
        int oh = (int)((o / OW) % OH);
        int oc = (int)((o / ((int64_t)OW * OH)) % OC);
        int n = (int)(o / ((int64_t)OW * OH * OC));
        double acc = dense_point(x, w, IC, H, W, R, S, sh, sw, ph, pw, n, oc, oh, ow);
        out[i] = epilogue(acc, oc, scale, shift, bias, residual, o, relu);
    }
    return 0;
}

/*
 * Depthwise fused conv2d, channel multiplier 1.  x [N][C][H][W], w [C][1][R][S],
 * y [N][C][OH][OW] (fp64).
 */
int oracle_dwconv2d_fused(const float *x, const float *w, const float *scale, const float *shift,
                          const float *bias, const float *residual, double *y,
                          int N, int C, int H, int W, int R, int S,
                          int sh, int sw, int ph, int pw, int relu)
{
    int OH = out_extent(H, ph, R, sh), OW = out_extent(W, pw, S, sw);
    if (OH < 1 || OW < 1) return -1;
    int64_t planes = (int64_t)N * C;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t plane = 0; plane < planes; ++plane) {
        int n = (int)(plane / C), c = (int)(plane % C);
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow) {
                int64_t o = (plane * OH + oh) * OW + ow;
                double acc = depthwise_point(x, w, C, H, W, R, S, sh, sw, ph, pw, n, c, oh, ow);
                y[o] = epilogue(acc, c, scale, shift, bias, residual, o, relu);
            }
    }
    return 0;
}

/*
 * Max-pool over a K x K window; taps that fall into the padding are ignored
 * (equivalent to padding with -infinity).  x [N][C][H][W] -> y [N][C][OH][OW].
 * Needed only by the ResNet-18 body workload (stem conv, then 3x3 stride-2
 * pad-1 pooling, which the 112 -> 56 size change of Table 2's C1 -> C2 forces).
 */
int oracle_maxpool2d(const float *x, double *y, int N, int C, int H, int W,
                     int K, int stride, int pad)
{
    int OH = out_extent(H, pad, K, stride), OW = out_extent(W, pad, K, stride);
    if (OH < 1 || OW < 1) return -1;
    int64_t planes = (int64_t)N * C;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t plane = 0; plane < planes; ++plane) {
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow) {
                double best = -INFINITY;
                for (int r = 0; r < K; ++r)
                    for (int s = 0; s < K; ++s) {
                        int ih = oh * stride - pad + r;
                        int iw = ow * stride - pad + s;
                        if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                        double v = (double)x[(plane * H + ih) * W + iw];
                        if (v > best) best = v;
                    }
                y[(plane * OH + oh) * OW + ow] = best;
            }
    }
    return 0;
}

/*
 * Round fp64 values to the nearest bfloat16 (ties to even) and return them as
 * floats.  bfloat16 = sign, 8 exponent bits, 7 fraction bits, i.e. 8
 * significant bits.  Used only where a workload says a layer's output is
 * stored as bf16 before the next layer reads it.  Finite inputs only;
 * bf16-subnormal magnitudes (below 2^-126) are flushed to signed zero, which
 * the synthetic workloads never produce other than exact zeros.
 */
void oracle_round_to_bf16(const double *in, float *out, int64_t count)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        double v = in[i];
        if (v == 0.0 || !isfinite(v)) { out[i] = (float)v; continue; }
        int e;
        double m = frexp(fabs(v), &e);          /* |v| = m * 2^e, m in [0.5, 1) */
        if (e - 1 < -126) { out[i] = copysignf(0.0f, (float)v); continue; }
        double scaled = ldexp(m, 8);            /* in [128, 256): 8 significant bits */
        double q = nearbyint(scaled);           /* default rounding mode: ties to even */
        double r = ldexp(q, e - 8);
        if (r > 3.3895313892515355e38) r = INFINITY;   /* above the largest bf16 */
        out[i] = (float)(v < 0 ? -r : r);
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
