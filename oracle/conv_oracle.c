/*
 * CPU oracle for the pattern-sparse 3x3 convolution.  TEST INFRASTRUCTURE ONLY: tests, the smoke check and the
 * bench's cpu_baseline leg use it; the product path never does and shares no code with it.
 *
 * What it computes.  Pattern pruning is an element-wise product of every 3x3 kernel with a binary mask taken from
 * the pattern library (paper, section 4.1 and the W o (sum_j z_j M_j) term of eq. (1) in section 5.1); connectivity
 * pruning removes whole kernels between an input and an output channel (sections 3 and 6.1).  The pruned layer is
 * therefore exactly an ordinary convolution whose weight tensor carries explicit zeros, and that is what is written
 * out here: a direct convolution over the masked dense weights Wm (built by oracle/pattern_oracle.py).
 *
 *   y[n][f][oy][ox] = bias[f] + sum_{c} sum_{ky} sum_{kx} Wm[f][c][ky][kx] * X(n, c, oy*s + ky - p, ox*s + kx - p)
 *
 * with X = x inside the image and 0 outside, Ho = floor((H + 2p - 3)/s) + 1 (same for Wo), no kernel flip
 * (cross-correlation, as in the deep-learning frameworks the paper trains with).  Accumulation is in double, in the
 * fixed order c, ky, kx ascending, starting from the bias; the result is returned in double, unrounded.  Taps whose
 * masked weight is exactly zero are skipped: for finite activations that changes nothing.
 *
 * Layouts: x [N][C][H][W] float, wm [F][C][3][3] float, bias [F] float or NULL, y [N][F][Ho][Wo] double.
 * fp16 workloads pass their fp16 values widened to float (lossless).
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static int out_dim(int in, int stride, int pad) {
    int t = in + 2 * pad - 3;
    if (t < 0) return 0;
    return t / stride + 1;
}

int oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int oracle_conv3x3(const float* x, const float* wm, const float* bias, int N, int C, int F, int H, int W, int stride,
                   int pad, int relu, double* y) {
    if (N < 0 || C <= 0 || F <= 0 || H <= 0 || W <= 0 || stride < 1 || pad < 0) return -1;
    const int Ho = out_dim(H, stride, pad), Wo = out_dim(W, stride, pad);
    const long plane_out = (long)Ho * Wo, plane_in = (long)H * W;
    const long jobs = (long)N * F;
#pragma omp parallel for schedule(dynamic, 1)
    for (long job = 0; job < jobs; ++job) {
        const int n = (int)(job / F), f = (int)(job % F);
        double* yp = y + ((long)n * F + f) * plane_out;
        const double b = bias ? (double)bias[f] : 0.0;
        for (long i = 0; i < plane_out; ++i) yp[i] = b;
        for (int c = 0; c < C; ++c) {
            const float* xp = x + ((long)n * C + c) * plane_in;
            for (int ky = 0; ky < 3; ++ky) {
                for (int kx = 0; kx < 3; ++kx) {
                    const double wv = (double)wm[(((long)f * C + c) * 3 + ky) * 3 + kx];
                    if (wv == 0.0) continue;
                    for (int oy = 0; oy < Ho; ++oy) {
                        const int iy = oy * stride + ky - pad;
                        if (iy < 0 || iy >= H) continue;
                        for (int ox = 0; ox < Wo; ++ox) {
                            const int ix = ox * stride + kx - pad;
                            if (ix < 0 || ix >= W) continue;
                            yp[(long)oy * Wo + ox] += wv * (double)xp[(long)iy * W + ix];
                        }
                    }
                }
            }
        }
        if (relu)
            for (long i = 0; i < plane_out; ++i)
                if (yp[i] < 0.0) yp[i] = 0.0;
    }
    return 0;
}

/* The same sum for a list of output coordinates (n, f, oy, ox), one at a time: used where a whole batch is too much
 * for the CPU.  coords is [npts][4] int32, out is [npts] double. */
int oracle_conv3x3_at(const float* x, const float* wm, const float* bias, int N, int C, int F, int H, int W,
                      int stride, int pad, int relu, const int32_t* coords, long npts, double* out) {
    if (N <= 0 || C <= 0 || F <= 0 || H <= 0 || W <= 0 || stride < 1 || pad < 0) return -1;
    const int Ho = out_dim(H, stride, pad), Wo = out_dim(W, stride, pad);
    const long plane_in = (long)H * W;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < npts; ++i) {
        const int n = coords[4 * i], f = coords[4 * i + 1], oy = coords[4 * i + 2], ox = coords[4 * i + 3];
        if (n < 0 || n >= N || f < 0 || f >= F || oy < 0 || oy >= Ho || ox < 0 || ox >= Wo) {
            bad = 1;
            continue;
        }
        double acc = bias ? (double)bias[f] : 0.0;
        for (int c = 0; c < C; ++c) {
            const float* xp = x + ((long)n * C + c) * plane_in;
            for (int ky = 0; ky < 3; ++ky) {
                const int iy = oy * stride + ky - pad;
                for (int kx = 0; kx < 3; ++kx) {
                    const int ix = ox * stride + kx - pad;
                    const double wv = (double)wm[(((long)f * C + c) * 3 + ky) * 3 + kx];
                    if (wv == 0.0 || iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                    acc += wv * (double)xp[(long)iy * W + ix];
                }
            }
        }
        out[i] = (relu && acc < 0.0) ? 0.0 : acc;
    }
    return bad ? -2 : 0;
}

/* 2x2 max-pool, stride 2, floor(H/2) x floor(W/2) outputs (the pooling between the VGG-16 stages). */
int oracle_maxpool2x2(const float* x, long planes, int H, int W, float* y) {
    if (planes < 0 || H <= 0 || W <= 0) return -1;
    const int Ho = H / 2, Wo = W / 2;
#pragma omp parallel for schedule(static)
    for (long p = 0; p < planes; ++p) {
        const float* xp = x + p * (long)H * W;
        float* yp = y + p * (long)Ho * Wo;
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox) {
                float m = xp[(long)(2 * oy) * W + 2 * ox];
                const float b = xp[(long)(2 * oy) * W + 2 * ox + 1];
                const float c = xp[(long)(2 * oy + 1) * W + 2 * ox];
                const float d = xp[(long)(2 * oy + 1) * W + 2 * ox + 1];
                if (b > m) m = b;
                if (c > m) m = c;
                if (d > m) m = d;
                yp[(long)oy * Wo + ox] = m;
            }
    }
    return 0;
}
