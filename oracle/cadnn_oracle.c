/*
 * CPU oracle for pruned-weight CNN inference layers.  TEST INFRASTRUCTURE ONLY:
 * it is imported by the tests, by the smoke check and by the benchmark's
 * cpu_baseline leg, never by the product path, and shares no code with the HIP
 * library.
 *
 * What it computes.  The paper prunes weights offline (Section 3) and then runs
 * ordinary inference over the pruned model, with convolution + batch-norm +
 * activation fused into one layer (Section 4, "Model computation fusion and
 * transformation").  With batch-norm folded into the weights and a per-channel
 * bias, a layer is therefore exactly
 *
 *   z[n,co,oh,ow] = sum_{ci,kh,kw} W[co,ci,kh,kw] * X~[n,ci,oh*s+kh-p,ow*s+kw-p]
 *   y             = act(z + bias[co] + residual[n,co,oh,ow])
 *
 * where X~ is X inside the image and 0 outside (cross-correlation, no kernel
 * flip), act is ReLU or identity, and zero weights contribute nothing.  This is
 * the plain definition written out over the DENSE pruned tensor: sums are taken
 * in double precision in fixed ci -> kh -> kw order and the result is handed
 * back in double so the caller rounds once to the storage type.  The only
 * liberty is skipping terms whose weight is exactly zero (which cannot change
 * the sum) with the weight loop outermost.
 *
 * Pinned by tests/test_oracle_*.py against brute-force loops, a hand-computed
 * example, numpy.matmul (1x1 conv and FC, Section 4: 1x1 convolution is a
 * matrix multiply), explicit im2col + matmul, torch's float64 conv2d, and the
 * invariants (zero-weight invariance, identity kernel, linearity, fused ==
 * unfused); the depthwise layer against the full convolution over the
 * block-diagonal expansion of its filters, a box-filter closed form and torch's
 * grouped float64 conv2d.  Whole-network outputs have no pin from the paper (it prints no
 * logits): parity unpinned beyond the per-layer pins.
 */
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int out_size(int size, int k, int stride, int pad) {
    int t = size + 2 * pad - k;
    if (t < 0) return 0;
    return t / stride + 1;
}

/* Fused conv layer.  x[n][cin][h][w], w[cout][cin][kh][kw], bias[cout] or NULL,
 * residual[n][cout][hout][wout] or NULL, y[n][cout][hout][wout] (double).
 * Returns 0, or -1 on bad arguments / allocation failure. */
int oracle_conv2d(const float* x, const float* w, const float* bias, const float* residual,
                  double* y, int n, int cin, int h, int wd, int cout, int kh, int kw,
                  int stride, int pad, int relu) {
    if (!x || !w || !y || n <= 0 || cin <= 0 || h <= 0 || wd <= 0 || cout <= 0 || kh <= 0 ||
        kw <= 0 || stride <= 0 || pad < 0)
        return -1;
    const int hout = out_size(h, kh, stride, pad), wout = out_size(wd, kw, stride, pad);
    if (hout <= 0 || wout <= 0) return -1;
    const long plane = (long)hout * wout;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int in = 0; in < n; ++in) {
        for (int co = 0; co < cout; ++co) {
            double* acc = y + ((long)in * cout + co) * plane;
            for (long i = 0; i < plane; ++i) acc[i] = 0.0;
            for (int ci = 0; ci < cin; ++ci) {
                const float* xp = x + ((long)in * cin + ci) * h * wd;
                for (int r = 0; r < kh; ++r) {
                    for (int c = 0; c < kw; ++c) {
                        const float wv = w[(((long)co * cin + ci) * kh + r) * kw + c];
                        if (wv == 0.0f) continue;           /* a zero weight adds nothing */
                        const double wvd = (double)wv;
                        for (int oh = 0; oh < hout; ++oh) {
                            const int ih = oh * stride + r - pad;
                            if (ih < 0 || ih >= h) continue;   /* outside the image: X~ = 0 */
                            for (int ow = 0; ow < wout; ++ow) {
                                const int iw = ow * stride + c - pad;
                                if (iw < 0 || iw >= wd) continue;
                                acc[(long)oh * wout + ow] += wvd * (double)xp[(long)ih * wd + iw];
                            }
                        }
                    }
                }
            }
            const double b = bias ? (double)bias[co] : 0.0;
            const float* rp = residual ? residual + ((long)in * cout + co) * plane : NULL;
            for (long i = 0; i < plane; ++i) {
                double t = acc[i] + b;
                if (rp) t += (double)rp[i];
                if (relu && !(t > 0.0)) t = 0.0;
                acc[i] = t;
            }
        }
    }
    return 0;
}

/* Fused depthwise convolution layer (Section 4 names depthwise convolution + batch-norm +
 * activation as one fused kernel of MobileNet-V1): every channel is filtered by its own
 * kh x kw filter and nothing is summed across channels,
 *
 *   y[n,c,oh,ow] = act( sum_{r,s} W[c,r,s] * X~[n,c,oh*stride+r-pad,ow*stride+s-pad] + bias[c] )
 *
 * x[n][ch][h][w], w[ch][kh][kw], bias[ch] or NULL, y[n][ch][hout][wout] (double).  Sums in
 * double, taps in r -> s order, zero taps skipped. */
int oracle_depthwise_conv2d(const float* x, const float* w, const float* bias, double* y, int n,
                            int ch, int h, int wd, int kh, int kw, int stride, int pad, int relu) {
    if (!x || !w || !y || n <= 0 || ch <= 0 || h <= 0 || wd <= 0 || kh <= 0 || kw <= 0 ||
        stride <= 0 || pad < 0)
        return -1;
    const int hout = out_size(h, kh, stride, pad), wout = out_size(wd, kw, stride, pad);
    if (hout <= 0 || wout <= 0) return -1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int in = 0; in < n; ++in) {
        for (int c = 0; c < ch; ++c) {
            const float* xp = x + ((long)in * ch + c) * h * wd;
            double* yp = y + ((long)in * ch + c) * hout * wout;
            for (int oh = 0; oh < hout; ++oh) {
                for (int ow = 0; ow < wout; ++ow) {
                    double t = 0.0;
                    for (int r = 0; r < kh; ++r) {
                        const int ih = oh * stride + r - pad;
                        if (ih < 0 || ih >= h) continue;       /* outside the image: X~ = 0 */
                        for (int q = 0; q < kw; ++q) {
                            const int iw = ow * stride + q - pad;
                            if (iw < 0 || iw >= wd) continue;
                            const float wv = w[((long)c * kh + r) * kw + q];
                            if (wv == 0.0f) continue;
                            t += (double)wv * (double)xp[(long)ih * wd + iw];
                        }
                    }
                    if (bias) t += (double)bias[c];
                    if (relu && !(t > 0.0)) t = 0.0;
                    yp[(long)oh * wout + ow] = t;
                }
            }
        }
    }
    return 0;
}

/* Fully connected layer: y[n][cout] = act(sum_i w[o][i] * x[n][i] + bias[o]). */
int oracle_fc(const float* x, const float* w, const float* bias, double* y, int n, int cin,
              int cout, int relu) {
    if (!x || !w || !y || n <= 0 || cin <= 0 || cout <= 0) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int in = 0; in < n; ++in) {
        for (int o = 0; o < cout; ++o) {
            double acc = 0.0;
            const float* wr = w + (long)o * cin;
            const float* xr = x + (long)in * cin;
            for (int i = 0; i < cin; ++i) {
                if (wr[i] == 0.0f) continue;
                acc += (double)wr[i] * (double)xr[i];
            }
            if (bias) acc += (double)bias[o];
            if (relu && !(acc > 0.0)) acc = 0.0;
            y[(long)in * cout + o] = acc;
        }
    }
    return 0;
}

/* Max pooling over the in-image part of each window (padding never wins). */
int oracle_maxpool(const float* x, double* y, int n, int c, int h, int wd, int k, int stride,
                   int pad) {
    if (!x || !y || n <= 0 || c <= 0 || h <= 0 || wd <= 0 || k <= 0 || stride <= 0 || pad < 0)
        return -1;
    const int hout = out_size(h, k, stride, pad), wout = out_size(wd, k, stride, pad);
    if (hout <= 0 || wout <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (long nc = 0; nc < (long)n * c; ++nc) {
        const float* xp = x + nc * h * wd;
        double* yp = y + nc * hout * wout;
        for (int oh = 0; oh < hout; ++oh)
            for (int ow = 0; ow < wout; ++ow) {
                int seen = 0;
                double m = 0.0;
                for (int r = 0; r < k; ++r)
                    for (int q = 0; q < k; ++q) {
                        const int ih = oh * stride + r - pad, iw = ow * stride + q - pad;
                        if (ih < 0 || ih >= h || iw < 0 || iw >= wd) continue;
                        const double v = (double)xp[(long)ih * wd + iw];
                        if (!seen || v > m) m = v;
                        seen = 1;
                    }
                yp[(long)oh * wout + ow] = m;   /* a window with no in-image element gives 0 */
            }
    }
    return 0;
}

/* Windowed average pooling (the 3x3 / stride 1 / padding 1 pools inside Inception-V3's
 * modules): the mean over the in-image part of each k x k window, i.e. padding is neither
 * summed nor counted.  A window with no in-image element gives 0. */
int oracle_avgpool(const float* x, double* y, int n, int c, int h, int wd, int k, int stride,
                   int pad) {
    if (!x || !y || n <= 0 || c <= 0 || h <= 0 || wd <= 0 || k <= 0 || stride <= 0 || pad < 0)
        return -1;
    const int hout = out_size(h, k, stride, pad), wout = out_size(wd, k, stride, pad);
    if (hout <= 0 || wout <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (long nc = 0; nc < (long)n * c; ++nc) {
        const float* xp = x + nc * h * wd;
        double* yp = y + nc * hout * wout;
        for (int oh = 0; oh < hout; ++oh)
            for (int ow = 0; ow < wout; ++ow) {
                int count = 0;
                double sum = 0.0;
                for (int r = 0; r < k; ++r)
                    for (int q = 0; q < k; ++q) {
                        const int ih = oh * stride + r - pad, iw = ow * stride + q - pad;
                        if (ih < 0 || ih >= h || iw < 0 || iw >= wd) continue;
                        sum += (double)xp[(long)ih * wd + iw];
                        ++count;
                    }
                yp[(long)oh * wout + ow] = count ? sum / (double)count : 0.0;
            }
    }
    return 0;
}

/* Global average pool: y[n][c] = mean over h*w. */
int oracle_global_avgpool(const float* x, double* y, int n, int c, int h, int wd) {
    if (!x || !y || n <= 0 || c <= 0 || h <= 0 || wd <= 0) return -1;
    const long hw = (long)h * wd;
    for (long nc = 0; nc < (long)n * c; ++nc) {
        double s = 0.0;
        for (long i = 0; i < hw; ++i) s += (double)x[nc * hw + i];
        y[nc] = s / (double)hw;
    }
    return 0;
}
