// Fused depthwise convolution layer: every channel is filtered by its own KH x KW filter,
// then bias and ReLU are applied, in one kernel (paper Section 4 names depthwise convolution
// + batch-norm + activation of MobileNet-V1 as one fused kernel).
//
// A wave owns one (image, channel) plane and a run of 64 x P output pixels of it, P adjacent
// pixels of one output row per lane, so the channel's filter taps are wave-uniform (scalar
// registers, zero taps skipped with a scalar branch) and each lane keeps a sliding row of
// (P-1)*S + KW inputs in registers that serves all its P outputs.  The layer moves every
// input and output element once and does KH*KW multiply-adds per output: it is bound by the
// launch itself at batch 1 and by memory traffic beyond.
#include "internal.h"

namespace cadnn {

struct DwLaunch {
    const void* x;
    void* y;
    const float* w;       // [channels][kh*kw], zeros where pruned
    const float* bias;    // [channels] or NULL
    TensorDesc xd, yd;
    int n, hout, wout, kh, kw, stride, pad, relu;
    int groups_per_row;   // wout / P
    int groups;           // hout * groups_per_row
    int tiles;            // ceil(groups / 64)
    long long waves;      // n * channels * tiles
};

// KH = KW = 0 selects the run-time filter size (any size, any stride), one pixel per lane.
template <typename T, int KH, int KW, int S, int P, bool HALO>
__global__ __launch_bounds__(256) void dwconv_kernel(DwLaunch a) {
    const int lane = threadIdx.x & 63;
    const long long wid = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4u + (threadIdx.x >> 6)));
    if (wid >= a.waves) return;
    const int tile = (int)(wid % a.tiles);
    const int ch = (int)((wid / a.tiles) % a.xd.c);
    const int img = (int)(wid / ((long long)a.tiles * a.xd.c));
    const int g = tile * 64 + lane;
    if (g >= a.groups) return;
    const int oh = g / a.groups_per_row;
    const int ow0 = (g - oh * a.groups_per_row) * P;
    const T* xp = (const T*)a.x + (size_t)img * a.xd.image + (size_t)ch * a.xd.plane + a.xd.origin;
    T* yp = (T*)a.y + (size_t)img * a.yd.image + (size_t)ch * a.yd.plane + a.yd.origin;
    const int kh = KH ? KH : a.kh, kw = KW ? KW : a.kw, st = KH ? S : a.stride;
    (void)st;
    const float* wt = a.w + (size_t)ch * kh * kw;
    const float b = a.bias ? a.bias[ch] : 0.0f;
    float acc[P];
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p] = 0.0f;
    if constexpr (KH != 0) {
        constexpr int SPAN = (P - 1) * S + KW;
        const int iw0 = ow0 * S - a.pad;
#pragma unroll
        for (int r = 0; r < KH; ++r) {
            const int ih = oh * S + r - a.pad;
            const bool row_ok = HALO || (ih >= 0 && ih < a.xd.h);
            const T* rowp = xp + (ptrdiff_t)ih * a.xd.pitch + iw0;
            float v[SPAN];
#pragma unroll
            for (int j = 0; j < SPAN; ++j) {
                const bool ok = row_ok && (HALO || (iw0 + j >= 0 && iw0 + j < a.xd.w));
                v[j] = ok ? (float)rowp[j] : 0.0f;
            }
#pragma unroll
            for (int q = 0; q < KW; ++q) {
                const float wv = wt[r * KW + q];
                if (wv != 0.0f) {
#pragma unroll
                    for (int p = 0; p < P; ++p) acc[p] = fmaf(wv, v[p * S + q], acc[p]);
                }
            }
        }
    } else {
        for (int r = 0; r < kh; ++r) {
            const int ih = oh * st + r - a.pad;
            if (ih < 0 || ih >= a.xd.h) continue;
            for (int q = 0; q < kw; ++q) {
                const int iw = ow0 * st + q - a.pad;
                const float wv = wt[r * kw + q];
                if (wv != 0.0f && iw >= 0 && iw < a.xd.w)
                    acc[0] = fmaf(wv, (float)xp[(ptrdiff_t)ih * a.xd.pitch + iw], acc[0]);
            }
        }
    }
    T* out = yp + (ptrdiff_t)oh * a.yd.pitch + ow0;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        float v = acc[p] + b;
        if (a.relu) v = v > 0.0f ? v : 0.0f;
        out[p] = (T)v;
    }
}

template <typename T, int KH, int KW, int S, int P, bool HALO>
static hipError_t launch_dw(const DwLaunch& a, hipStream_t s) {
    const long long blocks = (a.waves + 3) / 4;
    CADNN_LAUNCH((dwconv_kernel<T, KH, KW, S, P, HALO>), dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

template <typename T>
static cadnn_status launch_depthwise_t(DwLaunch a, hipStream_t s) {
    // the input's zero halo covers the padding: no bounds tests in the kernel
    const bool halo = a.xd.ph >= a.pad && a.xd.pw >= a.pad;
    const bool fast = a.kh == 3 && a.kw == 3 && (a.stride == 1 || a.stride == 2);
    // four pixels per lane when rows split evenly and there is enough work to keep the
    // chip busy with a quarter of the lanes
    const bool wide = fast && a.wout % 4 == 0 && (long long)a.n * a.xd.c * a.hout * a.wout >= 4ll * 64 * 1024;
    const int P = wide ? 4 : 1;
    a.groups_per_row = a.wout / P;
    a.groups = a.hout * a.groups_per_row;
    a.tiles = (a.groups + 63) / 64;
    a.waves = (long long)a.n * a.xd.c * a.tiles;
    if (a.waves > 0x7fffffffll - 4) return fail(CADNN_EUNSUPPORTED, "depthwise layer too large for one launch");
    hipError_t e;
    if (!fast) e = launch_dw<T, 0, 0, 1, 1, false>(a, s);
    else if (a.stride == 1)
        e = wide ? (halo ? launch_dw<T, 3, 3, 1, 4, true>(a, s) : launch_dw<T, 3, 3, 1, 4, false>(a, s))
                 : (halo ? launch_dw<T, 3, 3, 1, 1, true>(a, s) : launch_dw<T, 3, 3, 1, 1, false>(a, s));
    else
        e = wide ? (halo ? launch_dw<T, 3, 3, 2, 4, true>(a, s) : launch_dw<T, 3, 3, 2, 4, false>(a, s))
                 : (halo ? launch_dw<T, 3, 3, 2, 1, true>(a, s) : launch_dw<T, 3, 3, 2, 1, false>(a, s));
    CADNN_HIP(e);
    return CADNN_OK;
}

cadnn_status launch_depthwise(const cadnn_weights* w, const void* x, const TensorDesc& xd, void* y,
                              const TensorDesc& yd, int n, int stride, int pad, const float* bias, int relu,
                              hipStream_t s) {
    if (xd.s2d || yd.s2d) return fail(CADNN_EUNSUPPORTED, "depthwise layers read and write plain layouts only");
    DwLaunch a{};
    a.x = x; a.y = y; a.w = (const float*)w->d_dw.p; a.bias = bias;
    a.xd = xd; a.yd = yd; a.n = n;
    a.hout = yd.h; a.wout = yd.w; a.kh = w->kh; a.kw = w->kw; a.stride = stride; a.pad = pad; a.relu = relu;
    return w->dtype == CADNN_F16 ? launch_depthwise_t<_Float16>(a, s) : launch_depthwise_t<float>(a, s);
}

}  // namespace cadnn
