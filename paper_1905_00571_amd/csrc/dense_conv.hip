// Dense implicit-GEMM convolution on the matrix cores (MFMA), gfx950.
//
// Y[Cout x pixels] = W[Cout x K] * X~[K x pixels], K = Cin*Kh*Kw, where column q of X~ is
// the (never materialised) im2col window of output pixel q.  Used (a) as the dense
// comparator for the dense-vs-compressed comparison the paper reports (Section 5), and
// (b) as the fallback for layers that are not pruned (the first layer of the benchmark
// nets), where the layer really is a dense contraction.  Same fused epilogue as the sparse
// kernels (Section 4: conv + batch-norm + activation in one kernel).
//
// One workgroup (4 waves, 2 x 2) computes a 64 (channels) x 64 (pixels) tile; each wave
// owns a 32 x 32 sub-tile accumulated by v_mfma_f32_32x32x2_f32 (fp32 storage) or
// v_mfma_f32_32x32x8_f16 (fp16 storage, fp32 accumulate).  K is walked in chunks of 32:
// the weight chunk and the gathered activation chunk are staged in LDS (k fastest, rows
// padded against bank conflicts); global loads of chunk c+1 are issued before the MFMAs of
// chunk c and written to the other LDS buffer afterwards, one barrier per chunk.
#include "internal.h"

namespace cadnn {

namespace {

constexpr int BM = 64, BN = 64, BK = 32;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

struct DenseArgs {
    const void* w;        // [cout][K]
    const void* x;
    void* y;
    const float* bias;
    const void* residual;
    TensorDesc xd, yd, rd;
    int n, cout, K, kh, kw, stride, pad, relu;
    int hwout;
    uint32_t magic_taps, magic_kw;   // ceil(2^32 / d) for d = kh*kw and d = kw
};

template <typename T> struct Mma;
template <> struct Mma<float> {
    static constexpr int KSTEP = 2;      // k values consumed per instruction
    static constexpr int KLANE = 1;      // consecutive k held by one lane
    static constexpr int BKP = BK + 1;   // padded LDS row, in elements
    typedef float Frag;
    static __device__ __forceinline__ Frag load(const float* p) { return *p; }
    static __device__ __forceinline__ f32x16 mma(Frag a, Frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
};
template <> struct Mma<_Float16> {
    static constexpr int KSTEP = 8;
    static constexpr int KLANE = 4;
    static constexpr int BKP = BK + 4;
    typedef f16x4 Frag;
    static __device__ __forceinline__ Frag load(const _Float16* p) { return *(const f16x4*)p; }
    static __device__ __forceinline__ f32x16 mma(Frag a, Frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x8f16(a, b, c, 0, 0, 0);
    }
};

__device__ __forceinline__ uint32_t fast_div(uint32_t v, uint32_t magic) {
    return __umulhi(v, magic);
}

template <typename T>
__global__ __launch_bounds__(256) void dense_conv_kernel(const DenseArgs a) {
    using M = Mma<T>;
    constexpr int BKP = M::BKP;
    __shared__ __attribute__((aligned(16))) T As[2][BM * BKP];
    __shared__ __attribute__((aligned(16))) T Bs[2][BN * BKP];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = tid >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const int m0 = blockIdx.y * BM;
    const int q0 = blockIdx.x * BN;
    const int img = blockIdx.z;
    const int taps = a.kh * a.kw;

    const T* __restrict__ W = (const T*)a.w;
    const T* __restrict__ X = (const T*)a.x + (size_t)img * a.xd.image + a.xd.origin;

    // ---- this thread's share of the two staged chunks
    // weights: k = tid % 32 (contiguous in memory), rows tid/32 + 8*i
    const int a_k = tid & 31, a_m = tid >> 5;
    // activations: pixel tid % 64 (contiguous in memory), k = tid/64 + 4*i
    const int b_n = tid & 63, b_k = tid >> 6;
    const int q = q0 + b_n;
    const bool q_ok = q < a.hwout;
    const int oh = q / a.yd.w, ow = q - oh * a.yd.w;
    const int ih0 = oh * a.stride - a.pad, iw0 = ow * a.stride - a.pad;

    T ra[8], rb[8];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int m = m0 + a_m + 8 * i, k = k0 + a_k;
            ra[i] = (m < a.cout && k < a.K) ? W[(size_t)m * a.K + k] : (T)0.0f;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t k = (uint32_t)(k0 + b_k + 4 * i);
            const uint32_t ci = taps == 1 ? k : fast_div(k, a.magic_taps);
            const uint32_t t = k - ci * (uint32_t)taps;
            const uint32_t r = a.kw == 1 ? t : fast_div(t, a.magic_kw);
            const uint32_t c = t - r * (uint32_t)a.kw;
            const int ih = ih0 + (int)r, iw = iw0 + (int)c;
            const bool ok = q_ok && (int)k < a.K && ih >= 0 && ih < a.xd.h && iw >= 0 && iw < a.xd.w;
            rb[i] = ok ? X[(size_t)ci * a.xd.plane + ih * a.xd.pitch + iw] : (T)0.0f;
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 8; ++i) As[buf][(a_m + 8 * i) * BKP + a_k] = ra[i];
#pragma unroll
        for (int i = 0; i < 8; ++i) Bs[buf][b_n * BKP + b_k + 4 * i] = rb[i];
    };

    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;

    const int nchunks = (a.K + BK - 1) / BK;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < nchunks) fetch((c + 1) * BK);
        const T* ap = &As[buf][(wm * 32 + (lane & 31)) * BKP + (lane >> 5) * M::KLANE];
        const T* bp = &Bs[buf][(wn * 32 + (lane & 31)) * BKP + (lane >> 5) * M::KLANE];
#pragma unroll
        for (int k = 0; k < BK; k += M::KSTEP) acc = M::mma(M::load(ap + k), M::load(bp + k), acc);
        if (c + 1 < nchunks) stash(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds pixel (lane % 32) of 16 channels
    const int qo = q0 + wn * 32 + (lane & 31);
    if (qo >= a.hwout) return;
    const int oho = qo / a.yd.w, owo = qo - oho * a.yd.w;
    T* __restrict__ Y = (T*)a.y + (size_t)img * a.yd.image + a.yd.origin + oho * a.yd.pitch + owo;
    const T* __restrict__ R = a.residual
        ? (const T*)a.residual + (size_t)img * a.rd.image + a.rd.origin + oho * a.rd.pitch + owo : nullptr;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int co = m0 + wm * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (co >= a.cout) continue;
        float val = acc[v] + (a.bias ? a.bias[co] : 0.0f);
        if (R) val += (float)R[(size_t)co * a.rd.plane];
        if (a.relu) val = val > 0.0f ? val : 0.0f;
        Y[(size_t)co * a.yd.plane] = (T)val;
    }
}

// floor(v / d) == umulhi(v, ceil(2^32 / d)) for v * d < 2^32 (d = 1 is special-cased)
uint32_t magic_for(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((0x100000000ull + d - 1) / d); }

hipError_t launch_dense_variant(const ConvLaunch& l, hipStream_t s);

}  // namespace

const std::vector<ConvVariant>& all_dense_variants() {
    static const std::vector<ConvVariant> v = [] {
        std::vector<ConvVariant> out;
        for (int f16 = 0; f16 < 2; ++f16) {
            ConvVariant d{};
            d.name = f16 ? "dense_mfma__Float16_64x64x32" : "dense_mfma_float_64x64x32";
            d.family = FAM_DENSE;
            d.is_f16 = f16 != 0;
            d.nw = 4; d.rpw = 16; d.ks = 1; d.p = 1; d.unroll = 1;
            d.launch = &launch_dense_variant;
            out.push_back(d);
        }
        return out;
    }();
    return v;
}

// w: device [cout][cin*kh*kw] in the activation storage type.
cadnn_status dense_conv2d_desc(const void* w_dev, const void* x, const TensorDesc& xd, void* y,
                               const TensorDesc& yd, const void* residual, const TensorDesc& rd, int n,
                               int cout, int kh, int kw, int stride, int pad, const void* bias, int relu,
                               cadnn_dtype dtype, hipStream_t s) {
    DenseArgs a{};
    a.w = w_dev; a.x = x; a.y = y; a.bias = (const float*)bias; a.residual = residual;
    a.xd = xd; a.yd = yd; a.rd = rd;
    a.n = n; a.cout = cout; a.K = xd.c * kh * kw; a.kh = kh; a.kw = kw; a.stride = stride; a.pad = pad;
    a.relu = relu ? 1 : 0;
    a.hwout = yd.h * yd.w;
    a.magic_taps = magic_for((uint32_t)(kh * kw));
    a.magic_kw = magic_for((uint32_t)kw);
    dim3 grid((unsigned)((a.hwout + BN - 1) / BN), (unsigned)((cout + BM - 1) / BM), (unsigned)n);
    if (dtype == CADNN_F16)
        CADNN_LAUNCH(dense_conv_kernel<_Float16>, grid, dim3(256), 0, s, a);
    else
        CADNN_LAUNCH(dense_conv_kernel<float>, grid, dim3(256), 0, s, a);
    CADNN_HIP(hipGetLastError());
    return CADNN_OK;
}

namespace {
hipError_t launch_dense_variant(const ConvLaunch& l, hipStream_t s) {
    const cadnn_status st = dense_conv2d_desc(l.nz, l.x, l.xd, l.y, l.yd, l.residual, l.rd, l.n, l.cout, l.kh,
                                              l.kw, l.stride, l.pad, l.bias, l.relu,
                                              l.is_f16 ? CADNN_F16 : CADNN_F32, s);
    return st == CADNN_OK ? hipSuccess : hipErrorLaunchFailure;
}
}  // namespace

cadnn_status dense_conv2d_impl(const void* w_dev, const void* x, void* y, int n, int cin, int h, int wdt,
                               int cout, int kh, int kw, int stride, int pad, const void* bias,
                               const void* residual, int relu, cadnn_dtype dtype, hipStream_t s) {
    if (!w_dev || !x || !y) return fail(CADNN_EINVAL, "cadnn_dense_conv2d: NULL tensor");
    if (n <= 0 || cin <= 0 || h <= 0 || wdt <= 0 || cout <= 0 || kh <= 0 || kw <= 0)
        return fail(CADNN_EINVAL, "cadnn_dense_conv2d: non-positive size");
    if (stride <= 0 || pad < 0) return fail(CADNN_EINVAL, "cadnn_dense_conv2d: bad stride/pad");
    if (dtype != CADNN_F32 && dtype != CADNN_F16) return fail(CADNN_EINVAL, "cadnn_dense_conv2d: dtype");
    const int hout = conv_out(h, kh, stride, pad), wout = conv_out(wdt, kw, stride, pad);
    if (hout <= 0 || wout <= 0) return fail(CADNN_EINVAL, "cadnn_dense_conv2d: empty output");
    if (x == y) return fail(CADNN_EINVAL, "cadnn_dense_conv2d: y aliases x");
    if (n > 65535 || (cout + BM - 1) / BM > 65535) return fail(CADNN_EUNSUPPORTED, "cadnn_dense_conv2d: too large");
    if ((int64_t)cin * kh * kw > (1 << 24)) return fail(CADNN_EUNSUPPORTED, "cadnn_dense_conv2d: cin*kh*kw above 2^24");
    const TensorDesc yd = make_desc(cout, hout, wout);
    const int64_t elem = dtype == CADNN_F16 ? 2 : 4;
    // (the kernel addresses one image with 32-bit element offsets)
    if (desc_too_large(make_desc(cin, h, wdt)) || desc_too_large(yd) || (int64_t)cin * h * wdt * elem >= 0x7ffffff0ll ||
        yd.image * elem >= 0x7ffffff0ll)
        return fail(CADNN_EUNSUPPORTED, "cadnn_dense_conv2d: one image of a tensor is 2 GiB or more");
    // fp16 storage with whole 32-channel steps takes the 128 x 128-tile kernel
    if (cin % 32 == 0 && dense_wide_serves(dtype == CADNN_F16, cin, kh * kw, (int64_t)cin * h * wdt * elem * n, yd.image * elem * n,
                          (int64_t)n * hout * wout))
        return dense_wide_conv2d_raw(w_dev, x, make_desc(cin, h, wdt), y, yd, residual, yd, n, cout, kh, kw, stride, pad,
                                     bias, relu, s);
    return dense_conv2d_desc(w_dev, x, make_desc(cin, h, wdt), y, yd, residual, yd, n, cout, kh, kw, stride,
                             pad, bias, relu, dtype, s);
}

}  // namespace cadnn

extern "C" cadnn_status cadnn_dense_conv2d(const void* w_dev, const void* x, void* y, int n, int cin,
                                           int h, int wdt, int cout, int kh, int kw, int stride,
                                           int pad, const void* bias, const void* residual, int relu,
                                           cadnn_dtype dtype, void* stream) {
    return cadnn::dense_conv2d_impl(w_dev, x, y, n, cin, h, wdt, cout, kh, kw, stride, pad, bias,
                                    residual, relu, dtype, (hipStream_t)stream);
}
