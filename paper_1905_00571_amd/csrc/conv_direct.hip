// Staging-free sparse convolution for gfx950 (wave64).
//
// Lanes of a wave are consecutive flattened output pixels q = oh*wout + ow of one image.
// A wave walks the nonzeros of its packed rows; the weight and its input channel are
// wave-uniform (scalar loads, scalar FMA operand: a filter element is loaded once per wave,
// the paper's redundant filter-load elimination of Section 4), and the activation is read
// with ONE buffer load whose address is
//     base(image) + soffset(channel, uniform) + voffset(lane, tap).
// The per-lane voffset of every filter tap is computed once and kept in a register; taps
// that fall outside the image get an offset beyond the buffer's size, which the hardware
// range check turns into a zero (the implicit zero padding), so no bounds test or select
// is executed per nonzero.  To keep the tap offset a fixed register the plan regroups each
// row's nonzeros tap-major.  1x1 convolutions are the one-tap case of the same kernel: a
// sparse-matrix x dense-matrix product (Section 4: 1x1 convolution as matrix multiply).
//
// KS waves may split a row's input channels; their partial sums meet in LDS before the
// fused bias / residual / ReLU epilogue.
#include "internal.h"

namespace cadnn {

constexpr int kDirectUnroll = 4;
constexpr uint32_t kOutOfRange = 0x7ffffff0u;   // beyond any buffer this library accepts

template <typename T_, int KH_, int KW_, int P_, int RPW_, int KS_, int NW_>
struct DirectCfg {
    using T = T_;
    static constexpr int KH = KH_, KW = KW_, P = P_, RPW = RPW_, KS = KS_, NW = NW_;
    static constexpr int TAPS = KH * KW;
    static constexpr int RG = NW / KS;          // row slots per workgroup
    static constexpr int THREADS = NW * 64;
    static_assert(NW % KS == 0, "KS must divide the waves of a workgroup");
};

template <typename T>
__device__ __forceinline__ float load_act(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff);

template <>
__device__ __forceinline__ float load_act<float>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
}
template <>
__device__ __forceinline__ float load_act<_Float16>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    const unsigned short h = __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
    return (float)__builtin_bit_cast(_Float16, h);
}

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void sconv_direct_kernel(const ConvLaunch a) {
    using T = typename Cfg::T;
    constexpr int KW = Cfg::KW, P = Cfg::P, RPW = Cfg::RPW, KS = Cfg::KS, TAPS = Cfg::TAPS,
                  RG = Cfg::RG, U = kDirectUnroll;
    __shared__ float red[KS > 1 ? Cfg::NW * RPW * P * 64 : 1];

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rg = wv / KS, ks = wv % KS;
    const int n = blockIdx.z;
    const int q0 = blockIdx.x * (64 * P);
    const int row0 = (blockIdx.y * RG + rg) * RPW;

    // per-lane byte offset of every tap for each of the lane's pixels
    uint32_t voff[TAPS][P];
    int oh_[P], ow_[P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const int q = q0 + j * 64 + lane;
        const bool qok = q < a.hwout;
        const int oh = q / a.yd.w, ow = q - oh * a.yd.w;
        oh_[j] = oh; ow_[j] = ow;
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            const int ih = oh * a.stride + t / KW - a.pad;
            const int iw = ow * a.stride + t % KW - a.pad;
            const bool ok = qok && ih >= 0 && ih < a.xd.h && iw >= 0 && iw < a.xd.w;
            voff[t][j] = ok ? (uint32_t)(a.xd.origin + ih * a.xd.pitch + iw) * (uint32_t)sizeof(T) : kOutOfRange;
        }
    }

    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const char*)a.x + (size_t)n * a.image_bytes), 0, a.image_bytes, 0x00020000);
    const uint2* __restrict__ nz = a.nz;
    const uint32_t cs = (uint32_t)a.xd.plane * (uint32_t)sizeof(T);

    int co_[RPW];
    float bias_[RPW];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        co_[r] = a.perm[row0 + r];
        bias_[r] = (a.bias && co_[r] >= 0) ? a.bias[co_[r]] : 0.0f;
    }

    float acc[RPW][P];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
#pragma unroll
        for (int j = 0; j < P; ++j) acc[r][j] = 0.0f;
        const int32_t* __restrict__ seg = a.seg_ptr + ((size_t)(row0 + r) * KS + ks) * (TAPS + 1);
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            int i = seg[t];
            const int end = seg[t + 1];
            for (; i < end; i += U) {
                float xv[U][P];
                float wv_[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint2 pr = nz[i + u];
                    wv_[u] = __uint_as_float(pr.x);
                    const uint32_t soff = pr.y * cs;
#pragma unroll
                    for (int j = 0; j < P; ++j) xv[u][j] = load_act<T>(rsrc, voff[t][j], soff);
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int j = 0; j < P; ++j) acc[r][j] = fmaf(wv_[u], xv[u][j], acc[r][j]);
            }
        }
    }

    if (KS > 1) {
        // partial sums of the KS channel slices meet in LDS; slice 0 finishes the row
#pragma unroll
        for (int r = 0; r < RPW; ++r)
#pragma unroll
            for (int j = 0; j < P; ++j) red[((wv * RPW + r) * P + j) * 64 + lane] = acc[r][j];
        __syncthreads();
        if (ks != 0) return;
#pragma unroll
        for (int r = 0; r < RPW; ++r)
#pragma unroll
            for (int j = 0; j < P; ++j) {
                float s = acc[r][j];
#pragma unroll
                for (int k = 1; k < KS; ++k) s += red[(((wv + k) * RPW + r) * P + j) * 64 + lane];
                acc[r][j] = s;
            }
    }

    // ---- fused epilogue: + bias, + residual, ReLU, store at the original channel
    T* __restrict__ y = (T*)a.y + (size_t)n * a.yd.image + a.yd.origin;
    const T* __restrict__ res = a.residual ? (const T*)a.residual + (size_t)n * a.rd.image + a.rd.origin : nullptr;
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int co = co_[r];
        if (co < 0) continue;
        const float b = bias_[r];
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const int q = q0 + j * 64 + lane;
            if (q < a.hwout) {
                float v = acc[r][j] + b;
                if (res) v += (float)res[(size_t)co * a.rd.plane + oh_[j] * a.rd.pitch + ow_[j]];
                if (a.relu) v = v > 0.0f ? v : 0.0f;
                y[(size_t)co * a.yd.plane + oh_[j] * a.yd.pitch + ow_[j]] = (T)v;
            }
        }
    }
}

template <class Cfg>
static hipError_t launch_direct(const ConvLaunch& a, hipStream_t s) {
    dim3 grid((unsigned)a.tiles_x, (unsigned)a.row_groups, (unsigned)a.n);
    dim3 block(Cfg::THREADS);
    CADNN_LAUNCH(sconv_direct_kernel<Cfg>, grid, block, 0, s, a);
    return hipGetLastError();
}

template <class Cfg>
static ConvVariant make_direct(const char* name) {
    ConvVariant v{};
    v.name = name;
    v.family = FAM_DIRECT;
    v.is_f16 = sizeof(typename Cfg::T) == 2;
    v.kh = Cfg::KH; v.kw = Cfg::KW; v.stride = 0;
    v.p = Cfg::P; v.nw = Cfg::NW; v.rpw = Cfg::RPW; v.ks = Cfg::KS;
    v.unroll = kDirectUnroll;
    v.lds_bytes = Cfg::KS > 1 ? (size_t)Cfg::NW * Cfg::RPW * Cfg::P * 64 * 4 : 0;
    v.launch = &launch_direct<Cfg>;
    return v;
}

#define CADNN_DIRECT(T, KH, KW, P, RPW, KS, NW) \
    make_direct<DirectCfg<T, KH, KW, P, RPW, KS, NW>>( \
        "sdirect_" #T "_k" #KH "x" #KW "_p" #P "_r" #RPW "k" #KS "w" #NW)

#define CADNN_DIRECT_SHAPES(T, KH, KW)         \
    CADNN_DIRECT(T, KH, KW, 1, 1, 1, 4),       \
    CADNN_DIRECT(T, KH, KW, 1, 2, 1, 4),       \
    CADNN_DIRECT(T, KH, KW, 1, 4, 1, 4),       \
    CADNN_DIRECT(T, KH, KW, 2, 2, 1, 4),       \
    CADNN_DIRECT(T, KH, KW, 2, 4, 1, 4),       \
    CADNN_DIRECT(T, KH, KW, 4, 4, 1, 4),       \
    CADNN_DIRECT(T, KH, KW, 1, 1, 4, 4),       \
    CADNN_DIRECT(T, KH, KW, 1, 2, 4, 4),       \
    CADNN_DIRECT(T, KH, KW, 1, 1, 8, 8),       \
    CADNN_DIRECT(T, KH, KW, 1, 2, 2, 4)

const std::vector<ConvVariant>& all_direct_variants() {
    static const std::vector<ConvVariant> v = {
        CADNN_DIRECT_SHAPES(float, 3, 3), CADNN_DIRECT_SHAPES(_Float16, 3, 3)};
    return v;
}

}  // namespace cadnn
