// LDS-tiled sparse convolution for gfx950 (wave64).
//
// One workgroup computes a TW x TH tile of output pixels for G = NW*RPW packed rows
// (output channels, in the nnz-sorted order of the compact format).  Lanes of a wave are
// output pixels, so a nonzero weight and the tile offset of its tap are wave-uniform: they
// are fetched with scalar loads and the weight feeds the FMAs as a scalar operand, i.e. a
// filter element is loaded once per wave and reused for all of its pixels (the paper's
// redundant filter-load elimination, Section 4, mapped onto SGPR broadcast).  The input
// tile with its halo is staged once per channel chunk in LDS (zero-filled outside the
// image) and reused by every row of the group; bias, residual add and ReLU are fused in the
// epilogue (Section 4: conv + batch-norm + activation as one kernel).
//
// Strided layers: the staged tile is de-interleaved by the stride in both directions
// ("phases"), so that the lanes of a wave always read consecutive LDS words whatever the
// stride, and taps that a strided 1x1 filter never touches are not staged at all.
#include "internal.h"

namespace cadnn {

constexpr int kUnroll = 4;

constexpr int cmin(int a, int b) { return a < b ? a : b; }

// Smallest LDS row pitch >= need for which the lane rows that are read in the same
// 32-lane pass fall into disjoint bank windows (32 banks of 4 bytes).  Falls back to
// `need` when no pitch within one bank period achieves it.
constexpr int pick_pitch(int need, int tw) {
    if (tw >= 32) return need;
    const int rows = 32 / tw;
    for (int p = need; p < need + 32; ++p) {
        bool ok = true;
        for (int i = 0; i < rows && ok; ++i)
            for (int j = i + 1; j < rows && ok; ++j) {
                const int a = (i * p) % 32, b = (j * p) % 32;
                const int d = a > b ? a - b : b - a;
                if (d < tw || 32 - d < tw) ok = false;
            }
        if (ok) return p;
    }
    return need;
}

template <typename T_, int KH_, int KW_, int S_, int TW_, int P_, int NW_, int RPW_, int CCH_>
struct TileCfg {
    using T = T_;
    static constexpr int KH = KH_, KW = KW_, S = S_, TW = TW_, P = P_, NW = NW_, RPW = RPW_,
                         CCH = CCH_;
    static constexpr int RW = 64 / TW;          // lane rows per wave
    static constexpr int TH = RW * P;           // output rows per tile
    static constexpr int NRPH = cmin(S, KH);    // row phases staged
    static constexpr int RH = TH + (KH - 1) / S;
    static constexpr int NPH = cmin(S, KW);     // column phases staged
    static constexpr int CW = TW + (KW - 1) / S;
    static constexpr int PITCH = pick_pitch(NPH * CW, TW);
    static constexpr int PLANE = NRPH * RH * PITCH;
    static constexpr int THREADS = NW * 64;
    static constexpr size_t LDS_BYTES = (size_t)CCH * PLANE * sizeof(float);
    static_assert(64 % TW == 0, "TW must divide the wavefront");
    static_assert(LDS_BYTES <= 64 * 1024, "static LDS tile above 64 KiB");
};

template <typename T>
__device__ __forceinline__ float to_f32(T v) { return (float)v; }

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void sconv_tile_kernel(const ConvLaunch a) {
    using T = typename Cfg::T;
    constexpr int S = Cfg::S, TW = Cfg::TW, P = Cfg::P, NW = Cfg::NW, RPW = Cfg::RPW,
                  CCH = Cfg::CCH, RW = Cfg::RW, TH = Cfg::TH, RH = Cfg::RH, NPH = Cfg::NPH,
                  CW = Cfg::CW, PITCH = Cfg::PITCH, PLANE = Cfg::PLANE, U = kUnroll;
    constexpr int TOTAL = CCH * PLANE;
    constexpr int NIT = (TOTAL + Cfg::THREADS - 1) / Cfg::THREADS;   // staging passes per chunk
    constexpr int SB = NIT < 16 ? NIT : 16;                          // loads kept in flight
    __shared__ float lds[TOTAL];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tx = lane % TW, ty = lane / TW;
    const int tile_x = blockIdx.x % a.tiles_x, tile_y = blockIdx.x / a.tiles_x;
    const int n = blockIdx.z;
    const int oh0 = tile_y * TH, ow0 = tile_x * TW;
    const int ih0 = oh0 * S - a.pad, iw0 = ow0 * S - a.pad;
    const int row0 = (blockIdx.y * NW + wv) * RPW;
    const int cin = a.xd.c, h = a.xd.h, w = a.xd.w;

    const T* __restrict__ xn = (const T*)a.x + (size_t)n * a.xd.image + a.xd.origin;
    const uint2* __restrict__ nz = a.nz;
    const int32_t* __restrict__ seg = a.seg_ptr + (size_t)row0 * (a.nchunks + 1);

    float acc[RPW][P];
#pragma unroll
    for (int r = 0; r < RPW; ++r)
#pragma unroll
        for (int j = 0; j < P; ++j) acc[r][j] = 0.0f;

    const char* lane_ptr = (const char*)lds + (ty * PITCH + tx) * (int)sizeof(float);

    for (int c = 0; c < a.nchunks; ++c) {
        if (c) __syncthreads();
        // ---- stage CCH channels of the input tile (+halo), zero-filled outside the image;
        //      SB loads are issued before the first of them is stored
        const int c0 = c * CCH;
#pragma unroll
        for (int it0 = 0; it0 < NIT; it0 += SB) {
            float v[SB];
#pragma unroll
            for (int k = 0; k < SB; ++k) {
                const int e = tid + (it0 + k) * Cfg::THREADS;
                const int ch = e / PLANE;
                const int rem = e - ch * PLANE;
                const int rr = rem / PITCH;
                const int cc = rem - rr * PITCH;
                const int rph = rr / RH, ri = rr - rph * RH;
                const int cph = cc / CW, cj = cc - cph * CW;
                const int ci = c0 + ch;
                const int ih = ih0 + ri * S + rph;
                const int iw = iw0 + cj * S + cph;
                v[k] = 0.0f;
                if (it0 + k < NIT && e < TOTAL && cph < NPH && ci < cin && ih >= 0 && ih < h && iw >= 0 && iw < w)
                    v[k] = to_f32(xn[(size_t)ci * a.xd.plane + ih * a.xd.pitch + iw]);
            }
#pragma unroll
            for (int k = 0; k < SB; ++k) {
                const int e = tid + (it0 + k) * Cfg::THREADS;
                if (it0 + k < NIT && e < TOTAL) lds[e] = v[k];
            }
        }
        __syncthreads();
        // ---- stream this chunk's nonzeros of each of the wave's rows; the next group of
        //      (value, offset) pairs is fetched while the current one is consumed
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            int i = seg[r * (a.nchunks + 1) + c];
            const int end = seg[r * (a.nchunks + 1) + c + 1];
            if (i >= end) continue;
            uint2 cur[U];
#pragma unroll
            for (int u = 0; u < U; ++u) cur[u] = nz[i + u];
            for (i += U; i < end; i += U) {
                uint2 nxt[U];
#pragma unroll
                for (int u = 0; u < U; ++u) nxt[u] = nz[i + u];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float wval = __uint_as_float(cur[u].x);
                    const char* lp = lane_ptr + cur[u].y;
#pragma unroll
                    for (int j = 0; j < P; ++j)
                        acc[r][j] = fmaf(wval, *(const float*)(lp + j * RW * PITCH * (int)sizeof(float)),
                                         acc[r][j]);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) cur[u] = nxt[u];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float wval = __uint_as_float(cur[u].x);
                const char* lp = lane_ptr + cur[u].y;
#pragma unroll
                for (int j = 0; j < P; ++j)
                    acc[r][j] = fmaf(wval, *(const float*)(lp + j * RW * PITCH * (int)sizeof(float)),
                                     acc[r][j]);
            }
        }
    }

    // ---- fused epilogue: + bias, + residual, ReLU, store at the original channel
    const int ow = ow0 + tx;
    T* __restrict__ y = (T*)a.y + (size_t)n * a.yd.image + a.yd.origin;
    const T* __restrict__ res = a.residual ? (const T*)a.residual + (size_t)n * a.rd.image + a.rd.origin : nullptr;
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int co = a.perm[row0 + r];
        if (co < 0) continue;
        const float b = a.bias ? a.bias[co] : 0.0f;
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const int oh = oh0 + ty + j * RW;
            if (oh < a.yd.h && ow < a.yd.w) {
                float v = acc[r][j] + b;
                if (res) v += to_f32(res[(size_t)co * a.rd.plane + oh * a.rd.pitch + ow]);
                if (a.relu) v = v > 0.0f ? v : 0.0f;
                y[(size_t)co * a.yd.plane + oh * a.yd.pitch + ow] = (T)v;
            }
        }
    }
}

template <class Cfg>
static hipError_t launch_tile(const ConvLaunch& a, hipStream_t s) {
    dim3 grid((unsigned)(a.tiles_x * a.tiles_y), (unsigned)a.row_groups, (unsigned)a.n);
    dim3 block(Cfg::THREADS);
    CADNN_LAUNCH(sconv_tile_kernel<Cfg>, grid, block, 0, s, a);
    return hipGetLastError();
}

template <class Cfg>
static ConvVariant make_variant(const char* name) {
    ConvVariant v{};
    v.name = name;
    v.family = FAM_TILE;
    v.ks = 1;
    v.kh = Cfg::KH; v.kw = Cfg::KW; v.stride = Cfg::S;
    v.tw = Cfg::TW; v.rw = Cfg::RW; v.p = Cfg::P;
    v.nw = Cfg::NW; v.rpw = Cfg::RPW; v.cch = Cfg::CCH;
    v.th = Cfg::TH; v.rh = Cfg::RH; v.nrph = Cfg::NRPH; v.cw = Cfg::CW; v.nph = Cfg::NPH;
    v.pitch = Cfg::PITCH; v.plane = Cfg::PLANE;
    v.unroll = kUnroll;
    v.lds_bytes = Cfg::LDS_BYTES;
    v.elem_bytes = 4;   // the staged tile is fp32 whatever the storage type
    v.is_f16 = sizeof(typename Cfg::T) == 2;
    v.launch = &launch_tile<Cfg>;
    return v;
}

#define CADNN_VARIANT(T, KH, KW, S, TW, P, NW, RPW, CCH) \
    make_variant<TileCfg<T, KH, KW, S, TW, P, NW, RPW, CCH>>( \
        "sconv_" #T "_k" #KH "x" #KW "s" #S "_t" #TW "p" #P "_w" #NW "r" #RPW "c" #CCH)

#define CADNN_SHAPES(T)                                     \
    /* 3x3 */                                               \
    CADNN_VARIANT(T, 3, 3, 1, 32, 4, 4, 4, 32),             \
    CADNN_VARIANT(T, 3, 3, 1, 16, 2, 4, 4, 32),             \
    CADNN_VARIANT(T, 3, 3, 1, 8, 1, 4, 4, 64),              \
    CADNN_VARIANT(T, 3, 3, 2, 32, 2, 4, 4, 16),             \
    CADNN_VARIANT(T, 3, 3, 2, 16, 2, 4, 4, 16),             \
    CADNN_VARIANT(T, 3, 3, 2, 8, 1, 4, 4, 32),              \
    /* 1x1 */                                               \
    CADNN_VARIANT(T, 1, 1, 1, 32, 4, 4, 4, 64),             \
    CADNN_VARIANT(T, 1, 1, 1, 16, 2, 4, 4, 128),            \
    CADNN_VARIANT(T, 1, 1, 1, 8, 1, 4, 4, 256),             \
    CADNN_VARIANT(T, 1, 1, 2, 32, 2, 4, 4, 64),             \
    CADNN_VARIANT(T, 1, 1, 2, 16, 2, 4, 4, 128),            \
    CADNN_VARIANT(T, 1, 1, 2, 8, 1, 4, 4, 256),             \
    /* 7x7 */                                               \
    CADNN_VARIANT(T, 7, 7, 2, 32, 4, 4, 4, 3),              \
    CADNN_VARIANT(T, 7, 7, 2, 8, 1, 4, 4, 8),               \
    CADNN_VARIANT(T, 7, 7, 1, 32, 2, 4, 4, 4),              \
    CADNN_VARIANT(T, 7, 7, 1, 8, 1, 4, 4, 8)

const std::vector<ConvVariant>& all_tile_variants() {
    static const std::vector<ConvVariant> v = {CADNN_SHAPES(float), CADNN_SHAPES(_Float16)};
    return v;
}

}  // namespace cadnn
