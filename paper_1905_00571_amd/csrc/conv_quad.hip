// Linear-address sparse convolution for small images: four filter rows per wavefront (gfx950).
//
// On the last stage of a network an image has a few dozen pixels (7 x 7, 8 x 8) and a layer
// hundreds of thousands of nonzeros: with the pixels of ONE output channel as the lanes of a
// wave, most lanes idle, and every nonzero still costs the wave its own broadcast, address, load
// and multiply-add -- a chain of dependent instructions per nonzero (Section 4 of the paper
// counts loads per nonzero; here it is instructions per nonzero that bound the layer).  This
// kernel gives each quarter of a wave (16 lanes) its own packed row: a lane holds 4 adjacent
// pixels of one image row, 16 lanes cover an image of up to 16 such groups, and one pass of the
// loop -- one 16-byte load, four multiply-adds -- serves four nonzeros, one of each row.  (Or
// each half of a wave, with 2 pixels per lane: two rows per wave, twice the workgroups.)
//
// The stream is the linear-address plan (parts of KS waves per row at a fixed stride, headers
// {padded length, channel}); the four rows of a wave are walked in lock step up to the longest
// of them, the shorter ones running on into padding entries whose offset lies outside every
// buffer (they load zero).  A window of 16 entries per row arrives with one coalesced load and
// is handed to the row's lanes through a slot of LDS of the wave's own.  KS waves
// split every row's nonzeros; partial sums meet in LDS before the fused epilogue (Section 4:
// bias, residual, ReLU).  Addresses are those of the linear family: the input's zero halo covers
// the padding, a stride-2 layer reads a de-interleaved input as a plain view with unit stride.
#include <type_traits>

#include "internal.h"

namespace cadnn {

namespace {

typedef uint32_t u32x2q __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4q __attribute__((ext_vector_type(4)));

template <int I, int N, class F>
__device__ __forceinline__ void quad_static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>());
        quad_static_for<I + 1, N>(f);
    }
}

// R: packed rows per wave (4: quarters of 16 lanes with 4 adjacent pixels per lane; 2: halves of
//    32 lanes with 2 pixels per lane -- twice the workgroups for the same layer, which is what a
//    layer of a few hundred rows needs to reach every CU: the kernel is bound by the bytes the
//    activation loads move through the vector caches, 256 per nonzero, on the CUs that run it).
// B: nonzeros per row whose activations are requested in one go; two such sets take turns, so
//    2 B loads are in flight per lane.
template <typename T_, int R_, int KS_, int RG_, int B_>
struct QuadCfg {
    using T = T_;
    static constexpr int R = R_, KS = KS_, RG = RG_, B = B_, NW = KS_ * RG_, THREADS = NW * 64;
    static constexpr int WIN = 64 / R;          // lanes per row = entries per window of the stream
    static constexpr int PX = R == 4 ? 4 : 2;   // adjacent pixels per lane
    static constexpr int RD = 64 / WIN;         // windows in flight: 64 entries ahead
    static_assert(THREADS <= 1024 && (R == 2 || R == 4) && WIN % B == 0 && (RD * (WIN / B)) % 2 == 0, "shape");
};

// the activations of one nonzero for a lane's PX pixels, as loaded
template <typename T, int PX>
struct QuadX {
    uint32_t v[PX * (int)sizeof(T) / 4];
};

template <typename T, int PX>
__device__ __forceinline__ void quad_load(__amdgpu_buffer_rsrc_t r, uint32_t voff, QuadX<T, PX>& x) {
    constexpr int words = PX * (int)sizeof(T) / 4;
    if constexpr (words == 4) {
        const u32x4q v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, 0u, 0);
        x.v[0] = v[0]; x.v[1] = v[1]; x.v[2] = v[2]; x.v[3] = v[3];
    } else if constexpr (words == 2) {
        const u32x2q v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, 0u, 0);
        x.v[0] = v[0]; x.v[1] = v[1];
    } else {
        x.v[0] = __builtin_amdgcn_raw_buffer_load_b32(r, voff, 0u, 0);
    }
}

// acc + w * (low / high half of xh as binary16), product and sum in fp32: what a conversion
// followed by an fp32 FMA computes, bit for bit (w is a per-lane value here)
__device__ __forceinline__ float quad_mix_lo(float w, uint32_t xh, float acc) {
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[0,1,0]" : "=v"(d) : "v"(w), "v"(xh), "v"(acc));
    return d;
}
__device__ __forceinline__ float quad_mix_hi(float w, uint32_t xh, float acc) {
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,1,0] op_sel_hi:[0,1,0]" : "=v"(d) : "v"(w), "v"(xh), "v"(acc));
    return d;
}

template <typename T, int PX>
__device__ __forceinline__ void quad_mac(float w, const QuadX<T, PX>& x, float (&acc)[PX]) {
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int j = 0; j < PX; ++j) acc[j] = fmaf(w, __uint_as_float(x.v[j]), acc[j]);
    } else {
#pragma unroll
        for (int j = 0; j < PX / 2; ++j) {
            acc[2 * j] = quad_mix_lo(w, x.v[j], acc[2 * j]);
            acc[2 * j + 1] = quad_mix_hi(w, x.v[j], acc[2 * j + 1]);
        }
    }
}

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void sconv_quad_kernel(const ConvLaunch a) {
    using T = typename Cfg::T;
    constexpr int R = Cfg::R, KS = Cfg::KS, RG = Cfg::RG, B = Cfg::B, WIN = Cfg::WIN, PX = Cfg::PX, RD = Cfg::RD;
    __shared__ float red[KS > 1 ? Cfg::NW * PX * 64 : 1];
    __shared__ uint2 handoff[Cfg::NW][2][64];       // a wave's current window (and the one before)

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rg = wv / KS, ks = wv % KS;
    const int sub = lane / WIN, sl = lane % WIN;                // which of the wave's rows, lane within it
    const int n = (int)blockIdx.z;
    const int row = ((int)blockIdx.y * RG + rg) * R + sub;      // this lane's packed row

    // the lane's PX pixels: group sl of the image, groups enumerated over rows of wq = width
    // rounded up to PX positions (a group never straddles two rows; positions past a row's end
    // are computed and not stored)
    const int lpr = a.wq / PX;
    const int oh = sl / lpr, ow0 = (sl - oh * lpr) * PX;
    const bool live = oh < a.yd.h;
    const int base = a.xd.origin - a.pad * a.xd.pitch - a.pad;
    const uint32_t voff = live ? (uint32_t)(base + oh * a.stride * a.xd.pitch + ow0 * a.stride) * (uint32_t)sizeof(T)
                               : kPlanOutOfRange;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const char*)a.x + (size_t)n * a.image_bytes), 0, a.image_bytes, 0x00020000);

    // the part of the stream this wave walks for the lane's row, and its header
    const int part = row * KS + ks;
    const uint2* __restrict__ ent = a.nz + (size_t)part * a.nchunks;
    // Windows of the stream 64 entries ahead are in flight (it comes from memory); the
    // activations, which the caches hold, run one set ahead.
    // (The stream ends in spare entries: the windows requested past the last are in bounds.)
    uint2 ring[RD];
#pragma unroll
    for (int i = 0; i < RD; ++i) ring[i] = ent[WIN * i + sl];
    const int2 h = ((const int2*)a.seg_ptr)[part];
    const int co = h.y;
    int longest = h.x;
    if constexpr (R == 4) longest = max(longest, __shfl_xor(longest, 16, 64));
    longest = max(longest, __shfl_xor(longest, 32, 64));
    longest = __builtin_amdgcn_readfirstlane(longest);
    const float bias = (a.bias && co >= 0) ? a.bias[co] : 0.0f;

    float acc[PX];
#pragma unroll
    for (int j = 0; j < PX; ++j) acc[j] = 0.0f;
    // A window (lane l of a row's lanes holds entry l of the row) goes through LDS to the lanes
    // that need it: entries u0 .. u0 + B - 1 are read back one by one, all lanes of a row
    // reading the same 8 bytes -- (value, offset) of their own row in ONE broadcast read -- and
    // the activations are requested.  (The wave's own slot: no barrier, LDS keeps a wave's
    // accesses in order.)
    auto stage = [&](int slot, const uint2& win) __attribute__((always_inline)) { handoff[wv][slot][lane] = win; };
    auto fetch = [&](int slot, int u0, float (&w)[B], QuadX<T, PX> (&x)[B]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < B; ++u) {
            const uint2 e = handoff[wv][slot][sub * WIN + u0 + u];
            w[u] = __uint_as_float(e.x);
            quad_load<T, PX>(rsrc, voff + e.y, x[u]);
        }
    };
    auto mac = [&](const float (&w)[B], const QuadX<T, PX> (&x)[B]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < B; ++u) quad_mac<T, PX>(w[u], x[u], acc);
    };
    float wa[B], wb[B];
    QuadX<T, PX> xa[B], xb[B];
    if (longest > 0) {
        constexpr int SPW = WIN / B;      // sets per window; set number q uses registers q % 2
        stage(0, ring[0]);
        fetch(0, 0, wa, xa);
        for (int k0 = 0; k0 < longest; k0 += RD * WIN) {
            quad_static_for<0, RD>([&](auto I) {
                constexpr int i = decltype(I)::value;
                if (k0 + WIN * i < longest) {
                    const bool more = k0 + WIN * (i + 1) < longest;
                    quad_static_for<0, SPW>([&](auto H) {
                        constexpr int hh = decltype(H)::value;
                        constexpr bool odd = ((i * SPW + hh) & 1) != 0;
                        // the next set is requested into the other registers, then this one is used
                        if constexpr (hh + 1 < SPW) {
                            if constexpr (odd) fetch(i & 1, (hh + 1) * B, wa, xa);
                            else fetch(i & 1, (hh + 1) * B, wb, xb);
                        } else {
                            if (more) {
                                stage((i + 1) & 1, ring[(i + 1) % RD]);
                                if constexpr (odd) fetch((i + 1) & 1, 0, wa, xa);
                                else fetch((i + 1) & 1, 0, wb, xb);
                            }
                        }
                        if constexpr (odd) mac(wb, xb);
                        else mac(wa, xa);
                    });
                    ring[i] = ent[k0 + RD * WIN + WIN * i + sl];
                }
            });
        }
    }

    if (KS > 1) {
        // partial sums of the KS slices meet in LDS; slice 0 finishes the rows
#pragma unroll
        for (int j = 0; j < PX; ++j) red[(wv * PX + j) * 64 + lane] = acc[j];
        __syncthreads();
        if (ks != 0) return;
#pragma unroll
        for (int j = 0; j < PX; ++j) {
            float s = acc[j];
#pragma unroll
            for (int k = 1; k < KS; ++k) s += red[((wv + k) * PX + j) * 64 + lane];
            acc[j] = s;
        }
    }

    // ---- fused epilogue: + bias, + residual, ReLU, store at the original channel
    if (co < 0 || !live) return;
    T* __restrict__ y = (T*)a.y + (size_t)n * a.yd.image + (size_t)co * a.yd.plane + a.yd.origin + oh * a.yd.pitch + ow0;
    const T* __restrict__ res =
        a.residual ? (const T*)a.residual + (size_t)n * a.rd.image + (size_t)co * a.rd.plane + a.rd.origin + oh * a.rd.pitch + ow0
                   : nullptr;
#pragma unroll
    for (int j = 0; j < PX; ++j) {
        if (ow0 + j < a.yd.w) {
            float v = acc[j] + bias;
            if (res) v += (float)res[j];
            if (a.relu) v = v > 0.0f ? v : 0.0f;
            y[j] = (T)v;
        }
    }
}

template <class Cfg>
hipError_t launch_quad(const ConvLaunch& a, hipStream_t s) {
    dim3 grid(1u, (unsigned)a.row_groups, (unsigned)a.n);
    CADNN_LAUNCH(sconv_quad_kernel<Cfg>, grid, dim3(Cfg::THREADS), 0, s, a);
    return hipGetLastError();
}

template <class Cfg>
ConvVariant make_quad(const char* name) {
    ConvVariant v{};
    v.name = name;
    v.family = FAM_LINEAR;
    v.is_f16 = sizeof(typename Cfg::T) == 2;
    v.kh = 0; v.kw = 0; v.stride = 0;
    v.p = Cfg::PX; v.nw = Cfg::NW; v.rpw = Cfg::R; v.ks = Cfg::KS;
    v.unroll = Cfg::WIN;        // parts are padded to whole windows
    v.adjacent = 2;             // pixel groups enumerated over rows rounded up to PX positions
    v.quad = 1;
    v.lds_bytes = (Cfg::KS > 1 ? (size_t)Cfg::NW * Cfg::PX * 64 * 4 : 0) + (size_t)Cfg::NW * 2 * 64 * 8;
    v.launch = &launch_quad<Cfg>;
    return v;
}

#define CADNN_QUAD(T, R, KS, RG, B) make_quad<QuadCfg<T, R, KS, RG, B>>("squad_" #T "_r" #R "k" #KS "g" #RG "b" #B)
#define CADNN_QUAD_SHAPES(T)                                                                                             \
    CADNN_QUAD(T, 4, 1, 4, 8), CADNN_QUAD(T, 4, 2, 2, 8), CADNN_QUAD(T, 4, 4, 1, 8), CADNN_QUAD(T, 4, 4, 2, 8),          \
        CADNN_QUAD(T, 4, 8, 1, 8), CADNN_QUAD(T, 4, 8, 1, 16), CADNN_QUAD(T, 2, 2, 2, 8), CADNN_QUAD(T, 2, 4, 1, 8),     \
        CADNN_QUAD(T, 2, 4, 1, 16), CADNN_QUAD(T, 2, 8, 1, 8), CADNN_QUAD(T, 2, 8, 1, 16)

}  // namespace

const std::vector<ConvVariant>& all_quad_variants() {
    static const std::vector<ConvVariant> v = {CADNN_QUAD_SHAPES(float), CADNN_QUAD_SHAPES(_Float16)};
    return v;
}

}  // namespace cadnn
