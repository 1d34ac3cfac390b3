// Wave-sliced LDS-tile sparse convolution for gfx950 (wave64).
//
// A workgroup computes a TW x TH tile of output pixels for G packed rows (output channels
// in the nnz-sorted order of the compact format).  The input channels are cut into chunks
// of CCH; the NW waves of the workgroup take the chunks round-robin and each wave keeps a
// PRIVATE slice of LDS: it stages the input tile (+halo) of its chunk there, copies the
// chunk's nonzero stream of the G rows next to it, and accumulates all G rows over that
// chunk.  Nothing in the main loop needs a workgroup barrier, so one wave stages while
// another computes; the partial sums of the NW waves meet once in LDS before the fused
// bias / residual / ReLU epilogue (paper Section 4: conv + batch-norm + activation fused).
//
// Staging (fp32): `buffer_load ... lds` writes 64 consecutive LDS words per instruction
// straight from per-lane global offsets; the per-lane offsets of one channel plane are
// computed once per workgroup (positions outside the image or its zero halo are given an
// out-of-range offset, which the buffer range check turns into zeros), the channel enters
// as the scalar offset, so staging a chunk costs no vector ALU work at all.
// Strided layers: the tile is de-interleaved by the stride in both directions ("phases")
// so lanes always read consecutive LDS words, and taps a strided 1x1 filter never touches
// are not staged.
//
// Inner loop: lanes are pixels, so a nonzero's weight and tile offset are wave-uniform;
// they are fetched two at a time with one broadcast 128-bit LDS read, then one LDS read
// and one FMA per pixel.  A filter element is thus fetched once per wave and reused for
// all its pixels (the paper's redundant filter-load elimination, Section 4).
#include "internal.h"

namespace cadnn {


namespace {

constexpr int smin(int a, int b) { return a < b ? a : b; }
constexpr int smax(int a, int b) { return a > b ? a : b; }

// Smallest pitch >= need whose lane rows read in one 32-lane pass hit disjoint banks.
constexpr int spitch(int need, int tw) {
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

template <typename T_, int KH_, int KW_, int S_, int TW_, int P_, int NW_, int G_, int CCH_, int CF_>
struct StileCfg {
    using T = T_;
    static constexpr int KH = KH_, KW = KW_, S = S_, TW = TW_, P = P_, NW = NW_, G = G_, CCH = CCH_;
    static constexpr int RW = 64 / TW;
    static constexpr int TH = RW * P;
    static constexpr int NRPH = smin(S, KH);
    static constexpr int RH = TH + (KH - 1) / S;
    static constexpr int NPH = smin(S, KW);
    static constexpr int CW = TW + (KW - 1) / S;
    // CF = 1 pads the pitch until lane rows fall into disjoint banks; CF = 0 keeps the tile
    // compact (small images: more channels per slice at the price of 2-way conflicts)
    static constexpr int PITCH = CF_ ? spitch(NPH * CW, TW) : NPH * CW;
    static constexpr int PLANE = NRPH * RH * PITCH;
    static constexpr int NSTP = (PLANE + 63) / 64;          // staging instructions per channel
    static constexpr int PLANE_PAD = NSTP * 64;
    static constexpr int SLICE_BYTES = CCH * PLANE_PAD * 4;
    // nonzero-stream entries a wave buffers per (G rows, chunk): never more than the dense
    // count (+ segment padding); layers whose streams exceed the cap are not served
    static constexpr int CAP = smin(1024, (G * (CCH * KH * KW + 4) + 3) / 4 * 4);
    static constexpr int NZ_BYTES = ((CAP + 63) / 64 * 64 + 8) * 8;   // whole lanes + read-ahead slack
    static constexpr int RED_BYTES = G * P * 64 * 4;
    static constexpr int WAVE_BYTES = smax(SLICE_BYTES + NZ_BYTES, RED_BYTES);
    static constexpr int LDS_BYTES = NW * WAVE_BYTES;
    static constexpr int THREADS = NW * 64;
    static_assert(64 % TW == 0, "TW must divide the wavefront");
    static_assert(LDS_BYTES <= 160 * 1024, "beyond the LDS of a compute unit");
};

constexpr uint32_t kStileOob = 0x7ffffff0u;

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// Four nonzeros (two broadcast 128-bit pairs) against the P pixels of a lane.
template <int P, int STEP>
__device__ __forceinline__ void stile_fma4(float (&acc)[P], const char* lane_ptr, const uint4& q0, const uint4& q1) {
    const char* l0 = lane_ptr + q0.y;
    const char* l1 = lane_ptr + q0.w;
    const char* l2 = lane_ptr + q1.y;
    const char* l3 = lane_ptr + q1.w;
    float x0[P], x1[P], x2[P], x3[P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        x0[j] = *(const float*)(l0 + j * STEP);
        x1[j] = *(const float*)(l1 + j * STEP);
        x2[j] = *(const float*)(l2 + j * STEP);
        x3[j] = *(const float*)(l3 + j * STEP);
    }
#pragma unroll
    for (int j = 0; j < P; ++j) {
        acc[j] = fmaf(__uint_as_float(q0.x), x0[j], acc[j]);
        acc[j] = fmaf(__uint_as_float(q0.z), x1[j], acc[j]);
        acc[j] = fmaf(__uint_as_float(q1.x), x2[j], acc[j]);
        acc[j] = fmaf(__uint_as_float(q1.z), x3[j], acc[j]);
    }
}

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void sconv_stile_kernel(const ConvLaunch a) {
    using T = typename Cfg::T;
    constexpr int S = Cfg::S, TW = Cfg::TW, P = Cfg::P, NW = Cfg::NW, G = Cfg::G, CCH = Cfg::CCH,
                  RW = Cfg::RW, TH = Cfg::TH, RH = Cfg::RH, NPH = Cfg::NPH, CW = Cfg::CW,
                  PITCH = Cfg::PITCH, PLANE = Cfg::PLANE, NSTP = Cfg::NSTP, PLANE_PAD = Cfg::PLANE_PAD;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tx = lane % TW, ty = lane / TW;
    const int tile_x = blockIdx.x % a.tiles_x, tile_y = blockIdx.x / a.tiles_x;
    const int grp = blockIdx.y;
    const int n = blockIdx.z;
    const int oh0 = tile_y * TH, ow0 = tile_x * TW;
    const int ih0 = oh0 * S - a.pad, iw0 = ow0 * S - a.pad;
    const int cin = a.xd.c;

    unsigned char* wave_mem = smem + (size_t)wv * Cfg::WAVE_BYTES;
    float* slice = (float*)wave_mem;
    uint2* nzbuf = (uint2*)(wave_mem + Cfg::SLICE_BYTES);

    // per-lane global byte offset of every staged position of ONE channel plane
    uint32_t pre[NSTP];
#pragma unroll
    for (int it = 0; it < NSTP; ++it) {
        const int e = it * 64 + lane;
        const int rr = e / PITCH, cc = e - rr * PITCH;
        const int rph = rr / RH, ri = rr - rph * RH;
        const int cph = cc / CW, cj = cc - cph * CW;
        const int ih = ih0 + ri * S + rph;
        const int iw = iw0 + cj * S + cph;
        const bool ok = e < PLANE && cph < NPH && ih >= -a.xd.ph && ih < a.xd.h + a.xd.ph &&
                        iw >= -a.xd.pw && iw < a.xd.w + a.xd.pw;
        pre[it] = ok ? (uint32_t)(a.xd.origin + ih * a.xd.pitch + iw) * (uint32_t)sizeof(T) : kStileOob;
    }

    const char* ximg = (const char*)a.x + (size_t)n * a.image_bytes;
    const uint32_t plane_bytes = (uint32_t)a.xd.plane * (uint32_t)sizeof(T);
    const uint2* __restrict__ nz = a.nz;
    const int32_t* __restrict__ seg_grp = a.seg_ptr + (size_t)grp * a.nchunks * (G + 1);
    const char* lane_ptr = (const char*)slice + (ty * PITCH + tx) * 4;

    float acc[G][P];
#pragma unroll
    for (int r = 0; r < G; ++r)
#pragma unroll
        for (int j = 0; j < P; ++j) acc[r][j] = 0.0f;

    constexpr int NZR = (Cfg::CAP + 63) / 64;        // stream entries a lane carries per chunk
    // The nonzero stream of the wave's NEXT chunk is fetched into registers while the
    // current chunk is staged and consumed, so a chunk exposes one memory latency (its
    // staging), not three (segment table, stream, staging).
    uint2 nzr[NZR];
    int myseg = 0;
    if (wv < a.nchunks) {
        myseg = seg_grp[(size_t)wv * (G + 1) + (lane < G ? lane : G)];
        const int sb0 = __builtin_amdgcn_readlane(myseg, 0), se0 = __builtin_amdgcn_readlane(myseg, G);
#pragma unroll
        for (int k = 0; k < NZR; ++k) {
            const int i = sb0 + k * 64 + lane;
            nzr[k] = i < se0 ? nz[i] : make_uint2(0u, 0u);
        }
    }

    for (int c = wv; c < a.nchunks; c += NW) {
        // segment table of this (group, chunk), broadcast lane by lane
        int sg[G + 1];
#pragma unroll
        for (int r = 0; r <= G; ++r) sg[r] = __builtin_amdgcn_readlane(myseg, r);
        const int sb = sg[0], se = sg[G];
        // everything this wave read from its slice for the previous chunk has been consumed
        __builtin_amdgcn_wave_barrier();
        // ---- the chunk's nonzero stream goes next to the tile
#pragma unroll
        for (int k = 0; k < NZR; ++k)
            if (k * 64 < se - sb) nzbuf[k * 64 + lane] = nzr[k];
        // ---- fetch the next chunk's table and stream
        const int cn = c + NW;
        if (cn < a.nchunks) {
            myseg = seg_grp[(size_t)cn * (G + 1) + (lane < G ? lane : G)];
            const int sbn = __builtin_amdgcn_readlane(myseg, 0), sen = __builtin_amdgcn_readlane(myseg, G);
#pragma unroll
            for (int k = 0; k < NZR; ++k) {
                const int i = sbn + k * 64 + lane;
                nzr[k] = i < sen ? nz[i] : make_uint2(0u, 0u);
            }
        }
        if (sb == se) continue;                       // none of the G rows touches this chunk
        const int c0 = c * CCH;
        const int nch = smin(CCH, cin - c0);
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(ximg + (size_t)c0 * plane_bytes), 0, a.image_bytes - (uint32_t)c0 * plane_bytes,
            0x00020000);
        // ---- stage the chunk's channels
        for (int ch = 0; ch < nch; ++ch) {
            const uint32_t soff = (uint32_t)ch * plane_bytes;
#pragma unroll
            for (int it = 0; it < NSTP; ++it) {
                if (sizeof(T) == 4) {
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rsrc, (lds_ptr_t)(slice + ch * PLANE_PAD + it * 64), 4, pre[it], soff, 0, 0);
                } else {
                    const unsigned short hbits = __builtin_amdgcn_raw_buffer_load_b16(rsrc, pre[it], soff, 0);
                    slice[ch * PLANE_PAD + it * 64 + lane] = (float)__builtin_bit_cast(_Float16, hbits);
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
        // ---- accumulate.  Runs are padded to four entries; two register sets take turns so
        //      the (value, offset) pairs of the next four are in flight while these are used.
#pragma unroll
        for (int r = 0; r < G; ++r) {
            const uint4* p4 = (const uint4*)(nzbuf + (sg[r] - sb));
            int groups = (sg[r + 1] - sg[r]) >> 2;
            if (groups == 0) continue;
            uint4 a0 = p4[0], a1 = p4[1], b0, b1;
            while (true) {
                b0 = p4[2]; b1 = p4[3];               // next four (stays inside the buffer's slack)
                stile_fma4<P, RW * PITCH * 4>(acc[r], lane_ptr, a0, a1);
                if (groups == 1) break;
                a0 = p4[4]; a1 = p4[5];
                stile_fma4<P, RW * PITCH * 4>(acc[r], lane_ptr, b0, b1);
                if (groups == 2) break;
                groups -= 2;
                p4 += 4;
            }
        }
    }

    // ---- partial sums of the NW waves meet in LDS; each wave then finishes G/NW rows
    __syncthreads();
    float* red = (float*)wave_mem;
#pragma unroll
    for (int r = 0; r < G; ++r)
#pragma unroll
        for (int j = 0; j < P; ++j) red[(r * P + j) * 64 + lane] = acc[r][j];
    __syncthreads();

    const int ow = ow0 + tx;
    T* __restrict__ y = (T*)a.y + (size_t)n * a.yd.image + a.yd.origin;
    const T* __restrict__ res = a.residual ? (const T*)a.residual + (size_t)n * a.rd.image + a.rd.origin : nullptr;
    constexpr int RPF = (G + NW - 1) / NW;          // rows finished per wave
#pragma unroll
    for (int rr = 0; rr < RPF; ++rr) {
        const int r = wv * RPF + rr;
        if (r >= G) break;
        const int co = a.perm[grp * G + r];
        if (co < 0) continue;
        const float b = a.bias ? a.bias[co] : 0.0f;
#pragma unroll
        for (int j = 0; j < P; ++j) {
            float v = b;
#pragma unroll
            for (int k = 0; k < NW; ++k)
                v += ((const float*)(smem + (size_t)k * Cfg::WAVE_BYTES))[(r * P + j) * 64 + lane];
            const int oh = oh0 + ty + j * RW;
            if (oh < a.yd.h && ow < a.yd.w) {
                if (res) v += (float)res[(size_t)co * a.rd.plane + oh * a.rd.pitch + ow];
                if (a.relu) v = v > 0.0f ? v : 0.0f;
                y[(size_t)co * a.yd.plane + oh * a.yd.pitch + ow] = (T)v;
            }
        }
    }
}

template <class Cfg>
hipError_t launch_stile(const ConvLaunch& a, hipStream_t s) {
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void*)sconv_stile_kernel<Cfg>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    dim3 grid((unsigned)(a.tiles_x * a.tiles_y), (unsigned)a.row_groups, (unsigned)a.n);
    dim3 block(Cfg::THREADS);
    CADNN_LAUNCH(sconv_stile_kernel<Cfg>, grid, block, Cfg::LDS_BYTES, s, a);
    return hipGetLastError();
}

template <class Cfg>
ConvVariant make_stile(const char* name) {
    ConvVariant v{};
    v.name = name;
    v.family = FAM_STILE;
    v.is_f16 = sizeof(typename Cfg::T) == 2;
    v.kh = Cfg::KH; v.kw = Cfg::KW; v.stride = Cfg::S;
    v.tw = Cfg::TW; v.rw = Cfg::RW; v.p = Cfg::P;
    v.nw = Cfg::NW; v.rpw = Cfg::G; v.ks = Cfg::NW; v.cch = Cfg::CCH;
    v.th = Cfg::TH; v.rh = Cfg::RH; v.nrph = Cfg::NRPH; v.cw = Cfg::CW; v.nph = Cfg::NPH;
    v.pitch = Cfg::PITCH; v.plane = Cfg::PLANE_PAD;
    v.elem_bytes = 4;
    v.unroll = 4;
    v.nz_cap = Cfg::CAP;
    v.lds_bytes = Cfg::LDS_BYTES;
    v.launch = &launch_stile<Cfg>;
    return v;
}

}  // namespace

#define CADNN_STILE(T, KH, KW, S, TW, P, NW, G, CCH, CF) \
    make_stile<StileCfg<T, KH, KW, S, TW, P, NW, G, CCH, CF>>( \
        "stile_" #T "_k" #KH "x" #KW "s" #S "_t" #TW "p" #P "_w" #NW "g" #G "c" #CCH "f" #CF)

#define CADNN_STILE_SHAPES(T)                          \
    /* 3x3 stride 1: 56x56 / 28x28 images */           \
    CADNN_STILE(T, 3, 3, 1, 32, 4, 8, 8, 8, 1),        \
    CADNN_STILE(T, 3, 3, 1, 32, 2, 8, 8, 8, 1),        \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 8, 16, 8, 1),        \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 8, 8, 8, 1),         \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 16, 16, 4, 1),       \
    /* 3x3 stride 1: whole 14x14 / 7x7 image per tile */ \
    CADNN_STILE(T, 3, 3, 1, 16, 4, 8, 8, 8, 0),        \
    CADNN_STILE(T, 3, 3, 1, 16, 4, 8, 8, 4, 1),        \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 8, 8, 16, 0),        \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 16, 16, 4, 0),       \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 8, 2, 24, 0),        \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 4, 2, 32, 0),        \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 8, 4, 16, 0),        \
    CADNN_STILE(T, 3, 3, 1, 16, 4, 8, 1, 8, 0),        \
    CADNN_STILE(T, 3, 3, 1, 16, 4, 8, 2, 8, 0),        \
    CADNN_STILE(T, 3, 3, 1, 16, 4, 4, 2, 8, 0),        \
    /* 3x3 stride 2 */                                 \
    CADNN_STILE(T, 3, 3, 2, 8, 1, 8, 2, 8, 0),         \
    CADNN_STILE(T, 3, 3, 2, 16, 4, 8, 2, 2, 0),        \
    CADNN_STILE(T, 3, 3, 2, 32, 2, 8, 8, 4, 1),        \
    CADNN_STILE(T, 3, 3, 2, 8, 1, 8, 8, 8, 1),         \
    CADNN_STILE(T, 3, 3, 2, 16, 4, 8, 8, 2, 0),        \
    CADNN_STILE(T, 3, 3, 2, 8, 1, 8, 8, 8, 0),         \
    /* 1x1 stride 2 (projection shortcuts) */          \
    CADNN_STILE(T, 1, 1, 2, 32, 2, 8, 8, 16, 1),       \
    CADNN_STILE(T, 1, 1, 2, 16, 4, 8, 8, 16, 1),       \
    CADNN_STILE(T, 1, 1, 2, 8, 1, 8, 8, 32, 1),        \
    CADNN_STILE(T, 1, 1, 2, 8, 1, 16, 16, 16, 1),      \
    /* 1x1 stride 1 */                                 \
    CADNN_STILE(T, 1, 1, 1, 32, 2, 8, 8, 16, 1),       \
    CADNN_STILE(T, 1, 1, 1, 16, 4, 8, 8, 16, 1),       \
    CADNN_STILE(T, 1, 1, 1, 8, 1, 16, 16, 16, 1),      \
    /* 7x7 stride 2 */                                 \
    CADNN_STILE(T, 7, 7, 2, 32, 4, 4, 4, 1, 1)

const std::vector<ConvVariant>& all_stile_variants() {
    static const std::vector<ConvVariant> v = {CADNN_STILE_SHAPES(float), CADNN_STILE_SHAPES(_Float16)};
    return v;
}

}  // namespace cadnn
