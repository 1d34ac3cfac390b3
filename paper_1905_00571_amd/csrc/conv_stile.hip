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

template <typename T_, int KH_, int KW_, int S_, int TW_, int P_, int NW_, int G_, int CCH_>
struct StileCfg {
    using T = T_;
    static constexpr int KH = KH_, KW = KW_, S = S_, TW = TW_, P = P_, NW = NW_, G = G_, CCH = CCH_;
    static constexpr int RW = 64 / TW;
    static constexpr int TH = RW * P;
    static constexpr int NRPH = smin(S, KH);
    static constexpr int RH = TH + (KH - 1) / S;
    static constexpr int NPH = smin(S, KW);
    static constexpr int CW = TW + (KW - 1) / S;
    static constexpr int PITCH = spitch(NPH * CW, TW);
    static constexpr int PLANE = NRPH * RH * PITCH;
    static constexpr int NSTP = (PLANE + 63) / 64;          // staging instructions per channel
    static constexpr int PLANE_PAD = NSTP * 64;
    static constexpr int SLICE_BYTES = CCH * PLANE_PAD * 4;
    // nonzero-stream entries a wave buffers per (G rows, chunk): never more than the dense
    // count (+ segment padding); layers whose streams exceed the cap are not served
    static constexpr int CAP = smin(1024, (G * (CCH * KH * KW + 2) + 1) / 2 * 2);
    static constexpr int NZ_BYTES = CAP * 8;
    static constexpr int RED_BYTES = G * P * 64 * 4;
    static constexpr int WAVE_BYTES = smax(SLICE_BYTES + NZ_BYTES, RED_BYTES);
    static constexpr int LDS_BYTES = NW * WAVE_BYTES;
    static constexpr int THREADS = NW * 64;
    static_assert(64 % TW == 0, "TW must divide the wavefront");
    static_assert(G % NW == 0, "rows are finished NW waves at a time");
    static_assert(LDS_BYTES <= 160 * 1024, "beyond the LDS of a compute unit");
};

constexpr uint32_t kStileOob = 0x7ffffff0u;

typedef __attribute__((address_space(3))) void* lds_ptr_t;

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

    for (int c = wv; c < a.nchunks; c += NW) {
        const int32_t* __restrict__ seg = seg_grp + (size_t)c * (G + 1);
        const int sb = seg[0], se = seg[G];
        if (sb == se) continue;                       // none of the G rows touches this chunk
        // everything this wave read from its slice for the previous chunk has been consumed
        __builtin_amdgcn_wave_barrier();
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
        // ---- copy the nonzero stream of the G rows for this chunk next to the tile
        for (int i = sb + lane; i < se; i += 64) nzbuf[i - sb] = nz[i];
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
        // ---- accumulate: two (value, offset) pairs per broadcast read
#pragma unroll
        for (int r = 0; r < G; ++r) {
            const uint4* p4 = (const uint4*)(nzbuf + (seg[r] - sb));
            const uint4* e4 = (const uint4*)(nzbuf + (seg[r + 1] - sb));
            for (; p4 < e4; ++p4) {
                const uint4 pr = *p4;
                const float w0 = __uint_as_float(pr.x), w1 = __uint_as_float(pr.z);
                const char* l0 = lane_ptr + pr.y;
                const char* l1 = lane_ptr + pr.w;
#pragma unroll
                for (int j = 0; j < P; ++j) {
                    acc[r][j] = fmaf(w0, *(const float*)(l0 + j * RW * PITCH * 4), acc[r][j]);
                    acc[r][j] = fmaf(w1, *(const float*)(l1 + j * RW * PITCH * 4), acc[r][j]);
                }
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
    constexpr int RPF = G / NW;
#pragma unroll
    for (int rr = 0; rr < RPF; ++rr) {
        const int r = wv * RPF + rr;
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
    hipLaunchKernelGGL(sconv_stile_kernel<Cfg>, grid, block, Cfg::LDS_BYTES, s, a);
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
    v.unroll = 2;
    v.nz_cap = Cfg::CAP;
    v.lds_bytes = Cfg::LDS_BYTES;
    v.launch = &launch_stile<Cfg>;
    return v;
}

}  // namespace

#define CADNN_STILE(T, KH, KW, S, TW, P, NW, G, CCH) \
    make_stile<StileCfg<T, KH, KW, S, TW, P, NW, G, CCH>>( \
        "stile_" #T "_k" #KH "x" #KW "s" #S "_t" #TW "p" #P "_w" #NW "g" #G "c" #CCH)

#define CADNN_STILE_SHAPES(T)                       \
    /* 3x3 stride 1 */                              \
    CADNN_STILE(T, 3, 3, 1, 32, 4, 4, 4, 8),        \
    CADNN_STILE(T, 3, 3, 1, 32, 2, 4, 8, 8),        \
    CADNN_STILE(T, 3, 3, 1, 32, 2, 4, 4, 8),        \
    CADNN_STILE(T, 3, 3, 1, 16, 4, 4, 4, 8),        \
    CADNN_STILE(T, 3, 3, 1, 16, 4, 8, 8, 2),        \
    CADNN_STILE(T, 3, 3, 1, 16, 2, 4, 8, 8),        \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 4, 16, 16),       \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 4, 8, 16),        \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 8, 8, 8),         \
    CADNN_STILE(T, 3, 3, 1, 8, 1, 8, 16, 8),        \
    /* 3x3 stride 2 */                              \
    CADNN_STILE(T, 3, 3, 2, 32, 2, 4, 8, 4),        \
    CADNN_STILE(T, 3, 3, 2, 32, 2, 4, 4, 4),        \
    CADNN_STILE(T, 3, 3, 2, 16, 2, 4, 8, 4),        \
    CADNN_STILE(T, 3, 3, 2, 16, 4, 4, 4, 4),        \
    CADNN_STILE(T, 3, 3, 2, 8, 1, 4, 16, 8),        \
    CADNN_STILE(T, 3, 3, 2, 8, 1, 8, 8, 8),         \
    /* 1x1 stride 2 (projection shortcuts) */       \
    CADNN_STILE(T, 1, 1, 2, 32, 2, 4, 8, 32),       \
    CADNN_STILE(T, 1, 1, 2, 16, 4, 4, 8, 16),       \
    CADNN_STILE(T, 1, 1, 2, 16, 4, 8, 8, 16),       \
    CADNN_STILE(T, 1, 1, 2, 8, 1, 8, 16, 32),       \
    CADNN_STILE(T, 1, 1, 2, 8, 1, 4, 8, 32),        \
    /* 1x1 stride 1 */                              \
    CADNN_STILE(T, 1, 1, 1, 32, 2, 4, 8, 32),       \
    CADNN_STILE(T, 1, 1, 1, 16, 4, 4, 8, 16),       \
    CADNN_STILE(T, 1, 1, 1, 16, 4, 8, 8, 16),       \
    CADNN_STILE(T, 1, 1, 1, 8, 1, 8, 16, 32),       \
    /* 7x7 stride 2 */                              \
    CADNN_STILE(T, 7, 7, 2, 32, 4, 4, 4, 1),        \
    CADNN_STILE(T, 7, 7, 2, 32, 2, 4, 8, 1)

const std::vector<ConvVariant>& all_stile_variants() {
    static const std::vector<ConvVariant> v = {CADNN_STILE_SHAPES(float), CADNN_STILE_SHAPES(_Float16)};
    return v;
}

}  // namespace cadnn
