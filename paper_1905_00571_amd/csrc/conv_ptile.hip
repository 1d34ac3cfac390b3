// Shared-tile LDS sparse convolution for gfx950 (wave64).
//
// The vector L1 of a compute unit delivers far fewer bytes per clock than its LDS, and a
// kernel that feeds every FMA from global memory is bound by exactly that.  Filters larger
// than 1x1 reuse an input element for several taps and for every output channel, so here a
// workgroup stages the input region of one block of output pixels (7 rows x 7*P columns)
// in LDS once -- all input channels if they fit, else chunk after chunk -- and all its
// waves compute from it: the NW waves split G packed rows (output channels in the
// nnz-sorted order of the compact format) and, KS ways, each row's nonzeros.
//
// Lanes are pixels (an 8 x 8 lane grid of which 7 x 7 is used; pixel j of a lane is 7*j
// columns further right), so a nonzero's weight and tile offset are wave-uniform: they are
// streamed with coalesced 64-entry vector loads and broadcast lane by lane, and a filter
// element is fetched once per wave and reused for all its pixels (the paper's redundant
// filter-load elimination, Section 4).  Per nonzero a lane does one LDS read and one FMA
// per pixel.  Strided layers: the staged region is de-interleaved by the stride so lanes
// always read consecutive LDS words.  Out-of-image positions are staged as zeros (they get
// an out-of-range buffer offset), so the input needs no halo -- though it may have one.
// Partial sums of the KS slices meet in LDS before the fused bias / residual / ReLU
// epilogue (Section 4: conv + batch-norm + activation fused).
#include "internal.h"

namespace cadnn {

namespace {

constexpr uint32_t kPtOutOfRange = 0x7ffffff0u;

typedef __attribute__((address_space(3))) void* lds_ptr_t;

template <typename T_, int P_, int RPW_, int KS_, int NW_, int U_, int LW_ = 8>
struct PtileCfg {
    using T = T_;
    static constexpr int P = P_, RPW = RPW_, KS = KS_, NW = NW_, U = U_, LW = LW_;
    // LDS bytes between the pixels of a lane: 7 words to the right (LW = 8) or 4 rows of
    // 16 words further down (LW = 16)
    static constexpr int STEP = LW == 16 ? 4 * 16 * 4 : 7 * 4;
    static_assert(LW == 8 || LW == 16, "lane grid width");
    static constexpr int RG = NW / KS;
    static constexpr int THREADS = NW * 64;
    static_assert(NW % KS == 0, "KS must divide the waves of a workgroup");
};

template <int P, int STEP>
__device__ __forceinline__ void pt_fetch(const char* lane_ptr, uint32_t off, float (&x)[P]) {
    const char* p = lane_ptr + off;
#pragma unroll
    for (int j = 0; j < P; ++j) x[j] = *(const float*)(p + j * STEP);
}

// Broadcasts entries l0 .. l0+U-1 of a 64-entry window held one entry per lane.
template <int U>
__device__ __forceinline__ void pt_group(const uint2& win, int l0, float (&w)[U], uint32_t (&o)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        w[u] = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)win.x, l0 + u));
        o[u] = (uint32_t)__builtin_amdgcn_readlane((int)win.y, l0 + u);
    }
}

// Entries l0 .. l1-1 of one window against the P pixels of a lane, U at a time: U LDS reads
// in flight, then U FMAs per pixel.  The LDS latency of a group is covered by the other
// waves of the SIMD (a hand-pipelined loop made the compiler serialise the reads on false
// register hazards).
template <int U, int P, int STEP>
__device__ __forceinline__ void pt_window(const uint2& win, int l0, int l1, const char* lane_ptr, float (&acc)[P]) {
    for (; l0 < l1; l0 += U) {
        float w[U], x[U][P];
        uint32_t o[U];
        pt_group<U>(win, l0, w, o);
#pragma unroll
        for (int u = 0; u < U; ++u) pt_fetch<P, STEP>(lane_ptr, o[u], x[u]);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < P; ++j) acc[j] = fmaf(w[u], x[u][j], acc[j]);
    }
}

// fp16 element widened to fp32
__device__ __forceinline__ float pt_gload16(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    const unsigned short h = __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
    return (float)__builtin_bit_cast(_Float16, h);
}

}  // namespace

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void sconv_ptile_kernel(const ConvLaunch a) {
    using T = typename Cfg::T;
    constexpr int P = Cfg::P, RPW = Cfg::RPW, KS = Cfg::KS, RG = Cfg::RG, U = Cfg::U, NW = Cfg::NW;
    extern __shared__ float tile[];

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rg = wv / KS, ks = wv % KS;
    const int n = blockIdx.z;
    const int ty = blockIdx.x / a.tiles_x, tx = blockIdx.x - ty * a.tiles_x;
    const int row0 = (blockIdx.y * RG + rg) * RPW;
    const int nchunks = a.pt_nchunks;

    // ---- the wave's stream and part lengths are requested first: they do not depend on
    //      the tile.  A wave's parts (chunk by chunk, row by row within a chunk) lie back to
    //      back in one stream of fixed stride per wave, so two 64-entry windows can run
    //      ahead of the consumption across part boundaries without ever stalling on them.
    const int wsi = (blockIdx.y * RG + rg) * KS + ks;        // wave stream index
    const uint2* __restrict__ nzl = a.nz + (size_t)wsi * a.nchunks + lane;
    uint2 winA = nzl[0], winB = nzl[64];
    const int32_t* __restrict__ lens = a.seg_ptr + (size_t)wsi * nchunks * RPW;
    int co_[RPW], len_[RPW];
    float bias_[RPW];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        co_[r] = a.perm[row0 + r];
        len_[r] = lens[r];
    }
#pragma unroll
    for (int r = 0; r < RPW; ++r) bias_[r] = (a.bias && co_[r] >= 0) ? a.bias[co_[r]] : 0.0f;

    // ---- lane -> pixels
    constexpr int LW = Cfg::LW;
    constexpr int TILE_H = LW == 16 ? 4 * P : 7, TILE_W = LW == 16 ? 14 : 7 * P, USED = LW == 16 ? 14 : 7;
    const int li = lane / LW, lj = lane % LW;
    const bool lane_used = lj < USED && (LW == 16 || li < 7);
    int oidx[P], orow[P], ocol[P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        orow[j] = ty * TILE_H + li + (LW == 16 ? 4 * j : 0);
        ocol[j] = tx * TILE_W + lj + (LW == 16 ? 0 : 7 * j);
        oidx[j] = (lane_used && orow[j] < a.yd.h && ocol[j] < a.yd.w) ? orow[j] * a.yd.pitch + ocol[j] : -1;
    }
    // (the unused lanes of the grid read the tile origin: harmless and in range)
    const char* lane_ptr = (const char*)tile + (lane_used ? (li * a.pt_pitch + lj) * 4 : 0);

    // ---- residual up front: one more round trip off the tail
    const T* __restrict__ res = a.residual ? (const T*)a.residual + (size_t)n * a.rd.image + a.rd.origin : nullptr;
    float resv[RPW][P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const int ridx = orow[j] * a.rd.pitch + ocol[j];
#pragma unroll
        for (int r = 0; r < RPW; ++r)
            resv[r][j] = (res && ks == 0 && co_[r] >= 0 && oidx[j] >= 0) ? (float)res[(size_t)co_[r] * a.rd.plane + ridx] : 0.0f;
    }

    // ---- staging offsets: tile word p = lane + 64*t of a channel plane comes from here
    uint32_t goff[kPtileMaxSteps];
    {
        const int r_base = ty * TILE_H * a.stride - a.pad;     // image row of region row 0
        const int c_base = tx * TILE_W * a.stride - a.pad;
#pragma unroll
        for (int t = 0; t < kPtileMaxSteps; ++t) {
            const int p = lane + 64 * t;
            uint32_t off = kPtOutOfRange;
            if (t < a.pt_nstp && p < a.pt_plane) {
                const int phase = p / a.pt_sub, q = p - phase * a.pt_sub;
                const int pr = q / a.pt_pitch, pc = q - pr * a.pt_pitch;
                const int pa = phase / a.pt_nphc, pb = phase - pa * a.pt_nphc;
                const int u = pr * a.stride + pa, v = pc * a.stride + pb;
                const int row = r_base + u, col = c_base + v;
                if (phase < a.pt_nph && u < a.pt_in_rows && v < a.pt_in_cols && row >= -a.xd.ph &&
                    row < a.xd.h + a.xd.ph && col >= -a.xd.pw && col < a.xd.w + a.xd.pw)
                    off = (uint32_t)(a.xd.origin + row * a.xd.pitch + col) * (uint32_t)sizeof(T);
            }
            goff[t] = off;
        }
    }
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const char*)a.x + (size_t)n * a.image_bytes), 0, a.image_bytes, 0x00020000);
    const uint32_t plane_bytes = (uint32_t)a.xd.plane * (uint32_t)sizeof(T);
    const int cin = a.xd.c;

    float acc[RPW][P];
#pragma unroll
    for (int r = 0; r < RPW; ++r)
#pragma unroll
        for (int j = 0; j < P; ++j) acc[r][j] = 0.0f;

    // Staging of one chunk.  fp32: `buffer_load ... lds` moves 64 words per instruction
    // from per-lane global offsets straight to consecutive LDS words, with no register in
    // between, so a wave keeps all the loads of its channels in flight at once (lanes past
    // the end of a plane are masked off: they would land on the next channel) -- and the
    // kernel goes on computing on the other buffer meanwhile.  fp16: through registers,
    // widened to fp32 on the way, four channels at a time.
    const int chunk_words = a.pt_cch * a.pt_plane;
    auto stage = [&](int c, float* buf) {
        const int ch0 = c * a.pt_cch;
        const int cch = min(a.pt_cch, cin - ch0);
        if constexpr (sizeof(T) == 4) {
            for (int ch = wv; ch < cch; ch += NW) {
                const uint32_t soff = (uint32_t)(ch0 + ch) * plane_bytes;
#pragma unroll
                for (int t = 0; t < kPtileMaxSteps; ++t)
                    if (t < a.pt_nstp && lane + 64 * t < a.pt_plane)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)(buf + ch * a.pt_plane + 64 * t), 4,
                                                                 goff[t], soff, 0, 0);
            }
        } else {
            for (int ch = wv; ch < cch; ch += 4 * NW) {
                float v[4][kPtileMaxSteps];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int chk = min(ch + k * NW, cch - 1);
                    const uint32_t soff = (uint32_t)(ch0 + chk) * plane_bytes;
#pragma unroll
                    for (int t = 0; t < kPtileMaxSteps; ++t)
                        if (t < a.pt_nstp) v[k][t] = pt_gload16(rsrc, goff[t], soff);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (ch + k * NW >= cch) break;
#pragma unroll
                    for (int t = 0; t < kPtileMaxSteps; ++t) {
                        const int p = lane + 64 * t;
                        if (t < a.pt_nstp && p < a.pt_plane) buf[(ch + k * NW) * a.pt_plane + p] = v[k][t];
                    }
                }
            }
        }
    };

    // fp32 with several chunks: two LDS buffers, chunk c+1 lands while chunk c is consumed
    // (one barrier per chunk); otherwise one buffer, staged and consumed in turn.
    const bool twobuf = sizeof(T) == 4 && a.pt_nbuf == 2;
    int pos = 0;                 // entries of the wave's stream consumed so far
    int wbase = 0;               // stream index of entry 0 of the older window
    bool a_older = true;         // which of the two windows is the older one
    if (twobuf) stage(0, tile);
    for (int c = 0; c < nchunks; ++c) {
        float* buf = tile + ((twobuf && (c & 1)) ? chunk_words : 0);
        if (twobuf) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // this wave's share of chunk c landed
            __syncthreads();                                    // ... everyone's; and chunk c-1 is consumed
            if (c + 1 < nchunks) stage(c + 1, tile + ((c & 1) ? 0 : chunk_words));
        } else {
            if (c > 0) __syncthreads();                         // everyone is done reading the previous chunk
            stage(c, buf);
            if constexpr (sizeof(T) == 4) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
        const char* lp = lane_ptr + (buf - tile) * 4;
        // part lengths of the next chunk: needed only after the next barrier
        int nlen_[RPW];
#pragma unroll
        for (int r = 0; r < RPW; ++r) nlen_[r] = c + 1 < nchunks ? lens[(c + 1) * RPW + r] : 0;

        // ---- accumulate the wave's parts of this chunk
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            int left = len_[r];
            while (left > 0) {
                const int l0 = pos - wbase;                      // 0 .. 63, a multiple of U
                const int take = min(left, 64 - l0);
                if (a_older) pt_window<U, P, Cfg::STEP>(winA, l0, l0 + take, lp, acc[r]);
                else pt_window<U, P, Cfg::STEP>(winB, l0, l0 + take, lp, acc[r]);
                pos += take;
                left -= take;
                if (l0 + take == 64) {
                    // the older window is used up: refill it for 128 entries further on (the
                    // plan ends with spare entries, so the read-ahead stays inside it)
                    if (a_older) winA = nzl[wbase + 128]; else winB = nzl[wbase + 128];
                    wbase += 64;
                    a_older = !a_older;
                }
            }
        }
#pragma unroll
        for (int r = 0; r < RPW; ++r) len_[r] = nlen_[r];
    }

    if (KS > 1) {
        // partial sums of the KS slices meet in LDS (the tile is no longer needed)
        __syncthreads();
#pragma unroll
        for (int r = 0; r < RPW; ++r)
#pragma unroll
            for (int j = 0; j < P; ++j) tile[((wv * RPW + r) * P + j) * 64 + lane] = acc[r][j];
        __syncthreads();
        if (ks != 0) return;
#pragma unroll
        for (int r = 0; r < RPW; ++r)
#pragma unroll
            for (int j = 0; j < P; ++j) {
                float s = acc[r][j];
#pragma unroll
                for (int k = 1; k < KS; ++k) s += tile[(((wv + k) * RPW + r) * P + j) * 64 + lane];
                acc[r][j] = s;
            }
    }

    // ---- fused epilogue: + bias, + residual, ReLU, store at the original channel
    T* __restrict__ y = (T*)a.y + (size_t)n * a.yd.image + a.yd.origin;
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int co = co_[r];
        if (co < 0) continue;
        const float b = bias_[r];
#pragma unroll
        for (int j = 0; j < P; ++j) {
            if (oidx[j] >= 0) {
                float v = acc[r][j] + b;
                v += resv[r][j];
                if (a.relu) v = v > 0.0f ? v : 0.0f;
                y[(size_t)co * a.yd.plane + oidx[j]] = (T)v;
            }
        }
    }
}

template <class Cfg>
static hipError_t launch_ptile(const ConvLaunch& a, hipStream_t s) {
    // more than 64 KB of dynamic LDS has to be asked for once per kernel
    static const hipError_t attr = hipFuncSetAttribute((const void*)sconv_ptile_kernel<Cfg>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytesPerCU);
    if (attr != hipSuccess) return attr;
    dim3 grid((unsigned)(a.tiles_x * a.tiles_y), (unsigned)a.row_groups, (unsigned)a.n);
    dim3 block(Cfg::THREADS);
    CADNN_LAUNCH(sconv_ptile_kernel<Cfg>, grid, block, a.pt_lds_bytes, s, a);
    return hipGetLastError();
}

template <class Cfg>
static ConvVariant make_ptile(const char* name) {
    ConvVariant v{};
    v.name = name;
    v.family = FAM_PTILE;
    v.is_f16 = sizeof(typename Cfg::T) == 2;
    v.kh = 0; v.kw = 0; v.stride = 0;
    v.p = Cfg::P; v.nw = Cfg::NW; v.rpw = Cfg::RPW; v.ks = Cfg::KS;
    v.unroll = Cfg::U;
    v.tw = Cfg::LW;
    v.lds_bytes = 0;
    v.launch = &launch_ptile<Cfg>;
    return v;
}

#define CADNN_PTILE(T, P, RPW, KS, NW, U) \
    make_ptile<PtileCfg<T, P, RPW, KS, NW, U>>("sptile_" #T "_p" #P "_r" #RPW "k" #KS "w" #NW "u" #U)

#define CADNN_PTILE_WIDE(T, P, RPW, KS, NW, U) \
    make_ptile<PtileCfg<T, P, RPW, KS, NW, U, 16>>("sptile_" #T "_v" #P "_r" #RPW "k" #KS "w" #NW "u" #U)

#define CADNN_PTILE_SHAPES(T)         \
    CADNN_PTILE_WIDE(T, 1, 1, 1, 16, 4),  \
    CADNN_PTILE_WIDE(T, 1, 1, 2, 16, 4),  \
    CADNN_PTILE_WIDE(T, 1, 1, 4, 16, 4),  \
    CADNN_PTILE_WIDE(T, 1, 2, 1, 16, 4),  \
    CADNN_PTILE_WIDE(T, 2, 1, 1, 16, 4),  \
    CADNN_PTILE_WIDE(T, 2, 1, 2, 16, 4),  \
    CADNN_PTILE_WIDE(T, 2, 1, 4, 16, 4),  \
    CADNN_PTILE_WIDE(T, 2, 1, 8, 16, 4),  \
    CADNN_PTILE_WIDE(T, 2, 2, 1, 16, 4),  \
    CADNN_PTILE_WIDE(T, 2, 4, 1, 16, 4),  \
    CADNN_PTILE_WIDE(T, 4, 1, 1, 16, 4),  \
    CADNN_PTILE_WIDE(T, 4, 1, 2, 16, 4),  \
    CADNN_PTILE_WIDE(T, 4, 1, 4, 16, 4),  \
    CADNN_PTILE_WIDE(T, 4, 1, 8, 16, 4),  \
    CADNN_PTILE_WIDE(T, 4, 2, 1, 16, 4),  \
    CADNN_PTILE_WIDE(T, 4, 4, 1, 16, 4),  \
    CADNN_PTILE_WIDE(T, 4, 4, 1, 8, 4),   \
    CADNN_PTILE_WIDE(T, 4, 2, 2, 8, 4),   \
    CADNN_PTILE_WIDE(T, 4, 1, 2, 8, 4),   \
    CADNN_PTILE(T, 1, 1, 1, 16, 4),   \
    CADNN_PTILE(T, 1, 1, 2, 16, 4),   \
    CADNN_PTILE(T, 1, 1, 4, 16, 4),   \
    CADNN_PTILE(T, 1, 1, 8, 16, 4),   \
    CADNN_PTILE(T, 1, 1, 16, 16, 4),  \
    CADNN_PTILE(T, 1, 2, 1, 16, 4),   \
    CADNN_PTILE(T, 1, 2, 4, 16, 4),   \
    CADNN_PTILE(T, 1, 1, 1, 8, 4),    \
    CADNN_PTILE(T, 1, 1, 2, 8, 4),    \
    CADNN_PTILE(T, 1, 1, 4, 8, 4),    \
    CADNN_PTILE(T, 1, 1, 8, 8, 4),    \
    CADNN_PTILE(T, 2, 1, 1, 16, 4),   \
    CADNN_PTILE(T, 2, 1, 2, 16, 4),   \
    CADNN_PTILE(T, 2, 1, 4, 16, 4),   \
    CADNN_PTILE(T, 2, 1, 8, 16, 4),   \
    CADNN_PTILE(T, 2, 1, 16, 16, 4),  \
    CADNN_PTILE(T, 4, 1, 4, 16, 4),   \
    CADNN_PTILE(T, 4, 1, 8, 16, 4),   \
    CADNN_PTILE(T, 4, 1, 16, 16, 4),  \
    CADNN_PTILE(T, 4, 1, 1, 16, 4),   \
    CADNN_PTILE(T, 4, 2, 1, 16, 4),   \
    CADNN_PTILE(T, 4, 4, 1, 16, 4),   \
    CADNN_PTILE(T, 4, 4, 1, 8, 4),    \
    CADNN_PTILE(T, 4, 8, 1, 8, 4),    \
    CADNN_PTILE(T, 2, 4, 1, 16, 4),   \
    CADNN_PTILE(T, 2, 8, 1, 16, 4),   \
    CADNN_PTILE(T, 2, 8, 1, 8, 4),    \
    CADNN_PTILE(T, 1, 8, 1, 16, 4)

const std::vector<ConvVariant>& all_ptile_variants() {
    static const std::vector<ConvVariant> v = {CADNN_PTILE_SHAPES(float), CADNN_PTILE_SHAPES(_Float16)};
    return v;
}

}  // namespace cadnn
