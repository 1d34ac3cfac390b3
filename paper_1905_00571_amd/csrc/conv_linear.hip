// Linear-address sparse convolution for gfx950 (wave64): no staging, no bounds handling.
//
// Lanes of a wave are consecutive flattened output pixels of one image.  The input tensor
// is read in a layout whose zero halo covers the layer's padding (1x1 filters need none),
// so the address of the activation a nonzero weight multiplies is simply
//     base(image) + soffset(channel, tap: uniform, precomputed in the plan)
//                 + voffset(lane: fixed for the whole kernel)
// and the inner loop per nonzero is one buffer load and one FMA with the weight as scalar
// operand (a filter element is loaded once per wave and reused by all its pixels: the
// paper's redundant filter-load elimination, Section 4).  The (value, offset) pairs are
// streamed with coalesced vector loads, 64 pairs per wave-wide load and one such load
// ahead, and broadcast to scalar registers lane by lane: a scalar load per group of
// nonzeros would expose a cache-miss latency every few FMAs.  A 1x1 layer is the same
// loop: a sparse-matrix x dense-matrix product (Section 4: 1x1 convolution as matrix
// multiply).  Keeping the halo of every activation
// buffer at zero is the layout transformation ("padding", Section 4) that removes the
// irregular border handling from the hot loop.
//
// The loop is software-pipelined by hand: the activations of group g+1 are in flight
// while group g is accumulated.
// KS waves may split a row's nonzeros evenly; partial sums meet in LDS before the fused
// bias / residual / ReLU epilogue (Section 4: conv + batch-norm + activation fused).
#include "internal.h"

namespace cadnn {

constexpr int kDwPlaneMax = 30 * 30;            // fused depthwise: image sides up to 28, plus a 1-pixel halo
constexpr uint32_t kLinOutOfRange = 0x7ffffff0u;   // beyond any buffer this library accepts

// ADJ = 0: the P pixels of a lane are 64 apart (P wave-wide loads of one element each);
// ADJ = 1: they are P adjacent pixels of one output row fetched with ONE P-element load
//          (stride-1 layers whose output width is a multiple of P): fewer, wider loads and
//          fewer cache lines touched per useful byte.
// ADJ = 2: the same for rows that do NOT split into groups of P ("ragged"): the pixels are
//          enumerated over rows of wq = width rounded up to P positions, so a lane's group
//          never straddles two rows; the positions past a row's end are computed (their
//          loads stay inside the buffer or read as zero) and not stored.  Kept apart
//          because the extra bookkeeping costs the even-width layers about 1 %.
// S2D = 1: the instantiation understands de-interleaved tensors (TensorDesc::s2d) on its
//          output, residual and -- for pixel-wise layers -- input.  Kept apart because the
//          general address arithmetic costs every launch a fraction of a microsecond.
// DUAL = 1: a second sparse matrix on a second input tensor is accumulated into the same
//          outputs: a 1x1 projection shortcut fused into the layer it would have been the
//          residual of (the shortcut's kernel launch, its output write and the residual
//          read disappear).  A part of the stream is then the layer's entries followed by
//          the shortcut's, and the header is {length, channel, shortcut length, -}.
// POOL = 1: the layer's only reader is a global average pool and one pixel tile covers the
//          image: the epilogue averages the wave's pixels and writes the pooled vector;
//          the feature map itself is never written.
template <typename T_, int P_, int RPW_, int KS_, int NW_, int U_, int ADJ_ = 0, int S2D_ = 0, int DUAL_ = 0,
          int POOL_ = 0, int DW_ = 0>
struct LinearCfg {
    using T = T_;
    static constexpr int P = P_, RPW = RPW_, KS = KS_, NW = NW_, U = U_, ADJ = ADJ_, S2D = S2D_, DUAL = DUAL_,
                         POOL = POOL_, DW = DW_;
    static_assert(!(S2D && DUAL) && !(POOL && (S2D || DUAL || ADJ)), "not combined");
    static_assert(!(DW && (S2D || DUAL || POOL)), "not combined");
    static_assert(DW != 2 || (KS == 1 && ADJ == 0), "tile-per-wave depthwise fusion takes whole rows per wave");
    static_assert(!(ADJ && S2D), "adjacent pixels are not adjacent in a de-interleaved tensor");
    static_assert(ADJ != 2 || (!DUAL && !POOL), "not combined");
    static constexpr int RG = NW / KS;
    static constexpr int THREADS = NW * 64;
    static_assert(NW % KS == 0, "KS must divide the waves of a workgroup");
};

// Wave-wide window over the plan's (value, offset) stream: lane l of `cur` holds entry
// base + l, `nxt` the entry 64 further on (already in flight).
struct NzWindow {
    const uint2* __restrict__ nz;
    int lane;
    int base;
    uint2 cur, nxt;
    __device__ __forceinline__ void reset(int i) {
        base = i;
        cur = nz[base + lane];
        nxt = nz[base + 64 + lane];
    }
    __device__ __forceinline__ void seek(int i) {
        if (i < base || i >= base + 64) reset(i);
    }
    // Broadcasts the U entries starting at absolute index gi (a multiple of U past base).
    template <int U>
    __device__ __forceinline__ void group(int gi, float (&w)[U], uint32_t (&o)[U]) {
        if (gi - base >= 64) {
            cur = nxt;
            base += 64;
            nxt = nz[base + 64 + lane];
        }
        const int l0 = gi - base;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            w[u] = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)cur.x, l0 + u));
            o[u] = (uint32_t)__builtin_amdgcn_readlane((int)cur.y, l0 + u);
        }
    }
};

template <typename T>
__device__ __forceinline__ float lin_load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff);
template <>
__device__ __forceinline__ float lin_load<float>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
}
template <>
__device__ __forceinline__ float lin_load<_Float16>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    const unsigned short h = __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
    return (float)__builtin_bit_cast(_Float16, h);
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

// Activations of one nonzero for the P pixels of a lane: fp32 values, or -- in 2-byte storage --
// the raw halves as loaded (one per register when the pixels are 64 apart, packed pairs when
// they are adjacent), which the mixed-precision FMA below consumes without a conversion.
template <typename T, int P, int ADJ>
struct LinX {
    float v[P];
};
template <int P, int ADJ>
struct LinX<_Float16, P, ADJ> {
    uint32_t r[(ADJ != 0 && P > 1) ? P / 2 : P];
};

template <typename T, int P, int ADJ>
__device__ __forceinline__ void lin_fetch(__amdgpu_buffer_rsrc_t r, const uint32_t (&voff)[P], uint32_t soff,
                                          LinX<T, P, ADJ>& x) {
    if constexpr (sizeof(T) == 4) {
        if constexpr (ADJ == 0 || P == 1) {
#pragma unroll
            for (int j = 0; j < P; ++j) x.v[j] = lin_load<T>(r, voff[j], soff);
        } else if constexpr (P == 2) {
            const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, voff[0], soff, 0);
            x.v[0] = __uint_as_float(v[0]); x.v[1] = __uint_as_float(v[1]);
        } else {
            static_assert(P == 4, "unsupported adjacent-pixel width");
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff[0], soff, 0);
            x.v[0] = __uint_as_float(v[0]); x.v[1] = __uint_as_float(v[1]);
            x.v[2] = __uint_as_float(v[2]); x.v[3] = __uint_as_float(v[3]);
        }
    } else {
        if constexpr (ADJ == 0 || P == 1) {
#pragma unroll
            for (int j = 0; j < P; ++j) x.r[j] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, voff[j], soff, 0);
        } else if constexpr (P == 2) {
            x.r[0] = __builtin_amdgcn_raw_buffer_load_b32(r, voff[0], soff, 0);
        } else {
            static_assert(P == 4, "unsupported adjacent-pixel width");
            const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, voff[0], soff, 0);
            x.r[0] = v[0]; x.r[1] = v[1];
        }
    }
}

// acc + w * (the low / high half of xh as binary16), one instruction, the product and sum in
// fp32: what a conversion followed by an fp32 FMA computes, bit for bit.
__device__ __forceinline__ float fma_mix_lo(float w, uint32_t xh, float acc) {
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[0,1,0]" : "=v"(d) : "s"(w), "v"(xh), "v"(acc));
    return d;
}
__device__ __forceinline__ float fma_mix_hi(float w, uint32_t xh, float acc) {
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,1,0] op_sel_hi:[0,1,0]" : "=v"(d) : "s"(w), "v"(xh), "v"(acc));
    return d;
}

// acc[j] += w * x[j] for the P pixels of a lane (w is wave-uniform).
template <typename T, int P, int ADJ>
__device__ __forceinline__ void lin_mac(float w, const LinX<T, P, ADJ>& x, float (&acc)[P]) {
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int j = 0; j < P; ++j) acc[j] = fmaf(w, x.v[j], acc[j]);
    } else if constexpr (ADJ == 0 || P == 1) {
#pragma unroll
        for (int j = 0; j < P; ++j) acc[j] = fma_mix_lo(w, x.r[j], acc[j]);
    } else {
#pragma unroll
        for (int k = 0; k < P / 2; ++k) {
            acc[2 * k] = fma_mix_lo(w, x.r[k], acc[2 * k]);
            acc[2 * k + 1] = fma_mix_hi(w, x.r[k], acc[2 * k + 1]);
        }
    }
}

// Entries [i, end) of the stream (end - i a positive multiple of U) against the P pixels of
// a lane.  Two register sets (A, B) take turns: while one group is accumulated the
// activations of the next are in flight.
template <class Cfg>
__device__ __forceinline__ void lin_accumulate(__amdgpu_buffer_rsrc_t rsrc, const uint32_t (&voff)[Cfg::P], NzWindow& win,
                                               int i, int end, float (&acc)[Cfg::P]) {
    using T = typename Cfg::T;
    constexpr int P = Cfg::P, U = Cfg::U, ADJ = Cfg::ADJ;
    win.seek(i);
    int groups = (end - i) / U;
    float wa[U], wb[U];
    LinX<T, P, ADJ> xa[U], xb[U];
    uint32_t oa[U], ob[U];
    win.group<U>(i, wa, oa);
#pragma unroll
    for (int u = 0; u < U; ++u) lin_fetch<T, P, ADJ>(rsrc, voff, oa[u], xa[u]);
    while (true) {
        if (groups == 1) {
#pragma unroll
            for (int u = 0; u < U; ++u) lin_mac<T, P, ADJ>(wa[u], xa[u], acc);
            break;
        }
        win.group<U>(i + U, wb, ob);
#pragma unroll
        for (int u = 0; u < U; ++u) lin_fetch<T, P, ADJ>(rsrc, voff, ob[u], xb[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) lin_mac<T, P, ADJ>(wa[u], xa[u], acc);
        if (groups == 2) {
#pragma unroll
            for (int u = 0; u < U; ++u) lin_mac<T, P, ADJ>(wb[u], xb[u], acc);
            break;
        }
        win.group<U>(i + 2 * U, wa, oa);
#pragma unroll
        for (int u = 0; u < U; ++u) lin_fetch<T, P, ADJ>(rsrc, voff, oa[u], xa[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) lin_mac<T, P, ADJ>(wb[u], xb[u], acc);
        groups -= 2;
        i += 2 * U;
    }
}

// Output pixel served by flattened index q.  Normally row-major.  A pixel-wise layer on a
// de-interleaved input walks the pixels parity class by parity class instead (all pixels of
// one row/column parity, row-major, then the next class), which is the order they lie in
// memory: consecutive lanes then read consecutive elements again.
__device__ __forceinline__ void lin_pixel(const ConvLaunch& a, int q, int& oh, int& ow) {
    if (a.xd.s2d && a.stride == 1) {
        const int w2 = a.yd.w >> 1, hw2 = (a.yd.h >> 1) * w2;
        const int cls = q / hw2, rem = q - cls * hw2;
        const int i2 = rem / w2, j2 = rem - i2 * w2;
        oh = 2 * i2 + (cls >> 1);
        ow = 2 * j2 + (cls & 1);
    } else {
        oh = q / a.yd.w;
        ow = q - oh * a.yd.w;
    }
}

// One workgroup of one layer: pixel tile bx, row group by, image n.
template <class Cfg>
__device__ __forceinline__ void sconv_linear_block(const ConvLaunch& a, const int bx, const int by, const int n) {
    using T = typename Cfg::T;
    constexpr int P = Cfg::P, RPW = Cfg::RPW, KS = Cfg::KS, RG = Cfg::RG, ADJ = Cfg::ADJ;
    __shared__ float red[KS > 1 ? Cfg::NW * RPW * P * 64 : 1];

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // (DW = 2: the waves of a workgroup take the pixel tiles of ONE group of rows instead of
    // different rows of one pixel tile, so that a channel's whole image meets in LDS)
    constexpr bool TW = Cfg::DW == 2;
    const int rg = TW ? 0 : wv / KS, ks = TW ? 0 : wv % KS;
    // Workgroups in plain launch order.  (Die-aware placements were measured -- workgroup
    // L runs on die L % 8: giving each die its own pixel tiles leaves most of the chip idle
    // on layers with few tiles and gains nothing on the others, and giving each die its
    // own rows changes nothing.)
    const int tile = TW ? wv : bx, grp = by;
    const int q0 = tile * (64 * P);
    const int row0 = TW ? grp * RPW : (grp * RG + rg) * RPW;

    // byte offset of tap (0,0) of each of the lane's pixels inside the padded image (in a
    // de-interleaved input the taps of a stride-2 layer follow at the plan's offsets too)
    uint32_t voff[P];
    int oidx[P];
    const int base = a.xd.origin - a.pad * a.xd.pitch - a.pad;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const int q = ADJ ? q0 + lane * P + j : q0 + j * 64 + lane;
        int oh, ow;
        if constexpr (Cfg::S2D) {
            lin_pixel(a, q, oh, ow);
            oidx[j] = q < a.hwout ? tensor_off(a.yd, oh, ow) : -1;
            voff[j] = q < a.hwout
                          ? (uint32_t)tensor_off(a.xd, oh * a.stride - a.pad, ow * a.stride - a.pad) * (uint32_t)sizeof(T)
                          : kLinOutOfRange;
        } else if constexpr (ADJ == 2) {
            // ragged rows: the lane's one wide load starts at its first pixel, which is always
            // in the row; later pixels of the group may lie past the row's end
            oh = q / a.wq;
            ow = q - oh * a.wq;
            oidx[j] = (q < a.hwq && (j == 0 || ow < a.yd.w)) ? a.yd.origin + oh * a.yd.pitch + ow : -1;
            voff[j] = q < a.hwq
                          ? (uint32_t)(base + oh * a.stride * a.xd.pitch + ow * a.stride) * (uint32_t)sizeof(T)
                          : kLinOutOfRange;
        } else {
            oh = q / a.yd.w;
            ow = q - oh * a.yd.w;
            oidx[j] = q < a.hwout ? a.yd.origin + oh * a.yd.pitch + ow : -1;
            voff[j] = q < a.hwout
                          ? (uint32_t)(base + oh * a.stride * a.xd.pitch + ow * a.stride) * (uint32_t)sizeof(T)
                          : kLinOutOfRange;
        }
    }
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const char*)a.x + (size_t)n * a.image_bytes), 0, a.image_bytes, 0x00020000);
    // fused shortcut: the same pixels in the second input (a 1x1 filter: one tap, no padding)
    uint32_t voff2[Cfg::DUAL ? P : 1];
    __amdgpu_buffer_rsrc_t rsrc2 = rsrc;
    if constexpr (Cfg::DUAL) {
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const int q = ADJ ? q0 + lane * P + j : q0 + j * 64 + lane;
            const int oh = q / a.yd.w, ow = q - oh * a.yd.w;
            voff2[j] = q < a.hwout
                           ? (uint32_t)(a.x2d.origin + oh * a.stride2 * a.x2d.pitch + ow * a.stride2) * (uint32_t)sizeof(T)
                           : kLinOutOfRange;
        }
        rsrc2 = __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)a.x2 + (size_t)n * a.image2_bytes), 0,
                                                  a.image2_bytes, 0x00020000);
    }

    // Header {padded length, original channel} of each of the wave's parts.  A part starts
    // at (row*KS + ks) * stride, so the first window of the first row is requested in the
    // same breath as the headers and the bias follows one round trip later, in parallel
    // with the first activations.
    const int stride = a.nchunks;
    const int2* __restrict__ hdr = (const int2*)a.seg_ptr;
    NzWindow win;
    win.nz = a.nz;
    win.lane = lane;
    win.reset(((row0 + 0) * KS + ks) * stride);
    int co_[RPW], len_[RPW], len2_[RPW];
    float bias_[RPW];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        if constexpr (Cfg::DUAL) {
            const int4 h = ((const int4*)a.seg_ptr)[(row0 + r) * KS + ks];
            len_[r] = h.x;
            co_[r] = h.y;
            len2_[r] = h.z;
        } else {
            const int2 h = hdr[(row0 + r) * KS + ks];
            len_[r] = h.x;
            co_[r] = h.y;
            len2_[r] = 0;
        }
    }
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        bias_[r] = (a.bias && co_[r] >= 0) ? a.bias[co_[r]] : 0.0f;
        if constexpr (Cfg::DUAL) bias_[r] += (a.bias2 && co_[r] >= 0) ? a.bias2[co_[r]] : 0.0f;
    }

    // the residual is also fetched up front: one more round trip off the tail
    const T* __restrict__ res = a.residual ? (const T*)a.residual + (size_t)n * a.rd.image : nullptr;
    float resv[RPW][P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const int q = ADJ ? q0 + lane * P + j : q0 + j * 64 + lane;
        int oh, ow, ridx;
        if constexpr (Cfg::S2D) {
            lin_pixel(a, q, oh, ow);
            ridx = tensor_off(a.rd, oh, ow);
        } else {
            const int wq = ADJ == 2 ? a.wq : a.yd.w;
            oh = q / wq;
            ow = q - oh * wq;
            ridx = a.rd.origin + oh * a.rd.pitch + ow;
        }
#pragma unroll
        for (int r = 0; r < RPW; ++r)
            resv[r][j] = (res && ks == 0 && co_[r] >= 0 && oidx[j] >= 0) ? (float)res[(size_t)co_[r] * a.rd.plane + ridx] : 0.0f;
    }

    float acc[RPW][P];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
#pragma unroll
        for (int j = 0; j < P; ++j) acc[r][j] = 0.0f;
        const int i = ((row0 + r) * KS + ks) * stride;
        if (len_[r] > 0) lin_accumulate<Cfg>(rsrc, voff, win, i, i + len_[r], acc[r]);
        if constexpr (Cfg::DUAL) {
            if (len2_[r] > 0) lin_accumulate<Cfg>(rsrc2, voff2, win, i + len_[r], i + len_[r] + len2_[r], acc[r]);
        }
    }

    if (KS > 1) {
        // partial sums of the KS slices meet in LDS; slice 0 finishes the row
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

    if constexpr (Cfg::POOL) {
        // ---- fused epilogue + global average pool: every pixel of the channel is in this
        //      wave (each value rounded to the storage type first, as the separate pool
        //      would have read it), summed across the wavefront
        T* __restrict__ py = (T*)a.pool_y + (size_t)n * a.cout;
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const int co = co_[r];
            float sum = 0.0f;
#pragma unroll
            for (int j = 0; j < P; ++j) {
                float v = acc[r][j] + bias_[r] + resv[r][j];
                if (a.relu) v = v > 0.0f ? v : 0.0f;
                sum += oidx[j] >= 0 ? (float)(T)v : 0.0f;
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
            if (lane == 0 && co >= 0) py[co] = (T)(sum * a.pool_scale);
        }
        return;
    }

    if constexpr (Cfg::DW) {
        // ---- fused epilogue + 3x3 depthwise layer (padding 1): the whole image of each of the
        //      wave's channels is in this wave.  It goes, rounded to the storage type as the
        //      separate layer would have read it, into a zero-haloed LDS plane of the wave's
        //      own; the lanes then take the depthwise outputs of the channel from there.
        __shared__ float dwbuf[TW ? 1 : Cfg::RG][kDwPlaneMax];
        float* pl = dwbuf[rg];
        const int pitch = a.yd.w + 2;
        // who shares a plane: the wave alone, or (tile per wave) the whole workgroup
        const int me = TW ? (int)threadIdx.x : lane, team = TW ? Cfg::THREADS : 64;
        auto team_sync = [&]() {
            if constexpr (TW) {
                __syncthreads();
            } else {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        };
        for (int i = me; i < (a.yd.h + 2) * pitch; i += team) pl[i] = 0.0f;
        T* __restrict__ y2 = (T*)a.dw_y + (size_t)n * a.dw_yd.image;
        const int w2 = a.dw_yd.w, hw2 = a.dw_yd.h * w2;
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const int co = co_[r];
            if (co < 0) continue;
            // (the previous channel's reads are done before its plane is overwritten; co is the
            // same for every wave that shares the plane, so they all come here)
            team_sync();
#pragma unroll
            for (int j = 0; j < P; ++j) {
                if (oidx[j] >= 0) {
                    const int q = q0 + (ADJ ? lane * P + j : j * 64 + lane);
                    const int oh = q / a.yd.w, ow = q - oh * a.yd.w;
                    float v = acc[r][j] + bias_[r] + resv[r][j];
                    if (a.relu) v = v > 0.0f ? v : 0.0f;
                    pl[(oh + 1) * pitch + ow + 1] = (float)(T)v;
                }
            }
            team_sync();
            const float* __restrict__ wt = a.dw_w + (size_t)co * 9;
            const float b2 = a.dw_bias ? a.dw_bias[co] : 0.0f;
            for (int t = me; t < hw2; t += team) {
                const int oh2 = t / w2, ow2 = t - oh2 * w2;
                const float* tap = pl + oh2 * a.dw_stride * pitch + ow2 * a.dw_stride;
                float sum = 0.0f;
#pragma unroll
                for (int i = 0; i < 3; ++i)
#pragma unroll
                    for (int k = 0; k < 3; ++k) {
                        const float wv = wt[i * 3 + k];
                        if (wv != 0.0f) sum = fmaf(wv, tap[i * pitch + k], sum);
                    }
                float v2 = sum + b2;
                if (a.dw_relu) v2 = v2 > 0.0f ? v2 : 0.0f;
                y2[(size_t)co * a.dw_yd.plane + a.dw_yd.origin + oh2 * a.dw_yd.pitch + ow2] = (T)v2;
            }
        }
        return;
    }

    // ---- fused epilogue: + bias, + residual, ReLU, store at the original channel
    T* __restrict__ y = (T*)a.y + (size_t)n * a.yd.image;
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
__global__ __launch_bounds__(Cfg::THREADS) void sconv_linear_kernel(const ConvLaunch a) {
    sconv_linear_block<Cfg>(a, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z);
}

// Several independent layers in one launch (the branches of an Inception module at the same
// depth).  blockIdx.x runs over the workgroups of all layers, layer after layer -- first[k] is
// the first workgroup of layer k, first[layers] the total, at most kMaxCoLaunch layers --
// and blockIdx.y is the image, so no workgroup is launched in vain (a common bounding grid
// was measured first: 5000 workgroups outside their layer's own grid cost a 17x17 module 8 us).
// The layer's launch record is read from a table in device memory: a wave-uniform address,
// so it arrives through the scalar cache like the kernel arguments would.
struct CoLaunchHeader {
    int first[kMaxCoLaunch + 1];
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void sconv_linear_multi_kernel(const ConvLaunch* __restrict__ table,
                                                                         const CoLaunchHeader h, const int layers) {
    const int b = (int)blockIdx.x;
    int layer = 0, base = 0;
#pragma unroll
    for (int k = 1; k < kMaxCoLaunch; ++k)
        if (k < layers && b >= h.first[k]) { layer = k; base = h.first[k]; }
    const ConvLaunch a = table[layer];
    const int local = b - base;
    const int by = local / a.tiles_x, bx = local - by * a.tiles_x;
    const int n = (int)blockIdx.y;
    if (a.op_type != 0) {
        // a window pool riding along (a module's pooled branch): its output elements dealt
        // round robin to the threads of its workgroups
        using T = typename Cfg::T;
        const size_t elems = (size_t)a.yd.c * a.yd.h * a.yd.w, step = (size_t)a.tiles_x * a.row_groups * Cfg::THREADS;
        for (size_t r = (size_t)local * Cfg::THREADS + threadIdx.x; r < elems; r += step)
            windowpool_element<T>((const T*)a.x, (T*)a.y, a.xd, a.yd, n, r, a.pool_k, a.stride, a.pad, a.op_type == 2);
        return;
    }
    sconv_linear_block<Cfg>(a, bx, by, n);
}

template <class Cfg>
static hipError_t launch_linear(const ConvLaunch& a, hipStream_t s) {
    dim3 grid((unsigned)a.tiles_x, (unsigned)a.row_groups, (unsigned)a.n);
    dim3 block(Cfg::THREADS);
    CADNN_LAUNCH(sconv_linear_kernel<Cfg>, grid, block, 0, s, a);
    return hipGetLastError();
}

template <class Cfg>
static hipError_t launch_linear_multi(const ConvLaunch* table, const ConvLaunch* host_records, int layers, int images,
                                      hipStream_t s) {
    CoLaunchHeader h{};
    int total = 0;
    for (int k = 0; k < layers; ++k) {
        h.first[k] = total;
        total += host_records[k].tiles_x * host_records[k].row_groups;
    }
    for (int k = layers; k <= kMaxCoLaunch; ++k) h.first[k] = total;
    dim3 grid((unsigned)total, (unsigned)images, 1);
    dim3 block(Cfg::THREADS);
    CADNN_LAUNCH(sconv_linear_multi_kernel<Cfg>, grid, block, 0, s, table, h, layers);
    return hipGetLastError();
}

template <class Cfg>
static ConvVariant make_linear(const char* name) {
    ConvVariant v{};
    v.name = name;
    v.family = FAM_LINEAR;
    v.is_f16 = sizeof(typename Cfg::T) == 2;
    v.kh = 0; v.kw = 0; v.stride = 0;
    v.p = Cfg::P; v.nw = Cfg::NW; v.rpw = Cfg::RPW; v.ks = Cfg::KS;
    v.unroll = Cfg::U;
    v.adjacent = Cfg::ADJ;
    v.s2d = Cfg::S2D;
    v.dual = Cfg::DUAL;
    v.pool = Cfg::POOL;
    v.dw = Cfg::DW;
    if (Cfg::DW == 2) {
        v.nw = 1;                    // rows per workgroup = RPW: its waves split the pixels, not the rows
        v.tw = Cfg::NW;              // ... this many waves, i.e. pixel tiles
    }
    v.lds_bytes = Cfg::KS > 1 ? (size_t)Cfg::NW * Cfg::RPW * Cfg::P * 64 * 4 : 0;
    v.launch = &launch_linear<Cfg>;
    // (plain instantiations only: a fused second input, pool or depthwise epilogue, or a
    // de-interleaved tensor keeps a layer on a launch of its own)
    if constexpr (!Cfg::S2D && !Cfg::DUAL && !Cfg::POOL && !Cfg::DW) v.launch_multi = &launch_linear_multi<Cfg>;
    return v;
}

#define CADNN_LINEAR(T, P, RPW, KS, NW, U) \
    make_linear<LinearCfg<T, P, RPW, KS, NW, U>>("slinear_" #T "_p" #P "_r" #RPW "k" #KS "w" #NW "u" #U)

#define CADNN_LINEAR_ADJ(T, P, RPW, KS, NW, U) \
    make_linear<LinearCfg<T, P, RPW, KS, NW, U, 1>>("slinear_" #T "_a" #P "_r" #RPW "k" #KS "w" #NW "u" #U)

#define CADNN_LINEAR_RAGGED(T, P, RPW, KS, NW, U) \
    make_linear<LinearCfg<T, P, RPW, KS, NW, U, 2>>("slinear_" #T "_g" #P "_r" #RPW "k" #KS "w" #NW "u" #U)

#define CADNN_LINEAR_S2D(T, P, RPW, KS, NW, U) \
    make_linear<LinearCfg<T, P, RPW, KS, NW, U, 0, 1>>("slinear_" #T "_d" #P "_r" #RPW "k" #KS "w" #NW "u" #U)

#define CADNN_LINEAR_DUAL(T, P, RPW, KS, NW, U) \
    make_linear<LinearCfg<T, P, RPW, KS, NW, U, 0, 0, 1>>("slinear_" #T "_fp" #P "_r" #RPW "k" #KS "w" #NW "u" #U)

#define CADNN_LINEAR_DUAL_ADJ(T, P, RPW, KS, NW, U) \
    make_linear<LinearCfg<T, P, RPW, KS, NW, U, 1, 0, 1>>("slinear_" #T "_fa" #P "_r" #RPW "k" #KS "w" #NW "u" #U)

#define CADNN_LINEAR_POOL(T, P, RPW, KS, NW, U) \
    make_linear<LinearCfg<T, P, RPW, KS, NW, U, 0, 0, 0, 1>>("slinear_" #T "_gp" #P "_r" #RPW "k" #KS "w" #NW "u" #U)

#define CADNN_LINEAR_DW(T, P, RPW, KS, NW, U) \
    make_linear<LinearCfg<T, P, RPW, KS, NW, U, 0, 0, 0, 0, 1>>("slinear_" #T "_dw" #P "_r" #RPW "k" #KS "w" #NW "u" #U)

#define CADNN_LINEAR_DW_TILES(T, RPW, NW, U) \
    make_linear<LinearCfg<T, 1, RPW, 1, NW, U, 0, 0, 0, 0, 2>>("slinear_" #T "_dt1_r" #RPW "k1w" #NW "u" #U)

#define CADNN_LINEAR_SHAPES(T)          \
    CADNN_LINEAR_DW_TILES(T, 1, 4, 4), \
    CADNN_LINEAR_DW_TILES(T, 1, 4, 8), \
    CADNN_LINEAR_DW_TILES(T, 1, 4, 16), \
    CADNN_LINEAR_DW_TILES(T, 2, 4, 4), \
    CADNN_LINEAR_DW_TILES(T, 2, 4, 8), \
    CADNN_LINEAR_DW_TILES(T, 1, 16, 4), \
    CADNN_LINEAR_DW_TILES(T, 1, 16, 8), \
    CADNN_LINEAR_DW_TILES(T, 2, 16, 4), \
    CADNN_LINEAR_RAGGED(T, 2, 1, 1, 4, 4), \
    CADNN_LINEAR_RAGGED(T, 2, 1, 1, 4, 8), \
    CADNN_LINEAR_RAGGED(T, 2, 1, 2, 4, 4), \
    CADNN_LINEAR_RAGGED(T, 2, 1, 2, 4, 8), \
    CADNN_LINEAR_RAGGED(T, 2, 1, 4, 4, 4), \
    CADNN_LINEAR_RAGGED(T, 2, 1, 4, 4, 8), \
    CADNN_LINEAR_RAGGED(T, 2, 1, 8, 8, 4), \
    CADNN_LINEAR_RAGGED(T, 2, 2, 1, 4, 4), \
    CADNN_LINEAR_RAGGED(T, 4, 1, 1, 4, 4), \
    CADNN_LINEAR_RAGGED(T, 4, 1, 1, 4, 8), \
    CADNN_LINEAR_RAGGED(T, 4, 1, 2, 4, 4), \
    CADNN_LINEAR_RAGGED(T, 4, 1, 2, 4, 8), \
    CADNN_LINEAR_RAGGED(T, 4, 1, 4, 4, 4), \
    CADNN_LINEAR_RAGGED(T, 4, 1, 4, 4, 8), \
    CADNN_LINEAR_RAGGED(T, 4, 1, 8, 8, 4), \
    CADNN_LINEAR_RAGGED(T, 4, 2, 1, 4, 4), \
    CADNN_LINEAR_DW(T, 1, 1, 1, 4, 4), \
    CADNN_LINEAR_DW(T, 1, 1, 1, 4, 8), \
    CADNN_LINEAR_DW(T, 1, 1, 2, 4, 4), \
    CADNN_LINEAR_DW(T, 1, 1, 2, 4, 8), \
    CADNN_LINEAR_DW(T, 1, 1, 4, 4, 4), \
    CADNN_LINEAR_DW(T, 1, 1, 4, 4, 8), \
    CADNN_LINEAR_DW(T, 1, 1, 8, 8, 4), \
    CADNN_LINEAR_POOL(T, 1, 1, 1, 4, 4), \
    CADNN_LINEAR_POOL(T, 1, 1, 1, 4, 8), \
    CADNN_LINEAR_POOL(T, 1, 1, 2, 4, 4), \
    CADNN_LINEAR_POOL(T, 1, 1, 2, 4, 8), \
    CADNN_LINEAR_POOL(T, 1, 1, 4, 4, 4), \
    CADNN_LINEAR_POOL(T, 1, 1, 4, 4, 8), \
    CADNN_LINEAR_POOL(T, 1, 1, 8, 8, 4), \
    CADNN_LINEAR_POOL(T, 2, 1, 2, 4, 4), \
    CADNN_LINEAR_POOL(T, 4, 1, 2, 4, 4), \
    CADNN_LINEAR_DUAL(T, 1, 1, 1, 4, 4), \
    CADNN_LINEAR_DUAL(T, 1, 1, 1, 4, 8), \
    CADNN_LINEAR_DUAL(T, 1, 1, 2, 4, 4), \
    CADNN_LINEAR_DUAL(T, 1, 1, 2, 4, 8), \
    CADNN_LINEAR_DUAL(T, 1, 1, 4, 4, 4), \
    CADNN_LINEAR_DUAL(T, 1, 1, 4, 4, 8), \
    CADNN_LINEAR_DUAL(T, 1, 1, 8, 8, 4), \
    CADNN_LINEAR_DUAL(T, 1, 2, 1, 4, 4), \
    CADNN_LINEAR_DUAL(T, 2, 1, 1, 4, 4), \
    CADNN_LINEAR_DUAL(T, 2, 1, 2, 4, 4), \
    CADNN_LINEAR_DUAL_ADJ(T, 2, 1, 1, 4, 4), \
    CADNN_LINEAR_DUAL_ADJ(T, 2, 1, 2, 4, 4), \
    CADNN_LINEAR_DUAL_ADJ(T, 2, 1, 4, 4, 4), \
    CADNN_LINEAR_DUAL_ADJ(T, 4, 1, 1, 4, 4), \
    CADNN_LINEAR_DUAL_ADJ(T, 4, 1, 2, 4, 4), \
    CADNN_LINEAR_DUAL_ADJ(T, 4, 1, 4, 4, 4), \
    CADNN_LINEAR_S2D(T, 1, 1, 1, 4, 4), \
    CADNN_LINEAR_S2D(T, 1, 1, 1, 4, 8), \
    CADNN_LINEAR_S2D(T, 1, 1, 1, 4, 16), \
    CADNN_LINEAR_S2D(T, 1, 1, 2, 4, 4), \
    CADNN_LINEAR_S2D(T, 1, 1, 2, 4, 8), \
    CADNN_LINEAR_S2D(T, 1, 1, 4, 4, 4), \
    CADNN_LINEAR_S2D(T, 1, 1, 4, 4, 8), \
    CADNN_LINEAR_S2D(T, 1, 1, 8, 8, 4), \
    CADNN_LINEAR_S2D(T, 1, 2, 1, 4, 4), \
    CADNN_LINEAR_S2D(T, 1, 2, 1, 4, 8), \
    CADNN_LINEAR_S2D(T, 2, 1, 1, 4, 4), \
    CADNN_LINEAR_S2D(T, 2, 1, 2, 4, 4), \
    CADNN_LINEAR_S2D(T, 2, 1, 2, 4, 8), \
    CADNN_LINEAR_S2D(T, 2, 1, 4, 4, 4), \
    CADNN_LINEAR_S2D(T, 2, 2, 1, 4, 4), \
    CADNN_LINEAR_ADJ(T, 2, 1, 1, 4, 4), \
    CADNN_LINEAR_ADJ(T, 2, 1, 2, 4, 4), \
    CADNN_LINEAR_ADJ(T, 2, 1, 4, 4, 4), \
    CADNN_LINEAR_ADJ(T, 2, 1, 4, 4, 8), \
    CADNN_LINEAR_ADJ(T, 2, 1, 8, 8, 4), \
    CADNN_LINEAR_ADJ(T, 2, 2, 1, 4, 4), \
    CADNN_LINEAR_ADJ(T, 4, 1, 1, 4, 4), \
    CADNN_LINEAR_ADJ(T, 4, 1, 2, 4, 4), \
    CADNN_LINEAR_ADJ(T, 4, 1, 4, 4, 4), \
    CADNN_LINEAR_ADJ(T, 4, 1, 8, 8, 4), \
    CADNN_LINEAR_ADJ(T, 4, 2, 1, 4, 4), \
    CADNN_LINEAR_ADJ(T, 4, 1, 16, 16, 4), \
    CADNN_LINEAR_ADJ(T, 2, 1, 1, 4, 16), \
    CADNN_LINEAR_ADJ(T, 2, 1, 2, 4, 16), \
    CADNN_LINEAR_ADJ(T, 2, 1, 4, 4, 16), \
    CADNN_LINEAR_ADJ(T, 4, 1, 1, 4, 16), \
    CADNN_LINEAR_ADJ(T, 4, 1, 2, 4, 16), \
    CADNN_LINEAR_ADJ(T, 4, 1, 4, 4, 16), \
    CADNN_LINEAR_ADJ(T, 4, 1, 1, 4, 8),  \
    CADNN_LINEAR_ADJ(T, 4, 1, 2, 4, 8),  \
    CADNN_LINEAR_ADJ(T, 4, 1, 4, 4, 8),  \
    CADNN_LINEAR_ADJ(T, 2, 1, 1, 4, 8),  \
    CADNN_LINEAR_ADJ(T, 2, 1, 2, 4, 8),  \
    CADNN_LINEAR(T, 1, 1, 1, 4, 4),     \
    CADNN_LINEAR(T, 1, 1, 1, 4, 8),     \
    CADNN_LINEAR(T, 1, 1, 1, 4, 16),    \
    CADNN_LINEAR(T, 1, 1, 2, 4, 16),    \
    CADNN_LINEAR(T, 1, 1, 4, 4, 16),    \
    CADNN_LINEAR(T, 1, 1, 8, 8, 16),    \
    CADNN_LINEAR(T, 1, 1, 16, 16, 16),  \
    CADNN_LINEAR(T, 1, 1, 16, 16, 8),   \
    CADNN_LINEAR(T, 2, 1, 4, 4, 8),     \
    CADNN_LINEAR(T, 2, 1, 2, 4, 8),     \
    CADNN_LINEAR(T, 1, 2, 1, 4, 4),     \
    CADNN_LINEAR(T, 1, 2, 1, 4, 8),     \
    CADNN_LINEAR(T, 1, 4, 1, 4, 4),     \
    CADNN_LINEAR(T, 2, 1, 1, 4, 4),     \
    CADNN_LINEAR(T, 2, 2, 1, 4, 4),     \
    CADNN_LINEAR(T, 2, 4, 1, 4, 4),     \
    CADNN_LINEAR(T, 4, 2, 1, 4, 4),     \
    CADNN_LINEAR(T, 4, 4, 1, 4, 2),     \
    CADNN_LINEAR(T, 1, 1, 2, 4, 4),     \
    CADNN_LINEAR(T, 1, 1, 2, 4, 8),     \
    CADNN_LINEAR(T, 1, 1, 4, 4, 4),     \
    CADNN_LINEAR(T, 1, 1, 4, 4, 8),     \
    CADNN_LINEAR(T, 1, 2, 4, 4, 4),     \
    CADNN_LINEAR(T, 1, 1, 8, 8, 4),     \
    CADNN_LINEAR(T, 1, 1, 8, 8, 8),     \
    CADNN_LINEAR(T, 1, 1, 16, 16, 4),   \
    CADNN_LINEAR(T, 2, 1, 4, 4, 4)

const std::vector<ConvVariant>& all_linear_variants() {
    static const std::vector<ConvVariant> v = {CADNN_LINEAR_SHAPES(float), CADNN_LINEAR_SHAPES(_Float16)};
    return v;
}

}  // namespace cadnn
