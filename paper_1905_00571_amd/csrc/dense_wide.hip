// Dense implicit-GEMM convolution on the matrix cores for fp16 storage, large tiles (gfx950).
//
// Y[Cout x pixels] = W[Cout x K] * X~[K x pixels] with K ordered tap-major, k = tap * Cin + ci,
// so that the eight consecutive k values an MFMA lane supplies are eight consecutive input
// channels of one filter tap.  It is the dense side of the dense-vs-compressed comparison
// (paper Section 5) at the batch sizes where a layer is a real contraction, and a candidate
// the per-layer selection may pick for any layer in fp16 storage (Section 4, parameter
// selection by measurement), whatever its sparsity: a pruned layer run densely does 1 / density
// times the multiply-adds, at 32 times the vector-ALU rate.
//
// A fused 1x1 projection shortcut (Section 4, layer fusion) is more of K: its weights follow the
// layer's own in every row of the matrix and its input is gathered, with its own stride, for
// the steps behind the layer's own.  De-interleaved tensors are written and read in place.
//
// One workgroup (4 waves, 2 x 2) computes 128 output channels x 128 output pixels; a wave owns
// 64 x 64 as 2 x 2 accumulators of v_mfma_f32_32x32x16_f16 (instantiations with 64 channels
// and/or 64 pixels serve the layers too small to fill the chip with the large tile).  The pixels of a tile are numbered
// over the whole batch (n * Hout * Wout + q), so small images fill their tiles.  K is walked in
// steps of 32 = 32 channels of one tap:
//   * weights [128][32] arrive as 16-byte loads from the reordered matrix and lie in LDS with
//     rows 80 bytes apart (the 16-byte fragment reads of 16 lanes hit 16 different bank groups);
//   * activations [32][128]: gathered from NCHW with buffer loads of 1, 2 or 4 neighbouring
//     pixels of one channel -- address = the pixel group's own offset + tap offset + the
//     thread's first channel, in the vector part, + channel plane, in the scalar part.  With one
//     pixel per load a tap that falls outside the image for a pixel gets an out-of-range offset
//     and reads zero, so any padding works with or without a halo in memory; wider loads are
//     used where every tap of every pixel lies in memory.  The channels a thread holds of a
//     pixel are packed into one LDS write, [pixel][k] with rows 80 bytes apart like the
//     weights: the transposition NCHW needs on the way to the matrix cores happens in
//     registers, and both MFMA operands are single 16-byte LDS reads.
// Global loads run two stages ahead in two register sets.  Within a stage a wave requests the
// stage's fragments from LDS, issues the loads of stage s+2, waits for the set of stage s+1
// and writes it to the other LDS buffer, then multiplies: one barrier per stage.  Epilogue:
// bias, residual, ReLU fused (Section 4).
#include <type_traits>

#include "internal.h"

namespace cadnn {

namespace {

constexpr int WK = 32;
constexpr int kWideTableK = 256;      // longest K walked with a table
constexpr uint32_t kWideOutOfRange = 0x7ffffff0u;

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f32x16w __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4w __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2w __attribute__((ext_vector_type(2)));
typedef float f32x4w __attribute__((ext_vector_type(4)));
typedef float f32x2w __attribute__((ext_vector_type(2)));

struct WideArgs {
    const _Float16* w;        // [cout rounded up to 128][K] reordered tap-major, zero rows beyond cout
    const _Float16* x;
    _Float16* y;
    const float* bias;
    const _Float16* residual;
    TensorDesc xd, yd, rd;
    int n, cout, cin, kh, kw, stride, pad, relu;
    int hwout, total, K, csteps;   // total = n * hwout; csteps = cin / 32; K = row length of w
    // few input channels (cin not a multiple of 32; a network's first layer): K runs over
    // (ci, r, c) in the weights' own order, padded to whole steps, and the gather takes each k's
    // offset and tap from a table the workgroup builds in LDS (64-pixel tiles, one pixel per load)
    int table;
    // a fused 1x1 projection shortcut (x2 != NULL): csteps2 more steps of K read from x2, a
    // plain view walked with stride2 from pixel (0, 0); its bias is added as well
    const _Float16* x2;
    const float* bias2;
    TensorDesc x2d;
    int stride2, csteps2;
    // pixels a thread of the epilogue writes with one store (8, 4 or 2: they lie side by side
    // in the output and the residual, suitably aligned), or 0; then `rows`: pixels of one image
    // row a thread finishes together (8, 4 or 2: the rows split into such groups, whatever the
    // layout), or 0: one pixel per store straight from the accumulators
    int group, rows;
    // neighbouring pixels of a row one gather load takes (1, 2 or 4): the input is walked with unit
    // stride, every tap of every pixel lies in memory (no padding, or a halo that holds it), groups
    // do not straddle rows and there is no fused shortcut
    int gather;
    // K split over `sk` workgroups per output tile (blockIdx.z): each writes its fp32 partial
    // tile to `part`, the last to arrive (counted in `count`, which it leaves at zero) adds them
    // up in slice order and finishes the tile
    int sk;
    float* part;
    int* count;
};

template <int I, int N, class F>
__device__ __forceinline__ void wide_static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>());
        wide_static_for<I + 1, N>(f);
    }
}

// Waves per SIMD the register allocation is held to: the smallest tile with wide gathers fits
// 72 registers without spilling, and seven workgroups on a CU instead of five take the 1 568
// tiles of a 56 x 56 layer at batch 32 in one round.
#ifndef CADNN_WIDE_WAVES
#define CADNN_WIDE_WAVES(MI, NI, HS, G) ((MI) * (NI) == 1 && (HS) == 1 && (G) > 1 ? 7 : 1)
#endif
// MI x NI accumulators of 32 x 32 per wave: a workgroup's tile is 64 MI channels x 64 NI pixels.
// HS: 32-deep steps of K per stage, i.e. per barrier (a stage's LDS tile is 32 HS deep); with
// one or two workgroups on a CU the chain LDS write - barrier - LDS read - MFMA of a stage is
// not hidden by anything, so it has to be paid as seldom as the LDS size allows.
// D (even): register sets, that is how many stages ahead of the MFMAs the global loads run.
// G: neighbouring pixels per gather load (a quarter of the load instructions with 4; measured:
// a few percent of a layer's time, most where rows are short).
template <int MI, int NI, int HS, int D, int G>
__global__ __launch_bounds__(256, CADNN_WIDE_WAVES(MI, NI, HS, G)) void dense_wide_kernel(const WideArgs a) {
    constexpr int TM = 64 * MI, TN = 64 * NI;
    // a gather item is G pixels x CH channels of a step, fetched with CH loads; thread t takes
    // items t + 256 j, so that every wave's loads carry 64 lanes of wanted data
    constexpr int GROUPS = TN / G, CH = GROUPS / 8 < 8 ? GROUPS / 8 : 8, NB = GROUPS / 8 / CH;
    static_assert(CH >= 2 && GROUPS * (WK / CH) == 256 * NB, "256 threads cover a step's activations");
    constexpr int PITCH = WK * HS + 8;      // halves between rows in LDS: 80, 144 or 272 bytes, all conflict-free
    // (the two stage buffers of both operands; the epilogue reuses them for the output tile)
    constexpr int CPITCH = TN + 8;          // words between rows of the fp32 output tile
    constexpr int MAIN_BYTES = 2 * (TM + TN) * PITCH * 2, TILE_BYTES = 64 * CPITCH * 4, EPI_BYTES = TILE_BYTES + TM * 4;
    __shared__ __attribute__((aligned(16))) char smem[MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES];
    // (table mode: per k its byte offset from the pixel's own position and its tap; two stages
    // past the end of K are fetched, from entries that stay zero)
    constexpr bool TABLE = NI == 1 && G == 1;
    __shared__ int2 ktab[TABLE ? kWideTableK + 2 * WK * HS * D : 1];
    _Float16 (*As)[TM * PITCH] = (_Float16 (*)[TM * PITCH])smem;
    _Float16 (*Bs)[TN * PITCH] = (_Float16 (*)[TN * PITCH])(smem + 2 * TM * PITCH * 2);

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wv >> 1, wn = wv & 1;
    const int n0 = (int)blockIdx.x * TN, m0 = (int)blockIdx.y * TM;

    // ---- gather side: pixels n0 + lane (+ 64) -- byte offset of their own input position (tap
    //      offsets are added per step) and the taps that fall inside the image
    uint32_t gbase[NB], gbase2[NB];
    uint64_t gmask[NB];
    int grow[NB], gch[NB];        // first LDS row (pixel of the tile) and first channel of the item
#pragma unroll
    for (int h = 0; h < NB; ++h) {
        const int item = (int)threadIdx.x + 256 * h;
        grow[h] = (item % GROUPS) * G;
        gch[h] = item / GROUPS * CH;
        const int Q = n0 + grow[h];
        gbase[h] = 0;
        gbase2[h] = kWideOutOfRange;
        gmask[h] = 0;
        if (Q < a.total) {
            const int img = Q / a.hwout, q = Q - img * a.hwout;
            const int oh = q / a.yd.w, ow = q - oh * a.yd.w;
            // (de-interleaved input: a stride-2 layer walks the phase planes with unit stride,
            // a pixel-wise stride-1 layer takes each pixel's own place)
            const int at = !a.xd.s2d ? a.xd.origin + oh * a.stride * a.xd.pitch + ow * a.stride
                           : a.stride == 2 ? oh * a.xd.pitch + ow : tensor_off(a.xd, oh, ow);
            // (the item's first channel rides in the per-lane part: a wave may hold several)
            gbase[h] = (uint32_t)(img * (int)a.xd.image + (a.table ? 0 : gch[h]) * a.xd.plane + at) * 2u;
            if (a.x2)
                gbase2[h] = (uint32_t)(img * (int)a.x2d.image + gch[h] * a.x2d.plane + a.x2d.origin + oh * a.stride2 * a.x2d.pitch +
                                       ow * a.stride2) * 2u;
            if constexpr (G > 1) gmask[h] = ~(uint64_t)0;       // (every tap of every pixel lies in memory)
            else {
                // (the taps inside the image are a rectangle: rows times columns)
                uint32_t rows_in = 0, cols_in = 0;
                for (int r = 0; r < a.kh; ++r) {
                    const int ih = oh * a.stride + r - a.pad;
                    if (ih >= 0 && ih < a.xd.h) rows_in |= 1u << r;
                }
                for (int c = 0; c < a.kw; ++c) {
                    const int iw = ow * a.stride + c - a.pad;
                    if (iw >= 0 && iw < a.xd.w) cols_in |= 1u << c;
                }
                for (int r = 0; r < a.kh; ++r)
                    if ((rows_in >> r) & 1) gmask[h] |= (uint64_t)cols_in << (r * a.kw);
            }
        }
    }
    // (readfirstlane: the compiler must keep the buffer descriptors in scalar registers)
    const uint32_t xspan = __builtin_amdgcn_readfirstlane((uint32_t)(a.xd.image * 2) * (uint32_t)a.n);
    const uint32_t x2span = __builtin_amdgcn_readfirstlane(a.x2 ? (uint32_t)(a.x2d.image * 2) * (uint32_t)a.n : 0u);
    const uint32_t plane2_bytes = (uint32_t)a.x2d.plane * 2u;
    const int taps = a.kh * a.kw;
    const uint32_t plane_bytes = (uint32_t)a.xd.plane * 2u;

    // ---- weight side: thread t fetches 16-byte pieces t (+ 256) of a step's [TM][32] tile
    const int apart = (int)threadIdx.x & 3;
    const uint32_t wspan = __builtin_amdgcn_readfirstlane((uint32_t)(((a.cout + 127) / 128 * 128) * a.K * 2));
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, wspan, 0x00020000);
    uint32_t wrow[MI];
#pragma unroll
    for (int i = 0; i < MI; ++i) wrow[i] = (uint32_t)((m0 + (((int)threadIdx.x + 256 * i) >> 2)) * a.K + apart * 8) * 2u;

    // ---- the tile's bias values are requested now, one per thread: the epilogue finds them
    //      in a register instead of adding a memory round trip to the tail
    float my_bias = 0.0f;
    {
        // (row t of the tile in the order the epilogue walks it: pass t / 64, local row t % 64)
        const int t = (int)threadIdx.x, pass = t >> 6, r = t & 63;
        const int co = m0 + (r >> 5) * 32 * MI + pass * 32 + (r & 31);
        if (t < TM && co < a.cout) my_bias = (a.bias ? a.bias[co] : 0.0f) + (a.bias2 ? a.bias2[co] : 0.0f);
    }

    // D register sets: the loads of stage s + D are issued while stage s is multiplied and stage
    // s + 1, fetched D - 1 stages earlier, is written to LDS.
    u32x4w areg[D][HS][MI];
    // (2-byte elements are widened only when the set is used: see stash)
    typedef std::conditional_t<G == 1, unsigned short, std::conditional_t<G == 2, uint32_t, u32x2w>> gather_t;
    gather_t breg[D][HS][NB][CH];
    // Steps are fetched in order and a wave is one serial instruction stream, so what a step
    // costs in scalar bookkeeping it costs in time: the state of the walk over K is carried
    // along -- per step about ten scalar additions and a counter -- and everything that depends on
    // the tap (its offset, which pixels it reaches, the switch to a fused shortcut's input) is
    // redone only when the tap changes, behind a scalar branch that issues no load.  Past the
    // last step zeros are fetched (out-of-range offsets on both sides) rather than nothing, so
    // that the number of loads in flight is known at compile time.
    const int steps_all = a.table ? a.K / WK : taps * a.csteps + a.csteps2;
    if constexpr (TABLE) {
        if (a.table) {
            for (int k = (int)threadIdx.x; k < kWideTableK + 2 * WK * HS * D; k += 256) {
                const int ci = k / taps, t = k - ci * taps, r = t / a.kw, c = t - r * a.kw;
                ktab[k] = k < a.cin * taps ? make_int2((ci * a.xd.plane + (r - a.pad) * a.xd.pitch + (c - a.pad)) * 2, t) : make_int2(0, 0);
            }
            __syncthreads();
        }
    }
    // this workgroup's slice of K: steps [s_first, s_first + steps)
    // (integer divisions run on the vector ALU: their results are made scalar again, or every
    // address derived from them would be a per-lane value to the compiler)
    const int per_slice = __builtin_amdgcn_readfirstlane((steps_all + a.sk - 1) / a.sk);
    const int s_first = (int)blockIdx.z * per_slice;
    const int steps = min(per_slice, steps_all - s_first);
    const int stages = (steps + HS - 1) / HS;
    int f_tap = 0, f_r = 0, f_c = 0, f_left = 0, f_todo = steps, f_step = s_first;          // (scalar)
    bool f_second = false;
    uint32_t f_soffA = 0, f_inc = 0, f_pb = 0, f_soffB = 0;
    uint32_t f_vA[MI], f_vB[NB];
    // (past the slice only the per-lane parts of the addresses change, to out of range, which is
    // what the range check looks at; the scalar parts run on)
    auto end_walk = [&]() __attribute__((always_inline)) {
        f_left = 0x7fffffff;
#pragma unroll
        for (int h = 0; h < NB; ++h) f_vB[h] = kWideOutOfRange;
#pragma unroll
        for (int i = 0; i < MI; ++i) f_vA[i] = kWideOutOfRange;
    };
    // state of tap f_tap (f_r, f_c), entered at its channel block cb
    auto load_tap = [&](int cb) __attribute__((always_inline)) {
        f_second = f_tap >= taps;
        const int Rt = f_r - a.pad + a.xd.ph, Ct = f_c - a.pad + a.xd.pw;
        const int tap_el = !a.xd.s2d ? (f_r - a.pad) * a.xd.pitch + (f_c - a.pad)
                           : a.stride == 2 ? ((Rt & 1) * 2 + (Ct & 1)) * a.xd.sub + (Rt >> 1) * a.xd.pitch + (Ct >> 1) : 0;
        f_pb = f_second ? plane2_bytes : plane_bytes;
        f_inc = WK * f_pb;
        f_left = (f_second ? a.csteps2 : a.csteps) - cb;
        f_soffB = (uint32_t)(cb * WK) * f_pb;
#pragma unroll
        for (int h = 0; h < NB; ++h)
            f_vB[h] = f_second ? gbase2[h] : ((gmask[h] >> f_tap) & 1) ? gbase[h] + (uint32_t)(tap_el * 2) : kWideOutOfRange;
    };
    auto next_tap = [&]() __attribute__((always_inline)) {
        ++f_tap;
        if (++f_c == a.kw) { f_c = 0; ++f_r; }
        load_tap(0);
    };
#pragma unroll
    for (int i = 0; i < MI; ++i) f_vA[i] = wrow[i];
    if (a.table) {
        // (no tap walk: a pixel's own position, every k's offset from the table)
        f_left = 0x7fffffff;
#pragma unroll
        for (int h = 0; h < NB; ++h) f_vB[h] = (gmask[h] != 0) ? gbase[h] : kWideOutOfRange;
        f_soffA = (uint32_t)s_first * (WK * 2);
    } else {
        const int in_taps = taps * a.csteps;
        f_tap = __builtin_amdgcn_readfirstlane(s_first < in_taps ? s_first / a.csteps : taps);
        f_r = __builtin_amdgcn_readfirstlane(f_tap / a.kw);
        f_c = f_tap - f_r * a.kw;
        load_tap(s_first < in_taps ? s_first - f_tap * a.csteps : s_first - in_taps);
        f_soffA = (uint32_t)s_first * (WK * 2);
    }
    auto fetch = [&](auto SET) __attribute__((always_inline)) {
        constexpr int S = decltype(SET)::value;
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) {
            // (made scalar by hand: the compiler may fold this choice into per-lane control flow)
            const uint64_t xp = f_second ? (uint64_t)a.x2 : (uint64_t)a.x;
            // (the builtin returns a signed int: through uint32_t, or the low word's top bit smears over the high word)
            const uint64_t xps = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)xp) |
                                 ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(xp >> 32)) << 32);
            const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
                (void*)xps, 0, __builtin_amdgcn_readfirstlane(f_second ? x2span : xspan), 0x00020000);
#pragma unroll
            for (int i = 0; i < MI; ++i) areg[S][hs][i] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, f_vA[i], f_soffA, 0);
            if constexpr (TABLE) {
                if (a.table) {
                    // step f_step of K: this wave's eight k, each with its own offset and tap
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const int2 e = ktab[f_step * WK + wv * 8 + k];
                        const uint32_t vo = (f_vB[0] != kWideOutOfRange && ((gmask[0] >> e.y) & 1)) ? f_vB[0] + (uint32_t)e.x : kWideOutOfRange;
                        breg[S][hs][0][k] = __builtin_amdgcn_raw_buffer_load_b16(xrsrc, vo, 0u, 0);
                    }
                    f_soffA += WK * 2;
                    ++f_step;
                    if (--f_todo == 0) end_walk();
                    continue;
                }
            }
            uint32_t soff = f_soffB;         // (channel by channel: one running scalar instead of eight kept ones)
#pragma unroll
            for (int k = 0; k < CH; ++k) {
#pragma unroll
                for (int h = 0; h < NB; ++h) {
                    if constexpr (G == 1) breg[S][hs][h][k] = __builtin_amdgcn_raw_buffer_load_b16(xrsrc, f_vB[h], soff, 0);
                    else if constexpr (G == 2) breg[S][hs][h][k] = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, f_vB[h], soff, 0);
                    else breg[S][hs][h][k] = __builtin_amdgcn_raw_buffer_load_b64(xrsrc, f_vB[h], soff, 0);
                }
                soff += f_pb;
            }
            f_soffA += WK * 2;
            f_soffB += f_inc;
            if (--f_todo == 0) end_walk();
            else if (--f_left == 0) next_tap();
        }
    };
    auto stash = [&](int buf, auto SET) __attribute__((always_inline)) {
        constexpr int S = decltype(SET)::value;
        // The set is opaque to the compiler up to here, and its 2-byte elements are kept as
        // such: otherwise the first operation on every loaded register (the widening) -- and
        // with it the wait for the load -- is placed at the end of the loop iteration that
        // issued the load, which drains the loads in flight once per D stages.
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) {
#pragma unroll
            for (int i = 0; i < MI; ++i) asm volatile("" : "+v"(areg[S][hs][i]));
#pragma unroll
            for (int h = 0; h < NB; ++h)
#pragma unroll
                for (int k = 0; k < CH; ++k) asm volatile("" : "+v"(breg[S][hs][h][k]));
        }
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) {
#pragma unroll
            for (int i = 0; i < MI; ++i)
                *(u32x4w*)(&As[buf][(((int)threadIdx.x + 256 * i) >> 2) * PITCH + hs * WK + apart * 8]) = areg[S][hs][i];
#pragma unroll
            for (int h = 0; h < NB; ++h) {
                _Float16* dst = &Bs[buf][grow[h] * PITCH + hs * WK + gch[h]];
                if constexpr (G == 1) {
                    u32x4w pk;
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        pk[k] = (uint32_t)breg[S][hs][h][2 * k] | ((uint32_t)breg[S][hs][h][2 * k + 1] << 16);
                    *(u32x4w*)dst = pk;
                } else {
                    // a loaded word holds one channel of two neighbouring pixels: the low halves of
                    // two channels make a word of the first pixel, the high halves one of the second
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        uint32_t word[CH / 2];
#pragma unroll
                        for (int m = 0; m < CH / 2; ++m) {
                            uint32_t lo, hi;
                            if constexpr (G == 2) { lo = breg[S][hs][h][2 * m]; hi = breg[S][hs][h][2 * m + 1]; }
                            else { lo = breg[S][hs][h][2 * m][j >> 1]; hi = breg[S][hs][h][2 * m + 1][j >> 1]; }
                            word[m] = __builtin_amdgcn_perm(hi, lo, (j & 1) ? 0x07060302u : 0x05040100u);
                        }
                        if constexpr (CH == 2) *(uint32_t*)(dst + j * PITCH) = word[0];
                        else if constexpr (CH == 4) *(u32x2w*)(dst + j * PITCH) = u32x2w{word[0], word[1]};
                        else *(u32x4w*)(dst + j * PITCH) = u32x4w{word[0], word[1], word[2], word[3]};
                    }
                }
            }
        }
    };

    f32x16w acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.0f;

    const int fm = lane & 31, fk = lane >> 5;
    // stage s: LDS buffer s % 2 holds it; register set (s + j) % D holds stage s + j, 0 < j < D
    auto body = [&](auto PAR) __attribute__((always_inline)) {
        constexpr int P = decltype(PAR)::value;
        // A wave is one in-order instruction stream and there are few waves per SIMD, so the
        // order is chosen to keep a wait from standing right behind the request it waits for:
        // the stage's fragments are requested from LDS first; the global loads of stage s + D
        // are issued and the oldest set is waited for, packed and written to the LDS buffer
        // nobody reads during this stage while the fragments arrive; the products follow
        // without a wait in between and run on while the wave goes to the barrier.  (The
        // scheduler is held to this order.)
        h8 af[2 * HS][MI], bf[2 * HS][NI];
#pragma unroll
        for (int ks = 0; ks < 2 * HS; ++ks) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                af[ks][mi] = *(const h8*)(&As[P & 1][(wm * 32 * MI + mi * 32 + fm) * PITCH + ks * 16 + fk * 8]);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                bf[ks][ni] = *(const h8*)(&Bs[P & 1][(wn * 32 * NI + ni * 32 + fm) * PITCH + ks * 16 + fk * 8]);
        }
        __builtin_amdgcn_sched_barrier(0);
        fetch(std::integral_constant<int, P>());
        __builtin_amdgcn_sched_barrier(0);
        stash((P + 1) & 1, std::integral_constant<int, (P + 1) % D>());
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 2 * HS; ++ks)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[ks][mi], bf[ks][ni], acc[mi][ni], 0, 0, 0);
        __syncthreads();
    };
    wide_static_for<0, D>([&](auto J) { fetch(J); });
    stash(0, std::integral_constant<int, 0>());
    __syncthreads();
    int s = 0;
    for (; s + D <= stages; s += D) wide_static_for<0, D>([&](auto J) { body(J); });
    wide_static_for<0, D - 1>([&](auto J) {
        if (s + decltype(J)::value < stages) body(J);
    });

    // ---- K split over workgroups: the slices of a tile meet in memory
    if (a.sk > 1) {
        const size_t tile_id = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
        float* mine = a.part + (tile_id * a.sk + blockIdx.z) * (size_t)(TM * TN);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    __hip_atomic_store(mine + ((mi * NI + ni) * 16 + i) * 256 + threadIdx.x, acc[mi][ni][i], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        // Device-scope stores and loads go to the level all dies share, so the slices' tiles need
        // no cache write-back or invalidation (a release fence here writes back the whole L2 of
        // the die: 50 us per launch measured); what orders them against the count is that every
        // thread's stores are acknowledged before the workgroup's arrival is counted.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        int* flag = (int*)smem;           // (the stage buffers are no longer read: every wave is past the barrier)
        if (threadIdx.x == 0) {
            const int arrived = __hip_atomic_fetch_add(a.count + tile_id, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = arrived == a.sk - 1;
            if (arrived == a.sk - 1) a.count[tile_id] = 0;      // every other slice has counted itself: ready for the next launch
        }
        __syncthreads();
        const bool last = *flag != 0;
        __syncthreads();                  // (smem is reused below)
        if (!last) return;
        // slice order, whoever arrived last: the sum does not depend on the order of arrival
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.0f;
        for (int z = 0; z < a.sk; ++z) {
            const float* src = a.part + (tile_id * a.sk + z) * (size_t)(TM * TN);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        acc[mi][ni][i] += __hip_atomic_load(src + ((mi * NI + ni) * 16 + i) * 256 + threadIdx.x, __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    // ---- fused epilogue.  Lane l holds, per accumulator, pixel column l % 32 and the 16 rows
    //      8 * (i / 4) + 4 * (l / 32) + i % 4.
    const uint32_t yspan = __builtin_amdgcn_readfirstlane((uint32_t)(a.yd.image * 2) * (uint32_t)a.n);
    const uint32_t rspan = __builtin_amdgcn_readfirstlane(a.residual ? (uint32_t)(a.rd.image * 2) * (uint32_t)a.n : 0u);
    const __amdgpu_buffer_rsrc_t yrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a.y, 0, yspan, 0x00020000);
    const __amdgpu_buffer_rsrc_t rrsrc = __builtin_amdgcn_make_buffer_rsrc(
        a.residual ? (void*)a.residual : (void*)a.y, 0, rspan, 0x00020000);
    auto place = [&](int Q, uint32_t& yoff, uint32_t& roff) {
        yoff = kWideOutOfRange;
        roff = kWideOutOfRange;
        if (Q < a.total) {
            const int img = Q / a.hwout, q = Q - img * a.hwout;
            const int oh = q / a.yd.w, ow = q - oh * a.yd.w;
            yoff = (uint32_t)(img * (int)a.yd.image + tensor_off(a.yd, oh, ow)) * 2u;
            roff = (uint32_t)(img * (int)a.rd.image + tensor_off(a.rd, oh, ow)) * 2u;
        }
    };
    if (a.group || a.rows) {
        // Through LDS: the accumulators of 64 channels at a time are laid out [channel][pixel]
        // as fp32 and a thread takes `group` neighbouring pixels of one channel -- bias, residual,
        // ReLU, one rounding, ONE store of 4 to 16 bytes.  (A wave's own accumulator layout puts
        // 32 pixels of a channel side by side: 64-byte pieces written 2 bytes per lane, which
        // the memory pipeline takes at a fraction of the rate: 6 us per workgroup measured.)
        float* ct = (float*)smem;
        float* bl = (float*)(smem + TILE_BYTES);            // [pass][local row]
        auto run = [&](auto GG) __attribute__((always_inline)) {
            constexpr int SG = decltype(GG)::value, per_row = TN / SG, rows_per_sweep = 256 / per_row, sweeps = 64 / rows_per_sweep;
            const int cg = (int)threadIdx.x % per_row, r0 = (int)threadIdx.x / per_row;
            const int Q = n0 + cg * SG;
            uint32_t yoff = kWideOutOfRange, roff = kWideOutOfRange;
            if (Q < a.total) {          // (the images' pixel counts are multiples of the group: all of it or none)
                const int img = Q / a.hwout, q = Q - img * a.hwout;
                yoff = (uint32_t)(img * (int)a.yd.image + q) * 2u;
                roff = (uint32_t)(img * (int)a.rd.image + q) * 2u;
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                __syncthreads();        // the tile's last readers (the K loop, the previous pass) are done
                if (mi == 0 && threadIdx.x < TM) bl[threadIdx.x] = my_bias;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        ct[(wm * 32 + (i >> 2) * 8 + fk * 4 + (i & 3)) * CPITCH + wn * 32 * NI + ni * 32 + fm] = acc[mi][ni][i];
                __syncthreads();
#pragma unroll
                for (int k = 0; k < sweeps; ++k) {
                    const int r = r0 + k * rows_per_sweep;
                    const int co = m0 + (r >> 5) * 32 * MI + mi * 32 + (r & 31);
                    const bool live = co < a.cout && yoff != kWideOutOfRange;
                    const int cc = co < a.cout ? co : 0;
                    const float b = bl[mi * 64 + r];
                    const float* src = ct + r * CPITCH + cg * SG;
                    const uint32_t yo = live ? yoff + (uint32_t)cc * (uint32_t)a.yd.plane * 2u : kWideOutOfRange;
                    const uint32_t ro = live ? roff + (uint32_t)cc * (uint32_t)a.rd.plane * 2u : kWideOutOfRange;
                    auto finish = [&](float v, uint32_t rbits) __attribute__((always_inline)) {
                        v += b;
                        if (a.residual) v += (float)__builtin_bit_cast(_Float16, (unsigned short)rbits);
                        if (a.relu) v = v > 0.0f ? v : 0.0f;
                        return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)v);
                    };
                    if constexpr (SG == 8) {
                        const f32x4w lo = *(const f32x4w*)src, hi = *(const f32x4w*)(src + 4);
                        u32x4w rr = {0u, 0u, 0u, 0u};
                        if (a.residual) rr = __builtin_amdgcn_raw_buffer_load_b128(rrsrc, ro, 0u, 0);
                        u32x4w o;
                        o[0] = finish(lo[0], rr[0]) | (finish(lo[1], rr[0] >> 16) << 16);
                        o[1] = finish(lo[2], rr[1]) | (finish(lo[3], rr[1] >> 16) << 16);
                        o[2] = finish(hi[0], rr[2]) | (finish(hi[1], rr[2] >> 16) << 16);
                        o[3] = finish(hi[2], rr[3]) | (finish(hi[3], rr[3] >> 16) << 16);
                        __builtin_amdgcn_raw_buffer_store_b128(o, yrsrc, yo, 0u, 0);
                    } else if constexpr (SG == 4) {
                        const f32x4w lo = *(const f32x4w*)src;
                        u32x2w rr = {0u, 0u};
                        if (a.residual) rr = __builtin_amdgcn_raw_buffer_load_b64(rrsrc, ro, 0u, 0);
                        u32x2w o;
                        o[0] = finish(lo[0], rr[0]) | (finish(lo[1], rr[0] >> 16) << 16);
                        o[1] = finish(lo[2], rr[1]) | (finish(lo[3], rr[1] >> 16) << 16);
                        __builtin_amdgcn_raw_buffer_store_b64(o, yrsrc, yo, 0u, 0);
                    } else {
                        const f32x2w lo = *(const f32x2w*)src;
                        uint32_t rr = 0u;
                        if (a.residual) rr = __builtin_amdgcn_raw_buffer_load_b32(rrsrc, ro, 0u, 0);
                        __builtin_amdgcn_raw_buffer_store_b32(finish(lo[0], rr) | (finish(lo[1], rr >> 16) << 16), yrsrc, yo, 0u, 0);
                    }
                }
            }
        };
        // Any other layout whose rows split into groups of SG pixels (a halo, a de-interleaved
        // tensor): the group lies in one row, so in memory it is one run of SG elements, or -- de-
        // interleaved by column parity -- two runs of SG / 2 (pixels 0, 2, .. and 1, 3, ..).  A run
        // is stored 4 or 8 bytes at a time at whatever 2-byte alignment it has (checked on the box:
        // the buffer path takes such loads and stores).
        auto run_rows = [&](auto GG) __attribute__((always_inline)) {
            constexpr int SG = decltype(GG)::value, per_row = TN / SG, rows_per_sweep = 256 / per_row, sweeps = 64 / rows_per_sweep;
            const int cg = (int)threadIdx.x % per_row, r0 = (int)threadIdx.x / per_row;
            const int Q = n0 + cg * SG;
            uint32_t yo[2] = {kWideOutOfRange, kWideOutOfRange}, ro[2] = {kWideOutOfRange, kWideOutOfRange};
            if (Q < a.total) {
                const int img = Q / a.hwout, q = Q - img * a.hwout;
                const int oh = q / a.yd.w, ow = q - oh * a.yd.w;
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    yo[p] = (uint32_t)(img * (int)a.yd.image + tensor_off(a.yd, oh, ow + p)) * 2u;
                    ro[p] = (uint32_t)(img * (int)a.rd.image + tensor_off(a.rd, oh, ow + p)) * 2u;
                }
            }
            // N halves to / from one run, in pieces of at most 8 bytes
            auto load_run = [&](uint32_t off, auto NN, uint32_t (&h)[SG], int first, int step) __attribute__((always_inline)) {
                constexpr int N = decltype(NN)::value;
                uint32_t w[N / 2 > 0 ? N / 2 : 1];
                if constexpr (N == 1) {
                    h[first] = __builtin_amdgcn_raw_buffer_load_b16(rrsrc, off, 0u, 0);
                } else {
#pragma unroll
                    for (int i = 0; i < N / 2; i += 2) {
                        if constexpr (N >= 4) {
                            const u32x2w v = __builtin_amdgcn_raw_buffer_load_b64(rrsrc, off == kWideOutOfRange ? off : off + 4u * i, 0u, 0);
                            w[i] = v[0]; w[i + 1] = v[1];
                        } else {
                            w[i] = __builtin_amdgcn_raw_buffer_load_b32(rrsrc, off, 0u, 0);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < N; ++i) h[first + i * step] = (w[i / 2] >> (16 * (i & 1))) & 0xffffu;
                }
            };
            auto store_run = [&](uint32_t off, auto NN, const uint32_t (&h)[SG], int first, int step) __attribute__((always_inline)) {
                constexpr int N = decltype(NN)::value;
                if constexpr (N == 1) {
                    __builtin_amdgcn_raw_buffer_store_b16((unsigned short)h[first], yrsrc, off, 0u, 0);
                } else {
                    uint32_t w[N / 2];
#pragma unroll
                    for (int i = 0; i < N / 2; ++i) w[i] = h[first + 2 * i * step] | (h[first + (2 * i + 1) * step] << 16);
#pragma unroll
                    for (int i = 0; i < N / 2; i += 2) {
                        if constexpr (N >= 4)
                            __builtin_amdgcn_raw_buffer_store_b64(u32x2w{w[i], w[i + 1]}, yrsrc, off == kWideOutOfRange ? off : off + 4u * i, 0u, 0);
                        else
                            __builtin_amdgcn_raw_buffer_store_b32(w[i], yrsrc, off, 0u, 0);
                    }
                }
            };
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                __syncthreads();
                if (mi == 0 && threadIdx.x < TM) bl[threadIdx.x] = my_bias;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        ct[(wm * 32 + (i >> 2) * 8 + fk * 4 + (i & 3)) * CPITCH + wn * 32 * NI + ni * 32 + fm] = acc[mi][ni][i];
                __syncthreads();
#pragma unroll
                for (int k = 0; k < sweeps; ++k) {
                    const int r = r0 + k * rows_per_sweep;
                    const int co = m0 + (r >> 5) * 32 * MI + mi * 32 + (r & 31);
                    const bool live = co < a.cout && yo[0] != kWideOutOfRange;
                    const uint32_t cc = (uint32_t)(co < a.cout ? co : 0);
                    const float b = bl[mi * 64 + r];
                    const float* src = ct + r * CPITCH + cg * SG;
                    uint32_t res[SG], out[SG];
#pragma unroll
                    for (int j = 0; j < SG; ++j) res[j] = 0u;
                    if (a.residual) {
                        const uint32_t po = cc * (uint32_t)a.rd.plane * 2u;
                        if (a.rd.s2d) {
                            load_run(live ? ro[0] + po : kWideOutOfRange, std::integral_constant<int, SG / 2>(), res, 0, 2);
                            load_run(live ? ro[1] + po : kWideOutOfRange, std::integral_constant<int, SG / 2>(), res, 1, 2);
                        } else {
                            load_run(live ? ro[0] + po : kWideOutOfRange, std::integral_constant<int, SG>(), res, 0, 1);
                        }
                    }
#pragma unroll
                    for (int j = 0; j < SG; ++j) {
                        float v = src[j] + b;
                        if (a.residual) v += (float)__builtin_bit_cast(_Float16, (unsigned short)res[j]);
                        if (a.relu) v = v > 0.0f ? v : 0.0f;
                        out[j] = (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)v);
                    }
                    const uint32_t po = cc * (uint32_t)a.yd.plane * 2u;
                    if (a.yd.s2d) {
                        store_run(live ? yo[0] + po : kWideOutOfRange, std::integral_constant<int, SG / 2>(), out, 0, 2);
                        store_run(live ? yo[1] + po : kWideOutOfRange, std::integral_constant<int, SG / 2>(), out, 1, 2);
                    } else {
                        store_run(live ? yo[0] + po : kWideOutOfRange, std::integral_constant<int, SG>(), out, 0, 1);
                    }
                }
            }
        };
        if (a.group == 8) run(std::integral_constant<int, 8>());
        else if (a.group == 4) run(std::integral_constant<int, 4>());
        else if (a.group == 2) run(std::integral_constant<int, 2>());
        else if (a.rows == 8) run_rows(std::integral_constant<int, 8>());
        else if (a.rows == 4) run_rows(std::integral_constant<int, 4>());
        else run_rows(std::integral_constant<int, 2>());
    } else {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            uint32_t yoff, roff;
            place(n0 + wn * 32 * NI + ni * 32 + fm, yoff, roff);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int co = m0 + wm * 32 * MI + mi * 32 + (i >> 2) * 8 + fk * 4 + (i & 3);
                    const bool live = co < a.cout;
                    const int cc = live ? co : 0;
                    float v = acc[mi][ni][i] + ((a.bias ? a.bias[cc] : 0.0f) + (a.bias2 ? a.bias2[cc] : 0.0f));
                    if (a.residual)
                        v += (float)__builtin_bit_cast(
                            _Float16, __builtin_amdgcn_raw_buffer_load_b16(rrsrc, live ? roff + (uint32_t)cc * (uint32_t)a.rd.plane * 2u : kWideOutOfRange, 0u, 0));
                    if (a.relu) v = v > 0.0f ? v : 0.0f;
                    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, (_Float16)v), yrsrc,
                                                          live ? yoff + (uint32_t)cc * (uint32_t)a.yd.plane * 2u : kWideOutOfRange, 0u, 0);
                }
        }
    }
}

// [cout][cin][kh][kw] -> [cout rounded up to 128][tap * cin + ci], fp16, zero rows beyond cout.
__global__ __launch_bounds__(256) void dense_wide_reorder_kernel(const _Float16* __restrict__ w, _Float16* __restrict__ out,
                                                                 int cout, int cin, int taps, size_t total) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t K = (size_t)cin * taps;
        const int m = (int)(i / K);
        const int k = (int)(i - (size_t)m * K);
        const int tap = k / cin, ci = k - tap * cin;
        out[i] = m < cout ? w[((size_t)m * cin + ci) * taps + tap] : (_Float16)0.0f;
    }
}

// HS: 32-deep steps per stage.  Two halve the barriers of a long K; one keeps the LDS tile small
// (more workgroups per CU) and wastes nothing on layers whose K is a step or two: both are
// offered, except for the largest tile, whose registers only hold one.
#ifndef CADNN_WIDE_DEPTH
#define CADNN_WIDE_DEPTH 2
#endif
template <int MI, int NI, int HS>
hipError_t launch_wide_tile(const WideArgs& a, hipStream_t s) {
    dim3 grid((unsigned)((a.total + 64 * NI - 1) / (64 * NI)), (unsigned)((a.cout + 64 * MI - 1) / (64 * MI)), (unsigned)a.sk);
    if (a.gather == 4) CADNN_LAUNCH((dense_wide_kernel<MI, NI, HS, CADNN_WIDE_DEPTH, 4>), grid, dim3(256), 0, s, a);
    else if (a.gather == 2) CADNN_LAUNCH((dense_wide_kernel<MI, NI, HS, CADNN_WIDE_DEPTH, 2>), grid, dim3(256), 0, s, a);
    else CADNN_LAUNCH((dense_wide_kernel<MI, NI, HS, 2, 1>), grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_wide_args(const WideArgs& a, int tm, int tn, int hs, hipStream_t s) {
    // (K walked with a table: the 64-pixel tiles only, a K the table holds)
    if (a.table && (tn != 64 || a.K > kWideTableK || a.x2 || a.xd.s2d || a.sk > 1)) return hipErrorInvalidValue;
    if (tm == 128 && tn == 128) return launch_wide_tile<2, 2, 1>(a, s);
    if (tm == 128) return hs == 2 ? launch_wide_tile<2, 1, 2>(a, s) : launch_wide_tile<2, 1, 1>(a, s);
    if (tn == 128) return hs == 2 ? launch_wide_tile<1, 2, 2>(a, s) : launch_wide_tile<1, 2, 1>(a, s);
    return hs == 2 ? launch_wide_tile<1, 1, 2>(a, s) : launch_wide_tile<1, 1, 1>(a, s);
}

WideArgs wide_args(const void* w, const void* x, const TensorDesc& xd, void* y, const TensorDesc& yd, const void* residual,
                   const TensorDesc& rd, int n, int cout, int kh, int kw, int stride, int pad, const void* bias, int relu) {
    WideArgs a{};
    a.w = (const _Float16*)w; a.x = (const _Float16*)x; a.y = (_Float16*)y; a.bias = (const float*)bias;
    a.residual = (const _Float16*)residual;
    a.xd = xd; a.yd = yd; a.rd = rd;
    a.n = n; a.cout = cout; a.cin = xd.c; a.kh = kh; a.kw = kw; a.stride = stride; a.pad = pad; a.relu = relu ? 1 : 0;
    a.hwout = yd.h * yd.w;
    a.total = n * a.hwout;
    a.table = xd.c % WK != 0;
    a.K = a.table ? (xd.c * kh * kw + WK - 1) / WK * WK : xd.c * kh * kw;
    a.csteps = xd.c / WK;
    // the widest store the layouts allow: an image's pixels contiguous (no halo, not
    // de-interleaved), groups that neither straddle images nor leave their alignment
    auto group_of = [&](const TensorDesc& d, const void* p) {
        if (d.s2d || d.ph || d.pw || d.pitch != d.w) return 0;
        for (int g = 8; g >= 2; g >>= 1)
            if (a.hwout % g == 0 && d.plane % g == 0 && d.image % g == 0 && (uintptr_t)p % (2 * g) == 0) return g;
        return 0;
    };
    a.group = group_of(yd, y);
    if (residual) a.group = std::min(a.group, group_of(rd, residual));
    // any other layout (a halo, de-interleaved tensors): the widest groups the rows split into
    a.rows = 0;
    if (a.group == 0) a.rows = yd.w % 8 == 0 ? 8 : yd.w % 4 == 0 ? 4 : yd.w % 2 == 0 ? 2 : 0;
    a.gather = 1;
    const bool taps_in_memory = pad == 0 || (xd.ph >= pad && xd.pw >= pad);
    if (stride == 1 && !xd.s2d && taps_in_memory && !a.table)
        a.gather = yd.w % 4 == 0 ? 4 : yd.w % 2 == 0 ? 2 : 1;
    a.sk = 1;
    return a;
}

WideArgs wide_args(const ConvLaunch& l) {
    WideArgs a = wide_args(l.nz, l.x, l.xd, l.y, l.yd, l.residual, l.rd, l.n, l.cout, l.kh, l.kw, l.stride, l.pad, l.bias, l.relu);
    if (l.x2) {
        a.x2 = (const _Float16*)l.x2;
        a.bias2 = l.bias2;
        a.x2d = l.x2d;
        a.stride2 = l.stride2;
        a.csteps2 = l.x2d.c / WK;
        a.K += l.x2d.c;
        a.gather = 1;
    }
    a.sk = l.sk > 1 ? l.sk : 1;
    a.part = l.sk_part;
    a.count = l.sk_count;
    return a;
}

template <int TM, int TN, int HS = 2>
hipError_t launch_wide_variant(const ConvLaunch& l, hipStream_t s) {
    return launch_wide_args(wide_args(l), TM, TN, HS, s);
}

}  // namespace

bool dense_wide_serves(bool is_f16, int cin, int taps, int64_t in_bytes, int64_t out_bytes, int64_t pixels) {
    // (the whole batch sits behind 32-bit byte offsets)
    return is_f16 && (cin % WK == 0 || cin * taps <= kWideTableK) && taps <= 64 && in_bytes < 0x7ffffff0ll && out_bytes < 0x7ffffff0ll && pixels < 0x7fffff00ll;
}

// tw == 128 marks the tap-major weight matrix with rows padded to 128 (build_dense_plan); the
// tile is rpw * nw channels x 64 p pixels.
const std::vector<ConvVariant>& all_dense_wide_variants() {
    static const std::vector<ConvVariant> v = [] {
        std::vector<ConvVariant> out;
        auto add = [&](const char* name, int tm, int tn, hipError_t (*launch)(const ConvLaunch&, hipStream_t), int splitk = 1) {
            ConvVariant d{};
            d.splitk = splitk;
            d.name = name;
            d.family = FAM_DENSE;
            d.is_f16 = true;
            d.nw = 4; d.rpw = tm / 4; d.ks = 1; d.p = tn / 64; d.unroll = 1;
            d.tw = 128;
            d.launch = launch;
            out.push_back(d);
        };
        add("dense_mfma__Float16_128x128x32", 128, 128, &launch_wide_variant<128, 128>);
        add("dense_mfma__Float16_128x64x32", 128, 64, &launch_wide_variant<128, 64>);
        add("dense_mfma__Float16_64x128x32", 64, 128, &launch_wide_variant<64, 128>);
        add("dense_mfma__Float16_64x64x32w", 64, 64, &launch_wide_variant<64, 64>);
        add("dense_mfma__Float16_128x64x32_h1", 128, 64, &launch_wide_variant<128, 64, 1>);
        add("dense_mfma__Float16_64x128x32_h1", 64, 128, &launch_wide_variant<64, 128, 1>);
        add("dense_mfma__Float16_64x64x32w_h1", 64, 64, &launch_wide_variant<64, 64, 1>);
        // K split over 2 / 4 / 8 workgroups per tile, for layers whose tiles alone leave the chip idle
        add("dense_mfma__Float16_64x64x32w_k2", 64, 64, &launch_wide_variant<64, 64>, 2);
        add("dense_mfma__Float16_64x64x32w_k4", 64, 64, &launch_wide_variant<64, 64>, 4);
        add("dense_mfma__Float16_64x64x32w_k8", 64, 64, &launch_wide_variant<64, 64>, 8);
        add("dense_mfma__Float16_128x64x32_k2", 128, 64, &launch_wide_variant<128, 64>, 2);
        add("dense_mfma__Float16_128x64x32_k4", 128, 64, &launch_wide_variant<128, 64>, 4);
        return out;
    }();
    return v;
}

// The comparator on raw device weights [cout][cin][kh][kw] (fp16).  The tap-major copy of the
// weights is made on every call, in stream order (a caller that times the kernel alone packs
// the dense tensor into a weight handle and pins one of the variants above: then the copy is
// part of the plan).  The tile is the largest that still gives every CU two workgroups.
cadnn_status dense_wide_conv2d_raw(const void* w_dev, const void* x, const TensorDesc& xd, void* y, const TensorDesc& yd,
                                   const void* residual, const TensorDesc& rd, int n, int cout, int kh, int kw, int stride,
                                   int pad, const void* bias, int relu, hipStream_t s) {
    const size_t rows = (size_t)(cout + 127) / 128 * 128, K = (size_t)xd.c * kh * kw, total = rows * K;
    void* wr = nullptr;
    hipError_t e = hipMallocAsync(&wr, total * 2, s);
    if (e != hipSuccess) return fail(CADNN_ENOMEM, "hipMallocAsync(%zu) failed: %s", total * 2, hipGetErrorString(e));
    const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 4096);
    CADNN_LAUNCH(dense_wide_reorder_kernel, dim3(blocks), dim3(256), 0, s, (const _Float16*)w_dev, (_Float16*)wr, cout, xd.c,
                 kh * kw, total);
    const WideArgs a = wide_args(wr, x, xd, y, yd, residual, rd, n, cout, kh, kw, stride, pad, bias, relu);
    int tm = 128, tn = 128;
    auto blocks_of = [&](int m, int nn) { return (int64_t)((a.total + nn - 1) / nn) * ((cout + m - 1) / m); };
    if (blocks_of(tm, tn) < 512 && cout <= 64) tm = 64;
    if (blocks_of(tm, tn) < 512) tn = 64;
    if (blocks_of(tm, tn) < 512) tm = 64;
    e = launch_wide_args(a, tm, tn, a.csteps * kh * kw >= 8 ? 2 : 1, s);
    const hipError_t e2 = hipFreeAsync(wr, s);
    CADNN_HIP(e);
    CADNN_HIP(e2);
    return CADNN_OK;
}

}  // namespace cadnn
