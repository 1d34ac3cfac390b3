// Wide-read LDS sparse convolution for gfx950 (wave64): the kernel family in which one fetched
// activation vector feeds several FMAs and no FMA waits for a scalar copy of its weight.
//
// A workgroup stages the input region of one tile of output pixels in LDS -- all input
// channels if they fit half of a compute unit's LDS, else chunk after chunk, the next chunk
// landing in a second buffer while the current one is consumed -- and its NW waves share it:
// each wave owns RPW packed rows (output channels in the nnz-sorted order of the compact
// format, dealt out round robin so that the waves' shares are equal) and ALL pixels of the
// tile, P = 4 per lane.
//
// What differs from the other LDS families is how a nonzero reaches the arithmetic:
//   * the P activations a lane needs for a nonzero lie side by side in the staged tile (the
//     tile is laid out in slots of P words for exactly that, see WtileGeom) and arrive with
//     ONE 128-bit LDS read, feeding P FMAs;
//   * the nonzero's weight and tile offset are wave-uniform, but they are never copied to
//     scalar registers: a wave keeps 16 entries of its stream in two vector registers (lane l
//     holds entry l % 16) and entry k reaches the address add, and the weight a register of
//     its own, as a broadcast of lane k (`row_newbcast`).  Measured on the chip: a
//     lane-to-scalar copy costs about two vector-ALU slots, so the loop `2 copies + add + LDS
//     read + 4 FMA` runs at 37 clocks per nonzero per SIMD, `broadcasting add + LDS read +
//     broadcast copy + 4 FMA` at 27;
//   * the stream is compact: fp32 value + 16-bit offset (6 bytes per nonzero) in fp32
//     storage, fp16 value + 16-bit offset in one word (4 bytes) in fp16 storage -- the storage
//     accounting of the paper's Section 3 with its indices included.  An offset is the tap's
//     position in the staged chunk in units of 16 bytes.
//
// A filter element is fetched once per wave and reused by all its pixels, a staged activation
// is reused by every row of the workgroup and every tap (the paper's redundant-load
// elimination and layout transformation, Section 4); bias, residual and ReLU are fused into
// the epilogue (Section 4: conv + batch-norm + activation fused).
//
// 1x1 filters (a sparse matrix x dense matrix product, Section 4) take the "flat"
// instantiations: the pixels of the whole batch are numbered consecutively and a tile is
// 64 * P of them, so small images fill their tiles; any stride, any tensor layout.
// fp16 storage: an activation arrives in LDS as one binary16 value per word and is widened to
// fp32 in place by the wave that staged it; the weights are widened when a block of 16 entries
// is loaded; products and sums are fp32, as in every other family.
#include "internal.h"

namespace cadnn {

namespace {

constexpr uint32_t kWtOutOfRange = 0x7ffffff0u;

typedef __attribute__((address_space(3))) void* wt_lds_ptr_t;
typedef uint32_t wt_u4 __attribute__((ext_vector_type(4)));

template <typename T_, int FLAT_, int P_, int RPW_, int NW_, int LR_>
struct WtileCfg {
    using T = T_;
    static constexpr int FLAT = FLAT_, P = P_, RPW = RPW_, NW = NW_, LR = LR_, LC = 64 / LR_;
    static constexpr int THREADS = NW * 64;
    static_assert(P == 4, "a lane's pixels are one 128-bit LDS read");
    static_assert(64 % LR_ == 0, "lane grid");
};

// Lane K of the row's wv, in every lane of the row.  Every lane of the wave is active wherever
// this is used, so the lane read is always a live one.  (The FMA itself could read the lane
// -- v_fmac_f32_dpp -- but a lane-broadcast operand makes an instruction take about 1.5
// vector-ALU slots on this chip: one broadcast copy feeding P plain FMAs measures 27 clocks per
// nonzero per SIMD, P broadcasting FMAs 37.)
template <int K>
__device__ __forceinline__ float wt_bcast(float wv) {
    float r;
    asm("v_mov_b32_dpp %0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(wv), "n"(K));
    return r;
}
// (lane K of the row's ov) + base
template <int K>
__device__ __forceinline__ uint32_t wt_add(uint32_t ov, uint32_t base) {
    uint32_t r;
    asm("v_add_u32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(ov), "v"(base), "n"(K));
    return r;
}
// n / d for 0 <= n < 2^16 with m = ceil(2^32 / d), d < 2^16 (one multiply instead of a division
// sequence; the prologue below needs three of them per staged word).  d = 1 gives m = 2^32,
// which does not fit: callers pass m = 0 for it and get n back.
__device__ __forceinline__ int wt_div(int n, uint32_t m) { return m ? (int)__umulhi((uint32_t)n, m) : n; }
// n / d for any 0 <= n < 2^31, 0 < d < 2^24 through the float reciprocal, corrected by one step
__device__ __forceinline__ int wt_divf(int n, int d) {
    int q = (int)((float)n * __frcp_rn((float)d));
    int r = n - q * d;
    if (r < 0) { --q; r += d; }
    if (r < 0) { --q; r += d; }
    if (r >= d) { ++q; r -= d; }
    if (r >= d) ++q;
    return q;
}

// A register written by a vector-ALU instruction must not be read as a lane-broadcast source
// by the next two instructions; the compiler cannot see into the asm above, so the registers
// of a freshly loaded block pass through here first.
__device__ __forceinline__ void wt_settle(float& wv, uint32_t& ov) {
    asm volatile("s_nop 1" : "+v"(wv), "+v"(ov));
}

__device__ __forceinline__ wt_u4 wt_lds_read(uint32_t addr) {
    return *(const __attribute__((address_space(3))) wt_u4*)(uintptr_t)addr;
}

// Entries KB .. KB+N-1 of the block held in (wv, ov) against the P pixels of a lane: N LDS
// reads in flight, then per entry one broadcast copy of the weight and P FMAs.
template <typename T, int KB, int N, int U>
struct WtGroup {
    __device__ static __forceinline__ void fetch(uint32_t lane_base, uint32_t ov, wt_u4 (&x)[N]) {
        x[U] = wt_lds_read(wt_add<KB + U>(ov, lane_base));
        if constexpr (U + 1 < N) WtGroup<T, KB, N, U + 1>::fetch(lane_base, ov, x);
    }
    __device__ static __forceinline__ void mac(float wv, const wt_u4 (&x)[N], float (&acc)[4]) {
        const float w = wt_bcast<KB + U>(wv);
        acc[0] = fmaf(w, __uint_as_float(x[U][0]), acc[0]);
        acc[1] = fmaf(w, __uint_as_float(x[U][1]), acc[1]);
        acc[2] = fmaf(w, __uint_as_float(x[U][2]), acc[2]);
        acc[3] = fmaf(w, __uint_as_float(x[U][3]), acc[3]);
        if constexpr (U + 1 < N) WtGroup<T, KB, N, U + 1>::mac(wv, x, acc);
    }
};
template <typename T, int KB, int N>
__device__ __forceinline__ void wt_group(uint32_t lane_base, float wv, uint32_t ov, float (&acc)[4]) {
    wt_u4 x[N];
    WtGroup<T, KB, N, 0>::fetch(lane_base, ov, x);
    __builtin_amdgcn_sched_barrier(0);      // all N reads are in flight before the first FMA waits for one
    WtGroup<T, KB, N, 0>::mac(wv, x, acc);
}

// Lane (l % 16)'s entry of 16-entry block `blk` of the wave's stream: the weight as fp32 and
// the tile offset in bytes.  The lane's part of the address never changes and the block's part
// is a scalar, so a block costs no address arithmetic on the vector ALU.
template <typename T>
__device__ __forceinline__ void wt_load_block(__amdgpu_buffer_rsrc_t vals, __amdgpu_buffer_rsrc_t offs, int blk, uint32_t sub4,
                                              float& wv, uint32_t& ov) {
    if constexpr (sizeof(T) == 4) {
        wv = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(vals, sub4, (uint32_t)blk * 64u, 0));
        ov = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(offs, sub4 >> 1, (uint32_t)blk * 32u, 0) << 4;
    } else {
        const uint32_t e = __builtin_amdgcn_raw_buffer_load_b32(vals, sub4, (uint32_t)blk * 64u, 0);
        wv = (float)__builtin_bit_cast(_Float16, (unsigned short)(e & 0xffffu));
        ov = (e >> 16) << 4;
    }
}

}  // namespace

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void sconv_wtile_kernel(const ConvLaunch a) {
    using T = typename Cfg::T;
    constexpr int P = Cfg::P, RPW = Cfg::RPW, NW = Cfg::NW, LR = Cfg::LR, LC = Cfg::LC, FLAT = Cfg::FLAT;
    extern __shared__ __attribute__((aligned(16))) float wt_tile[];

    const int lane = threadIdx.x & 63;
    const int wv_id = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = FLAT ? 0 : (int)blockIdx.z;
    const int nchunks = a.wt_nchunks;

    // ---- the wave's stream: requested first, it does not depend on the tile
    // (row r of the wave is packed row  block * NW * RPW + wave + NW * r: the rows are sorted by
    // length, so dealing them out like this gives every wave of the workgroup the same share)
    const int wsi = (int)blockIdx.y * NW + wv_id;
    const int row0 = (int)blockIdx.y * (NW * RPW) + wv_id;
    const uint32_t sub4 = (uint32_t)(lane & 15) * 4u;
    // (buffer views of the wave's own stream: `a.nchunks` entries and the spare blocks behind them)
    const uint32_t stream_entries = (uint32_t)a.nchunks + 80u;
    const __amdgpu_buffer_rsrc_t vals = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const uint32_t*)a.nz + (size_t)wsi * a.nchunks), 0, stream_entries * 4u, 0x00020000);
    const __amdgpu_buffer_rsrc_t offs = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.nz_off + (sizeof(T) == 4 ? (size_t)wsi * a.nchunks : 0)), 0, stream_entries * 2u, 0x00020000);
    // (one block ahead)
    float w_cur, w_nxt;
    uint32_t o_cur, o_nxt;
    wt_load_block<T>(vals, offs, 0, sub4, w_cur, o_cur);
    wt_load_block<T>(vals, offs, 1, sub4, w_nxt, o_nxt);
    const int32_t* __restrict__ lens = a.seg_ptr + (size_t)wsi * nchunks * RPW;
    int co_[RPW], len_[RPW];
    float bias_[RPW];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        co_[r] = a.perm[row0 + NW * r];
        len_[r] = lens[r];
    }
#pragma unroll
    for (int r = 0; r < RPW; ++r) bias_[r] = (a.bias && co_[r] >= 0) ? a.bias[co_[r]] : 0.0f;

    // ---- lane -> output pixels: byte offsets inside y / the residual with the channel plane
    //      left out (it enters as the scalar part of the address); a pixel outside the tensor gets
    //      an out-of-range offset, which makes its loads read zero and drops its stores.
    //      (Flattened tiles run over the batch, whose tensors stay below 2^31 bytes.)
    const int hw = a.hwout;
    uint32_t yoff[P], roff[P];
    uint32_t lane_base = (uint32_t)(uintptr_t)(wt_lds_ptr_t)wt_tile;
    int ty = 0, tx = 0;
    if constexpr (FLAT) {
        const int total = a.n * hw;
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const int Q = (int)blockIdx.x * (64 * P) + lane * P + j;
            const int img = wt_divf(Q, hw), q = Q - img * hw;
            const int oh = wt_divf(q, a.yd.w), ow = q - oh * a.yd.w;
            yoff[j] = Q < total ? (uint32_t)(img * (int)a.yd.image + tensor_off(a.yd, oh, ow)) * (uint32_t)sizeof(T) : kWtOutOfRange;
            roff[j] = Q < total ? (uint32_t)(img * (int)a.rd.image + tensor_off(a.rd, oh, ow)) * (uint32_t)sizeof(T) : kWtOutOfRange;
        }
        lane_base += (uint32_t)(lane * P * 4);
    } else {
        ty = wt_divf((int)blockIdx.x, a.tiles_x);
        tx = (int)blockIdx.x - ty * a.tiles_x;
        const int lr = lane % LR, lc = lane / LR;
        const int orow = ty * LR + lr;
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const int ocol = tx * (LC * P) + lc + LC * j;
            const bool in = orow < a.yd.h && ocol < a.yd.w;
            yoff[j] = in ? (uint32_t)tensor_off(a.yd, orow, ocol) * (uint32_t)sizeof(T) : kWtOutOfRange;
            roff[j] = in ? (uint32_t)tensor_off(a.rd, orow, ocol) * (uint32_t)sizeof(T) : kWtOutOfRange;
        }
        lane_base += (uint32_t)((lr * a.wt_pitch + lc * P) * 4);
    }
    const uint32_t yspan = (uint32_t)(a.yd.image * (int64_t)sizeof(T)) * (FLAT ? (uint32_t)a.n : 1u);
    const uint32_t rspan = (uint32_t)(a.rd.image * (int64_t)sizeof(T)) * (FLAT ? (uint32_t)a.n : 1u);
    const __amdgpu_buffer_rsrc_t yrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((char*)a.y + (size_t)n * a.yd.image * sizeof(T)), 0, yspan, 0x00020000);

    // ---- residual up front: one more round trip off the tail
    float resv[RPW][P];
    {
        const __amdgpu_buffer_rsrc_t rrsrc = __builtin_amdgcn_make_buffer_rsrc(
            a.residual ? (void*)((const char*)a.residual + (size_t)n * a.rd.image * sizeof(T)) : (void*)a.y, 0,
            a.residual ? rspan : 0u, 0x00020000);
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            // (the scalar part of an address takes no part in the range check, so it is always a
            // real plane offset; a padding row -- a wave-uniform condition -- reads nothing)
            const uint32_t plane_off = (uint32_t)(co_[r] >= 0 ? co_[r] : 0) * (uint32_t)a.rd.plane * (uint32_t)sizeof(T);
#pragma unroll
            for (int j = 0; j < P; ++j) {
                if (co_[r] < 0) {
                    resv[r][j] = 0.0f;
                } else if constexpr (sizeof(T) == 4) {
                    resv[r][j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rrsrc, roff[j], plane_off, 0));
                } else {
                    resv[r][j] = (float)__builtin_bit_cast(_Float16, __builtin_amdgcn_raw_buffer_load_b16(rrsrc, roff[j], plane_off, 0));
                }
            }
        }
    }

    // ---- staging: a channel plane of the tile is `nstp` runs of 64 words, and a wave stages
    //      the SAME runs of every channel it is given -- run t = wave % nstp (and t + NW where
    //      there are more runs than waves) of the channels congruent to wave / nstp -- so that it
    //      needs the global offsets of one or two runs, not of the whole plane.
    constexpr int SPW = (kWtileMaxSteps + NW - 1) / NW;       // runs a wave may have to take
    const int nstp = a.wt_nstp;
    const int sets = nstp >= NW ? 1 : NW / nstp;              // waves that share a run split the channels
    const int my_set = nstp >= NW ? 0 : wv_id / nstp;
    const bool stages = nstp >= NW || wv_id < sets * nstp;
    uint32_t goff[SPW];
    int gword[SPW];
    {
        const int total = a.n * hw;
#pragma unroll
        for (int k = 0; k < SPW; ++k) {
            const int t = (nstp >= NW ? wv_id : wv_id % nstp) + k * NW;
            const int p = lane + 64 * t;
            gword[k] = (stages && t < nstp && p < a.wt_plane) ? p : -1;
            uint32_t off = kWtOutOfRange;
            if (gword[k] >= 0) {
                if constexpr (FLAT) {
                    const int Q = (int)blockIdx.x * (64 * P) + p;
                    if (Q < total) {
                        const int img = wt_divf(Q, hw), q = Q - img * hw;
                        const int oh = wt_divf(q, a.yd.w), ow = q - oh * a.yd.w;
                        off = (uint32_t)(img * (int)a.xd.image + tensor_off(a.xd, oh * a.stride, ow * a.stride)) * (uint32_t)sizeof(T);
                    }
                } else {
                    const int phase = wt_div(p, a.wt_m_sub), q = p - phase * a.wt_sub;
                    const int pr = wt_div(q, a.wt_m_pitch), rem = q - pr * a.wt_pitch;
                    const int slot = rem / P, j = rem - slot * P;
                    const int pa = wt_div(phase, a.wt_m_nphc), pb = phase - pa * a.wt_nphc;
                    const int row = (ty * LR + pr) * a.stride + pa - a.pad;
                    const int col = (tx * (LC * P) + slot + LC * j) * a.stride + pb - a.pad;
                    if (phase < a.wt_nph && slot < a.wt_ns && row >= 0 && row < a.xd.h && col >= 0 && col < a.xd.w)
                        off = (uint32_t)tensor_off(a.xd, row, col) * (uint32_t)sizeof(T);
                }
            }
            goff[k] = off;
        }
    }
    // flat tiles run over the images of the batch, so the buffer spans the whole tensor
    const uint32_t span = FLAT ? a.image_bytes * (uint32_t)a.n : a.image_bytes;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const char*)a.x + (size_t)n * a.image_bytes), 0, span, 0x00020000);
    const uint32_t plane_bytes = (uint32_t)a.xd.plane * (uint32_t)sizeof(T);
    const int cin = a.xd.c;

    float acc[RPW][P];
#pragma unroll
    for (int r = 0; r < RPW; ++r)
#pragma unroll
        for (int j = 0; j < P; ++j) acc[r][j] = 0.0f;

    // Staging of one chunk: `buffer_load ... lds` moves 64 elements per instruction from per-lane
    // global offsets straight to consecutive LDS words, no register in between (lanes past the
    // end of a plane are masked off: they would land on the next channel).  A 2-byte element
    // arrives zero-extended in a word of its own.
    const int chunk_words = a.wt_cch * a.wt_plane;
    auto stage = [&](int c, float* buf) {
        const int ch0 = c * a.wt_cch;
        const int cch = min(a.wt_cch, cin - ch0);
        for (int ch = my_set; ch < cch; ch += sets) {
            const uint32_t soff = (uint32_t)(ch0 + ch) * plane_bytes;
#pragma unroll
            for (int k = 0; k < SPW; ++k)
                if (gword[k] >= 0) {
                    float* dst = buf + ch * a.wt_plane + (gword[k] - lane);
                    if constexpr (sizeof(T) == 4)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (wt_lds_ptr_t)dst, 4, goff[k], soff, 0, 0);
                    else
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (wt_lds_ptr_t)dst, 2, goff[k], soff, 0, 0);
                }
        }
    };

    // 2-byte storage: once a wave's own share of a chunk has landed it widens it to fp32 in
    // place (the inner loop then runs the plain fp32 FMA, which issues faster than the
    // mixed-precision one: 27 against 34 clocks per nonzero measured).  A run is 16 groups of four
    // words, so the 64 lanes take the same run of four channels at a time.
    auto widen = [&](int c, float* buf) {
        if constexpr (sizeof(T) == 2) {
            const int cch = min(a.wt_cch, cin - c * a.wt_cch);
            const int quad = lane & 15, sub = lane >> 4;
#pragma unroll
            for (int k = 0; k < SPW; ++k) {
                const int t = (nstp >= NW ? wv_id : wv_id % nstp) + k * NW;
                if (!stages || t >= nstp) continue;
                const int word = 64 * t + 4 * quad;             // (a plane is a whole number of 4-word slots)
                if (word >= a.wt_plane) continue;
                for (int ch = my_set + sub * sets; ch < cch; ch += 4 * sets) {
                    wt_u4* q = (wt_u4*)(buf + ch * a.wt_plane + word);
                    const wt_u4 h = *q;
                    wt_u4 f;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        f[e] = __float_as_uint((float)__builtin_bit_cast(_Float16, (unsigned short)h[e]));
                    *q = f;
                }
            }
        }
    };

    // Several chunks: two LDS buffers, chunk c+1 lands while chunk c is consumed (one barrier
    // per chunk); a single chunk is staged and consumed.
    const bool twobuf = a.wt_nbuf == 2;
    int pos = 0;                 // entries of the wave's stream consumed so far (a multiple of 4)
    wt_settle(w_cur, o_cur);
    stage(0, wt_tile);
    for (int c = 0; c < nchunks; ++c) {
        float* buf = wt_tile + ((twobuf && (c & 1)) ? chunk_words : 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // this wave's share of chunk c landed
        widen(c, buf);
        __syncthreads();                                    // ... everyone's; and chunk c-1 is consumed
        if (c + 1 < nchunks) stage(c + 1, wt_tile + ((c & 1) ? 0 : chunk_words));
        const uint32_t lb = lane_base + (uint32_t)((buf - wt_tile) * 4);
        // part lengths of the next chunk: needed only after the next barrier
        int nlen_[RPW];
#pragma unroll
        for (int r = 0; r < RPW; ++r) nlen_[r] = c + 1 < nchunks ? lens[(c + 1) * RPW + r] : 0;

        // ---- accumulate the wave's parts of this chunk: whole blocks of 16 entries where the
        //      part has them, quarter blocks at its ragged ends (parts are padded to 4 entries)
        auto rotate = [&]() {
            // the block is used up: the one in flight becomes current, the one after that is
            // requested (the plan ends in spare blocks, so this stays inside it)
            w_cur = w_nxt;
            o_cur = o_nxt;
            wt_settle(w_cur, o_cur);
            wt_load_block<T>(vals, offs, (pos >> 4) + 2, sub4, w_nxt, o_nxt);
        };
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            int left = len_[r];
            while (left > 0) {
                const int quarter = (pos >> 2) & 3;
                if (quarter == 0 && left >= 16) {
                    wt_group<T, 0, 8>(lb, w_cur, o_cur, acc[r]);
                    wt_group<T, 8, 8>(lb, w_cur, o_cur, acc[r]);
                    rotate();
                    pos += 16;
                    left -= 16;
                    continue;
                }
                if (quarter == 0) wt_group<T, 0, 4>(lb, w_cur, o_cur, acc[r]);
                else if (quarter == 1) wt_group<T, 4, 4>(lb, w_cur, o_cur, acc[r]);
                else if (quarter == 2) wt_group<T, 8, 4>(lb, w_cur, o_cur, acc[r]);
                else {
                    wt_group<T, 12, 4>(lb, w_cur, o_cur, acc[r]);
                    rotate();
                }
                pos += 4;
                left -= 4;
            }
        }
#pragma unroll
        for (int r = 0; r < RPW; ++r) len_[r] = nlen_[r];
    }

    // ---- fused epilogue: + bias, + residual, ReLU, store at the original channel
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int co = co_[r];
        if (co < 0) continue;
        const float b = bias_[r];
        const uint32_t plane_off = (uint32_t)co * (uint32_t)a.yd.plane * (uint32_t)sizeof(T);
#pragma unroll
        for (int j = 0; j < P; ++j) {
            float v = acc[r][j] + b;
            v += resv[r][j];
            if (a.relu) v = v > 0.0f ? v : 0.0f;
            if constexpr (sizeof(T) == 4)
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), yrsrc, yoff[j], plane_off, 0);
            else
                __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, (_Float16)v), yrsrc, yoff[j], plane_off, 0);
        }
    }
}

template <class Cfg>
static hipError_t launch_wtile(const ConvLaunch& a, hipStream_t s) {
    // more than 64 KB of dynamic LDS has to be asked for once per kernel
    static const hipError_t attr = hipFuncSetAttribute((const void*)sconv_wtile_kernel<Cfg>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytesPerCU);
    if (attr != hipSuccess) return attr;
    dim3 grid((unsigned)a.wt_tiles, (unsigned)a.row_groups, Cfg::FLAT ? 1u : (unsigned)a.n);
    dim3 block(Cfg::THREADS);
    CADNN_LAUNCH(sconv_wtile_kernel<Cfg>, grid, block, a.wt_lds_bytes, s, a);
    return hipGetLastError();
}

template <class Cfg>
static ConvVariant make_wtile(const char* name) {
    ConvVariant v{};
    v.name = name;
    v.family = FAM_WTILE;
    v.is_f16 = sizeof(typename Cfg::T) == 2;
    v.kh = 0; v.kw = 0; v.stride = 0;
    v.p = Cfg::P; v.nw = Cfg::NW; v.rpw = Cfg::RPW; v.ks = 1;
    v.unroll = 4;
    v.rw = Cfg::LR;
    v.tw = Cfg::LC;
    v.flat = Cfg::FLAT;
    v.lds_bytes = 0;
    v.launch = &launch_wtile<Cfg>;
    return v;
}

#define CADNN_WTILE_FLAT(T, RPW, NW) \
    make_wtile<WtileCfg<T, 1, 4, RPW, NW, 64>>("swide_" #T "_f4_r" #RPW "w" #NW)
#define CADNN_WTILE_GRID(T, RPW, NW, LR) \
    make_wtile<WtileCfg<T, 0, 4, RPW, NW, LR>>("swide_" #T "_g4_r" #RPW "w" #NW "l" #LR)

#define CADNN_WTILE_SHAPES(T)         \
    CADNN_WTILE_FLAT(T, 1, 8),        \
    CADNN_WTILE_FLAT(T, 2, 8),        \
    CADNN_WTILE_FLAT(T, 4, 8),        \
    CADNN_WTILE_FLAT(T, 8, 8),        \
    CADNN_WTILE_FLAT(T, 1, 16),       \
    CADNN_WTILE_FLAT(T, 2, 16),       \
    CADNN_WTILE_FLAT(T, 4, 16),       \
    CADNN_WTILE_FLAT(T, 8, 16),       \
    CADNN_WTILE_GRID(T, 1, 8, 4),     \
    CADNN_WTILE_GRID(T, 2, 8, 4),     \
    CADNN_WTILE_GRID(T, 4, 8, 4),     \
    CADNN_WTILE_GRID(T, 8, 8, 4),     \
    CADNN_WTILE_GRID(T, 1, 16, 4),    \
    CADNN_WTILE_GRID(T, 2, 16, 4),    \
    CADNN_WTILE_GRID(T, 4, 16, 4),    \
    CADNN_WTILE_GRID(T, 8, 16, 4),    \
    CADNN_WTILE_GRID(T, 1, 8, 8),     \
    CADNN_WTILE_GRID(T, 2, 8, 8),     \
    CADNN_WTILE_GRID(T, 4, 8, 8),     \
    CADNN_WTILE_GRID(T, 8, 8, 8),     \
    CADNN_WTILE_GRID(T, 1, 16, 8),    \
    CADNN_WTILE_GRID(T, 2, 16, 8),    \
    CADNN_WTILE_GRID(T, 4, 16, 8),    \
    CADNN_WTILE_GRID(T, 8, 16, 8),    \
    CADNN_WTILE_GRID(T, 1, 8, 16),    \
    CADNN_WTILE_GRID(T, 2, 8, 16),    \
    CADNN_WTILE_GRID(T, 4, 8, 16),    \
    CADNN_WTILE_GRID(T, 8, 8, 16),    \
    CADNN_WTILE_GRID(T, 1, 16, 16),   \
    CADNN_WTILE_GRID(T, 2, 16, 16),   \
    CADNN_WTILE_GRID(T, 4, 16, 16),   \
    CADNN_WTILE_GRID(T, 8, 16, 16)

const std::vector<ConvVariant>& all_wtile_variants() {
    static const std::vector<ConvVariant> v = {CADNN_WTILE_SHAPES(float), CADNN_WTILE_SHAPES(_Float16)};
    return v;
}

}  // namespace cadnn
