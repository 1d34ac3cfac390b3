// Internal declarations shared by the translation units of libcadnn.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <array>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <functional>
#include <map>
#include <memory>
#include <mutex>
#include <string>
#include <tuple>
#include <vector>

#include "cadnn.h"

namespace cadnn {

// ---- error reporting -------------------------------------------------------
cadnn_status fail(cadnn_status code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

#define CADNN_HIP(expr)                                                                     \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            return ::cadnn::fail(CADNN_EHIP, "%s failed: %s (%s:%d)", #expr,                \
                                 hipGetErrorString(e_), __FILE__, __LINE__);                \
    } while (0)

inline int conv_out(int size, int k, int stride, int pad) {
    const int64_t t = (int64_t)size + 2 * (int64_t)pad - k;
    return t < 0 ? 0 : (int)std::min<int64_t>(t / stride + 1, INT32_MAX);
}

// ---- kernel launches -----------------------------------------------------------
// Every kernel of the library is launched through CADNN_LAUNCH.  Normally that is a plain
// launch.  While a LaunchTimer is installed on the thread (the in-order profile of a net), the
// launch takes the next pair of its events as the kernel's own start and stop marks, so that
// the elapsed time between them is the kernel's duration on the device and nothing else.
struct LaunchTimer {
    static constexpr int kMax = 8;                 // kernels one op may launch while timed
    hipEvent_t start[kMax], stop[kMax];
    int used = 0;
};
extern thread_local LaunchTimer* g_launch_timer;
}  // namespace cadnn
#include <hip/hip_ext.h>
#define CADNN_LAUNCH(kernel, grid, block, shmem, stream, ...)                                                  \
    do {                                                                                                       \
        ::cadnn::LaunchTimer* lt_ = ::cadnn::g_launch_timer;                                                   \
        if (lt_ && lt_->used < ::cadnn::LaunchTimer::kMax) {                                                   \
            hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, lt_->start[lt_->used], lt_->stop[lt_->used], \
                                  0, __VA_ARGS__);                                                             \
            ++lt_->used;                                                                                       \
        } else {                                                                                               \
            hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                               \
        }                                                                                                      \
    } while (0)
namespace cadnn {

// ---- device buffer with RAII -------------------------------------------------
struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
    bool on_host = false;     // filled while a HostPlans scope was alive: p is host memory
    DevBuf() = default;
    DevBuf(const DevBuf&) = delete;
    DevBuf& operator=(const DevBuf&) = delete;
    ~DevBuf() { release(); }
    void release();
    // Allocates (at least 16 bytes so that p is never NULL) and uploads `n` bytes from host.
    cadnn_status upload(const void* host, size_t n);
    // Allocates `n` bytes of device memory, zero-filled if asked (never in a HostPlans scope).
    cadnn_status alloc(size_t n, bool zero);
};

// ---- activation tensor layout --------------------------------------------------
// One image of an activation tensor is `c` planes of (h + 2*ph) rows of `pitch` elements;
// element (ch, i, j) of the image proper sits at ch*plane + origin + i*pitch + j.  With
// ph = pw = 0 this is plain contiguous NCHW.  A halo (ph, pw > 0) is kept at zero by
// whoever owns the buffer: kernels only ever write the image proper, so a consumer
// convolution can read its zero padding from memory instead of testing bounds.
//
// De-interleaved layout (s2d = 1), for tensors read by stride-2 convolutions: the padded
// plane is split by row and column parity into four sub-planes ("phases") of `sub`
// elements and `pitch` elements per row each; padded position (R, C) sits at
// ((R & 1) * 2 + (C & 1)) * sub + (R >> 1) * pitch + (C >> 1).  A stride-2 filter tap then
// walks one phase with unit stride, so such a layer reads memory as densely as a stride-1
// layer does (the paper's memory layout transformation, Section 4, applied to strides).
struct TensorDesc {
    int c, h, w;
    int ph, pw;
    int pitch, plane, origin;
    int64_t image;      // elements between consecutive images
    int s2d, sub;
};

// Element offset of image position (row, col) -- halo positions are row/col < 0 or
// >= h/w -- from the start of its channel plane.
__host__ __device__ inline int tensor_off(const TensorDesc& d, int row, int col) {
    const int R = row + d.ph, C = col + d.pw;
    return d.s2d ? ((R & 1) * 2 + (C & 1)) * d.sub + (R >> 1) * d.pitch + (C >> 1) : R * d.pitch + C;
}

// A plane of kMaxPlane elements or more does not fit the 32-bit element offsets the kernels
// use: its descriptor is clamped there (never used for addressing) and every entry point
// refuses it through desc_too_large.
constexpr int kMaxPlane = 1 << 30;
inline TensorDesc make_desc(int c, int h, int w, int ph = 0, int pw = 0) {
    TensorDesc d;
    d.c = c; d.h = h; d.w = w; d.ph = ph; d.pw = pw;
    const int64_t pitch = (int64_t)w + 2 * (int64_t)pw;
    const int64_t plane = ((int64_t)h + 2 * (int64_t)ph) * pitch;
    const bool fits = plane < kMaxPlane;
    d.pitch = fits ? (int)pitch : 0;
    d.plane = fits ? (int)plane : kMaxPlane;
    d.origin = fits ? ph * d.pitch + pw : 0;
    d.image = (int64_t)c * d.plane;
    d.s2d = 0; d.sub = 0;
    return d;
}
inline bool desc_too_large(const TensorDesc& d) { return d.plane >= kMaxPlane; }

// (callers have checked the plain descriptor of the same tensor with desc_too_large: the
// rounding up of odd sizes adds less than a row and a column)
inline TensorDesc make_desc_s2d(int c, int h, int w, int ph, int pw) {
    TensorDesc d;
    d.c = c; d.h = h; d.w = w; d.ph = ph; d.pw = pw;
    d.pitch = (w + 2 * pw + 1) / 2;
    d.sub = ((h + 2 * ph + 1) / 2) * d.pitch;
    d.plane = 4 * d.sub;
    d.origin = 0;
    d.image = (int64_t)c * d.plane;
    d.s2d = 1;
    return d;
}

// One output element of a k x k window pool (maximum, or the mean over the in-image part of
// the window): flat index r = (c * yd.h + oh) * yd.w + ow inside image `img`.
template <typename T>
__device__ __forceinline__ void windowpool_element(const T* __restrict__ x, T* __restrict__ y, const TensorDesc& xd,
                                                   const TensorDesc& yd, int img, size_t r, int k, int stride, int pad,
                                                   bool mean) {
    const int ow = (int)(r % yd.w);
    const int oh = (int)((r / yd.w) % yd.h);
    const int c = (int)(r / ((size_t)yd.w * yd.h));
    const T* xp = x + (size_t)img * xd.image + (size_t)c * xd.plane + xd.origin;
    int seen = 0;
    float m = 0.0f;
    for (int a = 0; a < k; ++a) {
        const int ih = oh * stride + a - pad;
        if (ih < 0 || ih >= xd.h) continue;
        for (int q = 0; q < k; ++q) {
            const int iw = ow * stride + q - pad;
            if (iw < 0 || iw >= xd.w) continue;
            const float v = (float)xp[(size_t)ih * xd.pitch + iw];
            if (mean) m += v;
            else if (!seen || v > m) m = v;
            ++seen;
        }
    }
    if (mean && seen) m /= (float)seen;
    // (tensor_off: the output may be a de-interleaved tensor -- a k = 1 pool is how one is made from a plain one)
    y[(size_t)img * yd.image + (size_t)c * yd.plane + tensor_off(yd, oh, ow)] = (T)m;
}

// ---- convolution kernel variants ------------------------------------------------
// A variant is one instantiation of a sparse convolution kernel.  Its compile-time
// geometry decides how a canonical column index k = (ci*KH + r)*KW + c is laid out in the
// device copy of the nonzero stream (a "plan"), so every variant owns its plans.
//
//  FAM_TILE   : activations staged per channel chunk in an LDS tile with halo; lanes are
//               the pixels of a TW x TH tile; entries are (value, byte offset in the tile).
//  FAM_DIRECT : no staging; lanes are flattened output pixels and read activations from
//               global memory through a buffer resource (out-of-image taps become
//               out-of-range buffer offsets, which read as zero); a row's entries are
//               regrouped tap-major so the per-lane tap offset is a fixed register;
//               entries are (value, input channel).
//  FAM_LINEAR : no staging and no bounds handling at all: the address of a tap is
//               lane offset + (channel, tap) offset, both linear in the padded layout.
//               Serves 1x1 filters on any input and larger filters on inputs whose zero
//               halo covers the padding; entries are (value, byte offset of the tap),
//               in canonical order, so a plan also depends on the input's plane/pitch.
//  FAM_DENSE  : the layer as a dense implicit GEMM on the matrix cores; the plan is the
//               unpacked [cout][K] weight matrix.  Offered only when at least a quarter
//               of the weights are nonzero (the unpruned first layer of a network).
//  FAM_STILE  : LDS tiles as FAM_TILE, but every wave of the workgroup stages and consumes
//               its own channel chunks (no barrier in the main loop) for all G rows of
//               the workgroup; the plan is chunk-major per group of G rows.
//  FAM_PTILE  : the workgroup stages ONE input tile (all channels, or channel chunks in
//               turn) in LDS for a 7-row block of output pixels and all its waves read it:
//               the waves split G rows and each row's nonzeros between them, so a staged
//               element is reused by every row of the group; entries are (value, byte
//               offset of the tap in the staged tile).
//  FAM_WTILE  : ("wide" tile) the workgroup stages one input tile in LDS as FAM_PTILE does, but
//               a lane owns P = 4 or 8 output pixels whose activations lie side by side in the
//               staged tile and arrive with ONE 128-bit LDS read per nonzero; the weight and
//               the tile offset of a nonzero reach the FMAs and the address add as lane
//               broadcasts inside those instructions (no scalar copy), and the stream is the
//               compact one: 32-bit value + 16-bit tile offset (fp32 storage), or 16-bit value +
//               16-bit tile offset (fp16 storage).
enum ConvFamily { FAM_TILE = 0, FAM_DIRECT = 1, FAM_LINEAR = 2, FAM_DENSE = 3, FAM_STILE = 4, FAM_PTILE = 5, FAM_WTILE = 6 };

struct ConvLaunch;
constexpr int kMaxCoLaunch = 8;   // layers (and riding pools) one launch can hold

struct ConvVariant {
    const char* name;
    int family;
    bool is_f16;          // activation storage type served (false = fp32, true = fp16)
    int kh, kw;           // filter geometry served (0 = any, FAM_LINEAR)
    int stride;           // stride served (0 = any)
    int p;                // output pixels per lane
    int nw, rpw;          // waves per workgroup, packed rows per wave
    int ks;               // waves that split one row's nonzeros (partial sums reduced in LDS)
    // FAM_TILE only
    int tw, rw;           // lanes along ow, lane rows per wave
    int cch;              // input channels staged per chunk
    int th;               // = rw * p   output rows per tile
    int rh, nrph;         // LDS rows per row phase, number of row phases
    int cw, nph;          // LDS columns per column phase, number of column phases
    int pitch, plane;     // LDS floats per tile row / per channel
    int elem_bytes;       // size of one staged tile element in LDS
    int unroll;           // nonzeros per scalar fetch; segments are padded to a multiple of it
    int adjacent;           // FAM_LINEAR: a lane's P pixels are adjacent in one output row (unit stride only)
    int s2d;              // FAM_LINEAR: understands de-interleaved output / residual / pixel-wise input
    int dual;             // FAM_LINEAR: accumulates a fused 1x1 shortcut on a second input
    int pool;             // FAM_LINEAR: global average pool fused into the epilogue
    int dw;               // FAM_LINEAR: a 3x3 depthwise layer fused into the epilogue
    int quad;             // FAM_LINEAR: rpw packed rows per wave side by side, 64 / rpw lanes x p adjacent pixels each (small images)
    int nz_cap;           // FAM_STILE: most stream entries per (row group, chunk) the kernel buffers
    int flat;             // FAM_WTILE: 1 = pixel-wise layers (1x1 filters), pixels flattened over the batch;
                          //            0 = filters with taps, lanes in an (rw x 64/rw) grid over a 2-D tile
    int splitk;           // FAM_DENSE, large tiles: workgroups that share one output tile, each a slice of K (0, 1: one)
    size_t lds_bytes;
    hipError_t (*launch)(const ConvLaunch&, hipStream_t);
    // several layers (at most kMaxCoLaunch) at once from a device table of launch records, of
    // which host_records is the host copy (NULL: not offered)
    hipError_t (*launch_multi)(const ConvLaunch* table_dev, const ConvLaunch* host_records, int layers, int images,
                               hipStream_t);
    int rows_per_block() const { return family == FAM_TILE || family == FAM_DENSE ? nw * rpw : (nw / ks) * rpw; }
};

struct ConvLaunch {
    const void* x;
    void* y;
    const float* bias;
    const void* residual;
    const uint2* nz;          // plan entries, segment-padded
    const uint16_t* nz_off;   // FAM_WTILE, fp32 storage: the entries' 16-bit tile offsets (nz holds the values)
    const int32_t* seg_ptr;   // plan segment table
    const int32_t* perm;      // [rows_padded] original channel, -1 for padding rows
    TensorDesc xd, yd, rd;    // layouts of x, y and residual
    int n, cout, stride, pad, relu, nchunks;
    int kh, kw, is_f16;
    int tiles_x, tiles_y, row_groups;
    int hwout;                // yd.h * yd.w
    // FAM_LINEAR ragged-row instantiations: output pixels are enumerated over rows of wq
    // positions, wq = yd.w rounded up to the adjacent pixels a lane takes, so that a lane's
    // group never straddles two rows; positions at or beyond yd.w are computed and not stored
    int wq, hwq;              // hwq = yd.h * wq
    // fused 1x1 shortcut (FAM_LINEAR dual instantiations): second input, plain view
    const void* x2;
    const float* bias2;
    TensorDesc x2d;
    int stride2;
    uint32_t image2_bytes;
    // fused global average pool (FAM_LINEAR pool instantiations): [n][cout] means
    void* pool_y;
    float pool_scale;
    // fused depthwise layer (FAM_LINEAR dw instantiations): its filter table, bias, output
    void* dw_y;
    const float* dw_w;
    const float* dw_bias;
    TensorDesc dw_yd;
    int dw_stride, dw_relu;
    // FAM_PTILE: geometry of the staged tile (see PtileGeom)
    int pt_pitch, pt_sub, pt_plane, pt_nphc, pt_nph, pt_in_rows, pt_in_cols, pt_cch, pt_nstp, pt_nchunks;
    uint32_t pt_lds_bytes;
    int pt_nbuf;
    // FAM_WTILE: geometry of the staged tile (see WtileGeom)
    int wt_lc, wt_ns, wt_pitch, wt_sub, wt_plane, wt_nphc, wt_nph, wt_cch, wt_nstp, wt_nchunks, wt_nbuf;
    int wt_tiles;             // pixel tiles per image (2-D tiles) or over the whole batch (flattened pixels)
    uint32_t wt_m_sub, wt_m_pitch, wt_m_nphc;   // ceil(2^32 / d) for d = wt_sub, wt_pitch, wt_nphc: n / d = mulhi(n, m) for n < 2^16
    uint32_t wt_lds_bytes;
    uint32_t image_bytes;     // xd.image * sizeof(element)
    // FAM_DENSE with K split over workgroups: the slices' fp32 partial tiles and one arrival
    // counter per output tile (zero between launches: the last arriver resets it)
    int sk;
    float* sk_part;
    int* sk_count;
    // launches of several layers (launch_multi) may carry window pools among them: 0 = a
    // convolution, 1 = a k x k maximum pool, 2 = a k x k mean pool (x, y, xd, yd, stride, pad
    // as for a layer; the output elements of image n are dealt round robin to the threads of
    // the tiles_x * row_groups workgroups)
    int op_type, pool_k;
};

struct ConvPlan {
    const ConvVariant* variant = nullptr;
    DevBuf nz, seg_ptr, perm;
    DevBuf nz_off;            // FAM_WTILE, fp32 storage: 16-bit tile offsets, one per entry of nz
    int64_t walked = 0;       // stream entries the kernels walk (real entries + the padding of the parts); the
                              // fixed stride between the parts of some layouts leaves gaps that are never read
    int entry_bytes = 8;      // bytes of one entry (value + index) as stored on the device
    int nchunks = 0;
    int rows_padded = 0;
    int64_t nz_padded = 0;
    // handed out for an ordinary launch (not only timed by a tuning pass): a captured graph or
    // a launch in flight may hold its device pointers, so it lives as long as the handle
    mutable bool in_use = false;
};

// While one of these is alive on a thread, DevBuf::upload keeps the data in host memory instead
// of sending it to the device: device layouts can then be built, measured and decoded without
// a GPU (cadnn_conv2d_plan_info, cadnn_conv2d_plan_unpack).
struct HostPlans {
    HostPlans();
    ~HostPlans();
    HostPlans(const HostPlans&) = delete;
    HostPlans& operator=(const HostPlans&) = delete;
};

// While one of these is alive on a thread, nothing may be allocated on the device: a device
// layout that is not there yet is an error (CADNN_EINVAL) instead of being built.
struct NoDeviceAlloc {
    NoDeviceAlloc();
    ~NoDeviceAlloc();
    NoDeviceAlloc(const NoDeviceAlloc&) = delete;
    NoDeviceAlloc& operator=(const NoDeviceAlloc&) = delete;
};

// While one of these is alive on a thread, the plans that thread asks for are trial plans of a
// tuning pass: they may be freed again when the pass ends (drop_unpinned_plans).
struct TrialPlans {
    TrialPlans();
    ~TrialPlans();
    TrialPlans(const TrialPlans&) = delete;
    TrialPlans& operator=(const TrialPlans&) = delete;
};

// Staged tile of the FAM_PTILE kernels for one layer geometry.  Two lane arrangements:
//   tw = 8 : an 8 x 8 lane grid of which 7 x 7 is used; pixel j of a lane lies 7*j columns
//            to the right: a tile serves 7 output rows x 7*P columns (image sizes that are
//            multiples of 7 but not of 14, and 7 x 7 images);
//   tw = 16: a 4 x 16 lane grid of which 4 x 14 is used; pixel j of a lane lies 4*j rows
//            further down: a tile serves 4*P output rows x 14 columns and the staged rows
//            are exactly 16 words apart, so the four lane rows of a 32-lane LDS access fall
//            into disjoint banks (filters up to 3 wide).
// The input region a tile needs is de-interleaved by the stride into
// nphr x nphc phases (sub-planes) so that lanes always read consecutive LDS words:
// input element (u, v) of the region sits at phase (u % S, v % S), position (u / S, v / S).
// `alias`: 3x3 / stride-1 tiles that span the whole image width drop the right halo column
// (its reads fall on the left halo of the next row, which is zero as well), which makes the
// pitch 8 words: bank-conflict free and small enough for 512 channels of a 7x7 image.
struct PtileGeom {
    int S, P;
    int tile_h, tile_w;       // output pixels of a tile
    int in_rows, in_cols;     // input region of a tile
    int nphr, nphc;           // phases used
    int pitch, sub, plane;    // words per tile row / per phase / per channel
    int nstp;                 // 64-word staging steps per channel
    int cch, nchunks;         // channels staged at a time, number of such chunks
    int nbuf;                 // LDS buffers: 2 = the next chunk is staged while one is consumed (fp32)
    int alias;
    size_t lds_bytes;
};
PtileGeom ptile_geom(const ConvVariant& v, int cin, int kh, int kw, int stride, int pad, int wout);   // v.is_f16 matters

// Staged tile of the FAM_WTILE kernels for one layer geometry.  A lane owns P output pixels.
//   flat = 1 (1x1 filters): the output pixels of the whole batch are numbered n * hout * wout + q and a
//            tile is 64 * P consecutive ones, lane l owning pixels P*l .. P*l + P-1; a channel plane of
//            the tile is those pixels' 64 * P activations in the same order.
//   flat = 0: the lanes form an lr x lc grid (lane l -> row l % lr, column l / lr); pixel j of a lane
//            lies lc * j columns to the right, so a tile is lr rows x lc * P columns of one image.  The
//            staged region is de-interleaved by the stride into nphr x nphc phases; a row of a phase
//            holds `ns` slots of P words -- word j of slot s is the phase's element at column
//            s + lc * j -- so the P activations a lane needs for a tap are the 16 or 32 consecutive
//            bytes of slot (lane column + tap column / stride).  Columns that two slots share are
//            staged twice.  Rows are `nsp` >= ns slots apart, chosen so that 16 consecutive lanes
//            read 16 different 16-byte bank groups.
// A tap's offset in a chunk is a multiple of 16 bytes and is stored divided by 16, in 16 bits.
struct WtileGeom {
    int flat, S, P;
    int lr, lc;               // lane grid (flat: 64 x 1)
    int tile_h, tile_w;       // output pixels of a tile (flat: 1 x 64*P)
    int nphr, nphc;           // phases used
    int ph_rows, ns, nsp;     // rows per phase, slots used per row, slots between rows
    int pitch, sub, plane;    // words per phase row / per phase / per channel
    int nstp;                 // 64-word staging steps per channel
    int cch, nchunks, nbuf;   // channels staged at a time, number of chunks, LDS buffers
    size_t lds_bytes;
};
WtileGeom wtile_geom(const ConvVariant& v, int cin, int kh, int kw, int stride);
constexpr int kWtileMaxSteps = 10;
// LDS a workgroup may take: half of a compute unit's for the 8-wave instantiations (two
// workgroups then share a compute unit and one computes while the other waits at a barrier),
// all of it for the 16-wave ones (fewer, larger channel chunks)
inline size_t wtile_lds_budget(const ConvVariant& v) { return v.nw >= 16 ? (size_t)160 * 1024 : (size_t)80 * 1024; }
constexpr int kPtileMaxSteps = 9;
constexpr size_t kLdsBytesPerCU = 160 * 1024;
// a plan entry's byte offset that no buffer this library accepts reaches: its load reads zero
constexpr uint32_t kPlanOutOfRange = 0x7ffffff0u;
constexpr int kFcTailEntries = 1024;   // 4 loads x 64 lanes x 4 entries

// (variant, a, b, shortcut weights, shortcut input plane): FAM_LINEAR a = input plane,
// b = input pitch; FAM_PTILE a = stride, b = alias flag; 0, 0 for layout-independent plans;
// the last two are NULL, 0 unless a 1x1 shortcut is fused into the layer
typedef std::tuple<const ConvVariant*, int, int, const void*, int> PlanKey;
// (n, h, w, stride, pad, input halo rows, input halo columns, flags: 1 = input
// de-interleaved, 2 = output or residual de-interleaved, 4 = a shortcut is fused in,
// 8 = a global average pool is fused in, 16 = a depthwise layer is fused in, 32 = with stride 2)
typedef std::array<int, 8> GeomKey;
struct SkScratch { DevBuf part, count; bool in_use = false; };

const std::vector<ConvVariant>& all_tile_variants();
const std::vector<ConvVariant>& all_direct_variants();
const std::vector<ConvVariant>& all_linear_variants();
// (the same plans and addresses, four rows per wave: conv_quad.hip)
const std::vector<ConvVariant>& all_quad_variants();
const std::vector<ConvVariant>& all_dense_variants();
// fp16 storage, 128 x 128 tiles, tap-major weight matrix (marked by tw == 128)
const std::vector<ConvVariant>& all_dense_wide_variants();
// (in_bytes / out_bytes: the whole batch of the largest tensor on each side)
bool dense_wide_serves(bool is_f16, int cin, int taps, int64_t in_bytes, int64_t out_bytes, int64_t pixels);
cadnn_status dense_wide_conv2d_raw(const void* w_dev, const void* x, const TensorDesc& xd, void* y, const TensorDesc& yd,
                                   const void* residual, const TensorDesc& rd, int n, int cout, int kh, int kw, int stride,
                                   int pad, const void* bias, int relu, hipStream_t s);
const std::vector<ConvVariant>& all_stile_variants();
const std::vector<ConvVariant>& all_ptile_variants();
const std::vector<ConvVariant>& all_wtile_variants();

}  // namespace cadnn

// ---- opaque handles ----------------------------------------------------------
struct cadnn_weights {
    int cout = 0, cin = 0, kh = 0, kw = 0;
    cadnn_dtype dtype = CADNN_F32;
    int64_t nnz = 0;
    // canonical form (host)
    std::vector<int32_t> perm, row_ptr, col_idx;
    std::vector<float> vals;       // fp32 values (for F16 handles: the binary16 value widened)
    std::vector<uint16_t> vals16;  // F16 handles only: binary16 bit patterns
    // device copies used by the FC kernel (canonical order)
    mutable cadnn::DevBuf d_row_ptr, d_perm, d_col, d_val;
    mutable bool fc_ready = false;
    // compact FC form (cin <= 65536): every row padded with zero entries to a multiple of
    // four, 16-bit columns, values in the handle's own precision; d_frow[r] is the row's
    // start in units of four entries.  kFcTailEntries zero entries follow the last row so
    // that a wave may read a whole chunk past a row's end.
    mutable cadnn::DevBuf d_frow, d_fcol, d_fval;
    mutable bool fc_compact = false;
    // depthwise filters (cin == 1): fp32 table [cout][kh*kw], zeros where pruned
    mutable cadnn::DevBuf d_dw;
    mutable bool dw_ready = false;
    // conv plans, built lazily
    mutable std::mutex mu;
    // (shared: a co-launch table of the net runner holds the plans its records point into)
    mutable std::map<cadnn::PlanKey, std::shared_ptr<cadnn::ConvPlan>> plans;
    // variant pinned for a geometry by tuning or by the caller
    mutable std::map<cadnn::GeomKey, const cadnn::ConvVariant*> chosen;
    // scratch of the split-K matrix-core variants, per (variant, layer geometry); never freed
    // or moved before the handle is (launch records and captured graphs point into it); two
    // launches of one layer that overlap in time would share it and race
    mutable std::map<std::pair<const cadnn::ConvVariant*, cadnn::GeomKey>, std::unique_ptr<cadnn::SkScratch>> sk_scratch;
    // FAM_STILE variants whose per-(row group, chunk) stream was measured against the kernel's buffer
    // (its own lock: candidates are also listed by callers that hold `mu`)
    mutable std::mutex stile_mu;
    mutable std::map<const cadnn::ConvVariant*, bool> stile_ok;
    size_t elem() const { return dtype == CADNN_F16 ? 2 : 4; }
};

namespace cadnn {
// A 1x1 projection shortcut fused into the layer whose residual it would have been
// (paper Section 4, layer fusion): its weights, the tensor it reads and that tensor's layout.
// Or (w == NULL, pool_y != NULL) a global average pool fused into the layer it reads: the
// layer writes the pooled [n][cout] vector to pool_y instead of its feature map.
struct ConvExtra {
    const cadnn_weights* w;
    const void* x;
    TensorDesc xd;
    int stride;
    const void* bias;     // device, fp32, may be NULL
    void* pool_y;
    // Or (dw != NULL) a 3x3 depthwise layer with padding 1 fused into the layer that produces
    // its input: the layer's own feature map is not written, the depthwise output is.
    const cadnn_weights* dw;
    const void* dw_bias;  // device, fp32, may be NULL
    int dw_stride, dw_relu;
    void* dw_y;
    TensorDesc dw_yd;
};

// stride / pad / wout matter to FAM_PTILE plans only.
// Whether every (row group, channel chunk) stream of these weights fits the buffer of a
// FAM_STILE variant (exact; cached on the handle).
bool stile_streams_fit(const cadnn_weights* w, const ConvVariant* v);
// Scratch of a split-K variant for one layer geometry: allocated (counters zeroed) on first use;
// like a plan it is dropped after tuning unless an ordinary launch has used it or its variant is pinned.
cadnn_status get_sk_scratch(const cadnn_weights* w, const ConvVariant* v, const GeomKey& key, size_t part_bytes,
                            size_t count_bytes, float** part, int** count);
cadnn_status get_conv_plan(const cadnn_weights* w, const ConvVariant* v, const TensorDesc& xd, int stride,
                           int pad, int wout, const ConvPlan** out, const ConvExtra* ex = nullptr,
                           std::shared_ptr<ConvPlan>* keep = nullptr);
void drop_unpinned_plans(const cadnn_weights* w);
// The plan of variant v for the layer, built in HOST memory (inside a HostPlans scope), never cached.
cadnn_status build_host_plan(const cadnn_weights* w, const ConvVariant* v, const TensorDesc& xd, int stride,
                             int pad, int wout, ConvPlan* plan);
// Dense [cout][cin*kh*kw] tensor rebuilt from the stream of a host-built FAM_WTILE plan.
cadnn_status wtile_plan_unpack(const cadnn_weights* w, const ConvVariant* v, int stride, const ConvPlan& plan, float* out);
cadnn_status ensure_fc_device(const cadnn_weights* w);
// A new handle whose rows are the rows of `parts` stacked in order (same cin, 1x1, same type):
// the layers that read one tensor pixel by pixel, merged into one layer with more channels.
cadnn_status merge_weights(const std::vector<const cadnn_weights*>& parts, cadnn_weights** out);
cadnn_status ensure_dw_device(const cadnn_weights* w);
uint16_t f32_to_f16_rne(float f);
float f16_to_f32(uint16_t h);

cadnn_status launch_fc(const cadnn_weights* w, const void* x, void* y, int n, const float* bias,
                       int relu, hipStream_t s);
cadnn_status launch_copy(const void* src, void* dst, size_t bytes, hipStream_t s);
cadnn_status launch_zero(void* dst, size_t bytes, hipStream_t s);
// Depthwise layer on plain (possibly haloed) tensors; yd carries the output size.
cadnn_status launch_depthwise(const cadnn_weights* w, const void* x, const TensorDesc& xd, void* y,
                              const TensorDesc& yd, int n, int stride, int pad, const float* bias, int relu,
                              hipStream_t s);
cadnn_status launch_maxpool(const void* x, const TensorDesc& xd, void* y, const TensorDesc& yd, int n,
                            int k, int stride, int pad, cadnn_dtype dt, hipStream_t s);
cadnn_status launch_avgpool2d(const void* x, const TensorDesc& xd, void* y, const TensorDesc& yd, int n,
                              int k, int stride, int pad, cadnn_dtype dt, hipStream_t s);
cadnn_status launch_avgpool(const void* x, const TensorDesc& xd, void* y, int n, cadnn_dtype dt,
                            hipStream_t s);

// Layer entry points on explicit layouts (the C ABI wraps them with contiguous layouts).
cadnn_status conv2d_impl(const cadnn_weights* w, const void* x, const TensorDesc& xd, void* y,
                         const TensorDesc& yd, const void* residual, const TensorDesc& rd, int n,
                         int stride, int pad, const void* bias, int relu, hipStream_t s,
                         const ConvExtra* ex = nullptr);
cadnn_status conv2d_tune_impl(const cadnn_weights* w, const void* x, const TensorDesc& xd, void* y,
                              const TensorDesc& yd, const void* residual, const TensorDesc& rd, int n,
                              int stride, int pad, const void* bias, int relu, hipStream_t s, int reps,
                              float* best_us, const std::function<cadnn_status()>* before = nullptr,
                              const ConvExtra* ex = nullptr);
// Independent layers launched as one kernel (the net runner's co-launch): one member.
struct ConvMember {
    const cadnn_weights* w;
    const void* x;
    TensorDesc xd;
    void* y;
    TensorDesc yd;
    const void* residual;   // may be NULL
    TensorDesc rd;
    int stride, pad;
    const void* bias;
    int relu;
    int pool_kind, pool_k;  // pool_kind 1 / 2: not a layer but a maximum / mean window pool (w = NULL) riding along
};
// Variants that can serve all members in one launch (none: they cannot share one) and the
// untuned pick among them.
cadnn_status conv2d_group_candidates(const std::vector<ConvMember>& members, int n,
                                     std::vector<const ConvVariant*>* out, const ConvVariant** pick);
// The members' launch records for variant v (plans are built on first use); `keep` receives
// the plans the records point into.
cadnn_status conv2d_group_records(const std::vector<ConvMember>& members, int n, const ConvVariant* v,
                                  std::vector<ConvLaunch>* records,
                                  std::vector<std::shared_ptr<ConvPlan>>* keep = nullptr);
// Times every such variant on the members' own buffers; *best_v stays NULL if none serves them.
cadnn_status conv2d_group_tune(const std::vector<ConvMember>& members, int n, hipStream_t s, int reps,
                               const std::function<cadnn_status()>* before, const ConvVariant** best_v,
                               float* best_us);
// Name of the variant that would serve the layer (NULL if none).
// `out_s2d`: the layer's output or residual is in the de-interleaved layout.
const char* conv2d_variant_name_impl(const cadnn_weights* w, const TensorDesc& xd, int n, int stride, int pad,
                                     int out_s2d = 0, const ConvExtra* ex = nullptr);
cadnn_status conv2d_list_variants_impl(const cadnn_weights* w, const TensorDesc& xd, int n, int stride, int pad,
                                       char* buf, size_t len, int out_s2d = 0, const ConvExtra* ex = nullptr);
cadnn_status conv2d_set_variant_impl(const cadnn_weights* w, const TensorDesc& xd, int n, int stride, int pad,
                                     const char* name, int out_s2d = 0, const ConvExtra* ex = nullptr);
cadnn_status conv2d_prepare_impl(const cadnn_weights* w, const TensorDesc& xd, int n, int stride, int pad,
                                 int out_s2d = 0, const ConvExtra* ex = nullptr);
cadnn_status dense_conv2d_desc(const void* w_dev, const void* x, const TensorDesc& xd, void* y,
                               const TensorDesc& yd, const void* residual, const TensorDesc& rd, int n,
                               int cout, int kh, int kw, int stride, int pad, const void* bias, int relu,
                               cadnn_dtype dtype, hipStream_t s);
cadnn_status dense_conv2d_impl(const void* w_dev, const void* x, void* y, int n, int cin, int h,
                               int wdt, int cout, int kh, int kw, int stride, int pad,
                               const void* bias, const void* residual, int relu, cadnn_dtype dtype,
                               hipStream_t s);
}  // namespace cadnn
