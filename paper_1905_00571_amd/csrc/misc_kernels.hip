// Sparse fully connected layer (row-per-wave SpMV / skinny SpMM) and the pooling layers
// that sit between the convolutions of the benchmark networks.
#include <algorithm>

#include "internal.h"

namespace cadnn {

// One wave per packed row: lanes stride over the row's nonzeros with coalesced loads of
// (value, column), gather the activations, and finish with a wavefront shuffle reduction.
// NB batch entries are carried per pass so the weights are streamed once per NB images.
template <typename T, int NB>
__global__ __launch_bounds__(256) void sfc_kernel(const int32_t* __restrict__ row_ptr,
                                                  const int32_t* __restrict__ perm,
                                                  const int32_t* __restrict__ col,
                                                  const float* __restrict__ val,
                                                  const T* __restrict__ x, T* __restrict__ y,
                                                  const float* __restrict__ bias, int n, int cin,
                                                  int cout, int relu) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= cout) return;
    const int n0 = blockIdx.y * NB;
    const int s = row_ptr[row], e = row_ptr[row + 1];
    float acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = 0.0f;
    for (int i = s + lane; i < e; i += 64) {
        const int c = col[i];
        const float v = val[i];
#pragma unroll
        for (int b = 0; b < NB; ++b)
            if (n0 + b < n) acc[b] = fmaf(v, (float)x[(size_t)(n0 + b) * cin + c], acc[b]);
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        float v = acc[b];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        acc[b] = v;
    }
    if (lane == 0) {
        const int co = perm[row];
        const float bv = bias ? bias[co] : 0.0f;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (n0 + b < n) {
                float v = acc[b] + bv;
                if (relu) v = v > 0.0f ? v : 0.0f;
                y[(size_t)(n0 + b) * cout + co] = (T)v;
            }
        }
    }
}

// The same product for matrices whose columns fit 16 bits, with the input vectors of NB
// images staged in LDS first.  The activation gather, which touches up to 64 different cache
// lines per wave instruction when it goes to the vector L1, becomes an LDS read, and the
// weights stream as aligned 16-byte (values) + 8-byte (columns) loads per lane, four
// nonzeros at a time, up to four such loads in flight per lane.  Row r goes to workgroup
// r % gridDim.x, so the rows, which are ordered by length, spread evenly over the workgroups.
// Rows are padded to a multiple of four entries and the arrays end in kFcTailEntries
// zero entries: a chunk may be read whole past the end of its row and masked afterwards.
typedef float fc_f4 __attribute__((ext_vector_type(4)));
typedef _Float16 fc_h4 __attribute__((ext_vector_type(4)));
typedef unsigned short fc_u4 __attribute__((ext_vector_type(4)));
template <typename T> struct FcVec { typedef fc_f4 type; };
template <> struct FcVec<_Float16> { typedef fc_h4 type; };

template <typename T, int NB, int U>
__device__ __forceinline__ void fc_use(const typename FcVec<T>::type (&v)[U], const fc_u4 (&c)[U],
                                       const T* xs, int cin, int nb, float (&acc)[NB]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float wv = (float)v[u][k];
            const int ci = c[u][k];
#pragma unroll
            for (int b = 0; b < NB; ++b)
                if (b < nb) acc[b] = fmaf(wv, (float)xs[b * cin + ci], acc[b]);
        }
    }
}

// Loads U x 64 groups of four entries starting at group `first` (this lane's), whole, and
// zeroes the values of the groups at or past e4, the end of the row; their columns become
// `safe`, columns of the row itself, so that the zero never meets an activation the row does
// not read (0 * Inf would be NaN).
template <typename T, int NB, int U>
__device__ __forceinline__ void fc_chunk(const typename FcVec<T>::type* __restrict__ val4,
                                         const fc_u4* __restrict__ col4, const T* xs, int cin, int nb,
                                         int first, int e4, const fc_u4 safe, float (&acc)[NB]) {
    typename FcVec<T>::type v[U];
    fc_u4 c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        v[u] = val4[first + u * 64];
        c[u] = col4[first + u * 64];
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (first + u * 64 >= e4) { v[u] = 0; c[u] = safe; }
    fc_use<T, NB, U>(v, c, xs, cin, nb, acc);
}

template <typename T, int NB, int THREADS>
__global__ __launch_bounds__(THREADS) void sfc_lds_kernel(const int32_t* __restrict__ row4,
                                                          const int32_t* __restrict__ perm,
                                                          const void* __restrict__ col,
                                                          const void* __restrict__ val,
                                                          const T* __restrict__ x, T* __restrict__ y,
                                                          const float* __restrict__ bias, int n, int cin,
                                                          int cout, int relu) {
    extern __shared__ __align__(16) unsigned char fc_smem[];
    T* xs = (T*)fc_smem;
    typedef typename FcVec<T>::type VT;
    constexpr int WPB = THREADS / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n0 = blockIdx.y * NB;
    const int nb = min(NB, n - n0);
    const VT* val4 = (const VT*)val;
    const fc_u4* col4 = (const fc_u4*)col;
    const int G = gridDim.x;
    const T* xg = x + (size_t)n0 * cin;
    for (int i = threadIdx.x; i < nb * cin; i += THREADS) xs[i] = xg[i];
    __syncthreads();
    for (int row = blockIdx.x + G * wave; row < cout; row += G * WPB) {
        const int s4 = row4[row], e4 = row4[row + 1];
        float acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = 0.0f;
        int base = s4;
        const fc_u4 safe = col4[s4];      // (the arrays end in spare entries: in range for an empty last row too)
        for (; e4 - base > 128; base += 256)
            fc_chunk<T, NB, 4>(val4, col4, xs, cin, nb, base + lane, e4, safe, acc);
        if (e4 - base > 64)
            fc_chunk<T, NB, 2>(val4, col4, xs, cin, nb, base + lane, e4, safe, acc);
        else if (e4 - base > 0)
            fc_chunk<T, NB, 1>(val4, col4, xs, cin, nb, base + lane, e4, safe, acc);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float v = acc[b];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
            acc[b] = v;
        }
        if (lane == 0) {
            const int co = perm[row];
            const float bv = bias ? bias[co] : 0.0f;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                if (b < nb) {
                    float v = acc[b] + bv;
                    if (relu) v = v > 0.0f ? v : 0.0f;
                    y[(size_t)(n0 + b) * cout + co] = (T)v;
                }
            }
        }
    }
}

template <typename T, int NB, int THREADS>
static hipError_t launch_fc_lds(const cadnn_weights* w, const void* x, void* y, int n, const float* bias,
                                int relu, hipStream_t s) {
    // more than 64 KB of dynamic LDS has to be asked for once per kernel
    static const hipError_t attr =
        hipFuncSetAttribute((const void*)sfc_lds_kernel<T, NB, THREADS>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytesPerCU);
    if (attr != hipSuccess) return attr;
    const size_t lds = (size_t)NB * w->cin * sizeof(T);
    constexpr int WPB = THREADS / 64;
    const int per_cu = (int)std::min<size_t>(2048 / THREADS, std::max<size_t>(1, kLdsBytesPerCU / std::max<size_t>(lds, 1)));
    const int gx = std::min((w->cout + WPB - 1) / WPB, 256 * per_cu);
    CADNN_LAUNCH((sfc_lds_kernel<T, NB, THREADS>), dim3((unsigned)gx, (unsigned)((n + NB - 1) / NB)),
                       dim3(THREADS), lds, s, (const int32_t*)w->d_frow.p, (const int32_t*)w->d_perm.p,
                       w->d_fcol.p, w->d_fval.p, (const T*)x, (T*)y, bias, n, w->cin, w->cout, relu);
    return hipGetLastError();
}

template <typename T>
static cadnn_status launch_fc_t(const cadnn_weights* w, const void* x, void* y, int n,
                                const float* bias, int relu, hipStream_t s) {
    // The staged kernel pays for itself once the gather is long (many nonzeros) or the weights
    // serve several images; small single-image products are latency-bound and skip the staging.
    if (w->fc_compact && (n > 1 || w->nnz >= (1 << 20))) {
        // images per pass: eight when their input vectors fit LDS together, else one
        const size_t vec = (size_t)w->cin * sizeof(T);
        const int nb = n > 1 && 8 * vec <= kLdsBytesPerCU ? 8 : (vec <= kLdsBytesPerCU && n <= 65535 ? 1 : 0);
        // 16 waves per workgroup once there are enough rows to give every wave one
        const bool big = w->cout > 256 * 4;
        if (nb == 8) {
            const hipError_t e = big ? launch_fc_lds<T, 8, 1024>(w, x, y, n, bias, relu, s)
                                     : launch_fc_lds<T, 8, 256>(w, x, y, n, bias, relu, s);
            CADNN_HIP(e);
            return CADNN_OK;
        }
        if (nb == 1) {
            const hipError_t e = big ? launch_fc_lds<T, 1, 1024>(w, x, y, n, bias, relu, s)
                                     : launch_fc_lds<T, 1, 256>(w, x, y, n, bias, relu, s);
            CADNN_HIP(e);
            return CADNN_OK;
        }
    }
    const int rows_per_block = 4;
    const unsigned gx = (unsigned)((w->cout + rows_per_block - 1) / rows_per_block);
    const int32_t* rp = (const int32_t*)w->d_row_ptr.p;
    const int32_t* pm = (const int32_t*)w->d_perm.p;
    const int32_t* cl = (const int32_t*)w->d_col.p;
    const float* vl = (const float*)w->d_val.p;
    if (n == 1) {
        CADNN_LAUNCH((sfc_kernel<T, 1>), dim3(gx, 1), dim3(256), 0, s, rp, pm, cl, vl,
                           (const T*)x, (T*)y, bias, n, w->cin, w->cout, relu);
    } else {
        constexpr int NB = 8;
        CADNN_LAUNCH((sfc_kernel<T, NB>), dim3(gx, (unsigned)((n + NB - 1) / NB)), dim3(256),
                           0, s, rp, pm, cl, vl, (const T*)x, (T*)y, bias, n, w->cin, w->cout, relu);
    }
    CADNN_HIP(hipGetLastError());
    return CADNN_OK;
}

cadnn_status launch_fc(const cadnn_weights* w, const void* x, void* y, int n, const float* bias,
                       int relu, hipStream_t s) {
    return w->dtype == CADNN_F16 ? launch_fc_t<_Float16>(w, x, y, n, bias, relu, s)
                                 : launch_fc_t<float>(w, x, y, n, bias, relu, s);
}

// Window pooling, one thread per output: the maximum (AVG = false) or the mean (AVG = true) over
// the in-image part of each k x k window; padding is never looked at, summed or counted.  With
// k = 1, stride 1 and no padding the max form is a layout-to-layout copy, which is how a tensor
// is moved into a channel slice of another.
template <typename T, bool AVG>
__global__ __launch_bounds__(256) void windowpool_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                         TensorDesc xd, TensorDesc yd, int n, int k,
                                                         int stride, int pad) {
    const size_t per_image = (size_t)yd.c * yd.h * yd.w;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= per_image * n) return;
    const int img = (int)(i / per_image);
    windowpool_element<T>(x, y, xd, yd, img, i - (size_t)img * per_image, k, stride, pad, AVG);
}

// 3 x 3 / 2 maximum pool, four neighbouring outputs of a row per thread: their windows span 9
// columns of 3 rows, fetched with three loads per row (4 + 4 + 1 elements, at whatever alignment
// the row has) instead of 9 per output.  Positions outside the image are never looked at: they
// enter the maximum as minus infinity (the loads themselves are range-checked buffer loads, so a
// window hanging over the first row or column reads nothing it should not).
typedef uint32_t u32x2m __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4m __attribute__((ext_vector_type(4)));
template <typename T>
__global__ __launch_bounds__(256) void maxpool3s2_kernel(const T* __restrict__ x, T* __restrict__ y, TensorDesc xd,
                                                         TensorDesc yd, int n, int pad) {
    const int groups = yd.w >> 2;
    const size_t per_image = (size_t)yd.c * yd.h * groups;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= per_image * n) return;
    const int img = (int)(i / per_image);
    const size_t r = i - (size_t)img * per_image;
    const int ow0 = (int)(r % groups) * 4;
    const int oh = (int)((r / groups) % yd.h);
    const int c = (int)(r / ((size_t)groups * yd.h));
    const uint32_t xbytes = (uint32_t)(xd.image * (int64_t)sizeof(T)), ybytes = (uint32_t)(yd.image * (int64_t)sizeof(T));
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc((void*)(x + (size_t)img * xd.image), 0, xbytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc((void*)(y + (size_t)img * yd.image), 0, ybytes, 0x00020000);
    const int iw0 = ow0 * 2 - pad;                    // first of the 9 columns
    // (a row's loads start inside the row: a load that begins in front of the buffer would be
    // dropped whole, valid columns included; the window's columns are the loaded ones shifted)
    const int start = iw0 < 0 ? 0 : iw0, shift = start - iw0;
    const float ninf = -__builtin_inff();
    float m[4] = {ninf, ninf, ninf, ninf};
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        const int ih = oh * 2 + a - pad;
        if (ih < 0 || ih >= xd.h) continue;
        const uint32_t off = (uint32_t)((int64_t)c * xd.plane + xd.origin + (int64_t)ih * xd.pitch + start) * (uint32_t)sizeof(T);
        float v[9];
        if constexpr (sizeof(T) == 2) {
            const u32x2m lo = __builtin_amdgcn_raw_buffer_load_b64(xr, off, 0u, 0);
            const u32x2m hi = __builtin_amdgcn_raw_buffer_load_b64(xr, off + 8u, 0u, 0);
            const uint32_t last = __builtin_amdgcn_raw_buffer_load_b16(xr, off + 16u, 0u, 0);
            const uint32_t w[5] = {lo[0], lo[1], hi[0], hi[1], last};
#pragma unroll
            for (int j = 0; j < 9; ++j) v[j] = (float)__builtin_bit_cast(_Float16, (unsigned short)(w[j >> 1] >> (16 * (j & 1))));
        } else {
            const u32x4m lo = __builtin_amdgcn_raw_buffer_load_b128(xr, off, 0u, 0);
            const u32x4m hi = __builtin_amdgcn_raw_buffer_load_b128(xr, off + 16u, 0u, 0);
            const uint32_t last = __builtin_amdgcn_raw_buffer_load_b32(xr, off + 32u, 0u, 0);
#pragma unroll
            for (int j = 0; j < 4; ++j) { v[j] = __uint_as_float(lo[j]); v[4 + j] = __uint_as_float(hi[j]); }
            v[8] = __uint_as_float(last);
        }
        if (shift) {        // (pad <= 1: by one column)
#pragma unroll
            for (int j = 8; j > 0; --j) v[j] = v[j - 1];
        }
#pragma unroll
        for (int j = 0; j < 9; ++j)
            if (iw0 + j < 0 || iw0 + j >= xd.w) v[j] = ninf;
#pragma unroll
        for (int j = 0; j < 4; ++j) m[j] = fmaxf(m[j], fmaxf(fmaxf(v[2 * j], v[2 * j + 1]), v[2 * j + 2]));
    }
    const uint32_t yoff = (uint32_t)((int64_t)c * yd.plane + yd.origin + (int64_t)oh * yd.pitch + ow0) * (uint32_t)sizeof(T);
    if constexpr (sizeof(T) == 2) {
        uint32_t h[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) h[j] = (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)m[j]);
        __builtin_amdgcn_raw_buffer_store_b64(u32x2m{h[0] | (h[1] << 16), h[2] | (h[3] << 16)}, yr, yoff, 0u, 0);
    } else {
        __builtin_amdgcn_raw_buffer_store_b128(u32x4m{__float_as_uint(m[0]), __float_as_uint(m[1]), __float_as_uint(m[2]), __float_as_uint(m[3])},
                                               yr, yoff, 0u, 0);
    }
}

// One wave per (n, c) plane; lanes stride over the plane, shuffle reduction at the end.
template <typename T>
__global__ __launch_bounds__(256) void avgpool_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                      TensorDesc xd, int n) {
    const int lane = threadIdx.x & 63;
    const int plane = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (plane >= n * xd.c) return;
    const int img = plane / xd.c, c = plane - img * xd.c;
    const T* xp = x + (size_t)img * xd.image + (size_t)c * xd.plane + xd.origin;
    const int hw = xd.h * xd.w;
    float s = 0.0f;
    for (int i = lane; i < hw; i += 64) {
        const int r = i / xd.w, q = i - r * xd.w;
        s += (float)xp[(size_t)r * xd.pitch + q];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) y[plane] = (T)(s / (float)hw);
}

// Plain streaming copy (16 bytes per thread per step); a known-traffic reference used to
// calibrate memory-traffic counters against.
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void zero_kernel(uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = make_uint4(0u, 0u, 0u, 0u);
}

// Zeroes `bytes` bytes (a multiple of 16, 16-byte aligned) with a kernel: usable where a memset
// node must not be recorded.
cadnn_status launch_zero(void* dst, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return CADNN_OK;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 16);
    CADNN_LAUNCH(zero_kernel, dim3(blocks), dim3(256), 0, s, (uint4*)dst, n16);
    CADNN_HIP(hipGetLastError());
    return CADNN_OK;
}

cadnn_status launch_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return CADNN_OK;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 16);
    CADNN_LAUNCH(copy_kernel, dim3(blocks), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n16);
    CADNN_HIP(hipGetLastError());
    return CADNN_OK;
}

template <bool AVG>
static cadnn_status launch_windowpool(const void* x, const TensorDesc& xd, void* y, const TensorDesc& yd, int n,
                                      int k, int stride, int pad, cadnn_dtype dt, hipStream_t s) {
    const size_t total = (size_t)n * yd.c * yd.h * yd.w;
    if ((total + 255) / 256 > 0x7fffffffull) return fail(CADNN_EUNSUPPORTED, "pooling layer too large for one launch");
    // the 3 x 3 / 2 maximum pool of the residual networks on plain tensors whose output rows split
    // into groups of 4: four outputs per thread (an image behind a 32-bit byte offset)
    const int64_t esz = dt == CADNN_F16 ? 2 : 4;
    if (!AVG && k == 3 && stride == 2 && pad <= 1 && !xd.s2d && !yd.s2d && yd.w % 4 == 0 && xd.image * esz < 0x7ffffff0ll &&
        yd.image * esz < 0x7ffffff0ll) {
        const unsigned blocks4 = (unsigned)((total / 4 + 255) / 256);
        if (dt == CADNN_F16)
            CADNN_LAUNCH((maxpool3s2_kernel<_Float16>), dim3(blocks4), dim3(256), 0, s, (const _Float16*)x, (_Float16*)y, xd, yd, n, pad);
        else
            CADNN_LAUNCH((maxpool3s2_kernel<float>), dim3(blocks4), dim3(256), 0, s, (const float*)x, (float*)y, xd, yd, n, pad);
        CADNN_HIP(hipGetLastError());
        return CADNN_OK;
    }
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dt == CADNN_F16)
        CADNN_LAUNCH((windowpool_kernel<_Float16, AVG>), dim3(blocks), dim3(256), 0, s, (const _Float16*)x,
                           (_Float16*)y, xd, yd, n, k, stride, pad);
    else
        CADNN_LAUNCH((windowpool_kernel<float, AVG>), dim3(blocks), dim3(256), 0, s, (const float*)x,
                           (float*)y, xd, yd, n, k, stride, pad);
    CADNN_HIP(hipGetLastError());
    return CADNN_OK;
}

cadnn_status launch_maxpool(const void* x, const TensorDesc& xd, void* y, const TensorDesc& yd, int n,
                            int k, int stride, int pad, cadnn_dtype dt, hipStream_t s) {
    return launch_windowpool<false>(x, xd, y, yd, n, k, stride, pad, dt, s);
}

cadnn_status launch_avgpool2d(const void* x, const TensorDesc& xd, void* y, const TensorDesc& yd, int n,
                              int k, int stride, int pad, cadnn_dtype dt, hipStream_t s) {
    return launch_windowpool<true>(x, xd, y, yd, n, k, stride, pad, dt, s);
}

cadnn_status launch_avgpool(const void* x, const TensorDesc& xd, void* y, int n, cadnn_dtype dt,
                            hipStream_t s) {
    const int nc = n * xd.c;
    const unsigned blocks = (unsigned)((nc + 3) / 4);
    if (dt == CADNN_F16)
        CADNN_LAUNCH(avgpool_kernel<_Float16>, dim3(blocks), dim3(256), 0, s, (const _Float16*)x,
                           (_Float16*)y, xd, n);
    else
        CADNN_LAUNCH(avgpool_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)x,
                           (float*)y, xd, n);
    CADNN_HIP(hipGetLastError());
    return CADNN_OK;
}

}  // namespace cadnn
