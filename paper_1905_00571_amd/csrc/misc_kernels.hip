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

template <typename T>
static cadnn_status launch_fc_t(const cadnn_weights* w, const void* x, void* y, int n,
                                const float* bias, int relu, hipStream_t s) {
    const int rows_per_block = 4;
    const unsigned gx = (unsigned)((w->cout + rows_per_block - 1) / rows_per_block);
    const int32_t* rp = (const int32_t*)w->d_row_ptr.p;
    const int32_t* pm = (const int32_t*)w->d_perm.p;
    const int32_t* cl = (const int32_t*)w->d_col.p;
    const float* vl = (const float*)w->d_val.p;
    if (n == 1) {
        hipLaunchKernelGGL((sfc_kernel<T, 1>), dim3(gx, 1), dim3(256), 0, s, rp, pm, cl, vl,
                           (const T*)x, (T*)y, bias, n, w->cin, w->cout, relu);
    } else {
        constexpr int NB = 8;
        hipLaunchKernelGGL((sfc_kernel<T, NB>), dim3(gx, (unsigned)((n + NB - 1) / NB)), dim3(256),
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

template <typename T>
__global__ __launch_bounds__(256) void maxpool_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                      TensorDesc xd, TensorDesc yd, int n, int k,
                                                      int stride, int pad) {
    const size_t per_image = (size_t)yd.c * yd.h * yd.w;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= per_image * n) return;
    const int img = (int)(i / per_image);
    const size_t r = i - (size_t)img * per_image;
    const int ow = (int)(r % yd.w);
    const int oh = (int)((r / yd.w) % yd.h);
    const int c = (int)(r / ((size_t)yd.w * yd.h));
    const T* xp = x + (size_t)img * xd.image + (size_t)c * xd.plane + xd.origin;
    bool seen = false;
    float m = 0.0f;
    for (int a = 0; a < k; ++a) {
        const int ih = oh * stride + a - pad;
        if (ih < 0 || ih >= xd.h) continue;
        for (int q = 0; q < k; ++q) {
            const int iw = ow * stride + q - pad;
            if (iw < 0 || iw >= xd.w) continue;
            const float v = (float)xp[(size_t)ih * xd.pitch + iw];
            if (!seen || v > m) m = v;
            seen = true;
        }
    }
    y[(size_t)img * yd.image + (size_t)c * yd.plane + yd.origin + (size_t)oh * yd.pitch + ow] = (T)m;
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

cadnn_status launch_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return CADNN_OK;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n16);
    CADNN_HIP(hipGetLastError());
    return CADNN_OK;
}

cadnn_status launch_maxpool(const void* x, const TensorDesc& xd, void* y, const TensorDesc& yd, int n,
                            int k, int stride, int pad, cadnn_dtype dt, hipStream_t s) {
    const size_t total = (size_t)n * yd.c * yd.h * yd.w;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dt == CADNN_F16)
        hipLaunchKernelGGL(maxpool_kernel<_Float16>, dim3(blocks), dim3(256), 0, s, (const _Float16*)x,
                           (_Float16*)y, xd, yd, n, k, stride, pad);
    else
        hipLaunchKernelGGL(maxpool_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)x,
                           (float*)y, xd, yd, n, k, stride, pad);
    CADNN_HIP(hipGetLastError());
    return CADNN_OK;
}

cadnn_status launch_avgpool(const void* x, const TensorDesc& xd, void* y, int n, cadnn_dtype dt,
                            hipStream_t s) {
    const int nc = n * xd.c;
    const unsigned blocks = (unsigned)((nc + 3) / 4);
    if (dt == CADNN_F16)
        hipLaunchKernelGGL(avgpool_kernel<_Float16>, dim3(blocks), dim3(256), 0, s, (const _Float16*)x,
                           (_Float16*)y, xd, n);
    else
        hipLaunchKernelGGL(avgpool_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)x,
                           (float*)y, xd, n);
    CADNN_HIP(hipGetLastError());
    return CADNN_OK;
}

}  // namespace cadnn
