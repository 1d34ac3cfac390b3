// Dense comparator / fallback convolution (implicit GEMM).
#include "internal.h"

namespace cadnn {

cadnn_status dense_conv2d_impl(const void*, const void*, void*, int, int, int, int, int, int, int,
                               int, int, const void*, const void*, int, cadnn_dtype, hipStream_t) {
    return fail(CADNN_EUNSUPPORTED, "cadnn_dense_conv2d: not built yet");
}

}  // namespace cadnn

extern "C" cadnn_status cadnn_dense_conv2d(const void* w_dev, const void* x, void* y, int n, int cin,
                                           int h, int wdt, int cout, int kh, int kw, int stride,
                                           int pad, const void* bias, const void* residual, int relu,
                                           cadnn_dtype dtype, void* stream) {
    return cadnn::dense_conv2d_impl(w_dev, x, y, n, cin, h, wdt, cout, kh, kw, stride, pad, bias,
                                    residual, relu, dtype, (hipStream_t)stream);
}
