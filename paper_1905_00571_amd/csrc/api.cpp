// C-ABI entry points for single layers: argument checks, variant selection, launch.
#include <cstring>

#include "internal.h"

using namespace cadnn;

namespace cadnn {

struct ConvGeom {
    int hout, wout;
    const TileVariant* variant;
};

static cadnn_status check_conv(const char* who, const cadnn_weights* w, int n, int h, int wdt,
                               int stride, int pad, ConvGeom* g) {
    if (!w) return fail(CADNN_EINVAL, "%s: NULL weight handle", who);
    if (n <= 0 || h <= 0 || wdt <= 0) return fail(CADNN_EINVAL, "%s: non-positive size", who);
    if (stride <= 0 || pad < 0) return fail(CADNN_EINVAL, "%s: bad stride/pad", who);
    g->hout = conv_out(h, w->kh, stride, pad);
    g->wout = conv_out(wdt, w->kw, stride, pad);
    if (g->hout <= 0 || g->wout <= 0) return fail(CADNN_EINVAL, "%s: empty output", who);
    if (n > 65535) return fail(CADNN_EUNSUPPORTED, "%s: batch above 65535", who);
    if ((int64_t)n * w->cin * h * wdt > (int64_t)INT32_MAX * 64 ||
        (int64_t)n * w->cout * g->hout * g->wout > (int64_t)INT32_MAX * 64)
        return fail(CADNN_EUNSUPPORTED, "%s: tensor too large", who);
    g->variant = select_tile_variant(w->kh, w->kw, stride, g->hout, g->wout, w->cout, w->dtype);
    if (!g->variant)
        return fail(CADNN_EUNSUPPORTED, "%s: no kernel for %dx%d filters with stride %d", who, w->kh,
                    w->kw, stride);
    return CADNN_OK;
}

cadnn_status conv2d_impl(const cadnn_weights* w, const void* x, void* y, int n, int h, int wdt,
                         int stride, int pad, const void* bias, const void* residual, int relu,
                         hipStream_t s) {
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_sparse_conv2d", w, n, h, wdt, stride, pad, &g);
    if (st != CADNN_OK) return st;
    if (!x || !y) return fail(CADNN_EINVAL, "cadnn_sparse_conv2d: NULL tensor");
    if (x == y) return fail(CADNN_EINVAL, "cadnn_sparse_conv2d: y aliases x");
    const ConvPlan* plan = nullptr;
    if ((st = get_conv_plan(w, g.variant, &plan)) != CADNN_OK) return st;
    const TileVariant* v = g.variant;
    ConvLaunch a{};
    a.x = x;
    a.y = y;
    a.bias = (const float*)bias;
    a.residual = residual;
    a.nz = (const uint2*)plan->nz.p;
    a.seg_ptr = (const int32_t*)plan->seg_ptr.p;
    a.perm = (const int32_t*)plan->perm.p;
    a.n = n; a.cin = w->cin; a.h = h; a.w = wdt; a.cout = w->cout;
    a.hout = g.hout; a.wout = g.wout; a.pad = pad; a.relu = relu ? 1 : 0;
    a.nchunks = plan->nchunks;
    a.tiles_x = (g.wout + v->tw - 1) / v->tw;
    a.tiles_y = (g.hout + v->th - 1) / v->th;
    a.row_groups = plan->rows_padded / (v->nw * v->rpw);
    if (a.row_groups > 65535) return fail(CADNN_EUNSUPPORTED, "cadnn_sparse_conv2d: too many rows");
    CADNN_HIP(v->launch(a, s));
    return CADNN_OK;
}

}  // namespace cadnn

extern "C" cadnn_status cadnn_sparse_conv2d(const cadnn_weights* w, const void* x, void* y, int n,
                                            int h, int wdt, int stride, int pad, const void* bias,
                                            const void* residual, int relu, void* stream) {
    return conv2d_impl(w, x, y, n, h, wdt, stride, pad, bias, residual, relu, (hipStream_t)stream);
}

extern "C" cadnn_status cadnn_conv2d_prepare(const cadnn_weights* w, int n, int h, int wdt,
                                             int stride, int pad) {
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_prepare", w, n, h, wdt, stride, pad, &g);
    if (st != CADNN_OK) return st;
    const ConvPlan* plan = nullptr;
    return get_conv_plan(w, g.variant, &plan);
}

extern "C" cadnn_status cadnn_conv2d_variant_name(const cadnn_weights* w, int n, int h, int wdt,
                                                  int stride, int pad, char* buf, size_t len) {
    if (!buf || len == 0) return fail(CADNN_EINVAL, "cadnn_conv2d_variant_name: NULL buffer");
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_variant_name", w, n, h, wdt, stride, pad, &g);
    if (st != CADNN_OK) return st;
    std::strncpy(buf, g.variant->name, len - 1);
    buf[len - 1] = '\0';
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_sparse_fc(const cadnn_weights* w, const void* x, void* y, int n,
                                        const void* bias, int relu, void* stream) {
    if (!w || !x || !y) return fail(CADNN_EINVAL, "cadnn_sparse_fc: NULL pointer");
    if (n <= 0) return fail(CADNN_EINVAL, "cadnn_sparse_fc: non-positive batch");
    if (w->kh != 1 || w->kw != 1)
        return fail(CADNN_EINVAL, "cadnn_sparse_fc: weights are a %dx%d filter bank", w->kh, w->kw);
    if (n > 8 * 65535) return fail(CADNN_EUNSUPPORTED, "cadnn_sparse_fc: batch too large");
    cadnn_status st = ensure_fc_device(w);
    if (st != CADNN_OK) return st;
    return launch_fc(w, x, y, n, (const float*)bias, relu ? 1 : 0, (hipStream_t)stream);
}

extern "C" cadnn_status cadnn_fc_prepare(const cadnn_weights* w) {
    if (!w) return fail(CADNN_EINVAL, "cadnn_fc_prepare: NULL handle");
    if (w->kh != 1 || w->kw != 1) return fail(CADNN_EINVAL, "cadnn_fc_prepare: weights are not a matrix");
    return ensure_fc_device(w);
}

extern "C" cadnn_status cadnn_maxpool2d(const void* x, void* y, int n, int c, int h, int wdt, int k,
                                        int stride, int pad, cadnn_dtype dtype, void* stream) {
    if (!x || !y) return fail(CADNN_EINVAL, "cadnn_maxpool2d: NULL tensor");
    if (n <= 0 || c <= 0 || h <= 0 || wdt <= 0 || k <= 0 || stride <= 0 || pad < 0)
        return fail(CADNN_EINVAL, "cadnn_maxpool2d: bad size");
    if (dtype != CADNN_F32 && dtype != CADNN_F16) return fail(CADNN_EINVAL, "cadnn_maxpool2d: dtype");
    if (conv_out(h, k, stride, pad) <= 0 || conv_out(wdt, k, stride, pad) <= 0)
        return fail(CADNN_EINVAL, "cadnn_maxpool2d: empty output");
    return launch_maxpool(x, y, n, c, h, wdt, k, stride, pad, dtype, (hipStream_t)stream);
}

extern "C" cadnn_status cadnn_global_avgpool(const void* x, void* y, int n, int c, int h, int wdt,
                                             cadnn_dtype dtype, void* stream) {
    if (!x || !y) return fail(CADNN_EINVAL, "cadnn_global_avgpool: NULL tensor");
    if (n <= 0 || c <= 0 || h <= 0 || wdt <= 0) return fail(CADNN_EINVAL, "cadnn_global_avgpool: bad size");
    if (dtype != CADNN_F32 && dtype != CADNN_F16) return fail(CADNN_EINVAL, "cadnn_global_avgpool: dtype");
    return launch_avgpool(x, y, n, c, h, wdt, dtype, (hipStream_t)stream);
}
