// C-ABI entry points for single layers: argument checks, variant selection, launch.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <algorithm>

#include "internal.h"

using namespace cadnn;

namespace cadnn {

struct ConvGeom {
    int n, h, w, stride, pad, hout, wout;
    std::array<int, 5> key() const { return {n, h, w, stride, pad}; }
};

static cadnn_status check_conv(const char* who, const cadnn_weights* w, int n, int h, int wdt,
                               int stride, int pad, ConvGeom* g) {
    if (!w) return fail(CADNN_EINVAL, "%s: NULL weight handle", who);
    if (n <= 0 || h <= 0 || wdt <= 0) return fail(CADNN_EINVAL, "%s: non-positive size", who);
    if (stride <= 0 || pad < 0) return fail(CADNN_EINVAL, "%s: bad stride/pad", who);
    *g = ConvGeom{n, h, wdt, stride, pad, conv_out(h, w->kh, stride, pad), conv_out(wdt, w->kw, stride, pad)};
    if (g->hout <= 0 || g->wout <= 0) return fail(CADNN_EINVAL, "%s: empty output", who);
    if (n > 65535) return fail(CADNN_EUNSUPPORTED, "%s: batch above 65535", who);
    if ((int64_t)n * w->cin * h * wdt > (int64_t)INT32_MAX * 64 ||
        (int64_t)n * w->cout * g->hout * g->wout > (int64_t)INT32_MAX * 64)
        return fail(CADNN_EUNSUPPORTED, "%s: tensor too large", who);
    return CADNN_OK;
}

static bool variant_fits(const ConvVariant& v, const cadnn_weights* w, const ConvGeom& g) {
    if (v.kh != w->kh || v.kw != w->kw) return false;
    if (v.is_f16 != (w->dtype == CADNN_F16)) return false;
    if (v.stride != 0 && v.stride != g.stride) return false;
    const int64_t esz = w->dtype == CADNN_F16 ? 2 : 4;
    if (v.family == FAM_DIRECT) {
        if ((int64_t)w->cin * g.h * g.w * esz >= 0x7ffffff0ll) return false;
        if ((w->cout + v.rows_per_block() - 1) / v.rows_per_block() > 65535) return false;
    } else {
        if ((w->cout + v.rows_per_block() - 1) / v.rows_per_block() > 65535) return false;
    }
    return true;
}

static std::vector<const ConvVariant*> candidates(const cadnn_weights* w, const ConvGeom& g) {
    std::vector<const ConvVariant*> out;
    for (const ConvVariant& v : all_direct_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    for (const ConvVariant& v : all_tile_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    return out;
}

// Default choice when nothing was tuned or pinned: a rough occupancy/latency model.
// A wave of a staging-free variant runs rpw * nnz_row / ks groups of loads one after the
// other; the chip wants at least a couple of waves on each of its 1024 SIMDs.
static const ConvVariant* heuristic_variant(const cadnn_weights* w, const ConvGeom& g) {
    const std::vector<const ConvVariant*> cand = candidates(w, g);
    if (cand.empty()) return nullptr;
    const double nnz_row = w->cout ? (double)w->nnz / w->cout : 0.0;
    const double pixels = (double)g.hout * g.wout;
    const ConvVariant* best = nullptr;
    double best_cost = 0.0;
    for (const ConvVariant* v : cand) {
        double cost;
        if (v->family == FAM_DIRECT) {
            const double tiles = std::ceil(pixels / (64.0 * v->p)) * g.n;
            const double blocks = tiles * std::ceil((double)w->cout / v->rows_per_block());
            const double waves = blocks * v->nw;
            const double iters = v->rpw * nnz_row / v->ks;            // loop trips per wave
            const double lane_eff = pixels * g.n / (tiles * 64.0 * v->p);
            // latency-bound part: one wave alone; throughput part: address units of a CU
            const double t_wave = 900.0 + iters / 4.0 * (160.0 + 40.0 * v->p) + (v->ks > 1 ? 300.0 : 0.0);
            const double rounds = std::ceil(waves / (1024.0 * 6.0));
            const double t_cu = waves * iters * v->p * 4.2 / 256.0;
            cost = std::max(t_wave * rounds, t_cu) / std::max(lane_eff, 0.05) * (lane_eff < 1 ? 1.0 : 1.0);
        } else {
            const double tiles = std::ceil((double)g.wout / v->tw) * std::ceil((double)g.hout / v->th) * g.n;
            const double blocks = tiles * std::ceil((double)w->cout / v->rows_per_block());
            const double nchunks = std::ceil((double)w->cin / v->cch);
            const double stage = nchunks * (1500.0 + (double)std::min(w->cin, v->cch) * v->plane / (v->nw * 64.0) * 24.0);
            const double iters = v->rpw * nnz_row;
            const double t_block = stage + iters * (10.0 + 6.0 * v->p) / 1.0;
            const double rounds = std::ceil(blocks / 256.0);
            cost = t_block * rounds * 3.0;   // until tuned, prefer the staging-free family
        }
        if (!best || cost < best_cost) { best = v; best_cost = cost; }
    }
    return best;
}

static const ConvVariant* pick_variant(const cadnn_weights* w, const ConvGeom& g) {
    {
        std::lock_guard<std::mutex> lock(w->mu);
        auto it = w->chosen.find(g.key());
        if (it != w->chosen.end()) return it->second;
    }
    return heuristic_variant(w, g);
}

static cadnn_status launch_variant(const cadnn_weights* w, const ConvVariant* v, const ConvGeom& g,
                                   const void* x, void* y, const void* bias, const void* residual,
                                   int relu, hipStream_t s) {
    const ConvPlan* plan = nullptr;
    cadnn_status st = get_conv_plan(w, v, &plan);
    if (st != CADNN_OK) return st;
    const uint32_t esz = w->dtype == CADNN_F16 ? 2 : 4;
    ConvLaunch a{};
    a.x = x;
    a.y = y;
    a.bias = (const float*)bias;
    a.residual = residual;
    a.nz = (const uint2*)plan->nz.p;
    a.seg_ptr = (const int32_t*)plan->seg_ptr.p;
    a.perm = (const int32_t*)plan->perm.p;
    a.n = g.n; a.cin = w->cin; a.h = g.h; a.w = g.w; a.cout = w->cout;
    a.hout = g.hout; a.wout = g.wout; a.stride = g.stride; a.pad = g.pad; a.relu = relu ? 1 : 0;
    a.nchunks = plan->nchunks;
    a.hwout = g.hout * g.wout;
    a.chan_stride_bytes = (uint32_t)g.h * (uint32_t)g.w * esz;
    a.image_bytes = (uint32_t)((int64_t)w->cin * g.h * g.w * esz > 0x7fffffffll ? 0 : (int64_t)w->cin * g.h * g.w * esz);
    if (v->family == FAM_DIRECT) {
        a.tiles_x = (a.hwout + 64 * v->p - 1) / (64 * v->p);
        a.tiles_y = 1;
        if (a.tiles_x > 0x7fffffff / 64) return fail(CADNN_EUNSUPPORTED, "cadnn_sparse_conv2d: image too large");
    } else {
        a.tiles_x = (g.wout + v->tw - 1) / v->tw;
        a.tiles_y = (g.hout + v->th - 1) / v->th;
    }
    a.row_groups = plan->rows_padded / v->rows_per_block();
    if (a.row_groups > 65535) return fail(CADNN_EUNSUPPORTED, "cadnn_sparse_conv2d: too many rows");
    CADNN_HIP(v->launch(a, s));
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
    const ConvVariant* v = pick_variant(w, g);
    if (!v)
        return fail(CADNN_EUNSUPPORTED, "cadnn_sparse_conv2d: no kernel for %dx%d filters with stride %d",
                    w->kh, w->kw, stride);
    return launch_variant(w, v, g, x, y, bias, residual, relu, s);
}

cadnn_status conv2d_tune_impl(const cadnn_weights* w, const void* x, void* y, int n, int h, int wdt,
                              int stride, int pad, const void* bias, const void* residual, int relu,
                              hipStream_t s, int reps, float* best_us) {
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_tune", w, n, h, wdt, stride, pad, &g);
    if (st != CADNN_OK) return st;
    if (!x || !y) return fail(CADNN_EINVAL, "cadnn_conv2d_tune: NULL tensor");
    if (reps <= 0) return fail(CADNN_EINVAL, "cadnn_conv2d_tune: reps must be positive");
    const std::vector<const ConvVariant*> cand = candidates(w, g);
    if (cand.empty())
        return fail(CADNN_EUNSUPPORTED, "cadnn_conv2d_tune: no kernel for %dx%d filters with stride %d",
                    w->kh, w->kw, stride);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    CADNN_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(CADNN_EHIP, "hipEventCreate failed"); }
    const ConvVariant* best = nullptr;
    float best_ms = 0.0f;
    for (const ConvVariant* v : cand) {
        for (int i = 0; i < 2 && st == CADNN_OK; ++i) st = launch_variant(w, v, g, x, y, bias, residual, relu, s);
        if (st != CADNN_OK) break;
        if (hipEventRecord(e0, s) != hipSuccess) { st = fail(CADNN_EHIP, "hipEventRecord failed"); break; }
        for (int i = 0; i < reps && st == CADNN_OK; ++i) st = launch_variant(w, v, g, x, y, bias, residual, relu, s);
        if (st != CADNN_OK) break;
        if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) { st = fail(CADNN_EHIP, "event wait failed"); break; }
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { st = fail(CADNN_EHIP, "hipEventElapsedTime failed"); break; }
        if (std::getenv("CADNN_TUNE_LOG"))
            std::fprintf(stderr, "[cadnn tune] cin=%d cout=%d k=%d s=%d hw=%dx%d nnz=%lld %-44s %8.2f us\n", w->cin,
                         w->cout, w->kh, stride, h, wdt, (long long)w->nnz, v->name, ms * 1e3f / reps);
        if (!best || ms < best_ms) { best = v; best_ms = ms; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != CADNN_OK) return st;
    {
        std::lock_guard<std::mutex> lock(w->mu);
        w->chosen[g.key()] = best;
    }
    drop_plans_except(w, best);
    if (best_us) *best_us = best_ms * 1e3f / reps;
    return CADNN_OK;
}

}  // namespace cadnn

extern "C" cadnn_status cadnn_sparse_conv2d(const cadnn_weights* w, const void* x, void* y, int n,
                                            int h, int wdt, int stride, int pad, const void* bias,
                                            const void* residual, int relu, void* stream) {
    return conv2d_impl(w, x, y, n, h, wdt, stride, pad, bias, residual, relu, (hipStream_t)stream);
}

extern "C" cadnn_status cadnn_conv2d_tune(const cadnn_weights* w, const void* x, void* y, int n, int h,
                                          int wdt, int stride, int pad, const void* bias,
                                          const void* residual, int relu, void* stream, int reps,
                                          float* best_us) {
    return conv2d_tune_impl(w, x, y, n, h, wdt, stride, pad, bias, residual, relu, (hipStream_t)stream,
                            reps, best_us);
}

extern "C" cadnn_status cadnn_conv2d_prepare(const cadnn_weights* w, int n, int h, int wdt,
                                             int stride, int pad) {
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_prepare", w, n, h, wdt, stride, pad, &g);
    if (st != CADNN_OK) return st;
    const ConvVariant* v = pick_variant(w, g);
    if (!v)
        return fail(CADNN_EUNSUPPORTED, "cadnn_conv2d_prepare: no kernel for %dx%d filters with stride %d",
                    w->kh, w->kw, stride);
    const ConvPlan* plan = nullptr;
    return get_conv_plan(w, v, &plan);
}

extern "C" cadnn_status cadnn_conv2d_variant_name(const cadnn_weights* w, int n, int h, int wdt,
                                                  int stride, int pad, char* buf, size_t len) {
    if (!buf || len == 0) return fail(CADNN_EINVAL, "cadnn_conv2d_variant_name: NULL buffer");
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_variant_name", w, n, h, wdt, stride, pad, &g);
    if (st != CADNN_OK) return st;
    const ConvVariant* v = pick_variant(w, g);
    if (!v)
        return fail(CADNN_EUNSUPPORTED, "cadnn_conv2d_variant_name: no kernel for %dx%d filters with stride %d",
                    w->kh, w->kw, stride);
    std::strncpy(buf, v->name, len - 1);
    buf[len - 1] = '\0';
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_conv2d_list_variants(const cadnn_weights* w, int n, int h, int wdt,
                                                   int stride, int pad, char* buf, size_t len) {
    if (!buf || len == 0) return fail(CADNN_EINVAL, "cadnn_conv2d_list_variants: NULL buffer");
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_list_variants", w, n, h, wdt, stride, pad, &g);
    if (st != CADNN_OK) return st;
    std::string all;
    for (const ConvVariant* v : candidates(w, g)) {
        if (!all.empty()) all += "\n";
        all += v->name;
    }
    if (all.size() + 1 > len) return fail(CADNN_EINVAL, "cadnn_conv2d_list_variants: buffer of %zu bytes, %zu needed", len, all.size() + 1);
    std::memcpy(buf, all.c_str(), all.size() + 1);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_conv2d_set_variant(const cadnn_weights* w, int n, int h, int wdt,
                                                 int stride, int pad, const char* name) {
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_set_variant", w, n, h, wdt, stride, pad, &g);
    if (st != CADNN_OK) return st;
    std::lock_guard<std::mutex> lock(w->mu);
    if (!name || !*name) {
        w->chosen.erase(g.key());
        return CADNN_OK;
    }
    for (const ConvVariant* v : candidates(w, g)) {
        if (std::strcmp(v->name, name) == 0) {
            w->chosen[g.key()] = v;
            return CADNN_OK;
        }
    }
    return fail(CADNN_EINVAL, "cadnn_conv2d_set_variant: '%s' does not serve this layer", name);
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
