// C-ABI entry points for single layers: argument checks, variant selection, launch.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <algorithm>

#include "internal.h"

using namespace cadnn;

namespace cadnn {

struct ConvGeom {
    int n, stride, pad, hout, wout;
    TensorDesc xd;
    int out_s2d = 0;          // output or residual de-interleaved
    const ConvExtra* ex = nullptr;   // fused 1x1 shortcut
    GeomKey key() const {
        return {n, xd.h, xd.w, stride, pad, xd.ph, xd.pw,
                (xd.s2d ? 1 : 0) | (out_s2d ? 2 : 0) | ((ex && ex->w) ? 4 : 0) | ((ex && ex->pool_y) ? 8 : 0) |
                    ((ex && ex->dw) ? (ex->dw_stride == 2 ? 48 : 16) : 0)};
    }
};

static cadnn_status check_conv(const char* who, const cadnn_weights* w, const TensorDesc& xd, int n,
                               int stride, int pad, ConvGeom* g, int out_s2d = 0, const ConvExtra* ex = nullptr) {
    if (!w) return fail(CADNN_EINVAL, "%s: NULL weight handle", who);
    if (n <= 0 || xd.h <= 0 || xd.w <= 0) return fail(CADNN_EINVAL, "%s: non-positive size", who);
    if (stride <= 0 || pad < 0) return fail(CADNN_EINVAL, "%s: bad stride/pad", who);
    if (xd.c != w->cin) return fail(CADNN_EINVAL, "%s: %d input channels, weights take %d", who, xd.c, w->cin);
    if (desc_too_large(xd)) return fail(CADNN_EUNSUPPORTED, "%s: a channel plane of 2^30 elements or more", who);
    g->n = n; g->stride = stride; g->pad = pad; g->xd = xd; g->out_s2d = out_s2d; g->ex = ex;
    if (ex && !ex->w && !ex->pool_y && !ex->dw) return fail(CADNN_EINVAL, "%s: empty fusion request", who);
    if (ex && ex->dw) {
        const cadnn_weights* d = ex->dw;
        if (ex->w || ex->pool_y) return fail(CADNN_EINVAL, "%s: one fusion at a time", who);
        if (d->cin != 1 || d->cout != w->cout || d->kh != 3 || d->kw != 3 || d->dtype != w->dtype ||
            (ex->dw_stride != 1 && ex->dw_stride != 2))
            return fail(CADNN_EINVAL, "%s: the fused depthwise layer must be 3x3, stride 1 or 2, one filter per output channel", who);
    }
    if (ex && ex->w) {
        if (!ex->x) return fail(CADNN_EINVAL, "%s: NULL fused shortcut", who);
        if (ex->w->kh != 1 || ex->w->kw != 1 || ex->w->cout != w->cout || ex->w->dtype != w->dtype ||
            ex->w->cin != ex->xd.c || ex->stride <= 0)
            return fail(CADNN_EINVAL, "%s: the fused shortcut must be a 1x1 layer of the same type and output channels", who);
        if (ex->xd.image * (int64_t)w->elem() >= 0x7ffffff0ll)
            return fail(CADNN_EUNSUPPORTED, "%s: one image of the shortcut's input is 2 GiB or more", who);
    }
    g->hout = conv_out(xd.h, w->kh, stride, pad);
    g->wout = conv_out(xd.w, w->kw, stride, pad);
    if (g->hout <= 0 || g->wout <= 0) return fail(CADNN_EINVAL, "%s: empty output", who);
    if (n > 65535) return fail(CADNN_EUNSUPPORTED, "%s: batch above 65535", who);
    if (xd.image * (int64_t)w->elem() >= 0x7ffffff0ll ||
        (double)w->cout * ((double)g->hout + 64.0) * ((double)g->wout + 64.0) * (double)w->elem() >= (double)0x7ffffff0ll)
        return fail(CADNN_EUNSUPPORTED, "%s: one image of the tensor is 2 GiB or more", who);
    return CADNN_OK;
}

// K split over workgroups (large-tile matrix-core variants with splitk > 1): the number of
// slices in use -- every slice gets at least one 32-deep step -- the output tiles, and the
// scratch the slices meet in: per (variant, layer geometry), allocated on first use and kept.
struct SplitK { int sk = 1; int64_t tiles = 0; };
static SplitK splitk_of(const ConvVariant& v, const cadnn_weights* w, const ConvGeom& g) {
    SplitK r;
    const int tm = v.rows_per_block(), tn = 64 * v.p;
    r.tiles = (((int64_t)g.n * g.hout * g.wout + tn - 1) / tn) * ((w->cout + tm - 1) / tm);
    const int steps = w->cin / 32 * w->kh * w->kw + ((g.ex && g.ex->w) ? g.ex->w->cin / 32 : 0);
    if (v.splitk > 1 && steps > 0) {
        const int per = (steps + v.splitk - 1) / v.splitk;
        r.sk = (steps + per - 1) / per;
    }
    return r;
}
static cadnn_status ensure_sk_scratch(const cadnn_weights* w, const ConvVariant* v, const ConvGeom& g, ConvLaunch* out) {
    const SplitK k = splitk_of(*v, w, g);
    if (k.sk <= 1) return CADNN_OK;
    float* part = nullptr;
    int* count = nullptr;
    const size_t tile_bytes = (size_t)v->rows_per_block() * 64 * v->p * sizeof(float);
    cadnn_status st = get_sk_scratch(w, v, g.key(), (size_t)k.tiles * k.sk * tile_bytes, (size_t)k.tiles * sizeof(int), &part, &count);
    if (st != CADNN_OK) return st;
    if (out) {
        out->sk = k.sk;
        out->sk_part = part;
        out->sk_count = count;
    }
    return CADNN_OK;
}

static bool variant_fits(const ConvVariant& v, const cadnn_weights* w, const ConvGeom& g, bool any_density = false) {
    if (v.is_f16 != (w->dtype == CADNN_F16)) return false;
    if (v.stride != 0 && v.stride != g.stride) return false;
    if ((w->cout + v.rows_per_block() - 1) / v.rows_per_block() > 65535) return false;
    // de-interleaved tensors and fused shortcuts are understood by the linear-address kernels
    // and by the large-tile matrix-core kernel (which fuses a projection shortcut as more of
    // K); the wide-tile family computes every address through the general layout function, so
    // it reads and writes de-interleaved tensors as well, and fuses nothing
    const bool wide_dense = v.family == FAM_DENSE && v.tw == 128;
    if (g.ex && v.family != FAM_LINEAR && !(wide_dense && g.ex->w && !g.ex->pool_y && !g.ex->dw)) return false;
    if ((g.xd.s2d || g.out_s2d) && v.family != FAM_LINEAR && v.family != FAM_WTILE && !wide_dense) return false;
    if (v.family == FAM_DENSE) {
        const bool dense_enough = (double)w->nnz >= 0.25 * (double)w->cout * w->cin * w->kh * w->kw;
        const int64_t pixels = (int64_t)g.n * g.hout * g.wout;
        // in 2-byte storage a candidate for the measured selection at any density, once the batch
        // of pixels gives the matrix cores a few tiles
        const bool by_tuning = v.is_f16 && pixels >= 96;
        if (!wide_dense) return any_density || dense_enough || by_tuning;
        int64_t in_bytes = g.xd.image * 2 * g.n;
        if (g.ex) {
            // (a de-interleaved shortcut input is handed over as the plain view of one phase)
            if (g.ex->w->cin % 32 != 0 || (g.ex->xd.s2d && g.ex->stride != 2)) return false;
            in_bytes = std::max<int64_t>(in_bytes, g.ex->xd.image * 2 * g.n);
        }
        if (!dense_wide_serves(v.is_f16, w->cin, w->kh * w->kw, in_bytes,
                               (int64_t)w->cout * (g.hout + 64) * (g.wout + 64) * 2 * g.n, pixels))
            return false;
        // few input channels: K is walked with a table of offsets by the 64-pixel tiles, on plain
        // tensors, with nothing fused and K in one piece
        if (w->cin % 32 != 0 && (v.p != 1 || g.ex || g.xd.s2d || v.splitk > 1)) return false;
        // a de-interleaved input is walked phase by phase (stride 2, taps starting inside the
        // halo) or pixel by pixel (stride 1, 1x1)
        if (g.xd.s2d && !(g.stride == 2 ? (g.xd.ph >= g.pad && g.xd.pw >= g.pad) : (g.stride == 1 && w->kh * w->kw == 1 && g.pad == 0)))
            return false;
        if (v.splitk > 1) {
            // K is split over workgroups where the tiles alone leave most of the chip idle and
            // every slice still gets a few stages; the scratch stays below 256 MiB
            const SplitK k = splitk_of(v, w, g);
            const int steps = w->cin / 32 * w->kh * w->kw + (g.ex ? g.ex->w->cin / 32 : 0);
            if (k.sk != v.splitk || k.tiles > 384 || steps < 8 * v.splitk ||
                k.tiles * k.sk * (int64_t)v.rows_per_block() * 64 * v.p * 4 > (256ll << 20))
                return false;
        }
        return any_density || dense_enough || by_tuning;
    }
    if (v.family == FAM_LINEAR) {
        const bool one = w->kh == 1 && w->kw == 1;
        if (g.xd.s2d) {
            // a stride-2 layer walks one phase per tap with unit stride (for filters larger
            // than 1x1 the taps must start on an even padded position); a stride-1 layer can
            // only be pixel-wise
            if (g.stride == 2) {
                if (!one && (((g.xd.ph - g.pad) & 1) || ((g.xd.pw - g.pad) & 1))) return false;
            } else if (g.stride != 1 || !one) {
                return false;
            }
        }
        // Writing a de-interleaved tensor, or reading one pixel by pixel, takes the
        // instantiations with the general address arithmetic; a stride-2 layer on a
        // de-interleaved input is handed a plain view of the phase it starts in.
        const bool general = g.out_s2d || (g.xd.s2d && g.stride == 1);
        if (general != (v.s2d != 0)) return false;
        // several rows per wave: the whole image in a row's share of the lanes, nothing fused
        if (v.quad && (g.ex || g.hout * ((g.wout + v.p - 1) / v.p) > 64 / v.rpw)) return false;
        // a fused shortcut takes the dual-input instantiations; its input must be walkable
        // with one stride (plain layout, or de-interleaved and read with stride 2)
        const bool shortcut = g.ex && g.ex->w, pooled = g.ex && g.ex->pool_y, dwf = g.ex && g.ex->dw;
        if (shortcut != (v.dual != 0) || pooled != (v.pool != 0) || dwf != (v.dw != 0)) return false;
        // a fused depthwise layer needs the whole image, at most 16 x 16, in one pixel tile
        // (one wavefront's pixels, or -- tile-per-wave instantiations -- those of all the waves of a workgroup)
        if (dwf && (general || g.hout * g.wout > 64 * v.p * (v.dw == 2 ? v.tw : 1) || g.hout > 28 || g.wout > 28)) return false;
        // a fused pool needs the whole image in one pixel tile of the variant
        if (pooled && (general || shortcut || g.hout * g.wout > 64 * v.p)) return false;
        if (shortcut) {
            if (general) return false;
            if (g.ex->xd.s2d && g.ex->stride != 2) return false;
            const int unit2 = g.ex->xd.s2d ? 2 : 1;
            if (v.adjacent && g.ex->stride != unit2) return false;
        }
        // a lane's adjacent pixels must be adjacent in memory, on both sides; rows that split
        // evenly into groups take the plain instantiations, the others the ragged-row ones
        const int unit = g.xd.s2d ? 2 : 1;
        if (v.adjacent && (g.stride != unit || (!v.quad && (g.wout % v.p != 0) != (v.adjacent == 2)))) return false;
        // The last group of a ragged row reads up to P-1 elements past its row.  Past the end
        // of the image that reads as zero dword by dword, which is fine for 4-byte storage; in
        // 2-byte storage the dword holding the image's last element would be dropped whole,
        // so there the input must end in a halo row instead.
        if (v.adjacent == 2 && v.is_f16 && g.xd.ph < 1 && !(v.quad && g.wout % v.p == 0)) return false;
        // 1x1 filters read only the image proper; larger filters need the zero halo
        if (one) return g.pad == 0;
        return g.xd.ph >= g.pad && g.xd.pw >= g.pad;
    }
    if (v.family == FAM_PTILE) {
        // staging pays only when a staged element is reused by several taps
        if (w->kh * w->kw == 1) return false;
        const PtileGeom pg = ptile_geom(v, w->cin, w->kh, w->kw, g.stride, g.pad, g.wout);
        return pg.nstp <= kPtileMaxSteps && (int64_t)pg.plane * 4 <= (int64_t)kLdsBytesPerCU;
    }
    if (v.family == FAM_WTILE) {
        // pixel-wise layers take the flattened-pixel instantiations, filters with taps the lane grids
        if ((w->kh * w->kw == 1) != (v.flat != 0)) return false;
        if (v.flat && g.pad != 0) return false;
        const WtileGeom wg = wtile_geom(v, w->cin, w->kh, w->kw, g.stride);
        if (wg.nstp > kWtileMaxSteps || wg.lds_bytes > kLdsBytesPerCU) return false;
        // a flattened tile runs over the images of the batch: the whole tensor behind one 32-bit offset
        if (v.flat && (g.xd.image * (int64_t)w->elem() * g.n >= 0x7ffffff0ll ||
                       (int64_t)w->cout * (g.hout + 64) * (g.wout + 64) * (int64_t)w->elem() * g.n >= 0x7ffffff0ll))
            return false;
        return true;
    }
    if (v.kh != w->kh || v.kw != w->kw) return false;
    // the wave-sliced LDS kernel buffers the stream of a (row group, channel chunk)
    return v.family != FAM_STILE || stile_streams_fit(w, &v);
}

static std::vector<const ConvVariant*> candidates(const cadnn_weights* w, const ConvGeom& g) {
    std::vector<const ConvVariant*> out;
    for (const ConvVariant& v : all_linear_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    for (const ConvVariant& v : all_quad_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    for (const ConvVariant& v : all_direct_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    for (const ConvVariant& v : all_tile_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    for (const ConvVariant& v : all_dense_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    for (const ConvVariant& v : all_dense_wide_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    for (const ConvVariant& v : all_stile_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    for (const ConvVariant& v : all_ptile_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    for (const ConvVariant& v : all_wtile_variants()) if (variant_fits(v, w, g)) out.push_back(&v);
    // No sparse kernel is instantiated for the geometry (say a 5x5 or a stride-3 7x7 filter on
    // an input without halo): the matrix-core kernel, which takes any geometry, serves it
    // whatever the density, so that every valid layer runs.
    if (out.empty())
        for (const ConvVariant& v : all_dense_variants()) if (variant_fits(v, w, g, true)) out.push_back(&v);
    return out;
}

// Default choice when nothing was tuned or pinned: a model of one launch on 256 CUs x 4
// SIMDs, in cycles.  For the staging-free families it is the largest of three terms --
// a wave's own latency chain times the rounds of waves the chip needs, the vector issue
// slots all waves consume (prologue + instructions per nonzero), and the L1 cache-line
// traffic (32 bytes per cycle per CU; a stride-2 lane pattern touches twice the lines) --
// with constants fitted to the tuner's timings of every variant on ResNet-50, VGG-16,
// MobileNet-V1 and Inception-V3 at batch 1 and ResNet-50 at batch 8 (its pick costs 8-15 %
// over the tuned choice; the fit leaves the L1 term almost no weight).
// Modelled cycles of one launch of variant v on the layer; negative: not modelled (the
// LDS-staged families, chosen by tuning only).
static double variant_cost(const cadnn_weights* w, const ConvGeom& g, const ConvVariant* v) {
    const double nnz_row = w->cout ? (double)w->nnz / w->cout : 0.0;
    const double pixels = (double)g.hout * g.wout;
    double cost;
    if (v->family == FAM_DENSE && v->tw == 128) {
        // large tiles, two workgroups per CU; for a pruned layer, and for K split over
        // workgroups, the measured selection decides
        if ((double)w->nnz < 0.25 * (double)w->cout * w->cin * w->kh * w->kw || v->splitk > 1) return -1.0;
        const double tm = v->rows_per_block(), tn = 64.0 * v->p;
        const double blocks = std::ceil(pixels * g.n / tn) * std::ceil(w->cout / tm);
        const double K = (double)w->cin * w->kh * w->kw;
        cost = 4000.0 + std::ceil(blocks / 512.0) * std::ceil(K / 32.0) * (300.0 + 1200.0 * tm * tn / 16384.0);
    } else if (v->family == FAM_DENSE) {
        // matrix cores: 64 x 64 tiles, ~1024 cycles per 32-deep chunk of K per tile
        if ((double)w->nnz < 0.25 * (double)w->cout * w->cin * w->kh * w->kw) return -1.0;   // by measurement only
        const double blocks = std::ceil(pixels / 64.0) * g.n * std::ceil(w->cout / 64.0);
        const double K = (double)w->cin * w->kh * w->kw;
        cost = 2500.0 + std::ceil(blocks / 256.0) * std::ceil(K / 32.0) * 1100.0;
    } else if (v->family == FAM_STILE || v->family == FAM_PTILE || v->family == FAM_WTILE) {
        return -1.0;
    } else if (v->quad) {
        return -1.0;
    } else if (v->family != FAM_TILE) {
        const int P = v->p;
        const double walked = v->adjacent == 2 ? (double)g.hout * ((g.wout + P - 1) / P * P) : pixels;
        const double tiles = std::ceil(walked / (64.0 * P)) * g.n;
        const double blocks = tiles * std::ceil((double)w->cout / v->rows_per_block());
        const double waves = blocks * v->nw;
        const double iters = v->rpw * nnz_row / v->ks;
        const double line_bytes = 256.0 * P * ((g.stride == 2 && !g.xd.s2d) ? 2.0 : 1.0);
        const double t_l1 = waves * iters * line_bytes / 32.0 / 256.0;
        const double instrs = v->adjacent ? 3.0 + P : 2.0 + 2.0 * P;
        const double t_issue = waves * (1787.0 + iters * instrs * 1.21) / 1024.0;
        const double per_nz = 77.4 * (1.0 + 0.51 * (P - 1)) / (1.0 + 0.079 * std::log2(v->unroll / 4.0));
        const double t_wave = 382.0 + iters * per_nz + (v->ks > 1 ? 338.0 * std::log2((double)v->ks) : 0.0);
        const double rounds = std::ceil(waves / (1024.0 * 2.3));
        cost = std::max(std::max(t_wave * rounds, t_issue), 0.078 * t_l1);
        if (v->family == FAM_DIRECT) cost *= 1.3;   // per-lane tap offsets, bounds by range check
    } else {
        const double tiles = std::ceil((double)g.wout / v->tw) * std::ceil((double)g.hout / v->th) * g.n;
        const double blocks = tiles * std::ceil((double)w->cout / v->rows_per_block());
        const double nchunks = std::ceil((double)w->cin / v->cch);
        const double stage = nchunks * (1500.0 + (double)std::min(w->cin, v->cch) * v->plane / (v->nw * 64.0) * 24.0);
        const double iters = v->rpw * nnz_row;
        const double t_block = stage + iters * (10.0 + 6.0 * v->p);
        const double rounds = std::ceil(blocks / 256.0);
        cost = t_block * rounds * 2.0;   // until tuned, prefer the staging-free families
    }
    return cost;
}

static const ConvVariant* heuristic_variant(const cadnn_weights* w, const ConvGeom& g) {
    const std::vector<const ConvVariant*> cand = candidates(w, g);
    if (cand.empty()) return nullptr;
    const double nnz_row = w->cout ? (double)w->nnz / w->cout : 0.0;
    const ConvVariant* best = nullptr;
    double best_cost = 0.0;
    for (const ConvVariant* v : cand) {
        const double cost = variant_cost(w, g, v);
        if (cost < 0.0) continue;   // chosen by tuning only
        if (!best || cost < best_cost) { best = v; best_cost = cost; }
    }
    if (!best) {
        // only LDS-staged variants serve the geometry (a 5x5 filter on a plain tensor): take
        // the one whose waves walk the fewest nonzeros each, the channel split priced as above
        for (const ConvVariant* v : cand) {
            const double cost = v->rpw * nnz_row / v->ks + (v->ks > 1 ? 338.0 / 77.4 * std::log2((double)v->ks) : 0.0);
            if (!best || cost < best_cost) { best = v; best_cost = cost; }
        }
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

// The launch record of variant v on the layer (builds and uploads the variant's plan on first use).
static cadnn_status make_launch(const cadnn_weights* w, const ConvVariant* v, const ConvGeom& g,
                                const void* x, void* y, const TensorDesc& yd, const void* residual,
                                const TensorDesc& rd, const void* bias, int relu, ConvLaunch* out,
                                std::shared_ptr<ConvPlan>* keep = nullptr) {
    const ConvPlan* plan = nullptr;
    cadnn_status st = get_conv_plan(w, v, g.xd, g.stride, g.pad, g.wout, &plan, g.ex, keep);
    if (st != CADNN_OK) return st;
    ConvLaunch a{};
    a.x = x;
    a.y = y;
    a.bias = (const float*)bias;
    a.residual = residual;
    a.nz = (const uint2*)plan->nz.p;
    a.nz_off = (const uint16_t*)plan->nz_off.p;
    a.seg_ptr = (const int32_t*)plan->seg_ptr.p;
    a.perm = (const int32_t*)plan->perm.p;
    a.xd = g.xd; a.yd = yd; a.rd = rd;
    a.n = g.n; a.cout = w->cout; a.stride = g.stride; a.pad = g.pad; a.relu = relu ? 1 : 0;
    if (g.ex && g.ex->pool_y) {
        a.pool_y = g.ex->pool_y;
        a.pool_scale = 1.0f / (float)(g.hout * g.wout);
    }
    if (g.ex && g.ex->dw) {
        if (!g.ex->dw->dw_ready) return fail(CADNN_EINVAL, "fused depthwise filters were not prepared");
        a.dw_y = g.ex->dw_y;
        a.dw_w = (const float*)g.ex->dw->d_dw.p;
        a.dw_bias = (const float*)g.ex->dw_bias;
        a.dw_yd = g.ex->dw_yd;
        a.dw_stride = g.ex->dw_stride;
        a.dw_relu = g.ex->dw_relu;
    }
    if (g.ex && g.ex->w) {
        // the shortcut's input as a plain view walked with one stride from pixel (0, 0)
        a.x2 = g.ex->x;
        a.bias2 = (const float*)g.ex->bias;
        a.x2d = g.ex->xd;
        a.stride2 = g.ex->stride;
        if (g.ex->xd.s2d) {
            a.x2d.origin = tensor_off(g.ex->xd, 0, 0);
            a.x2d.s2d = 0;
            a.stride2 = 1;
        }
        a.image2_bytes = (uint32_t)(g.ex->xd.image * (int64_t)w->elem());
    }
    if (g.xd.s2d && g.stride == 2 && v->family != FAM_DENSE) {
        // plain view for the kernel: unit stride over the rows of one phase, starting at the
        // position of tap (0, 0) of output pixel (0, 0); the plan's tap offsets pick the phase
        a.xd.origin = tensor_off(g.xd, -g.pad, -g.pad);
        a.xd.s2d = 0;
        a.stride = 1;
        a.pad = 0;
    }
    a.nchunks = plan->nchunks;
    a.kh = w->kh; a.kw = w->kw; a.is_f16 = w->dtype == CADNN_F16;
    a.hwout = g.hout * g.wout;
    a.image_bytes = (uint32_t)(g.xd.image * (int64_t)w->elem());
    if (v->family == FAM_PTILE) {
        const PtileGeom pg = ptile_geom(*v, w->cin, w->kh, w->kw, g.stride, g.pad, g.wout);
        a.tiles_x = (g.wout + pg.tile_w - 1) / pg.tile_w;
        a.tiles_y = (g.hout + pg.tile_h - 1) / pg.tile_h;
        a.pt_pitch = pg.pitch; a.pt_sub = pg.sub; a.pt_plane = pg.plane; a.pt_nphc = pg.nphc;
        a.pt_nph = pg.nphr * pg.nphc; a.pt_in_rows = pg.in_rows; a.pt_in_cols = pg.alias ? pg.in_cols - 1 : pg.in_cols;
        a.pt_cch = pg.cch; a.pt_nstp = pg.nstp; a.pt_nchunks = pg.nchunks;
        a.pt_lds_bytes = (uint32_t)pg.lds_bytes;
        a.pt_nbuf = pg.nbuf;
    } else if (v->family == FAM_WTILE) {
        const WtileGeom wg = wtile_geom(*v, w->cin, w->kh, w->kw, g.stride);
        if (wg.flat) {
            a.tiles_x = (int)(((int64_t)g.n * g.hout * g.wout + wg.tile_w - 1) / wg.tile_w);
            a.tiles_y = 1;
        } else {
            a.tiles_x = (g.wout + wg.tile_w - 1) / wg.tile_w;
            a.tiles_y = (g.hout + wg.tile_h - 1) / wg.tile_h;
        }
        a.wt_tiles = a.tiles_x * a.tiles_y;
        a.wt_lc = wg.lc; a.wt_ns = wg.ns; a.wt_pitch = wg.pitch; a.wt_sub = wg.sub; a.wt_plane = wg.plane;
        a.wt_nphc = wg.nphc; a.wt_nph = wg.nphr * wg.nphc; a.wt_cch = wg.cch; a.wt_nstp = wg.nstp;
        a.wt_nchunks = wg.nchunks; a.wt_nbuf = wg.nbuf;
        a.wt_lds_bytes = (uint32_t)wg.lds_bytes;
        auto magic = [](int d) { return (uint32_t)((((uint64_t)1 << 32) + (uint64_t)d - 1) / (uint64_t)d); };
        a.wt_m_sub = magic(wg.sub); a.wt_m_pitch = magic(wg.pitch); a.wt_m_nphc = magic(wg.nphc);
    } else if (v->family == FAM_TILE || v->family == FAM_STILE) {
        a.tiles_x = (g.wout + v->tw - 1) / v->tw;
        a.tiles_y = (g.hout + v->th - 1) / v->th;
    } else {
        a.wq = (v->family == FAM_LINEAR && v->adjacent == 2) ? (g.wout + v->p - 1) / v->p * v->p : g.wout;
        a.hwq = g.hout * a.wq;
        a.tiles_x = (a.hwq + 64 * v->p - 1) / (64 * v->p);
        if (v->family == FAM_LINEAR && v->dw == 2) a.tiles_x = 1;    // the workgroup's waves are the tiles
        a.tiles_y = 1;
    }
    a.row_groups = plan->rows_padded / v->rows_per_block();
    a.sk = 1;
    if (v->family == FAM_DENSE && v->splitk > 1 && (st = ensure_sk_scratch(w, v, g, &a)) != CADNN_OK) return st;
    *out = a;
    return CADNN_OK;
}

static cadnn_status launch_variant(const cadnn_weights* w, const ConvVariant* v, const ConvGeom& g,
                                   const void* x, void* y, const TensorDesc& yd, const void* residual,
                                   const TensorDesc& rd, const void* bias, int relu, hipStream_t s) {
    ConvLaunch a;
    cadnn_status st = make_launch(w, v, g, x, y, yd, residual, rd, bias, relu, &a);
    if (st != CADNN_OK) return st;
    CADNN_HIP(v->launch(a, s));
    return CADNN_OK;
}

// ---- independent layers in one launch ---------------------------------------------
static cadnn_status check_io(const char* who, const cadnn_weights* w, const ConvGeom& g, const void* x,
                             void* y, const TensorDesc& yd, const void* residual, const TensorDesc& rd);
static cadnn_status member_geom(const ConvMember& m, int n, ConvGeom* g) {
    if (m.pool_kind != 0) {
        // a window pool: only its tensors are checked, it constrains no variant
        if (!m.x || !m.y || m.x == m.y || m.pool_k <= 0 || m.stride <= 0 || m.pad < 0 || m.xd.s2d || m.yd.s2d ||
            m.yd.c != m.xd.c || m.yd.h != conv_out(m.xd.h, m.pool_k, m.stride, m.pad) ||
            m.yd.w != conv_out(m.xd.w, m.pool_k, m.stride, m.pad) || m.yd.h <= 0 || m.yd.w <= 0 || n <= 0)
            return fail(CADNN_EINVAL, "cadnn_net (co-launched layers): bad pool member");
        *g = ConvGeom{};
        return CADNN_OK;
    }
    cadnn_status st = check_conv("cadnn_net (co-launched layers)", m.w, m.xd, n, m.stride, m.pad, g,
                                 m.yd.s2d || (m.residual && m.rd.s2d), nullptr);
    if (st != CADNN_OK) return st;
    return check_io("cadnn_net (co-launched layers)", m.w, *g, m.x, m.y, m.yd, m.residual, m.rd);
}

cadnn_status conv2d_group_candidates(const std::vector<ConvMember>& members, int n,
                                     std::vector<const ConvVariant*>* out, const ConvVariant** pick) {
    out->clear();
    if (pick) *pick = nullptr;
    std::vector<ConvGeom> geoms(members.size());
    for (size_t k = 0; k < members.size(); ++k) {
        cadnn_status st = member_geom(members[k], n, &geoms[k]);
        if (st != CADNN_OK) return st;
    }
    if (members.empty()) return CADNN_OK;
    for (const ConvVariant& v : all_linear_variants()) {   // (the only family that offers it)
        if (!v.launch_multi) continue;
        bool all = true, any = false;
        for (size_t k = 0; k < members.size() && all; ++k) {
            if (members[k].pool_kind != 0) continue;
            any = true;
            all = variant_fits(v, members[k].w, geoms[k]);
        }
        if (all && any) out->push_back(&v);
    }
    // untuned pick: the layers run side by side, so the slowest of them decides
    double best = 0.0;
    for (const ConvVariant* v : *out) {
        double worst = 0.0;
        for (size_t k = 0; k < members.size(); ++k)
            if (members[k].pool_kind == 0) worst = std::max(worst, variant_cost(members[k].w, geoms[k], v));
        if (pick && (!*pick || worst < best)) { *pick = v; best = worst; }
    }
    return CADNN_OK;
}

cadnn_status conv2d_group_records(const std::vector<ConvMember>& members, int n, const ConvVariant* v,
                                  std::vector<ConvLaunch>* records, std::vector<std::shared_ptr<ConvPlan>>* keep) {
    records->resize(members.size());
    if (keep) keep->assign(members.size(), nullptr);
    if (members.size() > (size_t)kMaxCoLaunch) return fail(CADNN_EINVAL, "cadnn_net: more than %d layers in one launch", kMaxCoLaunch);
    int64_t total = 0;
    if (!v || !v->launch_multi) return fail(CADNN_EINVAL, "cadnn_net: variant cannot launch several layers");
    for (size_t k = 0; k < members.size(); ++k) {
        const ConvMember& m = members[k];
        ConvGeom g;
        cadnn_status st = member_geom(m, n, &g);
        if (st != CADNN_OK) return st;
        if (m.pool_kind != 0) {
            ConvLaunch a{};
            a.x = m.x; a.y = m.y; a.xd = m.xd; a.yd = m.yd; a.n = n; a.stride = m.stride; a.pad = m.pad;
            a.op_type = m.pool_kind; a.pool_k = m.pool_k;
            // the output elements of an image dealt round robin to the threads of at most 256
            // workgroups (one per compute unit)
            const int64_t threads = (int64_t)v->nw * 64;
            a.tiles_x = 1;
            a.tiles_y = 1;
            a.row_groups = (int)std::min<int64_t>(((int64_t)m.yd.c * m.yd.h * m.yd.w + threads - 1) / threads, 256);
            (*records)[k] = a;
            total += (int64_t)a.tiles_x * a.row_groups;
            continue;
        }
        if (!variant_fits(*v, m.w, g)) return fail(CADNN_EINVAL, "cadnn_net: '%s' does not serve every co-launched layer", v->name);
        if ((st = make_launch(m.w, v, g, m.x, m.y, m.yd, m.residual, m.rd, m.bias, m.relu, &(*records)[k],
                              keep ? &(*keep)[k] : nullptr)) != CADNN_OK) return st;
        total += (int64_t)(*records)[k].tiles_x * (*records)[k].row_groups;
    }
    if (n > 65535 || total > 0x7fffffffll)
        return fail(CADNN_EUNSUPPORTED, "cadnn_net: co-launched layers exceed the grid limits");
    return CADNN_OK;
}

// Times every variant that serves all members in one launch, the way conv2d_tune_impl times a
// single layer (caches swept, `before` launched, one event-timed launch per repeat).
cadnn_status conv2d_group_tune(const std::vector<ConvMember>& members, int n, hipStream_t s, int reps,
                               const std::function<cadnn_status()>* before, const ConvVariant** best_v,
                               float* best_us) {
    *best_v = nullptr;
    if (reps <= 0) return fail(CADNN_EINVAL, "cadnn_net: reps must be positive");
    std::vector<const ConvVariant*> cand;
    cadnn_status st = conv2d_group_candidates(members, n, &cand, nullptr);
    if (st != CADNN_OK) return st;
    if (cand.empty()) return CADNN_OK;
    DevBuf sweep;
    const size_t sweep_bytes = (size_t)64 << 20;
    if (hipMalloc(&sweep.p, 2 * sweep_bytes) != hipSuccess) {
        sweep.p = nullptr;
        return fail(CADNN_ENOMEM, "cadnn_net: no memory for the cache sweep buffer");
    }
    sweep.bytes = 2 * sweep_bytes;
    if (hipMemsetAsync(sweep.p, 0, 2 * sweep_bytes, s) != hipSuccess) return fail(CADNN_EHIP, "hipMemsetAsync failed");
    hipEvent_t e0 = nullptr, e1 = nullptr;
    CADNN_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(CADNN_EHIP, "hipEventCreate failed"); }
    float best_ms = 0.0f;
    std::vector<ConvLaunch> recs;
    const TrialPlans trial;
    for (const ConvVariant* v : cand) {
        if (conv2d_group_records(members, n, v, &recs) != CADNN_OK) continue;   // does not fit these weights
        DevBuf table;
        if ((st = table.upload(recs.data(), recs.size() * sizeof(ConvLaunch))) != CADNN_OK) break;
        const ConvLaunch* tab = (const ConvLaunch*)table.p;
        if (v->launch_multi(tab, recs.data(), (int)recs.size(), n, s) != hipSuccess) { st = fail(CADNN_EHIP, "co-launch failed"); break; }
        float total_ms = 0.0f;
        for (int i = 0; i < reps && st == CADNN_OK; ++i) {
            st = launch_copy(sweep.p, (char*)sweep.p + sweep_bytes, sweep_bytes, s);
            if (st != CADNN_OK) break;
            if (before && (st = (*before)()) != CADNN_OK) break;
            if (hipEventRecord(e0, s) != hipSuccess) { st = fail(CADNN_EHIP, "hipEventRecord failed"); break; }
            if (v->launch_multi(tab, recs.data(), (int)recs.size(), n, s) != hipSuccess) { st = fail(CADNN_EHIP, "co-launch failed"); break; }
            if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) { st = fail(CADNN_EHIP, "event wait failed"); break; }
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { st = fail(CADNN_EHIP, "hipEventElapsedTime failed"); break; }
            total_ms += ms;
        }
        if (st != CADNN_OK) break;
        if (hipStreamSynchronize(s) != hipSuccess) { st = fail(CADNN_EHIP, "hipStreamSynchronize failed"); break; }   // before the table goes
        if (std::getenv("CADNN_TUNE_LOG"))
            std::fprintf(stderr, "[cadnn tune] %zu layers at once %-44s %8.2f us\n", members.size(), v->name, total_ms * 1e3f / reps);
        if (!*best_v || total_ms < best_ms) { *best_v = v; best_ms = total_ms; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != CADNN_OK) return st;
    for (const ConvMember& m : members) if (m.w) drop_unpinned_plans(m.w);
    if (best_us) *best_us = best_ms * 1e3f / reps;
    return CADNN_OK;
}

static cadnn_status check_io(const char* who, const cadnn_weights* w, const ConvGeom& g, const void* x,
                             void* y, const TensorDesc& yd, const void* residual, const TensorDesc& rd) {
    if (!x || !y) return fail(CADNN_EINVAL, "%s: NULL tensor", who);
    if (x == y) return fail(CADNN_EINVAL, "%s: y aliases x", who);
    if (yd.c != w->cout || yd.h != g.hout || yd.w != g.wout) return fail(CADNN_EINVAL, "%s: output layout does not match the layer", who);
    if (residual && (rd.c != w->cout || rd.h != g.hout || rd.w != g.wout))
        return fail(CADNN_EINVAL, "%s: residual layout does not match the output", who);
    return CADNN_OK;
}

cadnn_status conv2d_impl(const cadnn_weights* w, const void* x, const TensorDesc& xd, void* y,
                         const TensorDesc& yd, const void* residual, const TensorDesc& rd, int n,
                         int stride, int pad, const void* bias, int relu, hipStream_t s, const ConvExtra* ex) {
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_sparse_conv2d", w, xd, n, stride, pad, &g, yd.s2d || (residual && rd.s2d), ex);
    if (st != CADNN_OK) return st;
    if ((st = check_io("cadnn_sparse_conv2d", w, g, x, y, yd, residual, rd)) != CADNN_OK) return st;
    const ConvVariant* v = pick_variant(w, g);
    if (!v)
        return fail(CADNN_EUNSUPPORTED, "cadnn_sparse_conv2d: no kernel for %dx%d filters with stride %d",
                    w->kh, w->kw, stride);
    return launch_variant(w, v, g, x, y, yd, residual, rd, bias, relu, s);
}

cadnn_status conv2d_prepare_impl(const cadnn_weights* w, const TensorDesc& xd, int n, int stride, int pad,
                                 int out_s2d, const ConvExtra* ex) {
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_prepare", w, xd, n, stride, pad, &g, out_s2d, ex);
    if (st != CADNN_OK) return st;
    const ConvVariant* v = pick_variant(w, g);
    if (!v)
        return fail(CADNN_EUNSUPPORTED, "cadnn_conv2d_prepare: no kernel for %dx%d filters with stride %d",
                    w->kh, w->kw, stride);
    const ConvPlan* plan = nullptr;
    if ((st = get_conv_plan(w, v, xd, g.stride, g.pad, g.wout, &plan, g.ex)) != CADNN_OK) return st;
    return ensure_sk_scratch(w, v, g, nullptr);
}

const char* conv2d_variant_name_impl(const cadnn_weights* w, const TensorDesc& xd, int n, int stride, int pad,
                                     int out_s2d, const ConvExtra* ex) {
    ConvGeom g;
    if (check_conv("cadnn_net_op_variant", w, xd, n, stride, pad, &g, out_s2d, ex) != CADNN_OK) return nullptr;
    const ConvVariant* v = pick_variant(w, g);
    if (!v) {
        (void)fail(CADNN_EUNSUPPORTED, "no kernel for %dx%d filters with stride %d", w->kh, w->kw, stride);
        return nullptr;
    }
    return v->name;
}

cadnn_status conv2d_list_variants_impl(const cadnn_weights* w, const TensorDesc& xd, int n, int stride, int pad,
                                       char* buf, size_t len, int out_s2d, const ConvExtra* ex) {
    if (!buf || len == 0) return fail(CADNN_EINVAL, "cadnn_conv2d_list_variants: NULL buffer");
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_list_variants", w, xd, n, stride, pad, &g, out_s2d, ex);
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

cadnn_status conv2d_set_variant_impl(const cadnn_weights* w, const TensorDesc& xd, int n, int stride, int pad,
                                     const char* name, int out_s2d, const ConvExtra* ex) {
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_set_variant", w, xd, n, stride, pad, &g, out_s2d, ex);
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

cadnn_status conv2d_tune_impl(const cadnn_weights* w, const void* x, const TensorDesc& xd, void* y,
                              const TensorDesc& yd, const void* residual, const TensorDesc& rd, int n,
                              int stride, int pad, const void* bias, int relu, hipStream_t s, int reps,
                              float* best_us, const std::function<cadnn_status()>* before, const ConvExtra* ex) {
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_tune", w, xd, n, stride, pad, &g, yd.s2d || (residual && rd.s2d), ex);
    if (st != CADNN_OK) return st;
    if ((st = check_io("cadnn_conv2d_tune", w, g, x, y, yd, residual, rd)) != CADNN_OK) return st;
    if (reps <= 0) return fail(CADNN_EINVAL, "cadnn_conv2d_tune: reps must be positive");
    const std::vector<const ConvVariant*> cand = candidates(w, g);
    if (cand.empty())
        return fail(CADNN_EUNSUPPORTED, "cadnn_conv2d_tune: no kernel for %dx%d filters with stride %d",
                    w->kh, w->kw, stride);
    // Inside a network a layer starts with cold L2 caches: its input was just written by
    // another kernel and its weights were last touched a whole forward pass ago.  Timing
    // back-to-back repeats would reward variants that only do well on cached data, so the
    // L2s are swept with a 64 MiB copy before every timed launch.
    DevBuf sweep;
    const size_t sweep_bytes = (size_t)64 << 20;
    if (hipMalloc(&sweep.p, 2 * sweep_bytes) != hipSuccess) {
        sweep.p = nullptr;
        return fail(CADNN_ENOMEM, "cadnn_conv2d_tune: no memory for the cache sweep buffer");
    }
    sweep.bytes = 2 * sweep_bytes;
    if (hipMemsetAsync(sweep.p, 0, 2 * sweep_bytes, s) != hipSuccess) return fail(CADNN_EHIP, "hipMemsetAsync failed");
    hipEvent_t e0 = nullptr, e1 = nullptr;
    CADNN_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(CADNN_EHIP, "hipEventCreate failed"); }
    const ConvVariant* best = nullptr;
    float best_ms = 0.0f;
    const TrialPlans trial;
    for (const ConvVariant* v : cand) {
        {
            const ConvPlan* probe = nullptr;
            if (get_conv_plan(w, v, g.xd, g.stride, g.pad, g.wout, &probe, g.ex) == CADNN_EUNSUPPORTED) continue;   // does not fit these weights
        }
        st = launch_variant(w, v, g, x, y, yd, residual, rd, bias, relu, s);
        float total_ms = 0.0f;
        for (int i = 0; i < reps && st == CADNN_OK; ++i) {
            st = launch_copy(sweep.p, (char*)sweep.p + sweep_bytes, sweep_bytes, s);
            if (st != CADNN_OK) break;
            // inside a net: the producer of the input runs right before, as it will
            if (before && (st = (*before)()) != CADNN_OK) break;
            if (hipEventRecord(e0, s) != hipSuccess) { st = fail(CADNN_EHIP, "hipEventRecord failed"); break; }
            st = launch_variant(w, v, g, x, y, yd, residual, rd, bias, relu, s);
            if (st != CADNN_OK) break;
            if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) { st = fail(CADNN_EHIP, "event wait failed"); break; }
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { st = fail(CADNN_EHIP, "hipEventElapsedTime failed"); break; }
            total_ms += ms;
        }
        if (st != CADNN_OK) break;
        const float ms = total_ms;
        if (std::getenv("CADNN_TUNE_LOG"))
            std::fprintf(stderr, "[cadnn tune] cin=%d cout=%d k=%d s=%d hw=%dx%d nnz=%lld %-44s %8.2f us\n", w->cin,
                         w->cout, w->kh, stride, xd.h, xd.w, (long long)w->nnz, v->name, ms * 1e3f / reps);
        if (!best || ms < best_ms) { best = v; best_ms = ms; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != CADNN_OK) return st;
    {
        std::lock_guard<std::mutex> lock(w->mu);
        w->chosen[g.key()] = best;
    }
    drop_unpinned_plans(w);
    if (best_us) *best_us = best_ms * 1e3f / reps;
    return CADNN_OK;
}

}  // namespace cadnn

static TensorDesc out_desc(const cadnn_weights* w, int h, int wdt, int stride, int pad) {
    if (stride <= 0 || pad < 0) return make_desc(0, 0, 0);   // rejected by the argument checks
    return make_desc(w ? w->cout : 0, w ? conv_out(h, w->kh, stride, pad) : 0, w ? conv_out(wdt, w->kw, stride, pad) : 0);
}

extern "C" cadnn_status cadnn_sparse_conv2d(const cadnn_weights* w, const void* x, void* y, int n,
                                            int h, int wdt, int stride, int pad, const void* bias,
                                            const void* residual, int relu, void* stream) {
    const TensorDesc yd = out_desc(w, h, wdt, stride, pad);
    return conv2d_impl(w, x, make_desc(w ? w->cin : 0, h, wdt), y, yd, residual, yd, n, stride, pad, bias,
                       relu, (hipStream_t)stream);
}

extern "C" cadnn_status cadnn_conv2d_tune(const cadnn_weights* w, const void* x, void* y, int n, int h,
                                          int wdt, int stride, int pad, const void* bias,
                                          const void* residual, int relu, void* stream, int reps,
                                          float* best_us) {
    const TensorDesc yd = out_desc(w, h, wdt, stride, pad);
    return conv2d_tune_impl(w, x, make_desc(w ? w->cin : 0, h, wdt), y, yd, residual, yd, n, stride, pad,
                            bias, relu, (hipStream_t)stream, reps, best_us);
}

extern "C" cadnn_status cadnn_conv2d_prepare(const cadnn_weights* w, int n, int h, int wdt,
                                             int stride, int pad) {
    return conv2d_prepare_impl(w, make_desc(w ? w->cin : 0, h, wdt), n, stride, pad);
}

extern "C" cadnn_status cadnn_conv2d_variant_name(const cadnn_weights* w, int n, int h, int wdt,
                                                  int stride, int pad, char* buf, size_t len) {
    if (!buf || len == 0) return fail(CADNN_EINVAL, "cadnn_conv2d_variant_name: NULL buffer");
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_variant_name", w, make_desc(w ? w->cin : 0, h, wdt), n, stride, pad, &g);
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
    return conv2d_list_variants_impl(w, make_desc(w ? w->cin : 0, h, wdt), n, stride, pad, buf, len);
}

extern "C" cadnn_status cadnn_conv2d_set_variant(const cadnn_weights* w, int n, int h, int wdt,
                                                 int stride, int pad, const char* name) {
    return conv2d_set_variant_impl(w, make_desc(w ? w->cin : 0, h, wdt), n, stride, pad, name);
}

// The variant `name` among those that serve the layer (NULL / "": the one that would be launched).
static cadnn_status named_variant(const char* who, const cadnn_weights* w, const ConvGeom& g, const char* name,
                                  const ConvVariant** out) {
    *out = nullptr;
    if (!name || !*name) {
        *out = pick_variant(w, g);
        if (!*out) return fail(CADNN_EUNSUPPORTED, "%s: no kernel for %dx%d filters with stride %d", who, w->kh, w->kw, g.stride);
        return CADNN_OK;
    }
    for (const ConvVariant* v : candidates(w, g))
        if (std::strcmp(v->name, name) == 0) { *out = v; return CADNN_OK; }
    return fail(CADNN_EINVAL, "%s: '%s' does not serve this layer", who, name);
}

extern "C" cadnn_status cadnn_conv2d_plan_info(const cadnn_weights* w, int n, int h, int wdt, int stride, int pad,
                                               const char* variant, cadnn_plan_info* out) {
    if (!out) return fail(CADNN_EINVAL, "cadnn_conv2d_plan_info: NULL pointer");
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_plan_info", w, make_desc(w ? w->cin : 0, h, wdt), n, stride, pad, &g);
    if (st != CADNN_OK) return st;
    const ConvVariant* v = nullptr;
    if ((st = named_variant("cadnn_conv2d_plan_info", w, g, variant, &v)) != CADNN_OK) return st;
    ConvPlan plan;
    if ((st = build_host_plan(w, v, g.xd, g.stride, g.pad, g.wout, &plan)) != CADNN_OK) return st;
    cadnn_plan_info info{};
    info.entries = plan.walked;
    info.stream_bytes = plan.walked * plan.entry_bytes;
    info.alloc_bytes = (int64_t)plan.nz.bytes + (int64_t)plan.nz_off.bytes;
    info.table_bytes = (int64_t)plan.seg_ptr.bytes + (int64_t)plan.perm.bytes;
    info.bytes_per_nonzero = w->nnz ? (double)info.stream_bytes / (double)w->nnz : 0.0;
    info.chunks = 1;
    info.lds_bytes = (int)v->lds_bytes;
    if (v->family == FAM_WTILE) {
        const WtileGeom wg = wtile_geom(*v, w->cin, w->kh, w->kw, g.stride);
        info.chunks = wg.nchunks;
        info.lds_bytes = (int)wg.lds_bytes;
    } else if (v->family == FAM_PTILE) {
        const PtileGeom pg = ptile_geom(*v, w->cin, w->kh, w->kw, g.stride, g.pad, g.wout);
        info.chunks = pg.nchunks;
        info.lds_bytes = (int)pg.lds_bytes;
    } else if (v->family == FAM_TILE || v->family == FAM_STILE) {
        info.chunks = plan.nchunks;
    }
    *out = info;
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_conv2d_plan_unpack(const cadnn_weights* w, int n, int h, int wdt, int stride, int pad,
                                                 const char* variant, float* w_host_out) {
    if (!w_host_out) return fail(CADNN_EINVAL, "cadnn_conv2d_plan_unpack: NULL pointer");
    ConvGeom g;
    cadnn_status st = check_conv("cadnn_conv2d_plan_unpack", w, make_desc(w ? w->cin : 0, h, wdt), n, stride, pad, &g);
    if (st != CADNN_OK) return st;
    const ConvVariant* v = nullptr;
    if ((st = named_variant("cadnn_conv2d_plan_unpack", w, g, variant, &v)) != CADNN_OK) return st;
    if (v->family != FAM_WTILE) return fail(CADNN_EUNSUPPORTED, "cadnn_conv2d_plan_unpack: '%s' has no compact tile-offset stream", v->name);
    ConvPlan plan;
    if ((st = build_host_plan(w, v, g.xd, g.stride, g.pad, g.wout, &plan)) != CADNN_OK) return st;
    return wtile_plan_unpack(w, v, g.stride, plan, w_host_out);
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

static cadnn_status check_depthwise(const char* who, const cadnn_weights* w, int n, int h, int wdt, int stride,
                                    int pad) {
    if (!w) return fail(CADNN_EINVAL, "%s: NULL handle", who);
    if (w->cin != 1) return fail(CADNN_EINVAL, "%s: weights have %d input channels per filter, a depthwise filter bank has 1", who, w->cin);
    if (n <= 0 || h <= 0 || wdt <= 0 || stride <= 0 || pad < 0) return fail(CADNN_EINVAL, "%s: bad size", who);
    if (conv_out(h, w->kh, stride, pad) <= 0 || conv_out(wdt, w->kw, stride, pad) <= 0)
        return fail(CADNN_EINVAL, "%s: empty output", who);
    if (desc_too_large(make_desc(1, h, wdt)) || desc_too_large(make_desc(1, conv_out(h, w->kh, stride, pad), conv_out(wdt, w->kw, stride, pad))))
        return fail(CADNN_EUNSUPPORTED, "%s: a channel plane of 2^30 elements or more", who);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_depthwise_conv2d(const cadnn_weights* w, const void* x, void* y, int n, int h,
                                               int wdt, int stride, int pad, const void* bias, int relu,
                                               void* stream) {
    if (!x || !y) return fail(CADNN_EINVAL, "cadnn_depthwise_conv2d: NULL tensor");
    cadnn_status st = check_depthwise("cadnn_depthwise_conv2d", w, n, h, wdt, stride, pad);
    if (st != CADNN_OK) return st;
    if ((st = ensure_dw_device(w)) != CADNN_OK) return st;
    const TensorDesc xd = make_desc(w->cout, h, wdt);
    const TensorDesc yd = make_desc(w->cout, conv_out(h, w->kh, stride, pad), conv_out(wdt, w->kw, stride, pad));
    return launch_depthwise(w, x, xd, y, yd, n, stride, pad, (const float*)bias, relu ? 1 : 0, (hipStream_t)stream);
}

extern "C" cadnn_status cadnn_depthwise_prepare(const cadnn_weights* w) {
    if (!w) return fail(CADNN_EINVAL, "cadnn_depthwise_prepare: NULL handle");
    if (w->cin != 1) return fail(CADNN_EINVAL, "cadnn_depthwise_prepare: not a depthwise filter bank");
    return ensure_dw_device(w);
}

extern "C" cadnn_status cadnn_device_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst) return fail(CADNN_EINVAL, "cadnn_device_copy: NULL pointer");
    if (bytes % 16) return fail(CADNN_EINVAL, "cadnn_device_copy: size must be a multiple of 16 bytes");
    return launch_copy(src, dst, bytes, (hipStream_t)stream);
}

// Measurement aid: what one kernel boundary costs inside a replayed HIP graph.  `launches`
// dependent 16-byte copies (the smallest kernel of the library) are captured into one graph,
// which is replayed `reps` times between two events.
extern "C" cadnn_status cadnn_graph_launch_floor(void* scratch32, int launches, int reps, void* stream,
                                                 float* us_per_launch) {
    if (!scratch32 || !us_per_launch) return fail(CADNN_EINVAL, "cadnn_graph_launch_floor: NULL pointer");
    if (launches <= 0 || launches > 4096 || reps <= 0) return fail(CADNN_EINVAL, "cadnn_graph_launch_floor: bad count");
    hipStream_t s = (hipStream_t)stream;
    hipStream_t cs = nullptr;
    CADNN_HIP(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    cadnn_status st = CADNN_OK;
    hipError_t e = hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) st = fail(CADNN_EHIP, "hipStreamBeginCapture failed: %s", hipGetErrorString(e));
    if (st == CADNN_OK) {
        for (int i = 0; i < launches && st == CADNN_OK; ++i) st = launch_copy(scratch32, (char*)scratch32 + 16, 16, cs);
        e = hipStreamEndCapture(cs, &graph);
        if (st == CADNN_OK && e != hipSuccess) st = fail(CADNN_EHIP, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
    }
    if (st == CADNN_OK && hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) != hipSuccess) st = fail(CADNN_EHIP, "hipGraphInstantiate failed");
    if (st == CADNN_OK && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) st = fail(CADNN_EHIP, "hipEventCreate failed");
    if (st == CADNN_OK) {
        bool ok = hipGraphLaunch(exec, s) == hipSuccess && hipEventRecord(e0, s) == hipSuccess;
        for (int r = 0; r < reps && ok; ++r) ok = hipGraphLaunch(exec, s) == hipSuccess;
        ok = ok && hipEventRecord(e1, s) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
        float ms = 0.0f;
        ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
        if (!ok) st = fail(CADNN_EHIP, "cadnn_graph_launch_floor: replay failed");
        else *us_per_launch = ms * 1e3f / (float)reps / (float)launches;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (exec) (void)hipGraphExecDestroy(exec);
    if (graph) (void)hipGraphDestroy(graph);
    (void)hipStreamDestroy(cs);
    return st;
}

extern "C" cadnn_status cadnn_maxpool2d(const void* x, void* y, int n, int c, int h, int wdt, int k,
                                        int stride, int pad, cadnn_dtype dtype, void* stream) {
    if (!x || !y) return fail(CADNN_EINVAL, "cadnn_maxpool2d: NULL tensor");
    if (n <= 0 || c <= 0 || h <= 0 || wdt <= 0 || k <= 0 || stride <= 0 || pad < 0)
        return fail(CADNN_EINVAL, "cadnn_maxpool2d: bad size");
    if (dtype != CADNN_F32 && dtype != CADNN_F16) return fail(CADNN_EINVAL, "cadnn_maxpool2d: dtype");
    if (conv_out(h, k, stride, pad) <= 0 || conv_out(wdt, k, stride, pad) <= 0)
        return fail(CADNN_EINVAL, "cadnn_maxpool2d: empty output");
    if (desc_too_large(make_desc(c, h, wdt)) || desc_too_large(make_desc(c, conv_out(h, k, stride, pad), conv_out(wdt, k, stride, pad))))
        return fail(CADNN_EUNSUPPORTED, "cadnn_maxpool2d: a channel plane of 2^30 elements or more");
    return launch_maxpool(x, make_desc(c, h, wdt), y,
                          make_desc(c, conv_out(h, k, stride, pad), conv_out(wdt, k, stride, pad)), n, k, stride,
                          pad, dtype, (hipStream_t)stream);
}

extern "C" cadnn_status cadnn_avgpool2d(const void* x, void* y, int n, int c, int h, int wdt, int k,
                                        int stride, int pad, cadnn_dtype dtype, void* stream) {
    if (!x || !y) return fail(CADNN_EINVAL, "cadnn_avgpool2d: NULL tensor");
    if (n <= 0 || c <= 0 || h <= 0 || wdt <= 0 || k <= 0 || stride <= 0 || pad < 0)
        return fail(CADNN_EINVAL, "cadnn_avgpool2d: bad size");
    if (dtype != CADNN_F32 && dtype != CADNN_F16) return fail(CADNN_EINVAL, "cadnn_avgpool2d: dtype");
    if (conv_out(h, k, stride, pad) <= 0 || conv_out(wdt, k, stride, pad) <= 0)
        return fail(CADNN_EINVAL, "cadnn_avgpool2d: empty output");
    if (desc_too_large(make_desc(c, h, wdt)) || desc_too_large(make_desc(c, conv_out(h, k, stride, pad), conv_out(wdt, k, stride, pad))))
        return fail(CADNN_EUNSUPPORTED, "cadnn_avgpool2d: a channel plane of 2^30 elements or more");
    return launch_avgpool2d(x, make_desc(c, h, wdt), y,
                            make_desc(c, conv_out(h, k, stride, pad), conv_out(wdt, k, stride, pad)), n, k, stride,
                            pad, dtype, (hipStream_t)stream);
}

extern "C" cadnn_status cadnn_global_avgpool(const void* x, void* y, int n, int c, int h, int wdt,
                                             cadnn_dtype dtype, void* stream) {
    if (!x || !y) return fail(CADNN_EINVAL, "cadnn_global_avgpool: NULL tensor");
    if (n <= 0 || c <= 0 || h <= 0 || wdt <= 0) return fail(CADNN_EINVAL, "cadnn_global_avgpool: bad size");
    if (dtype != CADNN_F32 && dtype != CADNN_F16) return fail(CADNN_EINVAL, "cadnn_global_avgpool: dtype");
    if (desc_too_large(make_desc(c, h, wdt))) return fail(CADNN_EUNSUPPORTED, "cadnn_global_avgpool: a channel plane of 2^30 elements or more");
    return launch_avgpool(x, make_desc(c, h, wdt), y, n, dtype, (hipStream_t)stream);
}
