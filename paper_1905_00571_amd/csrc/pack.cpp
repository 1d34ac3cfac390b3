// Host-side weight packing: dense pruned tensor -> canonical permuted row-compressed form
// (paper Section 3: pruned weights are exact zeros kept with their indices; Section 4:
// filter memory layout is transformed for the device) and the per-variant device plans.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <numeric>

#include "internal.h"

namespace cadnn {

static thread_local std::string g_last_error;
thread_local LaunchTimer* g_launch_timer = nullptr;

cadnn_status fail(cadnn_status code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}
void clear_error() { g_last_error.clear(); }

static thread_local int g_no_device_alloc = 0;
NoDeviceAlloc::NoDeviceAlloc() { ++g_no_device_alloc; }
NoDeviceAlloc::~NoDeviceAlloc() { --g_no_device_alloc; }

static thread_local int g_host_plans = 0;
HostPlans::HostPlans() { ++g_host_plans; }
HostPlans::~HostPlans() { --g_host_plans; }

void DevBuf::release() {
    if (p) {
        if (on_host) std::free(p);
        else (void)hipFree(p);
    }
    p = nullptr;
    bytes = 0;
    on_host = false;
}

cadnn_status DevBuf::upload(const void* host, size_t n) {
    if (g_no_device_alloc > 0 && g_host_plans == 0) return fail(CADNN_EINVAL, "this call may not allocate device memory");
    release();
    const size_t alloc = n < 16 ? 16 : n;
    if (g_host_plans > 0) {
        p = std::calloc(alloc, 1);
        if (!p) return fail(CADNN_ENOMEM, "out of host memory (%zu bytes)", alloc);
        on_host = true;
        bytes = alloc;
        if (n) std::memcpy(p, host, n);
        return CADNN_OK;
    }
    hipError_t e = hipMalloc(&p, alloc);
    if (e != hipSuccess) {
        p = nullptr;
        return fail(CADNN_ENOMEM, "hipMalloc(%zu) failed: %s", alloc, hipGetErrorString(e));
    }
    bytes = alloc;
    if (n) CADNN_HIP(hipMemcpy(p, host, n, hipMemcpyHostToDevice));
    return CADNN_OK;
}

cadnn_status DevBuf::alloc(size_t n, bool zero) {
    if (g_no_device_alloc > 0) return fail(CADNN_EINVAL, "this call may not allocate device memory");
    if (g_host_plans > 0) return fail(CADNN_EINVAL, "device scratch asked for while building host-only plans");
    release();
    const size_t sz = n < 16 ? 16 : n;
    hipError_t e = hipMalloc(&p, sz);
    if (e != hipSuccess) {
        p = nullptr;
        return fail(CADNN_ENOMEM, "hipMalloc(%zu) failed: %s", sz, hipGetErrorString(e));
    }
    bytes = sz;
    if (zero) CADNN_HIP(hipMemset(p, 0, sz));
    return CADNN_OK;
}

// IEEE binary32 -> binary16, round to nearest even (overflow -> inf, NaN kept quiet).
uint16_t f32_to_f16_rne(float f) {
    uint32_t x;
    std::memcpy(&x, &f, 4);
    const uint32_t sign = (x >> 16) & 0x8000u;
    const uint32_t absx = x & 0x7fffffffu;
    if (absx >= 0x7f800000u) {  // inf / NaN
        return (uint16_t)(sign | 0x7c00u | (absx > 0x7f800000u ? (0x200u | ((absx >> 13) & 0x3ffu)) : 0));
    }
    const int32_t exp = (int32_t)(absx >> 23) - 127;
    if (exp > 15) return (uint16_t)(sign | 0x7c00u);  // too large even before rounding
    uint32_t mant = absx & 0x7fffffu;
    if (exp >= -14) {
        // normal half candidate: keep 10 mantissa bits, round on the 13 dropped
        uint32_t half = ((uint32_t)(exp + 15) << 10) | (mant >> 13);
        const uint32_t rem = mant & 0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && (half & 1u))) ++half;  // carry may reach inf: correct
        return (uint16_t)(sign | half);
    }
    if (exp < -25) return (uint16_t)sign;  // below half of the smallest subnormal
    // subnormal half: value = mant24 * 2^(exp-23); unit = 2^-24
    mant |= 0x800000u;
    const int shift = -exp - 1;  // 14..24 -> bits dropped from the 24-bit significand: shift
    const uint32_t q = mant >> shift;
    const uint32_t rem = mant & ((1u << shift) - 1u);
    const uint32_t halfway = 1u << (shift - 1);
    uint32_t half = q;
    if (rem > halfway || (rem == halfway && (half & 1u))) ++half;
    return (uint16_t)(sign | half);
}

float f16_to_f32(uint16_t h) {
    const uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    const uint32_t exp = (h >> 10) & 0x1fu;
    uint32_t mant = h & 0x3ffu;
    uint32_t out;
    if (exp == 0) {
        if (mant == 0) {
            out = sign;
        } else {  // subnormal: normalise
            int e = -1;
            do {
                ++e;
                mant <<= 1;
            } while (!(mant & 0x400u));
            out = sign | ((uint32_t)(127 - 15 - e) << 23) | ((mant & 0x3ffu) << 13);
        }
    } else if (exp == 31) {
        out = sign | 0x7f800000u | (mant << 13);
    } else {
        out = sign | ((exp + 112u) << 23) | (mant << 13);
    }
    float f;
    std::memcpy(&f, &out, 4);
    return f;
}

// Pads a segment of a nonzero stream (its entries start at `first`) to a multiple of `unroll`
// with zero-valued entries that REPEAT the address word of the segment's last real entry: a
// padding entry then multiplies 0 with an activation the row reads anyway, never with one the
// definition of the layer does not touch (which could be Inf or NaN: 0 * Inf is NaN).
static void pad_segment(std::vector<uint2>& nz, size_t first, int unroll) {
    const uint32_t where = nz.size() > first ? nz.back().y : 0u;
    while (nz.size() % (size_t)unroll) nz.push_back(make_uint2(0u, where));
}

// Builds the device copy of the nonzero stream for one tile-kernel variant.
//
// Layout: packed rows are padded up to a multiple of the variant's rows-per-workgroup.
// For packed row i and channel chunk c, seg_ptr[i*(nchunks+1) + c .. + c+1] delimits that
// row's nonzeros whose input channel lies in [c*cch, (c+1)*cch); every segment is padded
// with zero-valued pairs to a multiple of `unroll` entries so the kernel can fetch
// fixed-size groups (see pad_segment).  Each entry is (fp32 value bits, byte offset of the tap inside the
// staged tile for output pixel (0,0) of the tile).
static cadnn_status build_tile_plan(const cadnn_weights* w, const ConvVariant* v, ConvPlan* plan) {
    const int g = v->nw * v->rpw;
    const int rows_padded = (w->cout + g - 1) / g * g;
    const int nchunks = (w->cin + v->cch - 1) / v->cch;
    const int taps = w->kh * w->kw;
    std::vector<int32_t> seg((size_t)rows_padded * (nchunks + 1), 0);
    std::vector<int32_t> perm(rows_padded, -1);
    std::vector<uint2> nz;
    nz.reserve((size_t)w->nnz + (size_t)rows_padded * nchunks * (v->unroll - 1) / 2 + 16);
    for (int i = 0; i < rows_padded; ++i) {
        if (i < w->cout) perm[i] = w->perm[i];
        int32_t cur = i < w->cout ? w->row_ptr[i] : 0;
        const int32_t end = i < w->cout ? w->row_ptr[i + 1] : 0;
        for (int c = 0; c < nchunks; ++c) {
            seg[(size_t)i * (nchunks + 1) + c] = (int32_t)nz.size();
            const size_t seg_first = nz.size();
            const int32_t k_end = (int32_t)std::min<int64_t>((int64_t)(c + 1) * v->cch, w->cin) * taps;
            while (cur < end && w->col_idx[cur] < k_end) {
                const int32_t k = w->col_idx[cur];
                const int ci = k / taps - c * v->cch;
                const int r = (k % taps) / w->kw;
                const int q = k % w->kw;
                const int lrow = (r % v->stride) * v->rh + r / v->stride;
                const int lcol = (q % v->stride) * v->cw + q / v->stride;
                const uint32_t off = (uint32_t)((ci * v->plane + lrow * v->pitch + lcol) * v->elem_bytes);
                uint32_t bits;
                std::memcpy(&bits, &w->vals[cur], 4);
                nz.push_back(make_uint2(bits, off));
                ++cur;
            }
            pad_segment(nz, seg_first, v->unroll);
        }
        seg[(size_t)i * (nchunks + 1) + nchunks] = (int32_t)nz.size();
    }
    if (nz.size() > (size_t)INT32_MAX) return fail(CADNN_EUNSUPPORTED, "plan too large");
    const int64_t walked_entries = (int64_t)nz.size();
    plan->variant = v;
    plan->nchunks = nchunks;
    plan->rows_padded = rows_padded;
    plan->nz_padded = (int64_t)nz.size();
    plan->walked = walked_entries;
    cadnn_status st;
    if ((st = plan->nz.upload(nz.data(), nz.size() * sizeof(uint2))) != CADNN_OK) return st;
    if ((st = plan->seg_ptr.upload(seg.data(), seg.size() * 4)) != CADNN_OK) return st;
    if ((st = plan->perm.upload(perm.data(), perm.size() * 4)) != CADNN_OK) return st;
    return CADNN_OK;
}

// Device copy of the nonzero stream for a staging-free (FAM_DIRECT) variant.
//
// Packed rows are padded to a multiple of the variant's rows-per-workgroup.  A row's
// input channels are cut into KS equal slices; inside a slice the entries are regrouped
// tap-major (tap t = r*KW + c), ascending channel inside a tap.  seg_ptr[((i*KS + s)*(T+1)
// + t .. t+1] delimits the entries of packed row i, slice s, tap t; every such segment is
// padded to a multiple of `unroll` with zero-valued entries (see pad_segment).  An entry is (fp32
// value bits, input channel).
static cadnn_status build_direct_plan(const cadnn_weights* w, const ConvVariant* v, ConvPlan* plan) {
    const int g = v->rows_per_block();
    const int rows_padded = (w->cout + g - 1) / g * g;
    const int taps = w->kh * w->kw;
    const int ks = v->ks;
    const int slice = (w->cin + ks - 1) / ks;
    std::vector<int32_t> seg((size_t)rows_padded * ks * (taps + 1), 0);
    std::vector<int32_t> perm(rows_padded, -1);
    std::vector<uint2> nz;
    nz.reserve((size_t)w->nnz + (size_t)w->cout * ks * taps * (v->unroll - 1) / 2 + 16);
    std::vector<std::vector<uint2>> bucket((size_t)ks * taps);
    for (int i = 0; i < rows_padded; ++i) {
        for (auto& b : bucket) b.clear();
        if (i < w->cout) {
            perm[i] = w->perm[i];
            for (int32_t j = w->row_ptr[i]; j < w->row_ptr[i + 1]; ++j) {
                const int32_t k = w->col_idx[j];
                const int ci = k / taps, t = k % taps;
                uint32_t bits;
                std::memcpy(&bits, &w->vals[j], 4);
                bucket[(size_t)(ci / slice) * taps + t].push_back(make_uint2(bits, (uint32_t)ci));
            }
        }
        for (int s = 0; s < ks; ++s) {
            int32_t* sp = &seg[((size_t)i * ks + s) * (taps + 1)];
            for (int t = 0; t < taps; ++t) {
                sp[t] = (int32_t)nz.size();
                const size_t seg_first = nz.size();
                const auto& b = bucket[(size_t)s * taps + t];
                nz.insert(nz.end(), b.begin(), b.end());
                pad_segment(nz, seg_first, v->unroll);
            }
            sp[taps] = (int32_t)nz.size();
        }
    }
    if (nz.size() > (size_t)INT32_MAX) return fail(CADNN_EUNSUPPORTED, "plan too large");
    const int64_t walked_entries = (int64_t)nz.size();
    plan->variant = v;
    plan->nchunks = 1;
    plan->rows_padded = rows_padded;
    plan->nz_padded = (int64_t)nz.size();
    plan->walked = walked_entries;
    cadnn_status st;
    if ((st = plan->nz.upload(nz.data(), nz.size() * sizeof(uint2))) != CADNN_OK) return st;
    if ((st = plan->seg_ptr.upload(seg.data(), seg.size() * 4)) != CADNN_OK) return st;
    if ((st = plan->perm.upload(perm.data(), perm.size() * 4)) != CADNN_OK) return st;
    return CADNN_OK;
}

// Device copy of the nonzero stream for a linear-address (FAM_LINEAR) variant.
//
// Entries stay in canonical order.  A packed row's entries are cut into KS contiguous
// parts of (nearly) equal length, each padded to a multiple of `unroll` with zero-valued
// entries that repeat the last real entry's offset.  Part s of packed row i starts at entry (i*KS + s)*stride, where `stride` is the
// longest padded part of the layer: the start of a part is therefore computable from the
// row number alone, and its first entries can be fetched together with its header instead
// of one memory round trip after it.  The header table (stored in the plan's segment
// buffer) holds, per part, {padded length, original channel of the row (-1: padding row)}.
// An entry is (fp32 value bits, byte offset of the tap relative to tap (0,0) of channel 0
// in the input's padded layout) -- hence the dependence on the input's plane and pitch.
// 128 spare zero entries end the stream: a wave reads it 64 entries at a time, one read
// ahead.
static cadnn_status build_linear_plan(const cadnn_weights* w, const ConvVariant* v, const TensorDesc& xd,
                                      ConvPlan* plan, const ConvExtra* ex) {
    if (ex && !ex->w) ex = nullptr;      // a fused pool does not touch the plan
    if ((v->dual != 0) != (ex != nullptr)) return fail(CADNN_EINVAL, "fused shortcut and kernel variant do not match");
    // fused 1x1 shortcut: its row for original channel co, wherever its own ordering put it
    std::vector<int32_t> row2;
    if (ex) {
        if (ex->w->cout != w->cout || ex->w->kh != 1 || ex->w->kw != 1)
            return fail(CADNN_EINVAL, "fused shortcut must be a 1x1 layer with the same output channels");
        row2.assign(w->cout, 0);
        for (int i = 0; i < ex->w->cout; ++i) row2[ex->w->perm[i]] = i;
    }
    const int hw = ex ? 4 : 2;      // header words per part
    const int g = v->rows_per_block();
    const int rows_padded = (w->cout + g - 1) / g * g;
    const int taps = w->kh * w->kw;
    const int ks = v->ks;
    const int U = v->unroll;
    const int64_t esz = (int64_t)w->elem();
    // longest padded part
    int64_t stride = U;
    for (int i = 0; i < w->cout; ++i) {
        const int32_t cnt = w->row_ptr[i + 1] - w->row_ptr[i];
        const int32_t per = (cnt + ks - 1) / ks;
        int64_t len = (int64_t)(per + U - 1) / U * U;
        if (ex) {
            const int i2 = row2[w->perm[i]];
            const int32_t per2 = (ex->w->row_ptr[i2 + 1] - ex->w->row_ptr[i2] + ks - 1) / ks;
            len += (int64_t)(per2 + U - 1) / U * U;
        }
        stride = std::max<int64_t>(stride, len);
    }
    const int64_t total = (int64_t)rows_padded * ks * stride + 128;
    if (total > (int64_t)INT32_MAX / 2) return fail(CADNN_EUNSUPPORTED, "plan too large");
    std::vector<int32_t> hdr((size_t)rows_padded * ks * hw, 0);
    std::vector<int32_t> perm(rows_padded, -1);
    // (four rows per wave are walked in lock step, the shorter ones into the unused end of their
    // part: there an entry must not touch memory)
    std::vector<uint2> nz((size_t)total, make_uint2(0u, v->quad ? kPlanOutOfRange : 0u));
    int64_t walked_entries = 0;
    for (int i = 0; i < rows_padded; ++i) {
        const int32_t b = i < w->cout ? w->row_ptr[i] : 0;
        const int32_t e = i < w->cout ? w->row_ptr[i + 1] : 0;
        if (i < w->cout) perm[i] = w->perm[i];
        const int32_t per = (e - b + ks - 1) / ks;
        for (int s = 0; s < ks; ++s) {
            const int32_t pb = (int32_t)std::min<int64_t>((int64_t)b + (int64_t)s * per, e);
            const int32_t pe = (int32_t)std::min<int64_t>((int64_t)pb + per, e);
            uint2* out = &nz[((size_t)i * ks + s) * (size_t)stride];
            for (int32_t j = pb; j < pe; ++j) {
                const int32_t k = w->col_idx[j];
                const int ci = k / taps, r = (k % taps) / w->kw, c = k % w->kw;
                // de-interleaved input (stride-2 layers): the tap picks the phase
                const int64_t tap = xd.s2d ? (int64_t)((r & 1) * 2 + (c & 1)) * xd.sub + (int64_t)(r >> 1) * xd.pitch + (c >> 1)
                                           : (int64_t)r * xd.pitch + c;
                const int64_t off = ((int64_t)ci * xd.plane + tap) * esz;
                uint32_t bits;
                std::memcpy(&bits, &w->vals[j], 4);
                out[j - pb] = make_uint2(bits, (uint32_t)off);
            }
            const int32_t len1 = (pe - pb + U - 1) / U * U;
            walked_entries += len1;
            // (padding repeats the last real entry's offset with a zero weight: see pad_segment)
            for (int32_t j = pe - pb; j < len1 && pe > pb; ++j) out[j] = make_uint2(0u, out[pe - pb - 1].y);
            hdr[((size_t)i * ks + s) * hw + 0] = len1;
            hdr[((size_t)i * ks + s) * hw + 1] = perm[i];
            if (ex && i < w->cout) {
                // the shortcut's slice follows the layer's own (padded) slice
                const int i2 = row2[w->perm[i]];
                const int32_t b2 = ex->w->row_ptr[i2], e2 = ex->w->row_ptr[i2 + 1];
                const int32_t per2 = (e2 - b2 + ks - 1) / ks;
                const int32_t qb = (int32_t)std::min<int64_t>((int64_t)b2 + (int64_t)s * per2, e2);
                const int32_t qe = (int32_t)std::min<int64_t>((int64_t)qb + per2, e2);
                for (int32_t j = qb; j < qe; ++j) {
                    const int64_t off = (int64_t)ex->w->col_idx[j] * ex->xd.plane * esz;   // 1x1: column = channel
                    uint32_t bits;
                    std::memcpy(&bits, &ex->w->vals[j], 4);
                    out[len1 + (j - qb)] = make_uint2(bits, (uint32_t)off);
                }
                const int32_t len2 = (qe - qb + U - 1) / U * U;
                for (int32_t j = qe - qb; j < len2 && qe > qb; ++j) out[len1 + j] = make_uint2(0u, out[len1 + qe - qb - 1].y);
                hdr[((size_t)i * ks + s) * hw + 2] = len2;
                walked_entries += len2;
            }
        }
    }
    plan->variant = v;
    plan->nchunks = (int)stride;
    plan->rows_padded = rows_padded;
    plan->nz_padded = (int64_t)nz.size();
    plan->walked = walked_entries;
    cadnn_status st;
    if ((st = plan->nz.upload(nz.data(), nz.size() * sizeof(uint2))) != CADNN_OK) return st;
    if ((st = plan->seg_ptr.upload(hdr.data(), hdr.size() * 4)) != CADNN_OK) return st;
    if ((st = plan->perm.upload(perm.data(), perm.size() * 4)) != CADNN_OK) return st;
    return CADNN_OK;
}

// Geometry of the staged tile of a FAM_PTILE variant for one layer (see PtileGeom).
PtileGeom ptile_geom(const ConvVariant& v, int cin, int kh, int kw, int stride, int pad, int wout) {
    PtileGeom g{};
    g.S = stride;
    g.P = v.p;
    const bool wide = v.tw == 16;
    g.tile_h = wide ? 4 * v.p : 7;
    g.tile_w = wide ? 14 : 7 * v.p;
    g.in_rows = (g.tile_h - 1) * stride + kh;
    g.in_cols = (g.tile_w - 1) * stride + kw;
    g.nphr = std::min(stride, kh);
    g.nphc = std::min(stride, kw);
    const int ph_r = (g.in_rows + stride - 1) / stride;
    const int ph_c = (g.in_cols + stride - 1) / stride;
    g.alias = (!wide && stride == 1 && kh == 3 && kw == 3 && pad == 1 && wout == 7 * v.p) ? 1 : 0;
    // the wide arrangement has its pitch compiled in (16); a region that does not fit makes
    // the plane larger than LDS below, which excludes the variant
    g.pitch = wide ? (ph_c <= 16 ? 16 : (1 << 20)) : (g.alias ? ph_c - 1 : ph_c);
    g.sub = ph_r * g.pitch;
    g.plane = g.nphr * g.nphc * g.sub + g.alias;
    g.nstp = (g.plane + 63) / 64;
    const size_t red_bytes = (size_t)v.nw * v.rpw * v.p * 64 * 4;
    const size_t plane_bytes = (size_t)g.plane * 4;
    if ((size_t)cin * plane_bytes <= kLdsBytesPerCU) {
        g.nbuf = 1; g.nchunks = 1; g.cch = cin;
    } else {
        // several chunks: fp32 stages chunk c+1 into a second buffer while chunk c is consumed
        g.nbuf = v.is_f16 ? 1 : 2;
        const int cch_max = (int)std::max<size_t>(1, kLdsBytesPerCU / g.nbuf / plane_bytes);
        g.nchunks = (cin + cch_max - 1) / cch_max;
        g.cch = (cin + g.nchunks - 1) / g.nchunks;
    }
    g.lds_bytes = std::max((size_t)g.nbuf * g.cch * plane_bytes, red_bytes);
    return g;
}

// Device copy of the nonzero stream for a shared-tile (FAM_PTILE) variant.
//
// The input channels are cut into `nchunks` chunks of `cch`.  A wave serves RPW packed rows
// and the `s`-th of KS even slices of each row's entries per chunk.  All its parts -- chunk
// by chunk, row by row within a chunk, each padded to the unroll -- lie back to back in one
// stream; stream w starts at w * stride entries (`stride` = the longest stream), w =
// (row / RPW) * KS + s, and the table holds the padded part lengths [w][chunk][row].  An
// entry is (fp32 value bits, byte offset of the tap in the staged chunk relative to the
// lane's pixel).  192 spare entries follow the last stream (the kernel reads two 64-entry
// windows ahead).
static cadnn_status build_ptile_plan(const cadnn_weights* w, const ConvVariant* v, int conv_stride, int pad,
                                     int wout, ConvPlan* plan) {
    const PtileGeom g = ptile_geom(*v, w->cin, w->kh, w->kw, conv_stride, pad, wout);
    const int rb = v->rows_per_block();
    const int rows_padded = (w->cout + rb - 1) / rb * rb;
    const int taps = w->kh * w->kw;
    const int ks = v->ks, rpw = v->rpw;
    const int U = v->unroll;
    const int nstreams = rows_padded / rpw * ks;
    // chunk boundaries of every row in the canonical stream
    std::vector<int32_t> cut((size_t)rows_padded * (g.nchunks + 1), 0);
    for (int i = 0; i < w->cout; ++i) {
        int32_t j = w->row_ptr[i];
        const int32_t e = w->row_ptr[i + 1];
        for (int c = 0; c < g.nchunks; ++c) {
            cut[(size_t)i * (g.nchunks + 1) + c] = j;
            const int32_t k_end = (int32_t)std::min<int64_t>((int64_t)(c + 1) * g.cch, w->cin) * taps;
            while (j < e && w->col_idx[j] < k_end) ++j;
        }
        cut[(size_t)i * (g.nchunks + 1) + g.nchunks] = e;
    }
    auto part_range = [&](int row, int c, int s, int32_t* pb, int32_t* pe) {
        const int32_t b = cut[(size_t)row * (g.nchunks + 1) + c], e = cut[(size_t)row * (g.nchunks + 1) + c + 1];
        const int32_t per = (e - b + ks - 1) / ks;
        *pb = (int32_t)std::min<int64_t>((int64_t)b + (int64_t)s * per, e);
        *pe = (int32_t)std::min<int64_t>((int64_t)*pb + per, e);
    };
    std::vector<int32_t> lens((size_t)nstreams * g.nchunks * rpw, 0);
    int64_t stride = U;
    for (int ws = 0; ws < nstreams; ++ws) {
        const int row0 = (ws / ks) * rpw, s = ws % ks;
        int64_t total = 0;
        for (int c = 0; c < g.nchunks; ++c)
            for (int r = 0; r < rpw; ++r) {
                int32_t pb, pe;
                part_range(row0 + r, c, s, &pb, &pe);
                const int32_t padded = (pe - pb + U - 1) / U * U;
                lens[((size_t)ws * g.nchunks + c) * rpw + r] = padded;
                total += padded;
            }
        stride = std::max(stride, total);
    }
    const int64_t total = (int64_t)nstreams * stride + 192;
    if (total > (int64_t)INT32_MAX / 2) return fail(CADNN_EUNSUPPORTED, "plan too large");
    std::vector<int32_t> perm(rows_padded, -1);
    for (int i = 0; i < w->cout; ++i) perm[i] = w->perm[i];
    std::vector<uint2> nz((size_t)total, make_uint2(0u, 0u));
    int64_t walked_entries = 0;
    for (int32_t l : lens) walked_entries += l;
    for (int ws = 0; ws < nstreams; ++ws) {
        const int row0 = (ws / ks) * rpw, s = ws % ks;
        uint2* out = &nz[(size_t)ws * (size_t)stride];
        for (int c = 0; c < g.nchunks; ++c)
            for (int r = 0; r < rpw; ++r) {
                int32_t pb, pe;
                part_range(row0 + r, c, s, &pb, &pe);
                for (int32_t j = pb; j < pe; ++j) {
                    const int32_t k = w->col_idx[j];
                    const int ci = k / taps - c * g.cch, tr = (k % taps) / w->kw, tc = k % w->kw;
                    const int phase = (tr % g.S) * g.nphc + (tc % g.S);
                    const int64_t off = ((int64_t)ci * g.plane + (int64_t)phase * g.sub + (tr / g.S) * g.pitch + tc / g.S) * 4;
                    uint32_t bits;
                    std::memcpy(&bits, &w->vals[j], 4);
                    out[j - pb] = make_uint2(bits, (uint32_t)off);
                }
                const int32_t padded = lens[((size_t)ws * g.nchunks + c) * rpw + r];
                for (int32_t j = pe - pb; j < padded && pe > pb; ++j) out[j] = make_uint2(0u, out[pe - pb - 1].y);
                out += padded;
            }
    }
    plan->variant = v;
    plan->nchunks = (int)stride;
    plan->rows_padded = rows_padded;
    plan->nz_padded = (int64_t)nz.size();
    plan->walked = walked_entries;
    cadnn_status st;
    if ((st = plan->nz.upload(nz.data(), nz.size() * sizeof(uint2))) != CADNN_OK) return st;
    if ((st = plan->seg_ptr.upload(lens.data(), lens.size() * 4)) != CADNN_OK) return st;
    if ((st = plan->perm.upload(perm.data(), perm.size() * 4)) != CADNN_OK) return st;
    return CADNN_OK;
}

// Geometry of the staged tile of a FAM_WTILE variant for one layer (see WtileGeom).
WtileGeom wtile_geom(const ConvVariant& v, int cin, int kh, int kw, int stride) {
    WtileGeom g{};
    g.flat = v.flat;
    g.S = stride;
    g.P = v.p;
    if (g.flat) {
        g.lr = 64; g.lc = 1;
        g.tile_h = 1; g.tile_w = 64 * g.P;
        g.nphr = g.nphc = 1;
        g.ph_rows = 1;
        g.ns = g.nsp = 64;
        g.pitch = g.sub = g.plane = 64 * g.P;
    } else {
        g.lr = v.rw; g.lc = 64 / v.rw;
        g.tile_h = g.lr; g.tile_w = g.lc * g.P;
        g.nphr = std::min(stride, kh);
        g.nphc = std::min(stride, kw);
        g.ph_rows = g.lr + (kh - 1) / stride;
        g.ns = g.lc + (kw - 1) / stride;
        // 16 consecutive lanes are min(lr, 16) rows x 16 / min(lr, 16) columns of the lane grid and
        // read slots (row * nsp + column + tap): they fall into 16 different 16-byte bank groups
        // when nsp is an odd multiple of 16 / min(lr, 16), modulo 16
        const int rows16 = std::min(g.lr, 16);
        const int unit = 16 / rows16;
        g.nsp = g.ns;
        while (g.nsp % (2 * unit) != unit % (2 * unit)) ++g.nsp;
        g.pitch = g.nsp * g.P;
        g.sub = g.ph_rows * g.pitch;
        g.plane = g.nphr * g.nphc * g.sub;
    }
    g.nstp = (g.plane + 63) / 64;
    const size_t plane_bytes = (size_t)g.plane * 4;
    const size_t budget = wtile_lds_budget(v);
    if ((size_t)cin * plane_bytes <= budget) {
        g.nbuf = 1; g.nchunks = 1; g.cch = cin;
    } else {
        // several chunks: chunk c+1 is staged into a second buffer while chunk c is consumed
        g.nbuf = 2;
        const int cch_max = (int)std::max<size_t>(1, budget / g.nbuf / plane_bytes);
        g.nchunks = (cin + cch_max - 1) / cch_max;
        g.cch = (cin + g.nchunks - 1) / g.nchunks;
    }
    g.lds_bytes = (size_t)g.nbuf * g.cch * plane_bytes;
    return g;
}

// Packed row number r of wave stream ws: the rows of a workgroup (nw * rpw consecutive packed
// rows, sorted by length) are dealt out to its waves round robin.
static inline size_t wtile_row(int ws, int r, int nw, int rpw) {
    return (size_t)(ws / nw) * (size_t)(nw * rpw) + (size_t)(ws % nw) + (size_t)nw * r;
}

// Host form of the nonzero stream of a FAM_WTILE variant (see build_wtile_plan).
struct WtileStream {
    WtileGeom g;
    int rows_padded = 0, nstreams = 0;
    int64_t stride = 0, total = 0;            // entries per wave stream, entries in all (spare blocks included)
    std::vector<int32_t> lens;                // [stream][chunk][row of the wave] padded part lengths
    std::vector<int32_t> perm;
    std::vector<uint32_t> vals;               // fp32 storage: value bits; fp16 storage: value | offset << 16
    std::vector<uint16_t> offs;               // fp32 storage only
};

// The input channels are cut into `nchunks` chunks of `cch`.  A wave serves RPW packed rows
// (wtile_row); its
// parts -- chunk by chunk, row by row within a chunk, each padded to 4 entries with zero-valued
// entries that repeat the last real entry's offset -- lie back to back in one stream; stream w
// starts at w * stride entries, stride = the longest stream rounded up to a block of 16, and
// the table holds the padded part lengths [w][chunk][row].  An entry is the value and the
// position of its tap in the staged chunk in units of 16 bytes (16 bits): two arrays in fp32
// storage (6 bytes per entry), one word holding the binary16 value and the offset in fp16
// storage (4 bytes).  Five spare blocks end the arrays: a wave reads two blocks ahead.
static cadnn_status make_wtile_stream(const cadnn_weights* w, const ConvVariant* v, int conv_stride, WtileStream* out) {
    WtileStream& st = *out;
    const WtileGeom g = wtile_geom(*v, w->cin, w->kh, w->kw, conv_stride);
    st.g = g;
    const int rb = v->rows_per_block();
    const int rows_padded = (w->cout + rb - 1) / rb * rb;
    const int taps = w->kh * w->kw;
    const int rpw = v->rpw;
    const int nstreams = rows_padded / rpw;
    const bool half = w->dtype == CADNN_F16;
    st.rows_padded = rows_padded;
    st.nstreams = nstreams;
    std::vector<int32_t> cut((size_t)rows_padded * (g.nchunks + 1), 0);
    for (int i = 0; i < w->cout; ++i) {
        int32_t j = w->row_ptr[i];
        const int32_t e = w->row_ptr[i + 1];
        for (int c = 0; c < g.nchunks; ++c) {
            cut[(size_t)i * (g.nchunks + 1) + c] = j;
            const int32_t k_end = (int32_t)std::min<int64_t>((int64_t)(c + 1) * g.cch, w->cin) * taps;
            while (j < e && w->col_idx[j] < k_end) ++j;
        }
        cut[(size_t)i * (g.nchunks + 1) + g.nchunks] = e;
    }
    st.lens.assign((size_t)nstreams * g.nchunks * rpw, 0);
    int64_t stride = 16;
    for (int ws = 0; ws < nstreams; ++ws) {
        int64_t total = 0;
        for (int c = 0; c < g.nchunks; ++c)
            for (int r = 0; r < rpw; ++r) {
                const size_t row = wtile_row(ws, r, v->nw, rpw);
                const int32_t cnt = cut[row * (g.nchunks + 1) + c + 1] - cut[row * (g.nchunks + 1) + c];
                const int32_t padded = (cnt + 3) / 4 * 4;
                st.lens[((size_t)ws * g.nchunks + c) * rpw + r] = padded;
                total += padded;
            }
        stride = std::max(stride, (total + 15) / 16 * 16);
    }
    const int64_t total = (int64_t)nstreams * stride + 80;
    if (total > (int64_t)INT32_MAX / 2) return fail(CADNN_EUNSUPPORTED, "plan too large");
    st.stride = stride;
    st.total = total;
    st.perm.assign(rows_padded, -1);
    for (int i = 0; i < w->cout; ++i) st.perm[i] = w->perm[i];
    st.vals.assign((size_t)total, 0u);
    if (!half) st.offs.assign((size_t)total, 0);
    for (int ws = 0; ws < nstreams; ++ws) {
        size_t o = (size_t)ws * (size_t)stride;
        for (int c = 0; c < g.nchunks; ++c)
            for (int r = 0; r < rpw; ++r) {
                const size_t row = wtile_row(ws, r, v->nw, rpw);
                const int32_t pb = cut[row * (g.nchunks + 1) + c], pe = cut[row * (g.nchunks + 1) + c + 1];
                const int32_t padded = st.lens[((size_t)ws * g.nchunks + c) * rpw + r];
                uint32_t last_off = 0;
                for (int32_t j = pb; j < pb + padded; ++j, ++o) {
                    uint32_t bits = 0, hbits = 0;
                    if (j < pe) {
                        const int32_t k = w->col_idx[j];
                        const int ci = k / taps - c * g.cch, tr = (k % taps) / w->kw, tc = k % w->kw;
                        const int64_t word = g.flat ? (int64_t)ci * g.plane
                                                    : (int64_t)ci * g.plane + (int64_t)((tr % g.S) * g.nphc + (tc % g.S)) * g.sub +
                                                          (int64_t)(tr / g.S) * g.pitch + (int64_t)(tc / g.S) * g.P;
                        if (word % 4 != 0 || word / 4 > 0xffff) return fail(CADNN_EUNSUPPORTED, "tile offset does not fit 16 bits");
                        last_off = (uint32_t)(word / 4);
                        std::memcpy(&bits, &w->vals[j], 4);
                        if (half) hbits = w->vals16[j];
                    }
                    if (half) {
                        st.vals[o] = hbits | (last_off << 16);
                    } else {
                        st.vals[o] = bits;
                        st.offs[o] = (uint16_t)last_off;
                    }
                }
            }
    }
    return CADNN_OK;
}

static cadnn_status build_wtile_plan(const cadnn_weights* w, const ConvVariant* v, int conv_stride, ConvPlan* plan) {
    WtileStream st;
    cadnn_status rc = make_wtile_stream(w, v, conv_stride, &st);
    if (rc != CADNN_OK) return rc;
    plan->variant = v;
    plan->nchunks = (int)st.stride;
    plan->rows_padded = st.rows_padded;
    plan->nz_padded = st.total;
    plan->walked = 0;
    for (int32_t l : st.lens) plan->walked += l;
    plan->entry_bytes = w->dtype == CADNN_F16 ? 4 : 6;
    if ((rc = plan->nz.upload(st.vals.data(), st.vals.size() * 4)) != CADNN_OK) return rc;
    if ((rc = plan->nz_off.upload(st.offs.data(), st.offs.size() * 2)) != CADNN_OK) return rc;
    if ((rc = plan->seg_ptr.upload(st.lens.data(), st.lens.size() * 4)) != CADNN_OK) return rc;
    if ((rc = plan->perm.upload(st.perm.data(), st.perm.size() * 4)) != CADNN_OK) return rc;
    return CADNN_OK;
}

bool stile_streams_fit(const cadnn_weights* w, const ConvVariant* v) {
    const int G = v->rpw, taps = w->kh * w->kw, U = v->unroll;
    const int nchunks = (w->cin + v->cch - 1) / v->cch;
    // a dense layer's stream is the longest possible one
    const int64_t dense_row = ((int64_t)std::min(w->cin, v->cch) * taps + U - 1) / U * U;
    if (dense_row * G <= v->nz_cap) return true;
    std::lock_guard<std::mutex> lock(w->stile_mu);
    auto it = w->stile_ok.find(v);
    if (it != w->stile_ok.end()) return it->second;
    bool ok = true;
    std::vector<int64_t> len(nchunks);
    for (int g0 = 0; g0 < w->cout && ok; g0 += G) {
        std::fill(len.begin(), len.end(), 0);
        for (int i = g0; i < std::min(g0 + G, w->cout); ++i) {
            int c = 0;
            int64_t run = 0;
            for (int32_t j = w->row_ptr[i]; j < w->row_ptr[i + 1]; ++j) {
                const int cj = (w->col_idx[j] / taps) / v->cch;
                if (cj != c) {
                    len[c] += (run + U - 1) / U * U;
                    run = 0;
                    c = cj;
                }
                ++run;
            }
            len[c] += (run + U - 1) / U * U;
        }
        for (int c = 0; c < nchunks; ++c) ok = ok && len[c] <= v->nz_cap;
    }
    w->stile_ok[v] = ok;
    return ok;
}

// Device copy of the nonzero stream for a wave-sliced tile (FAM_STILE) variant.
//
// Packed rows are taken G at a time (G = rows per workgroup).  For group g and channel
// chunk c the entries of the G rows whose channel lies in the chunk are laid out row after
// row, each row's run padded to a multiple of `unroll` with zero-valued entries (see pad_segment);
// seg_ptr[(g*nchunks + c)*(G+1) + r .. + 1] delimits row r's run.  An entry is (fp32 value
// bits, byte offset of the tap inside the wave's staged slice for pixel (0,0) of the tile).
// A (group, chunk) stream longer than the kernel's buffer makes the variant unusable for
// these weights (CADNN_EUNSUPPORTED).
static cadnn_status build_stile_plan(const cadnn_weights* w, const ConvVariant* v, ConvPlan* plan) {
    const int G = v->rpw;
    const int rows_padded = (w->cout + G - 1) / G * G;
    const int ngroups = rows_padded / G;
    const int nchunks = (w->cin + v->cch - 1) / v->cch;
    const int taps = w->kh * w->kw;
    std::vector<int32_t> seg((size_t)ngroups * nchunks * (G + 1), 0);
    std::vector<int32_t> perm(rows_padded, -1);
    std::vector<uint2> nz;
    nz.reserve((size_t)w->nnz + (size_t)rows_padded * nchunks + 16);
    std::vector<int32_t> cur(G), end(G);
    for (int g = 0; g < ngroups; ++g) {
        for (int r = 0; r < G; ++r) {
            const int i = g * G + r;
            if (i < w->cout) perm[i] = w->perm[i];
            cur[r] = i < w->cout ? w->row_ptr[i] : 0;
            end[r] = i < w->cout ? w->row_ptr[i + 1] : 0;
        }
        for (int c = 0; c < nchunks; ++c) {
            int32_t* sp = &seg[((size_t)g * nchunks + c) * (G + 1)];
            const size_t start = nz.size();
            const int32_t k_end = (int32_t)std::min<int64_t>((int64_t)(c + 1) * v->cch, w->cin) * taps;
            for (int r = 0; r < G; ++r) {
                sp[r] = (int32_t)nz.size();
                const size_t seg_first = nz.size();
                while (cur[r] < end[r] && w->col_idx[cur[r]] < k_end) {
                    const int32_t k = w->col_idx[cur[r]];
                    const int ci = k / taps - c * v->cch;
                    const int tr = (k % taps) / w->kw, tc = k % w->kw;
                    const int lrow = (tr % v->stride) * v->rh + tr / v->stride;
                    const int lcol = (tc % v->stride) * v->cw + tc / v->stride;
                    const uint32_t off = (uint32_t)((ci * v->plane + lrow * v->pitch + lcol) * 4);
                    uint32_t bits;
                    std::memcpy(&bits, &w->vals[cur[r]], 4);
                    nz.push_back(make_uint2(bits, off));
                    ++cur[r];
                }
                pad_segment(nz, seg_first, v->unroll);
            }
            sp[G] = (int32_t)nz.size();
            if (nz.size() - start > (size_t)v->nz_cap)
                return fail(CADNN_EUNSUPPORTED, "%s: %zu nonzeros in one (row group, channel chunk), buffer holds %d",
                            v->name, nz.size() - start, v->nz_cap);
        }
    }
    if (nz.size() > (size_t)INT32_MAX) return fail(CADNN_EUNSUPPORTED, "plan too large");
    const int64_t walked_entries = (int64_t)nz.size();
    plan->variant = v;
    plan->nchunks = nchunks;
    plan->rows_padded = rows_padded;
    plan->nz_padded = (int64_t)nz.size();
    plan->walked = walked_entries;
    cadnn_status st;
    if ((st = plan->nz.upload(nz.data(), nz.size() * sizeof(uint2))) != CADNN_OK) return st;
    if ((st = plan->seg_ptr.upload(seg.data(), seg.size() * 4)) != CADNN_OK) return st;
    if ((st = plan->perm.upload(perm.data(), perm.size() * 4)) != CADNN_OK) return st;
    return CADNN_OK;
}

// Plan of the dense kernels: the unpacked [cout][K] matrix in the storage type; for the
// 128 x 128-tile kernel with K ordered tap-major and the rows padded with zeros to whole tiles.
static cadnn_status build_dense_plan(const cadnn_weights* w, const ConvVariant* v, ConvPlan* plan, const ConvExtra* ex) {
    if (ex && !ex->w) ex = nullptr;
    if (ex && (v->tw != 128 || ex->w->cout != w->cout || ex->w->kh != 1 || ex->w->kw != 1 || ex->w->dtype != w->dtype))
        return fail(CADNN_EINVAL, "fused shortcut and kernel variant do not match");
    // (a fused 1x1 shortcut's weights follow the layer's own in every row)
    const size_t K1 = (size_t)w->cin * w->kh * w->kw;
    const size_t K = K1 + (ex ? (size_t)ex->w->cin : 0);
    plan->variant = v;
    plan->nchunks = 1;
    plan->rows_padded = (w->cout + 63) / 64 * 64;
    plan->nz_padded = (int64_t)((size_t)w->cout * K);
    plan->walked = plan->nz_padded;
    plan->entry_bytes = (int)w->elem();
    cadnn_status st;
    if (v->tw == 128 && w->cin % 32 != 0) {
        // few input channels (a network's first layer): the canonical order k = (ci, r, c), rows
        // padded with zeros to whole 32-deep steps; the kernel walks K with a table of offsets
        if (ex) return fail(CADNN_EINVAL, "fused shortcut and kernel variant do not match");
        const size_t Kp = (K1 + 31) / 32 * 32;
        plan->rows_padded = (w->cout + 127) / 128 * 128;
        plan->nz_padded = (int64_t)((size_t)plan->rows_padded * Kp);
        plan->walked = plan->nz_padded;
        std::vector<uint16_t> dense((size_t)plan->rows_padded * Kp, 0);
        for (int i = 0; i < w->cout; ++i)
            for (int32_t j = w->row_ptr[i]; j < w->row_ptr[i + 1]; ++j)
                dense[(size_t)w->perm[i] * Kp + (size_t)w->col_idx[j]] = w->vals16[j];
        st = plan->nz.upload(dense.data(), dense.size() * 2);
    } else if (v->tw == 128) {
        const int taps = w->kh * w->kw;
        plan->rows_padded = (w->cout + 127) / 128 * 128;
        plan->nz_padded = (int64_t)((size_t)plan->rows_padded * K);
        plan->walked = plan->nz_padded;
        std::vector<uint16_t> dense((size_t)plan->rows_padded * K, 0);
        for (int i = 0; i < w->cout; ++i)
            for (int32_t j = w->row_ptr[i]; j < w->row_ptr[i + 1]; ++j) {
                const int ci = w->col_idx[j] / taps, tap = w->col_idx[j] - ci * taps;
                dense[(size_t)w->perm[i] * K + (size_t)tap * w->cin + ci] = w->vals16[j];
            }
        if (ex)
            for (int i = 0; i < ex->w->cout; ++i)
                for (int32_t j = ex->w->row_ptr[i]; j < ex->w->row_ptr[i + 1]; ++j)
                    dense[(size_t)ex->w->perm[i] * K + K1 + (size_t)ex->w->col_idx[j]] = ex->w->vals16[j];
        st = plan->nz.upload(dense.data(), dense.size() * 2);
    } else if (w->dtype == CADNN_F16) {
        std::vector<uint16_t> dense((size_t)w->cout * K, 0);
        for (int i = 0; i < w->cout; ++i)
            for (int32_t j = w->row_ptr[i]; j < w->row_ptr[i + 1]; ++j)
                dense[(size_t)w->perm[i] * K + w->col_idx[j]] = w->vals16[j];
        st = plan->nz.upload(dense.data(), dense.size() * 2);
    } else {
        std::vector<float> dense((size_t)w->cout * K, 0.0f);
        for (int i = 0; i < w->cout; ++i)
            for (int32_t j = w->row_ptr[i]; j < w->row_ptr[i + 1]; ++j)
                dense[(size_t)w->perm[i] * K + w->col_idx[j]] = w->vals[j];
        st = plan->nz.upload(dense.data(), dense.size() * 4);
    }
    return st;
}

static cadnn_status build_plan(const cadnn_weights* w, const ConvVariant* v, const TensorDesc& xd, int stride,
                               int pad, int wout, ConvPlan* plan, const ConvExtra* ex) {
    if (ex && v->family != FAM_LINEAR && !(v->family == FAM_DENSE && v->tw == 128 && ex->w && !ex->pool_y && !ex->dw))
        return fail(CADNN_EINVAL, "a fused shortcut or pool needs a linear-address kernel");
    switch (v->family) {
        case FAM_PTILE: return build_ptile_plan(w, v, stride, pad, wout, plan);
        case FAM_WTILE: return build_wtile_plan(w, v, stride, plan);
        case FAM_DENSE: return build_dense_plan(w, v, plan, ex);
        case FAM_STILE: return build_stile_plan(w, v, plan);
        case FAM_DIRECT: return build_direct_plan(w, v, plan);
        case FAM_LINEAR: return build_linear_plan(w, v, xd, plan, ex);
        default: return build_tile_plan(w, v, plan);
    }
}

cadnn_status build_host_plan(const cadnn_weights* w, const ConvVariant* v, const TensorDesc& xd, int stride,
                             int pad, int wout, ConvPlan* plan) {
    const HostPlans host;
    try {
        return build_plan(w, v, xd, stride, pad, wout, plan, nullptr);
    } catch (const std::bad_alloc&) {
        return fail(CADNN_ENOMEM, "out of host memory building a conv plan");
    }
}

// The inverse of make_wtile_stream's layout transformation: every entry's 16-bit tile offset is
// taken apart into (channel, tap) again and its value added to that position of the row (the
// zero-valued padding entries add nothing).
cadnn_status wtile_plan_unpack(const cadnn_weights* w, const ConvVariant* v, int stride, const ConvPlan& plan, float* out) {
    if (v->family != FAM_WTILE || !plan.nz.on_host) return fail(CADNN_EINVAL, "not a host-built wide-tile plan");
    const WtileGeom g = wtile_geom(*v, w->cin, w->kh, w->kw, stride);
    const int64_t K = (int64_t)w->cin * w->kh * w->kw;
    std::memset(out, 0, (size_t)w->cout * K * sizeof(float));
    const bool half = w->dtype == CADNN_F16;
    const uint32_t* vals = (const uint32_t*)plan.nz.p;
    const uint16_t* offs = (const uint16_t*)plan.nz_off.p;
    const int32_t* lens = (const int32_t*)plan.seg_ptr.p;
    const int32_t* perm = (const int32_t*)plan.perm.p;
    const int rpw = v->rpw, nstreams = plan.rows_padded / rpw;
    for (int ws = 0; ws < nstreams; ++ws) {
        size_t o = (size_t)ws * (size_t)plan.nchunks;
        for (int c = 0; c < g.nchunks; ++c)
            for (int r = 0; r < rpw; ++r) {
                const int co = perm[wtile_row(ws, r, v->nw, rpw)];
                const int32_t len = lens[((size_t)ws * g.nchunks + c) * rpw + r];
                for (int32_t j = 0; j < len; ++j, ++o) {
                    const uint32_t off16 = half ? vals[o] >> 16 : offs[o];
                    const float val = half ? f16_to_f32((uint16_t)(vals[o] & 0xffffu)) : [&] { float f; std::memcpy(&f, &vals[o], 4); return f; }();
                    if (co < 0) {
                        if (val != 0.0f) return fail(CADNN_EINVAL, "a padding row carries a value");
                        continue;
                    }
                    const int64_t word = (int64_t)off16 * 4;
                    const int ci = (int)(word / g.plane) + c * g.cch;
                    int tr = 0, tc = 0;
                    if (!g.flat) {
                        const int64_t rem = word % g.plane;
                        const int phase = (int)(rem / g.sub), q = (int)(rem % g.sub);
                        tr = (q / g.pitch) * g.S + phase / g.nphc;
                        tc = ((q % g.pitch) / g.P) * g.S + phase % g.nphc;
                        if ((q % g.pitch) % g.P != 0) return fail(CADNN_EINVAL, "an offset does not point at a slot");
                    }
                    if (ci >= w->cin || tr >= w->kh || tc >= w->kw) return fail(CADNN_EINVAL, "an offset decodes to no tap of the filter");
                    out[(int64_t)co * K + ((int64_t)ci * w->kh + tr) * w->kw + tc] += val;
                }
            }
    }
    return CADNN_OK;
}

static PlanKey plan_key(const cadnn_weights* w, const ConvVariant* v, const TensorDesc& xd, int stride, int pad,
                        int wout, const ConvExtra* ex) {
    if (v->family == FAM_LINEAR)
        return PlanKey(v, xd.plane, xd.pitch | (xd.s2d ? 1 << 30 : 0), ex ? (const void*)ex->w : nullptr,
                       (ex && ex->w) ? ex->xd.plane : 0);
    if (v->family == FAM_PTILE)
        return PlanKey(v, stride, ptile_geom(*v, w->cin, w->kh, w->kw, stride, pad, wout).alias, nullptr, 0);
    if (v->family == FAM_WTILE) return PlanKey(v, stride, 0, nullptr, 0);
    if (v->family == FAM_DENSE) return PlanKey(v, 0, 0, (ex && ex->w) ? (const void*)ex->w : nullptr, 0);
    return PlanKey(v, 0, 0, nullptr, 0);
}

static thread_local int g_trial_plans = 0;
TrialPlans::TrialPlans() { ++g_trial_plans; }
TrialPlans::~TrialPlans() { --g_trial_plans; }

// Frees the trial plans of a tuning pass: every plan that was never handed out for an ordinary
// launch and whose variant is not pinned for some geometry of this handle.
void drop_unpinned_plans(const cadnn_weights* w) {
    std::lock_guard<std::mutex> lock(w->mu);
    for (auto it = w->plans.begin(); it != w->plans.end();) {
        bool pinned = it->second->in_use;
        for (const auto& c : w->chosen) pinned = pinned || c.second == std::get<0>(it->first);
        if (pinned) ++it; else it = w->plans.erase(it);
    }
    for (auto it = w->sk_scratch.begin(); it != w->sk_scratch.end();) {
        bool pinned = it->second->in_use;
        auto c = w->chosen.find(it->first.second);
        pinned = pinned || (c != w->chosen.end() && c->second == it->first.first);
        if (pinned) ++it; else it = w->sk_scratch.erase(it);
    }
}

cadnn_status get_sk_scratch(const cadnn_weights* w, const ConvVariant* v, const GeomKey& key, size_t part_bytes,
                            size_t count_bytes, float** part, int** count) {
    std::lock_guard<std::mutex> lock(w->mu);
    const auto k = std::make_pair(v, key);
    auto it = w->sk_scratch.find(k);
    if (it == w->sk_scratch.end()) {
        std::unique_ptr<SkScratch> sc(new (std::nothrow) SkScratch());
        if (!sc) return fail(CADNN_ENOMEM, "out of host memory");
        cadnn_status st = sc->part.alloc(part_bytes, false);
        if (st == CADNN_OK) st = sc->count.alloc(count_bytes, true);
        if (st != CADNN_OK) return st;
        it = w->sk_scratch.emplace(k, std::move(sc)).first;
    }
    if (g_trial_plans == 0) it->second->in_use = true;
    *part = (float*)it->second->part.p;
    *count = (int*)it->second->count.p;
    return CADNN_OK;
}

cadnn_status get_conv_plan(const cadnn_weights* w, const ConvVariant* v, const TensorDesc& xd, int stride,
                           int pad, int wout, const ConvPlan** out, const ConvExtra* ex,
                           std::shared_ptr<ConvPlan>* keep) {
    std::lock_guard<std::mutex> lock(w->mu);
    const PlanKey key = plan_key(w, v, xd, stride, pad, wout, ex);
    auto it = w->plans.find(key);
    if (it == w->plans.end()) {
        if (g_no_device_alloc > 0)
            return fail(CADNN_EINVAL, "the device layout of '%s' for this layer was not prepared, and this call may not allocate", v->name);
        std::shared_ptr<ConvPlan> plan(new (std::nothrow) ConvPlan());
        if (!plan) return fail(CADNN_ENOMEM, "out of host memory");
        cadnn_status st;
        try {
            st = build_plan(w, v, xd, stride, pad, wout, plan.get(), ex);
        } catch (const std::bad_alloc&) {
            return fail(CADNN_ENOMEM, "out of host memory building a conv plan");
        }
        if (st != CADNN_OK) return st;
        it = w->plans.emplace(key, std::move(plan)).first;
    }
    if (g_trial_plans == 0) it->second->in_use = true;
    *out = it->second.get();
    if (keep) *keep = it->second;
    return CADNN_OK;
}

// Device copies of the canonical arrays, used by the fully connected kernel.
cadnn_status ensure_fc_device(const cadnn_weights* w) {
    std::lock_guard<std::mutex> lock(w->mu);
    if (w->fc_ready) return CADNN_OK;
    cadnn_status st;
    if ((st = w->d_row_ptr.upload(w->row_ptr.data(), w->row_ptr.size() * 4)) != CADNN_OK) return st;
    if ((st = w->d_perm.upload(w->perm.data(), w->perm.size() * 4)) != CADNN_OK) return st;
    if ((st = w->d_col.upload(w->col_idx.data(), w->col_idx.size() * 4)) != CADNN_OK) return st;
    if ((st = w->d_val.upload(w->vals.data(), w->vals.size() * 4)) != CADNN_OK) return st;
    if (w->kh == 1 && w->kw == 1 && w->cin <= 65536) {
        try {
            std::vector<int32_t> frow((size_t)w->cout + 1);
            int64_t groups = 0;
            for (int r = 0; r < w->cout; ++r) {
                frow[r] = (int32_t)groups;
                groups += (w->row_ptr[r + 1] - w->row_ptr[r] + 3) / 4;
            }
            frow[w->cout] = (int32_t)groups;
            const size_t entries = (size_t)groups * 4 + kFcTailEntries;
            std::vector<uint16_t> fcol(entries, 0);
            const bool half = w->dtype == CADNN_F16;
            std::vector<float> fval(half ? 0 : entries, 0.0f);
            std::vector<uint16_t> fval16(half ? entries : 0, 0);
            for (int r = 0; r < w->cout; ++r) {
                size_t o = (size_t)frow[r] * 4;
                for (int32_t i = w->row_ptr[r]; i < w->row_ptr[r + 1]; ++i, ++o) {
                    fcol[o] = (uint16_t)w->col_idx[i];
                    if (half) fval16[o] = w->vals16[i];
                    else fval[o] = w->vals[i];
                }
                // the zero entries that fill the row's last group repeat its last column (a
                // zero weight must not meet an activation the row does not read)
                if (w->row_ptr[r + 1] > w->row_ptr[r])
                    for (; o < (size_t)frow[r + 1] * 4; ++o) fcol[o] = fcol[o - 1];
            }
            if ((st = w->d_frow.upload(frow.data(), frow.size() * 4)) != CADNN_OK) return st;
            if ((st = w->d_fcol.upload(fcol.data(), fcol.size() * 2)) != CADNN_OK) return st;
            st = half ? w->d_fval.upload(fval16.data(), fval16.size() * 2)
                      : w->d_fval.upload(fval.data(), fval.size() * 4);
            if (st != CADNN_OK) return st;
            w->fc_compact = true;
        } catch (const std::bad_alloc&) {
            return fail(CADNN_ENOMEM, "out of host memory building the fully connected layout");
        }
    }
    w->fc_ready = true;
    return CADNN_OK;
}

cadnn_status merge_weights(const std::vector<const cadnn_weights*>& parts, cadnn_weights** out) {
    *out = nullptr;
    if (parts.empty()) return fail(CADNN_EINVAL, "merge_weights: nothing to merge");
    std::unique_ptr<cadnn_weights> m;
    try {
        m.reset(new cadnn_weights());
        m->cin = parts[0]->cin;
        m->kh = m->kw = 1;
        m->dtype = parts[0]->dtype;
        int64_t cout = 0, nnz = 0;
        for (const cadnn_weights* p : parts) {
            if (p->cin != m->cin || p->kh != 1 || p->kw != 1 || p->dtype != m->dtype)
                return fail(CADNN_EINVAL, "merge_weights: layers of different shape or type");
            cout += p->cout;
            nnz += p->nnz;
        }
        if (cout > (1 << 24) || nnz > (int64_t)INT32_MAX) return fail(CADNN_EUNSUPPORTED, "merge_weights: too large");
        m->cout = (int)cout;
        m->nnz = nnz;
        // (part, packed row) of every merged channel, then the canonical order again: rows by
        // nonzero count, descending, ties by ascending (merged) channel
        struct Src { const cadnn_weights* p; int row; int32_t count; };
        std::vector<Src> src((size_t)cout);
        int base = 0;
        for (const cadnn_weights* p : parts) {
            for (int r = 0; r < p->cout; ++r)
                src[(size_t)base + p->perm[r]] = Src{p, r, p->row_ptr[r + 1] - p->row_ptr[r]};
            base += p->cout;
        }
        m->perm.resize((size_t)cout);
        std::iota(m->perm.begin(), m->perm.end(), 0);
        std::stable_sort(m->perm.begin(), m->perm.end(),
                         [&](int32_t a, int32_t b) { return src[a].count > src[b].count; });
        m->row_ptr.assign((size_t)cout + 1, 0);
        for (int i = 0; i < m->cout; ++i) m->row_ptr[i + 1] = m->row_ptr[i] + src[m->perm[i]].count;
        m->col_idx.resize((size_t)nnz);
        m->vals.resize((size_t)nnz);
        if (m->dtype == CADNN_F16) m->vals16.resize((size_t)nnz);
        for (int i = 0; i < m->cout; ++i) {
            const Src& s = src[m->perm[i]];
            const int32_t from = s.p->row_ptr[s.row];
            std::copy_n(s.p->col_idx.begin() + from, s.count, m->col_idx.begin() + m->row_ptr[i]);
            std::copy_n(s.p->vals.begin() + from, s.count, m->vals.begin() + m->row_ptr[i]);
            if (m->dtype == CADNN_F16)
                std::copy_n(s.p->vals16.begin() + from, s.count, m->vals16.begin() + m->row_ptr[i]);
        }
    } catch (const std::bad_alloc&) {
        return fail(CADNN_ENOMEM, "merge_weights: out of host memory");
    }
    *out = m.release();
    return CADNN_OK;
}

// Depthwise filters as a dense fp32 table [cout][kh*kw] (pruned taps are zeros, which the
// kernel skips); a depthwise handle is packed from [channels][1][kh][kw], so a row's column
// index is the tap index itself.
cadnn_status ensure_dw_device(const cadnn_weights* w) {
    std::lock_guard<std::mutex> lock(w->mu);
    if (w->dw_ready) return CADNN_OK;
    try {
        const size_t kk = (size_t)w->kh * w->kw;
        std::vector<float> table((size_t)w->cout * kk, 0.0f);
        for (int r = 0; r < w->cout; ++r)
            for (int32_t i = w->row_ptr[r]; i < w->row_ptr[r + 1]; ++i)
                table[(size_t)w->perm[r] * kk + w->col_idx[i]] = w->vals[i];
        cadnn_status st = w->d_dw.upload(table.data(), table.size() * 4);
        if (st != CADNN_OK) return st;
    } catch (const std::bad_alloc&) {
        return fail(CADNN_ENOMEM, "out of host memory building the depthwise filter table");
    }
    w->dw_ready = true;
    return CADNN_OK;
}

}  // namespace cadnn

using namespace cadnn;

extern "C" const char* cadnn_last_error(void) { return g_last_error.c_str(); }

extern "C" cadnn_status cadnn_pack_weights(const float* w_host, int cout, int cin, int kh, int kw,
                                           cadnn_dtype dtype, cadnn_weights** out) {
    if (out) *out = nullptr;
    if (!w_host || !out) return fail(CADNN_EINVAL, "cadnn_pack_weights: NULL pointer");
    if (cout <= 0 || cin <= 0 || kh <= 0 || kw <= 0)
        return fail(CADNN_EINVAL, "cadnn_pack_weights: non-positive size");
    if (dtype != CADNN_F32 && dtype != CADNN_F16)
        return fail(CADNN_EINVAL, "cadnn_pack_weights: unknown dtype %d", (int)dtype);
    const int64_t K = (int64_t)cin * kh * kw;
    if (K > (1 << 24) || cout > (1 << 24))
        return fail(CADNN_EUNSUPPORTED, "cadnn_pack_weights: cin*kh*kw or cout above 2^24");
    std::unique_ptr<cadnn_weights> w;
    try {
        w.reset(new cadnn_weights());
        w->cout = cout;
        w->cin = cin;
        w->kh = kh;
        w->kw = kw;
        w->dtype = dtype;
        // pass 1: nonzero count per row
        std::vector<int32_t> counts(cout);
        int64_t nnz = 0;
        for (int r = 0; r < cout; ++r) {
            const float* row = w_host + (int64_t)r * K;
            int32_t c = 0;
            for (int64_t k = 0; k < K; ++k) c += (row[k] != 0.0f);
            counts[r] = c;
            nnz += c;
        }
        if (nnz > (int64_t)INT32_MAX) return fail(CADNN_EUNSUPPORTED, "more than 2^31-1 nonzeros");
        w->nnz = nnz;
        // rows by nonzero count, descending; ties by ascending channel
        w->perm.resize(cout);
        std::iota(w->perm.begin(), w->perm.end(), 0);
        std::stable_sort(w->perm.begin(), w->perm.end(),
                         [&](int32_t a, int32_t b) { return counts[a] > counts[b]; });
        w->row_ptr.assign(cout + 1, 0);
        for (int i = 0; i < cout; ++i) w->row_ptr[i + 1] = w->row_ptr[i] + counts[w->perm[i]];
        w->col_idx.resize((size_t)nnz);
        w->vals.resize((size_t)nnz);
        if (dtype == CADNN_F16) w->vals16.resize((size_t)nnz);
        for (int i = 0; i < cout; ++i) {
            const float* row = w_host + (int64_t)w->perm[i] * K;
            int64_t o = w->row_ptr[i];
            for (int64_t k = 0; k < K; ++k) {
                if (row[k] != 0.0f) {
                    w->col_idx[o] = (int32_t)k;
                    if (dtype == CADNN_F16) {
                        const uint16_t hbits = f32_to_f16_rne(row[k]);
                        w->vals16[o] = hbits;
                        w->vals[o] = f16_to_f32(hbits);
                    } else {
                        w->vals[o] = row[k];
                    }
                    ++o;
                }
            }
        }
    } catch (const std::bad_alloc&) {
        return fail(CADNN_ENOMEM, "cadnn_pack_weights: out of host memory");
    }
    *out = w.release();
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_free_weights(cadnn_weights* w) {
    delete w;
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_packed_nnz(const cadnn_weights* w, int64_t* nnz) {
    if (!w || !nnz) return fail(CADNN_EINVAL, "cadnn_packed_nnz: NULL pointer");
    *nnz = w->nnz;
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_packed_export(const cadnn_weights* w, int32_t* perm, int32_t* row_ptr,
                                            int32_t* col_idx, void* vals) {
    if (!w) return fail(CADNN_EINVAL, "cadnn_packed_export: NULL handle");
    if (perm) std::memcpy(perm, w->perm.data(), w->perm.size() * 4);
    if (row_ptr) std::memcpy(row_ptr, w->row_ptr.data(), w->row_ptr.size() * 4);
    if (col_idx && w->nnz) std::memcpy(col_idx, w->col_idx.data(), w->col_idx.size() * 4);
    if (vals && w->nnz) {
        if (w->dtype == CADNN_F16)
            std::memcpy(vals, w->vals16.data(), w->vals16.size() * 2);
        else
            std::memcpy(vals, w->vals.data(), w->vals.size() * 4);
    }
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_unpack_weights(const cadnn_weights* w, float* out) {
    if (!w || !out) return fail(CADNN_EINVAL, "cadnn_unpack_weights: NULL pointer");
    const int64_t K = (int64_t)w->cin * w->kh * w->kw;
    std::memset(out, 0, (size_t)w->cout * K * sizeof(float));
    for (int i = 0; i < w->cout; ++i) {
        float* row = out + (int64_t)w->perm[i] * K;
        for (int32_t j = w->row_ptr[i]; j < w->row_ptr[i + 1]; ++j) row[w->col_idx[j]] = w->vals[j];
    }
    return CADNN_OK;
}
