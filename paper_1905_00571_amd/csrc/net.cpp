// Whole-network runner: an ordered op list over numbered activation buffers, launched
// back to back on one stream (optionally as one captured HIP graph) so that a single-image
// inference (the quantity the paper's evaluation reports, Section 5) costs one submission.
#include <algorithm>
#include <cstdlib>
#include <cstring>

#include <iterator>

#include "internal.h"

using namespace cadnn;

namespace {

enum OpKind { OP_CONV, OP_FC, OP_MAXPOOL, OP_AVGPOOL, OP_DEPTHWISE, OP_AVGPOOL2D, OP_CONCAT };

struct Shape {
    int n = 0, c = 0, h = 0, w = 0;
    size_t elems() const { return (size_t)n * c * h * w; }
    bool operator==(const Shape& o) const { return n == o.n && c == o.c && h == o.h && w == o.w; }
};

// Where a tensor lives: -1 = the caller's x, -2 = the caller's y, otherwise the output of
// op `inst` inside the workspace.  Every op output has a region of its own, so a halo
// that is zeroed once stays zero (kernels only write the image proper).
struct NetOp {
    OpKind kind;
    const cadnn_weights* w = nullptr;
    const void* bias = nullptr;
    int stride = 1, pad = 0, relu = 0, k = 0;
    int src = 0, dst = 0, res = -1;          // buffer ids as given by the caller
    Shape in, out;
    int src_inst = -1, res_inst = -1;        // producing op of each input (-1 = net input)
    TensorDesc xd, yd, rd;
    size_t y_off = 0;                        // byte offset of this op's output region
    int shortcut = -1;                       // conv: the 1x1 projection op fused into this one
    int pool_op = -1;                        // conv: the global average pool op fused into this one
    int dw_op = -1;                          // conv: the depthwise op fused into this one
    int fused_into = -1;                     // projection / pool / depthwise: the op that now computes it (it is skipped)
    // concatenation: its sources (src / src_inst repeat the first), the first output channel of
    // each, and whether the source's producer writes its slice of this op's region itself
    std::vector<int> srcs, src_insts, ch_off;
    std::vector<char> in_place;
    int slice_of = -1;                       // producer: the concatenation whose region it writes into ...
    int slice_ch = 0;                        // ... starting at this channel
    // 1x1 layers that read the same tensor pixel by pixel are merged into ONE launch with the
    // rows of all of them (a horizontal fusion): the first carries the others as `siblings`
    // and writes a region with the channels of all; a sibling is skipped (fused_into = the
    // first) and its output is the channel slice [sib_ch, sib_ch + cout) of that region
    std::vector<int> siblings;
    int sibling_of = -1, sib_ch = 0, launch_c = 0;   // launch_c: channels the launch writes (own + siblings')
    // Independent layers (different inputs, different weights) whose inputs are all ready when
    // the first of them runs are launched with it as ONE kernel: the first carries the others
    // as `comates`; a comate is skipped (fused_into = colaunch_of = the first).  Its tensors are
    // its own, untouched by this.
    std::vector<int> comates;
    int colaunch_of = -1;
    // A window pool is launched right after the op that completes its input (hoisted_to; that op
    // lists it in `hoisted`) instead of at its place in the op list, so that the layer reading
    // it can join the launch of layers that come before the pool in the list.  The members of
    // a group that tuning disbanded stay behind its first op the same way.
    int hoisted_to = -1;
    std::vector<int> hoisted;
    // A large stride-2 layer with a filter wider than 1x1 whose input could not be kept
    // de-interleaved where it is produced (odd sizes, other readers, a concatenation) reads a
    // de-interleaved copy made right before it: xd describes the copy at x_off, src_d the
    // tensor it is made from.
    bool restaged = false;
    size_t x_off = 0;
    TensorDesc src_d;
};

// The one kernel of a group of co-launched layers: the variant that serves them all and the
// members' launch records in device memory (with the plans they point into).
struct CoLaunch {
    const ConvVariant* v = nullptr;
    DevBuf table;
    std::vector<std::shared_ptr<ConvPlan>> plans;
    std::vector<ConvLaunch> records;   // host copy of the table (the launch derives the grid from it)
};

// Weights, bias and output layout an op is launched with: its own, or -- first op of a sibling
// group -- the merged ones.
const cadnn_weights* eff_w(const cadnn_net* net, const NetOp& op);
const void* eff_bias(const cadnn_net* net, const NetOp& op);
TensorDesc launch_yd(const NetOp& op) {
    TensorDesc d = op.yd;
    if (!op.siblings.empty()) d.c = op.launch_c;
    return d;
}

// Every op whose output `op` reads as an activation input (not as residual).
std::vector<int> input_insts(const NetOp& op) {
    if (op.kind == OP_CONCAT) return op.src_insts;
    return std::vector<int>{op.src_inst};
}

}  // namespace

// The workspace of nets that may not allocate (cadnn_run_net_noalloc): one array per GPU, held
// by the library until the process ends and shared by every such net on that GPU.  In host
// code the array's name is only a stand-in; its device address comes from static_workspace().
constexpr size_t kStaticWorkspaceBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device).
cadnn_status static_workspace(void** ptr) {
    int dev = -1;
    CADNN_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(CADNN_EUNSUPPORTED, "device %d: more than %d devices", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        CADNN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(CADNN_EHIP, "hipGetSymbolAddress returned no address for the static workspace");
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return CADNN_OK;
}
}  // namespace

struct cadnn_net {
    cadnn_dtype dtype = CADNN_F32;
    Shape input;
    std::vector<NetOp> ops;
    std::map<int, Shape> cur;        // shape currently held by each buffer id while building
    std::map<int, int> producer;     // op that last wrote each buffer id (-1 = net input)
    size_t ws_bytes = 0;
    bool laid_out = false;
    bool finalized = false;
    bool use_graph = false;
    bool want_tune = false;
    bool allow_s2d = true;
    bool allow_fusion = true;
    char* ws = nullptr;
    bool static_ws = false;          // the workspace is the library's static array (CADNN_NET_STATIC_WORKSPACE)
    std::map<int, std::unique_ptr<cadnn_weights>> merged_w;   // per first op of a sibling group
    std::map<int, std::unique_ptr<DevBuf>> merged_bias;
    std::map<int, std::unique_ptr<CoLaunch>> colaunch;        // per first op of a group of co-launched layers
    hipGraphExec_t exec = nullptr;
    const void* cap_x = nullptr;
    void* cap_y = nullptr;
    size_t elem() const { return dtype == CADNN_F16 ? 2 : 4; }
};

namespace {

const cadnn_weights* eff_w(const cadnn_net* net, const NetOp& op) {
    if (op.siblings.empty()) return op.w;
    auto it = net->merged_w.find((int)(&op - net->ops.data()));
    return it == net->merged_w.end() ? op.w : it->second.get();
}

const void* eff_bias(const cadnn_net* net, const NetOp& op) {
    if (op.siblings.empty()) return op.bias;
    auto it = net->merged_bias.find((int)(&op - net->ops.data()));
    return it == net->merged_bias.end() ? nullptr : it->second->p;
}

// One image of a tensor, with the zero halo a reader asks for, must stay addressable with the
// kernels' 32-bit offsets (with room for the rounding of the de-interleaved layout).
bool tensor_fits(const cadnn_net* net, const Shape& s, int halo) {
    if (halo > 65535) return false;
    const TensorDesc d = make_desc(s.c, s.h, s.w, halo, halo);
    return !desc_too_large(d) && d.image * (int64_t)net->elem() < 0x70000000ll;
}

cadnn_status note_output(cadnn_net* net, int dst, const Shape& s) {
    if (dst <= 0) return fail(CADNN_EINVAL, "cadnn_net: dst buffer must be >= 1 (0 is the input)");
    if (!tensor_fits(net, s, 0)) return fail(CADNN_EUNSUPPORTED, "cadnn_net: one image of buffer %d would be 1.75 GiB or more", dst);
    net->cur[dst] = s;
    net->producer[dst] = (int)net->ops.size();
    net->laid_out = false;
    return CADNN_OK;
}

cadnn_status src_shape(cadnn_net* net, int src, Shape* s, int* inst) {
    auto it = net->cur.find(src);
    if (it == net->cur.end()) return fail(CADNN_EINVAL, "cadnn_net: buffer %d read before it is written", src);
    *s = it->second;
    *inst = net->producer[src];
    return CADNN_OK;
}

// The layout of a net: where every op's output lives, what is fused into what and what is
// launched together.  The steps run in the order below; each reads what the ones before it
// decided.
struct Layout {
    cadnn_net* net;
    const int nops;
    std::vector<int> halo;          // zero halo rows / columns around every op's output
    std::vector<bool> flat;         // output kept without halo (read by an FC layer, or the net's output)
    std::vector<int> all_readers;   // ops that read each op's output (as input or as residual)
    std::vector<int> s2d, strided;  // de-interleaved layout: allowed for / wanted by the readers of each output
    size_t off = 0;                 // bytes of workspace handed out so far

    explicit Layout(cadnn_net* n)
        : net(n), nops((int)n->ops.size()), halo(nops, 0), flat(nops, false), all_readers(nops, 0), s2d(nops, 0),
          strided(nops, 0) {}

    // (Layers dense enough for the matrix-core kernels stay on plain layouts, which is all
    // those kernels read and write.)
    static bool sparse_enough(const NetOp& o) {
        return (double)o.w->nnz < 0.25 * (double)o.w->cout * o.w->cin * o.w->kh * o.w->kw;
    }
    static bool grouped(const NetOp& o) { return o.sibling_of >= 0 || !o.siblings.empty(); }

    // The halo of every op output: the largest padding among the convolutions with filters
    // larger than 1x1 that read it; none if a fully connected layer reads it or if it is the
    // net's output.
    void choose_halos() {
        for (const NetOp& op : net->ops) {
            if (op.src_inst < 0) continue;
            if (op.kind == OP_FC) flat[op.src_inst] = true;
            if ((op.kind == OP_CONV || op.kind == OP_DEPTHWISE) && (op.w->kh > 1 || op.w->kw > 1))
                halo[op.src_inst] = std::max(halo[op.src_inst], op.pad);
        }
        if (nops) flat[nops - 1] = true;
    }

    void place_concat_slices() {
        // A source of a concatenation that nothing else reads is written by its producer straight
        // into its channel slice of the concatenation's region (not when that region is the
        // caller's output tensor, and not for a producer that is itself a concatenation).
        for (const NetOp& op : net->ops) {
            for (int i : input_insts(op)) if (i >= 0) ++all_readers[i];
            if (op.res_inst >= 0) ++all_readers[op.res_inst];
        }
        for (NetOp& op : net->ops) { op.slice_of = -1; op.slice_ch = 0; }
        for (int k = 0; k < nops; ++k) {
            NetOp& cat = net->ops[k];
            if (cat.kind != OP_CONCAT) continue;
            cat.in_place.assign(cat.src_insts.size(), 0);
            for (size_t j = 0; j < cat.src_insts.size(); ++j) {
                const int p = cat.src_insts[j];
                if (p < 0 || k == nops - 1 || all_readers[p] != 1) continue;
                NetOp& prod = net->ops[p];
                if (prod.kind != OP_CONV && prod.kind != OP_DEPTHWISE && prod.kind != OP_MAXPOOL && prod.kind != OP_AVGPOOL2D)
                    continue;
                cat.in_place[j] = 1;
                prod.slice_of = k;
                prod.slice_ch = cat.ch_off[j];
            }
        }
    }

    void merge_siblings() {
        // Sibling groups: pixel-wise (1x1, stride 1) sparse layers without residual that read the
        // same tensor and are not concatenation slices become one launch over the rows of all of
        // them (the reduce layers of an Inception module's branches).  Their outputs share one
        // region, so they share its halo: the largest any of their readers needs.
        for (NetOp& op : net->ops) { op.siblings.clear(); op.sibling_of = -1; op.sib_ch = 0; op.launch_c = op.out.c; }
        net->merged_w.clear();
        if (net->allow_fusion) {
            auto eligible = [&](int k) {
                const NetOp& o = net->ops[k];
                return o.kind == OP_CONV && o.w->kh == 1 && o.w->kw == 1 && o.stride == 1 && o.pad == 0 && o.res < 0 &&
                       o.slice_of < 0 && o.sibling_of < 0 && o.siblings.empty() && !flat[k] && k != nops - 1 && sparse_enough(o);
            };
            for (int i = 0; i < nops; ++i) {
                if (!eligible(i)) continue;
                std::vector<const cadnn_weights*> parts{net->ops[i].w};
                std::vector<int> group;
                for (int j = i + 1; j < nops; ++j) {
                    const NetOp& a = net->ops[i];
                    const NetOp& b = net->ops[j];
                    if (!eligible(j) || b.src_inst != a.src_inst || b.src != a.src || b.relu != a.relu || b.w->cin != a.w->cin ||
                        (a.bias == nullptr) != (b.bias == nullptr))
                        continue;
                    // (the shared region must stay addressable like any tensor, under any reader's halo)
                    int total_c = b.out.c, h = std::max(halo[i], halo[j]);
                    for (const cadnn_weights* p : parts) total_c += p->cout;
                    for (int g : group) h = std::max(h, halo[g]);
                    if (!tensor_fits(net, Shape{a.out.n, total_c, a.out.h, a.out.w}, h)) continue;
                    parts.push_back(b.w);
                    group.push_back(j);
                }
                if (group.empty()) continue;
                cadnn_weights* merged = nullptr;
                if (merge_weights(parts, &merged) != CADNN_OK) continue;
                net->merged_w[i].reset(merged);
                NetOp& first = net->ops[i];
                int ch = first.out.c, h = halo[i];
                for (int j : group) {
                    NetOp& sib = net->ops[j];
                    sib.sibling_of = i;
                    sib.sib_ch = ch;
                    ch += sib.out.c;
                    h = std::max(h, halo[j]);
                    first.siblings.push_back(j);
                }
                first.launch_c = ch;
                halo[i] = h;
                for (int j : group) halo[j] = h;
            }
        }
    }

    void choose_deinterleaved() {
        // De-interleaved layout for the output of a convolution whose readers are all
        // convolutions, at least one of them with stride 2: every reader must be either a
        // stride-2 layer whose taps start on an even padded position (any 1x1; larger filters
        // when halo - pad is even) or a pixel-wise stride-1 layer, and both the producer and
        // the readers must be servable by the linear-address kernels.
        for (int i = 0; i < nops; ++i) {
            const NetOp& p = net->ops[i];
            bool ok = p.kind == OP_CONV && !flat[i] && (p.out.h % 2 == 0) && (p.out.w % 2 == 0) && sparse_enough(p) &&
                      p.siblings.empty() && p.sibling_of < 0;
            if (ok) {
                const bool one = p.w->kh == 1 && p.w->kw == 1;
                const int src_halo = p.src_inst < 0 ? 0 : (flat[p.src_inst] ? 0 : halo[p.src_inst]);
                ok = one ? p.pad == 0 : src_halo >= p.pad;
            }
            s2d[i] = ok ? 1 : 0;
        }
        for (const NetOp& op : net->ops) {
            if (op.res_inst >= 0) s2d[op.res_inst] = 0;
            if (op.kind == OP_CONCAT) {
                for (int i : op.src_insts) if (i >= 0) s2d[i] = 0;
                continue;
            }
            if (op.src_inst < 0) continue;
            const int i = op.src_inst;
            if (op.kind != OP_CONV || !sparse_enough(op)) { s2d[i] = 0; continue; }
            const bool one = op.w->kh == 1 && op.w->kw == 1;
            if (op.stride == 2 && (one ? op.pad == 0 : ((halo[i] - op.pad) & 1) == 0)) strided[i] = 1;
            else if (!(op.stride == 1 && one && op.pad == 0)) s2d[i] = 0;
        }
    }

    // The regions back to back, 256-byte aligned, in op order; slices take their place inside.
    void place_regions() {
        for (int i = 0; i < nops; ++i) {
            NetOp& op = net->ops[i];
            if (op.slice_of >= 0 || op.sibling_of >= 0) continue;   // lives inside another op's region, see below
            const int hp = flat[i] ? 0 : halo[i];
            op.yd = (s2d[i] && strided[i] && net->allow_s2d) ? make_desc_s2d(op.out.c, op.out.h, op.out.w, hp, hp)
                                                            : make_desc(op.launch_c, op.out.h, op.out.w, hp, hp);
            op.yd.c = op.out.c;                      // (with siblings the region holds launch_c channels; readers see the op's own)
            op.y_off = off;
            if (i != nops - 1) off += ((size_t)op.out.n * op.yd.image * net->elem() + 255) / 256 * 256;
        }
        for (NetOp& op : net->ops) {
            if (op.sibling_of < 0) continue;
            // a channel slice of the region the first op of the group writes
            const NetOp& first = net->ops[op.sibling_of];
            op.yd = first.yd;
            op.yd.c = op.out.c;
            op.y_off = first.y_off + (size_t)op.sib_ch * first.yd.plane * net->elem();
        }
        for (NetOp& op : net->ops) {
            if (op.slice_of < 0) continue;
            // a channel slice of the concatenation's region: its planes, its halo, its image stride
            const NetOp& cat = net->ops[op.slice_of];
            op.yd = cat.yd;
            op.yd.c = op.out.c;
            op.y_off = cat.y_off + (size_t)op.slice_ch * cat.yd.plane * net->elem();
        }
        for (NetOp& op : net->ops) {
            op.xd = op.src_inst < 0 ? make_desc(op.in.c, op.in.h, op.in.w) : net->ops[op.src_inst].yd;
            if (op.res >= 0)
                op.rd = op.res_inst < 0 ? make_desc(net->input.c, net->input.h, net->input.w) : net->ops[op.res_inst].yd;
            else
                op.rd = op.yd;
        }
        // De-interleaved copies: a stride-2 lane pattern on a plain tensor touches twice the
        // cache lines per load, which is what bounds a big layer (Inception-V3's 288 -> 384
        // 3x3/2 on 35 x 35: 35 us); a copy costs one small launch.
        for (NetOp& op : net->ops) {
            op.restaged = false;
            if (!net->allow_s2d || op.kind != OP_CONV || op.stride != 2 || (op.w->kh == 1 && op.w->kw == 1) || op.src_inst < 0 ||
                op.xd.s2d || !sparse_enough(op) || (double)op.w->nnz * op.out.h * op.out.w < 4e7 ||
                !tensor_fits(net, op.in, op.pad + 1))
                continue;
            op.restaged = true;
            op.src_d = op.xd;
            op.xd = make_desc_s2d(op.in.c, op.in.h, op.in.w, op.pad, op.pad);
            op.x_off = off;
            off += ((size_t)op.in.n * op.xd.image * net->elem() + 255) / 256 * 256;
        }
    }

    void fuse() {
        // A 1x1 projection shortcut whose only reader takes it as residual is computed inside
        // that reader (a second sparse matrix on a second input, same accumulators): one launch,
        // one output write and one residual read less (paper Section 4, layer fusion).
        for (NetOp& op : net->ops) { op.shortcut = -1; op.pool_op = -1; op.dw_op = -1; op.fused_into = op.sibling_of; }
        if (net->allow_fusion) {
            const std::vector<int>& readers = all_readers;
            for (int i = 0; i < nops; ++i) {
                NetOp& c = net->ops[i];
                if (c.kind != OP_CONV || c.res_inst < 0) continue;
                NetOp& p = net->ops[c.res_inst];
                const bool c_one = c.w->kh == 1 && c.w->kw == 1;
                const bool ok = p.kind == OP_CONV && !grouped(p) && p.w->kh == 1 && p.w->kw == 1 && p.pad == 0 && !p.relu && p.res < 0 &&
                                readers[c.res_inst] == 1 && c.res_inst != nops - 1 && p.w->cout == c.w->cout &&
                                sparse_enough(c) && sparse_enough(p) && !c.yd.s2d && !(c.xd.s2d && c.stride == 1) &&
                                (c_one ? c.pad == 0 : (c.xd.ph >= c.pad && c.xd.pw >= c.pad)) &&
                                (!c.xd.s2d || c_one || (((c.xd.ph - c.pad) & 1) == 0 && ((c.xd.pw - c.pad) & 1) == 0)) &&
                                (!p.xd.s2d || p.stride == 2);
                if (ok) {
                    c.shortcut = c.res_inst;
                    p.fused_into = i;
                }
            }
            // A global average pool that is the only reader of a convolution whose image fits one
            // pixel tile is computed in that convolution's epilogue; the feature map is not written.
            for (int i = 0; i < nops; ++i) {
                NetOp& a = net->ops[i];
                if (a.kind != OP_AVGPOOL || a.src_inst < 0) continue;
                NetOp& c = net->ops[a.src_inst];
                const bool c_one = c.kind == OP_CONV && c.w->kh == 1 && c.w->kw == 1;
                // (2-byte storage, whole 32-channel steps and a batch of a thousand pixels or more:
                // the matrix-core kernels, which fuse no pool, are the likely pick for the layer --
                // about three times the fused kernel's rate there -- so the pool keeps its launch)
                const bool mfma_likely = c.kind == OP_CONV && net->dtype == CADNN_F16 && c.w->cin % 32 == 0 &&
                                         (int64_t)c.out.n * c.out.h * c.out.w >= 1024;
                const bool ok = c.kind == OP_CONV && !grouped(c) && readers[a.src_inst] == 1 && c.shortcut < 0 && c.fused_into < 0 &&
                                sparse_enough(c) && !c.yd.s2d && !c.xd.s2d && !(c.res >= 0 && c.rd.s2d) &&
                                c.out.h * c.out.w <= 256 && !mfma_likely &&
                                (c_one ? c.pad == 0 : (c.xd.ph >= c.pad && c.xd.pw >= c.pad));
                if (ok) {
                    c.pool_op = i;
                    a.fused_into = a.src_inst;
                }
            }
            // A 3x3 depthwise layer (padding 1, stride 1 or 2) that is the only reader of a
            // convolution whose image is at most 28 x 28 is computed in that convolution's
            // epilogue: a wave (images of up to 64 pixels) or the 4 or 16 waves of a workgroup hold a
            // whole channel there, which is all a depthwise filter needs.  The convolution's own
            // feature map is not written.
            for (int i = 0; i < nops; ++i) {
                NetOp& d = net->ops[i];
                if (d.kind != OP_DEPTHWISE || d.src_inst < 0) continue;
                NetOp& c = net->ops[d.src_inst];
                const bool c_one = c.kind == OP_CONV && c.w->kh == 1 && c.w->kw == 1;
                const bool ok = c.kind == OP_CONV && !grouped(c) && readers[d.src_inst] == 1 && c.shortcut < 0 && c.pool_op < 0 &&
                                c.fused_into < 0 && sparse_enough(c) && !c.yd.s2d && !c.xd.s2d && !(c.res >= 0 && c.rd.s2d) &&
                                c.out.h <= 28 && c.out.w <= 28 && d.w->kh == 3 && d.w->kw == 3 && d.pad == 1 &&
                                (d.stride == 1 || d.stride == 2) && !d.yd.s2d &&
                                (c_one ? c.pad == 0 : (c.xd.ph >= c.pad && c.xd.pw >= c.pad));
                if (ok) {
                    c.dw_op = i;
                    d.fused_into = d.src_inst;
                }
            }
        }
    }

    void share_launches() {
        // Independent layers in one launch: sparse convolutions on plain tensors with nothing fused
        // into them, none of them touching the caller's x or y, whose inputs are all produced
        // before the first of them runs (the branches of an Inception module at the same depth).
        // Launched apart each would leave most of the chip idle and pay a launch of its own;
        // together they take about as long as the slowest.  A layer joins only while one kernel
        // variant still serves the whole group.
        for (NetOp& op : net->ops) { op.comates.clear(); op.colaunch_of = -1; op.hoisted_to = -1; op.hoisted.clear(); }
        // the op at whose launch op k's output becomes available: k itself, the op that computes
        // it (a sibling's or comate's first layer, the layer a pool is fused into), or the op a
        // hoisted pool is launched behind
        std::function<int(int)> ready_at = [&](int k) {
            const NetOp& o = net->ops[k];
            return o.hoisted_to >= 0 ? ready_at(o.hoisted_to) : o.fused_into >= 0 ? ready_at(o.fused_into) : k;
        };
        if (net->allow_fusion) {
            for (int p = 0; p + 1 < nops; ++p) {
                NetOp& o = net->ops[p];
                if ((o.kind == OP_MAXPOOL || o.kind == OP_AVGPOOL2D) && o.fused_into < 0 && o.src_inst >= 0 &&
                    ready_at(o.src_inst) < p - 1)
                    o.hoisted_to = o.src_inst;
            }
            auto member_of = [&](const NetOp& o) {
                // (pointers only have to be distinct and non-NULL here: nothing is launched)
                ConvMember m{};
                m.w = eff_w(net, o); m.x = (const void*)16; m.xd = o.xd; m.y = (void*)32; m.yd = launch_yd(o);
                m.residual = o.res >= 0 ? (const void*)48 : nullptr; m.rd = o.rd;
                m.stride = o.stride; m.pad = o.pad; m.bias = eff_bias(net, o); m.relu = o.relu;
                return m;
            };
            // a window pool on workspace tensors can ride along with such a group (it takes no part
            // in the choice of the variant): the pooled branch of a module
            auto solo_pool = [&](int k) {
                const NetOp& o = net->ops[k];
                return (o.kind == OP_MAXPOOL || o.kind == OP_AVGPOOL2D) && o.fused_into < 0 && o.colaunch_of < 0 &&
                       o.src_inst >= 0 && k != nops - 1 && !o.xd.s2d && !o.yd.s2d;
            };
            auto solo = [&](int k) {
                const NetOp& o = net->ops[k];
                return o.kind == OP_CONV && o.fused_into < 0 && o.shortcut < 0 && o.pool_op < 0 && o.dw_op < 0 &&
                       o.colaunch_of < 0 && o.comates.empty() && sparse_enough(o) && !o.yd.s2d && !(o.xd.s2d && !o.restaged) &&
                       !(o.res >= 0 && o.rd.s2d) && o.src_inst >= 0 && k != nops - 1 && (o.res < 0 || o.res_inst >= 0);
            };
            // the variants that can launch op k among several layers (sorted; listed once per op)
            std::vector<std::vector<const ConvVariant*>> multi(nops);
            std::vector<char> listed(nops, 0);
            auto multi_of = [&](int k) -> const std::vector<const ConvVariant*>& {
                if (!listed[k]) {
                    listed[k] = 1;
                    if (conv2d_group_candidates({member_of(net->ops[k])}, net->ops[k].in.n, &multi[k], nullptr) != CADNN_OK)
                        multi[k].clear();
                    std::sort(multi[k].begin(), multi[k].end());
                }
                return multi[k];
            };
            for (int i = 0; i < nops; ++i) {
                if (!solo(i)) continue;
                std::vector<const ConvVariant*> common = multi_of(i), narrowed;
                // (partners are looked for among the next 64 ops: a module's branches lie close together)
                for (int j = i + 1; j < std::min(nops, i + 65) && net->ops[i].comates.size() < (size_t)kMaxCoLaunch - 1 && !common.empty(); ++j) {
                    NetOp& b = net->ops[j];
                    if (solo_pool(j) && ready_at(b.src_inst) < i) {
                        b.hoisted_to = -1;
                        net->ops[i].comates.push_back(j);
                        b.colaunch_of = i;
                        b.fused_into = i;
                        continue;
                    }
                    if (!solo(j) || ready_at(b.src_inst) >= i || (b.res >= 0 && ready_at(b.res_inst) >= i)) continue;
                    const std::vector<const ConvVariant*>& theirs = multi_of(j);
                    narrowed.clear();
                    std::set_intersection(common.begin(), common.end(), theirs.begin(), theirs.end(), std::back_inserter(narrowed));
                    if (narrowed.empty()) continue;
                    common.swap(narrowed);
                    net->ops[i].comates.push_back(j);
                    net->ops[j].colaunch_of = i;
                    net->ops[j].fused_into = i;
                }
            }
            // every hoisted pool goes behind the op that really launches when its input completes
            for (int p = 0; p < nops; ++p)
                if (net->ops[p].hoisted_to >= 0) {
                    net->ops[p].hoisted_to = ready_at(p);
                    net->ops[net->ops[p].hoisted_to].hoisted.push_back(p);
                }
        }
    }

};

void layout(cadnn_net* net) {
    Layout l(net);
    l.choose_halos();
    l.place_concat_slices();
    l.merge_siblings();
    l.choose_deinterleaved();
    l.place_regions();
    l.fuse();
    l.share_launches();
    net->ws_bytes = l.off;
    net->laid_out = true;
}

int out_s2d(const NetOp& op) {
    return (op.yd.s2d || (op.res >= 0 && op.shortcut < 0 && op.rd.s2d)) ? 1 : 0;
}

const void* in_ptr(const cadnn_net* net, int inst, const void* x) {
    return inst < 0 ? x : (const void*)(net->ws + net->ops[inst].y_off);
}

void* out_ptr(const cadnn_net* net, size_t i, void* y) {
    return i + 1 == net->ops.size() ? y : (void*)(net->ws + net->ops[i].y_off);
}

void* out_ptr(const cadnn_net* net, size_t i, void* y);

// What is fused into op (if anything): a projection shortcut, reading from the caller's x or
// the workspace, or a global average pool, writing to the pool op's own output.
bool shortcut_of(const cadnn_net* net, const NetOp& op, const void* x, ConvExtra* ex, void* y = nullptr) {
    *ex = ConvExtra{};
    if (op.shortcut >= 0) {
        const NetOp& p = net->ops[op.shortcut];
        ex->w = p.w;
        ex->x = in_ptr(net, p.src_inst, x);
        ex->xd = p.xd;
        ex->stride = p.stride;
        ex->bias = p.bias;
        return true;
    }
    if (op.pool_op >= 0) {
        ex->pool_y = y ? out_ptr(net, (size_t)op.pool_op, y) : (void*)net;   // placeholder for geometry-only calls
        return true;
    }
    if (op.dw_op >= 0) {
        const NetOp& d = net->ops[op.dw_op];
        ex->dw = d.w;
        ex->dw_bias = d.bias;
        ex->dw_stride = d.stride;
        ex->dw_relu = d.relu;
        ex->dw_yd = d.yd;
        ex->dw_y = y ? out_ptr(net, (size_t)op.dw_op, y) : (void*)net;
        return true;
    }
    return false;
}

// Same for calls that only look at the geometry (the tensor pointer is a placeholder).
const ConvExtra* shortcut_geom(const cadnn_net* net, const NetOp& op, ConvExtra* ex) {
    return shortcut_of(net, op, (const void*)net, ex) ? ex : nullptr;
}

// The layers launched together with op i (itself first), on their own tensors: all of them
// live in the workspace, none reads the caller's x or writes the caller's y.
std::vector<ConvMember> colaunch_members(const cadnn_net* net, size_t i) {
    std::vector<int> idx{(int)i};
    idx.insert(idx.end(), net->ops[i].comates.begin(), net->ops[i].comates.end());
    std::vector<ConvMember> members;
    for (int k : idx) {
        const NetOp& o = net->ops[k];
        ConvMember m{};
        if (o.kind != OP_CONV) {
            m.pool_kind = o.kind == OP_MAXPOOL ? 1 : 2;
            m.pool_k = o.k;
            m.x = net->ws + net->ops[o.src_inst].y_off; m.xd = o.xd;
            m.y = net->ws + o.y_off; m.yd = o.yd;
            m.stride = o.stride; m.pad = o.pad;
            members.push_back(m);
            continue;
        }
        m.w = eff_w(net, o);
        m.x = o.restaged ? net->ws + o.x_off : net->ws + net->ops[o.src_inst].y_off; m.xd = o.xd;
        m.y = net->ws + o.y_off; m.yd = launch_yd(o);
        m.residual = o.res >= 0 ? net->ws + net->ops[o.res_inst].y_off : nullptr; m.rd = o.rd;
        m.stride = o.stride; m.pad = o.pad; m.bias = eff_bias(net, o); m.relu = o.relu;
        members.push_back(m);
    }
    return members;
}

// Builds the launch records of the group led by op i for variant v (NULL: the untuned pick)
// and puts them on the device.
cadnn_status set_colaunch_variant(cadnn_net* net, size_t i, const ConvVariant* v) {
    const std::vector<ConvMember> members = colaunch_members(net, i);
    const int n = net->ops[i].in.n;
    if (!v) {
        std::vector<const ConvVariant*> common;
        cadnn_status st = conv2d_group_candidates(members, n, &common, &v);
        if (st != CADNN_OK) return st;
        if (!v) return fail(CADNN_EUNSUPPORTED, "cadnn_net: no kernel variant serves the layers launched with op %zu", i);
    }
    std::unique_ptr<CoLaunch> c(new CoLaunch());
    cadnn_status st = conv2d_group_records(members, n, v, &c->records, &c->plans);
    if (st != CADNN_OK) return st;
    if ((st = c->table.upload(c->records.data(), c->records.size() * sizeof(ConvLaunch))) != CADNN_OK) return st;
    c->v = v;
    net->colaunch[(int)i] = std::move(c);
    return CADNN_OK;
}

// Back to one launch per layer (tuning found the group slower than its members apart).  The
// members keep their place in the launch order, right behind op i and ahead of anything
// already queued there: later groups were formed knowing their outputs complete at op i.
void disband_colaunch(cadnn_net* net, size_t i) {
    NetOp& lead = net->ops[i];
    for (int j : lead.comates) {
        net->ops[j].colaunch_of = -1;
        net->ops[j].fused_into = -1;
        net->ops[j].hoisted_to = (int)i;
    }
    lead.hoisted.insert(lead.hoisted.begin(), lead.comates.begin(), lead.comates.end());
    lead.comates.clear();
    net->colaunch.erase((int)i);
}

// ... outside tuning, where the members have no plans of their own yet.
cadnn_status take_apart(cadnn_net* net, size_t i) {
    const std::vector<int> members = net->ops[i].comates;
    disband_colaunch(net, i);
    for (int j : members) {
        const NetOp& m = net->ops[(size_t)j];
        if (m.kind != OP_CONV) continue;
        cadnn_status st = conv2d_prepare_impl(eff_w(net, m), m.xd, m.in.n, m.stride, m.pad, out_s2d(m), nullptr);
        if (st != CADNN_OK) return st;
    }
    return CADNN_OK;
}

// The de-interleaved copy a restaged layer reads (a k = 1 pool from the source's layout).
cadnn_status restage_input(cadnn_net* net, const NetOp& op, const void* x, hipStream_t s) {
    if (!op.restaged) return CADNN_OK;
    return launch_maxpool(in_ptr(net, op.src_inst, x), op.src_d, net->ws + op.x_off, op.xd, op.in.n, 1, 1, 0, net->dtype, s);
}

cadnn_status launch_one(cadnn_net* net, size_t i, const void* x, void* y, hipStream_t s) {
    const NetOp& op = net->ops[i];
    if (op.fused_into >= 0) return CADNN_OK;     // computed inside (or launched with) another op
    cadnn_status rs = restage_input(net, op, x, s);
    for (size_t k = 0; k < op.comates.size() && rs == CADNN_OK; ++k) rs = restage_input(net, net->ops[(size_t)op.comates[k]], x, s);
    if (rs != CADNN_OK) return rs;
    if (!op.comates.empty()) {
        auto it = net->colaunch.find((int)i);
        if (it == net->colaunch.end()) return fail(CADNN_EINVAL, "cadnn_net: co-launch table of op %zu is missing", i);
        const CoLaunch& c = *it->second;
        CADNN_HIP(c.v->launch_multi((const ConvLaunch*)c.table.p, c.records.data(), (int)c.records.size(), op.in.n, s));
        return CADNN_OK;
    }
    const void* src = op.restaged ? (const void*)(net->ws + op.x_off) : in_ptr(net, op.src_inst, x);
    void* dst = out_ptr(net, i, y);
    ConvExtra ex;
    const bool fused = shortcut_of(net, op, x, &ex, y);
    switch (op.kind) {
        case OP_CONV:
            return conv2d_impl(eff_w(net, op), src, op.xd, dst, launch_yd(op),
                               (op.res >= 0 && op.shortcut < 0) ? in_ptr(net, op.res_inst, x) : nullptr, op.rd, op.in.n,
                               op.stride, op.pad, eff_bias(net, op), op.relu, s, fused ? &ex : nullptr);
        case OP_DEPTHWISE:
            return launch_depthwise(op.w, src, op.xd, dst, op.yd, op.in.n, op.stride, op.pad, (const float*)op.bias,
                                    op.relu, s);
        case OP_FC:
            return launch_fc(op.w, src, dst, op.in.n, (const float*)op.bias, op.relu, s);
        case OP_MAXPOOL:
            return launch_maxpool(src, op.xd, dst, op.yd, op.in.n, op.k, op.stride, op.pad, net->dtype, s);
        case OP_AVGPOOL2D:
            return launch_avgpool2d(src, op.xd, dst, op.yd, op.in.n, op.k, op.stride, op.pad, net->dtype, s);
        case OP_CONCAT: {
            // only the sources that were not written in place need moving
            for (size_t j = 0; j < op.srcs.size(); ++j) {
                if (op.in_place[j]) continue;
                const int p = op.src_insts[j];
                const TensorDesc from = p < 0 ? make_desc(net->input.c, net->input.h, net->input.w) : net->ops[p].yd;
                TensorDesc to = op.yd;
                to.c = from.c;
                char* slice = (char*)dst + (size_t)op.ch_off[j] * op.yd.plane * net->elem();
                cadnn_status st = launch_maxpool(in_ptr(net, p, x), from, slice, to, op.in.n, 1, 1, 0, net->dtype, s);
                if (st != CADNN_OK) return st;
            }
            return CADNN_OK;
        }
        case OP_AVGPOOL:
            return launch_avgpool(src, op.xd, dst, op.in.n, net->dtype, s);
    }
    return fail(CADNN_EINVAL, "cadnn_net: unknown op kind");
}

// The ops in launch order: the op list's, but for the hoisted pools.
cadnn_status launch_all(cadnn_net* net, const void* x, void* y, hipStream_t s) {
    for (size_t i = 0; i < net->ops.size(); ++i) {
        if (net->ops[i].hoisted_to >= 0) continue;
        cadnn_status st = launch_one(net, i, x, y, s);
        for (size_t k = 0; k < net->ops[i].hoisted.size() && st == CADNN_OK; ++k)
            st = launch_one(net, (size_t)net->ops[i].hoisted[k], x, y, s);
        if (st != CADNN_OK) return st;
    }
    return CADNN_OK;
}

void drop_graph(cadnn_net* net) {
    if (net->exec) (void)hipGraphExecDestroy(net->exec);
    net->exec = nullptr;
    net->cap_x = nullptr;
    net->cap_y = nullptr;
}

// Live tuning (CADNN_NET_TUNE, on the first run): every convolution's candidates are timed on
// the data an ordinary pass leaves in its input region, then every group of co-launched layers
// as a whole; a group stays only if it beats its layers launched apart.
cadnn_status tune_net(cadnn_net* net, const void* x, void* y, hipStream_t s) {
    // every layer is timed on the data an ordinary pass leaves in its input region
    cadnn_status st = launch_all(net, x, y, s);
    std::vector<float> alone_us(net->ops.size(), 0.0f);
    for (size_t i = 0; i < net->ops.size() && st == CADNN_OK; ++i) {
        const NetOp& op = net->ops[i];
        // (co-launched layers are timed one by one too: the group must beat their sum)
        if (op.kind != OP_CONV || (op.fused_into >= 0 && op.colaunch_of < 0)) continue;
        const std::function<cadnn_status()> producer = [&]() {
            return op.src_inst >= 0 ? launch_one(net, (size_t)op.src_inst, x, y, s) : CADNN_OK;
        };
        ConvExtra ex;
        const bool fused = shortcut_of(net, op, x, &ex, y);
        st = conv2d_tune_impl(eff_w(net, op), op.restaged ? (const void*)(net->ws + op.x_off) : in_ptr(net, op.src_inst, x), op.xd,
                              out_ptr(net, i, y), launch_yd(op),
                              (op.res >= 0 && op.shortcut < 0) ? in_ptr(net, op.res_inst, x) : nullptr, op.rd, op.in.n,
                              op.stride, op.pad, eff_bias(net, op), op.relu, s, 20, &alone_us[i], &producer,
                              fused ? &ex : nullptr);
    }
    // then every group as a whole, over the variants that serve all its layers
    for (size_t i = 0; i < net->ops.size() && st == CADNN_OK; ++i) {
        if (net->ops[i].comates.empty()) continue;
        // (a pool that rides along would cost a launch of its own: about 3.5 us at these sizes)
        float apart = alone_us[i];
        for (int j : net->ops[i].comates) apart += net->ops[j].kind == OP_CONV ? alone_us[(size_t)j] : 3.5f;
        const std::function<cadnn_status()> producer = [&]() {
            return launch_one(net, (size_t)net->ops[i].src_inst, x, y, s);
        };
        const ConvVariant* best = nullptr;
        float together = 0.0f;
        st = conv2d_group_tune(colaunch_members(net, i), net->ops[i].in.n, s, 20, &producer, &best, &together);
        if (st != CADNN_OK) break;
        if (best && together < apart) st = set_colaunch_variant(net, i, best);
        else disband_colaunch(net, i);
    }
    return st;
}

}  // namespace

extern "C" cadnn_status cadnn_net_create(cadnn_dtype dtype, int n, int c, int h, int w,
                                         cadnn_net** out) {
    if (out) *out = nullptr;
    if (!out) return fail(CADNN_EINVAL, "cadnn_net_create: NULL out");
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return fail(CADNN_EINVAL, "cadnn_net_create: bad shape");
    if (dtype != CADNN_F32 && dtype != CADNN_F16) return fail(CADNN_EINVAL, "cadnn_net_create: dtype");
    if (desc_too_large(make_desc(c, h, w)) || (int64_t)c * h * w * (dtype == CADNN_F16 ? 2 : 4) >= 0x7ffffff0ll)
        return fail(CADNN_EUNSUPPORTED, "cadnn_net_create: one input image is 2 GiB or more");
    cadnn_net* net = new (std::nothrow) cadnn_net();
    if (!net) return fail(CADNN_ENOMEM, "cadnn_net_create: out of memory");
    net->dtype = dtype;
    net->input = Shape{n, c, h, w};
    net->cur[0] = net->input;
    net->producer[0] = -1;
    *out = net;
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_add_conv(cadnn_net* net, const cadnn_weights* w, const void* bias,
                                           int stride, int pad, int relu, int src, int dst, int res) {
    if (!net || !w) return fail(CADNN_EINVAL, "cadnn_net_add_conv: NULL pointer");
    if (net->finalized) return fail(CADNN_EINVAL, "cadnn_net_add_conv: net already finalized");
    if (w->dtype != net->dtype) return fail(CADNN_EINVAL, "cadnn_net_add_conv: dtype of weights and net differ");
    if (src == dst || res == dst) return fail(CADNN_EINVAL, "cadnn_net_add_conv: dst aliases an input");
    NetOp op;
    cadnn_status st = src_shape(net, src, &op.in, &op.src_inst);
    if (st != CADNN_OK) return st;
    if (op.in.c != w->cin) return fail(CADNN_EINVAL, "cadnn_net_add_conv: %d input channels, weights take %d", op.in.c, w->cin);
    if (stride <= 0 || pad < 0) return fail(CADNN_EINVAL, "cadnn_net_add_conv: bad stride/pad");
    if (!tensor_fits(net, op.in, pad)) return fail(CADNN_EUNSUPPORTED, "cadnn_net_add_conv: one padded input image would be 1.75 GiB or more");
    op.out = Shape{op.in.n, w->cout, conv_out(op.in.h, w->kh, stride, pad), conv_out(op.in.w, w->kw, stride, pad)};
    if (op.out.h <= 0 || op.out.w <= 0) return fail(CADNN_EINVAL, "cadnn_net_add_conv: empty output");
    if (res >= 0) {
        Shape r;
        if ((st = src_shape(net, res, &r, &op.res_inst)) != CADNN_OK) return st;
        if (!(r == op.out)) return fail(CADNN_EINVAL, "cadnn_net_add_conv: residual shape differs from output");
    }
    op.kind = OP_CONV; op.w = w; op.bias = bias; op.stride = stride; op.pad = pad; op.relu = relu;
    op.src = src; op.dst = dst; op.res = res < 0 ? -1 : res;
    if ((st = note_output(net, dst, op.out)) != CADNN_OK) return st;
    net->ops.push_back(op);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_add_depthwise(cadnn_net* net, const cadnn_weights* w, const void* bias,
                                                int stride, int pad, int relu, int src, int dst) {
    if (!net || !w) return fail(CADNN_EINVAL, "cadnn_net_add_depthwise: NULL pointer");
    if (net->finalized) return fail(CADNN_EINVAL, "cadnn_net_add_depthwise: net already finalized");
    if (w->dtype != net->dtype) return fail(CADNN_EINVAL, "cadnn_net_add_depthwise: dtype of weights and net differ");
    if (w->cin != 1) return fail(CADNN_EINVAL, "cadnn_net_add_depthwise: weights are not a depthwise filter bank");
    if (src == dst) return fail(CADNN_EINVAL, "cadnn_net_add_depthwise: dst aliases src");
    NetOp op;
    cadnn_status st = src_shape(net, src, &op.in, &op.src_inst);
    if (st != CADNN_OK) return st;
    if (op.in.c != w->cout) return fail(CADNN_EINVAL, "cadnn_net_add_depthwise: %d channels, %d filters", op.in.c, w->cout);
    if (stride <= 0 || pad < 0) return fail(CADNN_EINVAL, "cadnn_net_add_depthwise: bad stride/pad");
    if (!tensor_fits(net, op.in, pad)) return fail(CADNN_EUNSUPPORTED, "cadnn_net_add_depthwise: one padded input image would be 1.75 GiB or more");
    op.out = Shape{op.in.n, op.in.c, conv_out(op.in.h, w->kh, stride, pad), conv_out(op.in.w, w->kw, stride, pad)};
    if (op.out.h <= 0 || op.out.w <= 0) return fail(CADNN_EINVAL, "cadnn_net_add_depthwise: empty output");
    op.kind = OP_DEPTHWISE; op.w = w; op.bias = bias; op.stride = stride; op.pad = pad; op.relu = relu;
    op.src = src; op.dst = dst;
    if ((st = note_output(net, dst, op.out)) != CADNN_OK) return st;
    net->ops.push_back(op);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_add_maxpool(cadnn_net* net, int k, int stride, int pad, int src,
                                              int dst) {
    if (!net) return fail(CADNN_EINVAL, "cadnn_net_add_maxpool: NULL net");
    if (net->finalized) return fail(CADNN_EINVAL, "cadnn_net_add_maxpool: net already finalized");
    if (k <= 0 || stride <= 0 || pad < 0 || src == dst) return fail(CADNN_EINVAL, "cadnn_net_add_maxpool: bad argument");
    NetOp op;
    cadnn_status st = src_shape(net, src, &op.in, &op.src_inst);
    if (st != CADNN_OK) return st;
    op.out = Shape{op.in.n, op.in.c, conv_out(op.in.h, k, stride, pad), conv_out(op.in.w, k, stride, pad)};
    if (op.out.h <= 0 || op.out.w <= 0) return fail(CADNN_EINVAL, "cadnn_net_add_maxpool: empty output");
    op.kind = OP_MAXPOOL; op.k = k; op.stride = stride; op.pad = pad; op.src = src; op.dst = dst;
    if ((st = note_output(net, dst, op.out)) != CADNN_OK) return st;
    net->ops.push_back(op);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_add_avgpool(cadnn_net* net, int k, int stride, int pad, int src,
                                              int dst) {
    if (!net) return fail(CADNN_EINVAL, "cadnn_net_add_avgpool: NULL net");
    if (net->finalized) return fail(CADNN_EINVAL, "cadnn_net_add_avgpool: net already finalized");
    if (k <= 0 || stride <= 0 || pad < 0 || src == dst) return fail(CADNN_EINVAL, "cadnn_net_add_avgpool: bad argument");
    NetOp op;
    cadnn_status st = src_shape(net, src, &op.in, &op.src_inst);
    if (st != CADNN_OK) return st;
    op.out = Shape{op.in.n, op.in.c, conv_out(op.in.h, k, stride, pad), conv_out(op.in.w, k, stride, pad)};
    if (op.out.h <= 0 || op.out.w <= 0) return fail(CADNN_EINVAL, "cadnn_net_add_avgpool: empty output");
    op.kind = OP_AVGPOOL2D; op.k = k; op.stride = stride; op.pad = pad; op.src = src; op.dst = dst;
    if ((st = note_output(net, dst, op.out)) != CADNN_OK) return st;
    net->ops.push_back(op);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_add_concat(cadnn_net* net, const int* srcs, int count, int dst) {
    if (!net || !srcs) return fail(CADNN_EINVAL, "cadnn_net_add_concat: NULL pointer");
    if (net->finalized) return fail(CADNN_EINVAL, "cadnn_net_add_concat: net already finalized");
    if (count <= 0) return fail(CADNN_EINVAL, "cadnn_net_add_concat: no sources");
    NetOp op;
    int channels = 0;
    for (int j = 0; j < count; ++j) {
        if (srcs[j] == dst) return fail(CADNN_EINVAL, "cadnn_net_add_concat: dst aliases a source");
        Shape sh;
        int inst = -1;
        cadnn_status st = src_shape(net, srcs[j], &sh, &inst);
        if (st != CADNN_OK) return st;
        if (j == 0) {
            op.in = sh;
            op.src = srcs[0];
            op.src_inst = inst;
        } else if (sh.n != op.in.n || sh.h != op.in.h || sh.w != op.in.w) {
            return fail(CADNN_EINVAL, "cadnn_net_add_concat: source %d is %dx%dx%d, the first is %dx%dx%d", j, sh.n,
                        sh.h, sh.w, op.in.n, op.in.h, op.in.w);
        }
        op.srcs.push_back(srcs[j]);
        op.src_insts.push_back(inst);
        op.ch_off.push_back(channels);
        channels += sh.c;
    }
    op.in_place.assign((size_t)count, 0);
    op.out = Shape{op.in.n, channels, op.in.h, op.in.w};
    op.kind = OP_CONCAT; op.dst = dst;
    cadnn_status st = note_output(net, dst, op.out);
    if (st != CADNN_OK) return st;
    net->ops.push_back(op);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_add_global_avgpool(cadnn_net* net, int src, int dst) {
    if (!net) return fail(CADNN_EINVAL, "cadnn_net_add_global_avgpool: NULL net");
    if (net->finalized) return fail(CADNN_EINVAL, "cadnn_net_add_global_avgpool: net already finalized");
    if (src == dst) return fail(CADNN_EINVAL, "cadnn_net_add_global_avgpool: dst aliases src");
    NetOp op;
    cadnn_status st = src_shape(net, src, &op.in, &op.src_inst);
    if (st != CADNN_OK) return st;
    op.out = Shape{op.in.n, op.in.c, 1, 1};
    op.kind = OP_AVGPOOL; op.src = src; op.dst = dst;
    if ((st = note_output(net, dst, op.out)) != CADNN_OK) return st;
    net->ops.push_back(op);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_add_fc(cadnn_net* net, const cadnn_weights* w, const void* bias,
                                         int relu, int src, int dst) {
    if (!net || !w) return fail(CADNN_EINVAL, "cadnn_net_add_fc: NULL pointer");
    if (net->finalized) return fail(CADNN_EINVAL, "cadnn_net_add_fc: net already finalized");
    if (w->dtype != net->dtype) return fail(CADNN_EINVAL, "cadnn_net_add_fc: dtype of weights and net differ");
    if (w->kh != 1 || w->kw != 1) return fail(CADNN_EINVAL, "cadnn_net_add_fc: weights are not a matrix");
    if (src == dst) return fail(CADNN_EINVAL, "cadnn_net_add_fc: dst aliases src");
    NetOp op;
    cadnn_status st = src_shape(net, src, &op.in, &op.src_inst);
    if (st != CADNN_OK) return st;
    if ((size_t)op.in.c * op.in.h * op.in.w != (size_t)w->cin)
        return fail(CADNN_EINVAL, "cadnn_net_add_fc: %zu input features, weights take %d",
                    (size_t)op.in.c * op.in.h * op.in.w, w->cin);
    op.out = Shape{op.in.n, w->cout, 1, 1};
    op.kind = OP_FC; op.w = w; op.bias = bias; op.relu = relu; op.src = src; op.dst = dst;
    if ((st = note_output(net, dst, op.out)) != CADNN_OK) return st;
    net->ops.push_back(op);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_workspace_bytes(const cadnn_net* net, size_t* bytes) {
    if (!net || !bytes) return fail(CADNN_EINVAL, "cadnn_net_workspace_bytes: NULL pointer");
    if (net->ops.empty()) return fail(CADNN_EINVAL, "cadnn_net_workspace_bytes: empty net");
    if (!net->laid_out) layout(const_cast<cadnn_net*>(net));
    *bytes = net->ws_bytes;
    return CADNN_OK;
}

// (Re)does the layout if the flags that matter to it changed.
static void layout_for(cadnn_net* net, int flags) {
    const bool allow = (flags & CADNN_NET_PLAIN_LAYOUT) == 0;
    const bool fuse = (flags & CADNN_NET_NO_FUSION) == 0;
    if (!net->laid_out || allow != net->allow_s2d || fuse != net->allow_fusion) {
        net->allow_s2d = allow;
        net->allow_fusion = fuse;
        layout(net);
    }
}

extern "C" cadnn_status cadnn_net_op_info(cadnn_net* net, int op_index, int flags, cadnn_op_info* out) {
    if (!net || !out) return fail(CADNN_EINVAL, "cadnn_net_op_info: NULL pointer");
    if (op_index < 0 || op_index >= (int)net->ops.size()) return fail(CADNN_EINVAL, "cadnn_net_op_info: no op %d", op_index);
    if (net->finalized) {
        const int now = (net->allow_s2d ? 0 : CADNN_NET_PLAIN_LAYOUT) | (net->allow_fusion ? 0 : CADNN_NET_NO_FUSION);
        if ((flags & (CADNN_NET_PLAIN_LAYOUT | CADNN_NET_NO_FUSION)) != now)
            return fail(CADNN_EINVAL, "cadnn_net_op_info: the net was finalized with other flags");
    } else {
        layout_for(net, flags);
    }
    const NetOp& op = net->ops[op_index];
    out->halo_h = op.yd.ph;
    out->halo_w = op.yd.pw;
    out->pitch = op.yd.pitch;
    out->plane = op.yd.plane;
    out->image = op.yd.image;
    out->deinterleaved = op.yd.s2d;
    out->offset = (int64_t)op.y_off + (op.yd.s2d ? 0 : (int64_t)op.yd.origin * (int64_t)net->elem());
    out->fused_into = op.fused_into;
    out->slice_of = op.slice_of;
    out->slice_channel = op.sibling_of >= 0 ? op.sib_ch : op.slice_ch;
    out->launched_with = op.colaunch_of >= 0 ? 1 : 0;
    out->launched_after = op.hoisted_to;
    out->input_copy = op.restaged ? (int64_t)op.x_off : -1;
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_finalize(cadnn_net* net, void* ws, size_t bytes, int flags) {
    if (!net) return fail(CADNN_EINVAL, "cadnn_net_finalize: NULL net");
    if (net->ops.empty()) return fail(CADNN_EINVAL, "cadnn_net_finalize: empty net");
    // (a plain layout never needs more room than the de-interleaved one that
    // cadnn_net_workspace_bytes reports)
    layout_for(net, flags);
    net->static_ws = (flags & CADNN_NET_STATIC_WORKSPACE) != 0;
    if (net->static_ws) {
        if (net->ws_bytes > kStaticWorkspaceBytes)
            return fail(CADNN_EUNSUPPORTED, "cadnn_net_finalize: the net needs %zu bytes of workspace, the static workspace holds %zu",
                        net->ws_bytes, kStaticWorkspaceBytes);
        cadnn_status st = static_workspace(&ws);
        if (st != CADNN_OK) return st;
        bytes = kStaticWorkspaceBytes;
    }
    if (net->ws_bytes > 0 && !ws) return fail(CADNN_EINVAL, "cadnn_net_finalize: NULL workspace");
    if (bytes < net->ws_bytes) return fail(CADNN_EINVAL, "cadnn_net_finalize: workspace of %zu bytes, %zu needed", bytes, net->ws_bytes);
    drop_graph(net);
    net->ws = (char*)ws;
    // halos are read as the zero padding of the consumer layers and are never written again
    if (net->ws_bytes) {
        CADNN_HIP(hipMemset(ws, 0, net->ws_bytes));
        CADNN_HIP(hipDeviceSynchronize());
    }
    // biases of a sibling group, stacked like the rows of its merged weights
    net->merged_bias.clear();
    for (size_t i = 0; i < net->ops.size(); ++i) {
        const NetOp& op = net->ops[i];
        if (op.siblings.empty() || !op.bias) continue;
        std::vector<float> zeros((size_t)op.launch_c, 0.0f);
        std::unique_ptr<DevBuf> buf(new DevBuf());
        cadnn_status st = buf->upload(zeros.data(), zeros.size() * 4);
        if (st != CADNN_OK) return st;
        CADNN_HIP(hipMemcpy(buf->p, op.bias, (size_t)op.out.c * 4, hipMemcpyDeviceToDevice));
        for (int j : op.siblings) {
            const NetOp& sib = net->ops[j];
            CADNN_HIP(hipMemcpy((char*)buf->p + (size_t)sib.sib_ch * 4, sib.bias, (size_t)sib.out.c * 4, hipMemcpyDeviceToDevice));
        }
        net->merged_bias[(int)i] = std::move(buf);
    }
    for (const NetOp& op : net->ops) {
        cadnn_status st = CADNN_OK;
        ConvExtra ex;
        if (op.kind == OP_CONV && op.fused_into < 0)
            st = conv2d_prepare_impl(eff_w(net, op), op.xd, op.in.n, op.stride, op.pad, out_s2d(op), shortcut_geom(net, op, &ex));
        if (op.kind == OP_FC) st = cadnn_fc_prepare(op.w);
        if (op.kind == OP_DEPTHWISE) st = ensure_dw_device(op.w);
        if (st != CADNN_OK) return st;
    }
    net->colaunch.clear();
    for (size_t i = 0; i < net->ops.size(); ++i) {
        if (net->ops[i].comates.empty()) continue;
        cadnn_status st = set_colaunch_variant(net, i, nullptr);
        if (st != CADNN_OK) return st;
    }
    net->use_graph = (flags & CADNN_NET_GRAPH) != 0;
    net->want_tune = (flags & CADNN_NET_TUNE) != 0;
    net->finalized = true;
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_run_net(cadnn_net* net, const void* x, void* y, void* stream) {
    if (!net || !x || !y) return fail(CADNN_EINVAL, "cadnn_run_net: NULL pointer");
    if (!net->finalized) return fail(CADNN_EINVAL, "cadnn_run_net: net not finalized");
    hipStream_t s = (hipStream_t)stream;
    if (net->want_tune) {
        cadnn_status st = tune_net(net, x, y, s);
        if (st != CADNN_OK) return st;
        net->want_tune = false;
        drop_graph(net);
    }
    if (!net->use_graph) return launch_all(net, x, y, s);
    if (!net->exec || net->cap_x != x || net->cap_y != y) {
        drop_graph(net);
        hipStream_t cs = nullptr;
        CADNN_HIP(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
        hipGraph_t graph = nullptr;
        hipError_t e = hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal);
        cadnn_status st = CADNN_OK;
        if (e != hipSuccess) {
            st = fail(CADNN_EHIP, "hipStreamBeginCapture failed: %s", hipGetErrorString(e));
        } else {
            st = launch_all(net, x, y, cs);
            e = hipStreamEndCapture(cs, &graph);
            if (st == CADNN_OK && e != hipSuccess)
                st = fail(CADNN_EHIP, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
        }
        if (st == CADNN_OK) {
            e = hipGraphInstantiate(&net->exec, graph, nullptr, nullptr, 0);
            if (e != hipSuccess) {
                net->exec = nullptr;
                st = fail(CADNN_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
            }
        }
        if (graph) (void)hipGraphDestroy(graph);
        (void)hipStreamDestroy(cs);
        if (st != CADNN_OK) return st;
        net->cap_x = x;
        net->cap_y = y;
    }
    CADNN_HIP(hipGraphLaunch(net->exec, s));
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_run_net_noalloc(cadnn_net* net, const void* x, void* y, void* stream) {
    if (!net || !x || !y) return fail(CADNN_EINVAL, "cadnn_run_net_noalloc: NULL pointer");
    if (!net->finalized) return fail(CADNN_EINVAL, "cadnn_run_net_noalloc: net not finalized");
    if (!net->static_ws) return fail(CADNN_EINVAL, "cadnn_run_net_noalloc: the net was not finalized with CADNN_NET_STATIC_WORKSPACE");
    if (net->want_tune) return fail(CADNN_EINVAL, "cadnn_run_net_noalloc: tuning (CADNN_NET_TUNE) allocates; run cadnn_run_net once first");
    if (net->ws_bytes > kStaticWorkspaceBytes) return fail(CADNN_EUNSUPPORTED, "cadnn_run_net_noalloc: workspace above the static limit");
    hipStream_t s = (hipStream_t)stream;
    void* ptr = nullptr;
    cadnn_status st = static_workspace(&ptr);
    if (st != CADNN_OK) return st;
    if (ptr != (void*)net->ws) return fail(CADNN_EINVAL, "cadnn_run_net_noalloc: the net was finalized on another device");
    const NoDeviceAlloc guard;
    // The array is shared by every such net on this GPU and keeps what the last call left: the
    // halos this net reads as zero padding are cleared again (with a kernel, so that a caller
    // under graph capture records no memset node).
    if (net->ws_bytes && (st = launch_zero(ptr, (net->ws_bytes + 15) / 16 * 16, s)) != CADNN_OK) return st;
    return launch_all(net, x, y, s);
}

extern "C" cadnn_status cadnn_net_num_ops(const cadnn_net* net, int* num_ops) {
    if (!net || !num_ops) return fail(CADNN_EINVAL, "cadnn_net_num_ops: NULL pointer");
    *num_ops = (int)net->ops.size();
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_profile(cadnn_net* net, const void* x, void* y, void* stream,
                                          int repeats, float* ms_per_op) {
    if (!net || !x || !y || !ms_per_op) return fail(CADNN_EINVAL, "cadnn_net_profile: NULL pointer");
    if (!net->finalized) return fail(CADNN_EINVAL, "cadnn_net_profile: net not finalized");
    if (repeats <= 0) return fail(CADNN_EINVAL, "cadnn_net_profile: repeats must be positive");
    hipStream_t s = (hipStream_t)stream;
    const size_t nops = net->ops.size();
    std::vector<hipEvent_t> ev(nops + 1, nullptr);
    cadnn_status st = CADNN_OK;
    for (size_t i = 0; i <= nops && st == CADNN_OK; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) st = fail(CADNN_EHIP, "hipEventCreate failed");
    // Every op is idempotent (it reads its sources and overwrites its destination), so op i
    // is launched `repeats` times back to back between two events on the caller's stream.
    for (size_t i = 0; i < nops && st == CADNN_OK; ++i) {
        if (hipEventRecord(ev[i], s) != hipSuccess) { st = fail(CADNN_EHIP, "hipEventRecord failed"); break; }
        for (int r = 0; r < repeats && st == CADNN_OK; ++r) st = launch_one(net, i, x, y, s);
    }
    if (st == CADNN_OK && hipEventRecord(ev[nops], s) != hipSuccess) st = fail(CADNN_EHIP, "hipEventRecord failed");
    if (st == CADNN_OK && hipStreamSynchronize(s) != hipSuccess) st = fail(CADNN_EHIP, "hipStreamSynchronize failed");
    for (size_t i = 0; i < nops && st == CADNN_OK; ++i) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, ev[i], ev[i + 1]) != hipSuccess) st = fail(CADNN_EHIP, "hipEventElapsedTime failed");
        ms_per_op[i] = ms / (float)repeats;
    }
    for (hipEvent_t e : ev) if (e) (void)hipEventDestroy(e);
    return st;
}

// Per-op device time with the ops IN LAUNCH ORDER, as a forward pass runs them: every op finds
// the caches as the real pass leaves them (its input just written by its producer, its weights
// last touched a whole pass ago) instead of warm from its own previous launch.  Every kernel
// carries its own start and stop marks (LaunchTimer), so an op's figure is the device time of
// its kernels and nothing else -- what a kernel trace of the same pass reports.
extern "C" cadnn_status cadnn_net_profile_in_order(cadnn_net* net, const void* x, void* y, void* stream,
                                                   int repeats, float* ms_per_op) {
    if (!net || !x || !y || !ms_per_op) return fail(CADNN_EINVAL, "cadnn_net_profile_in_order: NULL pointer");
    if (!net->finalized) return fail(CADNN_EINVAL, "cadnn_net_profile_in_order: net not finalized");
    if (repeats <= 0) return fail(CADNN_EINVAL, "cadnn_net_profile_in_order: repeats must be positive");
    hipStream_t s = (hipStream_t)stream;
    const size_t nops = net->ops.size();
    std::vector<size_t> order;
    for (size_t i = 0; i < nops; ++i) {
        if (net->ops[i].hoisted_to >= 0) continue;
        order.push_back(i);
        for (int h : net->ops[i].hoisted) order.push_back((size_t)h);
    }
    std::vector<LaunchTimer> timers(order.size());
    cadnn_status st = CADNN_OK;
    for (LaunchTimer& t : timers)
        for (int k = 0; k < LaunchTimer::kMax; ++k) { t.start[k] = nullptr; t.stop[k] = nullptr; }
    for (LaunchTimer& t : timers)
        for (int k = 0; k < LaunchTimer::kMax && st == CADNN_OK; ++k)
            if (hipEventCreate(&t.start[k]) != hipSuccess || hipEventCreate(&t.stop[k]) != hipSuccess)
                st = fail(CADNN_EHIP, "hipEventCreate failed");
    std::vector<double> sum(nops, 0.0);
    for (int r = 0; r < repeats && st == CADNN_OK; ++r) {
        for (size_t k = 0; k < order.size() && st == CADNN_OK; ++k) {
            timers[k].used = 0;
            g_launch_timer = &timers[k];
            st = launch_one(net, order[k], x, y, s);
            g_launch_timer = nullptr;
        }
        if (st == CADNN_OK && hipStreamSynchronize(s) != hipSuccess) st = fail(CADNN_EHIP, "hipStreamSynchronize failed");
        for (size_t k = 0; k < order.size() && st == CADNN_OK; ++k)
            for (int q = 0; q < timers[k].used; ++q) {
                float ms = 0.0f;
                if (hipEventElapsedTime(&ms, timers[k].start[q], timers[k].stop[q]) != hipSuccess) { st = fail(CADNN_EHIP, "hipEventElapsedTime failed"); break; }
                sum[order[k]] += ms;
            }
    }
    g_launch_timer = nullptr;
    for (LaunchTimer& t : timers)
        for (int k = 0; k < LaunchTimer::kMax; ++k) {
            if (t.start[k]) (void)hipEventDestroy(t.start[k]);
            if (t.stop[k]) (void)hipEventDestroy(t.stop[k]);
        }
    if (st != CADNN_OK) return st;
    for (size_t i = 0; i < nops; ++i) ms_per_op[i] = (float)(sum[i] / repeats);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_op_variant(const cadnn_net* net, int op_index, char* buf, size_t len) {
    if (!net || !buf || len == 0) return fail(CADNN_EINVAL, "cadnn_net_op_variant: NULL pointer");
    if (!net->finalized) return fail(CADNN_EINVAL, "cadnn_net_op_variant: net not finalized");
    if (op_index < 0 || op_index >= (int)net->ops.size()) return fail(CADNN_EINVAL, "cadnn_net_op_variant: no op %d", op_index);
    const NetOp& op = net->ops[op_index];
    const char* name = "";
    switch (op.kind) {
        case OP_CONV: {
            ConvExtra ex;
            auto co = net->colaunch.find(op_index);
            name = op.fused_into >= 0 ? "fused"
                   : (!op.comates.empty() && co != net->colaunch.end()) ? co->second->v->name
                                      : conv2d_variant_name_impl(eff_w(net, op), op.xd, op.in.n, op.stride, op.pad, out_s2d(op),
                                                                 shortcut_geom(net, op, &ex));
            break;
        }
        case OP_FC: name = "sfc"; break;
        case OP_DEPTHWISE: name = op.fused_into >= 0 ? "fused" : "dwconv"; break;
        case OP_MAXPOOL: name = op.fused_into >= 0 ? "fused" : "maxpool"; break;
        case OP_AVGPOOL: name = op.fused_into >= 0 ? "fused" : "avgpool"; break;
        case OP_AVGPOOL2D: name = op.fused_into >= 0 ? "fused" : "avgpool2d"; break;
        case OP_CONCAT:
            name = std::all_of(op.in_place.begin(), op.in_place.end(), [](char c) { return c != 0; }) ? "in place" : "concat";
            break;
    }
    if (!name) return CADNN_EUNSUPPORTED;
    std::strncpy(buf, name, len - 1);
    buf[len - 1] = '\0';
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_op_candidates(const cadnn_net* net, int op_index, char* buf, size_t len) {
    if (!net || !buf || len == 0) return fail(CADNN_EINVAL, "cadnn_net_op_candidates: NULL pointer");
    if (!net->finalized) return fail(CADNN_EINVAL, "cadnn_net_op_candidates: net not finalized");
    if (op_index < 0 || op_index >= (int)net->ops.size()) return fail(CADNN_EINVAL, "cadnn_net_op_candidates: no op %d", op_index);
    const NetOp& op = net->ops[op_index];
    if (op.kind != OP_CONV) return fail(CADNN_EINVAL, "cadnn_net_op_candidates: op %d is not a convolution", op_index);
    if (op.fused_into >= 0) return fail(CADNN_EINVAL, "cadnn_net_op_candidates: op %d is computed inside op %d", op_index, op.fused_into);
    if (!op.comates.empty()) {
        // the variants that serve the whole group
        std::vector<const ConvVariant*> common;
        cadnn_status st = conv2d_group_candidates(colaunch_members(net, (size_t)op_index), op.in.n, &common, nullptr);
        if (st != CADNN_OK) return st;
        std::string all;
        for (const ConvVariant* v : common) {
            if (!all.empty()) all += "\n";
            all += v->name;
        }
        if (all.size() + 1 > len) return fail(CADNN_EINVAL, "cadnn_net_op_candidates: buffer of %zu bytes, %zu needed", len, all.size() + 1);
        std::memcpy(buf, all.c_str(), all.size() + 1);
        return CADNN_OK;
    }
    ConvExtra ex;
    return conv2d_list_variants_impl(eff_w(net, op), op.xd, op.in.n, op.stride, op.pad, buf, len, out_s2d(op), shortcut_geom(net, op, &ex));
}

extern "C" cadnn_status cadnn_net_set_op_variant(cadnn_net* net, int op_index, const char* name) {
    if (!net) return fail(CADNN_EINVAL, "cadnn_net_set_op_variant: NULL net");
    if (!net->finalized) return fail(CADNN_EINVAL, "cadnn_net_set_op_variant: net not finalized");
    if (op_index < 0 || op_index >= (int)net->ops.size()) return fail(CADNN_EINVAL, "cadnn_net_set_op_variant: no op %d", op_index);
    const NetOp& op = net->ops[op_index];
    if (op.kind != OP_CONV) return fail(CADNN_EINVAL, "cadnn_net_set_op_variant: op %d is not a convolution", op_index);
    if (op.fused_into >= 0) return CADNN_OK;     // nothing to pin: computed inside, or launched with, another op
    if (!op.comates.empty() && name && std::strcmp(name, "apart") == 0) {
        // the group's layers one launch each from now on (what tuning does to a group that loses)
        drop_graph(net);
        CADNN_HIP(hipDeviceSynchronize());
        return take_apart(net, (size_t)op_index);
    }
    if (!op.comates.empty()) {
        const ConvVariant* v = nullptr;
        if (name && *name) {
            std::vector<const ConvVariant*> common;
            cadnn_status st = conv2d_group_candidates(colaunch_members(net, (size_t)op_index), op.in.n, &common, nullptr);
            if (st != CADNN_OK) return st;
            for (const ConvVariant* c : common) if (std::strcmp(c->name, name) == 0) v = c;
            if (!v) return fail(CADNN_EINVAL, "cadnn_net_set_op_variant: '%s' does not serve every layer launched with op %d", name, op_index);
        }
        drop_graph(net);
        // (the stream may still be running the old table's launches)
        CADNN_HIP(hipDeviceSynchronize());
        return set_colaunch_variant(net, (size_t)op_index, v);
    }
    ConvExtra ex;
    cadnn_status st = conv2d_set_variant_impl(eff_w(net, op), op.xd, op.in.n, op.stride, op.pad, name, out_s2d(op), shortcut_geom(net, op, &ex));
    if (st != CADNN_OK) return st;
    drop_graph(net);
    return conv2d_prepare_impl(eff_w(net, op), op.xd, op.in.n, op.stride, op.pad, out_s2d(op), shortcut_geom(net, op, &ex));
}

extern "C" cadnn_status cadnn_net_read_buffer(cadnn_net* net, int buf, void* host_out, size_t bytes,
                                              void* stream) {
    if (!net || !host_out) return fail(CADNN_EINVAL, "cadnn_net_read_buffer: NULL pointer");
    if (!net->finalized) return fail(CADNN_EINVAL, "cadnn_net_read_buffer: net not finalized");
    auto it = net->producer.find(buf);
    if (it == net->producer.end() || it->second < 0 || it->second + 1 == (int)net->ops.size())
        return fail(CADNN_EINVAL, "cadnn_net_read_buffer: buffer %d is not in the workspace", buf);
    const NetOp& op = net->ops[it->second];
    // (a fused pool's vector is written, by the convolution; a fused projection's map is not)
    if (op.fused_into >= 0 && op.kind == OP_CONV && op.sibling_of < 0 && op.colaunch_of < 0)
        return fail(CADNN_EINVAL, "cadnn_net_read_buffer: buffer %d is never materialised (its op is computed inside op %d)", buf, op.fused_into);
    if (op.pool_op >= 0)
        return fail(CADNN_EINVAL, "cadnn_net_read_buffer: buffer %d is never materialised (op %d pools it on the fly)", buf, it->second);
    if (op.dw_op >= 0)
        return fail(CADNN_EINVAL, "cadnn_net_read_buffer: buffer %d is never materialised (op %d filters it on the fly)", buf, it->second);
    const size_t e = net->elem();
    if (bytes != op.out.elems() * e)
        return fail(CADNN_EINVAL, "cadnn_net_read_buffer: buffer %d holds %zu bytes, %zu asked", buf, op.out.elems() * e, bytes);
    CADNN_HIP(hipStreamSynchronize((hipStream_t)stream));
    if (op.yd.s2d) {
        // de-interleaved region: fetch it whole and pick the image positions on the host
        const size_t total = (size_t)op.out.n * op.yd.image * e;
        std::vector<char> raw(total);
        CADNN_HIP(hipMemcpy(raw.data(), net->ws + op.y_off, total, hipMemcpyDeviceToHost));
        for (int n = 0; n < op.out.n; ++n)
            for (int c = 0; c < op.out.c; ++c)
                for (int i = 0; i < op.out.h; ++i)
                    for (int j = 0; j < op.out.w; ++j) {
                        const size_t src = ((size_t)n * op.yd.image + (size_t)c * op.yd.plane + tensor_off(op.yd, i, j)) * e;
                        const size_t dst = ((((size_t)n * op.out.c + c) * op.out.h + i) * op.out.w + j) * e;
                        std::memcpy((char*)host_out + dst, raw.data() + src, e);
                    }
        return CADNN_OK;
    }
    // strip the halo: one 2-D copy per (image, channel) plane
    for (int n = 0; n < op.out.n; ++n)
        for (int c = 0; c < op.out.c; ++c) {
            const char* src = net->ws + op.y_off + ((size_t)n * op.yd.image + (size_t)c * op.yd.plane + op.yd.origin) * e;
            char* dst = (char*)host_out + ((size_t)n * op.out.c + c) * op.out.h * op.out.w * e;
            CADNN_HIP(hipMemcpy2D(dst, (size_t)op.out.w * e, src, (size_t)op.yd.pitch * e, (size_t)op.out.w * e,
                                  (size_t)op.out.h, hipMemcpyDeviceToHost));
        }
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_free(cadnn_net* net) {
    if (net) {
        drop_graph(net);
        delete net;
    }
    return CADNN_OK;
}
