// Whole-network runner: an ordered op list over numbered activation buffers, launched
// back to back on one stream (optionally as one captured HIP graph) so that a single-image
// inference (the quantity the paper's evaluation reports, Section 5) costs one submission.
#include <algorithm>
#include <cstring>

#include "internal.h"

using namespace cadnn;

namespace {

enum OpKind { OP_CONV, OP_FC, OP_MAXPOOL, OP_AVGPOOL };

struct Shape {
    int n = 0, c = 0, h = 0, w = 0;
    size_t elems() const { return (size_t)n * c * h * w; }
    bool operator==(const Shape& o) const { return n == o.n && c == o.c && h == o.h && w == o.w; }
};

struct NetOp {
    OpKind kind;
    const cadnn_weights* w = nullptr;
    const void* bias = nullptr;
    int stride = 1, pad = 0, relu = 0, k = 0;
    int src = 0, dst = 0, res = -1;
    Shape in, out;
};

}  // namespace

struct cadnn_net {
    cadnn_dtype dtype = CADNN_F32;
    Shape input;
    std::vector<NetOp> ops;
    std::map<int, Shape> cur;        // current shape held by each buffer while building
    std::map<int, size_t> max_elems; // largest element count each buffer ever holds
    std::map<int, size_t> offset;    // byte offset of each workspace buffer
    int out_buf = -1;
    size_t ws_bytes = 0;
    bool finalized = false;
    bool use_graph = false;
    bool want_tune = false;
    char* ws = nullptr;
    // captured graph
    hipGraphExec_t exec = nullptr;
    const void* cap_x = nullptr;
    void* cap_y = nullptr;
    size_t elem() const { return dtype == CADNN_F16 ? 2 : 4; }
};

namespace {

cadnn_status note_output(cadnn_net* net, int dst, const Shape& s) {
    if (dst <= 0) return fail(CADNN_EINVAL, "cadnn_net: dst buffer must be >= 1 (0 is the input)");
    net->cur[dst] = s;
    size_t& m = net->max_elems[dst];
    m = std::max(m, s.elems());
    net->out_buf = dst;
    return CADNN_OK;
}

cadnn_status src_shape(cadnn_net* net, int src, Shape* s) {
    auto it = net->cur.find(src);
    if (it == net->cur.end()) return fail(CADNN_EINVAL, "cadnn_net: buffer %d read before it is written", src);
    *s = it->second;
    return CADNN_OK;
}

void* buf_ptr(cadnn_net* net, int buf, const void* x, void* y) {
    if (buf == 0) return const_cast<void*>(x);
    if (buf == net->out_buf) return y;
    return net->ws + net->offset[buf];
}

cadnn_status launch_one(cadnn_net* net, size_t i, const void* x, void* y, hipStream_t s) {
    const NetOp& op = net->ops[i];
    const void* src = buf_ptr(net, op.src, x, y);
    void* dst = buf_ptr(net, op.dst, x, y);
    switch (op.kind) {
        case OP_CONV:
            return conv2d_impl(op.w, src, dst, op.in.n, op.in.h, op.in.w, op.stride, op.pad, op.bias,
                               op.res >= 0 ? buf_ptr(net, op.res, x, y) : nullptr, op.relu, s);
        case OP_FC:
            return launch_fc(op.w, src, dst, op.in.n, (const float*)op.bias, op.relu, s);
        case OP_MAXPOOL:
            return launch_maxpool(src, dst, op.in.n, op.in.c, op.in.h, op.in.w, op.k, op.stride,
                                  op.pad, net->dtype, s);
        case OP_AVGPOOL:
            return launch_avgpool(src, dst, op.in.n, op.in.c, op.in.h, op.in.w, net->dtype, s);
    }
    return fail(CADNN_EINVAL, "cadnn_net: unknown op kind");
}

cadnn_status launch_all(cadnn_net* net, const void* x, void* y, hipStream_t s) {
    for (size_t i = 0; i < net->ops.size(); ++i) {
        cadnn_status st = launch_one(net, i, x, y, s);
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

}  // namespace

extern "C" cadnn_status cadnn_net_create(cadnn_dtype dtype, int n, int c, int h, int w,
                                         cadnn_net** out) {
    if (out) *out = nullptr;
    if (!out) return fail(CADNN_EINVAL, "cadnn_net_create: NULL out");
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return fail(CADNN_EINVAL, "cadnn_net_create: bad shape");
    if (dtype != CADNN_F32 && dtype != CADNN_F16) return fail(CADNN_EINVAL, "cadnn_net_create: dtype");
    cadnn_net* net = new (std::nothrow) cadnn_net();
    if (!net) return fail(CADNN_ENOMEM, "cadnn_net_create: out of memory");
    net->dtype = dtype;
    net->input = Shape{n, c, h, w};
    net->cur[0] = net->input;
    *out = net;
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_add_conv(cadnn_net* net, const cadnn_weights* w, const void* bias,
                                           int stride, int pad, int relu, int src, int dst, int res) {
    if (!net || !w) return fail(CADNN_EINVAL, "cadnn_net_add_conv: NULL pointer");
    if (net->finalized) return fail(CADNN_EINVAL, "cadnn_net_add_conv: net already finalized");
    if (w->dtype != net->dtype) return fail(CADNN_EINVAL, "cadnn_net_add_conv: dtype of weights and net differ");
    if (src == dst || res == dst) return fail(CADNN_EINVAL, "cadnn_net_add_conv: dst aliases an input");
    Shape in;
    cadnn_status st = src_shape(net, src, &in);
    if (st != CADNN_OK) return st;
    if (in.c != w->cin) return fail(CADNN_EINVAL, "cadnn_net_add_conv: %d input channels, weights take %d", in.c, w->cin);
    if (stride <= 0 || pad < 0) return fail(CADNN_EINVAL, "cadnn_net_add_conv: bad stride/pad");
    Shape o{in.n, w->cout, conv_out(in.h, w->kh, stride, pad), conv_out(in.w, w->kw, stride, pad)};
    if (o.h <= 0 || o.w <= 0) return fail(CADNN_EINVAL, "cadnn_net_add_conv: empty output");
    if (res >= 0) {
        Shape r;
        if ((st = src_shape(net, res, &r)) != CADNN_OK) return st;
        if (!(r == o)) return fail(CADNN_EINVAL, "cadnn_net_add_conv: residual shape differs from output");
    }
    if ((st = cadnn_conv2d_prepare(w, in.n, in.h, in.w, stride, pad)) != CADNN_OK) return st;
    NetOp op;
    op.kind = OP_CONV; op.w = w; op.bias = bias; op.stride = stride; op.pad = pad; op.relu = relu;
    op.src = src; op.dst = dst; op.res = res < 0 ? -1 : res; op.in = in; op.out = o;
    if ((st = note_output(net, dst, o)) != CADNN_OK) return st;
    net->ops.push_back(op);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_add_maxpool(cadnn_net* net, int k, int stride, int pad, int src,
                                              int dst) {
    if (!net) return fail(CADNN_EINVAL, "cadnn_net_add_maxpool: NULL net");
    if (net->finalized) return fail(CADNN_EINVAL, "cadnn_net_add_maxpool: net already finalized");
    if (k <= 0 || stride <= 0 || pad < 0 || src == dst) return fail(CADNN_EINVAL, "cadnn_net_add_maxpool: bad argument");
    Shape in;
    cadnn_status st = src_shape(net, src, &in);
    if (st != CADNN_OK) return st;
    Shape o{in.n, in.c, conv_out(in.h, k, stride, pad), conv_out(in.w, k, stride, pad)};
    if (o.h <= 0 || o.w <= 0) return fail(CADNN_EINVAL, "cadnn_net_add_maxpool: empty output");
    NetOp op;
    op.kind = OP_MAXPOOL; op.k = k; op.stride = stride; op.pad = pad; op.src = src; op.dst = dst;
    op.in = in; op.out = o;
    if ((st = note_output(net, dst, o)) != CADNN_OK) return st;
    net->ops.push_back(op);
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_add_global_avgpool(cadnn_net* net, int src, int dst) {
    if (!net) return fail(CADNN_EINVAL, "cadnn_net_add_global_avgpool: NULL net");
    if (net->finalized) return fail(CADNN_EINVAL, "cadnn_net_add_global_avgpool: net already finalized");
    if (src == dst) return fail(CADNN_EINVAL, "cadnn_net_add_global_avgpool: dst aliases src");
    Shape in;
    cadnn_status st = src_shape(net, src, &in);
    if (st != CADNN_OK) return st;
    Shape o{in.n, in.c, 1, 1};
    NetOp op;
    op.kind = OP_AVGPOOL; op.src = src; op.dst = dst; op.in = in; op.out = o;
    if ((st = note_output(net, dst, o)) != CADNN_OK) return st;
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
    Shape in;
    cadnn_status st = src_shape(net, src, &in);
    if (st != CADNN_OK) return st;
    if ((size_t)in.c * in.h * in.w != (size_t)w->cin)
        return fail(CADNN_EINVAL, "cadnn_net_add_fc: %zu input features, weights take %d",
                    (size_t)in.c * in.h * in.w, w->cin);
    if ((st = cadnn_fc_prepare(w)) != CADNN_OK) return st;
    Shape o{in.n, w->cout, 1, 1};
    NetOp op;
    op.kind = OP_FC; op.w = w; op.bias = bias; op.relu = relu; op.src = src; op.dst = dst;
    op.in = in; op.out = o;
    if ((st = note_output(net, dst, o)) != CADNN_OK) return st;
    net->ops.push_back(op);
    return CADNN_OK;
}

static void layout_workspace(cadnn_net* net) {
    size_t off = 0;
    net->offset.clear();
    for (const auto& kv : net->max_elems) {
        if (kv.first == net->out_buf) continue;
        net->offset[kv.first] = off;
        off += (kv.second * net->elem() + 255) / 256 * 256;
    }
    net->ws_bytes = off;
}

extern "C" cadnn_status cadnn_net_workspace_bytes(const cadnn_net* net, size_t* bytes) {
    if (!net || !bytes) return fail(CADNN_EINVAL, "cadnn_net_workspace_bytes: NULL pointer");
    if (net->ops.empty()) return fail(CADNN_EINVAL, "cadnn_net_workspace_bytes: empty net");
    layout_workspace(const_cast<cadnn_net*>(net));
    *bytes = net->ws_bytes;
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_finalize(cadnn_net* net, void* ws, size_t bytes, int flags) {
    if (!net) return fail(CADNN_EINVAL, "cadnn_net_finalize: NULL net");
    if (net->ops.empty()) return fail(CADNN_EINVAL, "cadnn_net_finalize: empty net");
    // the output buffer is the caller's y: it must not also be read after a later write
    // to another buffer with the same id -- it is simply the last op's dst.
    for (const NetOp& op : net->ops)
        if (op.dst == net->out_buf && &op != &net->ops.back() && net->max_elems[op.dst] > net->ops.back().out.elems())
            return fail(CADNN_EINVAL, "cadnn_net_finalize: output buffer %d is also used for a larger intermediate", op.dst);
    layout_workspace(net);
    if (net->ws_bytes > 0 && !ws) return fail(CADNN_EINVAL, "cadnn_net_finalize: NULL workspace");
    if (bytes < net->ws_bytes) return fail(CADNN_EINVAL, "cadnn_net_finalize: workspace of %zu bytes, %zu needed", bytes, net->ws_bytes);
    drop_graph(net);
    net->ws = (char*)ws;
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
        // the inputs of every layer must hold finite, representative data while it is timed
        cadnn_status st = launch_all(net, x, y, s);
        for (size_t i = 0; i < net->ops.size() && st == CADNN_OK; ++i) {
            const NetOp& op = net->ops[i];
            if (op.kind != OP_CONV) continue;
            st = conv2d_tune_impl(op.w, buf_ptr(net, op.src, x, y), buf_ptr(net, op.dst, x, y), op.in.n,
                                  op.in.h, op.in.w, op.stride, op.pad, op.bias,
                                  op.res >= 0 ? buf_ptr(net, op.res, x, y) : nullptr, op.relu, s, 20, nullptr);
        }
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

extern "C" cadnn_status cadnn_net_read_buffer(cadnn_net* net, int buf, void* host_out, size_t bytes,
                                              void* stream) {
    if (!net || !host_out) return fail(CADNN_EINVAL, "cadnn_net_read_buffer: NULL pointer");
    if (!net->finalized) return fail(CADNN_EINVAL, "cadnn_net_read_buffer: net not finalized");
    auto it = net->offset.find(buf);
    if (it == net->offset.end()) return fail(CADNN_EINVAL, "cadnn_net_read_buffer: buffer %d is not in the workspace", buf);
    if (bytes > net->max_elems[buf] * net->elem()) return fail(CADNN_EINVAL, "cadnn_net_read_buffer: buffer %d is smaller than %zu bytes", buf, bytes);
    CADNN_HIP(hipStreamSynchronize((hipStream_t)stream));
    CADNN_HIP(hipMemcpy(host_out, net->ws + it->second, bytes, hipMemcpyDeviceToHost));
    return CADNN_OK;
}

extern "C" cadnn_status cadnn_net_free(cadnn_net* net) {
    if (net) {
        drop_graph(net);
        delete net;
    }
    return CADNN_OK;
}
