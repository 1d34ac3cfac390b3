/*
 * libcadnn -- sparse-weight x dense-activation CNN inference layers for AMD gfx950.
 *
 * The operations follow the CADNN paper's statement of the problem: weights are
 * pruned offline to unstructured sparsity (Section 3), stored compactly with
 * their indices, and each layer runs as convolution + folded batch-norm (bias)
 * + activation in ONE fused kernel (Section 4, "Model computation fusion and
 * transformation"); 1x1 convolutions are matrix multiplies (same paragraph) and
 * the filter layout is transformed for the device (Section 4, "Memory layout
 * transformation and load optimization").
 *
 * General conventions
 *   - Every call returns a cadnn_status; nothing throws or aborts.  The text of
 *     the last failure on the calling thread is available from cadnn_last_error().
 *   - Activations are NCHW, contiguous, in DEVICE memory owned by the caller.
 *     Element type is float for CADNN_F32 handles and IEEE binary16 for
 *     CADNN_F16 handles (products and sums are always taken in fp32).
 *     Bias vectors are always fp32 device arrays of `cout` elements.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Compute calls are asynchronous on that stream and do not synchronise.
 *   - Handles are opaque, owned by the library until the matching free call,
 *     and bound to the device that was current when they were created.
 *   - Host pointers are only read/written during the call that receives them.
 */
#ifndef CADNN_H
#define CADNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CADNN_OK = 0,
    CADNN_EINVAL = 1,        /* NULL pointer, non-positive size, empty output, mismatched handle */
    CADNN_EUNSUPPORTED = 2,  /* valid request this build has no kernel for */
    CADNN_ENOMEM = 3,        /* host or device allocation failed */
    CADNN_EHIP = 4           /* a HIP runtime call failed (text in cadnn_last_error) */
} cadnn_status;

typedef enum {
    CADNN_F32 = 0,           /* fp32 storage, fp32 accumulate */
    CADNN_F16 = 1,           /* fp16 storage (weights, activations, residual, output), fp32 accumulate */
    /* (not storage types: these two give the enumeration the range of int, so that any value
     * a caller passes is an argument the library can check and refuse with CADNN_EINVAL) */
    CADNN_DTYPE_RANGE_LO_ = -0x7fffffff - 1,
    CADNN_DTYPE_RANGE_HI_ = 0x7fffffff
} cadnn_dtype;

typedef struct cadnn_weights cadnn_weights;
typedef struct cadnn_net cadnn_net;

/* Text of the most recent error on this thread ("" if none).  Never NULL. */
const char* cadnn_last_error(void);

/* ------------------------------------------------------------------------- *
 * Weight packing (Section 3: pruned weights are exact zeros stored with their
 * indices; Section 4: filter layout transformed for the device).
 *
 * w_host: HOST pointer to the dense pruned tensor [cout][cin][kh][kw], fp32.
 * A fully connected layer is kh = kw = 1.  An entry is a nonzero iff its fp32
 * value != 0.  The canonical compact form is: row co = filter of output channel
 * co flattened over k = (ci*kh_ + r)*kw_ + c; entries of a row in ascending k;
 * rows ordered by nonzero count, descending, ties by ascending channel (so that
 * neighbouring rows -- which share a wavefront or workgroup -- carry balanced
 * work).  For CADNN_F16 values are rounded to nearest-even binary16 after the
 * fp32 nonzero test.  An all-zero tensor is valid.  Packing is pure host work
 * (no GPU needed); device-side layouts derived from the canonical form are
 * built on the first use of a layer geometry, on the device current at that
 * time (see cadnn_conv2d_prepare / cadnn_fc_prepare).
 * Errors: EINVAL for NULL / non-positive sizes; EUNSUPPORTED if cin*kh*kw or
 * cout exceed 2^24; ENOMEM.  *out is set to NULL on failure.
 * ------------------------------------------------------------------------- */
cadnn_status cadnn_pack_weights(const float* w_host, int cout, int cin, int kh, int kw,
                                cadnn_dtype dtype, cadnn_weights** out);
cadnn_status cadnn_free_weights(cadnn_weights* w);   /* NULL is accepted */

/* Number of stored nonzeros. */
cadnn_status cadnn_packed_nnz(const cadnn_weights* w, int64_t* nnz);
/* Copies the canonical form to HOST arrays: perm[cout], row_ptr[cout+1],
 * col_idx[nnz] (int32 k), vals[nnz] (float for F32 handles, uint16 binary16 bit
 * patterns for F16 handles).  Any output pointer may be NULL to skip it. */
cadnn_status cadnn_packed_export(const cadnn_weights* w, int32_t* perm, int32_t* row_ptr,
                                 int32_t* col_idx, void* vals);
/* Inverse of packing: writes the dense HOST tensor [cout][cin][kh][kw] (fp32;
 * for F16 handles the binary16 values widened exactly), zeros elsewhere. */
cadnn_status cadnn_unpack_weights(const cadnn_weights* w, float* w_host_out);

/* ------------------------------------------------------------------------- *
 * Fused sparse convolution layer (Section 4: conv + batch-norm + activation in
 * one kernel; batch-norm arrives pre-folded as `bias`):
 *
 *   y[n][co][oh][ow] = act( sum_{ci,r,c} W[co][ci][r][c] * X~[n][ci][oh*stride+r-pad][ow*stride+c-pad]
 *                           + bias[co] + residual[n][co][oh][ow] )
 *
 * X~ is x inside the image and 0 outside; hout = (h + 2*pad - kh)/stride + 1
 * (floor), wout likewise; act = ReLU if relu != 0 else identity.
 * x: device [n][cin][h][wdt]; y: device [n][cout][hout][wout]; bias: device
 * fp32 [cout] or NULL; residual: device, same shape/type as y, or NULL.
 * y must not overlap x.  residual may be y itself (in-place add: each element
 * is read before the same thread writes it) but must not partially overlap it.
 * The first call with a new (h, wdt, stride, pad, n) geometry may build and
 * upload a device layout (allocates, synchronous); call cadnn_conv2d_prepare
 * beforehand to keep the timed call allocation-free.
 * Sparse kernels serve 1x1 and 3x3 filters at any stride, 7x7 filters at strides 1 and 2,
 * other filter sizes while a tile of the input fits the LDS, and every filter size inside a
 * net (whose tensors carry zero halos); a geometry none of them serves, and any layer with
 * at least a quarter of its weights nonzero, may take the dense matrix-core kernel.
 * Errors: EINVAL (NULL x/y/w, sizes <= 0, stride <= 0, pad < 0, empty output);
 * EUNSUPPORTED (batch above 65535, a channel plane of 2^30 elements or more, or one
 * image of x or y of 2 GiB or more: the kernels address an image with 32-bit offsets); EHIP.
 * ------------------------------------------------------------------------- */
cadnn_status cadnn_sparse_conv2d(const cadnn_weights* w, const void* x, void* y, int n, int h,
                                 int wdt, int stride, int pad, const void* bias,
                                 const void* residual, int relu, void* stream);
/* Builds whatever device layout cadnn_sparse_conv2d would need for this geometry. */
cadnn_status cadnn_conv2d_prepare(const cadnn_weights* w, int n, int h, int wdt, int stride,
                                  int pad);

/* Kernel-variant selection (Section 4, "Optimization parameters selection": tile sizes
 * and work splits are chosen per layer).  cadnn_conv2d_tune times every kernel variant
 * that can serve this layer on the given tensors (`reps` launches each, events on
 * `stream`, synchronises, overwrites y) and pins the fastest for this (n, h, wdt,
 * stride, pad); best_us (may be NULL) receives its time per launch in microseconds.
 * Every timed launch follows a 64 MiB device copy that sweeps the L2 caches, because
 * inside a network a layer always starts cold (allocates 128 MiB for the duration).
 * cadnn_conv2d_list_variants writes the newline-separated names of the variants that
 * can serve the layer; cadnn_conv2d_set_variant pins one by name (NULL or "" removes
 * the pin, returning to the built-in heuristic).
 * Tuning frees only the trial layouts it built itself: a device layout that an ordinary
 * launch (or a finalized net, whose captured graph holds its address) has used stays
 * alive until cadnn_free_weights, so a handle may be tuned while a net uses it.  Launches
 * and tuning of ONE handle from several threads at once are serialised by the caller. */
cadnn_status cadnn_conv2d_tune(const cadnn_weights* w, const void* x, void* y, int n, int h,
                               int wdt, int stride, int pad, const void* bias,
                               const void* residual, int relu, void* stream, int reps,
                               float* best_us);
cadnn_status cadnn_conv2d_list_variants(const cadnn_weights* w, int n, int h, int wdt, int stride,
                                        int pad, char* buf, size_t len);
cadnn_status cadnn_conv2d_set_variant(const cadnn_weights* w, int n, int h, int wdt, int stride,
                                      int pad, const char* name);

/* Sparse fully connected layer: y[n][o] = act( sum_i W[o][i]*x[n][i] + bias[o] ).
 * (Section 3: the fully connected layers are pruned like the convolutions and kept as
 * values with indices; Section 4: a 1x1 convolution is a matrix product -- this is that
 * product on a one-pixel image, the classifier that ends each network of Section 5's
 * model table.)
 * w must have kh = kw = 1; x: device [n][cin]; y: device [n][cout]; bias: device fp32
 * [cout] or NULL.  Asynchronous on `stream`.  A zero weight (pruned, or the padding of the
 * device layout) never meets an activation its row does not read.  Errors: NULL pointer,
 * n <= 0, a handle that is a filter bank (CADNN_EINVAL); n above 8 * 65535
 * (CADNN_EUNSUPPORTED). */
cadnn_status cadnn_sparse_fc(const cadnn_weights* w, const void* x, void* y, int n,
                             const void* bias, int relu, void* stream);
/* Uploads the device arrays cadnn_sparse_fc needs (otherwise done on its first call). */
cadnn_status cadnn_fc_prepare(const cadnn_weights* w);

/* ------------------------------------------------------------------------- *
 * Fused depthwise convolution layer (Section 4 names depthwise convolution +
 * batch-norm + activation, as in MobileNet-V1, among the fused kernels): each
 * channel is filtered by its own kh x kw filter and channels are not summed,
 *
 *   y[n][c][oh][ow] = act( sum_{r,s} W[c][0][r][s] * X~[n][c][oh*stride+r-pad][ow*stride+s-pad] + bias[c] )
 *
 * w: a handle packed from the HOST tensor [channels][1][kh][kw] (cin = 1, cout =
 * channels); taps that are exactly zero are skipped.  x: device [n][channels][h][wdt];
 * y: device [n][channels][hout][wout], sizes as for cadnn_sparse_conv2d; bias: device fp32
 * [channels] or NULL.  y must not overlap x.  The first call uploads the filter
 * table (allocates, synchronous) unless cadnn_depthwise_prepare was called.
 * Errors: EINVAL (NULL pointer, sizes <= 0, pad < 0, empty output, a handle with
 * cin != 1); EUNSUPPORTED (more than 2^31 wavefronts of work); EHIP.
 * ------------------------------------------------------------------------- */
cadnn_status cadnn_depthwise_conv2d(const cadnn_weights* w, const void* x, void* y, int n, int h,
                                    int wdt, int stride, int pad, const void* bias, int relu,
                                    void* stream);
cadnn_status cadnn_depthwise_prepare(const cadnn_weights* w);

/* Pooling layers used between the convolutions of the benchmark networks.
 * (The paper describes no pooling operation; these are the layers that the published
 * architectures of the models in Section 5's model table place between convolutions.
 * No passage to cite.)
 * Max pooling takes the maximum over the in-image part of each k x k window
 * (padding never wins); windowed average pooling takes the mean over the in-image
 * part of each window (padding is neither summed nor counted; the 3x3 / stride 1
 * pools inside Inception-V3's modules); global average pooling writes
 * y[n][c] = mean over h*w. */
cadnn_status cadnn_maxpool2d(const void* x, void* y, int n, int c, int h, int wdt, int k,
                             int stride, int pad, cadnn_dtype dtype, void* stream);
cadnn_status cadnn_avgpool2d(const void* x, void* y, int n, int c, int h, int wdt, int k,
                             int stride, int pad, cadnn_dtype dtype, void* stream);
cadnn_status cadnn_global_avgpool(const void* x, void* y, int n, int c, int h, int wdt,
                                  cadnn_dtype dtype, void* stream);

/* Host-only view of the device layout ("plan") a kernel variant would read for this layer
 * (Section 3 counts the storage of a pruned model with and without its indices; Section 4
 * transforms the filter layout per device): no GPU is needed, nothing is uploaded or cached.
 * `variant` is a name from cadnn_conv2d_list_variants (NULL or "": the variant
 * cadnn_sparse_conv2d would launch).
 *   entries          stream entries the kernels walk: the nonzeros plus the zero-valued
 *                    entries that pad every part of a row to the kernels' unroll
 *   stream_bytes     bytes of values + indices of those entries as stored on the device
 *   alloc_bytes      device bytes of the stream arrays (parts start at a fixed stride in
 *                    some layouts; the gaps between them are allocated and never read)
 *   table_bytes      bytes of the per-row / per-part tables beside the stream
 *   bytes_per_nonzero  stream_bytes / nonzeros of the layer (0 if it has none)
 *   chunks           input-channel chunks an LDS-staged variant works through (else 1)
 *   lds_bytes        dynamic LDS of one workgroup (0: none or compiled in)
 * Errors: as cadnn_sparse_conv2d; CADNN_EINVAL if the name does not serve the layer. */
typedef struct cadnn_plan_info {
    int64_t entries;
    int64_t stream_bytes;
    int64_t alloc_bytes;
    int64_t table_bytes;
    double bytes_per_nonzero;
    int chunks;
    int lds_bytes;
} cadnn_plan_info;
cadnn_status cadnn_conv2d_plan_info(const cadnn_weights* w, int n, int h, int wdt, int stride, int pad,
                                    const char* variant, cadnn_plan_info* out);
/* The inverse of that layout transformation, for the variants with the compact 16-bit
 * tile-offset stream ("swide_*"): rebuilds the dense [cout][cin][kh][kw] fp32 tensor on the
 * HOST from the stream the kernel would read.  Equal to cadnn_unpack_weights element by
 * element when the layout loses nothing.  CADNN_EUNSUPPORTED for the other variants. */
cadnn_status cadnn_conv2d_plan_unpack(const cadnn_weights* w, int n, int h, int wdt, int stride, int pad,
                                      const char* variant, float* w_host_out);

/* Measurement aid, not part of the paper's method: a plain device-to-device streaming copy
 * of `bytes` bytes (a multiple of 16; 16-byte aligned pointers), whose memory traffic is
 * known exactly and against which hardware traffic counters are calibrated. */
cadnn_status cadnn_device_copy(const void* src, void* dst, size_t bytes, void* stream);

/* Measurement aid: the cost of one kernel boundary inside a replayed HIP graph, in
 * microseconds: `launches` (1..4096) dependent 16-byte copies are captured into a graph that
 * is replayed `reps` times on `stream` between two events.  scratch32: 32 bytes of device
 * memory the copies may overwrite.  Synchronises. */
cadnn_status cadnn_graph_launch_floor(void* scratch32, int launches, int reps, void* stream,
                                      float* us_per_launch);

/* Dense comparator on the same ABI (implicit-GEMM convolution over the dense
 * [cout][cin][kh][kw] DEVICE weight tensor, same fused epilogue), used for the
 * dense-vs-compressed comparison the paper reports (Section 5) and as the
 * fallback for layers that are not pruned. */
cadnn_status cadnn_dense_conv2d(const void* w_dev, const void* x, void* y, int n, int cin, int h,
                                int wdt, int cout, int kh, int kw, int stride, int pad,
                                const void* bias, const void* residual, int relu,
                                cadnn_dtype dtype, void* stream);

/* ------------------------------------------------------------------------- *
 * Whole-network runner (Section 5 measures single-image latency of a whole
 * network): an ordered list of ops over numbered activation buffers.  Buffer 0
 * is the network input (shape given at creation); the last op's dst buffer is
 * the network output.  All other tensors live in one caller-provided device
 * workspace, one region per op output; an output that feeds a padded convolution is
 * stored with a zero halo of that padding around every channel plane (the halo is
 * zeroed once in cadnn_net_finalize and never written), so those convolutions read
 * their zero padding from memory.  Buffer ids only express the wiring.  Weight
 * handles and bias arrays must outlive the net.
 *   create -> add_* (shapes are inferred and checked op by op) ->
 *   workspace_bytes -> finalize(workspace) -> run (any number of times) -> free
 * cadnn_run_net launches every op on `stream` in order (as one HIP graph launch
 * when graph capture was requested in finalize); x / y are the device input and
 * output tensors.  No host synchronisation inside.
 * ------------------------------------------------------------------------- */
cadnn_status cadnn_net_create(cadnn_dtype dtype, int n, int c, int h, int w, cadnn_net** out);
cadnn_status cadnn_net_add_conv(cadnn_net* net, const cadnn_weights* w, const void* bias_dev,
                                int stride, int pad, int relu, int src_buf, int dst_buf,
                                int residual_buf /* -1 = none */);
/* Depthwise layer (see cadnn_depthwise_conv2d); w must have cin = 1 and as many filters as
 * src_buf has channels. */
cadnn_status cadnn_net_add_depthwise(cadnn_net* net, const cadnn_weights* w, const void* bias_dev,
                                     int stride, int pad, int relu, int src_buf, int dst_buf);
cadnn_status cadnn_net_add_maxpool(cadnn_net* net, int k, int stride, int pad, int src_buf,
                                   int dst_buf);
cadnn_status cadnn_net_add_avgpool(cadnn_net* net, int k, int stride, int pad, int src_buf,
                                   int dst_buf);
cadnn_status cadnn_net_add_global_avgpool(cadnn_net* net, int src_buf, int dst_buf);
/* Channel concatenation (the branches of an Inception module): dst_buf holds the `count`
 * source buffers stacked along the channel axis in the given order; they must agree in batch,
 * height and width.  A source whose only reader is this op is written in place, into its
 * channel slice of dst_buf, by the op that produces it (no copy is launched for it); any
 * other source is copied. */
cadnn_status cadnn_net_add_concat(cadnn_net* net, const int* src_bufs, int count, int dst_buf);
cadnn_status cadnn_net_add_fc(cadnn_net* net, const cadnn_weights* w, const void* bias_dev,
                              int relu, int src_buf, int dst_buf);
/* Size of the workspace cadnn_net_finalize needs.  It depends on the layout flags below
 * (CADNN_NET_PLAIN_LAYOUT, CADNN_NET_NO_FUSION): the value is for flags 0 unless
 * cadnn_net_op_info has been called with other flags since the last op was added; finalize
 * refuses a workspace smaller than its own flags need. */
cadnn_status cadnn_net_workspace_bytes(const cadnn_net* net, size_t* bytes);
/* flags: CADNN_NET_GRAPH -- cadnn_run_net replays a captured HIP graph (re-captured
 * when x / y change between calls); CADNN_NET_TUNE -- the first cadnn_run_net call
 * first runs cadnn_conv2d_tune on every convolution with the net's own buffers, the
 * op that produces its input launched before every timed launch so that the caches are
 * as they will be (that first call synchronises and takes a fraction of a second);
 * CADNN_NET_PLAIN_LAYOUT -- keep every intermediate tensor in plain (haloed) NCHW; by
 * default the output of a convolution that is read by stride-2 convolutions is kept
 * de-interleaved by row/column parity, so those layers read it with unit stride (and a
 * large stride-2 layer whose input cannot be kept that way reads a de-interleaved copy made
 * right before it: cadnn_op_info.input_copy);
 * CADNN_NET_NO_FUSION -- launch every op on its own, in op-list order.  By default:
 *   - a 1x1 projection shortcut whose only reader adds it as residual is computed inside
 *     that reader; a global average pool that is the only reader of a small-image
 *     convolution is computed in that convolution's epilogue, and so is a 3x3 depthwise layer
 *     (padding 1, stride 1 or 2) that is the only reader of a convolution with an image of at
 *     most 28 x 28.  The skipped op reports fused_into, profile time zero and variant name
 *     "fused"; a buffer that is no longer written is refused by cadnn_net_read_buffer.
 *   - 1x1 stride-1 sparse convolutions with the same activation and no residual that read
 *     the same tensor are launched as one layer over the rows of all of them: the later ones
 *     report fused_into = the first one; their outputs are channel slices of the first
 *     one's region, from channel slice_channel on, and stay readable.
 *   - sparse convolutions on plain tensors whose inputs are all ready when an earlier one
 *     runs (the branches of an Inception module at the same depth; up to eight, window pools
 *     on workspace tensors included) are launched with it as one kernel over a table of
 *     launch records, while one variant serves all the layers: they report fused_into = that
 *     op and launched_with = 1; the op's variant name is the group's, and
 *     cadnn_net_op_candidates / cadnn_net_set_op_variant on it list / pin variants for the
 *     whole group.  Tuning (CADNN_NET_TUNE) keeps a group only if it beats its layers
 *     launched apart.
 *   - a window pool that rides on no launch moves up in the launch order to where its input
 *     completes (launched_after). */
#define CADNN_NET_GRAPH 1
#define CADNN_NET_TUNE 2
#define CADNN_NET_PLAIN_LAYOUT 4
#define CADNN_NET_NO_FUSION 8
/* CADNN_NET_STATIC_WORKSPACE -- the net's workspace is the library's own static device array
 * (workspace_dev and bytes are ignored): see cadnn_run_net_noalloc. */
#define CADNN_NET_STATIC_WORKSPACE 16
cadnn_status cadnn_net_finalize(cadnn_net* net, void* workspace_dev, size_t bytes, int flags);
/* Where the runner puts op `op_index`'s output and what it does with the op, as decided for
 * `flags` (the CADNN_NET_PLAIN_LAYOUT / CADNN_NET_NO_FUSION bits matter).  Pure host work: it
 * may be called before cadnn_net_finalize and needs no GPU.  cadnn_net_workspace_bytes reports
 * the size for the flags of the most recent of cadnn_net_op_info / cadnn_net_finalize (default
 * 0). */
typedef struct {
    int halo_h, halo_w;      /* zero halo rows / columns around every channel plane */
    int pitch;               /* elements per stored row */
    int64_t plane;           /* elements per stored channel plane */
    int64_t image;           /* elements from one image to the next */
    int deinterleaved;       /* 1 = split by row / column parity (read by stride-2 layers) */
    int64_t offset;          /* byte offset of channel 0 of image 0 in the workspace (the last
                                op writes the caller's y: its offset is 0 and means nothing) */
    int fused_into;          /* >= 0: the op launches nothing of its own: it is computed inside
                                that op, or (launched_with = 1) by the same kernel launch */
    int slice_of;            /* >= 0: the op writes in place into that concatenation's region */
    int slice_channel;       /* ... starting at this channel of it (for a sibling layer: of
                                the region of the op named by fused_into) */
    int launched_with;       /* 1: an independent layer that shares the kernel launch of op
                                fused_into; its tensors and its region are its own */
    int launched_after;      /* >= 0: the op is launched right behind that op instead of at its
                                place in the op list: a window pool moved up to where its
                                input completes (so that its reader can share an earlier
                                launch), or a member of a group that tuning took apart */
    int64_t input_copy;      /* >= 0: a large stride-2 layer (filter wider than 1x1) whose input is
                                not de-interleaved where it is produced reads a de-interleaved
                                copy of it, made right before the layer at this byte offset of
                                the workspace (not with CADNN_NET_PLAIN_LAYOUT) */
} cadnn_op_info;
cadnn_status cadnn_net_op_info(cadnn_net* net, int op_index, int flags, cadnn_op_info* out);
cadnn_status cadnn_run_net(cadnn_net* net, const void* x, void* y, void* stream);
/* cadnn_run_net for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  It allocates nothing, on the device or through any
 * allocating library routine, and launches the net's kernels one by one on `stream` (no graph
 * of its own).  The net's workspace -- every intermediate tensor -- is a static device array
 * of the library, 16 MiB per GPU, held until the process ends: the net must have been
 * finalized with CADNN_NET_STATIC_WORKSPACE (on the device that is current now), which
 * refuses a net that needs more with CADNN_EUNSUPPORTED and builds every device layout the
 * net's layers use.  x and y are the caller's, as in cadnn_run_net.  Every such net on a GPU
 * shares that one array, which keeps what the last call left: each call clears the part it
 * uses first (with a kernel), and calls that overlap on one GPU -- two streams, two threads --
 * race and must be serialised by the caller.  Errors: CADNN_EINVAL (NULL pointer, a net that
 * is not finalized, not finalized with CADNN_NET_STATIC_WORKSPACE, finalized on another
 * device or still waiting to be tuned, or a layer whose device layout is missing). */
cadnn_status cadnn_run_net_noalloc(cadnn_net* net, const void* x, void* y, void* stream);
/* Number of ops, and per-op device time: op i is launched `repeats` times back
 * to back between two HIP events on `stream` and the average is written to
 * ms_per_op[i] (cadnn_net_num_ops entries).  Synchronises the stream. */
cadnn_status cadnn_net_num_ops(const cadnn_net* net, int* num_ops);
cadnn_status cadnn_net_profile(cadnn_net* net, const void* x, void* y, void* stream, int repeats,
                               float* ms_per_op);
/* The same per-op times with the ops in launch order, as a forward pass runs them: an op then
 * finds the caches as the real pass leaves them (input just written by its producer, weights
 * last touched a pass ago) and not warm from its own previous launch.  Every kernel is
 * launched with start and stop marks of its own, so ms_per_op[i] is the device time of op i's
 * kernels and nothing else (what a kernel trace of the same pass reports), averaged over
 * `repeats` passes; 0 for ops that launch nothing.  Synchronises the stream. */
cadnn_status cadnn_net_profile_in_order(cadnn_net* net, const void* x, void* y, void* stream, int repeats,
                                        float* ms_per_op);
/* Name of the kernel serving op `op_index` (a conv variant name, "dwconv", "sfc", "maxpool",
 * "avgpool2d", "avgpool", "concat", or "fused" / "in place" for an op that launches nothing),
 * NUL-terminated into buf. */
cadnn_status cadnn_net_op_variant(const cadnn_net* net, int op_index, char* buf, size_t len);
/* Newline-separated names of the variants that can serve convolution op `op_index` in
 * the layout the net gave its input (a halo opens the linear-address kernels to 3x3). */
cadnn_status cadnn_net_op_candidates(const cadnn_net* net, int op_index, char* buf, size_t len);
/* Pins the kernel variant of convolution op `op_index` by name (as reported by
 * cadnn_net_op_variant after tuning), e.g. to replay a saved tuning result.  NULL or ""
 * returns the op to the built-in heuristic.  The net must be finalized.  On the first op of
 * a group of layers that share a launch the name pins the group's variant; "apart" there
 * takes the group apart for good: its layers are launched one by one, right behind that op. */
cadnn_status cadnn_net_set_op_variant(cadnn_net* net, int op_index, const char* name);
/* Copies the current contents of activation buffer `buf` (as left by the last
 * run) to a HOST array of `bytes` bytes; synchronises `stream`. */
cadnn_status cadnn_net_read_buffer(cadnn_net* net, int buf, void* host_out, size_t bytes,
                                   void* stream);
cadnn_status cadnn_net_free(cadnn_net* net);          /* NULL is accepted */

/* Name of the kernel variant cadnn_sparse_conv2d / cadnn_sparse_fc would launch
 * for this geometry, written to buf (NUL-terminated, truncated to len). */
cadnn_status cadnn_conv2d_variant_name(const cadnn_weights* w, int n, int h, int wdt, int stride,
                                       int pad, char* buf, size_t len);

#ifdef __cplusplus
}
#endif
#endif /* CADNN_H */
