"""GPU parity: every layer kind through the C ABI against the CPU oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from util import (TOL_F32, TOL_F16, F16_ULP, SUM_TOL, assert_close, assert_layer_close, assert_chain_close,
                  assert_net_close, cond_conv, cond_fc, cond_depthwise, chain_bounds, assert_within_bound)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def cad():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1905_00571_amd as cad
    cad.lib()
    return cad


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_conv(cad, x, w, b, r, stride, pad, relu, dtype=None):
    dtype = dtype if dtype is not None else cad.F32
    npdt = np.float16 if dtype == cad.F16 else np.float32
    xs = x.astype(npdt)
    rs = None if r is None else r.astype(npdt)
    h = cad.cadnn_pack_weights(w, dtype)
    y = cad.cadnn_sparse_conv2d(h, dev(xs), stride, pad, None if b is None else dev(b),
                                None if rs is None else dev(rs), relu)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    ref = oracle.conv2d(xs, w.astype(npdt), b, rs, stride, pad, relu, npdt)
    cond = cond_conv(xs, w.astype(npdt), b, rs, stride, pad)
    h.free()
    return got, ref, cond


def test_config0_single_conv(cad):
    """64->64 3x3 @56x56, 90 % sparse, stride 1, pad 1, bias, fused ReLU."""
    x = wl.activation((1, 64, 56, 56), "c0", 0, relu=True)
    w = wl.pruned_weights(64, 64, 3, 3, 0.9, "c0", 1)
    b = wl.bias_vector(64, "c0", 1)
    got, ref, cond = run_conv(cad, x, w, b, None, 1, 1, True)
    assert got.shape == (1, 64, 56, 56)
    print("C0", assert_layer_close(got, ref, cond, TOL_F32, "config 0"))


def test_config1_bottleneck_layers_and_chain(cad):
    ops = wl.bottleneck_conv2x_ops(0.85)
    shape = (1, 256, 56, 56)
    x, ws, bs = wl.net_tensors(ops, "c1", shape, input_relu=True)
    ref, ins, outs = oracle.run_net(ops, x, ws, bs)
    # each layer in isolation on the oracle's own input
    for i, op in enumerate(ops):
        h = cad.cadnn_pack_weights(ws[i])
        res = dev(ins[0]) if op.res == 0 else None
        y = cad.cadnn_sparse_conv2d(h, dev(ins[i]), op.stride, op.pad, dev(bs[i]), res, op.relu)
        torch.cuda.synchronize()
        cond = cond_conv(ins[i], ws[i], bs[i], ins[0] if op.res == 0 else None, op.stride, op.pad)
        assert_layer_close(y.cpu().numpy(), outs[i], cond, TOL_F32, f"bottleneck layer {op.name}")
        h.free()
    # and chained through the net runner, eager and graph
    for graph in (False, True):
        net = cad.build_net(ops, ws, bs, shape, cad.F32, use_graph=graph)
        xd = dev(x)
        for _ in range(3):
            y = net.run(xd)
            torch.cuda.synchronize()
            assert_chain_close(y.cpu().numpy(), ref, cond_conv(ins[2], ws[2], bs[2], ins[0], 1, 0),
                               TOL_F32, f"bottleneck chain graph={graph}")
        net.free()


GEOMS = [
    # cin, cout, k, stride, pad, h, w, sparsity
    (5, 7, 1, 1, 0, 9, 11, 0.5),
    (16, 24, 1, 2, 0, 14, 14, 0.9),
    (8, 8, 3, 1, 1, 7, 7, 0.5),
    (8, 8, 3, 1, 0, 9, 8, 0.0),
    (37, 19, 3, 1, 1, 30, 33, 0.9),       # ragged channels and tiles, several channel chunks
    (40, 20, 3, 2, 1, 29, 31, 0.8),
    (16, 16, 3, 2, 1, 14, 14, 0.99),
    (3, 8, 7, 2, 3, 37, 41, 0.0),
    (4, 6, 7, 1, 3, 12, 12, 0.5),
    (3, 5, 3, 1, 3, 6, 6, 0.3),           # pad larger than the kernel radius
    (300, 10, 1, 1, 0, 5, 5, 0.9),        # more channels than one 1x1 chunk
    (70, 33, 1, 1, 0, 40, 40, 0.7),
]


@pytest.mark.parametrize("geom", GEOMS)
def test_property_sweep(cad, geom):
    cin, cout, k, stride, pad, h, w_, s = geom
    tag = "sweep-%d-%d-%d-%d-%d" % (cin, cout, k, stride, pad)
    for n in (1, 3):
        x = wl.activation((n, cin, h, w_), tag, n, relu=False)
        w = wl.pruned_weights(cout, cin, k, k, s, tag, 1, mask="random")
        b = wl.bias_vector(cout, tag, 1, sigma=0.5)
        hout, wout = oracle.out_size(h, k, stride, pad), oracle.out_size(w_, k, stride, pad)
        r = wl.activation((n, cout, hout, wout), tag, 2, relu=False, role="r")
        for bias, res, relu in [(None, None, False), (b, r, True), (b, None, True), (None, r, False)]:
            got, ref, cond = run_conv(cad, x, w, bias, res, stride, pad, relu)
            assert_layer_close(got, ref, cond, TOL_F32, f"{geom} n={n} bias={bias is not None} res={res is not None}")


def test_degenerate_rows_and_all_zero(cad):
    x = wl.activation((2, 16, 12, 12), "degen", 0, relu=False)
    w = wl.pruned_weights(20, 16, 3, 3, 0.9, "degen", 1, row_skew=2.0)
    w[4] = 0
    w[11] = np.float32(0.125)
    b = wl.bias_vector(20, "degen", 1, sigma=1.0)
    r = wl.activation((2, 20, 12, 12), "degen", 2, relu=False, role="r")
    got, ref, cond = run_conv(cad, x, w, b, r, 1, 1, True)
    assert_layer_close(got, ref, cond, TOL_F32, "skewed rows")
    # all-zero weights: exactly act(bias + residual)
    got, ref, _ = run_conv(cad, x, np.zeros_like(w), b, r, 1, 1, True)
    assert np.array_equal(got, ref)
    # identity kernel: exactly ReLU(x)
    wi = np.zeros((16, 16, 3, 3), np.float32)
    for c in range(16):
        wi[c, c, 1, 1] = 1
    got, _, _ = run_conv(cad, x, wi, None, None, 1, 1, True)
    assert np.array_equal(got, np.maximum(x, 0))


def test_nan_poison_catches_unwritten_outputs(cad):
    x = wl.activation((1, 8, 19, 23), "poison", 0, relu=False)
    w = wl.pruned_weights(5, 8, 3, 3, 0.5, "poison", 1)
    h = cad.cadnn_pack_weights(w)
    out = torch.full((1, 5, 19, 23), float("nan"), device="cuda")
    cad.cadnn_sparse_conv2d(h, dev(x), 1, 1, None, None, False, out=out)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    h.free()


@pytest.mark.parametrize("geom", [(16, 24, 3, 1, 1, 14, 14, 0.8, 1), (32, 40, 1, 1, 0, 14, 14, 0.8, 2),
                                  (16, 24, 3, 2, 1, 15, 15, 0.7, 1), (24, 36, 3, 1, 1, 7, 7, 0.85, 3)])
def test_pruned_positions_never_touch_the_activation(cad, geom):
    """The definition of the layer does not read an activation whose weight is pruned, so a
    non-finite value there must not reach any output: input channel 0 is pruned in every row
    and holds Inf at every pixel.  The padding entries of the device plans (rows are padded to
    the kernels' unroll) carry a zero weight and must therefore point at an activation the row
    reads anyway -- 0 * Inf would be NaN.  Every sparse variant, both storage types."""
    cin, cout, k, stride, pad, h, w_, s, n = geom
    tag = "inf-%d-%d-%d-%d" % (cin, cout, k, stride)
    x = wl.activation((n, cin, h, w_), tag, 0, relu=False)
    x[:, 0] = np.inf
    w = wl.pruned_weights(cout, cin, k, k, s, tag, 1, row_skew=0.5)
    w[:, 0] = 0.0
    b = wl.bias_vector(cout, tag, 1, sigma=0.5)
    for dtype, npdt, tol in ((cad.F32, np.float32, TOL_F32), (cad.F16, np.float16, TOL_F16)):
        xs = x.astype(npdt)
        ref = oracle.conv2d(xs, w.astype(npdt), b, None, stride, pad, True, npdt)
        assert np.isfinite(ref).all()
        cond = cond_conv(xs, w.astype(npdt), b, None, stride, pad)
        hnd = cad.cadnn_pack_weights(w, dtype)
        names = [nm for nm in cad.cadnn_conv2d_list_variants(hnd, n, h, w_, stride, pad) if not nm.startswith("dense")]
        assert names, geom
        xd, bd = dev(xs), dev(b)
        for name in names:
            cad.cadnn_conv2d_set_variant(hnd, n, h, w_, stride, pad, name)
            y = cad.cadnn_sparse_conv2d(hnd, xd, stride, pad, bd, None, True)
            torch.cuda.synchronize()
            assert_layer_close(y.cpu().numpy(), ref, cond, tol, f"{geom} {name}", f16=dtype == cad.F16)
        hnd.free()
    # fully connected: column 0 pruned in every row, Inf there; row lengths of every remainder
    # modulo the kernels' group of four, with and without the LDS-staged kernel (batch > 1)
    for nb in (1, 3):
        xf = wl.activation((nb, 300), "inf-fc", 0, relu=False)
        xf[:, 0] = np.inf
        wf = wl.pruned_weights(50, 300, 1, 1, 0.7, "inf-fc", 1, row_skew=0.5)
        wf[:, 0] = 0.0
        for dtype, npdt, tol in ((cad.F32, np.float32, TOL_F32), (cad.F16, np.float16, TOL_F16)):
            hnd = cad.cadnn_pack_weights(wf, dtype)
            y = cad.cadnn_sparse_fc(hnd, dev(xf.astype(npdt)), None, False)
            torch.cuda.synchronize()
            ref = oracle.fc(xf.astype(npdt), wf.astype(npdt), None, False, npdt)
            assert_layer_close(y.cpu().numpy(), ref, cond_fc(xf.astype(npdt), wf.astype(npdt), None), tol,
                               f"fc batch {nb}", f16=dtype == cad.F16)
            hnd.free()


@pytest.mark.parametrize("n,cin,cout,s,relu", [(1, 2048, 1000, 0.9, False), (1, 300, 70, 0.5, True),
                                               (8, 512, 100, 0.96, True), (11, 64, 9, 0.0, False),
                                               (1, 25088, 256, 0.96, True), (3, 25088, 64, 0.96, True), (1, 25088, 1100, 0.96, True),
                                               (9, 2048, 1000, 0.9, False), (1, 48, 20000, 0.5, True),
                                               (2, 300, 1500, 0.3, True), (1, 70000, 12, 0.9, False),
                                               (10, 70000, 5, 0.99, True)])
def test_sparse_fc(cad, n, cin, cout, s, relu):
    tag = f"fc-{n}-{cin}-{cout}"
    x = wl.activation((n, cin), tag, 0, relu=True)
    w = wl.pruned_weights(cout, cin, 1, 1, s, tag, 1)
    if cout > 5:
        w[2] = 0
    b = wl.bias_vector(cout, tag, 1, sigma=0.1)
    h = cad.cadnn_pack_weights(w)
    y = cad.cadnn_sparse_fc(h, dev(x), dev(b), relu)
    torch.cuda.synchronize()
    assert_layer_close(y.cpu().numpy(), oracle.fc(x, w, b, relu), cond_fc(x, w, b), TOL_F32, tag)
    h.free()


@pytest.mark.parametrize("n,ch,h,w,kh,kw,stride,pad,s", [
    (1, 32, 112, 112, 3, 3, 1, 1, 0.0),     # MobileNet dw1: four pixels per lane
    (1, 64, 112, 112, 3, 3, 2, 1, 0.0),     # dw2: stride 2, four pixels per lane
    (2, 19, 23, 17, 3, 3, 1, 1, 0.3),       # ragged sizes, pruned taps, one pixel per lane
    (1, 1024, 7, 7, 3, 3, 1, 1, 0.0),       # dw13: 49 of 64 lanes
    (3, 7, 20, 24, 3, 3, 2, 0, 0.2),        # no padding
    (1, 6, 15, 13, 5, 3, 1, 2, 0.0),        # rectangular filter: run-time size path
    (2, 5, 16, 16, 3, 3, 3, 1, 0.0),        # stride 3: run-time path
    (1, 3, 9, 9, 1, 1, 1, 0, 0.0),          # 1x1 depthwise = per-channel scale
])
def test_depthwise(cad, n, ch, h, w, kh, kw, stride, pad, s):
    tag = f"dw-{n}-{ch}-{h}-{w}-{kh}{kw}-{stride}-{pad}"
    x = wl.activation((n, ch, h, w), tag, 0, relu=False)
    wt = wl.pruned_weights(ch, 1, kh, kw, s, tag, 1)
    if ch > 4:
        wt[3] = 0                                      # an all-zero filter: output = act(bias)
    b = wl.bias_vector(ch, tag, 1, sigma=0.1)
    hd = cad.cadnn_pack_weights(wt)
    for relu in (True, False):
        y = cad.cadnn_depthwise_conv2d(hd, dev(x), stride, pad, dev(b), relu)
        torch.cuda.synchronize()
        ref = oracle.depthwise_conv2d(x, wt, b, stride, pad, relu)
        assert_layer_close(y.cpu().numpy(), ref, cond_depthwise(x, wt, b, stride, pad), TOL_F32, tag)
    y = cad.cadnn_depthwise_conv2d(hd, dev(x), stride, pad, None, False)
    torch.cuda.synchronize()
    assert_layer_close(y.cpu().numpy(), oracle.depthwise_conv2d(x, wt, None, stride, pad, False),
                       cond_depthwise(x, wt, None, stride, pad), TOL_F32, tag + " no bias")
    hd.free()


def test_depthwise_fp16_and_errors(cad):
    x = wl.activation((2, 24, 28, 28), "dwh", 0, relu=True).astype(np.float16)
    wt = wl.pruned_weights(24, 1, 3, 3, 0.0, "dwh", 1)
    b = wl.bias_vector(24, "dwh", 1)
    hd = cad.cadnn_pack_weights(wt, cad.F16)
    w16 = wt.astype(np.float16)
    for stride in (1, 2):
        y = cad.cadnn_depthwise_conv2d(hd, dev(x), stride, 1, dev(b), True)
        torch.cuda.synchronize()
        assert y.dtype == torch.float16
        ref = oracle.depthwise_conv2d(x, w16, b, stride, 1, True, dtype=np.float16)
        assert_layer_close(y.cpu().numpy(), ref, cond_depthwise(x, w16, b, stride, 1), TOL_F16, "dw fp16", f16=True)
    hd.free()
    full = cad.cadnn_pack_weights(wl.pruned_weights(8, 8, 3, 3, 0.5, "dwh", 2))
    with pytest.raises(cad.CadnnError):
        cad.cadnn_depthwise_conv2d(full, dev(wl.activation((1, 8, 9, 9), "dwh", 3, relu=False)), 1, 1)
    full.free()


def test_pools(cad):
    x = wl.activation((2, 5, 23, 17), "pool", 0, relu=False)
    for k, s, p in [(3, 2, 1), (2, 2, 0)]:
        y = cad.cadnn_maxpool2d(dev(x), k, s, p)
        assert np.array_equal(y.cpu().numpy(), oracle.maxpool(x, k, s, p))
    y = cad.cadnn_global_avgpool(dev(x))
    assert_close(y.cpu().numpy(), oracle.global_avgpool(x), 1e-6, "avgpool")
    x16 = x.astype(np.float16)
    y = cad.cadnn_maxpool2d(dev(x16), 3, 2, 1)
    assert np.array_equal(y.cpu().numpy(), oracle.maxpool(x16, 3, 2, 1))
    # output rows that split into groups of 4 take the kernel with four outputs per thread; the
    # values are all negative, so a padding position read as zero would show
    for shape, p in [((2, 5, 24, 31), 1), ((3, 4, 25, 33), 0), ((1, 3, 8, 8), 1)]:
        xn = -np.abs(wl.activation(shape, "pool4", p, relu=False)) - 0.5
        for xx in (xn, xn.astype(np.float16)):
            y = cad.cadnn_maxpool2d(dev(xx), 3, 2, p)
            assert np.array_equal(y.cpu().numpy(), oracle.maxpool(xx, 3, 2, p)), (shape, p, xx.dtype)
    for k, s, p in [(3, 1, 1), (3, 2, 0), (2, 2, 0), (5, 1, 2)]:
        y = cad.cadnn_avgpool2d(dev(x), k, s, p)
        # an fp32 sum of at most k*k terms against the mean of their magnitudes
        d = np.abs(y.cpu().numpy().astype(np.float64) - oracle.avgpool(x, k, s, p, dtype=np.float64))
        assert (d <= 2e-6 * oracle.avgpool(np.abs(x), k, s, p, dtype=np.float64) + 1e-30).all(), (k, s, p, d.max())
    y = cad.cadnn_avgpool2d(dev(x16), 3, 1, 1)
    # fp16 storage: the same fp32 sum, rounded once to fp16 (both sides round a value that
    # agrees to the summation bound, so they differ by at most one rounding step)
    ref16 = oracle.avgpool(x16, 3, 1, 1, dtype=np.float64)
    d = np.abs(y.cpu().numpy().astype(np.float64) - oracle.avgpool(x16, 3, 1, 1).astype(np.float64))
    assert (d <= 2e-6 * oracle.avgpool(np.abs(x16), 3, 1, 1, dtype=np.float64) + F16_ULP * np.abs(ref16) + 1e-30).all(), d.max()


def test_fp16_storage_variant(cad):
    x = wl.activation((2, 32, 28, 28), "h", 0, relu=True)
    w = wl.pruned_weights(48, 32, 3, 3, 0.8, "h", 1)
    b = wl.bias_vector(48, "h", 1)
    r = wl.activation((2, 48, 28, 28), "h", 2, relu=False, role="r")
    got, ref, cond = run_conv(cad, x, w, b, r, 1, 1, True, dtype=cad.F16)
    assert got.dtype == np.float16
    assert_layer_close(got, ref, cond, TOL_F16, "fp16 3x3", f16=True)
    w1 = wl.pruned_weights(40, 32, 1, 1, 0.5, "h", 3)
    got, ref, cond = run_conv(cad, x, w1, None, None, 2, 0, False, dtype=cad.F16)
    assert_layer_close(got, ref, cond, TOL_F16, "fp16 1x1 s2", f16=True)
    # fc
    xf = wl.activation((3, 200), "h", 4, relu=True).astype(np.float16)
    wf = wl.pruned_weights(30, 200, 1, 1, 0.7, "h", 5)
    h = cad.cadnn_pack_weights(wf, cad.F16)
    y = cad.cadnn_sparse_fc(h, dev(xf), None, False)
    torch.cuda.synchronize()
    assert_layer_close(y.cpu().numpy(), oracle.fc(xf, wf.astype(np.float16), None, False, np.float16),
                       cond_fc(xf, wf.astype(np.float16), None), TOL_F16, "fp16 fc", f16=True)
    h.free()


def test_runtime_error_paths(cad):
    h = cad.cadnn_pack_weights(wl.pruned_weights(8, 4, 3, 3, 0.5, "err", 1))
    x = dev(wl.activation((1, 4, 8, 8), "err", 0, relu=False))
    L = cad.lib()
    y = torch.empty((1, 8, 8, 8), device="cuda")
    assert L.cadnn_sparse_conv2d(h.handle, x.data_ptr(), x.data_ptr(), 1, 8, 8, 1, 1, None, None, 0, None) == 1
    assert L.cadnn_sparse_conv2d(h.handle, x.data_ptr(), None, 1, 8, 8, 1, 1, None, None, 0, None) == 1
    assert L.cadnn_sparse_conv2d(h.handle, x.data_ptr(), y.data_ptr(), 1, 8, 8, 1, 1, None, None, 0, None) == 0
    torch.cuda.synchronize()
    h.free()


VARIANT_GEOMS = [
    # cin, cout, k, stride, pad, h, w, sparsity, n
    (24, 20, 3, 1, 1, 19, 21, 0.8, 2),
    (40, 12, 3, 2, 1, 30, 27, 0.7, 1),
    (70, 37, 1, 1, 0, 23, 9, 0.85, 2),
    (48, 16, 1, 2, 0, 14, 14, 0.5, 1),
    (3, 9, 7, 2, 3, 40, 33, 0.0, 1),
    (520, 6, 3, 1, 1, 7, 7, 0.9, 1),      # long rows: exercises the channel-split variants
    (37, 70, 3, 2, 1, 21, 17, 0.5, 2),    # dense enough for the matrix-core fallback too
    (19, 33, 1, 1, 0, 9, 9, 0.0, 1),
    (40, 24, 1, 1, 0, 12, 20, 0.8, 2),    # even width: adjacent-pixel wide loads
    (40, 3, 3, 2, 1, 30, 27, 0.0, 2),     # unpruned, few input channels (a network's first layer)
    # whole 32-channel steps and a few thousand pixels: the 128 x 128-tile matrix-core kernel
    # is a candidate too (fp16 storage), whatever the sparsity
    (64, 150, 3, 1, 1, 30, 25, 0.8, 3),
    (32, 40, 3, 2, 1, 41, 37, 0.6, 4),
    (96, 130, 1, 1, 0, 29, 31, 0.85, 3),
    # long K on few pixels: the variants that split K over several workgroups per output tile
    (160, 70, 3, 1, 1, 12, 11, 0.8, 2),
    (256, 40, 3, 1, 1, 9, 9, 0.9, 4),
    # images of at most 16 groups of 4 adjacent pixels: four packed rows per wave (pixel-wise, and
    # a 3x3 filter without padding, which needs no halo on a plain tensor)
    (96, 50, 1, 1, 0, 7, 7, 0.8, 3),
    (72, 41, 3, 1, 0, 9, 10, 0.85, 2),
]


@pytest.mark.parametrize("geom", [(12, 9, 5, 1, 2, 19, 23, 0.8, 2), (5, 11, 7, 3, 3, 19, 9, 0.9, 1),
                                  (6, 4, 5, 2, 0, 11, 13, 1.0, 1), (7, 5, 2, 1, 1, 9, 8, 0.85, 1)])
def test_geometries_without_a_sparse_kernel_run_dense(cad, geom):
    """Filter sizes and strides off the beaten track on a plain tensor (5x5, 7x7 at stride 3,
    2x2): whatever serves them -- the LDS-staged family while a tile of the input fits, else
    the matrix-core kernel at any sparsity, an all-zero filter bank included -- every valid
    geometry has at least one variant and each of them meets the bar."""
    cin, cout, k, stride, pad, h, w_, s, n = geom
    tag = "odd-%d-%d-%d-%d" % (cin, cout, k, stride)
    x = wl.activation((n, cin, h, w_), tag, 0, relu=False)
    w = wl.pruned_weights(cout, cin, k, k, s, tag, 1)
    b = wl.bias_vector(cout, tag, 1, sigma=0.5)
    for dtype, npdt, tol in ((cad.F32, np.float32, TOL_F32), (cad.F16, np.float16, TOL_F16)):
        xs = x.astype(npdt)
        hnd = cad.cadnn_pack_weights(w, dtype)
        names = cad.cadnn_conv2d_list_variants(hnd, n, h, w_, stride, pad)
        assert names, geom
        if stride == 3:
            assert all(nm.startswith("dense_mfma") for nm in names), names
        ref = oracle.conv2d(xs, w.astype(npdt), b, None, stride, pad, True, npdt)
        cond = cond_conv(xs, w.astype(npdt), b, None, stride, pad)
        for name in [None] + names:
            cad.cadnn_conv2d_set_variant(hnd, n, h, w_, stride, pad, name)
            y = cad.cadnn_sparse_conv2d(hnd, dev(xs), stride, pad, dev(b), None, True)
            torch.cuda.synchronize()
            assert_layer_close(y.cpu().numpy(), ref, cond, tol, f"{geom} {name}", f16=dtype == cad.F16)
        hnd.free()


@pytest.mark.parametrize("geom", VARIANT_GEOMS)
def test_every_kernel_variant(cad, geom):
    """Each instantiated kernel variant that can serve a layer is pinned in turn and must
    meet the same bar (both activation storage types)."""
    cin, cout, k, stride, pad, h, w_, s, n = geom
    tag = "var-%d-%d-%d-%d" % (cin, cout, k, stride)
    x = wl.activation((n, cin, h, w_), tag, 0, relu=False)
    w = wl.pruned_weights(cout, cin, k, k, s, tag, 1, row_skew=0.5)
    b = wl.bias_vector(cout, tag, 1, sigma=0.5)
    hout, wout = oracle.out_size(h, k, stride, pad), oracle.out_size(w_, k, stride, pad)
    r = wl.activation((n, cout, hout, wout), tag, 2, relu=False, role="r")
    for dtype, npdt, tol in ((cad.F32, np.float32, TOL_F32), (cad.F16, np.float16, TOL_F16)):
        xs, rs = x.astype(npdt), r.astype(npdt)
        ref = oracle.conv2d(xs, w.astype(npdt), b, rs, stride, pad, True, npdt)
        cond = cond_conv(xs, w.astype(npdt), b, rs, stride, pad)
        hnd = cad.cadnn_pack_weights(w, dtype)
        names = cad.cadnn_conv2d_list_variants(hnd, n, h, w_, stride, pad)
        assert names, geom
        if dtype == cad.F16 and cin % 32 == 0 and n * hout * wout >= 2048:
            assert "dense_mfma__Float16_128x128x32" in names, names
        if dtype == cad.F16 and cin * k * k // 32 >= 64 and cin % 32 == 0:
            assert "dense_mfma__Float16_64x64x32w_k8" in names, names
        # (in 2-byte storage a row that does not split into groups of 4 needs a halo row behind the image)
        if pad == 0 and stride == 1 and hout * ((wout + 3) // 4) <= 16 and (dtype == cad.F32 or wout % 4 == 0):
            assert [nm for nm in names if nm.startswith("squad_") and "_r4" in nm] and [nm for nm in names if "_r2" in nm], names
        xd, rd, bd = dev(xs), dev(rs), dev(b)
        for name in names:
            cad.cadnn_conv2d_set_variant(hnd, n, h, w_, stride, pad, name)
            assert cad.cadnn_conv2d_variant_name(hnd, n, h, w_, stride, pad) == name
            out = torch.full((n, cout, hout, wout), float("nan"), device="cuda", dtype=xd.dtype)
            cad.cadnn_sparse_conv2d(hnd, xd, stride, pad, bd, rd, True, out=out)
            torch.cuda.synchronize()
            assert_layer_close(out.cpu().numpy(), ref, cond, tol, f"{geom} {name}", f16=dtype == cad.F16)
        # tuning pins one of them and the result still matches
        out = torch.empty((n, cout, hout, wout), device="cuda", dtype=xd.dtype)
        us = cad.cadnn_conv2d_tune(hnd, xd, out, stride, pad, bd, rd, True, reps=3)
        assert us > 0 and cad.cadnn_conv2d_variant_name(hnd, n, h, w_, stride, pad) in names
        cad.cadnn_sparse_conv2d(hnd, xd, stride, pad, bd, rd, True, out=out)
        torch.cuda.synchronize()
        assert_layer_close(out.cpu().numpy(), ref, cond, tol, f"{geom} tuned", f16=dtype == cad.F16)
        cad.cadnn_conv2d_set_variant(hnd, n, h, w_, stride, pad, None)
        hnd.free()


@pytest.mark.parametrize("geom", [(3, 64, 7, 2, 3, 56, 56, 1), (64, 64, 3, 1, 1, 28, 28, 2),
                                  (100, 70, 1, 1, 0, 13, 13, 1), (33, 40, 3, 2, 1, 19, 23, 1),
                                  (16, 8, 5, 1, 2, 11, 11, 1),
                                  # whole 32-channel steps: in fp16 storage the 128 x 128-tile kernel
                                  (32, 200, 3, 2, 1, 19, 23, 3), (96, 130, 1, 1, 0, 13, 13, 2),
                                  (32, 16, 7, 2, 3, 30, 30, 1), (64, 70, 5, 1, 2, 11, 11, 1),
                                  (128, 129, 3, 1, 2, 9, 14, 5)])
def test_dense_comparator(cad, geom):
    """cadnn_dense_conv2d (matrix-core implicit GEMM over the dense tensor) meets the same bar."""
    cin, cout, k, stride, pad, h, w_, n = geom
    tag = "dense-%d-%d-%d-%d" % (cin, cout, k, stride)
    x = wl.activation((n, cin, h, w_), tag, 0, relu=False)
    w = wl.pruned_weights(cout, cin, k, k, 0.3, tag, 1)
    b = wl.bias_vector(cout, tag, 1, sigma=0.5)
    hout, wout = oracle.out_size(h, k, stride, pad), oracle.out_size(w_, k, stride, pad)
    r = wl.activation((n, cout, hout, wout), tag, 2, relu=False, role="r")
    for npdt, tol, f16 in ((np.float32, TOL_F32, False), (np.float16, TOL_F16, True)):
        xs, rs, wsd = x.astype(npdt), r.astype(npdt), w.astype(npdt)
        ref = oracle.conv2d(xs, wsd, b, rs, stride, pad, True, npdt)
        cond = cond_conv(xs, wsd, b, rs, stride, pad)
        y = cad.cadnn_dense_conv2d(dev(wsd), dev(xs), stride, pad, dev(b), dev(rs), True)
        torch.cuda.synchronize()
        assert_layer_close(y.cpu().numpy(), ref, cond, tol, f"dense {geom} f16={f16}", f16=f16)
        y = cad.cadnn_dense_conv2d(dev(wsd), dev(xs), stride, pad, None, None, False)
        torch.cuda.synchronize()
        ref = oracle.conv2d(xs, wsd, None, None, stride, pad, False, npdt)
        assert_layer_close(y.cpu().numpy(), ref, cond_conv(xs, wsd, None, None, stride, pad), tol,
                           f"dense {geom} plain f16={f16}", f16=f16)


@pytest.mark.parametrize("geom", [(24, 20, 3, 1, 1, 18, 20, 0.8, 2), (16, 12, 3, 2, 1, 15, 17, 0.7, 1),
                                  # odd widths over several pixel tiles: the ragged-row variants
                                  (24, 20, 3, 1, 1, 13, 19, 0.8, 2), (10, 14, 5, 1, 2, 21, 35, 0.8, 1),
                                  (130, 9, 3, 1, 1, 7, 7, 0.9, 1), (12, 10, 3, 1, 1, 14, 14, 0.5, 1),
                                  # enough channels that the LDS families stage them chunk by chunk
                                  (600, 12, 3, 1, 1, 14, 14, 0.9, 1), (520, 8, 3, 2, 1, 14, 14, 0.9, 2)])
def test_every_variant_on_a_haloed_input(cad, geom):
    """Inside a net the input of a 3x3 layer carries a zero halo, which opens the
    linear-address kernels to it: a 1x1 producer feeds the 3x3 layer and every variant that
    can serve the 3x3 layer there is pinned in turn (both storage types)."""
    cin, cout, k, stride, pad, h, w_, s, n = geom
    tag = "halo-%d-%d-%d-%d" % (cin, cout, k, stride)
    ops = [wl.Op("conv", "pre", 0, 1, 8, cin, 1, 1, 0, 0.3, True),
           wl.Op("conv", "main", 1, 2, cin, cout, k, stride, pad, s, True),
           wl.Op("conv", "post", 2, 3, cout, 6, 1, 1, 0, 0.2, False)]
    shape = (n, 8, h, w_)
    x, ws, bs = wl.net_tensors(ops, tag, shape, input_relu=True)
    for dtype, npdt, tol in ((cad.F32, np.float32, TOL_F32), (cad.F16, np.float16, TOL_F16)):
        xs = x.astype(npdt)
        ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
        cond = cond_conv(ins[1], ws[1].astype(npdt), bs[1], None, stride, pad)
        net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False)
        names = net.op_candidates(1)
        assert any(nm.startswith("slinear") for nm in names), names
        if stride == 1 and w_ % 2 == 1:
            assert any("_g2_" in nm for nm in names) and any("_g4_" in nm for nm in names), names
        xd = dev(xs)
        for name in names:
            net.set_op_variant(1, name)
            assert net.op_variant(1) == name
            y = net.run(xd)
            torch.cuda.synchronize()
            mid = net.read_buffer(2, outs[1].shape)
            assert_layer_close(mid, outs[1], cond, tol, f"{geom} {name}", f16=dtype == cad.F16)
        net.free()


@pytest.mark.parametrize("geom", [(12, 12, 1), (20, 28, 2), (14, 14, 3)])
def test_every_variant_on_deinterleaved_tensors(cad, geom):
    """The output of a convolution read by stride-2 convolutions is kept de-interleaved by
    row/column parity inside a net.  A downsampling bottleneck (1x1 -> 3x3/2 -> 1x1 plus a
    1x1/2 projection shortcut) behind a 1x1 producer exercises every role: writing such a
    tensor, reading it pixel-wise, reading it with a strided 3x3 and with a strided 1x1.
    Every variant that can serve each layer is pinned in turn and every intermediate tensor
    is compared with the oracle; the same net in plain layout must agree."""
    h, w_, n = geom
    # (layers around a de-interleaved tensor must be too sparse for the dense family)
    ops = [wl.Op("conv", "t", 0, 1, 8, 16, 1, 1, 0, 0.8, True),
           wl.Op("conv", "a", 1, 2, 16, 8, 1, 1, 0, 0.8, True),
           wl.Op("conv", "b", 2, 3, 8, 8, 3, 2, 1, 0.85, True),
           wl.Op("conv", "p", 1, 4, 16, 16, 1, 2, 0, 0.8, False),
           wl.Op("conv", "c", 3, 5, 8, 16, 1, 1, 0, 0.3, True, 4),
           wl.Op("conv", "post", 5, 6, 16, 6, 1, 1, 0, 0.2, False)]
    shape = (n, 8, h, w_)
    x, ws, bs = wl.net_tensors(ops, "s2d-%d-%d" % (h, w_), shape, input_relu=True)
    for dtype, npdt, tol in ((cad.F32, np.float32, TOL_F32), (cad.F16, np.float16, TOL_F16)):
        xs = x.astype(npdt)
        ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
        net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False, fuse=False)
        plain = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False, plain_layout=True, fuse=False)
        xd = dev(xs)
        for i in range(5):
            names = net.op_candidates(i)
            # (in 2-byte storage the large-tile matrix-core kernels are candidates as well)
            assert names and (i == 4 or all(nm.startswith(("slinear", "squad", "swide", "dense_mfma__Float16_")) for nm in names)), (i, names)
            r = outs[3] if ops[i].res >= 0 else None
            cond = cond_conv(ins[i], ws[i].astype(npdt), bs[i], r, ops[i].stride, ops[i].pad)
            for name in names:
                net.set_op_variant(i, name)
                assert net.op_variant(i) == name
                net.run(xd)
                torch.cuda.synchronize()
                got = net.read_buffer(ops[i].dst, outs[i].shape)
                assert_layer_close(got, outs[i], cond, tol, f"{geom} op {ops[i].name} {name}", f16=dtype == cad.F16)
        y = net.run(xd)
        yp = plain.run(xd)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), yp.cpu().numpy()) or np.allclose(
            y.cpu().numpy().astype(np.float64), yp.cpu().numpy().astype(np.float64), rtol=0, atol=tol * np.abs(ref).max())
        net.free()
        plain.free()


@pytest.mark.parametrize("geom", [(12, 12, 1, 2), (20, 28, 2, 2), (14, 14, 3, 1), (9, 11, 2, 1)])
def test_fused_projection_shortcut(cad, geom):
    """A 1x1 projection shortcut whose only reader adds it as residual is computed inside
    that reader: the projection op reports "fused", its buffer is never materialised, and
    every dual-input variant of the reader must reproduce the oracle's block output -- with
    the block input de-interleaved (stride-2 block) or plain (stride-1 block), both storage
    types, and the same as the net without fusion."""
    h, w_, n, stride = geom
    ops = [wl.Op("conv", "t", 0, 1, 8, 16, 1, 1, 0, 0.8, True),
           wl.Op("conv", "a", 1, 2, 16, 8, 1, 1, 0, 0.8, True),
           wl.Op("conv", "b", 2, 3, 8, 8, 3, stride, 1, 0.85, True),
           wl.Op("conv", "p", 1, 4, 16, 24, 1, stride, 0, 0.8, False),
           wl.Op("conv", "c", 3, 5, 8, 24, 1, 1, 0, 0.8, True, 4),
           wl.Op("conv", "post", 5, 6, 24, 6, 1, 1, 0, 0.2, False)]
    shape = (n, 8, h, w_)
    x, ws, bs = wl.net_tensors(ops, "fuse-%d-%d-%d" % (h, w_, stride), shape, input_relu=True)
    for dtype, npdt, tol in ((cad.F32, np.float32, TOL_F32), (cad.F16, np.float16, TOL_F16)):
        xs = x.astype(npdt)
        ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
        net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False)
        unfused = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False, fuse=False)
        xd = dev(xs)
        assert net.op_variant(3) == "fused" and unfused.op_variant(3) != "fused"
        with pytest.raises(cad.CadnnError):
            net.read_buffer(4, outs[3].shape)
        names = net.op_candidates(4)
        assert names and all("_f" in nm for nm in names), names
        # what is summed now: the layer's own terms and the shortcut's
        cond = cond_conv(ins[4], ws[4].astype(npdt), bs[4], None, 1, 0) + \
            cond_conv(ins[3], ws[3].astype(npdt), bs[3], None, stride, 0)
        for name in names:
            net.set_op_variant(4, name)
            assert net.op_variant(4) == name
            y = net.run(xd)
            torch.cuda.synchronize()
            got = net.read_buffer(5, outs[4].shape)
            # fp16: the unfused definition rounds the shortcut to fp16 before adding it
            extra_tol = 2.0 ** -10 * np.abs(outs[3].astype(np.float64)) if dtype == cad.F16 else 0.0
            d = np.abs(got.astype(np.float64) - outs[4].astype(np.float64))
            bound = 1e-4 * cond + (2.0 ** -10 if dtype == cad.F16 else 0.0) * np.abs(outs[4].astype(np.float64)) + extra_tol + 1e-30
            assert (d <= bound).all(), f"{geom} {name}: worst ratio {(d / bound).max():.3f}"
            assert d.max() / np.abs(outs[4]).max() <= tol
        yf = net.run(xd).cpu().numpy().astype(np.float64)
        yu = unfused.run(xd).cpu().numpy().astype(np.float64)
        torch.cuda.synchronize()
        assert np.abs(yf - yu).max() <= tol * np.abs(ref).max()
        net.free()
        unfused.free()


@pytest.mark.parametrize("geom", [(20, 28, 2, 2), (13, 11, 7, 2), (14, 14, 2, 1)])
def test_matrix_core_variants_in_a_bottleneck(cad, geom):
    """In 2-byte storage the large-tile matrix-core kernels are candidates for every layer with
    whole 32-channel steps, whatever its sparsity.  A downsampling bottleneck with such channel
    counts puts them in every role a net has: writing and reading de-interleaved tensors
    (pixel-wise, with a strided 3x3 and with a strided 1x1), reading a haloed input, adding a
    residual, and computing a fused projection shortcut as more of the contraction.  Each is
    pinned in turn and the layer's output compared with the oracle."""
    h, w_, n, stride = geom
    ops = [wl.Op("conv", "t", 0, 1, 8, 64, 1, 1, 0, 0.5, True),
           wl.Op("conv", "a", 1, 2, 64, 32, 1, 1, 0, 0.8, True),
           wl.Op("conv", "b", 2, 3, 32, 32, 3, stride, 1, 0.85, True),
           wl.Op("conv", "p", 1, 4, 64, 136, 1, stride, 0, 0.8, False),
           wl.Op("conv", "c", 3, 5, 32, 136, 1, 1, 0, 0.8, True, 4),
           wl.Op("conv", "post", 5, 6, 136, 6, 1, 1, 0, 0.2, False)]
    shape = (n, 8, h, w_)
    x, ws, bs = wl.net_tensors(ops, "mfma-%d-%d-%d" % (h, w_, stride), shape, input_relu=True)
    npdt, tol = np.float16, TOL_F16
    xs = x.astype(npdt)
    ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
    bounds = chain_bounds(ops, ins, outs, ws, bs, True)
    xd = dev(xs)
    for fuse in (False, True):
        net = cad.build_net(ops, ws, bs, shape, cad.F16, use_graph=False, fuse=fuse)
        assert (net.op_variant(3) == "fused") == fuse
        for i in (1, 2, 3, 4):
            if fuse and i == 3:
                continue
            names = [nm for nm in net.op_candidates(i) if nm.startswith("dense_mfma__Float16_") and not nm.endswith("_64x64x32")]
            assert len([nm for nm in names if "_k" not in nm and "_h" not in nm]) == 4, (i, net.op_candidates(i))
            for name in names:
                net.set_op_variant(i, name)
                assert net.op_variant(i) == name
                net.run(xd)
                torch.cuda.synchronize()
                got = net.read_buffer(ops[i].dst, outs[i].shape)
                # (the layer's input is what the net's own earlier layers left: the bound of
                # the chain up to here, not of the layer alone)
                assert_within_bound(got, outs[i], bounds[i], f"{geom} fuse={fuse} op {ops[i].name} {name}")
                assert np.abs(got.astype(np.float64) - outs[i].astype(np.float64)).max() <= tol * np.abs(outs[i]).max()
        net.free()


@pytest.mark.parametrize("dtype_name", ["f32", "f16"])
@pytest.mark.parametrize("geom", [(7, 7, 2, 1), (14, 14, 1, 2), (8, 8, 3, 1), (5, 6, 2, 1), (16, 12, 2, 2), (10, 6, 2, 1)])
def test_several_rows_per_wave_in_a_bottleneck(cad, geom, dtype_name):
    """The small-image kernels (four packed rows per wave with 16 lanes of 4 adjacent pixels per
    row, or two with 32 lanes of 2 pixels)
    in the roles a net gives them: pixel-wise on a plain tensor, a 3x3 filter on a tensor with
    a halo, a strided 3x3 on a de-interleaved tensor, widths that do and do not split into
    groups of 4, a residual.  Each instantiation is pinned in turn and the layer's output
    compared with the oracle."""
    h, w_, n, stride = geom
    ops = [wl.Op("conv", "t", 0, 1, 8, 40, 1, 1, 0, 0.5, True),
           wl.Op("conv", "a", 1, 2, 40, 24, 1, 1, 0, 0.8, True),
           wl.Op("conv", "b", 2, 3, 24, 50, 3, stride, 1, 0.85, True),
           wl.Op("conv", "p", 1, 4, 40, 70, 1, stride, 0, 0.8, False),
           wl.Op("conv", "c", 3, 5, 50, 70, 1, 1, 0, 0.8, True, 4),
           wl.Op("conv", "post", 5, 6, 70, 6, 1, 1, 0, 0.2, False)]
    shape = (n, 8, h, w_)
    f16 = dtype_name == "f16"
    npdt, tol = (np.float16, TOL_F16) if f16 else (np.float32, TOL_F32)
    x, ws, bs = wl.net_tensors(ops, "quad-%d-%d-%d" % (h, w_, stride), shape, input_relu=True)
    xs = x.astype(npdt)
    ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
    bounds = chain_bounds(ops, ins, outs, ws, bs, f16)
    xd = dev(xs)
    net = cad.build_net(ops, ws, bs, shape, cad.F16 if f16 else cad.F32, use_graph=False, fuse=False)
    seen = 0
    for i in (1, 2, 4):
        names = [nm for nm in net.op_candidates(i) if nm.startswith("squad_")]
        small = outs[i].shape[2] * ((outs[i].shape[3] + 3) // 4) <= 16      # (10 x 6: only two rows per wave fit)
        # (the layer in front of a strided 3x3 writes a de-interleaved tensor: not offered there)
        # and in 2-byte storage ragged rows need an input with a halo, which only the 3x3 layer has)
        if small and not (i == 1 and stride == 2) and (not f16 or i == 2 or outs[i].shape[3] % 4 == 0):
            assert len(names) >= 5, (i, net.op_candidates(i))
        for name in names:
            net.set_op_variant(i, name)
            assert net.op_variant(i) == name
            net.run(xd)
            torch.cuda.synchronize()
            got = net.read_buffer(ops[i].dst, outs[i].shape)
            assert_within_bound(got, outs[i], bounds[i], f"{geom} {dtype_name} op {ops[i].name} {name}")
            assert np.abs(got.astype(np.float64) - outs[i].astype(np.float64)).max() <= tol * max(np.abs(outs[i]).max(), 1e-3)
            seen += 1
    assert seen >= 5
    net.free()


def test_split_k_sums_in_slice_order(cad):
    """The matrix-core variants that split K over several workgroups per output tile add the
    slices' partial tiles in slice order, whoever arrives last: repeated launches give
    bit-identical outputs, the arrival counters are back at zero after every launch (a stale
    count would make a later launch finish a tile early, with slices missing), and the result
    meets the bar of the unsplit kernel."""
    cin, cout, k, stride, pad, h, w_, s, n = 256, 72, 3, 1, 1, 10, 9, 0.9, 5
    x = wl.activation((n, cin, h, w_), "splitk", 0, relu=False).astype(np.float16)
    w = wl.pruned_weights(cout, cin, k, k, s, "splitk", 1)
    b = wl.bias_vector(cout, "splitk", 1, sigma=0.5)
    r = wl.activation((n, cout, h, w_), "splitk", 2, relu=False, role="r").astype(np.float16)
    ref = oracle.conv2d(x, w.astype(np.float16), b, r, stride, pad, True, np.float16)
    cond = cond_conv(x, w.astype(np.float16), b, r, stride, pad)
    hnd = cad.cadnn_pack_weights(w, cad.F16)
    names = [nm for nm in cad.cadnn_conv2d_list_variants(hnd, n, h, w_, stride, pad) if "_k" in nm]
    assert "dense_mfma__Float16_64x64x32w_k8" in names and "dense_mfma__Float16_128x64x32_k4" in names, names
    xd, rd, bd = dev(x), dev(r), dev(b)
    for name in names:
        cad.cadnn_conv2d_set_variant(hnd, n, h, w_, stride, pad, name)
        outs = []
        for rep in range(6):
            out = torch.full((n, cout, h, w_), float("nan"), device="cuda", dtype=torch.float16)
            cad.cadnn_sparse_conv2d(hnd, xd, stride, pad, bd, rd, True, out=out)
            torch.cuda.synchronize()
            outs.append(out.cpu().numpy())
        assert_layer_close(outs[0], ref, cond, TOL_F16, f"split K {name}", f16=True)
        for rep in range(1, 6):
            assert np.array_equal(outs[0].view(np.uint16), outs[rep].view(np.uint16)), f"{name}: launch {rep} differs from launch 0"
    hnd.free()


@pytest.mark.parametrize("geom", [(7, 7, 1, 1), (7, 7, 3, 3), (14, 14, 2, 1), (9, 5, 2, 3)])
def test_fused_global_average_pool(cad, geom):
    """A global average pool that is the only reader of a small-image convolution is computed
    in that convolution's epilogue: the pool op reports "fused", the feature map is never
    materialised, and every pooling variant of the convolution must reproduce the oracle's
    pooled vector (and the logits of the FC behind it), with and without an identity
    residual, both storage types."""
    h, w_, n, k = geom
    ops = [wl.Op("conv", "pre", 0, 1, 8, 24, 1, 1, 0, 0.8, True),
           wl.Op("conv", "mid", 1, 2, 24, 24, k, 1, k // 2, 0.85, True),
           wl.Op("conv", "last", 2, 3, 24, 24, 1, 1, 0, 0.8, True, 1),
           wl.Op("avgpool", "gap", 3, 4, 0, 0, 0, 1, 0, 0.0, False),
           wl.Op("fc", "fc", 4, 5, 24, 10, 1, 1, 0, 0.5, False)]
    shape = (n, 8, h, w_)
    x, ws, bs = wl.net_tensors(ops, "gap-%d-%d-%d" % (h, w_, k), shape, input_relu=True)
    for dtype, npdt, tol in ((cad.F32, np.float32, TOL_F32), (cad.F16, np.float16, TOL_F16)):
        xs = x.astype(npdt)
        ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
        net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False)
        unfused = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False, fuse=False)
        xd = dev(xs)
        assert net.op_variant(3) == "fused" and unfused.op_variant(3) == "avgpool"
        with pytest.raises(cad.CadnnError):
            net.read_buffer(3, outs[2].shape)
        names = net.op_candidates(2)
        assert names and all("_gp" in nm for nm in names), names
        pooled = outs[3].reshape(n, 24).astype(np.float64)
        scale = np.abs(pooled).max()
        ulp = F16_ULP if dtype == cad.F16 else 0.0
        cond_last = cond_conv(ins[2], ws[2].astype(npdt), bs[2], outs[0], 1, 0)
        bound_mean = (SUM_TOL * cond_last + ulp * np.abs(outs[2].astype(np.float64))).mean(axis=(2, 3))
        for name in names:
            net.set_op_variant(2, name)
            y = net.run(xd)
            torch.cuda.synchronize()
            got = net.read_buffer(4, outs[3].shape).reshape(n, 24).astype(np.float64)
            # the mean of values that each obey the layer bound (so the mean of those bounds
            # bounds it), rounded once more to the storage type
            assert (np.abs(got - pooled) <= bound_mean + ulp * np.abs(pooled) + 1e-30).all(), \
                f"{name}: worst ratio {(np.abs(got - pooled) / (bound_mean + ulp * np.abs(pooled) + 1e-30)).max():.3f}"
            assert np.abs(got - pooled).max() <= tol * scale, name
            assert np.abs(y.cpu().numpy().astype(np.float64) - ref.astype(np.float64)).max() <= tol * np.abs(ref).max()
        yu = unfused.run(xd).cpu().numpy().astype(np.float64)
        torch.cuda.synchronize()
        assert np.abs(yu - ref.astype(np.float64)).max() <= tol * np.abs(ref).max()
        net.free()
        unfused.free()


@pytest.mark.parametrize("geom", [(7, 7, 1, 1, 1), (8, 8, 2, 3, 2), (5, 9, 3, 1, 2), (4, 16, 1, 3, 1),
                                  (14, 14, 1, 1, 1), (14, 14, 2, 3, 2), (16, 16, 1, 3, 1), (9, 13, 2, 1, 2),
                                  (28, 28, 1, 1, 2), (20, 27, 2, 3, 1)])
def test_fused_depthwise_epilogue(cad, geom):
    """A 3x3 depthwise layer that is the only reader of a convolution whose image is at most
    28 x 28 (one wavefront's pixels, or those of the 4 or 16 waves of a workgroup) is computed
    in that convolution's epilogue: the depthwise op reports "fused",
    the convolution's own map is never materialised, and every such variant of the convolution
    must reproduce the oracle's depthwise output (checked element by element against the
    depthwise layer's own bound on the oracle's input) and the layers behind it."""
    h, w_, n, k, ds = geom
    ops = [wl.Op("conv", "pre", 0, 1, 8, 24, 1, 1, 0, 0.8, True),
           wl.Op("conv", "mid", 1, 2, 24, 40, k, 1, k // 2, 0.85, True),
           wl.Op("dwconv", "dw", 2, 3, 40, 40, 3, ds, 1, 0.2, True),
           wl.Op("conv", "post", 3, 4, 40, 16, 1, 1, 0, 0.5, False)]
    shape = (n, 8, h, w_)
    x, ws, bs = wl.net_tensors(ops, "dwf-%d-%d-%d-%d" % (h, w_, k, ds), shape, input_relu=True)
    for dtype, npdt, tol in ((cad.F32, np.float32, TOL_F32), (cad.F16, np.float16, TOL_F16)):
        f16 = dtype == cad.F16
        xs = x.astype(npdt)
        ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
        net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False)
        unfused = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False, fuse=False)
        xd = dev(xs)
        assert net.op_variant(2) == "fused" and unfused.op_variant(2) == "dwconv"
        with pytest.raises(cad.CadnnError):
            net.read_buffer(2, outs[1].shape)
        names = net.op_candidates(1)
        assert names and all("_dw" in nm or "_dt" in nm for nm in names), names
        dw_ref = outs[2].astype(np.float64)
        # bound of the fused pair on the oracle's input to the pair: the depthwise layer's own
        # condition sum plus what the first layer's rounding error becomes behind |filters|
        wd = ws[2].astype(npdt)
        cond_mid = cond_conv(ins[1], ws[1].astype(npdt), bs[1], None, 1, k // 2)
        cond = cond_depthwise(outs[1], wd, bs[2], ds, 1) + cond_depthwise(cond_mid.astype(np.float32), wd, None, ds, 1)
        if f16:   # the intermediate map is rounded to fp16 on both sides, possibly to neighbouring values
            cond = cond + 2.0 ** -10 / 1e-4 * cond_depthwise(np.abs(outs[1]).astype(np.float32), wd, None, ds, 1)
        for name in names:
            net.set_op_variant(1, name)
            y = net.run(xd)
            torch.cuda.synchronize()
            got = net.read_buffer(3, outs[2].shape)
            assert_layer_close(got, dw_ref, cond, tol, f"{geom} {name}", f16=f16)
            assert np.abs(y.cpu().numpy().astype(np.float64) - ref.astype(np.float64)).max() <= tol * np.abs(ref).max(), name
        yu = unfused.run(xd).cpu().numpy().astype(np.float64)
        torch.cuda.synchronize()
        assert np.abs(yu - ref.astype(np.float64)).max() <= tol * np.abs(ref).max()
        net.free()
        unfused.free()


@pytest.mark.parametrize("dtype_name", ["f32", "f16"])
def test_concat_in_place_and_copied(cad, dtype_name):
    """Channel concatenation inside a net: branch outputs that only the concatenation reads are
    written by their producers (convolution, depthwise, max pool, average pool) straight into
    their channel slices, whose zero halo the 3x3 reader behind relies on; a source with another
    reader, the net input, and a nested concatenation are copied.  Every intermediate buffer and
    the output are compared with the oracle."""
    f16 = dtype_name == "f16"
    dtype, npdt, tol = (cad.F16, np.float16, TOL_F16) if f16 else (cad.F32, np.float32, TOL_F32)
    Op = wl.Op
    ops = [Op("conv", "b1", 0, 1, 6, 10, 1, 1, 0, 0.5, True),
           Op("conv", "b2a", 0, 2, 6, 8, 1, 1, 0, 0.5, True),
           Op("conv", "b2b", 2, 3, 8, 12, 3, 1, 1, 0.7, True),
           Op("dwconv", "b3", 2, 4, 8, 8, 3, 1, 1, 0.0, True),          # buffer 2 has two readers
           Op("maxpool", "b4", 0, 5, k=3, stride=1, pad=1),
           Op("avgpool2d", "b5", 0, 6, k=3, stride=1, pad=1),
           Op("concat", "inner", 5, 7, srcs=(5, 6)),
           Op("concat", "cat", 1, 8, srcs=(1, 3, 4, 7, 0, 2)),          # 10 + 12 + 8 + 12 + 6 + 8 = 56
           Op("conv", "post", 8, 9, 56, 16, 3, 1, 1, 0.8, True),
           Op("concat", "tail", 9, 10, srcs=(9, 9))]                      # the last op: copies into y
    shape = (3, 6, 11, 13)
    x, ws, bs = wl.net_tensors(ops, "cat", shape, input_relu=True)
    xs = x.astype(npdt)
    ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
    assert ref.shape == (3, 32, 11, 13)
    for kw in ({}, {"plain_layout": True, "fuse": False}):
        net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=True, **kw)
        names = [net.op_variant(i) for i in range(len(ops))]
        assert names[6] == "in place" and names[7] == "concat" and names[9] == "concat", names
        for rep in range(2):
            y = net.run(dev(xs))
            torch.cuda.synchronize()
            assert_close(y.cpu().numpy(), ref, tol, f"concat net {kw} (replay {rep})")
        for i in (0, 2, 3, 4, 5, 6, 7):
            got = net.read_buffer(ops[i].dst, outs[i].shape)
            assert_close(got, outs[i], tol, f"buffer of {ops[i].name}")
        net.free()


@pytest.mark.parametrize("dtype_name", ["f32", "f16"])
def test_sibling_layers_in_one_launch(cad, dtype_name):
    """Pixel-wise sparse layers that read the same tensor are merged into one launch over the
    rows of all of them, their outputs channel slices of one region whose halo serves the most
    demanding reader (5x5 here).  Every variant of the merged layer, tuned or not, must leave
    each sibling's output and everything behind it as the oracle has them; a layer with a
    different activation, a concatenation slice and a residual layer stay out of the group."""
    f16 = dtype_name == "f16"
    dtype, npdt, tol = (cad.F16, np.float16, TOL_F16) if f16 else (cad.F32, np.float32, TOL_F32)
    Op = wl.Op
    ops = [Op("conv", "stem", 0, 1, 6, 32, 1, 1, 0, 0.8, True),
           Op("conv", "s1", 1, 2, 32, 12, 1, 1, 0, 0.8, True),          # group of three: s1, s2, s3
           Op("conv", "s2", 1, 3, 32, 20, 1, 1, 0, 0.9, True),
           Op("conv", "lin", 1, 4, 32, 8, 1, 1, 0, 0.8, False),         # no ReLU: not in the group
           Op("conv", "s3", 1, 5, 32, 9, 1, 1, 0, 0.85, True),
           Op("conv", "slice", 1, 6, 32, 10, 1, 1, 0, 0.8, True),       # only read by the concatenation: in place there
           Op("conv", "r3", 2, 7, 12, 16, 3, 1, 1, 0.8, True),          # halo 1
           Op("conv", "r5", 3, 8, 20, 16, 5, 1, 2, 0.9, True),          # halo 2: the group's halo
           Op("conv", "r1", 5, 9, 9, 16, 1, 1, 0, 0.8, True),
           Op("conv", "rl", 4, 10, 8, 16, 1, 1, 0, 0.8, True),
           Op("concat", "cat", 7, 11, srcs=(7, 8, 9, 10, 6)),
           Op("conv", "post", 11, 12, 74, 12, 1, 1, 0, 0.8, False)]
    shape = (2, 6, 13, 11)
    x, ws, bs = wl.net_tensors(ops, "sib", shape, input_relu=True)
    xs = x.astype(npdt)
    ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
    infos, _ = cad.plan_net(ops, ws, shape, dtype)
    # s2 and s3 are rows of s1's launch; lin and slice, which could not be, are independent layers
    # that share its kernel launch all the same (with r3 / r5 / r1 / rl one level down)
    assert [(i["fused_into"], i["launched_with"]) for i in infos[:6]] == [(-1, 0), (-1, 0), (1, 0), (1, 1), (1, 0), (1, 1)]
    assert [(i["fused_into"], i["launched_with"]) for i in infos[6:10]] == [(-1, 0), (6, 1), (6, 1), (6, 1)]
    assert infos[1]["halo_h"] == infos[2]["halo_h"] == infos[4]["halo_h"] == 2 and infos[5]["slice_of"] == 10
    for kw in ({}, {"tune": True}, {"fuse": False}):
        net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=True, **kw)
        merged = kw.get("fuse", True)
        assert (net.op_variant(2) == "fused") == merged and (net.op_variant(4) == "fused") == merged
        names = [net.op_variant(1)] if kw else net.op_candidates(1)
        assert names
        for name in names:
            net.set_op_variant(1, name)
            y = net.run(dev(xs))
            torch.cuda.synchronize()
            assert_net_close(y.cpu().numpy(), ref, tol, f"sibling net {kw} {name}")
            for i in (1, 2, 3, 4, 5):
                cond = cond_conv(ins[i], ws[i].astype(npdt), bs[i], None, 1, 0)
                got = net.read_buffer(ops[i].dst, outs[i].shape)
                assert_layer_close(got, outs[i], cond + (2.0 ** -10 / 1e-4 * np.abs(outs[i]) if f16 else 0), tol,
                                   f"{ops[i].name} {kw} {name}", f16=f16)
        if not kw:
            # the second level: a 3x3, a 5x5 and two 1x1 layers on four different tensors share
            # every launch; each variant that serves all four must leave the concatenation right
            assert [net.op_variant(i) for i in (7, 8, 9)] == ["fused"] * 3
            names = net.op_candidates(6)
            assert len(names) > 4 and net.op_variant(6) in names
            cat = np.concatenate([outs[i] for i in (6, 7, 8, 9, 5)], axis=1)
            for name in names:
                net.set_op_variant(6, name)
                assert net.op_variant(6) == name
                y = net.run(dev(xs))
                torch.cuda.synchronize()
                assert_net_close(net.read_buffer(11, cat.shape), cat, tol, f"co-launched {name}")
                assert_net_close(y.cpu().numpy(), ref, tol, f"co-launched net {name}")
            with pytest.raises(cad.CadnnError):
                net.set_op_variant(6, "slinear_float_d1_r1k1w4u4")        # not a variant for several layers
        net.free()


@pytest.mark.parametrize("dtype_name", ["f32", "f16"])
def test_group_taken_apart_keeps_the_launch_order(cad, dtype_name):
    """A pooled branch: the pool rides along with the module's first layers and its 1x1 layer
    with the second ones, whose launch comes BEFORE the pool's place in the op list.  When the
    first group is taken apart (as tuning does to a group that loses) the pool must still run
    ahead of that second launch.  Checked on two different inputs in a row: on a repeated
    input the stale pool output of the previous run would hide a wrong order."""
    f16 = dtype_name == "f16"
    dtype, npdt, tol = (cad.F16, np.float16, TOL_F16) if f16 else (cad.F32, np.float32, TOL_F32)
    Op = wl.Op
    ops = [Op("conv", "stem", 0, 1, 6, 24, 1, 1, 0, 0.8, True),
           Op("conv", "a", 1, 2, 24, 12, 1, 1, 0, 0.8, True),            # leads the first launch: a, b (no ReLU: not a sibling), pool
           Op("conv", "b", 1, 3, 24, 10, 1, 1, 0, 0.8, False),
           Op("conv", "a2", 2, 4, 12, 16, 3, 1, 1, 0.8, True),           # leads the second: a2, b2, p1
           Op("conv", "b2", 3, 5, 10, 16, 1, 1, 0, 0.8, True),
           Op("avgpool2d", "pool", 1, 6, k=3, stride=1, pad=1),
           Op("conv", "p1", 6, 7, 24, 8, 1, 1, 0, 0.8, True),
           Op("concat", "cat", 4, 8, srcs=(4, 5, 7)),
           Op("conv", "post", 8, 9, 40, 9, 1, 1, 0, 0.8, False)]
    shape = (2, 6, 12, 10)
    x, ws, bs = wl.net_tensors(ops, "apart", shape, input_relu=True)
    xs = x.astype(npdt)
    xs2 = wl.activation(shape, "apart", 99, relu=True).astype(npdt)
    refs = [oracle.run_net(ops, v, ws, bs, dtype=npdt)[0] for v in (xs, xs2)]
    net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=True)
    info = [net.op_info(i) for i in range(len(ops))]
    assert [(info[i]["fused_into"], info[i]["launched_with"]) for i in (2, 5, 4, 6)] == [(1, 1), (1, 1), (3, 1), (3, 1)]
    for step in ("together", "apart"):
        if step == "apart":
            net.set_op_variant(1, "apart")
            info = [net.op_info(i) for i in range(len(ops))]
            assert [(info[i]["fused_into"], info[i]["launched_after"]) for i in (2, 5)] == [(-1, 1), (-1, 1)]
            assert info[6]["fused_into"] == 3                     # the second group is untouched
            assert net.op_variant(5) == "avgpool2d" and net.op_variant(2).startswith("slinear")
        for v, ref in ((xs, refs[0]), (xs2, refs[1]), (xs, refs[0])):
            y = net.run(dev(v))
            torch.cuda.synchronize()
            assert_net_close(y.cpu().numpy(), ref, tol, f"{step}")
    net.free()


@pytest.mark.parametrize("dtype_name", ["f32", "f16"])
def test_big_strided_layer_reads_a_deinterleaved_copy(cad, dtype_name):
    """A large 3x3 stride-2 layer on an odd-sized tensor (Inception-V3's 288 -> 384 on 35 x 35)
    cannot have its input de-interleaved where it is produced; the runner makes a de-interleaved
    copy right before it.  Every variant that serves the layer there, on two inputs in a row,
    and the same net in plain layout."""
    f16 = dtype_name == "f16"
    dtype, npdt, tol = (cad.F16, np.float16, TOL_F16) if f16 else (cad.F32, np.float32, TOL_F32)
    Op = wl.Op
    ops = [Op("conv", "pre", 0, 1, 8, 288, 1, 1, 0, 0.5, True),
           Op("conv", "main", 1, 2, 288, 384, 3, 2, 0, 0.8, True),
           Op("maxpool", "pool", 1, 3, k=3, stride=2, pad=0),            # a second reader of the same tensor
           Op("concat", "cat", 2, 4, srcs=(2, 3)),
           Op("conv", "post", 4, 5, 672, 6, 1, 1, 0, 0.8, False)]
    shape = (2, 8, 35, 35)
    x, ws, bs = wl.net_tensors(ops, "restage", shape, input_relu=True)
    xs = x.astype(npdt)
    xs2 = wl.activation(shape, "restage", 99, relu=True).astype(npdt)
    refs = [oracle.run_net(ops, v, ws, bs, dtype=npdt) for v in (xs, xs2)]
    net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=True)
    plain = cad.build_net(ops, ws, bs, shape, dtype, use_graph=True, plain_layout=True)
    assert net.op_info(1)["input_copy"] >= 0 and plain.op_info(1)["input_copy"] == -1
    assert all(net.op_info(i)["input_copy"] == -1 for i in (0, 2, 4))
    names = net.op_candidates(1)
    assert any("_a4_" in nm or "_g4_" in nm for nm in names) or f16, names     # unit-stride wide loads on the copy
    for name in [None] + names:
        net.set_op_variant(1, name)
        for v, (ref, ins, outs) in ((xs, refs[0]), (xs2, refs[1])):
            y = net.run(dev(v))
            torch.cuda.synchronize()
            cond = cond_conv(ins[1], ws[1].astype(npdt), bs[1], None, 2, 0)
            got = net.read_buffer(2, outs[1].shape)
            assert_layer_close(got, outs[1], cond + (2.0 ** -10 / 1e-4 * np.abs(outs[1]) if f16 else 0), tol,
                               f"restaged {name}", f16=f16)
            assert_net_close(y.cpu().numpy(), ref, tol, f"restaged net {name}")
    y = plain.run(dev(xs2))
    torch.cuda.synchronize()
    assert_net_close(y.cpu().numpy(), refs[1][0], tol, "plain layout")
    net.free()
    plain.free()
