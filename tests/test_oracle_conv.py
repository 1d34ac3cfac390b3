"""Pins for the CPU oracle's layers (no GPU).

Each test checks the C oracle against something other than itself: a brute-force
loop nest written here, hand arithmetic, a library routine (matmul / torch
float64 conv) or an invariant of the definition.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_conv(x, w, bias, res, stride, pad, relu):
    """The definition as a 7-deep scalar loop in Python floats (double)."""
    n, cin, h, wd = x.shape
    cout, _, kh, kw = w.shape
    hout = (h + 2 * pad - kh) // stride + 1
    wout = (wd + 2 * pad - kw) // stride + 1
    y = np.zeros((n, cout, hout, wout))
    for b in range(n):
        for co in range(cout):
            for oh in range(hout):
                for ow in range(wout):
                    s = 0.0
                    for ci in range(cin):
                        for r in range(kh):
                            for c in range(kw):
                                ih, iw = oh * stride + r - pad, ow * stride + c - pad
                                if 0 <= ih < h and 0 <= iw < wd:
                                    s += float(w[co, ci, r, c]) * float(x[b, ci, ih, iw])
                    if bias is not None:
                        s += float(bias[co])
                    if res is not None:
                        s += float(res[b, co, oh, ow])
                    if relu:
                        s = max(s, 0.0)
                    y[b, co, oh, ow] = s
    return y


def rnd(shape, seed, sparsity=0.0):
    g = np.random.default_rng(seed)
    a = g.standard_normal(shape).astype(np.float32)
    if sparsity > 0:
        a = np.where(g.random(shape) < sparsity, np.float32(0), a).astype(np.float32)
    return a


def read_golden(name):
    sections, cur = {}, None
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            cur = line.strip("[]")
            sections[cur] = []
        else:
            sections[cur].append([float(t) for t in line.split()])
    return {k: np.array(v, dtype=np.float32) for k, v in sections.items()}


def test_hand_example():
    g = read_golden("conv3x3_hand_example.txt")
    x = g["x"].reshape(1, 1, 4, 4)
    w = g["w"].reshape(1, 1, 3, 3)
    z = oracle.conv2d_f64(x, w, None, None, 1, 1, False)
    assert np.array_equal(z[0, 0], g["z"].astype(np.float64))
    y = oracle.conv2d(x, w, g["bias"].reshape(1), None, 1, 1, True)
    assert np.array_equal(y[0, 0], g["y"])


@pytest.mark.parametrize("k,stride,pad", [(1, 1, 0), (1, 2, 0), (3, 1, 1), (3, 2, 1), (3, 1, 0),
                                          (7, 2, 3), (3, 2, 3), (7, 1, 3)])
def test_brute_force(k, stride, pad):
    seed = 100 * k + 10 * stride + pad
    x = rnd((2, 3, 7, 6), seed)
    w = rnd((4, 3, k, k), seed + 1, sparsity=0.5)
    b = rnd((4,), seed + 2)
    hout = (7 + 2 * pad - k) // stride + 1
    wout = (6 + 2 * pad - k) // stride + 1
    if hout <= 0 or wout <= 0:
        pytest.skip("empty")
    r = rnd((2, 4, hout, wout), seed + 3)
    for bias, res, relu in [(None, None, False), (b, None, True), (b, r, True), (b, r, False)]:
        got = oracle.conv2d_f64(x, w, bias, res, stride, pad, relu)
        ref = brute_conv(x, w, bias, res, stride, pad, relu)
        assert got.shape == ref.shape
        np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)


def test_non_square_kernel_and_image_brute_force():
    x = rnd((1, 2, 5, 8), 7)
    w = rnd((3, 2, 1, 7), 8, sparsity=0.3)
    got = oracle.conv2d_f64(x, w, None, None, 1, 2, False)
    np.testing.assert_allclose(got, brute_conv(x, w, None, None, 1, 2, False), rtol=1e-13, atol=1e-13)


def test_1x1_is_matmul():
    # Section 4: a 1x1 convolution is a matrix multiply W[Cout x Cin] @ X[Cin x HW].
    x = rnd((2, 16, 9, 11), 1)
    w = rnd((24, 16, 1, 1), 2, sparsity=0.8)
    got = oracle.conv2d_f64(x, w)
    ref = np.einsum("oc,nchw->nohw", w[:, :, 0, 0].astype(np.float64), x.astype(np.float64))
    ref2 = np.stack([w[:, :, 0, 0].astype(np.float64) @ x[i].reshape(16, -1).astype(np.float64)
                     for i in range(2)]).reshape(2, 24, 9, 11)
    np.testing.assert_allclose(got, ref2, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_1x1_stride2_is_matmul_on_subsampled_input():
    x = rnd((1, 8, 10, 10), 3)
    w = rnd((5, 8, 1, 1), 4, sparsity=0.5)
    got = oracle.conv2d_f64(x, w, stride=2)
    xs = x[:, :, ::2, ::2]
    ref = (w[:, :, 0, 0].astype(np.float64) @ xs[0].reshape(8, -1).astype(np.float64)).reshape(1, 5, 5, 5)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("k,stride,pad", [(3, 1, 1), (3, 2, 1), (7, 2, 3), (5, 1, 2)])
def test_im2col_matmul(k, stride, pad):
    x = rnd((2, 5, 12, 13), 11)
    w = rnd((6, 5, k, k), 12, sparsity=0.7)
    n, cin, h, wd = x.shape
    hout, wout = (h + 2 * pad - k) // stride + 1, (wd + 2 * pad - k) // stride + 1
    xp = np.pad(x.astype(np.float64), ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    cols = np.zeros((n, cin * k * k, hout * wout))
    for ci in range(cin):
        for r in range(k):
            for c in range(k):
                patch = xp[:, ci, r:r + stride * hout:stride, c:c + stride * wout:stride]
                cols[:, (ci * k + r) * k + c, :] = patch.reshape(n, -1)
    ref = (w.reshape(6, -1).astype(np.float64) @ cols).reshape(n, 6, hout, wout)
    got = oracle.conv2d_f64(x, w, None, None, stride, pad, False)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("k,stride,pad", [(1, 1, 0), (3, 1, 1), (3, 2, 1), (7, 2, 3)])
def test_against_torch_float64(k, stride, pad):
    torch = pytest.importorskip("torch")
    x = rnd((2, 6, 15, 14), 21)
    w = rnd((8, 6, k, k), 22, sparsity=0.6)
    b = rnd((8,), 23)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     torch.from_numpy(b).double(), stride=stride, padding=pad)
    got = oracle.conv2d_f64(x, w, b, None, stride, pad, False)
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-12, atol=1e-12)
    got_r = oracle.conv2d_f64(x, w, b, None, stride, pad, True)
    np.testing.assert_allclose(got_r, torch.relu(ref).numpy(), rtol=1e-12, atol=1e-12)


def test_zero_weight_invariance_and_all_zero():
    x = rnd((1, 4, 8, 8), 31)
    w = rnd((5, 4, 3, 3), 32, sparsity=0.7)
    b = rnd((5,), 33)
    r = rnd((1, 5, 8, 8), 34)
    base = oracle.conv2d_f64(x, w, b, r, 1, 1, True)
    # -0.0 in place of +0.0 at pruned positions must change nothing (bit-exact)
    w2 = np.where(w == 0, np.float32(-0.0), w)
    assert np.array_equal(base, oracle.conv2d_f64(x, w2, b, r, 1, 1, True))
    # removing an input channel whose weights are all zero changes nothing
    w3 = w.copy()
    w3[:, 2] = 0
    full = oracle.conv2d_f64(x, w3, b, r, 1, 1, True)
    cut = oracle.conv2d_f64(np.delete(x, 2, axis=1), np.delete(w3, 2, axis=1), b, r, 1, 1, True)
    assert np.array_equal(full, cut)
    # all-zero weights: y == act(bias + residual) exactly
    z = oracle.conv2d_f64(x, np.zeros_like(w), b, r, 1, 1, True)
    ref = np.maximum(b.astype(np.float64)[None, :, None, None] + r.astype(np.float64), 0.0)
    assert np.array_equal(z, ref)


def test_identity_kernel_gives_relu_of_input():
    x = rnd((2, 6, 9, 9), 41)
    for k, pad in [(1, 0), (3, 1), (7, 3)]:
        w = np.zeros((6, 6, k, k), np.float32)
        for c in range(6):
            w[c, c, k // 2, k // 2] = 1.0
        y = oracle.conv2d(x, w, None, None, 1, pad, True)
        assert np.array_equal(y, np.maximum(x, 0))


def test_shifted_delta_kernel_shifts_the_image():
    # W = delta at (kh=0, kw=2) of a 3x3, pad 1: y[oh][ow] = x[oh-1][ow+1] (0 outside).
    # Catches a transposed kernel or a flipped (true-convolution) index.
    x = rnd((1, 1, 6, 7), 43)
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, 0, 2] = 1.0
    y = oracle.conv2d_f64(x, w, None, None, 1, 1, False)[0, 0]
    ref = np.zeros((6, 7))
    ref[1:, :-1] = x[0, 0, :-1, 1:]
    assert np.array_equal(y, ref)


def test_linearity_pre_activation():
    x = rnd((1, 5, 10, 10), 51)
    w1 = rnd((4, 5, 3, 3), 52, 0.5)
    w2 = rnd((4, 5, 3, 3), 53, 0.5)
    a, b = np.float32(0.5), np.float32(-2.0)   # exact scalings in binary fp
    lhs = oracle.conv2d_f64(x, (a * w1 + b * w2).astype(np.float32), None, None, 2, 1, False)
    rhs = a * oracle.conv2d_f64(x, w1, None, None, 2, 1, False) + \
        b * oracle.conv2d_f64(x, w2, None, None, 2, 1, False)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-6, atol=1e-6)


def test_fused_equals_unfused():
    x = rnd((2, 4, 8, 8), 61)
    w = rnd((6, 4, 3, 3), 62, 0.6)
    b = rnd((6,), 63)
    r = rnd((2, 6, 8, 8), 64)
    fused = oracle.conv2d_f64(x, w, b, r, 1, 1, True)
    z = oracle.conv2d_f64(x, w, None, None, 1, 1, False)
    unfused = np.maximum(z + b.astype(np.float64)[None, :, None, None] + r.astype(np.float64), 0.0)
    np.testing.assert_allclose(fused, unfused, rtol=1e-14, atol=1e-14)


def test_fc_is_matmul():
    x = rnd((3, 50), 71)
    w = rnd((20, 50, 1, 1), 72, 0.9)
    b = rnd((20,), 73)
    got = oracle.fc_f64(x, w, b, relu=True)
    ref = np.maximum(x.astype(np.float64) @ w.reshape(20, 50).astype(np.float64).T + b.astype(np.float64), 0)
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)
    got2 = oracle.fc_f64(x, w, None, relu=False)
    np.testing.assert_allclose(got2, x.astype(np.float64) @ w.reshape(20, 50).astype(np.float64).T,
                               rtol=1e-13, atol=1e-13)


def test_pools():
    x = rnd((2, 3, 9, 8), 81)
    for k, s, p in [(3, 2, 1), (2, 2, 0), (3, 1, 1)]:
        got = oracle.maxpool(x, k, s, p)
        hout, wout = (9 + 2 * p - k) // s + 1, (8 + 2 * p - k) // s + 1
        ref = np.zeros((2, 3, hout, wout), np.float32)
        for n in range(2):
            for c in range(3):
                for oh in range(hout):
                    for ow in range(wout):
                        vals = [x[n, c, oh * s + r - p, ow * s + q - p]
                                for r in range(k) for q in range(k)
                                if 0 <= oh * s + r - p < 9 and 0 <= ow * s + q - p < 8]
                        ref[n, c, oh, ow] = max(vals)
        assert np.array_equal(got, ref)
    # a negative image keeps its negative maxima at the border (padding never wins)
    xn = -np.abs(x) - 1
    assert (oracle.maxpool(xn, 3, 2, 1) < 0).all()
    g = oracle.global_avgpool(x)
    np.testing.assert_allclose(g[:, :, 0, 0], x.astype(np.float64).mean(axis=(2, 3)), rtol=1e-6)


def test_output_shape_ladder():
    g = {}
    for line in open(os.path.join(GOLDEN, "resnet50_shapes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        t = line.split()
        g[t[0]] = [int(v) for v in t[1:]]
    assert oracle.out_size(224, 7, 2, 3) == g["conv1"][0]
    assert oracle.out_size(112, 3, 2, 1) == g["pool1"][0]
    assert oracle.out_size(56, 3, 1, 1) == g["conv2"][0]
    assert oracle.out_size(56, 3, 2, 1) == g["conv3"][0]
    assert oracle.out_size(28, 3, 2, 1) == g["conv4"][0]
    assert oracle.out_size(14, 3, 2, 1) == g["conv5"][0]
    assert oracle.out_size(56, 1, 2, 0) == 28
    x = np.zeros((1, 1, 224, 224), np.float32)
    w = np.zeros((1, 1, 7, 7), np.float32)
    assert oracle.conv2d_f64(x, w, None, None, 2, 3, False).shape == (1, 1, 112, 112)


def test_fp16_variant_single_rounding():
    x = rnd((1, 8, 6, 6), 91).astype(np.float16)
    w = rnd((4, 8, 3, 3), 92, 0.5).astype(np.float16)
    y64 = oracle.conv2d_f64(x, w, None, None, 1, 1, False)
    # inputs are widened exactly: same result as the float64 brute force over the fp16 values
    ref = brute_conv(x.astype(np.float64), w.astype(np.float64), None, None, 1, 1, False)
    np.testing.assert_allclose(y64, ref, rtol=1e-13, atol=1e-13)
    y16 = oracle.conv2d(x, w, None, None, 1, 1, False, dtype=np.float16)
    assert y16.dtype == np.float16
    assert np.array_equal(y16, ref.astype(np.float16))


# ---------------------------------------------------------------------------
# Depthwise layer (paper Section 4: depthwise convolution + batch-norm + activation fused)
# ---------------------------------------------------------------------------

def brute_depthwise(x, w, bias, stride, pad, relu):
    """Each channel against its own filter, as scalar loops in Python floats."""
    n, ch, h, wd = x.shape
    kh, kw = w.shape[2], w.shape[3]
    hout = (h + 2 * pad - kh) // stride + 1
    wout = (wd + 2 * pad - kw) // stride + 1
    y = np.zeros((n, ch, hout, wout))
    for b in range(n):
        for c in range(ch):
            for oh in range(hout):
                for ow in range(wout):
                    s = 0.0
                    for r in range(kh):
                        for q in range(kw):
                            ih, iw = oh * stride + r - pad, ow * stride + q - pad
                            if 0 <= ih < h and 0 <= iw < wd:
                                s += float(w[c, 0, r, q]) * float(x[b, c, ih, iw])
                    if bias is not None:
                        s += float(bias[c])
                    y[b, c, oh, ow] = max(s, 0.0) if relu else s
    return y


@pytest.mark.parametrize("kh,kw,stride,pad", [(3, 3, 1, 1), (3, 3, 2, 1), (5, 3, 1, 2), (1, 1, 1, 0), (3, 3, 2, 0)])
def test_depthwise_brute_force(kh, kw, stride, pad):
    x = rnd((2, 5, 9, 8), 70 + kh)
    w = rnd((5, 1, kh, kw), 71 + kw, sparsity=0.3)
    b = rnd((5,), 72)
    got = oracle.depthwise_conv2d_f64(x, w, b, stride, pad, True)
    np.testing.assert_allclose(got, brute_depthwise(x, w, b, stride, pad, True), rtol=1e-13, atol=1e-13)
    got = oracle.depthwise_conv2d_f64(x, w, None, stride, pad, False)
    np.testing.assert_allclose(got, brute_depthwise(x, w, None, stride, pad, False), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("stride", [1, 2])
def test_depthwise_is_full_conv_with_block_diagonal_filters(stride):
    """Placing filter c at [c, c] of an otherwise zero [C][C][kh][kw] tensor turns the
    depthwise layer into an ordinary convolution (which has its own pins above)."""
    x = rnd((2, 6, 11, 10), 80)
    w = rnd((6, 1, 3, 3), 81)
    b = rnd((6,), 82)
    full = np.zeros((6, 6, 3, 3), np.float32)
    for c in range(6):
        full[c, c] = w[c, 0]
    want = oracle.conv2d_f64(x, full, b, None, stride, 1, True)
    got = oracle.depthwise_conv2d_f64(x, w, b, stride, 1, True)
    np.testing.assert_allclose(got, want, rtol=1e-14, atol=1e-14)


def test_depthwise_box_filter_closed_form():
    """All-ones 3x3 filters on an all-ones image count the in-image taps: 9 inside,
    6 on edges, 4 in corners; a channel scaled by a gives a times that."""
    x = np.ones((1, 3, 6, 7), np.float32)
    x[0, 1] *= 2.0
    x[0, 2] *= -0.5
    w = np.ones((3, 1, 3, 3), np.float32)
    got = oracle.depthwise_conv2d_f64(x, w, None, 1, 1, False)
    rows = np.array([2, 3, 3, 3, 3, 2], float)[:, None]
    cols = np.array([2, 3, 3, 3, 3, 3, 2], float)[None, :]
    for c, a in enumerate([1.0, 2.0, -0.5]):
        assert np.array_equal(got[0, c], a * rows * cols)


def test_depthwise_against_torch_grouped_float64():
    torch = pytest.importorskip("torch")
    x = rnd((2, 7, 13, 12), 90)
    w = rnd((7, 1, 3, 3), 91, sparsity=0.2)
    b = rnd((7,), 92)
    for stride in (1, 2):
        want = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                          torch.from_numpy(b).double(), stride=stride, padding=1, groups=7)
        got = oracle.depthwise_conv2d_f64(x, w, b, stride, 1, False)
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-12)


def test_depthwise_channels_do_not_mix_and_fp16_rounds_once():
    x = rnd((1, 4, 8, 8), 95)
    w = rnd((4, 1, 3, 3), 96)
    base = oracle.depthwise_conv2d_f64(x, w, None, 1, 1, False)
    x2 = x.copy()
    x2[0, 2] += 1.0                      # only channel 2 of the output may move
    moved = oracle.depthwise_conv2d_f64(x2, w, None, 1, 1, False)
    assert np.array_equal(moved[0, [0, 1, 3]], base[0, [0, 1, 3]])
    assert not np.array_equal(moved[0, 2], base[0, 2])
    x16, w16 = x.astype(np.float16), w.astype(np.float16)
    y16 = oracle.depthwise_conv2d(x16, w16, None, 1, 1, True, dtype=np.float16)
    assert y16.dtype == np.float16
    assert np.array_equal(y16, oracle.depthwise_conv2d_f64(x16, w16, None, 1, 1, True).astype(np.float16))


# ---------------------------------------------------------------------------
# Rectangular filters carried in square banks (Inception-V3's 1x7 / 7x1 layers)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("kh,kw", [(1, 7), (7, 1), (1, 3), (3, 5)])
def test_rectangular_filter_centred_in_a_square_one(kh, kw):
    """A kh x kw filter with padding ((kh-1)/2, (kw-1)/2) equals the same filter centred in a
    zero k x k one with padding (k-1)/2: checked against torch's float64 convolution with
    rectangular padding, which never sees the square form."""
    torch = pytest.importorskip("torch")
    import workloads as wl
    k = max(kh, kw)
    x = rnd((2, 5, 11, 13), 200 + kh)
    w = rnd((6, 5, kh, kw), 201 + kw, sparsity=0.4)
    b = rnd((6,), 202)
    for stride in (1, 2):
        want = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                          torch.from_numpy(b).double(), stride=stride,
                                          padding=((kh - 1) // 2, (kw - 1) // 2))
        got = oracle.conv2d_f64(x, wl.embed_filter(w, k), b, None, stride, (k - 1) // 2, False)
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-12)
    assert np.count_nonzero(wl.embed_filter(w, k)) == np.count_nonzero(w)


# ---------------------------------------------------------------------------
# Windowed average pool and channel concatenation (Inception-V3 modules)
# ---------------------------------------------------------------------------

def test_avgpool_window_mean_excludes_padding():
    torch = pytest.importorskip("torch")
    x = rnd((2, 3, 9, 11), 300)
    for k, s, p in [(3, 1, 1), (3, 2, 1), (2, 2, 0), (5, 1, 2)]:
        want = torch.nn.functional.avg_pool2d(torch.from_numpy(x).double(), k, s, p, count_include_pad=False)
        got = oracle.avgpool(x, k, s, p, dtype=np.float64)
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-13, atol=1e-13)
    # brute force on a tiny case
    k, s, p = 3, 1, 1
    got = oracle.avgpool(x[:1, :1], k, s, p, dtype=np.float64)[0, 0]
    for oh in range(9):
        for ow in range(11):
            vals = [float(x[0, 0, i, j]) for i in range(oh - 1, oh + 2) for j in range(ow - 1, ow + 2)
                    if 0 <= i < 9 and 0 <= j < 11]
            assert abs(got[oh, ow] - sum(vals) / len(vals)) < 1e-12
    # a constant image stays constant (the border is not dimmed by the padding)
    c = np.full((1, 2, 6, 5), 2.5, np.float32)
    assert np.array_equal(oracle.avgpool(c, 3, 1, 1, dtype=np.float64), np.full((1, 2, 6, 5), 2.5))


def test_run_net_concat_stacks_channels_in_order():
    from workloads import Op
    ops = [Op("maxpool", "a", 0, 1, k=3, stride=1, pad=1),
           Op("avgpool2d", "b", 0, 2, k=3, stride=1, pad=1),
           Op("concat", "cat", 1, 3, srcs=(1, 0, 2))]
    x = rnd((2, 3, 5, 6), 301)
    y, ins, outs = oracle.run_net(ops, x, [None] * 3, [None] * 3)
    assert y.shape == (2, 9, 5, 6)
    assert np.array_equal(y[:, 0:3], oracle.maxpool(x, 3, 1, 1))
    assert np.array_equal(y[:, 3:6], x)
    assert np.array_equal(y[:, 6:9], oracle.avgpool(x, 3, 1, 1))
