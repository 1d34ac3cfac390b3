"""Pins for the reference packer (canonical compact format) and the net interpreter."""
import numpy as np
import pytest

import oracle
import workloads as wl


def small_w(seed, shape=(7, 3, 3, 3), sparsity=0.7):
    g = np.random.default_rng(seed)
    w = g.standard_normal(shape).astype(np.float32)
    return np.where(g.random(shape) < sparsity, np.float32(0), w).astype(np.float32)


def test_hand_written_pack():
    # 3 rows, K = 4: row0 has 1 nonzero, row1 has 3, row2 has 1 (tie with row0 -> row0 first)
    w = np.array([[0, 5, 0, 0], [1, 0, 2, 3], [0, 0, 0, 7]], np.float32).reshape(3, 4, 1, 1)
    p = oracle.pack(w)
    assert p["perm"].tolist() == [1, 0, 2]
    assert p["row_ptr"].tolist() == [0, 3, 4, 5]
    assert p["col_idx"].tolist() == [0, 2, 3, 1, 3]
    assert p["vals"].tolist() == [1, 2, 3, 5, 7]


def test_column_index_is_ci_kh_kw_row_major():
    w = np.zeros((1, 2, 3, 3), np.float32)
    w[0, 1, 2, 0] = 4.0      # k = (1*3 + 2)*3 + 0 = 15
    w[0, 0, 1, 2] = -1.0     # k = (0*3 + 1)*3 + 2 = 5
    p = oracle.pack(w)
    assert p["col_idx"].tolist() == [5, 15]
    assert p["vals"].tolist() == [-1.0, 4.0]


@pytest.mark.parametrize("seed", range(5))
def test_pack_properties_and_roundtrip(seed):
    w = small_w(seed, shape=(9, 4, 3, 3), sparsity=[0.0, 0.5, 0.9, 0.99, 1.0][seed])
    if seed == 2:
        w[3] = 0          # an all-zero row
        w[5] = 1.5        # a fully dense row
    p = oracle.pack(w)
    cout = w.shape[0]
    assert sorted(p["perm"].tolist()) == list(range(cout))
    assert p["row_ptr"][0] == 0 and p["row_ptr"][-1] == np.count_nonzero(w)
    nnz = np.diff(p["row_ptr"])
    assert (nnz[:-1] >= nnz[1:]).all()
    for i in range(cout):
        cols = p["col_idx"][p["row_ptr"][i]:p["row_ptr"][i + 1]]
        assert (np.diff(cols) > 0).all()
        assert np.count_nonzero(w[p["perm"][i]]) == len(cols)
    # ties keep ascending channel order
    for i in range(cout - 1):
        if nnz[i] == nnz[i + 1]:
            assert p["perm"][i] < p["perm"][i + 1]
    u = oracle.unpack(p)
    assert np.array_equal(u, w)
    assert np.array_equal(u.view(np.uint32), np.where(w == 0, np.float32(0), w).view(np.uint32))


def test_pack_negative_zero_denormal_nan():
    w = np.zeros((2, 4, 1, 1), np.float32)
    w[0, 0] = -0.0
    w[0, 1] = np.float32(1e-42)      # denormal: kept
    w[1, 2] = np.nan                 # NaN != 0: kept
    w[1, 3] = np.inf
    p = oracle.pack(w)
    assert p["row_ptr"].tolist() == [0, 2, 3]
    assert p["perm"].tolist() == [1, 0]
    assert p["col_idx"].tolist() == [2, 3, 1]


def test_pack_fp16_keeps_fp32_nonzero_test():
    w = np.zeros((1, 3, 1, 1), np.float32)
    w[0, 0] = 1e-10       # rounds to fp16 zero but stays an explicit entry
    w[0, 2] = 0.1
    p = oracle.pack(w, np.float16)
    assert p["col_idx"].tolist() == [0, 2]
    assert p["vals"].dtype == np.float16
    assert p["vals"][0] == 0 and p["vals"][1] == np.float16(0.1)


def test_conv_from_unpacked_equals_conv_from_dense():
    w = small_w(11, (6, 5, 3, 3), 0.8)
    x = np.random.default_rng(12).standard_normal((1, 5, 8, 8)).astype(np.float32)
    a = oracle.conv2d_f64(x, w, None, None, 1, 1, True)
    b = oracle.conv2d_f64(x, oracle.unpack(oracle.pack(w)), None, None, 1, 1, True)
    assert np.array_equal(a, b)


def test_run_net_matches_manual_composition():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    ops = [
        wl.Op("conv", "c1", 0, 1, 3, 8, 3, 2, 1, 0.0, True),
        wl.Op("maxpool", "p", 1, 2, k=3, stride=2, pad=1),
        wl.Op("conv", "a", 2, 3, 8, 4, 1, 1, 0, 0.5, True),
        wl.Op("conv", "b", 3, 4, 4, 4, 3, 1, 1, 0.5, True),
        wl.Op("conv", "p", 2, 5, 8, 16, 1, 1, 0, 0.5, False),
        wl.Op("conv", "c", 4, 6, 4, 16, 1, 1, 0, 0.5, True, res=5),
        wl.Op("avgpool", "g", 6, 7),
        wl.Op("fc", "fc", 7, 8, 16, 5, sparsity=0.5, relu=False),
    ]
    x, ws, bs = wl.net_tensors(ops, "unit-net", (2, 3, 17, 17))
    y, ins, outs = oracle.run_net(ops, x, ws, bs)
    t = lambda a: torch.from_numpy(np.asarray(a)).double()
    h = torch.relu(F.conv2d(t(x), t(ws[0]), t(bs[0]), stride=2, padding=1))
    h = F.max_pool2d(h, 3, 2, 1)
    a = torch.relu(F.conv2d(h, t(ws[2]), t(bs[2])))
    b = torch.relu(F.conv2d(a, t(ws[3]), t(bs[3]), padding=1))
    p = F.conv2d(h, t(ws[4]), t(bs[4]))
    c = torch.relu(F.conv2d(b, t(ws[5]), t(bs[5])) + p)
    g = c.mean(dim=(2, 3))
    ref = g @ t(ws[7]).reshape(5, 16).T + t(bs[7])
    assert y.shape == (2, 5, 1, 1)
    np.testing.assert_allclose(y[:, :, 0, 0], ref.numpy(), rtol=2e-5, atol=2e-6)
    assert len(ins) == len(outs) == len(ops)
    assert np.array_equal(ins[5], outs[3])


def _torch_fp16_net(ops, x, ws, bs, jitter=None):
    """The same op list evaluated with torch float64 primitives and an explicit rounding of
    every weight tensor and every layer output to IEEE binary16 (bias stays fp32): the fp16
    storage semantics written out independently of oracle.run_net.  `jitter`, if given,
    perturbs every pre-rounding layer result relatively (a stand-in for another summation
    order) and is used to exercise the propagated error bound."""
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).double()
    h16 = lambda v: v.to(torch.float16).double()
    bufs = {0: h16(t(x))}
    outs = []
    rng = np.random.default_rng(5)
    for i, op in enumerate(ops):
        src = bufs[op.src]
        if op.kind == "conv":
            y = F.conv2d(src, h16(t(ws[i])), t(bs[i]), stride=op.stride, padding=op.pad)
            if op.res >= 0:
                y = y + bufs[op.res]
        elif op.kind == "dwconv":
            y = F.conv2d(src, h16(t(ws[i])), t(bs[i]), stride=op.stride, padding=op.pad, groups=src.shape[1])
        elif op.kind == "fc":
            y = src.reshape(src.shape[0], -1) @ h16(t(ws[i])).reshape(op.cout, -1).T + t(bs[i])
            y = y.reshape(y.shape[0], y.shape[1], 1, 1)
        elif op.kind == "maxpool":
            y = F.max_pool2d(src, op.k, op.stride, op.pad)
        elif op.kind == "avgpool2d":
            y = F.avg_pool2d(src, op.k, op.stride, op.pad, count_include_pad=False)
        elif op.kind == "avgpool":
            y = src.mean(dim=(2, 3), keepdim=True)
        elif op.kind == "concat":
            y = torch.cat([bufs[b] for b in op.srcs], dim=1)
        if op.kind in ("conv", "dwconv", "fc") and op.relu:
            y = torch.relu(y)
        if jitter and op.kind in ("conv", "dwconv", "fc"):
            y = y * t(1.0 + jitter * rng.uniform(-1.0, 1.0, size=tuple(y.shape)))
        y = h16(y)
        bufs[op.dst] = y
        outs.append(y.numpy())
    return outs


def _fp16_dw_net():
    ops = [
        wl.Op("conv", "stem", 0, 1, 3, 8, 3, 2, 1, 0.0, True),
        wl.Op("dwconv", "dw1", 1, 2, 8, 8, 3, 1, 1, 0.0, True),
        wl.Op("conv", "pw1", 2, 3, 8, 12, 1, 1, 0, 0.5, False),
        wl.Op("dwconv", "dw2", 3, 4, 12, 12, 3, 2, 1, 0.3, True),
        wl.Op("conv", "pw2", 4, 5, 12, 12, 1, 1, 0, 0.5, True),
        wl.Op("conv", "b", 5, 6, 12, 12, 3, 1, 1, 0.6, True, res=4),
        wl.Op("avgpool2d", "ap", 6, 7, k=3, stride=1, pad=1),
        wl.Op("maxpool", "mp", 6, 8, k=3, stride=1, pad=1),
        wl.Op("concat", "cat", 7, 9, srcs=(7, 8, 5)),
        wl.Op("avgpool", "g", 9, 10),
        wl.Op("fc", "fc", 10, 11, 36, 5, sparsity=0.5, relu=False),
    ]
    return ops, (2, 3, 19, 17)


def test_run_net_fp16_with_depthwise_matches_explicit_rounding():
    """Pins the interpreter's fp16 mode and its depthwise dispatch: weights and every
    activation rounded to binary16, sums in higher precision, one rounding per layer."""
    ops, shape = _fp16_dw_net()
    x, ws, bs = wl.net_tensors(ops, "unit-net-16", shape)
    y, ins, outs = oracle.run_net(ops, x.astype(np.float16), ws, bs, dtype=np.float16)
    assert y.dtype == np.float16 and all(o.dtype == np.float16 for o in outs)
    want = _torch_fp16_net(ops, x, ws, bs)
    for i, op in enumerate(ops):
        a, b = outs[i].astype(np.float64), want[i]
        assert a.shape == b.shape, op.name
        # both are a correctly rounded value of the same exact sum up to float64 noise: equal,
        # except where that noise straddles a rounding boundary (one fp16 step, rarely)
        step = 2.0 ** -10 * np.maximum(np.abs(a), 2.0 ** -14)
        assert (np.abs(a - b) <= step).all(), op.name
        assert (a == b).mean() > 0.995, (op.name, (a == b).mean())
    # the fp32 mode of the same graph, for the depthwise dispatch alone
    y32, _, outs32 = oracle.run_net(ops, x, ws, bs)
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).double()
    ref_dw1 = torch.relu(F.conv2d(t(outs32[0]), t(ws[1]), t(bs[1]), padding=1, groups=8)).numpy()
    np.testing.assert_allclose(outs32[1], ref_dw1, rtol=1e-6, atol=1e-7)


def test_propagated_chain_bound_holds_and_is_not_vacuous():
    """util.chain_bounds (the gate of the chained GPU tests): an independent evaluation whose
    every layer is off by up to 3e-5 relative before rounding -- what another summation order
    may do -- stays inside the bound, in both storage types; an evaluation with a dropped
    term does not; and the bound is a small fraction of the tensor's scale."""
    from util import chain_bounds, assert_within_bound
    ops, shape = _fp16_dw_net()
    x, ws, bs = wl.net_tensors(ops, "unit-net-16", shape)
    y, ins, outs = oracle.run_net(ops, x.astype(np.float16), ws, bs, dtype=np.float16)
    bounds = chain_bounds(ops, ins, outs, ws, bs, True)
    other = _torch_fp16_net(ops, x, ws, bs, jitter=3e-5)
    for i, op in enumerate(ops):
        assert_within_bound(other[i], outs[i], bounds[i], op.name)
    assert bounds[-1].max() < 0.05 * np.abs(outs[-1].astype(np.float64)).max()
    broken = [w.copy() for w in ws[:5]] + list(ws[5:])
    nz = np.flatnonzero(broken[2])
    broken[2].reshape(-1)[nz[0]] = 0.0                         # one pointwise weight dropped
    bad = _torch_fp16_net(ops, x, broken, bs)
    with pytest.raises(AssertionError):
        for i, op in enumerate(ops):
            assert_within_bound(bad[i], outs[i], bounds[i], op.name)
