"""The seeded generators: determinism, exact sparsity, exact zeros, layer tables."""
import os

import numpy as np

import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_deterministic_and_distinct():
    a = wl.pruned_weights(8, 4, 3, 3, 0.9, "t", 1)
    b = wl.pruned_weights(8, 4, 3, 3, 0.9, "t", 1)
    c = wl.pruned_weights(8, 4, 3, 3, 0.9, "t", 2)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert a.dtype == np.float32 and a.flags.c_contiguous


def test_sparsity_is_exact_and_zeros_are_positive_zero():
    for s, mask in [(0.9, "magnitude"), (0.8, "magnitude"), (0.85, "random"), (0.0, "magnitude"), (1.0, "magnitude")]:
        w = wl.pruned_weights(64, 64, 3, 3, s, "t", 3, mask)
        assert np.count_nonzero(w) == wl.keep_count(w.size, s)
        z = w[w == 0]
        assert not np.signbit(z).any()
    assert wl.keep_count(36864, 0.9) == 3686          # 64x64x3x3 at 90 %
    assert wl.keep_count(10, 0.25) == 8 and wl.keep_count(10, 0.75) == 2   # 7.5 -> 8, 2.5 -> 2 (half-even)


def test_magnitude_mask_keeps_the_largest():
    w = wl.pruned_weights(16, 16, 3, 3, 0.9, "t", 4)
    dense = wl.pruned_weights(16, 16, 3, 3, 0.0, "t", 4)
    kept = np.abs(dense[w != 0])
    dropped = np.abs(dense[w == 0])
    assert kept.min() >= dropped.max()
    assert np.array_equal(w[w != 0], dense[w != 0])


def test_he_normal_scale_and_inputs():
    w = wl.pruned_weights(128, 64, 3, 3, 0.0, "t", 5)
    assert abs(w.std() / np.sqrt(2.0 / 576) - 1) < 0.02
    x = wl.activation((1, 64, 56, 56), "t", 0, relu=True)
    assert (x >= 0).all() and abs((x == 0).mean() - 0.5) < 0.01
    b = wl.bias_vector(1000, "t", 1)
    assert abs(b.std() / 0.01 - 1) < 0.1


def test_row_skew_changes_row_counts_only():
    a = wl.pruned_weights(64, 64, 3, 3, 0.9, "t", 6)
    b = wl.pruned_weights(64, 64, 3, 3, 0.9, "t", 6, row_skew=1.0)
    assert np.count_nonzero(a) == np.count_nonzero(b)
    ra = (a.reshape(64, -1) != 0).sum(1)
    rb = (b.reshape(64, -1) != 0).sum(1)
    assert rb.std() > 2 * ra.std()


def test_resnet50_table():
    g = {}
    for line in open(os.path.join(GOLDEN, "resnet50_shapes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        t = line.split()
        g[t[0]] = [int(v) for v in t[1:]]
    ops = wl.resnet50_ops()
    convs = [o for o in ops if o.kind == "conv"]
    assert len(convs) == g["convs"][0] and sum(o.kind == "fc" for o in ops) == g["fcs"][0]
    cur = {0: (1, 3, 224, 224)}
    macs = weights = 0
    for o in ops:
        n, c, h, w = cur[o.src]
        if o.kind == "conv":
            ho = wl.conv_out_size(h, o.k, o.stride, o.pad)
            macs += o.cout * o.cin * o.k * o.k * ho * ho
            weights += o.cout * o.cin * o.k * o.k
            cur[o.dst] = (n, o.cout, ho, ho)
            if o.res >= 0:
                assert cur[o.res] == cur[o.dst]
        elif o.kind == "maxpool":
            ho = wl.conv_out_size(h, o.k, o.stride, o.pad)
            cur[o.dst] = (n, c, ho, ho)
        elif o.kind == "avgpool":
            cur[o.dst] = (n, c, 1, 1)
        else:
            macs_fc = o.cin * o.cout
            cur[o.dst] = (n, o.cout, 1, 1)
    assert macs == g["dense_conv_macs"][0]
    assert macs + macs_fc == g["dense_total_macs"][0]
    assert weights == g["dense_conv_weights"][0]
    by_name = {o.name: o for o in ops}
    assert by_name["conv3_1b"].stride == 2 and by_name["conv3_1a"].stride == 1
    assert by_name["conv3_1p"].stride == 2 and not by_name["conv3_1p"].relu
    assert by_name["conv1"].sparsity == 0.0 and by_name["conv2_1b"].sparsity == 0.8
    assert by_name["conv2_1a"].sparsity == 0.9 and by_name["fc"].sparsity == 0.9
    shapes = wl.buffer_shapes(ops, (1, 3, 224, 224))
    assert shapes[8] == (1, 1000, 1, 1) and shapes[1] == (1, 64, 112, 112)


def test_vgg16_table():
    ops = wl.vgg16_ops()
    assert sum(o.kind == "conv" for o in ops) == 13
    assert sum(o.kind == "maxpool" for o in ops) == 5
    fcs = [o for o in ops if o.kind == "fc"]
    assert [(o.cin, o.cout) for o in fcs] == [(25088, 4096), (4096, 4096), (4096, 1000)]
    assert [o.relu for o in fcs] == [True, True, False]
    shapes = wl.buffer_shapes(ops, (1, 3, 224, 224))
    assert shapes[5] == (1, 1000, 1, 1)


def test_mobilenet_v1_table():
    ops = wl.mobilenet_v1_ops()
    kinds = [o.kind for o in ops]
    assert kinds.count("dwconv") == 13 and kinds.count("conv") == 14 and kinds.count("fc") == 1
    assert kinds.count("avgpool") == 1 and len(ops) == 29
    # 28 weight layers (the count the architecture is known by) and 4.2 M weights
    x, ws, bs = wl.net_tensors(ops, "mbtest", (1, 3, 224, 224))
    total = sum(w.size for w in ws if w is not None)
    assert 4.1e6 < total < 4.3e6, total
    shapes = wl.buffer_shapes(ops, (1, 3, 224, 224))
    assert shapes[ops[-1].dst] == (1, 1000, 1, 1)
    for o, w in zip(ops, ws):
        if o.kind == "dwconv":
            assert w.shape == (o.cin, 1, 3, 3) and np.count_nonzero(w) == w.size
        if o.kind == "conv" and o.k == 1:
            assert abs(1 - np.count_nonzero(w) / w.size - 0.8) < 1e-3
    # strides: four stride-2 depthwise layers and the stride-2 first layer take 224 down to 7
    assert [o.stride for o in ops if o.kind == "dwconv"].count(2) == 4 and ops[0].stride == 2


def test_mobilenet_v2_table():
    ops = wl.mobilenet_v2_ops()
    kinds = [o.kind for o in ops]
    assert kinds.count("dwconv") == 17 and kinds.count("conv") == 35 and kinds.count("fc") == 1
    assert sum(o.res >= 0 for o in ops) == 10           # blocks with stride 1 and equal widths
    assert all(not o.relu for o in ops if o.name.endswith("_project"))
    x, ws, bs = wl.net_tensors(ops, "mbtest2", (1, 3, 224, 224))
    total = sum(w.size for w in ws if w is not None)
    assert 3.4e6 < total < 3.55e6, total
    shapes = wl.buffer_shapes(ops, (1, 3, 224, 224))
    assert shapes[ops[-1].dst] == (1, 1000, 1, 1)
    # a residual is read from a buffer no op of its block overwrites
    for i, o in enumerate(ops):
        if o.res >= 0:
            blk = o.name.split("_")[0]
            assert all(p.dst != o.res for p in ops[:i + 1] if p.name.startswith(blk + "_"))


def test_embed_filter_and_factorized_branch_table():
    w = wl.pruned_weights(4, 3, 1, 7, 0.5, "emb", 1)
    e = wl.embed_filter(w, 7)
    assert e.shape == (4, 3, 7, 7) and np.array_equal(e[:, :, 3, :], w[:, :, 0, :])
    assert np.count_nonzero(e) == np.count_nonzero(w)
    e[:, :, 3, :] = 0
    assert not e.any()
    with np.testing.assert_raises(ValueError):
        wl.embed_filter(wl.pruned_weights(2, 2, 2, 7, 0.0, "emb", 2), 7)      # even height cannot be centred
    ops = wl.factorized_7x7_branch_ops()
    assert [(o.kh, o.kw) for o in ops] == [(0, 0), (7, 1), (1, 7), (7, 1), (1, 7)]
    x, ws, bs = wl.net_tensors(ops, "embt", (1, 768, 17, 17))
    for o, wt in zip(ops[1:], ws[1:]):
        assert wt.shape == (o.cout, o.cin, 7, 7)
        rows = np.abs(wt).sum(axis=(0, 1, 3)) > 0
        cols = np.abs(wt).sum(axis=(0, 1, 2)) > 0
        assert rows.sum() == o.kh and cols.sum() == o.kw      # nonzeros only on the centred kh x kw taps
    assert wl.buffer_shapes(ops, (1, 768, 17, 17))[ops[-1].dst] == (1, 192, 17, 17)
