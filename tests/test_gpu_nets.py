"""GPU parity for whole networks through cadnn_run_net (full-size configurations)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from util import (TOL_F32, TOL_F16, F16_ULP, assert_close, assert_layer_close, assert_chain_close,
                  assert_net_close, cond_conv, cond_fc, cond_depthwise, rel_errors)

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


def check_layers_in_isolation(cad, ops, ws, bs, ins, outs, tol, dtype, which=None):
    """Each conv/fc of the net on the ORACLE's input for that layer (sensitive to a bug in
    one branch, which an end-to-end check dominated by identity shortcuts can hide)."""
    worst = 0.0
    f16 = dtype == cad.F16
    npdt = np.float16 if f16 else np.float32
    for i, op in enumerate(ops):
        if which is not None and i not in which:
            continue
        if op.kind == "conv":
            h = cad.cadnn_pack_weights(ws[i], dtype)
            res = None
            if op.res >= 0:
                j = max(k for k in range(i) if ops[k].dst == op.res) if op.res != 0 else -1
                res = outs[j] if j >= 0 else ins[0]
            y = cad.cadnn_sparse_conv2d(h, dev(ins[i]), op.stride, op.pad, dev(bs[i]),
                                        None if res is None else dev(res), op.relu)
            cond = cond_conv(ins[i], ws[i].astype(npdt), bs[i], res, op.stride, op.pad)
        elif op.kind == "dwconv":
            h = cad.cadnn_pack_weights(ws[i], dtype)
            y = cad.cadnn_depthwise_conv2d(h, dev(ins[i]), op.stride, op.pad, dev(bs[i]), op.relu)
            cond = cond_depthwise(ins[i], ws[i].astype(npdt), bs[i], op.stride, op.pad)
        elif op.kind == "fc":
            h = cad.cadnn_pack_weights(ws[i], dtype)
            y = cad.cadnn_sparse_fc(h, dev(ins[i].reshape(ins[i].shape[0], -1)), dev(bs[i]), op.relu)
            y = y.reshape(outs[i].shape)
            cond = cond_fc(ins[i], ws[i].astype(npdt), bs[i]).reshape(outs[i].shape)
        elif op.kind == "maxpool":
            y = cad.cadnn_maxpool2d(dev(ins[i]), op.k, op.stride, op.pad)
            h = None
        elif op.kind == "avgpool2d":
            y = cad.cadnn_avgpool2d(dev(ins[i]), op.k, op.stride, op.pad)
            h = None
        elif op.kind == "concat":
            continue
        else:
            y = cad.cadnn_global_avgpool(dev(ins[i]))
            h = None
        torch.cuda.synchronize()
        if op.kind in ("conv", "fc", "dwconv"):
            e = assert_layer_close(y.cpu().numpy(), outs[i], cond, tol, f"layer {i} {op.name}", f16=f16)
        else:
            # pools: the maximum is exact; a mean is an fp32 sum of the window rounded once to
            # the storage type (one fp16 step where both sides round values that agree to 1e-6)
            e = assert_close(y.cpu().numpy(), outs[i], F16_ULP if f16 else 1e-6, f"layer {i} {op.name}")
        worst = max(worst, e[0])
        if h is not None:
            h.free()
    return worst


def test_config2_resnet50_fp32(cad):
    ops = wl.resnet50_ops()
    shape = (1, 3, 224, 224)
    x, ws, bs = wl.net_tensors(ops, "c2", shape)
    ref, ins, outs = oracle.run_net(ops, x, ws, bs)
    worst = check_layers_in_isolation(cad, ops, ws, bs, ins, outs, TOL_F32, cad.F32)
    print("resnet50 per-layer worst E_inf", worst)
    net = cad.build_net(ops, ws, bs, shape, cad.F32, use_graph=True)
    xd = dev(x)
    for rep in range(3):
        y = net.run(xd)
        torch.cuda.synchronize()
        e = assert_chain_close(y.cpu().numpy(), ref, cond_fc(ins[-1], ws[-1], bs[-1]), TOL_F32,
                               f"resnet50 end to end (replay {rep})")
    print("resnet50 end-to-end", e)
    ms = net.profile(xd, y, repeats=2)
    assert ms.shape == (len(ops),) and (ms > 0).all()
    net.free()


def test_config2_resnet50_fp32_in_the_benchmark_configuration(cad):
    """The launch configuration bench.py times: the saved per-layer kernel choice that ships
    with the package, default layouts and fusions, one HIP graph replayed."""
    import json
    import os
    path = os.path.join(os.path.dirname(cad.__file__), "tuned", "resnet50_c2_f32_n1.json")
    names = json.load(open(path))["variants"]
    ops = wl.resnet50_ops()
    assert len(names) == len(ops)
    shape = (1, 3, 224, 224)
    x, ws, bs = wl.net_tensors(ops, "c2", shape)
    ref, ins, outs = oracle.run_net(ops, x, ws, bs)
    net = cad.build_net(ops, ws, bs, shape, cad.F32, use_graph=True)
    net.set_variants(names)                      # raises if a saved name does not fit this build
    assert net.variants() == names
    kinds = {n.split("_")[0] for n in names}
    assert {"slinear", "dense", "fused", "sfc"} <= kinds, kinds
    xd = dev(x)
    cond = cond_fc(ins[-1], ws[-1], bs[-1])
    for rep in range(3):
        y = net.run(xd)
        torch.cuda.synchronize()
        e = assert_chain_close(y.cpu().numpy(), ref, cond, TOL_F32, f"resnet50 saved tuning (replay {rep})")
    # sampled intermediate tensors of the same run against the oracle's
    for name in ("conv4_6c", "conv5_3a", "conv5_3b"):
        i = next(k for k, o in enumerate(ops) if o.name == name)
        if any(o.dst == ops[i].dst for o in ops[i + 1:]):
            continue                              # buffer id reused by a later op
        got = net.read_buffer(ops[i].dst, outs[i].shape)
        assert_net_close(got, outs[i], TOL_F32, name + " inside the tuned net")
    print("resnet50 saved tuning end-to-end", e)
    net.free()


def test_config4_vgg16_fp32(cad):
    ops = wl.vgg16_ops()
    shape = (1, 3, 224, 224)
    x, ws, bs = wl.net_tensors(ops, "c4", shape)
    ref, ins, outs = oracle.run_net(ops, x, ws, bs)
    worst = check_layers_in_isolation(cad, ops, ws, bs, ins, outs, TOL_F32, cad.F32)
    print("vgg16 per-layer worst E_inf", worst)
    net = cad.build_net(ops, ws, bs, shape, cad.F32, use_graph=True)
    y = net.run(dev(x))
    torch.cuda.synchronize()
    print("vgg16 end-to-end", assert_chain_close(y.cpu().numpy(), ref, cond_fc(ins[-1], ws[-1], bs[-1]),
                                                 TOL_F32, "vgg16 end to end"))
    net.free()


@pytest.mark.parametrize("version,dtype_name,n", [(1, "f32", 1), (1, "f16", 4), (2, "f32", 1), (2, "f16", 2)])
def test_mobilenet(cad, version, dtype_name, n):
    """Second workload family (the paper's Table 2 lists MobileNet-V1 and -V2): depthwise layers
    chained with pruned pointwise layers (V2: with residual adds on linear projections), every
    layer in isolation and the whole net, with and without the net-level fusions and layouts."""
    f16 = dtype_name == "f16"
    dtype, npdt, tol = (cad.F16, np.float16, TOL_F16) if f16 else (cad.F32, np.float32, TOL_F32)
    ops = wl.mobilenet_v1_ops() if version == 1 else wl.mobilenet_v2_ops()
    ndw = sum(o.kind == "dwconv" for o in ops)
    assert ndw == (13 if version == 1 else 17)
    shape = (n, 3, 224, 224)
    x, ws, bs = wl.net_tensors(ops, f"mbv{version}", shape)
    xs = x.astype(npdt)
    ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
    which = None if not f16 else set(range(0, len(ops), 3))
    worst = check_layers_in_isolation(cad, ops, ws, bs, ins, outs, tol, dtype, which=which)
    print("mobilenet per-layer worst E_inf", worst)
    cond = cond_fc(ins[-1], ws[-1].astype(npdt), bs[-1])
    for kw in ({}, {"plain_layout": True, "fuse": False}):
        net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=True, **kw)
        names = [net.op_variant(i) for i, o in enumerate(ops) if o.kind == "dwconv"]
        # depthwise layers on images of at most 28 x 28 run inside the layer that feeds them
        fused = 0 if kw else (9 if version == 1 else 13)
        assert names.count("fused") == fused and names.count("dwconv") == ndw - fused, names
        xd = dev(xs)
        for rep in range(2):
            y = net.run(xd)
            torch.cuda.synchronize()
            e = assert_chain_close(y.cpu().numpy(), ref, cond, tol, f"mobilenet end to end {kw} (replay {rep})")
        # the last depthwise output (no later op reuses its buffer id), read back from the workspace
        i = max(k for k, o in enumerate(ops) if o.kind == "dwconv")
        assert not any(o.dst == ops[i].dst for o in ops[i + 1:])
        got = net.read_buffer(ops[i].dst, outs[i].shape)
        assert_net_close(got, outs[i], tol, "last depthwise output inside the net")
        net.free()
    print("mobilenet end-to-end", e)


def stage_ends(ops):
    """First and last convolution of every stage of the ResNet-50 ladder (plus the stem and
    the FC): the layers whose shapes differ most, each checked in isolation."""
    pick = {0, len(ops) - 1}
    for stage in (2, 3, 4, 5):
        idx = [i for i, o in enumerate(ops) if o.kind == "conv" and o.name.startswith(f"conv{stage}_")]
        pick.update({idx[0], idx[1], idx[-2], idx[-1]})     # 1x1 reduce + 3x3 of the first block, 3x3 + 1x1 expand of the last
    return pick


@pytest.mark.parametrize("n,s", [(1, 0.8), (8, 0.5), (32, 0.8), (1, 0.5), (1, 0.7), (1, 0.9), (1, 0.95), (8, 0.7), (8, 0.95), (32, 0.5)])
def test_config3_resnet50_fp16(cad, n, s):
    """configs[3]: the ResNet-50 stack in fp16 storage over the batch sizes and the uniform
    sparsity sweep it names.  Layers in isolation on the oracle's own inputs (a spread of
    layers at small batch; the first and last layers of every stage at batch 32), then the
    whole chain; the chain is run twice with a second input in between, so that a replay
    cannot lean on what the first left behind."""
    ops = wl.resnet50_ops(uniform=s)
    shape = (n, 3, 224, 224)
    x, ws, bs = wl.net_tensors(ops, f"c3-{s}", shape)
    x16 = x.astype(np.float16)
    ref, ins, outs = oracle.run_net(ops, x16, ws, bs, dtype=np.float16)
    convs = [i for i, o in enumerate(ops) if o.kind in ("conv", "fc")]
    subset = stage_ends(ops) if n >= 32 else set(convs[:3] + convs[-4:] + convs[20:23])
    worst = check_layers_in_isolation(cad, ops, ws, bs, ins, outs, TOL_F16, cad.F16, which=subset)
    net = cad.build_net(ops, ws, bs, shape, cad.F16, use_graph=True)
    cond = cond_fc(ins[-1], ws[-1].astype(np.float16), bs[-1])
    xd = dev(x16)
    y = net.run(xd)
    torch.cuda.synchronize()
    e = assert_chain_close(y.cpu().numpy(), ref, cond, TOL_F16, "fp16 chain")
    if n <= 8:
        x2 = wl.activation(shape, f"c3-{s}", 99, relu=False).astype(np.float16)
        ref2, ins2, _ = oracle.run_net(ops, x2, ws, bs, dtype=np.float16)
        y2 = net.run(dev(x2))
        torch.cuda.synchronize()
        assert_chain_close(y2.cpu().numpy(), ref2, cond_fc(ins2[-1], ws[-1].astype(np.float16), bs[-1]), TOL_F16,
                           "fp16 chain, second input")
    print("resnet50 fp16", n, s, "per-layer worst E_inf", worst, "end-to-end", e)
    net.free()


@pytest.mark.parametrize("dtype_name", ["f32", "f16"])
def test_factorized_7x7_branch(cad, dtype_name):
    """Inception-V3's 1x7 / 7x1 layers (the paper's Table 2 names the model) through the same
    ABI: each rectangular filter bank is centred in a 7x7 one with padding 3, whose extra taps
    are exact zeros and are never stored.  Each layer alone on a plain tensor (LDS-staged
    kernels) and the chain inside a net (halo layouts, linear-address kernels)."""
    f16 = dtype_name == "f16"
    dtype, npdt, tol = (cad.F16, np.float16, TOL_F16) if f16 else (cad.F32, np.float32, TOL_F32)
    ops = wl.factorized_7x7_branch_ops()
    shape = (2, 768, 17, 17)
    x, ws, bs = wl.net_tensors(ops, "incep", shape, input_relu=True)
    xs = x.astype(npdt)
    ref, ins, outs = oracle.run_net(ops, xs, ws, bs, dtype=npdt)
    for i, op in enumerate(ops):
        if op.kh:
            h = cad.cadnn_pack_weights(ws[i], dtype)
            assert cad.cadnn_packed_nnz(h) == wl.keep_count(op.cout * op.cin * op.kh * op.kw, op.sparsity)
            h.free()
    check_layers_in_isolation(cad, ops, ws, bs, ins, outs, tol, dtype)
    net = cad.build_net(ops, ws, bs, shape, dtype, use_graph=True)
    names = [net.op_variant(i) for i in range(len(ops))]
    assert all(n.startswith("slinear") for n in names), names
    for rep in range(2):
        y = net.run(dev(xs))
        torch.cuda.synchronize()
        cond = cond_conv(ins[-1], ws[-1].astype(npdt), bs[-1], None, 1, 3)
        e = assert_chain_close(y.cpu().numpy(), ref, cond, tol, f"factorized branch (replay {rep})")
    print("factorized 7x7 branch", names, e)
    net.free()


def test_inception_v3(cad):
    """The fourth model of the paper's Table 2: 94 convolutions (5x5, 3x3, strided, and 1x7 / 7x1 /
    1x3 / 3x1 filters carried in square banks), 9 windowed average pools, 4 max pools and 11
    channel concatenations whose sources are written in place.  A sample of layers in isolation on
    the oracle's inputs, then the whole net."""
    ops = wl.inception_v3_ops()
    shape = (1, 3, 299, 299)
    x, ws, bs = wl.net_tensors(ops, "iv3", shape)
    ref, ins, outs = oracle.run_net(ops, x, ws, bs)
    which = set(range(0, len(ops), 5)) | {i for i, o in enumerate(ops) if o.kind == "avgpool2d"}
    worst = check_layers_in_isolation(cad, ops, ws, bs, ins, outs, TOL_F32, cad.F32, which=which)
    print("inception per-layer worst E_inf", worst)
    net = cad.build_net(ops, ws, bs, shape, cad.F32, use_graph=True)
    names = [net.op_variant(i) for i in range(len(ops))]
    assert [n for n, o in zip(names, ops) if o.kind == "concat"] == ["in place"] * 11, names
    xd = dev(x)
    cond = cond_fc(ins[-1], ws[-1], bs[-1])
    for rep in range(2):
        y = net.run(xd)
        torch.cuda.synchronize()
        e = assert_chain_close(y.cpu().numpy(), ref, cond, TOL_F32, f"inception end to end (replay {rep})")
    for name in ("a3_cat", "c2_cat", "e1_cat"):
        i = next(k for k, o in enumerate(ops) if o.name == name)
        got = net.read_buffer(ops[i].dst, outs[i].shape)
        assert_net_close(got, outs[i], TOL_F32, name + " inside the net")
    print("inception end-to-end", e)
    net.free()


def test_runs_are_bit_identical(cad):
    """Nothing on the path uses atomics or depends on scheduling: repeated graph replays, a run
    without a graph and a second net built from the same tensors give the same bits."""
    ops = wl.resnet50_ops()
    shape = (2, 3, 224, 224)
    x, ws, bs = wl.net_tensors(ops, "c2", shape)
    xd = dev(x)
    net = cad.build_net(ops, ws, bs, shape, cad.F32, use_graph=True)
    first = net.run(xd).clone()
    torch.cuda.synchronize()
    for _ in range(20):
        y = net.run(xd)
    torch.cuda.synchronize()
    assert torch.equal(y, first)
    eager = cad.build_net(ops, ws, bs, shape, cad.F32, use_graph=False)
    y2 = eager.run(xd)
    torch.cuda.synchronize()
    assert torch.equal(y2, first)
    net.free()
    eager.free()
