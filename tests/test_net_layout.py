"""CPU-only checks of the net runner's layout decisions (no GPU): halos, de-interleaved
tensors, fusions and in-place concatenation, through cadnn_net_op_info."""
import numpy as np
import pytest

import workloads as wl
import paper_1905_00571_amd as cad


def plan(ops, shape, tag, **kw):
    _, ws, _ = wl.net_tensors(ops, tag, shape)
    return cad.plan_net(ops, ws, shape, **kw)


def region_bytes(info, n, elem=4):
    return (n * info["image"] * elem + 255) // 256 * 256


def test_resnet50_layout():
    ops = wl.resnet50_ops()
    infos, nbytes = plan(ops, (1, 3, 224, 224), "c2")
    by = {o.name: i for o, i in zip(ops, infos)}
    idx = {o.name: k for k, o in enumerate(ops)}
    # a zero halo of the reader's padding around everything a 3x3 layer reads, none elsewhere
    for o, i in zip(ops, infos):
        readers = [r for r in ops if r.src == o.dst and ops.index(r) > ops.index(o)]
        nxt = next((r for r in ops[idx[o.name] + 1:] if r.src == o.dst), None)
        if nxt is not None and nxt.kind == "conv" and nxt.k == 3:
            assert (i["halo_h"], i["halo_w"]) == (1, 1), o.name
        elif o.name != "conv1":
            assert (i["halo_h"], i["halo_w"]) == (0, 0), o.name
    # the four projection shortcuts are computed inside the layers that add them, the pool inside the last layer
    fused = {o.name: ops[i["fused_into"]].name for o, i in zip(ops, infos) if i["fused_into"] >= 0}
    assert fused == {"conv2_1p": "conv2_1c", "conv3_1p": "conv3_1c", "conv4_1p": "conv4_1c",
                     "conv5_1p": "conv5_1c", "gap": "conv5_3c"}
    # tensors read by stride-2 layers are de-interleaved: a block input read by a strided
    # projection (through the layer it is fused into) and the 1x1 output read by a strided 3x3
    s2d = sorted(o.name for o, i in zip(ops, infos) if i["deinterleaved"])
    assert s2d == sorted(["conv2_3c", "conv3_1a", "conv3_4c", "conv4_1a", "conv4_6c", "conv5_1a"])
    assert by["conv3_1a"]["pitch"] == (56 + 2 + 1) // 2
    # regions back to back, 256-byte aligned, in op order; the last op writes the caller's tensor
    off = 0
    for o, i in zip(ops[:-1], infos[:-1]):
        origin = 0 if i["deinterleaved"] else (i["halo_h"] * i["pitch"] + i["halo_w"]) * 4
        assert i["offset"] == off + origin, o.name
        off += region_bytes(i, 1)
    assert nbytes == off
    assert all(i["slice_of"] == -1 for i in infos)


def test_layout_flags_turn_the_options_off():
    ops = wl.resnet50_ops()
    infos, nbytes = plan(ops, (2, 3, 224, 224), "c2", plain_layout=True, fuse=False)
    assert not any(i["deinterleaved"] for i in infos)
    assert all(i["fused_into"] == -1 for i in infos)
    full, nfull = plan(ops, (2, 3, 224, 224), "c2")
    assert nbytes <= nfull          # a plain layout never needs more room


def test_mobilenet_layout():
    for ops, fused_names in ((wl.mobilenet_v1_ops(), ["dw%d" % i for i in range(5, 14)]),
                             (wl.mobilenet_v2_ops(), ["b%d_dw" % i for i in range(5, 18)])):
        infos, _ = plan(ops, (1, 3, 224, 224), "mb")
        got = [o.name for o, i in zip(ops, infos) if o.kind == "dwconv" and i["fused_into"] >= 0]
        assert got == fused_names
        for o, i in zip(ops, infos):
            if o.kind == "dwconv" and i["fused_into"] >= 0:
                assert ops[i["fused_into"]].dst == o.src          # computed by the layer that feeds it
            nxt = next((r for r in ops[ops.index(o) + 1:] if r.src == o.dst), None)
            if nxt is not None and nxt.kind == "dwconv":
                assert (i["halo_h"], i["halo_w"]) == (1, 1), o.name
        assert not any(i["deinterleaved"] for i in infos)         # depthwise readers take plain tensors


def test_inception_concatenations_are_written_in_place():
    ops = wl.inception_v3_ops()
    infos, nbytes = plan(ops, (1, 3, 299, 299), "iv3")
    idx_of_dst = {o.dst: k for k, o in enumerate(ops)}
    cats = [k for k, o in enumerate(ops) if o.kind == "concat"]
    assert len(cats) == 11
    shapes = wl.buffer_shapes(ops, (1, 3, 299, 299))
    total_slices = 0
    for k in cats:
        cat, ci = ops[k], infos[k]
        ch = 0
        for b in cat.srcs:
            p = idx_of_dst[b]
            pi = infos[p]
            assert pi["slice_of"] == k and pi["slice_channel"] == ch, (cat.name, ops[p].name)
            # same planes, same halo, same image stride; starts ch planes into the region
            assert (pi["halo_h"], pi["halo_w"], pi["pitch"], pi["plane"], pi["image"]) == \
                   (ci["halo_h"], ci["halo_w"], ci["pitch"], ci["plane"], ci["image"])
            assert pi["offset"] == ci["offset"] + ch * ci["plane"] * 4
            ch += shapes[b][1]
            total_slices += 1
        assert ch == shapes[cat.dst][1] and ci["image"] == ch * ci["plane"]
    assert total_slices == 46
    # concatenations are read by 1x1 layers and pools only: no halo; the halo of a branch's
    # intermediate tensor is the padding of the filter that reads it (5x5: 2, 7 taps: 3, 3x3: 1)
    assert all(infos[k]["halo_h"] == 0 and infos[k]["halo_w"] == 0 for k in cats)
    halo = {o.name: (i["halo_h"], i["halo_w"]) for o, i in zip(ops, infos)}
    # (a1_3x3a shares the region of a1_5x5a, see the sibling test below, hence its halo)
    assert halo["a1_5x5a"] == (2, 2) and halo["c1_7a"] == (3, 3) and halo["a1_3x3a"] == (2, 2)
    assert halo["a1_3x3b"] == (1, 1) and halo["e1_3a"] == (1, 1) and halo["stem3"] == (0, 0) and halo["stem2"] == (1, 1)
    # the workspace holds every region that is not a slice of another (a concatenation's, or
    # the region of the first layer of a sibling group)
    off = sum(region_bytes(i, 1) for o, i in zip(ops[:-1], infos[:-1])
              if i["slice_of"] < 0 and not (o.kind == "conv" and i["fused_into"] >= 0 and not i["launched_with"]))
    # ... and the de-interleaved copy of its input that the big 3x3/2 layer of the first grid
    # reduction reads (288 channels of 35 x 35, four 18 x 18 phases each), the only such layer
    copies = {o.name: i["input_copy"] for o, i in zip(ops, infos) if i["input_copy"] >= 0}
    assert copies == {"b_3x3": off}
    assert nbytes == off + 288 * 4 * 18 * 18 * 4


def test_concat_copy_cases_are_not_in_place():
    Op = wl.Op
    ops = [Op("conv", "a", 0, 1, 4, 6, 1, 1, 0, 0.5, True),
           Op("conv", "b", 1, 2, 6, 6, 3, 1, 1, 0.5, True),            # buffer 1 has a second reader
           Op("concat", "inner", 1, 3, srcs=(1, 2)),
           Op("concat", "outer", 3, 4, srcs=(3, 0))]                    # a concatenation and the net input
    infos, _ = plan(ops, (1, 4, 8, 8), "cc")
    assert infos[0]["slice_of"] == -1            # two readers
    assert infos[1]["slice_of"] == 2 and infos[1]["slice_channel"] == 6
    assert infos[2]["slice_of"] == -1            # a nested concatenation is copied


def test_op_info_errors():
    L = cad.lib()
    import ctypes
    net = ctypes.c_void_p()
    assert L.cadnn_net_create(0, 1, 4, 8, 8, ctypes.byref(net)) == 0
    assert L.cadnn_net_add_maxpool(net, 2, 2, 0, 0, 1) == 0
    info = cad.OpInfo()
    assert L.cadnn_net_op_info(net, 1, 0, ctypes.byref(info)) == 1
    assert L.cadnn_net_op_info(net, 0, 0, None) == 1
    assert L.cadnn_net_op_info(net, 0, 0, ctypes.byref(info)) == 0 and info.pitch == 4
    srcs = (ctypes.c_int * 2)(0, 1)
    assert L.cadnn_net_add_concat(net, srcs, 2, 2) == 1           # 8x8 and 4x4 do not stack
    assert L.cadnn_net_add_concat(net, srcs, 0, 2) == 1
    assert L.cadnn_net_add_avgpool(net, 3, 1, 1, 1, 1) == 1       # dst aliases src
    assert L.cadnn_net_add_avgpool(net, 3, 1, 1, 1, 2) == 0
    assert L.cadnn_net_free(net) == 0


def test_inception_sibling_layers_share_a_launch():
    """The 1x1 reduce layers of an Inception module's branches read the same tensor pixel by
    pixel: those that are not concatenation slices become one launch and one region."""
    ops = wl.inception_v3_ops()
    infos, _ = plan(ops, (1, 3, 299, 299), "iv3")
    name_of = [o.name for o in ops]
    merged = {o.name: name_of[i["fused_into"]] for o, i in zip(ops, infos)
              if o.kind == "conv" and i["fused_into"] >= 0 and not i["launched_with"]}
    want = {}
    for m in ("a1", "a2", "a3"):
        want[m + "_3x3a"] = m + "_5x5a"
    for m in ("c1", "c2", "c3", "c4"):
        want[m + "_dbl_a"] = m + "_7a"
    want["d_7a"] = "d_3x3a"
    want["e1_dbl_a"] = "e1_3a"
    want["e2_dbl_a"] = "e2_3a"
    assert merged == want
    by = {o.name: i for o, i in zip(ops, infos)}
    shapes = wl.buffer_shapes(ops, (1, 3, 299, 299))
    for sib, first in want.items():
        a, b = by[first], by[sib]
        c_first = next(o.cout for o in ops if o.name == first)
        # one region: same planes and halo (the larger of the two readers' paddings), the
        # sibling's slice behind the first layer's channels
        assert (b["halo_h"], b["pitch"], b["plane"], b["image"]) == (a["halo_h"], a["pitch"], a["plane"], a["image"])
        assert b["offset"] == a["offset"] + c_first * a["plane"] * 4
        assert b["slice_channel"] == c_first and b["slice_of"] == -1
    assert by["a1_5x5a"]["halo_h"] == 2 and by["c1_7a"]["halo_h"] == 3 and by["d_3x3a"]["halo_h"] == 3
    # without fusion nothing is merged
    plain, nplain = plan(ops, (1, 3, 299, 299), "iv3", fuse=False)
    assert all(i["fused_into"] == -1 for i in plain)
    # ... and every layer has a region of its own again: the workspace size follows the flags
    # (plus the de-interleaved input copy of the one big strided layer, a layout matter, not a fusion)
    assert nplain == sum(region_bytes(i, 1) for i in plain[:-1] if i["slice_of"] < 0) + 288 * 4 * 18 * 18 * 4


def test_inception_independent_layers_share_a_launch():
    """Layers of different branches whose inputs are ready at the same point are launched as one
    kernel (up to eight, while one variant serves them all): they keep their own regions, and
    a layer joins the launch of an EARLIER op only -- never one that produces its input."""
    ops = wl.inception_v3_ops()
    infos, _ = plan(ops, (1, 3, 299, 299), "iv3")
    idx = {o.name: k for k, o in enumerate(ops)}
    groups = {}
    for o, i in zip(ops, infos):
        if i["launched_with"]:
            groups.setdefault(ops[i["fused_into"]].name, []).append(o.name)
    # (a module's pool rides along with its first layers, the pooled branch's 1x1 layer with the second ones)
    assert groups["c1_1x1"] == ["c1_7a", "c1_pool"] and groups["c1_7b"] == ["c1_dbl_b", "c1_pool1x1"]
    assert groups["c1_7c"] == ["c1_dbl_c"] and groups["b_3x3"] == ["b_dbl_a", "b_pool"] and groups["d_3x3a"] == ["d_pool"]
    assert groups["e1_3b"] == ["e1_3c", "e1_dbl_b", "e1_pool1x1"] and groups["e2_dbl_c"] == ["e2_dbl_d"]
    assert groups["a1_5x5b"] == ["a1_3x3b", "a1_pool1x1"] and groups["d_3x3b"] == ["d_7b"]
    assert sum(len(m) for m in groups.values()) == 48
    def ready(k):
        nxt = infos[k]["launched_after"] if infos[k]["launched_after"] >= 0 else infos[k]["fused_into"]
        return ready(nxt) if nxt >= 0 else k
    producer = {}
    for k, o in enumerate(ops):
        if infos[k]["launched_with"]:
            assert o.kind in ("conv", "maxpool", "avgpool2d")
            lead = infos[k]["fused_into"]
            assert lead < k and ops[lead].kind == "conv" and infos[lead]["fused_into"] < 0
            assert ready(producer[o.src]) < lead, o.name           # its input is complete before the shared launch
            assert infos[k]["slice_of"] >= 0 or infos[k]["offset"] != infos[lead]["offset"]   # a region of its own
        producer[o.dst] = k
    # chains have nothing to launch together; without fusion nothing is
    for other in (wl.resnet50_ops(), wl.mobilenet_v1_ops()):
        inf, _ = plan(other, (1, 3, 224, 224), "chain")
        assert not any(i["launched_with"] for i in inf)
    plain, _ = plan(ops, (1, 3, 299, 299), "iv3", fuse=False)
    assert not any(i["launched_with"] or i["launched_after"] >= 0 for i in plain)


def test_random_net_layouts_keep_their_invariants():
    """Host-only properties of the layout of 150 seeded random op graphs (the generator of the
    GPU parity test), with every combination of the layout flags: materialised regions do not
    overlap and lie inside the workspace; a slice lies inside the region it belongs to; an op
    that rides on another op's launch does so on an EARLIER op that really launches, and
    everything it reads is complete by then; an op moved in the launch order goes behind an op
    that launches."""
    import importlib.util
    import os
    spec = importlib.util.spec_from_file_location("random_nets", os.path.join(os.path.dirname(__file__), "test_gpu_random_nets.py"))
    rnd = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(rnd)
    seen = {"launched_with": 0, "launched_after": 0, "slices": 0}
    for seed in range(150):
        ops, shape = rnd.random_net(seed)
        _, ws, _ = wl.net_tensors(ops, f"rnd{seed}", shape)
        n = shape[0]
        for kw in ({}, {"fuse": False}, {"plain_layout": True}):
            infos, nbytes = cad.plan_net(ops, ws, shape, **kw)

            def ready(k):
                nxt = infos[k]["launched_after"] if infos[k]["launched_after"] >= 0 else infos[k]["fused_into"]
                return ready(nxt) if 0 <= nxt < k else k     # (a projection is fused into a LATER op: not a launch it rides on)

            producer = {0: -1}
            spans = []
            for k, (o, i) in enumerate(zip(ops, infos)):
                srcs = list(o.srcs) if o.kind == "concat" else [o.src]
                if o.kind == "conv" and o.res >= 0:
                    srcs.append(o.res)
                seen["launched_with"] += i["launched_with"]
                seen["launched_after"] += i["launched_after"] >= 0
                seen["slices"] += i["slice_of"] >= 0
                if i["launched_with"]:
                    lead = i["fused_into"]
                    assert 0 <= lead < k and infos[lead]["fused_into"] < 0 and ops[lead].kind == "conv", (seed, kw, o.name)
                    assert all(producer[b] >= 0 and ready(producer[b]) < lead for b in srcs), (seed, kw, o.name)
                if i["launched_after"] >= 0:
                    host = i["launched_after"]
                    assert host < k and infos[host]["fused_into"] < 0 and infos[host]["launched_after"] < 0, (seed, kw, o.name)
                    assert all(producer[b] >= 0 and ready(producer[b]) <= host for b in srcs), (seed, kw, o.name)
                producer[o.dst] = k
                if k == len(ops) - 1:
                    continue
                start = i["offset"] - (0 if i["deinterleaved"] else (i["halo_h"] * i["pitch"] + i["halo_w"]) * 4)
                spans.append((k, start, i))
            shapes = wl.buffer_shapes(ops, shape)
            regions = []
            for k, start, i in spans:
                o = ops[k]
                c = shapes[o.dst][1]
                end = start + ((n - 1) * i["image"] + c * i["plane"]) * 4
                assert 0 <= start and end <= nbytes, (seed, kw, o.name)
                sibling = o.kind == "conv" and i["fused_into"] >= 0 and not i["launched_with"] and i["fused_into"] < k
                never_written = i["fused_into"] > k       # a projection computed inside the layer that adds it
                if i["slice_of"] >= 0 or sibling:
                    host = i["slice_of"] if i["slice_of"] >= 0 else i["fused_into"]
                    hs = next(s for kk, s, _ in spans if kk == host)
                    hi = infos[host]
                    assert hs <= start and end <= hs + n * hi["image"] * 4, (seed, kw, o.name)
                elif not never_written:
                    regions.append((start, start + n * i["image"] * 4, o.name))
            regions.sort()
            for (a0, a1, an), (b0, b1, bn) in zip(regions, regions[1:]):
                assert a1 <= b0, (seed, kw, an, bn)
    assert min(seen.values()) >= 20, seen         # the nets do contain what is being checked
