#!/usr/bin/env python3
"""Benchmark of the sparse-inference hot path on one MI355X.

Workload: the full ResNet-50 stack at batch 1 in fp32 (53 pruned convolutions + pools +
the 2048->1000 FC; conv1 dense, 3x3 convs 80 % sparse, 1x1 convs and FC 90 % sparse) on
seeded synthetic tensors.  A step is one whole forward pass through cadnn_run_net (one HIP
graph launch).  Prints ONE JSON line; a per-layer table goes to --layers-out if given.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
TUNED_DIR = os.path.join(ROOT, "paper_1905_00571_amd", "tuned")
DEFAULT_TUNE = os.path.join(TUNED_DIR, "resnet50_c2_f32_n1.json")      # saved per-layer kernel choice
DEFAULT_TRAFFIC = os.path.join(TUNED_DIR, "traffic_resnet50_c2_f32_n1.json")  # measured HBM bytes per launch
FP32_VECTOR_TFLOPS = 157.3   # MI355X vector fp32 (256 CU x 2.4 GHz x 256 flop/clk)
MFMA_FP16_TFLOPS = 2500.0    # MI355X dense fp16 matrix cores


def layer_costs(ops, weights, in_shape, elem):
    """Algorithmic flops and bytes of every op: each activation read once, each output
    written once, each nonzero (value + 16-bit index) read once; flops over nonzero MACs."""
    import numpy as np
    from workloads import conv_out_size
    cur = {0: tuple(in_shape)}
    rows = []
    for i, op in enumerate(ops):
        n, c, h, w = cur[op.src]
        if op.kind == "conv":
            ho, wo = conv_out_size(h, op.k, op.stride, op.pad), conv_out_size(w, op.k, op.stride, op.pad)
            nnz = int(np.count_nonzero(weights[i]))
            out = (n, op.cout, ho, wo)
            flops = 2.0 * nnz * ho * wo * n
            byts = (n * c * h * w + n * op.cout * ho * wo * (2 if op.res >= 0 else 1)) * elem \
                + nnz * (elem + 2) + (op.cout + 1) * 4 + op.cout * 4 + op.cout * 4
            # run as a dense contraction (a matrix-core kernel): every position of the matrix
            dense_flops = 2.0 * op.cout * c * op.k * op.k * ho * wo * n
            dense_byts = byts - nnz * (elem + 2) + op.cout * c * op.k * op.k * elem
        elif op.kind == "dwconv":
            ho, wo = conv_out_size(h, op.k, op.stride, op.pad), conv_out_size(w, op.k, op.stride, op.pad)
            nnz = int(np.count_nonzero(weights[i]))
            out = (n, c, ho, wo)
            flops = 2.0 * nnz * ho * wo * n
            byts = (n * c * h * w + n * c * ho * wo) * elem + c * op.k * op.k * 4 + c * 4
        elif op.kind == "fc":
            nnz = int(np.count_nonzero(weights[i]))
            out = (n, op.cout, 1, 1)
            flops = 2.0 * nnz * n
            byts = (n * c * h * w + n * op.cout) * elem + nnz * (elem + 2) + (op.cout + 1) * 4 + op.cout * 8
        elif op.kind in ("maxpool", "avgpool2d"):
            ho, wo = conv_out_size(h, op.k, op.stride, op.pad), conv_out_size(w, op.k, op.stride, op.pad)
            out = (n, c, ho, wo)
            nnz, flops = 0, 0.0
            byts = (n * c * h * w + n * c * ho * wo) * elem
        elif op.kind == "concat":
            # its sources are written in place by their producers: nothing moves
            c = sum(cur[b][1] for b in op.srcs)
            out = (n, c, h, w)
            nnz, flops, byts = 0, 0.0, 0.0
        else:
            out = (n, c, 1, 1)
            nnz, flops = 0, float(n * c * h * w)
            byts = (n * c * h * w + n * c) * elem
        cur[op.dst] = out
        rows.append({"op": op.name, "kind": op.kind, "in": [n, c, h, w], "out": list(out), "nnz": nnz,
                     "flops": flops, "bytes": float(byts)})
        if op.kind == "conv":
            rows[-1].update({"dense_flops": dense_flops, "dense_bytes": float(dense_byts), "nnz_own": nnz,
                             "bytes_own": float(byts)})
    return rows


KERNEL_OF_PREFIX = {"slinear": "sconv_linear_kernel", "squad": "sconv_quad_kernel", "stile": "sconv_stile_kernel", "sptile": "sconv_ptile_kernel",
                    "swide": "sconv_wtile_kernel",
                    "sdirect": "sconv_direct_kernel", "sconv": "sconv_tile_kernel",
                    "dense": "dense_conv_kernel", "sfc": "sfc_kernel", "dwconv": "dwconv_kernel", "maxpool": "windowpool_kernel",
                    "avgpool": "avgpool_kernel", "avgpool2d": "windowpool_kernel", "concat": "windowpool_kernel",
                    "fused": "(computed inside another op)", "in place": "(written by its producers)"}


def kernel_of(variant: str) -> str:
    """The __global__ function a variant name is an instantiation of."""
    if variant.startswith("dense_mfma") and not variant.endswith("_64x64x32"):
        return "dense_wide_kernel"
    return KERNEL_OF_PREFIX.get(variant.split("_")[0], variant)


MFMA_KERNELS = ("dense_conv_kernel", "dense_wide_kernel")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--layers-out", type=str, default="")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-tune", action="store_true")
    ap.add_argument("--save-tune", type=str, default="", help="write the tuned variant names (JSON)")
    ap.add_argument("--load-tune", type=str, default=DEFAULT_TUNE if os.path.exists(DEFAULT_TUNE) else "",
                    help="pin saved variant names instead of tuning (default: the saved choice for this "
                         "workload that ships with the package)")
    ap.add_argument("--retune", action="store_true", help="ignore --load-tune and time every variant per layer now")
    ap.add_argument("--traffic", type=str, default=DEFAULT_TRAFFIC,
                    help="JSON of HBM bytes per launch per kernel measured with rocprofv3 --pmc "
                         "(written by paper_1905_00571_amd/profile_summary.py)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 256 MiB device copy 10 times (known traffic, for counter calibration)")
    ap.add_argument("--workload", choices=["c2", "c3", "c4", "mobilenet", "mobilenet2", "inception"], default="c2",
                    help="c2 (default, the metric's workload): ResNet-50 fp32, conv1 dense / 3x3 80 %% / 1x1+FC 90 %%; "
                         "c3: ResNet-50 with uniform --sparsity in --dtype at --batch; c4: VGG-16 conv 90 %% / FC 96 %%; "
                         "mobilenet / mobilenet2: MobileNet-V1 / -V2, dense first layer and depthwise filters, "
                         "pointwise 80 %% / FC 90 %%; inception: Inception-V3 at 299x299, first layer dense, "
                         "other convolutions 80 %% / FC 90 %%")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--sparsity", type=float, default=0.8, help="uniform sparsity of workload c3")
    ap.add_argument("--dtype", choices=["f32", "f16"], default="", help="storage type (default f32; c3: f16)")
    ap.add_argument("--dense-compare", action="store_true", default=None,
                    help="also time every distinct convolution shape of the workload as a DENSE layer on the same "
                         "GPU: the library's own MFMA implicit GEMM and MIOpen through torch.nn.functional.conv2d "
                         "(the only use of torch compute anywhere: a comparator).  On by default for the metric's "
                         "workload (a few seconds)")
    ap.add_argument("--no-dense-compare", dest="dense_compare", action="store_false")
    ap.add_argument("--no-fusion", action="store_true", help="launch every op on its own (CADNN_NET_NO_FUSION)")
    ap.add_argument("--plain-layout", action="store_true", help="no de-interleaved tensors (CADNN_NET_PLAIN_LAYOUT)")
    ap.add_argument("--no-layer-profile", action="store_true",
                    help="skip the per-op event pass (for clean rocprofv3 kernel statistics)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives or sharding are part of it); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import workloads as wl
    import paper_1905_00571_amd as cad

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    cad.lib()
    torch.cuda.set_device(0)

    n = args.batch
    shape = (n, 3, 224, 224)
    dt = args.dtype or ("f16" if args.workload == "c3" else "f32")
    if args.workload == "c2":
        ops, tag = wl.resnet50_ops(), "c2"
        desc = "resnet50-sparse %s batch %d (configs[2]): 53 convs + FC, conv1 0 %%, 3x3 80 %%, 1x1+FC 90 %% " \
               "unstructured sparsity, %dx3x224x224 input" % (dt, n, n)
    elif args.workload == "c3":
        ops, tag = wl.resnet50_ops(uniform=args.sparsity), "c3-%s" % args.sparsity
        desc = "resnet50-sparse %s batch %d (configs[3]): every layer %.0f %% unstructured sparsity" % (dt, n, 100 * args.sparsity)
    elif args.workload == "mobilenet":
        ops, tag = wl.mobilenet_v1_ops(), "mbv1"
        desc = "mobilenet-v1-sparse %s batch %d: conv1 and 13 depthwise 3x3 dense, 13 pointwise 80 %%, FC 90 %% " \
               "unstructured sparsity" % (dt, n)
    elif args.workload == "inception":
        shape = (n, 3, 299, 299)
        ops, tag = wl.inception_v3_ops(), "iv3"
        desc = "inception-v3-sparse %s batch %d: first layer dense, 93 convolutions 80 %%, FC 90 %% unstructured " \
               "sparsity, %dx3x299x299 input" % (dt, n, n)
    elif args.workload == "mobilenet2":
        ops, tag = wl.mobilenet_v2_ops(), "mbv2"
        desc = "mobilenet-v2-sparse %s batch %d: conv1 and 17 depthwise 3x3 dense, 34 pointwise 80 %%, FC 90 %% " \
               "unstructured sparsity" % (dt, n)
    else:
        ops, tag = wl.vgg16_ops(), "c4"
        desc = "vgg16-sparse %s batch %d (configs[4]): 13 convs 90 %%, 3 FC 96 %% unstructured sparsity" % (dt, n)
    is_default = args.workload == "c2" and n == 1 and dt == "f32"
    x, ws, bs = wl.net_tensors(ops, tag, shape)
    npdt = np.float16 if dt == "f16" else np.float32
    tdt = torch.float16 if dt == "f16" else torch.float32
    elem = 2 if dt == "f16" else 4
    if args.retune or args.no_tune or (not is_default and args.load_tune == DEFAULT_TUNE):
        args.load_tune = ""     # (the saved choice that ships with the package is for the default workload)
    def make_net(live_tune):
        return cad.build_net(ops, ws, bs, shape, cad.F16 if dt == "f16" else cad.F32, use_graph=not args.no_graph,
                             tune=live_tune, fuse=not args.no_fusion, plain_layout=args.plain_layout)

    net = make_net(not (args.no_tune or args.load_tune))
    tuning = "none" if args.no_tune else "live"
    if args.load_tune:
        try:
            with open(args.load_tune) as f:
                net.set_variants(json.load(f)["variants"])
            tuning = "saved:" + os.path.relpath(args.load_tune, ROOT)
        except Exception as e:      # a saved choice from another build of the library: tune now instead
            print("bench.py: saved tuning not usable (%s); tuning live" % e, file=sys.stderr)
            net.free()
            net = make_net(True)
    xd = torch.from_numpy(x.astype(npdt)).cuda()            # inputs resident in HBM before timing
    y = torch.empty(net.out_shape, dtype=tdt, device="cuda")
    stream = torch.cuda.current_stream()

    if args.dense_compare is None:
        args.dense_compare = is_default
    for _ in range(max(args.warmup, 1)):
        net.run(xd, y, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        net.run(xd, y, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # the spread of single passes: one event between consecutive passes of a second, untimed run
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(min(args.steps, 500) + 1)]
    marks[0].record(stream)
    for m in marks[1:]:
        net.run(xd, y, stream)
        m.record(stream)
    torch.cuda.synchronize()
    per_pass = np.array([a_.elapsed_time(b_) for a_, b_ in zip(marks[:-1], marks[1:])])
    pass_ms = {"p10": float(np.percentile(per_pass, 10)), "median": float(np.median(per_pass)),
               "p90": float(np.percentile(per_pass, 90))}

    # single-inference latency with a host sync after every pass (median)
    lat = []
    for _ in range(min(args.steps, 200)):
        a = time.perf_counter()
        net.run(xd, y, stream)
        torch.cuda.synchronize()
        lat.append((time.perf_counter() - a) * 1e3)
    lat_sync_ms = float(np.median(lat))

    # ---- per-op device time with HIP events on the launch stream, grouped by kernel function
    # (all tile-shape instantiations of one __global__ template count as one kernel)
    if args.calibrate_copy:
        a_ = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b_ = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        a_.zero_()
        for _ in range(10):
            cad.cadnn_device_copy(a_, b_, stream)
        torch.cuda.synchronize()
    if args.save_tune:
        with open(args.save_tune, "w") as f:
            json.dump({"workload": "resnet50-%s-%s-n%d" % (args.workload, dt, n), "variants": net.variants()}, f, indent=1)
    if args.no_layer_profile:
        print(json.dumps({"metric": "sparse ResNet-50 batch-1 latency" if is_default else "latency of " + desc,
                          "value": ms_per_step, "unit": "ms", "note": "per-op pass skipped"}))
        net.free()
        return 0
    # cold caches: a 512 MiB copy (twice the Infinity Cache) before every pass, the pass
    # itself timed with events on the launch stream; the copy also gives an achieved HBM rate
    big_a = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    big_b = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    big_a.zero_()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e2 = torch.cuda.Event(enable_timing=True)
    cold, copy_ms = [], []
    for _ in range(20):
        e0.record(stream)
        cad.cadnn_device_copy(big_a, big_b, stream)
        e1.record(stream)
        net.run(xd, y, stream)
        e2.record(stream)
        torch.cuda.synchronize()
        copy_ms.append(e0.elapsed_time(e1))
        cold.append(e1.elapsed_time(e2))
    lat_cold_ms = float(np.median(cold))
    copy_gbs = 2.0 * (512 << 20) / (float(np.median(copy_ms)) * 1e-3) / 1e9
    del big_a, big_b

    # per-op device time, two ways: every op 20 times back to back (warm caches), and the ops in
    # launch order as a forward pass runs them, every kernel carrying its own start and stop
    # marks.  The second is what the kernels take inside a pass -- the figure a rocprofv3 kernel
    # trace of this command reports -- and is the one used below.
    per_op_ms_warm = net.profile(xd, y, repeats=20, stream=stream)
    per_op_ms = net.profile_in_order(xd, y, repeats=30, stream=stream)
    scratch = torch.zeros(64, dtype=torch.uint8, device="cuda")
    floor_us = cad.cadnn_graph_launch_floor(scratch, 64, 20, stream)
    costs = layer_costs(ops, ws, shape, elem)
    groups = {}
    names = [net.op_variant(i) for i in range(len(ops))]
    # a projection shortcut computed inside its reader: its multiply-adds, input and weights
    # move to the reader; its output write and the reader's residual read no longer exist
    for i, op in enumerate(ops):
        if names[i] != "fused":
            continue
        info = net.op_info(i)
        if info["launched_with"]:
            # an independent layer (or a pool riding along) in another op's kernel launch: nothing
            # is saved but the launch; its work is accounted where it runs
            j = info["fused_into"]
            for key in ("flops", "bytes", "nnz"):
                costs[j][key] = costs[j].get(key, 0) + costs[i].get(key, 0)
            costs[i]["flops"] = costs[i]["bytes"] = 0.0
            continue
        if op.kind in ("avgpool", "dwconv"):
            # pooled (or depthwise-filtered) in the epilogue of the convolution that feeds it: that
            # layer's feature map is neither written nor read back; only the fused op's output is
            j = max(k for k, o in enumerate(ops[:i]) if o.dst == op.src)
            map_bytes = float(np.prod(costs[i]["in"])) * elem
            costs[j]["flops"] += costs[i]["flops"]
            costs[j]["bytes"] += costs[i]["bytes"] - 2.0 * map_bytes
            costs[i]["flops"] = costs[i]["bytes"] = 0.0
            continue
        j = info["fused_into"]
        if j < i:
            # rows of an earlier 1x1 layer's launch on the same input, which is read once; its
            # work moves there
            shared_in = float(np.prod(costs[i]["in"])) * elem
            while names[j] == "fused":       # (the first layer of a sibling group may itself ride on another launch)
                j = net.op_info(j)["fused_into"]
            costs[j]["flops"] += costs[i]["flops"]
            costs[j]["bytes"] += costs[i]["bytes"] - shared_in
            costs[j]["nnz"] += costs[i]["nnz"]
            costs[i]["flops"] = costs[i]["bytes"] = 0.0
            continue
        out_bytes = float(np.prod(costs[i]["out"])) * elem
        costs[j]["flops"] += costs[i]["flops"]
        costs[j]["bytes"] += costs[i]["bytes"] - out_bytes - out_bytes
        costs[j]["nnz"] += costs[i]["nnz"]
        costs[i]["flops"] = costs[i]["bytes"] = 0.0
    for i, op in enumerate(ops):
        name = names[i]
        costs[i]["kernel"] = name
        if name in ("fused", "in place"):
            per_op_ms[i] = 0.0
        costs[i]["ms"] = float(per_op_ms[i])
        costs[i]["ms_warm"] = float(per_op_ms_warm[i])
        t = costs[i]["ms"] * 1e-3
        costs[i]["gflops"] = costs[i]["flops"] / t / 1e9 if t > 0 else 0.0
        costs[i]["gbs"] = costs[i]["bytes"] / t / 1e9 if t > 0 else 0.0
        costs[i]["frac_hbm"] = costs[i]["gbs"] / HBM_PEAK_GBS
        costs[i]["frac_fp32"] = costs[i]["gflops"] / (FP32_VECTOR_TFLOPS * 1e3)
        g = groups.setdefault(kernel_of(name), {"ms": 0.0, "ms_warm": 0.0, "launches": 0, "flops": 0.0, "bytes": 0.0})
        g["ms"] += costs[i]["ms"]
        g["ms_warm"] += costs[i]["ms_warm"]
        g["launches"] += 1
        # a matrix-core kernel's algorithm is the dense contraction: it is priced with that
        # (a fused projection's share is added at the sparse count: a slight under-count)
        mfma = kernel_of(name) in MFMA_KERNELS
        g["flops"] += costs[i]["flops"] + ((costs[i]["dense_flops"] - 2.0 * costs[i]["nnz_own"] * np.prod(costs[i]["out"][2:]) * costs[i]["out"][0]) if mfma else 0.0)
        g["bytes"] += costs[i]["bytes"] + ((costs[i]["dense_bytes"] - costs[i]["bytes_own"]) if mfma else 0.0)
    dom_name, dom = max(groups.items(), key=lambda kv: kv[1]["ms"])
    avg_s = dom["ms"] * 1e-3 / dom["launches"]
    t_hbm = dom["bytes"] / dom["launches"] / (HBM_PEAK_GBS * 1e9)
    t_alu = dom["flops"] / dom["launches"] / (FP32_VECTOR_TFLOPS * 1e12)
    if dom_name in MFMA_KERNELS:
        peak = MFMA_FP16_TFLOPS if dt == "f16" else FP32_VECTOR_TFLOPS     # (dense fp32 MFMA: 157.3 as well)
        achieved = dom["flops"] / dom["launches"] / avg_s / 1e12
        gbs = dom["bytes"] / dom["launches"] / avg_s / 1e9
        note = ("the dense contraction the kernel performs (every position of the weight matrix), not the nonzero "
                "count; both roofs are given, 'bound' is the one that allows the launch less time")
        if t_hbm > dom["flops"] / dom["launches"] / (peak * 1e12):
            roofline = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                        "traffic": None}
        else:
            roofline = {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                        "traffic": None}
        roofline.update({"note": note, "mfma_tflops": achieved, "frac_of_mfma_peak": achieved / peak,
                         "hbm_gbs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS})
    elif t_alu >= t_hbm:
        achieved = dom["flops"] / dom["launches"] / avg_s / 1e12
        roofline = {"bound": "alu", "achieved": achieved, "peak": FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / FP32_VECTOR_TFLOPS, "traffic": None}
    else:
        achieved = dom["bytes"] / dom["launches"] / avg_s / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": None}
    if is_default and args.traffic and os.path.exists(args.traffic):
        with open(args.traffic) as f:
            measured = json.load(f).get("kernels", {})
        if dom_name in measured:
            roofline["traffic"] = measured[dom_name]["hbm_bytes_per_launch"]
            roofline["traffic_source"] = ("not measured in this run: FETCH_SIZE + WRITE_SIZE of the committed rocprofv3 "
                                          "--pmc runs of this command (profiles/), read from " + os.path.relpath(args.traffic, ROOT))
    roofline.update({"kernel": dom_name, "launches_per_step": dom["launches"],
                     "avg_launch_us": avg_s * 1e6,
                     "avg_launch_us_warm": dom["ms_warm"] * 1e3 / dom["launches"],
                     "timing": "ops in launch order, each kernel's own start/stop marks "
                               "(avg_launch_us_warm: each op 20x back to back between two events)",
                     "algorithmic_flops_per_launch": dom["flops"] / dom["launches"],
                     "algorithmic_bytes_per_launch": dom["bytes"] / dom["launches"]})

    roofline["frac_of_measured_copy_rate"] = (roofline["achieved"] / copy_gbs) if roofline["bound"] == "hbm" else None

    # ---- the same layers as dense convolutions on this GPU (comparators)
    dense_cmp = None
    if args.dense_compare:
        def time_us(fn, reps=10):
            for _ in range(5):
                fn()
            a_ = torch.cuda.Event(enable_timing=True)
            b_ = torch.cuda.Event(enable_timing=True)
            a_.record(stream)
            for _ in range(reps):
                fn()
            b_.record(stream)
            torch.cuda.synchronize()
            return a_.elapsed_time(b_) * 1e3 / reps

        memo = {}
        pending = {}
        tot = {"sparse": 0.0, "mfma": 0.0, "miopen": 0.0}
        wins = cnt = by_mfma = 0
        for i, op in enumerate(ops):
            if op.kind != "conv":
                continue
            nn_, c_, h_, w_ = costs[i]["in"]
            key = (c_, op.cout, op.k, op.stride, op.pad, h_, w_)
            if key not in memo:
                xin = torch.randn(nn_, c_, h_, w_, device="cuda").relu_().to(tdt)
                wd = torch.from_numpy(ws[i]).cuda().to(tdt)
                bd = torch.from_numpy(bs[i]).cuda()
                yo = torch.empty(costs[i]["out"], dtype=tdt, device="cuda")
                t_mfma = time_us(lambda: cad.cadnn_dense_conv2d(wd, xin, op.stride, op.pad, bd, None, True, out=yo,
                                                                stream=stream))
                if dt == "f16":
                    # the matrix-core variants through a weight handle (their weight matrix is
                    # part of the plan, as in a net): the best of them is the dense time
                    hd = cad.cadnn_pack_weights(ws[i], cad.F16)
                    for nm in cad.cadnn_conv2d_list_variants(hd, nn_, h_, w_, op.stride, op.pad):
                        if nm.startswith("dense_mfma"):
                            cad.cadnn_conv2d_set_variant(hd, nn_, h_, w_, op.stride, op.pad, nm)
                            t_mfma = min(t_mfma, time_us(lambda: cad.cadnn_sparse_conv2d(
                                hd, xin, op.stride, op.pad, bd, None, True, out=yo, stream=stream)))
                    hd.free()
                bt = bd.to(tdt)
                t_mio = time_us(lambda: torch.relu_(torch.nn.functional.conv2d(xin, wd, bt, stride=op.stride,
                                                                                padding=op.pad)))
                memo[key] = (t_mfma, t_mio)
            costs[i]["dense_mfma_us"], costs[i]["miopen_us"] = memo[key]
            if names[i] == "fused":            # compared together with the layer that computes it
                j = next((k for k in range(i + 1, len(ops)) if ops[k].kind == "conv" and ops[k].res == op.dst), None)
                if j is not None:
                    pending[j] = memo[key]
                continue
            t_mfma, t_mio = memo[key][0] + pending.get(i, (0.0, 0.0))[0], memo[key][1] + pending.get(i, (0.0, 0.0))[1]
            density = np.count_nonzero(ws[i]) / float(ws[i].size)
            if density <= 0.2001:              # layers pruned to >= 80 % sparsity (up to nnz rounding)
                cnt += 1
                tot["sparse"] += costs[i]["ms"] * 1e3
                tot["mfma"] += t_mfma
                tot["miopen"] += t_mio
                wins += int(costs[i]["ms"] * 1e3 < min(t_mfma, t_mio))
                by_mfma += int(names[i].startswith("dense_mfma"))
        dense_cmp = {"layers_at_80pct_or_more": cnt, "net_faster_than_both_on": wins,
                     "of_which_the_selection_runs_on_matrix_cores": by_mfma,
                     "sum_net_us": tot["sparse"], "sum_own_mfma_dense_us": tot["mfma"],
                     "sum_miopen_dense_us": tot["miopen"],
                     "note": "per-layer times, back-to-back launches; 'net' is the kernel the measured selection runs for "
                             "the pruned layer (a compressed-format kernel, or in 2-byte storage a matrix-core kernel "
                             "over the zero-filled matrix where that is faster); the dense columns run the same layer "
                             "shape unpruned"}

    total_flops = sum(c["flops"] for c in costs)
    total_bytes = sum(c["bytes"] for c in costs)

    # ---- CPU baseline: the oracle as it stands, one full forward pass of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: the first image of the batch through the whole net
        times = []
        for _ in range(5):
            a = time.perf_counter()
            ref, _, _ = oracle.run_net(ops, x[:1].astype(npdt), ws, bs, dtype=npdt)
            times.append((time.perf_counter() - a) * 1e3)
        cpu_ms = float(np.median(times))
        got = y[:1].float().cpu().numpy()
        ref = ref.astype(np.float32)
        err = float(np.abs(got - ref).max() / np.abs(ref).max())
        # ... and once more on an input the net has not seen: after hundreds of passes over one
        # input the workspace holds every intermediate tensor of it, which would hide an op that
        # reads its input before this pass wrote it
        x2 = wl.activation(shape, tag, 99, relu=False).astype(npdt)
        y2 = net.run(torch.from_numpy(x2).cuda(), None, stream)
        torch.cuda.synchronize()
        ref2 = oracle.run_net(ops, x2[:1], ws, bs, dtype=npdt)[0].astype(np.float32)
        err2 = float(np.abs(y2[:1].float().cpu().numpy() - ref2).max() / np.abs(ref2).max())
        cpu = {"value": cpu_ms, "unit": "ms", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "full forward pass of ONE image of the same workload (every conv + pools + FC), "
                         "median of 5 passes",
               "gpu_vs_oracle_max_rel_err": err, "gpu_vs_oracle_max_rel_err_fresh_input": err2}

    if args.layers_out:
        with open(args.layers_out, "w") as f:
            json.dump({"layers": costs, "groups": groups}, f, indent=1)

    line = {
        "metric": "sparse ResNet-50 batch-1 latency" if is_default else "latency of one forward pass",
        "value": ms_per_step,
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": dt,
        "data": "synthetic",
        "config": {"workload": desc, "graph": not args.no_graph, "per_layer_kernel_tuning": tuning},
        "images_per_s": n * 1e3 / ms_per_step,
        "ms_per_step_spread": pass_ms,
        "launches_per_step": int(sum(1 for nm in names if nm not in ("fused", "in place"))),
        "graph_kernel_boundary_us": floor_us,
        "launch_floor_ms": floor_us * 1e-3 * sum(1 for nm in names if nm not in ("fused", "in place")),
        "latency_with_host_sync_ms": lat_sync_ms,
        "latency_cold_caches_ms": lat_cold_ms,
        "measured_copy_rate_gbs": copy_gbs,
        "dense_comparison": dense_cmp,
        "effective_gflops_nonzero_macs": total_flops / (ms_per_step * 1e-3) / 1e9,
        "effective_gbs_algorithmic": total_bytes / (ms_per_step * 1e-3) / 1e9,
        "sum_of_kernel_ms": float(per_op_ms.sum()),
        "sum_of_kernel_ms_warm": float(per_op_ms_warm.sum()),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "paper_context": "26 ms (title) / 21 ms (text) ResNet-50 on a Snapdragon 835 phone; other hardware, not a target",
    }
    print(json.dumps(line))
    net.free()
    return 0


if __name__ == "__main__":
    sys.exit(main())
