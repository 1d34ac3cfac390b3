"""CPU-only checks of the product library: it loads, exports every declared symbol, and its
host-side packer agrees with the oracle's reference packer bit for bit."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import workloads as wl
import paper_1905_00571_amd as cad
from paper_1905_00571_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cadnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cadnn_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = cad.lib()
    names = declared_symbols()
    assert len(names) >= 20
    raw = ctypes.CDLL(cad.lib_path())
    for n in names:
        assert hasattr(raw, n), f"{n} declared in cadnn.h but not exported"
    assert L.cadnn_last_error() is not None


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1905_00571_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src, f
                assert "cadnn_oracle" not in src, f


def cmp_pack(w, dtype_flag, np_dtype):
    ref = oracle.pack(w, np_dtype)
    h = cad.cadnn_pack_weights(w, dtype_flag)
    got = cad.cadnn_packed_export(h)
    assert cad.cadnn_packed_nnz(h) == int(ref["row_ptr"][-1])
    for k in ("perm", "row_ptr", "col_idx"):
        assert got[k].dtype == ref[k].dtype and got[k].tobytes() == ref[k].tobytes(), k
    assert got["vals"].tobytes() == ref["vals"].tobytes()
    un = cad.cadnn_unpack_weights(h)
    ref_un = oracle.unpack(ref).astype(np.float32)
    assert un.tobytes() == ref_un.tobytes()
    h.free()
    return ref


@pytest.mark.parametrize("shape,s", [((64, 64, 3, 3), 0.9), ((256, 64, 1, 1), 0.85),
                                     ((64, 3, 7, 7), 0.0), ((1000, 2048, 1, 1), 0.9),
                                     ((7, 5, 3, 3), 1.0), ((9, 4, 1, 7), 0.5)])
def test_pack_matches_oracle_bit_exact_fp32(shape, s):
    w = wl.pruned_weights(*shape, s, "packtest", 1)
    ref = cmp_pack(w, cad.F32, np.float32)
    assert np.array_equal(oracle.unpack(ref), w)


def test_pack_skewed_rows_empty_rows_dense_rows():
    w = wl.pruned_weights(32, 16, 3, 3, 0.9, "packtest", 2, row_skew=1.5)
    w[3] = 0
    w[7] = np.float32(0.25)
    cmp_pack(w, cad.F32, np.float32)


def test_pack_special_values():
    w = np.zeros((3, 4, 1, 1), np.float32)
    w[0, 0] = -0.0
    w[0, 1] = np.float32(1e-42)
    w[1, 2] = np.inf
    w[2, 3] = np.float32(-3.5)
    w[2, 0] = np.float32(65520.0)     # rounds to fp16 inf
    cmp_pack(w, cad.F32, np.float32)
    cmp_pack(w, cad.F16, np.float16)


def test_pack_fp16_rounding_matches_numpy():
    g = np.random.default_rng(5)
    vals = np.concatenate([
        g.standard_normal(20000).astype(np.float32) * np.float32(0.05),
        (g.standard_normal(5000) * 1e-6).astype(np.float32),        # fp16 subnormals
        (g.standard_normal(2000) * 1e-8).astype(np.float32),        # round to zero / smallest
        np.array([6.1035e-05, 6.0976e-05, 5.96e-08, 2.98e-08, 2.9802322e-08, 8.9e-08, 65504.0,
                  65519.9, 1.0009765625, 1.00048828125, 1.0014648, 0.33325195], np.float32),
    ])
    w = vals.reshape(1, -1, 1, 1).copy()
    w[w == 0] = 1.0
    cmp_pack(np.ascontiguousarray(w), cad.F16, np.float16)


def test_pack_errors():
    L = cad.lib()
    out = ctypes.c_void_p()
    w = np.ones(4, np.float32)
    p = w.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
    assert L.cadnn_pack_weights(None, 1, 1, 2, 2, 0, ctypes.byref(out)) == 1
    assert b"NULL" in L.cadnn_last_error()
    assert L.cadnn_pack_weights(p, 0, 1, 2, 2, 0, ctypes.byref(out)) == 1
    assert L.cadnn_pack_weights(p, 1, 1, 2, -2, 0, ctypes.byref(out)) == 1
    assert L.cadnn_pack_weights(p, 1, 1, 2, 2, 7, ctypes.byref(out)) == 1
    assert out.value is None
    assert L.cadnn_packed_nnz(None, None) == 1
    assert L.cadnn_free_weights(None) == 0
    assert L.cadnn_net_free(None) == 0
    assert L.cadnn_unpack_weights(None, None) == 1


def test_layer_argument_checks_without_a_gpu():
    """Argument errors are reported before anything touches the device."""
    L = cad.lib()
    h = cad.cadnn_pack_weights(wl.pruned_weights(8, 4, 3, 3, 0.5, "packtest", 3))
    assert L.cadnn_sparse_conv2d(None, None, None, 1, 8, 8, 1, 1, None, None, 0, None) == 1
    assert L.cadnn_sparse_conv2d(h.handle, None, None, 1, 8, 8, 0, 1, None, None, 0, None) == 1
    assert L.cadnn_sparse_conv2d(h.handle, None, None, 1, 2, 2, 1, 0, None, None, 0, None) == 1   # empty output
    h5 = cad.cadnn_pack_weights(wl.pruned_weights(8, 4, 5, 5, 0.9, "packtest", 4))
    assert cad.cadnn_conv2d_list_variants(h5, 1, 8, 8, 1, 2)                                         # 5x5: LDS-staged or dense kernels
    buf = ctypes.create_string_buffer(4096)
    assert L.cadnn_conv2d_list_variants(h.handle, 1, 8, 8, 1, 1, buf, 4096) == 0
    names = buf.value.decode().split("\n")
    assert len(names) >= 4 and all("float" in n for n in names) and any("3x3" in n for n in names)
    assert L.cadnn_conv2d_set_variant(h.handle, 1, 8, 8, 1, 1, b"no-such-kernel") == 1
    assert L.cadnn_conv2d_set_variant(h.handle, 1, 8, 8, 1, 1, names[-1].encode()) == 0
    assert L.cadnn_conv2d_variant_name(h.handle, 1, 8, 8, 1, 1, buf, 4096) == 0
    assert buf.value.decode() == names[-1]
    assert L.cadnn_conv2d_set_variant(h.handle, 1, 8, 8, 1, 1, None) == 0
    h5.free()
    assert L.cadnn_sparse_fc(h.handle, 1, 1, 1, None, 0, None) == 1                                # 3x3 handle in fc
    assert L.cadnn_maxpool2d(None, None, 1, 1, 4, 4, 2, 2, 0, 0, None) == 1
    net = ctypes.c_void_p()
    assert L.cadnn_net_create(0, 1, 4, 8, 8, ctypes.byref(net)) == 0
    assert L.cadnn_net_add_maxpool(net, 2, 2, 0, 3, 1) == 1          # reads an unwritten buffer
    assert L.cadnn_net_add_maxpool(net, 2, 2, 0, 0, 0) == 1          # dst aliases src
    assert L.cadnn_net_add_maxpool(net, 2, 2, 0, 0, 1) == 0
    assert L.cadnn_run_net(net, 1, 1, None) == 1                      # not finalized
    n = ctypes.c_int()
    assert L.cadnn_net_num_ops(net, ctypes.byref(n)) == 0 and n.value == 1
    assert L.cadnn_net_free(net) == 0
    h.free()


def test_depthwise_argument_checks_without_a_gpu():
    L = cad.lib()
    dw = cad.cadnn_pack_weights(wl.pruned_weights(4, 1, 3, 3, 0.0, "packtest", 5))
    full = cad.cadnn_pack_weights(wl.pruned_weights(4, 4, 3, 3, 0.5, "packtest", 6))
    assert L.cadnn_depthwise_conv2d(None, 1, 1, 1, 8, 8, 1, 1, None, 0, None) == 1
    assert L.cadnn_depthwise_conv2d(dw.handle, None, None, 1, 8, 8, 1, 1, None, 0, None) == 1      # NULL tensors
    assert L.cadnn_depthwise_conv2d(full.handle, 1, 1, 1, 8, 8, 1, 1, None, 0, None) == 1          # cin != 1
    assert b"depthwise" in L.cadnn_last_error()
    assert L.cadnn_depthwise_conv2d(dw.handle, 1, 1, 1, 2, 2, 1, 0, None, 0, None) == 1            # empty output
    assert L.cadnn_depthwise_conv2d(dw.handle, 1, 1, 1, 8, 8, 0, 1, None, 0, None) == 1            # stride 0
    assert L.cadnn_depthwise_prepare(full.handle) == 1
    net = ctypes.c_void_p()
    assert L.cadnn_net_create(0, 1, 4, 8, 8, ctypes.byref(net)) == 0
    assert L.cadnn_net_add_depthwise(net, full.handle, None, 1, 1, 1, 0, 1) == 1     # not a depthwise bank
    assert L.cadnn_net_add_depthwise(net, dw.handle, None, 1, 1, 1, 0, 0) == 1       # dst aliases src
    assert L.cadnn_net_add_depthwise(net, dw.handle, None, 1, 1, 1, 0, 1) == 0
    dw8 = cad.cadnn_pack_weights(wl.pruned_weights(8, 1, 3, 3, 0.0, "packtest", 7))
    assert L.cadnn_net_add_depthwise(net, dw8.handle, None, 1, 1, 1, 1, 2) == 1      # 8 filters on 4 channels
    assert L.cadnn_net_add_depthwise(net, dw.handle, None, 2, 1, 1, 1, 2) == 0
    nbytes = ctypes.c_size_t()
    assert L.cadnn_net_workspace_bytes(net, ctypes.byref(nbytes)) == 0
    assert nbytes.value >= 4 * 10 * 10 * 4           # first output: 4 planes of 8x8 inside a 1-pixel zero halo
    assert L.cadnn_net_free(net) == 0
    for h in (dw, full, dw8):
        h.free()


def test_sizes_beyond_32_bit_offsets_are_refused_on_the_host():
    """Tensors whose channel plane or image does not fit the kernels' 32-bit offsets, and
    paddings that would overflow the size arithmetic, are refused (CADNN_EUNSUPPORTED = 2, or
    EINVAL = 1 for an empty output) before anything touches a device."""
    L = cad.lib()
    h = cad.cadnn_pack_weights(wl.pruned_weights(4, 2, 3, 3, 0.5, "big", 1))
    one = ctypes.c_void_p(16)          # never dereferenced: the checks come first
    big = 1 << 16
    assert L.cadnn_sparse_conv2d(h.handle, one, one, 1, big, big, 1, 1, None, None, 0, None) == 2
    assert L.cadnn_sparse_conv2d(h.handle, one, one, 1, 8, 8, 1, 1 << 30, None, None, 0, None) == 2
    assert L.cadnn_conv2d_prepare(h.handle, 1, 40000, 40000, 1, 1) == 2
    assert L.cadnn_conv2d_prepare(h.handle, 1, 20000, 20000, 1, 1) == 2          # 2 x 4e8 x 4 bytes: above 2 GiB
    assert L.cadnn_maxpool2d(one, one, 1, 1, big, big, 2, 2, 0, 0, None) == 2
    assert L.cadnn_avgpool2d(one, one, 1, 1, big, big, 3, 1, 1, 0, None) == 2
    assert L.cadnn_global_avgpool(one, one, 1, 1, big, big, 0, None) == 2
    assert L.cadnn_dense_conv2d(one, one, ctypes.c_void_p(32), 1, 2, big, big, 4, 3, 3, 1, 1, None, None, 0, 0, None) == 2
    dw = cad.cadnn_pack_weights(wl.pruned_weights(2, 1, 3, 3, 0.0, "big", 2))
    assert L.cadnn_depthwise_conv2d(dw.handle, one, one, 1, big, big, 1, 1, None, 0, None) == 2
    net = ctypes.c_void_p()
    assert L.cadnn_net_create(0, 1, 64, 4096, 4096, ctypes.byref(net)) == 2 and not net.value
    assert L.cadnn_net_create(0, 1, 2, 4096, 4096, ctypes.byref(net)) == 0
    assert L.cadnn_net_add_conv(net, h.handle, None, 1, 70000, 1, 0, 1, -1) == 2       # halo beyond the limit
    assert L.cadnn_net_add_conv(net, h.handle, None, 1, 8000, 1, 0, 1, -1) == 2        # padded image above the limit
    assert L.cadnn_net_add_conv(net, h.handle, None, 1, 1, 1, 0, 1, -1) == 0
    wide = cad.cadnn_pack_weights(wl.pruned_weights(64, 4, 1, 1, 0.5, "big", 3))
    assert L.cadnn_net_add_conv(net, wide.handle, None, 1, 0, 1, 1, 2, -1) == 2        # 64 x 4096 x 4096 x 4 bytes
    assert b"GiB" in L.cadnn_last_error()
    assert L.cadnn_net_free(net) == 0
    for x in (h, dw, wide):
        x.free()


def test_listed_variants_can_all_serve_the_layer():
    """Listing and pinning variants is host work.  A variant of the wave-sliced LDS family
    buffers the nonzeros of a (row group, channel chunk): it is listed only for weights whose
    longest such stream fits its buffer, so a dense 3x3 bank loses the 16-row x 8-channel one
    that an 80 % sparse bank keeps; every geometry has some variant (5x5 and stride-3 7x7
    filters on a plain tensor included) and every listed name can be pinned."""
    counts = {}
    for s in (0.0, 0.8, 1.0):
        h = cad.cadnn_pack_weights(wl.pruned_weights(75, 332, 3, 3, s, "variants", 1))
        names = cad.cadnn_conv2d_list_variants(h, 2, 34, 11, 1, 1)
        counts[s] = {nm for nm in names if nm.startswith("stile")}
        for nm in names:
            cad.cadnn_conv2d_set_variant(h, 2, 34, 11, 1, 1, nm)
        assert cad.cadnn_conv2d_variant_name(h, 2, 34, 11, 1, 1) == names[-1]
        cad.cadnn_conv2d_set_variant(h, 2, 34, 11, 1, 1, None)
        assert cad.cadnn_conv2d_variant_name(h, 2, 34, 11, 1, 1) in names     # the untuned pick
        h.free()
    assert counts[0.8] == counts[1.0] and counts[0.0] < counts[0.8]
    assert any("g16c8" in nm for nm in counts[0.8]) and not any("g16c8" in nm for nm in counts[0.0])
    for (cin, cout, k, stride, pad, hh, ww, s) in [(12, 9, 5, 1, 2, 19, 23, 0.8), (5, 11, 7, 3, 3, 19, 9, 0.9),
                                                  (6, 4, 2, 1, 1, 9, 8, 0.85), (300, 8, 5, 2, 2, 40, 40, 0.9)]:
        h = cad.cadnn_pack_weights(wl.pruned_weights(cout, cin, k, k, s, "variants", 2))
        names = cad.cadnn_conv2d_list_variants(h, 1, hh, ww, stride, pad)
        assert names, (cin, cout, k, stride)
        assert cad.cadnn_conv2d_variant_name(h, 1, hh, ww, stride, pad) in names
        h.free()


def test_binding_exposes_the_c_names():
    for n in declared_symbols():
        if n.startswith("cadnn_net_") or n in ("cadnn_last_error",):
            continue
        assert hasattr(cad, n) or hasattr(binding, n), n
