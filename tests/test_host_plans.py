"""CPU-only checks of the device layouts ("plans") the kernels read: every plan builder runs on
the host through cadnn_conv2d_plan_info (also under the sanitizers, see test_host_sanitizers),
the compact streams cost the bytes per nonzero the storage accounting promises, and the layout
transformation of the wide-tile family loses nothing (its inverse gives the tensor back)."""
import numpy as np
import pytest

import workloads as wl
import paper_1905_00571_amd as cad

# (cin, cout, k, stride, pad, h, w, sparsity, batch)
LAYERS = [
    (64, 64, 3, 1, 1, 56, 56, 0.9, 1),       # configs[0]
    (256, 64, 1, 1, 0, 56, 56, 0.85, 1),     # conv2_x reduce
    (64, 256, 1, 1, 0, 56, 56, 0.85, 2),     # conv2_x expand
    (128, 128, 3, 2, 1, 56, 56, 0.8, 1),     # strided 3x3
    (512, 512, 3, 1, 1, 14, 14, 0.9, 1),     # VGG conv5: many channel chunks
    (1024, 2048, 1, 2, 0, 14, 14, 0.9, 4),   # strided projection
    (24, 40, 5, 1, 2, 17, 17, 0.8, 1),       # a filter size only the LDS families serve on a plain tensor
    (7, 9, 3, 1, 1, 5, 5, 0.5, 3),           # tiny and ragged
]


@pytest.mark.parametrize("layer", LAYERS)
@pytest.mark.parametrize("dtype_name", ["f32", "f16"])
def test_every_plan_builds_on_the_host_and_counts_its_bytes(layer, dtype_name):
    cin, cout, k, stride, pad, h, w_, s, n = layer
    dtype = cad.F16 if dtype_name == "f16" else cad.F32
    w = wl.pruned_weights(cout, cin, k, k, s, "plan-%d-%d-%d" % (cin, cout, k), 0, row_skew=0.5)
    w[cout // 2] = 0.0                                     # an empty row among the others
    hnd = cad.cadnn_pack_weights(w, dtype)
    nnz = cad.cadnn_packed_nnz(hnd)
    names = cad.cadnn_conv2d_list_variants(hnd, n, h, w_, stride, pad)
    assert names
    wide = [nm for nm in names if nm.startswith("swide_")]
    if k in (1, 3) and stride == 1:
        assert wide, names
    for nm in names:
        info = cad.cadnn_conv2d_plan_info(hnd, n, h, w_, stride, pad, nm)
        if nm.startswith("dense"):
            # (the tap-major matrix of the large-tile kernels pads its rows to whole 128-row tiles)
            # (and, for few input channels, its K to whole 32-deep steps)
            large = not nm.endswith("_64x64x32")
            rows = (cout + 127) // 128 * 128 if large else cout
            K = (cin * k * k + 31) // 32 * 32 if large and cin % 32 else cin * k * k
            assert info["stream_bytes"] == rows * K * (2 if dtype == cad.F16 else 4)
            continue
        assert info["entries"] >= nnz and info["stream_bytes"] > 0 and info["chunks"] >= 1, (nm, info)
        per_entry = info["stream_bytes"] / info["entries"]
        if nm.startswith("swide_"):
            # fp32 value + 16-bit tile offset, or fp16 value + 16-bit tile offset
            assert per_entry == (4.0 if dtype == cad.F16 else 6.0), (nm, info)
            assert 0 < info["lds_bytes"] <= 160 * 1024
        else:
            assert per_entry == 8.0, (nm, info)
    # the variant that would be launched, by default
    assert cad.cadnn_conv2d_plan_info(hnd, n, h, w_, stride, pad)["entries"] >= nnz
    with pytest.raises(cad.CadnnError):
        cad.cadnn_conv2d_plan_info(hnd, n, h, w_, stride, pad, "no_such_variant")
    # the wide-tile layout transformation has an inverse, and it returns the packed tensor
    ref = cad.cadnn_unpack_weights(hnd)
    for nm in wide:
        back = cad.cadnn_conv2d_plan_unpack(hnd, n, h, w_, stride, pad, nm)
        assert np.array_equal(back, ref), nm
    other = [nm for nm in names if not nm.startswith("swide_")]
    if other:
        with pytest.raises(cad.CadnnError):
            cad.cadnn_conv2d_plan_unpack(hnd, n, h, w_, stride, pad, other[0])
    hnd.free()


def test_compact_stream_bytes_per_nonzero_on_the_benchmark_layers():
    """Section 3 of the paper counts storage without indices; with them the compact stream is
    6 bytes per nonzero in fp32 storage and 4 in fp16, padding of the parts included up to a
    few percent on the weight-bound layers (stage-5 3x3 of ResNet-50, VGG-16's conv5)."""
    for cin, cout, k, hw, s in [(512, 512, 3, 7, 0.8), (512, 512, 3, 14, 0.9), (2048, 512, 1, 7, 0.9)]:
        w = wl.pruned_weights(cout, cin, k, k, s, "bpn-%d-%d" % (cin, k), 0)
        for dtype, bar in ((cad.F32, 6.0), (cad.F16, 4.0)):
            hnd = cad.cadnn_pack_weights(w, dtype)
            # batch 8: the 7 x 7 images then fill the tiles of the flattened-pixel variants
            names = [nm for nm in cad.cadnn_conv2d_list_variants(hnd, 8, hw, hw, 1, k // 2) if nm.startswith("swide_")]
            assert names
            best = min(cad.cadnn_conv2d_plan_info(hnd, 8, hw, hw, 1, k // 2, nm)["bytes_per_nonzero"] for nm in names)
            assert bar <= best <= bar * 1.25, (cin, k, dtype, best)
            linear = [nm for nm in cad.cadnn_conv2d_list_variants(hnd, 8, hw, hw, 1, k // 2) if nm.startswith(("slinear_", "sdirect_"))]
            if linear:
                assert cad.cadnn_conv2d_plan_info(hnd, 8, hw, hw, 1, k // 2, linear[0])["bytes_per_nonzero"] >= 8.0
            hnd.free()
