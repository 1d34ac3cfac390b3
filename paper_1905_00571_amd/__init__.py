"""Thin Python binding over libcadnn.so (argument marshalling only).

Every function here has the name of the C entry point it forwards to (see
include/cadnn.h); all arithmetic runs in the HIP kernels behind the C ABI.
PyTorch is used only to own device memory and streams.  If the shared library
has not been built the import fails loudly: there is no CPU fallback.
"""
from .binding import (  # noqa: F401
    CadnnError,
    F32,
    F16,
    lib,
    lib_path,
    Weights,
    Net,
    cadnn_pack_weights,
    cadnn_free_weights,
    cadnn_packed_nnz,
    cadnn_packed_export,
    cadnn_unpack_weights,
    cadnn_sparse_conv2d,
    cadnn_conv2d_prepare,
    cadnn_conv2d_variant_name,
    cadnn_conv2d_list_variants,
    cadnn_conv2d_plan_info,
    cadnn_graph_launch_floor,
    cadnn_conv2d_plan_unpack,
    cadnn_conv2d_set_variant,
    cadnn_conv2d_tune,
    cadnn_sparse_fc,
    cadnn_fc_prepare,
    cadnn_depthwise_conv2d,
    cadnn_depthwise_prepare,
    cadnn_device_copy,
    cadnn_maxpool2d,
    cadnn_avgpool2d,
    cadnn_global_avgpool,
    cadnn_dense_conv2d,
    cadnn_run_net,
    cadnn_run_net_noalloc,
    build_net,
    plan_net,
    OpInfo,
)
