"""Seeded synthetic workloads (tensors and layer tables) shared by the tests,
the oracle-side harness and the HIP-side harness.

Nothing in this package performs any of the method's arithmetic: it only draws
random tensors, prunes them to a requested sparsity (input preparation that the
paper does offline, Section 3) and lists layer shapes.
"""
from .gen import (  # noqa: F401
    MASTER_SEED,
    rng_for,
    activation,
    bias_vector,
    pruned_weights,
    keep_count,
    conv_out_size,
    embed_filter,
)
from .nets import (  # noqa: F401
    Op,
    resnet50_ops,
    vgg16_ops,
    mobilenet_v1_ops,
    mobilenet_v2_ops,
    factorized_7x7_branch_ops,
    inception_v3_ops,
    bottleneck_conv2x_ops,
    single_conv_ops,
    net_tensors,
    buffer_shapes,
)
