"""CPU fp64 oracle of the compressed-activation convolution step.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports it and it
never imports the product package.
"""
from .cac_oracle import (  # noqa: F401
    EDGE_CEIL_VALID,
    EDGE_FLOOR_DROP,
    ConvGeom,
    avgpool,
    bias_grad,
    bn_bwd,
    bn_relu,
    build,
    conv_dw,
    conv_dw_entries,
    conv_dw_from_tile_sums,
    conv_dx,
    conv_dx_entries,
    conv_fwd,
    conv_fwd_entries,
    cosine,
    inflate,
    maxpool,
    num_threads,
    out_shape,
    pooled_shape,
    saved_bytes,
    tile_sums,
)
