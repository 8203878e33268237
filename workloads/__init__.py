"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package only draws random tensors and describes their shapes.  It holds
none of the arithmetic of the operators under test: no convolution, pooling,
normalisation or folding lives here.  Both the oracle and the HIP library take
what this module produces as plain inputs.
"""
from .resnet18 import (  # noqa: F401
    ENTROPY, BN_EPS, CONV_SPECS, STAGE_IO, NUM_CLASSES, FC_IN,
    rng_for, make_input, make_conv_weight, make_bn, make_resnet18_params,
    round_to_bf16, bf16_bits, bf16_from_bits, conv_out_hw, SWEEP_OPS,
)
