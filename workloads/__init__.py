"""Seeded synthetic inputs and layer tables for the ternary pointwise-conv path.

This package holds no arithmetic of the method itself: it only draws the
random tensors (activations, ternary weights, bias, requantisation
parameters, residuals) and enumerates layer shapes.  Both the CPU oracle's
tests and the HIP path's tests/bench take their inputs from here.
"""
from .generators import (  # noqa: F401
    SplitMix64, PwLayerInputs, DwLayerInputs, BlockInputs,
    make_pw_layer, make_dw_layer, make_block, make_gconv_layer, GconvLayerInputs, float_conv_weights, prelu_mult_neg, CONFIG_SEED_BASE,
)
from .mobilenetv2 import (  # noqa: F401
    PwShape, DwShape, BlockShape, mobilenetv2_pointwise_layers, mobilenetv2_depthwise_layers,
    mobilenetv2_blocks,
    mobilenetv2_param_counts, BASELINE_CONFIGS,
)
from .grouped import (  # noqa: F401,E402
    GconvShape, regnetx_400mf_grouped_layers, resnext50_32x4d_grouped_layers,
    regnetx_400mf_pointwise_layers, resnext50_32x4d_pointwise_layers,
)
