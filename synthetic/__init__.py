"""Seeded synthetic inputs and layer-shape tables.

This package holds no arithmetic of the block-sparse method itself: it only
draws random tensors and masks and lists layer shapes.  It is the one module
both the CPU oracle's tests and the HIP path's tests/bench may import.
"""
from .gen import (  # noqa: F401
    LayerCase,
    bf16_grid,
    draw_layer,
    draw_mask,
    seed_for,
)
from .layers import (  # noqa: F401
    ConvSpec,
    config_cases,
    inception_v3_layers,
    resnet50_layers,
    vgg16_layers,
)
