"""Seeded synthetic inputs (slides, weights, labels) shared by the CPU oracle and the HIP path.

This package holds shapes, names and random-number recipes only: none of the
method's arithmetic (no encoder, pool, loss or gradient code) lives here.
"""
from .slide_inputs import (  # noqa: F401
    SlideConfig, CONFIGS, SEEDS, param_shapes, make_params, make_pixels,
    make_label, make_features, to_bf16_grid,
)
from .resnet_inputs import (  # noqa: F401
    ResNetConfig, RESNET_CONFIGS, RESNET_SEEDS, resnet_blocks, resnet_param_shapes, make_resnet_params,
)
