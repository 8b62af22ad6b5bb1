"""Seeded synthetic inputs and network descriptions.

This package is the only code shared by the CPU oracle's tests and the HIP
path's tests.  It holds data recipes only: tensor shapes, seeds, value
distributions, layer lists and route tables.  None of the method's arithmetic
(slicing, gating, convolution, normalisation, attention) lives here.
"""
from .nets import (  # noqa: F401
    BASE_SEED,
    mbnet_arch,
    mbnet_pp_arch,
    mbnet_params,
    resnet_arch,
    resnet_params,
    vit_arch,
    vit_params,
    bn_tables,
    seeded_logit_bias,
    images,
)
from .configs import CONFIG1_MIXED_SEEDS, config1, config2  # noqa: F401
