"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

Nothing in this package performs any of the method's arithmetic (no convolution,
no factorisation, no greedy allocation): it only draws random tensors and shape
descriptors, and converts between fp32 and the 16-bit storage encodings.
"""
from .rng import normal, uniform_int, geometric, bits64          # noqa: F401
from .storage import to_storage, from_storage, storage_bytes     # noqa: F401
from .configs import (                                           # noqa: F401
    LayerShape, config1, config2, vgg16_shape, resnet18_shape, resnet50_shape, wrn28_4_shape,
    he_weight, skewed_g, draw_g, pruned_weight,
)
