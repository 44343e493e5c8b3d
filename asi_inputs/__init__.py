"""Seeded synthetic inputs for the ASI hot path.

This package only *makes inputs*: layer tables, random tensors with a chosen
spectrum, rounding to the storage dtype.  It holds none of the method's steps
(no subspace iteration, no projection, no weight gradient) and is the one
module both the CPU oracle's tests and the GPU harness may import.
"""
from .configs import CONFIGS, Layer, layers_of  # noqa: F401
from .synth import (  # noqa: F401
    LayerStream,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_seed,
    random_orthonormal,
    tucker_tensor,
)
