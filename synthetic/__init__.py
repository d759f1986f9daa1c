"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package only *generates inputs* (block lists, dense weights, activations, and
the 16-bit encodings of them).  It contains none of the method's arithmetic: no
packing, no rotation, no product.  Neither the oracle nor the HIP library imports it;
the tests and the benchmark feed its outputs to both sides.
"""
from .configs import (CONFIGS, EXTRA_CONFIGS, LayerConfig, aligned_twin,   # noqa: F401
                      get_config)
from .masks import select_blocks, target_block_count           # noqa: F401
from .tensors import (make_weights, make_activations, encode,  # noqa: F401
                      decode_f64, make_layer)
