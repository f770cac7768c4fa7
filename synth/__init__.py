"""Seeded synthetic inputs for the DSVT hot path.

This package only draws numbers: voxel coordinates, features and weights, all
from counter-based Philox streams with fixed seeds.  It holds none of the
method's arithmetic (no window ids, no set maps, no attention), so the CPU
oracle and the HIP path can both be fed from it without sharing any logic.
"""
from .frames import (CONFIGS, make_frame, make_features, round_bf16,  # noqa: F401
                     bf16_bits, frame_uniform, frame_radial, frame_skewed, make_points)
from .weights import make_layer_weights, make_pool_weights, make_vfe_weights, rel_table_size  # noqa: F401
