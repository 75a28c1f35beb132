"""Seeded synthetic inputs for Flattened Window Attention (FWA).

This module only draws random numbers and shapes them into the inputs the
method consumes (integer BEV coordinates, feature rows, layer parameters).
It contains none of the method's arithmetic: no window keys, no sorting, no
attention.  Both the CPU oracle's tests and the GPU path's tests feed on it,
and neither of those two imports the other.
"""
from .bf16 import bf16_round, f16_round, f32_to_bf16_bits, bf16_bits_to_f32
from .frames import (unique_uniform_cells, lidar_frame, merged_sweep,
                     frame_batch, row_major_order, lidar_points)
from .weights import layer_params, stack_params, PARAM_NAMES
from .configs import CONFIGS, make_config, layer_schedule

__all__ = [
    "bf16_round", "f16_round", "f32_to_bf16_bits", "bf16_bits_to_f32",
    "unique_uniform_cells", "lidar_frame", "merged_sweep", "frame_batch",
    "row_major_order", "lidar_points", "layer_params", "stack_params", "PARAM_NAMES",
    "CONFIGS", "make_config", "layer_schedule",
]
