"""CPU oracle for Flattened Window Attention -- TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 statement of what the FWA hot path computes, written
from the paper's definitions (Sec. 4.2: Eq. (1) window-based sorting, equal-size
grouping, axis alternation, window shift; Eq. (2) the group attention layer).
It shares no code with the GPU path and must never be imported by it: only the
tests, the smoke check and the benchmark's CPU-baseline leg may call it.

Parity status: every function here is pinned by tests that do not depend on
the oracle itself (brute force on tiny inputs, library special cases, closed
forms, invariants); nothing is "parity unpinned".
"""
from .flatten import (Geometry, shift_amount, window_tuple, pack_key, sort_tuple_order,
                      flatten, frame_segments, Geometry3, window_tuple3, flatten3d)
from .layer import layer_norm, gelu_erf, softmax_rows, group_layer, layer, stack
from .pillars import point_cells, voxelize, bev_scatter

__all__ = ["Geometry", "shift_amount", "window_tuple", "pack_key", "sort_tuple_order",
           "flatten", "frame_segments", "Geometry3", "window_tuple3", "flatten3d", "layer_norm", "gelu_erf", "softmax_rows",
           "group_layer", "layer", "stack", "point_cells", "voxelize", "bev_scatter"]
