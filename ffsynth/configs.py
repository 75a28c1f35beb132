"""The five benchmark configurations, as seeded recipes.

`make_config(i)` returns a dict with: coords int32 [n,3] (b,x,y), feats float32
[n,C] (bf16-representable when dtype == "bf16"), layers (list of parameter
dicts), geometry and the layer schedule.  Layer l sorts along axis l % 2
(0 = x-major, 1 = y-major) with the half-window shift on when (l // 2) % 2 == 1,
i.e. x, y, shifted-x, shifted-y, x, y, ...
"""
import numpy as np
from .bf16 import bf16_round
from .frames import unique_uniform_cells, lidar_frame, merged_sweep, frame_batch, GRID
from .weights import stack_params

CONFIGS = {
    1: dict(name="tiny", n=2000, grid=64, B=1, window=8, G=32, C=64, heads=4, F=128,
            layers=2, dtype="f32"),
    2: dict(name="waymo_frame", n=30000, grid=GRID, B=1, window=13, G=64, C=128, heads=8,
            F=256, layers=4, dtype="bf16"),
    3: dict(name="full_backbone", n=30000, grid=GRID, B=1, window=13, G=64, C=128, heads=8,
            F=256, layers=8, dtype="bf16"),
    4: dict(name="sweep3", n=80000, grid=GRID, B=1, window=13, G=128, C=128, heads=8,
            F=256, layers=8, dtype="bf16", per_frame=46000),
    5: dict(name="batch8", n=240000, grid=GRID, B=8, window=9, G=69, C=256, heads=8,
            F=512, layers=8, dtype="bf16",
            targets=(20000, 23000, 26000, 29000, 31000, 34000, 37000, 40000)),
}


def layer_schedule(num_layers):
    """[(axis, shift)] for layers 0..num_layers-1."""
    return [(l % 2, (l // 2) % 2) for l in range(num_layers)]


def _coords(i, c):
    if i == 1:
        return unique_uniform_cells(c["n"], c["grid"], seed=0)
    if i in (2, 3):
        return lidar_frame(seed=0, target=c["n"])
    if i == 4:
        return merged_sweep((0, 1, 2), (0.0, 0.5, 1.0), c["per_frame"], c["n"])
    if i == 5:
        return frame_batch(range(8), c["targets"], shuffle_seed=99)
    raise KeyError(i)


def make_config(i, num_layers=None, with_feats=True):
    c = dict(CONFIGS[i])
    L = c["layers"] if num_layers is None else num_layers
    coords = _coords(i, c)
    out = dict(c)
    out["id"] = i
    out["coords"] = coords
    out["n"] = int(coords.shape[0])
    out["schedule"] = layer_schedule(L)
    bf16 = c["dtype"] == "bf16"
    if with_feats:
        rng = np.random.default_rng(7 + i)
        feats = rng.standard_normal((out["n"], c["C"]), dtype=np.float32)
        out["feats"] = bf16_round(feats) if bf16 else feats
        out["layer_params"] = stack_params(c["C"], c["F"], c["heads"], L, bf16=bf16)
    return out
