"""Seeded parameters of one FWA transformer layer.

Layout follows the usual linear-layer convention y = x @ W.T + b with W stored
[out_features, in_features] row-major:
  w_qkv [3C, C] rows 0..C-1 = query, C..2C-1 = key, 2C..3C-1 = value projection;
        head h uses rows h*d..(h+1)*d-1 of each third;
  w_o [C, C]; w1 [F, C]; w2 [C, F].
Xavier-uniform per logical matrix (W_q, W_k, W_v each C x C).  Biases and the
LayerNorm affine parameters are drawn non-trivial on purpose so that a dropped
term shows up in a comparison.
"""
import numpy as np
from .bf16 import bf16_round

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


def _xavier(rng, out_f, in_f):
    a = np.sqrt(6.0 / (in_f + out_f))
    return rng.uniform(-a, a, size=(out_f, in_f)).astype(np.float32)


def layer_params(C, F, heads, seed, bf16=False, ln_eps=1e-5):
    rng = np.random.default_rng(seed)
    p = {}
    p["ln1_g"] = rng.uniform(0.9, 1.1, size=C).astype(np.float32)
    p["ln1_b"] = rng.uniform(-0.1, 0.1, size=C).astype(np.float32)
    p["w_qkv"] = np.concatenate([_xavier(rng, C, C) for _ in range(3)], axis=0)
    p["b_qkv"] = rng.uniform(-0.1, 0.1, size=3 * C).astype(np.float32)
    p["w_o"] = _xavier(rng, C, C)
    p["b_o"] = rng.uniform(-0.1, 0.1, size=C).astype(np.float32)
    p["ln2_g"] = rng.uniform(0.9, 1.1, size=C).astype(np.float32)
    p["ln2_b"] = rng.uniform(-0.1, 0.1, size=C).astype(np.float32)
    p["w1"] = _xavier(rng, F, C)
    p["b1"] = rng.uniform(-0.1, 0.1, size=F).astype(np.float32)
    p["w2"] = _xavier(rng, C, F)
    p["b2"] = rng.uniform(-0.1, 0.1, size=C).astype(np.float32)
    if bf16:
        for k in PARAM_NAMES:
            p[k] = bf16_round(p[k])
    p["C"], p["F"], p["heads"], p["ln_eps"] = int(C), int(F), int(heads), float(ln_eps)
    return p


def stack_params(C, F, heads, num_layers, bf16=False, base_seed=1000):
    """Layer l uses seed base_seed + l."""
    return [layer_params(C, F, heads, base_seed + l, bf16=bf16) for l in range(num_layers)]
