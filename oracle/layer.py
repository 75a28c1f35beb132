"""Oracle for the group attention layer (paper Sec. 4.2.2, Eq. (2)).

TEST INFRASTRUCTURE ONLY -- see the package docstring.

    F'  = F  + MHSA(LN(F))          standard softmax multi-head self-attention
    F'' = F' + FFN(LN(F'))          FFN = Linear -> GELU -> Linear

computed independently inside each group of the flattened order, in float64,
with scores and probabilities materialised (no tiling, no masking, no padding:
a short tail group simply attends over its real members).

Eq. (2) hands the attention a second argument, PE(C), which the paper calls a
global absolute positional embedding and gives no formula for.  Here it is an
optional per-pillar array of the features' shape, computed by the caller, and it
enters the way the detection transformers this design follows use it: queries
and keys are projected from LN(F) + PE, values from LN(F) alone.

Linear layers follow y = x @ W.T + b with W stored [out, in].
"""
import numpy as np
from scipy.special import erf as _erf


def layer_norm(x, gamma, beta, eps):
    """Per-row normalisation with biased variance, then affine."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma + beta


def gelu_erf(x):
    """Exact GELU: x * Phi(x)."""
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def softmax_rows(s):
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def _f64(p, name):
    return np.asarray(p[name], dtype=np.float64)


def group_layer(X, p, pe=None):
    """One transformer layer on the m x C features of ONE group; pe: None or the
    m x C positional embedding of the group's members (added to the inputs of
    the query and key projections only)."""
    X = np.asarray(X, dtype=np.float64)
    m, C = X.shape
    heads = int(p["heads"])
    d = C // heads
    eps = float(p["ln_eps"])
    U = layer_norm(X, _f64(p, "ln1_g"), _f64(p, "ln1_b"), eps)
    Uqk = U if pe is None else U + np.asarray(pe, dtype=np.float64)
    W, b = _f64(p, "w_qkv"), _f64(p, "b_qkv")
    Q = Uqk @ W[:C].T + b[:C]
    K = Uqk @ W[C:2 * C].T + b[C:2 * C]
    V = U @ W[2 * C:].T + b[2 * C:]
    O = np.empty((m, C), dtype=np.float64)
    for h in range(heads):
        sl = slice(h * d, (h + 1) * d)
        S = (Q[:, sl] @ K[:, sl].T) / np.sqrt(float(d))
        P = softmax_rows(S)
        O[:, sl] = P @ V[:, sl]
    X1 = X + O @ _f64(p, "w_o").T + _f64(p, "b_o")
    H = gelu_erf(layer_norm(X1, _f64(p, "ln2_g"), _f64(p, "ln2_b"), eps)
                 @ _f64(p, "w1").T + _f64(p, "b1"))
    return X1 + H @ _f64(p, "w2").T + _f64(p, "b2")


def layer(feats, perm, group_offsets, p, groups=None, dropped_passthrough=True, group_size=None,
          pos_embed=None):
    """Gather each group's rows, apply `group_layer`, scatter back.

    feats [n, C] in pillar order; perm / group_offsets from `flatten`.  With
    `groups` (an iterable of group indices) only those groups are computed; all
    other rows of the result are NaN.  Rows that belong to no group (dropped
    tails) pass through unchanged when every group is computed.
    With `group_size` given, `group_offsets` is the list of group starts that
    `flatten(..., tail="drop")` returns ('Drop Residual', Sec. 4.3): no closing
    entry, every group has exactly `group_size` members.
    `pos_embed`, if given, is [n, C] in pillar order like feats (see `group_layer`).
    Returns float64 [n, C].
    """
    feats = np.asarray(feats, dtype=np.float64)
    n = feats.shape[0]
    perm = np.asarray(perm)
    off = np.asarray(group_offsets)
    if group_size is None:
        num_groups = len(off) - 1
        ends = off[1:]
    else:
        num_groups = len(off)
        ends = off + int(group_size)
    if groups is None:
        out = feats.copy() if dropped_passthrough else np.full_like(feats, np.nan)
        groups = range(num_groups)
    else:
        out = np.full_like(feats, np.nan)
    for g in groups:
        rows = perm[int(off[g]):int(ends[g])]
        out[rows] = group_layer(feats[rows], p, None if pos_embed is None else np.asarray(pos_embed)[rows])
    return out


def stack(feats, perms, offsets, layer_params, schedule, between=None, pos_embed=None):
    """Layers applied in order; layer l uses the cached flatten of its
    (axis, shift) pair ('Reuse Sorting').  perms / offsets: dicts keyed by
    (axis, shift).  `between`, if given, is applied to the features after each
    layer (e.g. the storage rounding of a bf16 buffer).  `pos_embed` [n, C], if
    given, is handed to every layer.  Returns the list of all intermediate
    feature arrays, input first."""
    cur = np.asarray(feats, dtype=np.float64)
    trace = [cur]
    for p, key in zip(layer_params, schedule):
        cur = layer(cur, perms[key], offsets[key], p, pos_embed=pos_embed)
        if between is not None:
            cur = np.asarray(between(cur), dtype=np.float64)
        trace.append(cur)
    return trace
