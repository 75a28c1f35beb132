"""Pins for the layer oracle: a hand-worked case, the textbook pre-LN encoder
layer of a library (float64, CPU), closed forms and invariances."""
import math
import os

import numpy as np
import pytest
import torch

import ffsynth
import oracle
from oracle import Geometry

GOLD = os.path.join(os.path.dirname(__file__), "golden", "eq2_hand_worked.txt")


def _params(C=32, F=48, heads=4, seed=0):
    return ffsynth.layer_params(C, F, heads, seed)


def test_hand_worked_two_tokens():
    vals = {}
    with open(GOLD) as f:
        for line in f:
            if line[0] in "XOT":
                k, *v = line.split()
                vals[k] = list(map(float, v))
    X = np.array(vals["X"]).reshape(2, 2)
    rng = np.random.default_rng(0)
    I = np.eye(2)
    p = dict(C=2, F=3, heads=1, ln_eps=1e-5,
             ln1_g=np.ones(2), ln1_b=np.zeros(2),
             w_qkv=np.concatenate([rng.normal(size=(2, 2)), rng.normal(size=(2, 2)), I]),
             b_qkv=np.zeros(6), w_o=I, b_o=np.zeros(2),
             ln2_g=rng.normal(size=2), ln2_b=rng.normal(size=2),
             w1=rng.normal(size=(3, 2)), b1=rng.normal(size=3),
             w2=np.zeros((2, 3)), b2=np.array([0.5, 0.25]))
    out = oracle.group_layer(X, p)
    assert np.abs(out.reshape(-1) - np.array(vals["OUT"])).max() <= vals["TOL"][0]


def _torch_encoder_layer(p):
    C, F, heads = p["C"], p["F"], p["heads"]
    m = torch.nn.TransformerEncoderLayer(C, heads, dim_feedforward=F, dropout=0.0,
                                         activation="gelu", batch_first=True,
                                         norm_first=True, dtype=torch.float64)
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        m.self_attn.in_proj_weight.copy_(t(p["w_qkv"]))
        m.self_attn.in_proj_bias.copy_(t(p["b_qkv"]))
        m.self_attn.out_proj.weight.copy_(t(p["w_o"]))
        m.self_attn.out_proj.bias.copy_(t(p["b_o"]))
        m.linear1.weight.copy_(t(p["w1"])); m.linear1.bias.copy_(t(p["b1"]))
        m.linear2.weight.copy_(t(p["w2"])); m.linear2.bias.copy_(t(p["b2"]))
        m.norm1.weight.copy_(t(p["ln1_g"])); m.norm1.bias.copy_(t(p["ln1_b"]))
        m.norm2.weight.copy_(t(p["ln2_g"])); m.norm2.bias.copy_(t(p["ln2_b"]))
    m.norm1.eps = m.norm2.eps = p["ln_eps"]
    m.train()          # training mode with dropout 0: takes the plain (unfused) code path
    return m


@pytest.mark.parametrize("C,F,heads,m", [(32, 48, 4, 11), (64, 128, 4, 32), (128, 256, 8, 64)])
def test_against_library_pre_ln_encoder_layer(C, F, heads, m):
    p = ffsynth.layer_params(C, F, heads, seed=5)
    X = np.random.default_rng(1).standard_normal((m, C))
    with torch.no_grad():
        want = _torch_encoder_layer(p)(torch.tensor(X)[None])[0].numpy()
    got = oracle.group_layer(X, p)
    assert np.abs(got - want).max() < 1e-12


def test_masked_padding_equals_short_group():
    """A padded, key-masked group must equal attention over the real members."""
    p = _params()
    rng = np.random.default_rng(2)
    m, G = 5, 8
    X = rng.standard_normal((m, 32))
    Xp = np.concatenate([X, rng.standard_normal((G - m, 32)) * 50.0])
    mask = torch.tensor([False] * m + [True] * (G - m))[None]
    with torch.no_grad():
        want = _torch_encoder_layer(p)(torch.tensor(Xp)[None], src_key_padding_mask=mask)[0].numpy()
    got = oracle.group_layer(X, p)
    assert np.abs(got - want[:m]).max() < 1e-12


def test_pointwise_functions_against_library():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((7, 19)) * 3
    g, b = rng.standard_normal(19), rng.standard_normal(19)
    want = torch.nn.functional.layer_norm(torch.tensor(x), (19,), torch.tensor(g), torch.tensor(b), 1e-5)
    assert np.abs(oracle.layer_norm(x, g, b, 1e-5) - want.numpy()).max() < 1e-13
    want = torch.nn.functional.gelu(torch.tensor(x)).numpy()
    assert np.abs(oracle.gelu_erf(x) - want).max() < 1e-14
    for v in (-3.0, -0.5, 0.0, 0.7, 4.0):
        assert abs(oracle.gelu_erf(np.array(v)) - 0.5 * v * (1 + math.erf(v / math.sqrt(2)))) < 1e-15
    P = oracle.softmax_rows(x)
    assert np.abs(P.sum(-1) - 1).max() < 1e-14
    assert np.abs(P - torch.softmax(torch.tensor(x), -1).numpy()).max() < 1e-15
    assert np.isfinite(oracle.softmax_rows(x + 1e4)).all()       # max-subtracted


def test_zero_query_projection_gives_mean_of_values():
    p = _params()
    C = 32
    p["w_qkv"][:C] = 0
    p["b_qkv"][:C] = 0
    rng = np.random.default_rng(4)
    X = rng.standard_normal((13, C))
    U = oracle.layer_norm(X, p["ln1_g"], p["ln1_b"], p["ln_eps"])
    Vmean = (U @ p["w_qkv"][2 * C:].astype(np.float64).T + p["b_qkv"][2 * C:]).mean(0)
    X1 = X + Vmean @ p["w_o"].astype(np.float64).T + p["b_o"]
    H = oracle.layer_norm(X1, p["ln2_g"], p["ln2_b"], p["ln_eps"]) @ p["w1"].astype(np.float64).T + p["b1"]
    H = np.array([[0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in r] for r in H])
    want = X1 + H @ p["w2"].astype(np.float64).T + p["b2"]
    assert np.abs(oracle.group_layer(X, p) - want).max() < 1e-12


def test_group_size_one_is_a_per_row_mlp(cfg):
    """G = 1: softmax over one key is 1, so attention returns the value row."""
    c = cfg(1)
    p = c["layer_params"][0]
    C = c["C"]
    feats = c["feats"][:300].astype(np.float64)
    coords = c["coords"][:300]
    g = Geometry(1, 64, 64, 8, 8)
    W = lambda k: p[k].astype(np.float64)
    U = oracle.layer_norm(feats, W("ln1_g"), W("ln1_b"), p["ln_eps"])
    X1 = feats + (U @ W("w_qkv")[2 * C:].T + W("b_qkv")[2 * C:]) @ W("w_o").T + W("b_o")
    Hn = oracle.layer_norm(X1, W("ln2_g"), W("ln2_b"), p["ln_eps"]) @ W("w1").T + W("b1")
    want = X1 + oracle.gelu_erf(Hn) @ W("w2").T + W("b2")
    for axis, shift in [(0, 0), (1, 1)]:
        perm, off, _ = oracle.flatten(coords, g, axis, shift, 1)
        assert len(off) == 301
        got = oracle.layer(feats, perm, off, p)
        assert np.abs(got - want).max() < 1e-12


def test_group_covering_everything_ignores_the_sort(cfg):
    """G >= n: one global attention; without positional terms the result in
    pillar order cannot depend on axis, shift or window."""
    c = cfg(1)
    p = c["layer_params"][0]
    feats = c["feats"][:200].astype(np.float64)
    coords = c["coords"][:200]
    want = oracle.group_layer(feats, p)
    for w, axis, shift in [(8, 0, 0), (8, 1, 1), (3, 0, 1), (64, 1, 0)]:
        perm, off, _ = oracle.flatten(coords, Geometry(1, 64, 64, w, w), axis, shift, 200)
        assert off.tolist() == [0, 200]
        got = oracle.layer(feats, perm, off, p)
        assert np.abs(got - want).max() < 1e-12


def test_input_permutation_equivariance(cfg):
    c = cfg(1)
    p = c["layer_params"][1]
    n = 500
    feats, coords = c["feats"][:n].astype(np.float64), c["coords"][:n]
    g = Geometry(1, 64, 64, 8, 8)
    pi = np.random.default_rng(6).permutation(n)
    perm, off, _ = oracle.flatten(coords, g, 1, 1, 32)
    a = oracle.layer(feats, perm, off, p)
    perm2, off2, _ = oracle.flatten(coords[pi], g, 1, 1, 32)
    b = oracle.layer(feats[pi], perm2, off2, p)
    assert np.abs(a[pi] - b).max() < 1e-12


def test_zero_output_projections_give_identity():
    p = _params()
    for k in ("w_o", "b_o", "w2", "b2"):
        p[k] = np.zeros_like(p[k])
    X = np.random.default_rng(7).standard_normal((9, 32))
    assert np.array_equal(oracle.group_layer(X, p), X)


def test_layer_scatter_and_partial_groups(cfg):
    c = cfg(1)
    p = c["layer_params"][0]
    n = 333
    feats, coords = c["feats"][:n], c["coords"][:n]
    perm, off, _ = oracle.flatten(coords, Geometry(1, 64, 64, 8, 8), 0, 0, 32)
    full = oracle.layer(feats, perm, off, p)
    assert np.isfinite(full).all()
    some = oracle.layer(feats, perm, off, p, groups=[0, len(off) - 2])
    rows = np.concatenate([perm[off[0]:off[1]], perm[off[-2]:off[-1]]])
    assert np.array_equal(some[rows], full[rows])
    rest = np.setdiff1d(np.arange(n), rows)
    assert np.isnan(some[rest]).all()
    # tail group (13 members) equals the single-group function on its rows
    tail = perm[off[-2]:off[-1]]
    assert len(tail) == n - 32 * (n // 32)
    assert np.abs(full[tail] - oracle.group_layer(feats[tail].astype(np.float64), p)).max() == 0


def test_stack_uses_four_sorts_and_drop_passthrough(cfg):
    c = cfg(1, 4)
    n = 400
    feats, coords = c["feats"][:n], c["coords"][:n]
    g = Geometry(1, 64, 64, 8, 8)
    sched = ffsynth.layer_schedule(4)
    perms, offs = {}, {}
    for key in set(sched):
        perms[key], offs[key], _ = oracle.flatten(coords, g, key[0], key[1], 32)
    trace = oracle.stack(feats, perms, offs, c["layer_params"], sched)
    assert len(trace) == 5
    cur = feats.astype(np.float64)
    for l, key in enumerate(sched):                         # recomputed sorts give the same
        pr, of, _ = oracle.flatten(coords, g, key[0], key[1], 32)
        cur = oracle.layer(cur, pr, of, c["layer_params"][l])
    assert np.array_equal(cur, trace[-1])
    # drop mode: rows of the short tail pass through unchanged
    pr, starts, _ = oracle.flatten(coords, g, 0, 0, 32, tail="drop")
    off_full = np.concatenate([starts, [starts[-1] + 32]]).astype(np.int32)
    out = oracle.layer(feats, pr, off_full, c["layer_params"][0])
    tail_rows = pr[off_full[-1]:]
    assert len(tail_rows) == 16 and np.array_equal(out[tail_rows], feats[tail_rows].astype(np.float64))


def test_drop_residual_with_several_frames(cfg):
    """'Drop Residual' (Sec. 4.3) over four frames, one of them shorter than a group: the listed
    groups are exactly the full runs of G inside each frame, their rows equal the group layer of
    those rows, and every other row is the input row."""
    c = cfg(1, 1)
    rng = np.random.default_rng(5)
    counts = [70, 9, 64, 45]                                # frame sizes: 2+0+2+1 full groups of 32
    coords = np.concatenate([np.column_stack([np.full(k, b), rng.permutation(40 * 40)[:k] // 40,
                                              rng.permutation(40 * 40)[:k] % 40])
                             for b, k in enumerate(counts)]).astype(np.int32)
    coords = coords[rng.permutation(len(coords))]
    n, G = len(coords), 32
    feats = c["feats"][:n]
    g = Geometry(4, 40, 40, 8, 8)
    perm, starts, _ = oracle.flatten(coords, g, 1, 1, G, tail="drop")
    frame_start = np.concatenate([[0], np.cumsum(counts)])
    want = [int(frame_start[b]) + k * G for b in range(4) for k in range(counts[b] // G)]
    assert starts.tolist() == want                          # brute force from the frame sizes
    out = oracle.layer(feats, perm, starts, c["layer_params"][0], group_size=G)
    grouped = np.zeros(n, bool)
    for s0 in want:
        rows = perm[s0:s0 + G]
        assert len(set(coords[rows, 0])) == 1               # a group never spans two frames
        assert np.array_equal(out[rows], oracle.group_layer(feats[rows].astype(np.float64), c["layer_params"][0]))
        grouped[rows] = True
    assert grouped.sum() == G * len(want) and (~grouped).sum() == 6 + 9 + 0 + 13
    assert np.array_equal(out[~grouped], feats[~grouped].astype(np.float64))
    # the masked list restricted to its full groups is the same list
    _, off, _ = oracle.flatten(coords, g, 1, 1, G)
    assert [int(a) for a, b in zip(off[:-1], off[1:]) if b - a == G] == want


@pytest.mark.parametrize("C,F,heads,m", [(32, 48, 4, 11), (128, 256, 8, 64)])
def test_positional_embedding_against_library_attention(C, F, heads, m):
    """PE(C) of Eq. (2) as read here: queries and keys from LN(F) + PE, values from LN(F).  The
    library's attention module takes the three inputs separately."""
    p = ffsynth.layer_params(C, F, heads, seed=6)
    rng = np.random.default_rng(2)
    X, pe = rng.standard_normal((m, C)), 0.5 * rng.standard_normal((m, C))
    enc = _torch_encoder_layer(p)
    with torch.no_grad():
        x = torch.tensor(X)[None]
        u = enc.norm1(x)
        qk = u + torch.tensor(pe)[None]
        x1 = x + enc.self_attn(qk, qk, u, need_weights=False)[0]
        want = (x1 + enc.linear2(torch.nn.functional.gelu(enc.linear1(enc.norm2(x1)))))[0].numpy()
    got = oracle.group_layer(X, p, pe)
    assert np.abs(got - want).max() < 1e-12
    assert np.abs(got - oracle.group_layer(X, p)).max() > 1e-3          # the embedding matters
    assert np.array_equal(oracle.group_layer(X, p, np.zeros((m, C))), oracle.group_layer(X, p))
    # with no query and key projection the embedding cannot reach the output
    p0 = dict(p)
    p0["w_qkv"] = np.array(p["w_qkv"], dtype=np.float64)
    p0["w_qkv"][:2 * C] = 0.0
    assert np.array_equal(oracle.group_layer(X, p0, pe), oracle.group_layer(X, p0))


def test_positional_embedding_rows_follow_the_pillars(cfg):
    """layer() hands each group the embedding rows of its own members (pillar order, like feats)."""
    c = cfg(1, 1)
    n = 200
    feats, coords, p = c["feats"][:n], c["coords"][:n], c["layer_params"][0]
    pe = np.random.default_rng(3).standard_normal(feats.shape)
    perm, off, _ = oracle.flatten(coords, Geometry(1, 64, 64, 8, 8), 1, 0, 32)
    out = oracle.layer(feats, perm, off, p, pos_embed=pe)
    for g in range(len(off) - 1):
        rows = perm[off[g]:off[g + 1]]
        assert np.array_equal(out[rows], oracle.group_layer(feats[rows].astype(np.float64), p, pe[rows]))
    tr = oracle.stack(feats, {(1, 0): perm}, {(1, 0): off}, [p], [(1, 0)], pos_embed=pe)
    assert np.array_equal(tr[-1], out)
