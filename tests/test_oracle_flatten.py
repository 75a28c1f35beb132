"""Pins for the flatten oracle: hand-worked cases, brute force, library special
cases and invariants.  None of these uses the oracle to check itself."""
import itertools
import os

import numpy as np
import pytest

import ffsynth
import oracle
from oracle import Geometry

GOLD = os.path.join(os.path.dirname(__file__), "golden", "eq1_hand_worked.txt")


def _gold_lines(tag):
    with open(GOLD) as f:
        for line in f:
            if line.startswith(tag + " "):
                yield line[len(tag) + 1:].strip()


def test_hand_worked_tuples():
    n = 0
    for line in _gold_lines("TUPLE"):
        lhs, rhs = line.split("->")
        b, x, y, wx, wy, axis, shift = map(int, lhs.split())
        want = tuple(map(int, rhs.split()))
        g = Geometry(16, 1000, 1000, wx, wy)
        assert oracle.window_tuple(b, x, y, g, axis, shift) == want, line
        n += 1
    assert n >= 8


def test_hand_worked_keys():
    for line in _gold_lines("KEY"):
        lhs, rhs = line.split("->")
        assert oracle.pack_key(tuple(map(int, lhs.split()))) == int(rhs), line


def test_hand_worked_sort():
    pts = list(map(int, next(_gold_lines("POINTS")).split()))
    coords = np.array([[0, pts[2 * i], pts[2 * i + 1]] for i in range(6)], dtype=np.int32)
    g = Geometry(1, 4, 4, 2, 2)
    for line in _gold_lines("SORT"):
        lhs, rhs = line.split("->")
        axis, shift = map(int, lhs.split())
        perm_s, off_s = rhs.split(";")
        perm, off, keys = oracle.flatten(coords, g, axis, shift, 4)
        assert perm.tolist() == list(map(int, perm_s.split())), line
        assert off.tolist() == list(map(int, off_s.split())), line


def _brute_tuple(b, x, y, wx, wy, axis, shift):
    """Independent restatement with divmod and explicit branches."""
    sx = wx // 2 if shift else 0
    sy = wy // 2 if shift else 0
    Wx, Lx = divmod(x + sx, wx)
    Wy, Ly = divmod(y + sy, wy)
    return (b, Wx, Wy, Lx, Ly) if axis == 0 else (b, Wy, Wx, Ly, Lx)


@pytest.mark.parametrize("w", [1, 2, 3, 8])
def test_tuple_exhaustive_small_grids(w):
    g = Geometry(2, 8, 8, w, w)
    for b, x, y, axis, shift in itertools.product(range(2), range(8), range(8), (0, 1), (0, 1)):
        t = oracle.window_tuple(b, x, y, g, axis, shift)
        assert t == _brute_tuple(b, x, y, w, w, axis, shift)
        # Eq. (1) is invertible: window * w + local gives the (shifted) coordinate back
        s = w // 2 if shift else 0
        if axis == 0:
            assert (t[1] * w + t[3] - s, t[2] * w + t[4] - s) == (x, y)
        else:
            assert (t[2] * w + t[4] - s, t[1] * w + t[3] - s) == (x, y)


def test_key_order_equals_tuple_order_and_overflow():
    rng = np.random.default_rng(0)
    ts = [tuple(int(v) for v in (rng.integers(0, 65536), rng.integers(0, 65536),
                                 rng.integers(0, 65536), rng.integers(0, 256),
                                 rng.integers(0, 256))) for _ in range(2000)]
    ts += [(65535, 65535, 65535, 255, 255), (0, 0, 0, 0, 0)]
    ks = [oracle.pack_key(t) for t in ts]
    assert max(ks) == 2 ** 64 - 1
    order_t = sorted(range(len(ts)), key=lambda i: ts[i])
    order_k = sorted(range(len(ts)), key=lambda i: ks[i])
    assert [ts[i] for i in order_t] == [ts[i] for i in order_k]
    for bad in [(65536, 0, 0, 0, 0), (0, 65536, 0, 0, 0), (0, 0, 0, 256, 0), (0, 0, 0, 0, 256)]:
        with pytest.raises(OverflowError):
            oracle.pack_key(bad)


def _rand_unique(n, B, gx, gy, seed):
    rng = np.random.default_rng(seed)
    ids = rng.permutation(B * gx * gy)[:n]
    b, r = np.divmod(ids, gx * gy)
    x, y = np.divmod(r, gy)
    return np.stack([b, x, y], axis=1).astype(np.int32)


@pytest.mark.parametrize("axis,shift", [(0, 0), (1, 0), (0, 1), (1, 1)])
def test_bruteforce_comparison_sort(axis, shift):
    """Selection sort with an explicit field-by-field comparison."""
    coords = _rand_unique(150, 2, 12, 10, seed=3)
    coords = np.concatenate([coords, coords[:7]])          # duplicates: ties by index
    g = Geometry(2, 12, 10, 4, 3)
    perm, off, keys = oracle.flatten(coords, g, axis, shift, 16)

    def less(i, j):
        ti = _brute_tuple(*map(int, coords[i]), 4, 3, axis, shift)
        tj = _brute_tuple(*map(int, coords[j]), 4, 3, axis, shift)
        for a, b in zip(ti, tj):
            if a != b:
                return a < b
        return i < j
    rest = list(range(len(coords)))
    want = []
    while rest:
        m = rest[0]
        for c in rest[1:]:
            if less(c, m):
                m = c
        want.append(m)
        rest.remove(m)
    assert perm.tolist() == want


@pytest.mark.parametrize("axis", [0, 1])
def test_window_one_or_whole_grid_is_lexsort(axis):
    """Without quantisation the order is the plain coordinate sort."""
    coords = _rand_unique(3000, 3, 40, 50, seed=1)
    if axis == 0:
        want = np.lexsort((coords[:, 2], coords[:, 1], coords[:, 0]))
    else:
        want = np.lexsort((coords[:, 1], coords[:, 2], coords[:, 0]))
    for w in (1, 64):
        g = Geometry(3, 40, 50, w, w)
        perm, _, _ = oracle.flatten(coords, g, axis, 0, 10)
        assert np.array_equal(perm, want)


def test_invariants_on_config1(cfg):
    c = cfg(1)
    coords = c["coords"]
    n = c["n"]
    g = Geometry(1, 64, 64, 8, 8)
    members = {}
    for axis, shift in [(0, 0), (1, 0), (0, 1), (1, 1)]:
        perm, off, keys = oracle.flatten(coords, g, axis, shift, 32)
        assert np.array_equal(np.sort(perm), np.arange(n))                 # bijection
        assert np.all(keys[1:] > keys[:-1])                                # unique coords
        # each window's members are contiguous in the order
        s = 4 if shift else 0
        win = ((coords[perm, 1] + s) // 8) * 100 + (coords[perm, 2] + s) // 8
        change = np.flatnonzero(win[1:] != win[:-1])
        assert len(change) + 1 == len(np.unique(win))
        members[(axis, shift)] = {w: frozenset(perm[win == w].tolist()) for w in np.unique(win)}
        # grouping: every group G long except the last one
        d = np.diff(off)
        assert off[0] == 0 and off[-1] == n and np.all(d[:-1] == 32) and 1 <= d[-1] <= 32
        assert len(off) - 1 == -(-n // 32)
    # both axes agree on which pillars share a window
    assert members[(0, 0)] == members[(1, 0)]
    assert members[(0, 1)] == members[(1, 1)]


def test_axis_swap_and_shift_identities():
    coords = _rand_unique(2500, 2, 37, 41, seed=5)
    g = Geometry(2, 37, 41, 5, 7)
    swapped = coords[:, [0, 2, 1]]
    gs = Geometry(2, 41, 37, 7, 5)
    for shift in (0, 1):
        p1, o1, k1 = oracle.flatten(coords, g, 1, shift, 9)
        p0, o0, k0 = oracle.flatten(swapped, gs, 0, shift, 9)
        assert np.array_equal(p1, p0) and np.array_equal(k1, k0) and np.array_equal(o1, o0)
    moved = coords.copy()
    moved[:, 1] += 5 // 2
    moved[:, 2] += 7 // 2
    for axis in (0, 1):
        ps, _, ks = oracle.flatten(coords, g, axis, 1, 9)
        pm, _, km = oracle.flatten(moved, Geometry(2, 39, 44, 5, 7), axis, 0, 9)
        assert np.array_equal(ps, pm) and np.array_equal(ks, km)
    # translating by whole windows changes window ids but not the order
    far = coords.copy()
    far[:, 1] += 3 * 5
    for axis in (0, 1):
        pa, _, _ = oracle.flatten(coords, g, axis, 0, 9)
        pb, _, _ = oracle.flatten(far, Geometry(2, 52, 41, 5, 7), axis, 0, 9)
        assert np.array_equal(pa, pb)


def test_input_permutation_equivariance():
    coords = _rand_unique(800, 1, 30, 30, seed=8)
    g = Geometry(1, 30, 30, 4, 4)
    pi = np.random.default_rng(2).permutation(800)
    p_a, _, k_a = oracle.flatten(coords, g, 0, 1, 7)
    p_b, _, k_b = oracle.flatten(coords[pi], g, 0, 1, 7)
    assert np.array_equal(pi[p_b], p_a) and np.array_equal(k_a, k_b)


@pytest.mark.parametrize("axis,shift", [(0, 0), (1, 1)])
def test_rank_by_occupancy_bitmap(axis, shift):
    """Third derivation for unique cells: walk the cells in traversal order and
    number the occupied ones."""
    B, gx, gy, w = 2, 20, 23, 6
    coords = _rand_unique(500, B, gx, gy, seed=11)
    g = Geometry(B, gx, gy, w, w)
    perm, _, _ = oracle.flatten(coords, g, axis, shift, 13)
    s = w // 2 if shift else 0
    occ = {(int(b), int(x), int(y)): i for i, (b, x, y) in enumerate(coords)}
    nwx, nwy = -(-(gx + s) // w), -(-(gy + s) // w)
    walk = []
    for b in range(B):
        if axis == 0:
            for Wx, Wy, Lx, Ly in itertools.product(range(nwx), range(nwy), range(w), range(w)):
                walk.append((b, Wx * w + Lx - s, Wy * w + Ly - s))
        else:
            for Wy, Wx, Ly, Lx in itertools.product(range(nwy), range(nwx), range(w), range(w)):
                walk.append((b, Wx * w + Lx - s, Wy * w + Ly - s))
    want = [occ[c] for c in walk if c in occ]
    assert perm.tolist() == want


def test_grouping_per_frame_and_edge_cases():
    coords = _rand_unique(1000, 4, 25, 25, seed=4)
    coords = coords[coords[:, 0] != 2]                     # frame 2 is empty
    g = Geometry(4, 25, 25, 5, 5)
    G = 17
    perm, off, keys = oracle.flatten(coords, g, 0, 0, G)
    counts = np.bincount(coords[:, 0], minlength=4)
    assert counts[2] == 0
    assert len(off) - 1 == sum(-(-int(c) // G) for c in counts)
    fb = coords[perm, 0]
    starts = np.concatenate([[0], np.cumsum(counts)])
    for gi in range(len(off) - 1):
        seg = fb[off[gi]:off[gi + 1]]
        assert seg.min() == seg.max()                      # never spans two frames
        b = int(seg[0])
        last_of_frame = off[gi + 1] == starts[b + 1]
        assert (off[gi] - starts[b]) % G == 0
        assert len(seg) == G or (last_of_frame and 1 <= len(seg) < G)
    # drop mode keeps only full groups
    _, full, _ = oracle.flatten(coords, g, 0, 0, G, tail="drop")
    assert len(full) == sum(int(c) // G for c in counts)
    assert set(full.tolist()) <= set(off.tolist())
    # n = 0 and n divisible by G
    p0, o0, k0 = oracle.flatten(np.zeros((0, 3), np.int32), g, 0, 0, G)
    assert p0.shape == (0,) and o0.tolist() == [0] and k0.shape == (0,)
    c2 = _rand_unique(64, 1, 25, 25, seed=9)
    _, o2, _ = oracle.flatten(c2, Geometry(1, 25, 25, 5, 5), 1, 1, 16)
    assert o2.tolist() == [0, 16, 32, 48, 64]


def test_generator_shapes(cfg):
    c = cfg(1)
    assert c["coords"].shape == (2000, 3) and c["coords"].dtype == np.int32
    assert c["feats"].shape == (2000, 64) and c["schedule"] == [(0, 0), (1, 0)]
    assert ffsynth.layer_schedule(8) == [(0, 0), (1, 0), (0, 1), (1, 1)] * 2
    assert len(set(ffsynth.layer_schedule(8))) == 4        # 8 layers share 4 sorts
    x = np.array([1.0, 1.00390625, 1.01171875, -3.3895314e38, 1e-40], dtype=np.float32)
    r = ffsynth.bf16_round(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625)  # ties to even
    assert np.array_equal(ffsynth.bf16_round(r), r)


def test_three_dimensional_windows():
    """3-D windows (footnote of Sec. 4.2.1): reduces to the BEV case for a flat grid, agrees with a
    lexicographic library sort of the explicit seven-field tuples, keeps the grouping rules."""
    rng = np.random.default_rng(11)
    n = 600
    ids = rng.permutation(2 * 12 * 10 * 6)[:n]
    b, r = np.divmod(ids, 12 * 10 * 6)
    x, r = np.divmod(r, 10 * 6)
    y, z = np.divmod(r, 6)
    c4 = np.stack([b, x, y, z], 1).astype(np.int32)
    g3 = oracle.Geometry3(2, 12, 10, 6, 5, 3, 4)
    for axis in (0, 1):
        for shift in (0, 1):
            perm, off = oracle.flatten3d(c4, g3, axis, shift, 17)
            sx, sy, sz = (5 // 2, 3 // 2, 4 // 2) if shift else (0, 0, 0)
            X, Y, Z = c4[:, 1] + sx, c4[:, 2] + sy, c4[:, 3] + sz
            f = [c4[:, 0], X // 5, Y // 3, Z // 4, X % 5, Y % 3, Z % 4]
            if axis == 1:
                f = [f[0], f[2], f[1], f[3], f[5], f[4], f[6]]
            want = np.lexsort(tuple(reversed(f)))                      # library sort, first field most significant
            assert np.array_equal(perm, want)                          # coordinates are unique: no ties
            counts = np.bincount(c4[:, 0], minlength=2)
            assert len(off) - 1 == sum(-(-int(k) // 17) for k in counts) and off[-1] == n
            _, starts = oracle.flatten3d(c4, g3, axis, shift, 17, tail="drop")
            assert len(starts) == sum(int(k) // 17 for k in counts)
    # a grid that is one voxel high with a window one voxel high is the BEV case
    c3 = _rand_unique(500, 3, 20, 20, seed=12)
    c4 = np.concatenate([c3, np.zeros((500, 1), np.int32)], axis=1)
    for axis, shift in [(0, 0), (1, 1)]:
        p2, o2, _ = oracle.flatten(c3, Geometry(3, 20, 20, 6, 4), axis, shift, 9)
        p3, o3 = oracle.flatten3d(c4, oracle.Geometry3(3, 20, 20, 1, 6, 4, 1), axis, shift, 9)
        assert np.array_equal(p2, p3) and np.array_equal(o2, o3)
