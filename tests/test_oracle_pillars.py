"""Pins for the voxelisation / BEV-scatter oracle: library routines (unique, bincount, add.at),
closed forms and invariants on small inputs."""
import numpy as np

import oracle
from oracle import Geometry


def _points(m, B, seed, span=12.0):
    rng = np.random.default_rng(seed)
    xy = rng.uniform(-span, span, size=(m, 2)).astype(np.float32)
    frame = rng.integers(0, B, size=m).astype(np.int32)
    pf = rng.standard_normal((m, 5)).astype(np.float32)
    return xy, frame, pf


def test_voxelize_against_unique_and_add_at():
    g = Geometry(3, 64, 48, 1, 1)
    xy, frame, pf = _points(5000, 3, seed=1)
    xmin, ymin, vx, vy = -10.24, -7.68, 0.32, 0.32                   # part of the cloud lies outside
    coords, feats, p2p = oracle.voxelize(xy, frame, pf, g, xmin, ymin, vx, vy)
    cx = np.floor((xy[:, 0] - np.float32(xmin)) / np.float32(vx)).astype(np.int64)
    cy = np.floor((xy[:, 1] - np.float32(ymin)) / np.float32(vy)).astype(np.int64)
    keep = (cx >= 0) & (cx < 64) & (cy >= 0) & (cy < 48)
    assert 0 < keep.sum() < len(xy)
    ids = (frame.astype(np.int64) * 64 + cx) * 48 + cy
    uniq, inv, cnt = np.unique(ids[keep], return_inverse=True, return_counts=True)   # ascending id = ascending (b, x, y)
    assert len(coords) == len(uniq)
    assert np.array_equal((coords[:, 0].astype(np.int64) * 64 + coords[:, 1]) * 48 + coords[:, 2], uniq)
    sums = np.zeros((len(uniq), 5))
    np.add.at(sums, inv, pf[keep].astype(np.float64))
    assert np.abs(feats - sums / cnt[:, None]).max() < 1e-12
    assert np.array_equal(p2p[keep], inv) and (p2p[~keep] == -1).all()
    assert np.array_equal(np.bincount(p2p[keep], minlength=len(uniq)), cnt)


def test_voxelize_closed_forms():
    g = Geometry(1, 4, 4, 1, 1)
    # four points in one cell, one on a cell edge (belongs to the upper cell), one outside
    xy = np.array([[0.1, 0.1], [0.2, 0.3], [0.9, 0.9], [0.5, 0.5], [1.0, 0.0], [4.0, 0.0], [-0.001, 0.0]], np.float32)
    pf = np.arange(7, dtype=np.float32)[:, None] * np.ones((1, 2), np.float32)
    coords, feats, p2p = oracle.voxelize(xy, np.zeros(7, np.int32), pf, g, 0.0, 0.0, 1.0, 1.0)
    assert coords.tolist() == [[0, 0, 0], [0, 1, 0]]
    assert np.allclose(feats, [[1.5, 1.5], [4.0, 4.0]])
    assert p2p.tolist() == [0, 0, 0, 0, 1, -1, -1]
    # one point per cell: pillars are the points in (b, x, y) order, features unchanged
    xs, ys = np.meshgrid(np.arange(4), np.arange(4), indexing="ij")
    xy = np.stack([xs.ravel() + 0.5, ys.ravel() + 0.5], 1).astype(np.float32)
    perm = np.random.default_rng(0).permutation(16)
    pf = np.random.default_rng(1).standard_normal((16, 3)).astype(np.float32)
    coords, feats, p2p = oracle.voxelize(xy[perm], np.zeros(16, np.int32), pf[perm], g, 0.0, 0.0, 1.0, 1.0)
    assert np.array_equal(coords[:, 1] * 4 + coords[:, 2], np.arange(16))
    assert np.array_equal(feats, pf.astype(np.float64)) and np.array_equal(p2p, perm)


def test_bev_scatter_against_fancy_indexing_and_roundtrip():
    g = Geometry(2, 9, 7, 1, 1)
    rng = np.random.default_rng(3)
    ids = rng.permutation(2 * 9 * 7)[:40]
    b, r = np.divmod(ids, 63)
    x, y = np.divmod(r, 7)
    coords = np.stack([b, x, y], 1).astype(np.int32)
    feats = rng.standard_normal((40, 6)).astype(np.float32)
    bev = oracle.bev_scatter(feats, coords, g)
    want = np.zeros((2, 7, 9, 6), np.float32)
    want[b, y, x] = feats                                       # library scatter
    assert bev.shape == (2, 7, 9, 6) and np.array_equal(bev, want)
    assert np.array_equal(bev[coords[:, 0], coords[:, 2], coords[:, 1]], feats)      # gather back
    assert (np.abs(bev).sum(axis=-1) > 0).sum() == 40                                 # nothing else is set
    coords[0] = (2, 0, 0)                                       # outside: skipped
    assert np.array_equal(oracle.bev_scatter(feats, coords, g)[b[1:], y[1:], x[1:]], feats[1:])
