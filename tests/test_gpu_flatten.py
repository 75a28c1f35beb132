"""GPU parity: ff_flatten must equal the oracle bit for bit (keys, perm, group offsets)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2301_08739_amd as ff
from gpu_util import geoms, gpu_flatten

pytestmark = pytest.mark.gpu

SORTS = [(0, 0), (1, 0), (0, 1), (1, 1)]


def _check(coords, g, og, axis, shift, G):
    perm, off, ng, keys, _ = gpu_flatten(coords, g, axis, shift, G)
    wperm, woff, wkeys = oracle.flatten(coords, og, axis, shift, G)
    assert ng == len(woff) - 1
    assert np.array_equal(off, woff)
    assert np.array_equal(perm, wperm)
    assert np.array_equal(keys, wkeys)


@pytest.mark.parametrize("i", [1, 2, 4, 5])
def test_configs_bit_exact(cfg, i):
    c = cfg(i)
    g, og = geoms(c)
    for axis, shift in SORTS:
        print(f"flatten cfg{i} axis={axis} shift={shift} n={c['n']}", flush=True)
        _check(c["coords"], g, og, axis, shift, c["G"])


def _rand_coords(n, B, gx, gy, seed, unique=True):
    rng = np.random.default_rng(seed)
    if unique:
        ids = rng.permutation(B * gx * gy)[:n]
    else:
        ids = rng.integers(0, B * gx * gy, size=n)
    b, r = np.divmod(ids, gx * gy)
    x, y = np.divmod(r, gy)
    return np.stack([b, x, y], axis=1).astype(np.int32)


@pytest.mark.parametrize("n", [0, 1, 2, 63, 64, 65, 2047, 2048, 2049, 4095, 4096, 4097, 5000, 12288, 65536, 65537, 131072, 131073])
def test_sizes_around_tile_edges(n):
    gx, gy = (90, 70) if n <= 3 * 90 * 70 else (300, 200)
    coords = _rand_coords(n, 3, gx, gy, seed=n, unique=True)
    g, og = ff.Geometry(3, gx, gy, 7, 5), oracle.Geometry(3, gx, gy, 7, 5)
    for axis, shift in [(0, 1), (1, 0)]:
        _check(coords, g, og, axis, shift, 10)


def test_duplicates_keep_index_order():
    coords = _rand_coords(20000, 2, 20, 20, seed=1, unique=False)      # heavy duplication
    g, og = ff.Geometry(2, 20, 20, 4, 4), oracle.Geometry(2, 20, 20, 4, 4)
    for axis, shift in SORTS:
        _check(coords, g, og, axis, shift, 33)
    same = np.zeros((3000, 3), dtype=np.int32)                          # all keys equal
    _check(same, ff.Geometry(1, 1, 1, 1, 1), oracle.Geometry(1, 1, 1, 1, 1), 0, 0, 7)  # zero key bits
    _check(same, g, og, 1, 1, 7)


def test_degenerate_windows_and_groups():
    coords = _rand_coords(3000, 1, 300, 200, seed=2)
    for w in (1, 256):
        g, og = ff.Geometry(1, 300, 200, w, w), oracle.Geometry(1, 300, 200, w, w)
        for axis, shift in [(0, 0), (1, 1)]:
            _check(coords, g, og, axis, shift, 64)
    g, og = ff.Geometry(1, 300, 200, 13, 9), oracle.Geometry(1, 300, 200, 13, 9)
    for G in (1, 2999, 3000, 3001, 100000):
        _check(coords, g, og, 0, 1, G)


def test_many_frames_with_empty_ones():
    B = 700
    coords = _rand_coords(9000, B, 16, 16, seed=3)
    coords = coords[(coords[:, 0] % 7 != 3) & (coords[:, 0] != B - 1)]  # empty frames incl. the last
    g, og = ff.Geometry(B, 16, 16, 4, 4), oracle.Geometry(B, 16, 16, 4, 4)
    for axis, shift in [(0, 0), (1, 1)]:
        _check(coords, g, og, axis, shift, 5)


def test_maximum_field_widths():
    # 65535 frames x 65535 windows on one axis, window 256 on the other: 16+16+8(+0+0) key bits
    rng = np.random.default_rng(4)
    n = 4000
    coords = np.stack([rng.integers(0, 65535, n), rng.integers(0, 65535, n), rng.integers(0, 256, n)], 1).astype(np.int32)
    coords[0] = (65534, 65534, 255)
    g, og = ff.Geometry(65535, 65535, 256, 1, 256), oracle.Geometry(65535, 65535, 256, 1, 256)
    _check(coords, g, og, 0, 0, 3)
    _check(coords, g, og, 1, 0, 3)


def test_errors_and_determinism():
    coords = torch.zeros((10, 3), dtype=torch.int32, device="cuda")
    with pytest.raises(ff.FlatformerError):
        ff.ff_flatten(coords, ff.Geometry(1, 10, 10, 0, 1), 0, 0, 4)          # window 0
    with pytest.raises(ff.FlatformerError):
        ff.ff_flatten(coords, ff.Geometry(1, 10, 10, 2, 2), 2, 0, 4)          # axis 2
    with pytest.raises(ff.FlatformerError):
        ff.ff_flatten(coords, ff.Geometry(1, 10, 10, 2, 2), 0, 0, 0)          # G 0
    with pytest.raises(ff.FlatformerError):
        ff.ff_flatten(coords, ff.Geometry(1, 10, 10, 2, 2), 0, 0, 4, tail=2)  # no such tail mode
    with pytest.raises(ff.FlatformerError):                                   # 16+16+16+8+8 key bits + index
        ff.ff_flatten(coords, ff.Geometry(65535, 65535 * 256, 65535 * 256, 256, 256), 0, 0, 4)
    c = _rand_coords(50000, 2, 300, 300, seed=5)
    g = ff.Geometry(2, 300, 300, 13, 13)
    a = gpu_flatten(c, g, 0, 1, 64)
    b = gpu_flatten(c, g, 0, 1, 64)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[3], b[3])


@pytest.mark.parametrize("n", [262144, 262145, 700001, 1572864, 1572865])
def test_tile_size_changes_with_cloud_size(n):
    """The sort picks tiles of 1024, 2048 or 4096 words by the number of pillars: both sides of each change."""
    coords = _rand_coords(n, 8, 512, 512, seed=n)
    g, og = ff.Geometry(8, 512, 512, 13, 13), oracle.Geometry(8, 512, 512, 13, 13)
    print(f"flatten n={n}", flush=True)
    _check(coords, g, og, 0, 1, 64)
    _check(coords, g, og, 1, 0, 69)


def test_more_than_1024_tiles():
    """4.2 M pillars: the digit tables have more than 1024 rows, which the column scan takes in
    narrower strips.  One sort configuration against the oracle's tuple sort (about half a minute of
    host time)."""
    n = 4200001
    coords = _rand_coords(n, 8, 1024, 1024, seed=6)
    g, og = ff.Geometry(8, 1024, 1024, 13, 13), oracle.Geometry(8, 1024, 1024, 13, 13)
    print(f"flatten n={n}: oracle sort running", flush=True)
    _check(coords, g, og, 1, 1, 64)


@pytest.mark.parametrize("i,tail", [(1, ff.FF_TAIL_MASK), (2, ff.FF_TAIL_MASK), (2, ff.FF_TAIL_DROP), (5, ff.FF_TAIL_MASK)])
def test_batched_sorts_equal_single_sorts(cfg, i, tail):
    """ff_flatten_batch (the four sort configurations of a block in one launch set, 'Reuse Sorting') gives
    what four ff_flatten calls give; those are held against the oracle above."""
    c = cfg(i, 1)
    g, _ = geoms(c)
    ct = torch.from_numpy(c["coords"]).to("cuda")
    sorts = [(0, 0), (1, 0), (0, 1), (1, 1)]
    for S in (4, 3, 1):
        got = ff.ff_flatten_batch(ct, g, sorts[:S], c["G"], tail=tail)
        torch.cuda.synchronize()
        for (axis, shift), (perm, goff, ng) in zip(sorts, got):
            wperm, wgoff, wng, _ = ff.ff_flatten(ct, g, axis, shift, c["G"], tail=tail)
            k = int(wng.item())
            assert int(ng.item()) == k
            assert torch.equal(perm, wperm) and torch.equal(goff[:k + 1], wgoff[:k + 1])
    with pytest.raises(ff.FlatformerError):
        ff.ff_flatten_batch(ct, g, sorts + [(0, 0)], c["G"])
    with pytest.raises(ff.FlatformerError):
        ff.ff_flatten_batch(ct, g, [(0, 2)], c["G"])


def test_few_frames_single_duplicates_and_sparse_ranges():
    """Up to eight frames with an empty one, a single duplicated pair at the front, in the middle and at the end
    of an otherwise duplicate-free cloud, a handful of pillars at the grid's corners, windows of 1 and of 256,
    nine frames, dropped tails through the batched call: all equal to the oracle."""
    g, og = ff.Geometry(8, 468, 468, 13, 13), oracle.Geometry(8, 468, 468, 13, 13)
    coords = _rand_coords(40000, 8, 468, 468, seed=5)
    coords[:, 0] = np.where(coords[:, 0] == 3, 5, coords[:, 0])           # frame 3 is empty
    for axis, shift in SORTS:
        _check(coords, g, og, axis, shift, 64)
    for at, src in [(0, 1), (20000, 7), (39999, 39998)]:                  # one duplicated pair
        c2 = coords.copy()
        c2[at] = c2[src]
        _check(c2, g, og, 0, 1, 64)
        _check(c2, g, og, 1, 0, 50)
    corners = np.array([[0, 0, 0], [7, 467, 467], [0, 467, 0], [7, 0, 467], [4, 233, 233]], dtype=np.int32)
    for axis, shift in SORTS:
        _check(corners, g, og, axis, shift, 2)
    g1, og1 = ff.Geometry(1, 700, 650, 1, 256), oracle.Geometry(1, 700, 650, 1, 256)   # windows of 1 and of 256
    c1 = _rand_coords(30000, 1, 700, 650, seed=9)
    for axis, shift in SORTS:
        _check(c1, g1, og1, axis, shift, 64)
    g9, og9 = ff.Geometry(9, 468, 468, 13, 13), oracle.Geometry(9, 468, 468, 13, 13)
    _check(coords, g9, og9, 0, 0, 64)
    # drop mode through the batched call
    ct = torch.from_numpy(coords).to("cuda")
    for (axis, shift), (perm, goff, ng) in zip(SORTS, ff.ff_flatten_batch(ct, g, SORTS, 64, tail=ff.FF_TAIL_DROP)):
        wperm, starts, _ = oracle.flatten(coords, og, axis, shift, 64, tail="drop")
        k = int(ng.item())
        assert k == len(starts)
        assert np.array_equal(perm.cpu().numpy(), wperm) and np.array_equal(goff.cpu().numpy()[:k], starts)
        assert int(goff[k].item()) == coords.shape[0]


def test_coordinate_check_and_safety_outside_the_geometry():
    """ff_check_coords counts the rows outside the geometry and names the first; ff_flatten on such a cloud still
    returns a permutation and touches nothing outside its buffers (guard words around perm stay intact)."""
    g = ff.Geometry(2, 100, 80, 7, 5)
    coords = _rand_coords(5000, 2, 100, 80, seed=11)
    ct = torch.from_numpy(coords).to("cuda")
    assert ff.ff_check_coords(ct, g).cpu().tolist() == [0, 5000]
    assert ff.ff_check_coords(ct[:0], g).cpu().tolist() == [0, 0]
    bad = coords.copy()
    bad[77] = (2, 5, 5)            # frame beyond the last
    bad[300] = (0, -1, 5)          # negative x
    bad[301] = (1, 99, 80)         # y == grid_y
    bad[4999] = (-3, 2**30, -2**31)
    bt = torch.from_numpy(bad).to("cuda")
    assert ff.ff_check_coords(bt, g).cpu().tolist() == [4, 77]
    for axis, shift in SORTS:
        perm, goff, ng, _ = ff.ff_flatten(bt, g, axis, shift, 16)
        torch.cuda.synchronize()
        assert np.array_equal(np.sort(perm.cpu().numpy()), np.arange(5000))
        k = int(ng.item())
        assert 0 < k <= 5000 // 16 + 3 and int(goff[k].item()) == 5000
