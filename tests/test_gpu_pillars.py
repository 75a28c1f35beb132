"""GPU parity for the steps either side of the FWA blocks: dense BEV scatter (bit-exact)."""
import numpy as np
import pytest
import torch

import ffsynth
import oracle
import paper_2301_08739_amd as ff
from gpu_util import DEV, geoms, to_dev_feats

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("i,dt", [(1, ff.FF_F32), (2, ff.FF_BF16), (2, ff.FF_F16), (5, ff.FF_BF16)])
def test_bev_scatter_bit_exact(cfg, i, dt):
    c = cfg(i, 1)
    g, og = geoms(c)
    n = c["n"] if i != 5 else 60000
    coords, feats = c["coords"][:n], c["feats"][:n]
    x = to_dev_feats(feats, dt)
    bev = ff.ff_bev_scatter(x, torch.from_numpy(coords).to(DEV), g, dt)
    torch.cuda.synchronize()
    want = oracle.bev_scatter(x.cpu().view(torch.int16 if dt != ff.FF_F32 else torch.int32).numpy(), coords, og)
    got = bev.cpu().view(torch.int16 if dt != ff.FF_F32 else torch.int32).numpy()
    assert got.shape == want.shape and np.array_equal(got, want)


def test_bev_scatter_edges():
    g, og = ff.Geometry(2, 5, 3, 1, 1), oracle.Geometry(2, 5, 3, 1, 1)
    empty = ff.ff_bev_scatter(torch.zeros((0, 8), device=DEV), torch.zeros((0, 3), dtype=torch.int32, device=DEV), g, ff.FF_F32)
    assert empty.shape == (2, 3, 5, 8) and not empty.any()
    coords = np.array([[0, 0, 0], [1, 4, 2], [2, 0, 0], [0, 5, 0], [0, 0, -1]], np.int32)      # three outside
    feats = np.arange(5 * 8, dtype=np.float32).reshape(5, 8) + 1
    out = torch.full((2, 3, 5, 8), 9.0, device=DEV)                                           # stale contents are overwritten
    got = ff.ff_bev_scatter(torch.from_numpy(feats).to(DEV), torch.from_numpy(coords).to(DEV), g, ff.FF_F32, out=out)
    assert np.array_equal(got.cpu().numpy(), oracle.bev_scatter(feats, coords, og))
    with pytest.raises(ff.FlatformerError):
        ff.ff_bev_scatter(torch.zeros((4, 3), device=DEV), torch.zeros((4, 3), dtype=torch.int32, device=DEV), g, ff.FF_F32)


def _voxelize_case(m, B, Cp, seed, gx=468, gy=468, voxel=0.32, half=74.88):
    xy, frame, pf = ffsynth.lidar_points(seed, m, B, Cp)
    g, og = ff.Geometry(B, gx, gy, 13, 13), oracle.Geometry(B, gx, gy, 13, 13)
    grid = ff.VoxelGrid(-half, -half, voxel, voxel)
    coords, feats, npil, p2p = ff.ff_voxelize(torch.from_numpy(xy).to(DEV), torch.from_numpy(frame).to(DEV),
                                              torch.from_numpy(pf).to(DEV), g, grid)
    torch.cuda.synchronize()
    n = int(npil.item())
    wc, wf, wp = oracle.voxelize(xy, frame, pf, og, -half, -half, voxel, voxel)
    assert n == len(wc), (n, len(wc))
    assert np.array_equal(coords[:n].cpu().numpy(), wc)                 # cells and their order: bit-exact
    assert np.array_equal(p2p.cpu().numpy(), wp)
    err = np.abs(feats[:n].cpu().numpy().astype(np.float64) - wf).max() if n else 0.0
    counts = np.bincount(wp[wp >= 0], minlength=max(n, 1))
    print(f"voxelize m={m} B={B} Cp={Cp}: {n} pillars, {int((wp < 0).sum())} points dropped, "
          f"largest pillar {int(counts.max()) if n else 0} points, max abs err of the means {err:.2e}", flush=True)
    assert err <= 1e-5          # float32 sums of at most a few hundred N(0,1) values, then one division
    return n


@pytest.mark.parametrize("m,B,Cp", [(0, 1, 4), (1, 1, 4), (1000, 2, 3), (5000, 1, 9), (180000, 1, 4), (400000, 3, 5)])
def test_voxelize_against_oracle(m, B, Cp):
    _voxelize_case(m, B, Cp, seed=100 + m + B)


def test_voxelize_small_grid_and_everything_outside():
    # coarse cells: many points per pillar; then a grid nothing falls into
    assert _voxelize_case(20000, 2, 4, seed=7, gx=40, gy=30, voxel=4.0, half=60.0) > 0
    assert _voxelize_case(3000, 1, 4, seed=8, gx=4, gy=4, voxel=0.01, half=500.0) == 0


def test_voxelize_then_flatten_then_bev(cfg):
    """The three steps in a row: points -> pillars -> (sorted for a layer) -> dense map."""
    xy, frame, pf = ffsynth.lidar_points(5, 120000, 1, 8)
    g = ff.Geometry(1, 468, 468, 13, 13)
    coords, feats, npil, _ = ff.ff_voxelize(torch.from_numpy(xy).to(DEV), None, torch.from_numpy(pf).to(DEV), g,
                                            ff.VoxelGrid(-74.88, -74.88, 0.32, 0.32), want_map=False)
    n = int(npil.item())
    coords, feats = coords[:n].contiguous(), feats[:n].contiguous()
    perm, goff, ng, _ = ff.ff_flatten(coords, g, 1, 1, 64)
    assert torch.equal(torch.sort(perm.long())[0], torch.arange(n, device=DEV))
    bev = ff.ff_bev_scatter(feats, coords, g, ff.FF_F32)
    torch.cuda.synchronize()
    c = coords.long()
    assert torch.equal(bev[c[:, 0], c[:, 2], c[:, 1]], feats) and int((bev.abs().sum(-1) > 0).sum()) <= n
