"""Oracle for the two steps either side of the FWA blocks (paper Sec. 5.1 'Model').

TEST INFRASTRUCTURE ONLY -- see the package docstring.

Before the blocks the point cloud is voxelised into sparse bird's-eye-view
pillars (0.32 m x 0.32 m in the paper); after them the pillar features go to a
regular BEV encoder, which wants a dense map.  The paper refers to PointPillars
for the first and gives no formula for either, so both are written out here in
their plainest form:

  voxelize     a point belongs to the cell floor((x - x_min) / voxel_x),
               floor((y - y_min) / voxel_y) of its frame (float32 arithmetic: the
               cell index is an integer decided by floating point, so it is
               decided in the precision the kernels use); points outside the grid
               are dropped; a pillar is a non-empty cell, its feature vector the
               mean of its points' feature vectors; pillars are listed in
               ascending (frame, x, y) order.  The learned per-point network
               PointPillars puts in front of the pooling is not part of this.
  bev_scatter  bev[b, y, x, :] = feats[i] for pillar i = (b, x, y), zero elsewhere.
"""
import numpy as np


def point_cells(xy, frame, geom, x_min, y_min, voxel_x, voxel_y):
    """(cells int64 [m, 3] as (b, x, y), keep bool [m]); float32 arithmetic."""
    xy = np.asarray(xy, dtype=np.float32)
    cx = np.floor((xy[:, 0] - np.float32(x_min)) / np.float32(voxel_x))
    cy = np.floor((xy[:, 1] - np.float32(y_min)) / np.float32(voxel_y))
    frame = np.asarray(frame, dtype=np.int64)
    keep = ((cx >= 0) & (cx < geom.grid_x) & (cy >= 0) & (cy < geom.grid_y) &
            (frame >= 0) & (frame < geom.num_frames))
    cells = np.stack([frame, np.where(keep, cx, 0).astype(np.int64), np.where(keep, cy, 0).astype(np.int64)], axis=1)
    return cells, keep


def voxelize(xy, frame, pfeats, geom, x_min, y_min, voxel_x, voxel_y):
    """Returns (coords int32 [n, 3], feats float64 [n, Cp], point_to_pillar int32 [m], -1 for dropped points)."""
    cells, keep = point_cells(xy, frame, geom, x_min, y_min, voxel_x, voxel_y)
    pfeats = np.asarray(pfeats, dtype=np.float64)
    members = {}
    for i in range(len(cells)):                      # plain loop: a dictionary of member lists
        if keep[i]:
            members.setdefault(tuple(int(v) for v in cells[i]), []).append(i)
    order = sorted(members)                          # ascending (b, x, y)
    coords = np.asarray(order, dtype=np.int32).reshape(len(order), 3)
    feats = np.zeros((len(order), pfeats.shape[1]), dtype=np.float64)
    p2p = np.full(len(cells), -1, dtype=np.int32)
    for k, cell in enumerate(order):
        idx = members[cell]
        feats[k] = pfeats[idx].sum(axis=0) / len(idx)
        p2p[idx] = k
    return coords, feats, p2p


def bev_scatter(feats, coords, geom):
    """Dense map [num_frames, grid_y, grid_x, C]; pillars outside the grid are skipped."""
    feats = np.asarray(feats)
    bev = np.zeros((geom.num_frames, geom.grid_y, geom.grid_x, feats.shape[1]), dtype=feats.dtype)
    for i, (b, x, y) in enumerate(np.asarray(coords)):
        if 0 <= b < geom.num_frames and 0 <= x < geom.grid_x and 0 <= y < geom.grid_y:
            bev[b, y, x, :] = feats[i]
    return bev
