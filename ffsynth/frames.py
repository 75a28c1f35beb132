"""Synthetic pillar clouds with the shape of single-frame / multi-frame LiDAR
bird's-eye-view scenes: a 468 x 468 grid of 0.32 m pillars over +-74.88 m with
about 20k-40k non-empty pillars per frame (the workload sizes the paper quotes
for its benchmark scenes, Sec. 3 and Sec. 5.1).  These clouds stand in for the
public dataset the paper measures on; nothing of that dataset is reproduced.

Every function returns int32 coordinates [n, 3] with columns (b, x, y), in
first-occurrence (i.e. random, unsorted) order, all rows distinct.
"""
import numpy as np

GRID = 468            # pillars per axis
CELL = 0.32           # metres per pillar
HALF = 74.88          # half extent in metres (GRID * CELL / 2)
MEAN_RANGE = 20.0     # mean of the exponential radial law, metres
N_CLUSTERS = 50       # Gaussian object clusters per frame
CLUSTER_SIGMA = 1.0   # metres
CLUSTER_FRACTION = 0.2
CHUNK = 8192


def _first_occurrence_unique(cells, have, order, target):
    """Append unseen cell ids from `cells` (in order) to `order` until target."""
    _, first = np.unique(cells, return_index=True)
    first.sort()
    for c in cells[first]:
        c = int(c)
        if c not in have:
            have.add(c)
            order.append(c)
            if len(order) >= target:
                return True
    return False


def unique_uniform_cells(n, grid, seed):
    """n distinct cells drawn uniformly on a grid x grid board, b = 0."""
    if n > grid * grid:
        raise ValueError("more cells requested than the grid holds")
    rng = np.random.default_rng(seed)
    have, order = set(), []
    while len(order) < n:
        x = rng.integers(0, grid, size=CHUNK)
        y = rng.integers(0, grid, size=CHUNK)
        if _first_occurrence_unique(x * grid + y, have, order, n):
            break
    ids = np.asarray(order[:n], dtype=np.int64)
    out = np.zeros((n, 3), dtype=np.int32)
    out[:, 1] = ids // grid
    out[:, 2] = ids % grid
    return out


def _lidar_cells(rng, centres, x_offset):
    """One chunk of raw points -> in-range cell ids (row-major id = x*GRID+y)."""
    is_obj = rng.random(CHUNK) < CLUSTER_FRACTION
    r = rng.exponential(MEAN_RANGE, size=CHUNK)
    th = rng.uniform(0.0, 2.0 * np.pi, size=CHUNK)
    px = r * np.cos(th)
    py = r * np.sin(th)
    which = rng.integers(0, N_CLUSTERS, size=CHUNK)
    jitter = rng.normal(0.0, CLUSTER_SIGMA, size=(CHUNK, 2))
    px = np.where(is_obj, centres[which, 0] + jitter[:, 0], px) + x_offset
    py = np.where(is_obj, centres[which, 1] + jitter[:, 1], py)
    keep = (px >= -HALF) & (px < HALF) & (py >= -HALF) & (py < HALF)
    cx = np.floor((px[keep] + HALF) / CELL).astype(np.int64)
    cy = np.floor((py[keep] + HALF) / CELL).astype(np.int64)
    keep2 = (cx >= 0) & (cx < GRID) & (cy >= 0) & (cy < GRID)
    return cx[keep2] * GRID + cy[keep2]


def lidar_frame(seed, target, x_offset=0.0, b=0):
    """`target` distinct pillars of one synthetic LiDAR frame.

    Background returns have range ~ Exponential(mean 20 m) and uniform azimuth;
    one point in five belongs to one of 50 Gaussian object clusters (sigma 1 m)
    whose centres follow the same radial law.  `x_offset` (metres) moves the
    whole frame along x before quantisation (ego motion between sweeps).
    """
    rng = np.random.default_rng(seed)
    cr = rng.exponential(MEAN_RANGE, size=N_CLUSTERS)
    ct = rng.uniform(0.0, 2.0 * np.pi, size=N_CLUSTERS)
    centres = np.stack([cr * np.cos(ct), cr * np.sin(ct)], axis=1)
    have, order = set(), []
    while len(order) < target:
        if _first_occurrence_unique(_lidar_cells(rng, centres, x_offset),
                                    have, order, target):
            break
    ids = np.asarray(order[:target], dtype=np.int64)
    out = np.empty((target, 3), dtype=np.int32)
    out[:, 0] = b
    out[:, 1] = ids // GRID
    out[:, 2] = ids % GRID
    return out


def merged_sweep(seeds, offsets_m, per_frame, total):
    """Several frames with ego offsets merged into one cloud (b = 0), duplicates
    removed keeping the first occurrence, cut to exactly `total` pillars."""
    parts = [lidar_frame(s, per_frame, x_offset=o) for s, o in zip(seeds, offsets_m)]
    allc = np.concatenate(parts, axis=0)
    ids = allc[:, 1].astype(np.int64) * GRID + allc[:, 2]
    _, first = np.unique(ids, return_index=True)
    first.sort()
    if first.size < total:
        raise ValueError(f"union has only {first.size} pillars, need {total}")
    return np.ascontiguousarray(allc[first[:total]])


def frame_batch(seeds, targets, shuffle_seed):
    """Independent frames, b = frame index, rows globally shuffled so that a
    sort really has to separate the frames."""
    parts = [lidar_frame(s, t, b=i) for i, (s, t) in enumerate(zip(seeds, targets))]
    allc = np.concatenate(parts, axis=0)
    rng = np.random.default_rng(shuffle_seed)
    return np.ascontiguousarray(allc[rng.permutation(allc.shape[0])])


def row_major_order(coords):
    """The same pillars in (b, x, y) row-major order: the order a voxeliser's
    `unique` would emit.  Input-order variant for locality measurements."""
    idx = np.lexsort((coords[:, 2], coords[:, 1], coords[:, 0]))
    return np.ascontiguousarray(coords[idx])


def lidar_points(seed, m, num_frames=1, feat_dim=4):
    """Raw points of synthetic LiDAR frames, before any voxelisation: (xy float32 [m, 2] in metres,
    frame int32 [m], point features float32 [m, feat_dim]).  Same spatial law as `lidar_frame`
    (exponential range, uniform azimuth, one point in five in one of 50 Gaussian clusters), a few
    percent of the points fall outside +-74.88 m.  The features are N(0, 1) stand-ins for height,
    intensity and the like."""
    rng = np.random.default_rng(seed)
    frame = rng.integers(0, num_frames, size=m).astype(np.int32)
    cr = rng.exponential(MEAN_RANGE, size=(num_frames, N_CLUSTERS))
    ct = rng.uniform(0.0, 2.0 * np.pi, size=(num_frames, N_CLUSTERS))
    centres = np.stack([cr * np.cos(ct), cr * np.sin(ct)], axis=2)          # [frames, clusters, 2]
    is_obj = rng.random(m) < CLUSTER_FRACTION
    r = rng.exponential(MEAN_RANGE, size=m)
    th = rng.uniform(0.0, 2.0 * np.pi, size=m)
    which = rng.integers(0, N_CLUSTERS, size=m)
    jitter = rng.normal(0.0, CLUSTER_SIGMA, size=(m, 2))
    px = np.where(is_obj, centres[frame, which, 0] + jitter[:, 0], r * np.cos(th))
    py = np.where(is_obj, centres[frame, which, 1] + jitter[:, 1], r * np.sin(th))
    xy = np.stack([px, py], axis=1).astype(np.float32)
    feats = rng.standard_normal((m, feat_dim)).astype(np.float32)
    return xy, frame, feats
