"""Oracle for window-based sorting and equal-size grouping (paper Sec. 4.2.1).

TEST INFRASTRUCTURE ONLY -- see the package docstring.

Everything is done with Python integers and an explicit tuple comparison; the
packed 64-bit key is produced separately so that the packing itself is checked
against the tuple order rather than assumed.
"""
from collections import namedtuple
import numpy as np

# B frames; coords[:,0] in [0,B), coords[:,1] in [0,grid_x), coords[:,2] in [0,grid_y)
Geometry = namedtuple("Geometry", "num_frames grid_x grid_y win_x win_y")


def shift_amount(w, shift):
    """Window shift (Sec. 4.2.2 'Window Shift'): translate by half a window.
    Integer coordinates and odd windows: floor(w / 2), added, so coordinates
    stay non-negative."""
    return (w // 2) if shift else 0


def window_tuple(b, x, y, geom, axis, shift):
    """Eq. (1): (window coords, local coords) of one pillar, batch index first.

    axis 0: x has priority  -> (b, Wx, Wy, Lx, Ly)
    axis 1: y has priority  -> (b, Wy, Wx, Ly, Lx)   ('Alternate Sorting Axis')
    """
    X = int(x) + shift_amount(geom.win_x, shift)
    Y = int(y) + shift_amount(geom.win_y, shift)
    Wx = X // geom.win_x
    Wy = Y // geom.win_y
    Lx = X - Wx * geom.win_x
    Ly = Y - Wy * geom.win_y
    if axis == 0:
        return (int(b), Wx, Wy, Lx, Ly)
    return (int(b), Wy, Wx, Ly, Lx)


def pack_key(t):
    """Canonical 64-bit key: fields 16 | 16 | 16 | 8 | 8 bits, most significant
    first, so that integer order equals tuple order."""
    b, w1, w2, l1, l2 = t
    if not (0 <= b < 1 << 16 and 0 <= w1 < 1 << 16 and 0 <= w2 < 1 << 16
            and 0 <= l1 < 1 << 8 and 0 <= l2 < 1 << 8):
        raise OverflowError("key field out of range: %r" % (t,))
    return (b << 48) | (w1 << 32) | (w2 << 16) | (l1 << 8) | l2


def sort_tuple_order(tuples):
    """Stable ascending order of the tuples; ties broken by original index."""
    return sorted(range(len(tuples)), key=lambda i: (tuples[i], i))


def frame_segments(sorted_b, num_frames):
    """[start, end) of each frame in an array of non-decreasing frame ids."""
    segs = []
    pos = 0
    n = len(sorted_b)
    for b in range(num_frames):
        start = pos
        while pos < n and sorted_b[pos] == b:
            pos += 1
        segs.append((start, pos))
    if pos != n:
        raise ValueError("frame ids not sorted or out of range")
    return segs


def flatten(coords, geom, axis, shift, G, tail="mask"):
    """Sort pillars by their window tuple and cut each frame's sorted run into
    consecutive groups of G ('Equal-Size Grouping').

    Returns (perm int32 [n], group_offsets int32 [num_groups+1], keys_sorted uint64 [n]).
    perm[p] is the original index of the pillar at sorted position p.  Groups
    never cross frames; only a frame's last group may have fewer than G members
    (tail == "mask").  With tail == "drop" ('Drop Residual') those short groups
    are left out of the list: the result is then (perm, group_starts, keys)
    where group_starts lists only full groups and there is no closing entry.
    """
    coords = np.asarray(coords)
    n = coords.shape[0]
    tuples = [window_tuple(coords[i, 0], coords[i, 1], coords[i, 2], geom, axis, shift)
              for i in range(n)]
    order = sort_tuple_order(tuples)
    perm = np.asarray(order, dtype=np.int32).reshape(n)
    keys = np.asarray([pack_key(tuples[i]) for i in order], dtype=np.uint64).reshape(n)
    sorted_b = [tuples[i][0] for i in order]
    offsets = []
    for (s, e) in frame_segments(sorted_b, geom.num_frames):
        p = s
        while p < e:
            if tail == "drop" and e - p < G:
                break
            offsets.append(p)
            p += G
    if tail == "mask":
        offsets.append(n)
    elif tail != "drop":
        raise ValueError(tail)
    return perm, np.asarray(offsets, dtype=np.int32), keys


# ---- three-dimensional windows (footnote of Sec. 4.2.1: the method applies to 3-D point clouds) --------
# coords[:, 0] frame, coords[:, 1..3] = (x, y, z) voxel indices
Geometry3 = namedtuple("Geometry3", "num_frames grid_x grid_y grid_z win_x win_y win_z")


def window_tuple3(b, x, y, z, geom, axis, shift):
    """Eq. (1) with a third coordinate: window coordinates, then local coordinates.  The paper
    states the 3-D case in a footnote only; the reading taken keeps the two-axis alternation of
    the BEV case and appends z to both halves of the tuple:

    axis 0 -> (b, Wx, Wy, Wz, Lx, Ly, Lz)       axis 1 -> (b, Wy, Wx, Wz, Ly, Lx, Lz)
    """
    X = int(x) + shift_amount(geom.win_x, shift)
    Y = int(y) + shift_amount(geom.win_y, shift)
    Z = int(z) + shift_amount(geom.win_z, shift)
    Wx, Wy, Wz = X // geom.win_x, Y // geom.win_y, Z // geom.win_z
    Lx, Ly, Lz = X - Wx * geom.win_x, Y - Wy * geom.win_y, Z - Wz * geom.win_z
    if axis == 0:
        return (int(b), Wx, Wy, Wz, Lx, Ly, Lz)
    return (int(b), Wy, Wx, Wz, Ly, Lx, Lz)


def flatten3d(coords, geom, axis, shift, G, tail="mask"):
    """`flatten` for voxels with coordinates (b, x, y, z).  Returns (perm, group_offsets); the
    packed 64-bit key of the BEV case has no room for seven fields and is not produced."""
    coords = np.asarray(coords)
    n = coords.shape[0]
    tuples = [window_tuple3(*coords[i], geom, axis, shift) for i in range(n)]
    order = sort_tuple_order(tuples)
    perm = np.asarray(order, dtype=np.int32).reshape(n)
    sorted_b = [tuples[i][0] for i in order]
    offsets = []
    for (s, e) in frame_segments(sorted_b, geom.num_frames):
        p = s
        while p < e:
            if tail == "drop" and e - p < G:
                break
            offsets.append(p)
            p += G
    if tail == "mask":
        offsets.append(n)
    elif tail != "drop":
        raise ValueError(tail)
    return perm, np.asarray(offsets, dtype=np.int32)
