"""GPU: ff_flatten_noalloc (the sort on the library's static scratch array, for callers that cannot allocate)
gives exactly what ff_flatten gives, on two calls in a row, the second with a smaller cloud, and again after
a larger one; a cloud beyond the array is refused with a status code."""
import numpy as np
import pytest
import torch

import paper_2301_08739_amd as ff
from gpu_util import DEV, geoms

pytestmark = pytest.mark.gpu


def _both(coords, g, axis, shift, G, tail):
    ct = torch.from_numpy(np.ascontiguousarray(coords, dtype=np.int32)).to(DEV)
    n = ct.shape[0]
    want = ff.ff_flatten(ct, g, axis, shift, G, tail=tail, want_keys=True)
    cap = -(-n // G) + g.num_frames + 1
    perm = torch.full((n,), -7, dtype=torch.int32, device=DEV)
    goff = torch.full((cap,), -1, dtype=torch.int32, device=DEV)
    ng = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    keys = torch.full((n,), -7, dtype=torch.int64, device=DEV)
    ff.ff_flatten_noalloc(ct, g, axis, shift, G, perm, goff, ng, keys=keys, tail=tail)
    torch.cuda.synchronize()
    k = int(ng.item())
    assert k == int(want[2].item())
    assert torch.equal(perm, want[0])
    assert torch.equal(goff[:k + 1], want[1][:k + 1])
    assert torch.equal(keys, want[3])
    return k


def test_noalloc_flatten_equals_flatten_on_consecutive_calls(cfg):
    big, small = cfg(5, 1), cfg(2, 1)
    gb, _ = geoms(big)
    gs, _ = geoms(small)
    print("noalloc: config 5 cloud, 240000 pillars, 8 frames, G=69", flush=True)
    _both(big["coords"], gb, 0, 1, big["G"], ff.FF_TAIL_MASK)
    print("noalloc: config 2 cloud, 30000 pillars, G=64 (smaller, right after)", flush=True)
    _both(small["coords"], gs, 1, 0, small["G"], ff.FF_TAIL_MASK)
    print("noalloc: 1003 pillars, dropped tails", flush=True)
    _both(small["coords"][:1003], gs, 1, 1, 64, ff.FF_TAIL_DROP)
    print("noalloc: config 5 cloud again, other axis", flush=True)
    _both(big["coords"], gb, 1, 0, big["G"], ff.FF_TAIL_MASK)
    print("noalloc: empty cloud", flush=True)
    _both(small["coords"][:0], gs, 0, 0, 64, ff.FF_TAIL_MASK)


def test_noalloc_flatten_refuses_what_does_not_fit(cfg):
    c = cfg(2, 1)
    g, _ = geoms(c)
    n = 600000                      # needs more than FF_NOALLOC_SCRATCH_BYTES of scratch
    assert ff.ff_flatten_workspace_bytes(n, g) > ff.FF_NOALLOC_SCRATCH_BYTES
    rng = np.random.default_rng(3)
    coords = np.zeros((n, 3), dtype=np.int32)
    coords[:, 1:] = rng.integers(0, c["grid"], size=(n, 2))
    ct = torch.from_numpy(coords).to(DEV)
    perm = torch.full((n,), -7, dtype=torch.int32, device=DEV)
    goff = torch.full((n // 64 + 3,), -1, dtype=torch.int32, device=DEV)
    ng = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    with pytest.raises(ff.FlatformerError, match="unsupported"):
        ff.ff_flatten_noalloc(ct, g, 0, 0, 64, perm, goff, ng)
    torch.cuda.synchronize()
    assert int(ng.item()) == -1 and int(perm[0].item()) == -7                  # nothing was written
