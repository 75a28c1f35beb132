"""Helpers shared by the GPU parity tests (not a test module)."""
import numpy as np
import torch

import ffsynth
import oracle
import paper_2301_08739_amd as ff

DEV = "cuda"


def geoms(c):
    return (ff.Geometry(c["B"], c["grid"], c["grid"], c["window"], c["window"]),
            oracle.Geometry(c["B"], c["grid"], c["grid"], c["window"], c["window"]))


def to_dev_feats(feats, dtype):
    t = torch.from_numpy(np.ascontiguousarray(feats, dtype=np.float32))
    return t.to(DEV).to({ff.FF_F32: torch.float32, ff.FF_BF16: torch.bfloat16, ff.FF_F16: torch.float16}[dtype])


def to_host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def dtype_of(c):
    return ff.FF_F32 if c["dtype"] == "f32" else ff.FF_BF16


def gpu_flatten(coords, g, axis, shift, G, want_keys=True, tail=ff.FF_TAIL_MASK):
    """(perm, group_offsets[:num_groups + 1], num_groups, keys, device tensors), on the host."""
    ct = torch.from_numpy(np.ascontiguousarray(coords, dtype=np.int32)).to(DEV)
    perm, goff, ng, keys = ff.ff_flatten(ct, g, axis, shift, G, tail=tail, want_keys=want_keys)
    torch.cuda.synchronize()
    k = int(ng.item())
    return (perm.cpu().numpy(), goff.cpu().numpy()[:k + 1], k,
            None if keys is None else keys.cpu().numpy().view(np.uint64), (perm, goff, ng))


def bf16_half_ulp(y):
    """Largest error of rounding to nearest bf16 at magnitude |y|: half a unit in the last place of an 8-bit
    significand, 2^(e-8) for 2^e <= |y| < 2^(e+1) (0.0156 on [4, 8), 0.031 on [8, 16)); between |y| / 512 at the
    top of a binade and |y| / 256 at its bottom."""
    a = np.abs(np.asarray(y, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -126)))
    return np.ldexp(1.0, (e - 8).astype(np.int64))


def assert_bf16_bar(wide, narrow, want, rows=None):
    """The bf16 bar of the layer tests: (a) the result before storage rounding within 2e-2 of the oracle
    everywhere, (c) the bf16 buffer within 2e-2 + half an ulp of the stored value everywhere and within plain
    2e-2 where |reference| < 2.  ((b), buffer == RNE(wide), is asserted by the caller that produced both.)
    Returns (max error of wide, max error of narrow)."""
    if rows is not None:
        wide, narrow, want = wide[rows], narrow[rows], want[rows]
    e_wide = np.abs(wide - want).max()
    assert e_wide <= 2e-2, e_wide
    err = np.abs(narrow - want)
    assert np.all(err <= 2e-2 + bf16_half_ulp(narrow))
    small = np.abs(want) < 2.0
    assert err[small].max() <= 2e-2, err[small].max()
    return e_wide, err.max()
