"""GPU: the fused matrix-core layer at its third shape, (C, head dim, F) = (64, 16, 128) — configuration 1's
layer in 16-bit storage — against the oracle (Eq. (2)), over group sizes with short tails, and the host-side
query that tells which kernels a call takes."""
import numpy as np
import pytest
import torch

import ffsynth
import oracle
import paper_2301_08739_amd as ff
from gpu_util import DEV, assert_bf16_bar, geoms, gpu_flatten, to_dev_feats, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("G", [1, 7, 32, 33, 64, 100, 128])
def test_narrow_layer_bf16_and_f16(cfg, G):
    c = dict(cfg(1, 1))
    n = 1003
    coords = np.ascontiguousarray(c["coords"][:n])
    g, _ = geoms(c)
    perm, off, ng, _, dev = gpu_flatten(coords, g, 1, 1, G, want_keys=False)
    mg = -(-n // G) + 1
    for dt, rnd, tol in ((ff.FF_BF16, ffsynth.bf16_round, 2e-2), (ff.FF_F16, ffsynth.f16_round, 2.5e-3)):
        p = ffsynth.stack_params(64, 128, 4, 1, bf16=False)[0]
        p = {k: (rnd(np.asarray(v, dtype=np.float32)) if isinstance(v, np.ndarray) else v) for k, v in p.items()}
        feats = rnd(np.random.default_rng(5).standard_normal((n, 64)).astype(np.float32))
        want = oracle.layer(feats, perm, off, p)
        lw = ff.LayerWeights(p, dt, DEV)
        assert ff.ff_group_attention_path(lw, G, dt) == ff.FF_PATH_FUSED
        x = to_dev_feats(feats, dt)
        wide = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], mg, lw, G, dt, ff.FF_FLAG_OUT_F32))
        narrow = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], mg, lw, G, dt, 0))
        plain = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], mg, lw, G, dt,
                                              ff.FF_FLAG_OUT_F32 | ff.FF_FLAG_FORCE_GENERIC))
        err = np.abs(wide - want).max()
        print(f"narrow layer G={G} dtype={dt}: fused max abs err {err:.3e}, plain kernels {np.abs(plain - want).max():.3e}",
              flush=True)
        assert err <= tol
        assert np.abs(plain - want).max() <= tol
        assert np.array_equal(rnd(wide.astype(np.float32)).astype(np.float64), narrow)
        if dt == ff.FF_BF16:
            assert_bf16_bar(wide, narrow, want)


def test_narrow_block_equals_layer_calls(cfg):
    """Configuration 1 (two layers, x then y) with bf16 storage through ff_fwa_block, chained in sorted order."""
    c = cfg(1)
    g, _ = geoms(c)
    params = ffsynth.stack_params(64, 128, 4, 2, bf16=True)
    layers = [ff.LayerWeights(p, ff.FF_BF16, DEV) for p in params]
    ct = torch.from_numpy(c["coords"]).to(DEV)
    x = to_dev_feats(ffsynth.bf16_round(c["feats"]), ff.FF_BF16)
    out = ff.ff_fwa_block(ct, g, c["G"], layers, ff.FF_BF16, x)
    cur = x
    for l, key in enumerate(c["schedule"]):
        perm, goff, ng, _ = ff.ff_flatten(ct, g, key[0], key[1], c["G"])
        cur = ff.ff_group_attention(cur, perm, goff, ng, -(-c["n"] // c["G"]) + 1, layers[l], c["G"], ff.FF_BF16)
    torch.cuda.synchronize()
    assert torch.equal(out, cur)


def test_path_query():
    mk = lambda C, F, h: ff.LayerWeights(ffsynth.layer_params(C, F, h, seed=3), ff.FF_BF16, DEV)
    a, b, c3, odd = mk(128, 256, 8), mk(256, 512, 8), mk(64, 128, 4), mk(96, 160, 3)
    for lw in (a, b, c3):
        assert ff.ff_group_attention_path(lw, 64, ff.FF_BF16) == ff.FF_PATH_FUSED
        assert ff.ff_group_attention_path(lw, 128, ff.FF_F16) == ff.FF_PATH_FUSED
        assert ff.ff_group_attention_path(lw, 129, ff.FF_BF16) == ff.FF_PATH_PLAIN           # groups beyond 128
        assert ff.ff_group_attention_path(lw, 64, ff.FF_BF16, ff.FF_FLAG_FORCE_GENERIC) == ff.FF_PATH_PLAIN
    assert ff.ff_group_attention_path(odd, 64, ff.FF_BF16) == ff.FF_PATH_PLAIN               # no fused instantiation
    assert ff.ff_group_attention_path(mk(128, 512, 8), 64, ff.FF_BF16) == ff.FF_PATH_PLAIN
    f32 = ff.LayerWeights(ffsynth.layer_params(128, 256, 8, seed=3), ff.FF_F32, DEV)
    assert ff.ff_group_attention_path(f32, 64, ff.FF_F32) == ff.FF_PATH_PLAIN
    with pytest.raises(ff.FlatformerError):
        ff.ff_group_attention_path(a, 0, ff.FF_BF16)
    with pytest.raises(ff.FlatformerError):
        ff.ff_group_attention_path(a, 2000, ff.FF_BF16)
