"""GPU parity for IEEE half storage (FF_F16, the paper's inference precision): the fused kernel and
the plain kernels against the oracle on inputs rounded to half precision once.

Tolerance: the error model is the one of the bf16 path (operands of every product rounded to the
storage type, fp32 accumulation), with a unit roundoff of 2^-11 instead of 2^-8, so the bf16 bar of
2e-2 scales to 2.5e-3.  The stored half buffer must be the round-to-nearest-even of the fp32-stored
result, bit for bit."""
import numpy as np
import pytest
import torch

import ffsynth
import oracle
import paper_2301_08739_amd as ff
from gpu_util import DEV, geoms, gpu_flatten, to_dev_feats, to_host

pytestmark = pytest.mark.gpu

TOL = 2.5e-3
F16 = ff.FF_F16


def _half_params(p):
    q = dict(p)
    for k, v in p.items():
        if isinstance(v, np.ndarray):
            q[k] = ffsynth.f16_round(v)
    return q


def _case(c, n):
    return c["coords"][:n], ffsynth.f16_round(c["feats"][:n]), _half_params(c["layer_params"][0])


def _check(wide, narrow, want, what):
    err = np.abs(wide - want).max()
    print(f"{what}: max abs err {err:.3e} (max |ref| {np.abs(want).max():.2f})", flush=True)
    assert err <= TOL, (what, err)
    assert np.array_equal(ffsynth.f16_round(wide.astype(np.float32)).astype(np.float64), narrow), what


@pytest.mark.parametrize("i,G,variants", [(2, 32, (0, 1, 10)), (2, 64, (0, 2, 6, 7, 11, 12)), (2, 100, (0, 4, 9)),
                                          (5, 64, (0, 2, 5)), (5, 69, (0, 3, 6)), (5, 128, (0, 4))])
def test_fused_kernel_mappings(cfg, i, G, variants):
    c = cfg(i, 1)
    coords, feats, p = _case(c, 1003)
    g, og = geoms(c)
    perm, off, ng, _, dev = gpu_flatten(coords, g, 1, 1, G, want_keys=False)
    want = oracle.layer(feats, perm, off, p)
    lw = ff.LayerWeights(p, F16, DEV)
    x = to_dev_feats(feats, F16)
    for v in variants:
        fl = ff.FF_FLAG_VARIANT(v)
        wide = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], ng + 1, lw, G, F16, fl | ff.FF_FLAG_OUT_F32))
        narrow = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], ng + 1, lw, G, F16, fl))
        _check(wide, narrow, want, f"fp16 cfg{i} G={G} variant {v}")
    lw.pack()
    packed = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], ng + 1, lw, G, F16, 0))
    assert np.array_equal(packed, narrow if variants[-1] == 0 else
                          to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], ng + 1, ff.LayerWeights(p, F16, DEV), G, F16, 0)))
    plain = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], ng + 1, lw, G, F16,
                                          ff.FF_FLAG_OUT_F32 | ff.FF_FLAG_FORCE_GENERIC))
    assert np.abs(plain - want).max() <= TOL


def test_config2_every_layer_teacher_forced(cfg):
    c = cfg(2, 4)
    g, og = geoms(c)
    cur = ffsynth.f16_round(c["feats"])
    for l, key in enumerate(c["schedule"]):
        p = _half_params(c["layer_params"][l])
        perm, off, ng, _, dev = gpu_flatten(c["coords"], g, key[0], key[1], c["G"], want_keys=False)
        lw = ff.LayerWeights(p, F16, DEV)
        x = to_dev_feats(cur, F16)
        mg = -(-c["n"] // c["G"]) + c["B"]
        wide = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], mg, lw, c["G"], F16, ff.FF_FLAG_OUT_F32))
        narrow = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], mg, lw, c["G"], F16, 0))
        want = oracle.layer(cur, perm, off, p)
        _check(wide, narrow, want, f"fp16 cfg2 layer {l} sort {key}")
        cur = ffsynth.f16_round(want.astype(np.float32))


def test_drop_and_positional_embedding(cfg):
    c = cfg(2, 1)
    coords, feats, p = _case(c, 1003)
    g, og = geoms(c)
    G = 64
    pe = ffsynth.f16_round(0.5 * np.random.default_rng(21).standard_normal(feats.shape).astype(np.float32))
    lw = ff.LayerWeights(p, F16, DEV)
    x, pe_d = to_dev_feats(feats, F16), to_dev_feats(pe, F16)
    perm, starts, _ = oracle.flatten(coords, og, 0, 1, G, tail="drop")
    dperm, dgoff, dng, _ = ff.ff_flatten(torch.from_numpy(coords).to(DEV), g, 0, 1, G, tail=ff.FF_TAIL_DROP)
    want = oracle.layer(feats, perm, starts, p, group_size=G, pos_embed=pe)
    for fl in (0, ff.FF_FLAG_FORCE_GENERIC):
        wide = to_host(ff.ff_group_attention(x, dperm, dgoff, dng, 1003 // G, lw, G, F16,
                                             fl | ff.FF_FLAG_OUT_F32 | ff.FF_FLAG_TAIL_DROP, pos_embed=pe_d))
        narrow = to_host(ff.ff_group_attention(x, dperm, dgoff, dng, 1003 // G, lw, G, F16,
                                               fl | ff.FF_FLAG_TAIL_DROP, pos_embed=pe_d))
        _check(wide, narrow, want, f"fp16 drop + pos embed flags {fl}")
        skipped = np.ones(1003, bool)
        for s0 in starts:
            skipped[perm[s0:s0 + G]] = False
        assert skipped.sum() == 1003 % G and np.array_equal(narrow[skipped], feats[skipped].astype(np.float64))


def test_block_and_rows(cfg):
    c = cfg(2, 4)
    g, og = geoms(c)
    ct = torch.from_numpy(c["coords"]).to(DEV)
    layers = [ff.LayerWeights(_half_params(p), F16, DEV) for p in c["layer_params"]]
    x = to_dev_feats(ffsynth.f16_round(c["feats"]), F16)
    out = ff.ff_fwa_block(ct, g, c["G"], layers, F16, x)
    cur = x
    for l, key in enumerate(c["schedule"]):
        perm, goff, ng, _ = ff.ff_flatten(ct, g, key[0], key[1], c["G"])
        cur = ff.ff_group_attention(cur, perm, goff, ng, -(-c["n"] // c["G"]) + c["B"], layers[l], c["G"], F16)
    torch.cuda.synchronize()
    assert out.dtype == torch.float16 and torch.equal(out, cur) and torch.isfinite(out).all()
    gth = ff.ff_gather(x, perm, F16)
    assert torch.equal(gth, x[perm.long()]) and torch.equal(ff.ff_scatter(gth, perm, F16), x)


@pytest.mark.parametrize("i", [4, 5])
def test_full_size_sampled_groups_all_options(cfg, i):
    """Full-size configurations with every option at once (half storage, dropped short groups,
    positional embedding), in the launch configuration bench.py times: sampled groups against the
    oracle one by one, skipped rows exact, everything finite."""
    c = cfg(i, 1)
    g, og = geoms(c)
    n, G = c["n"], c["G"]
    feats = ffsynth.f16_round(c["feats"])
    p = _half_params(c["layer_params"][0])
    pe = ffsynth.f16_round(0.5 * np.random.default_rng(40 + i).standard_normal(feats.shape).astype(np.float32))
    ct = torch.from_numpy(c["coords"]).to(DEV)
    perm_d, goff_d, ng_d, _ = ff.ff_flatten(ct, g, 1, 1, G, tail=ff.FF_TAIL_DROP)
    torch.cuda.synchronize()
    ng = int(ng_d.item())
    perm, starts = perm_d.cpu().numpy(), goff_d.cpu().numpy()[:ng]
    lw = ff.LayerWeights(p, F16, DEV).pack()
    x, pe_d = to_dev_feats(feats, F16), to_dev_feats(pe, F16)
    mg = n // G + c["B"]
    wide = to_host(ff.ff_group_attention(x, perm_d, goff_d, ng_d, mg, lw, G, F16,
                                         ff.FF_FLAG_OUT_F32 | ff.FF_FLAG_TAIL_DROP, pos_embed=pe_d))
    narrow = to_host(ff.ff_group_attention(x, perm_d, goff_d, ng_d, mg, lw, G, F16, ff.FF_FLAG_TAIL_DROP, pos_embed=pe_d))
    pick = sorted(set([0, 1, ng // 2, ng - 1] + np.random.default_rng(i).integers(0, ng, 12).tolist()))
    rows = np.concatenate([perm[starts[k]:starts[k] + G] for k in pick])
    want = oracle.layer(feats, perm, starts[pick], p, groups=range(len(pick)), group_size=G, pos_embed=pe)
    err = np.abs(wide[rows] - want[rows]).max()
    grouped = np.zeros(n, bool)
    for s0 in starts:
        grouped[perm[s0:s0 + G]] = True
    print(f"cfg{i} fp16 + drop + pos embed: {len(pick)} of {ng} groups, {int((~grouped).sum())} rows skipped, "
          f"max abs err {err:.3e}", flush=True)
    assert err <= TOL
    assert np.array_equal(ffsynth.f16_round(wide.astype(np.float32)).astype(np.float64), narrow)
    assert np.array_equal(narrow[~grouped], feats[~grouped].astype(np.float64)) and np.isfinite(narrow).all()
