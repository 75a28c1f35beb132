"""GPU parity for the positional-embedding input of Eq. (2): queries and keys from LN(F) + PE,
values from LN(F); plain fp32 kernels and the fused bf16 kernel against the oracle."""
import numpy as np
import pytest
import torch

import ffsynth
import oracle
import paper_2301_08739_amd as ff
from gpu_util import DEV, dtype_of, geoms, gpu_flatten, to_dev_feats, to_host

pytestmark = pytest.mark.gpu


def _pe(shape, seed, bf16):
    pe = 0.5 * np.random.default_rng(seed).standard_normal(shape).astype(np.float32)
    return ffsynth.bf16_round(pe).astype(np.float32) if bf16 else pe


def test_fp32_layers_and_block(cfg):
    c = cfg(1)
    g, og = geoms(c)
    pe = _pe(c["feats"].shape, 11, False)
    perms, offs = {}, {}
    for key in set(c["schedule"]):
        perms[key], offs[key], _ = oracle.flatten(c["coords"], og, key[0], key[1], c["G"])
    trace = oracle.stack(c["feats"], perms, offs, c["layer_params"], c["schedule"], pos_embed=pe)
    pe_d = to_dev_feats(pe, ff.FF_F32)
    for l, key in enumerate(c["schedule"]):
        perm, off, ng, _, dev = gpu_flatten(c["coords"], g, key[0], key[1], c["G"], want_keys=False)
        lw = ff.LayerWeights(c["layer_params"][l], ff.FF_F32, DEV)
        got = to_host(ff.ff_group_attention(to_dev_feats(trace[l].astype(np.float32), ff.FF_F32), dev[0], dev[1], dev[2],
                                            ng + 1, lw, c["G"], ff.FF_F32, pos_embed=pe_d))
        want = oracle.layer(trace[l].astype(np.float32), perm, off, c["layer_params"][l], pos_embed=pe)
        assert np.abs(got - want).max() <= 1e-4
        assert np.abs(want - oracle.layer(trace[l].astype(np.float32), perm, off, c["layer_params"][l])).max() > 1e-2
    layers = [ff.LayerWeights(p, ff.FF_F32, DEV) for p in c["layer_params"]]
    out = ff.ff_fwa_block(torch.from_numpy(c["coords"]).to(DEV), g, c["G"], layers, ff.FF_F32,
                          to_dev_feats(c["feats"], ff.FF_F32), pos_embed=pe_d)
    torch.cuda.synchronize()
    assert np.abs(to_host(out) - trace[-1]).max() <= 1e-4


@pytest.mark.parametrize("i,G,variants", [(2, 32, (0, 10)), (2, 64, (0, 2, 6, 7, 12)), (2, 100, (0, 4, 9)),
                                          (5, 64, (0, 2, 5)), (5, 69, (0, 6)), (5, 128, (0, 4))])
def test_bf16_fused_kernel(cfg, i, G, variants):
    c = dict(cfg(i, 1))
    n = 1003
    c["coords"], feats = c["coords"][:n], c["feats"][:n]
    p = c["layer_params"][0]
    g, og = geoms(c)
    pe = _pe(feats.shape, 12 + G, True)
    perm, off, ng, _, dev = gpu_flatten(c["coords"], g, 1, 1, G, want_keys=False)
    want = oracle.layer(feats, perm, off, p, pos_embed=pe)
    lw = ff.LayerWeights(p, ff.FF_BF16, DEV).pack()
    x, pe_d = to_dev_feats(feats, ff.FF_BF16), to_dev_feats(pe, ff.FF_BF16)
    for v in variants:
        print(f"pos embed cfg{i} G={G} variant {v}", flush=True)
        fl = ff.FF_FLAG_VARIANT(v)
        wide = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], ng + 1, lw, G, ff.FF_BF16,
                                             fl | ff.FF_FLAG_OUT_F32, pos_embed=pe_d))
        narrow = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], ng + 1, lw, G, ff.FF_BF16, fl, pos_embed=pe_d))
        err = np.abs(wide - want).max()
        assert err <= 2e-2, (v, err)
        assert np.array_equal(ffsynth.bf16_round(wide.astype(np.float32)).astype(np.float64), narrow)
    plain = to_host(ff.ff_group_attention(x, dev[0], dev[1], dev[2], ng + 1, lw, G, ff.FF_BF16,
                                          ff.FF_FLAG_OUT_F32 | ff.FF_FLAG_FORCE_GENERIC, pos_embed=pe_d))
    assert np.abs(plain - want).max() <= 2e-2
    assert np.abs(want - oracle.layer(feats, perm, off, p)).max() > 1e-2      # the embedding matters here


def test_mappings_without_registers_for_the_embedding_refuse(cfg):
    c = dict(cfg(2, 1))
    n = 500
    c["coords"], feats = c["coords"][:n], c["feats"][:n]
    g, og = geoms(c)
    perm, off, ng, _, dev = gpu_flatten(c["coords"], g, 0, 0, 32, want_keys=False)
    lw = ff.LayerWeights(c["layer_params"][0], ff.FF_BF16, DEV)
    x = to_dev_feats(feats, ff.FF_BF16)
    with pytest.raises(ff.FlatformerError):
        ff.ff_group_attention(x, dev[0], dev[1], dev[2], ng + 1, lw, 32, ff.FF_BF16, ff.FF_FLAG_VARIANT(1), pos_embed=x)
    with pytest.raises(ff.FlatformerError):                                   # three groups per workgroup: 168 registers
        ff.ff_group_attention(x, dev[0], dev[1], dev[2], ng + 1, lw, 32, ff.FF_BF16, ff.FF_FLAG_VARIANT(11), pos_embed=x)


def test_bf16_block_matches_layer_calls(cfg):
    c = cfg(2, 4)
    g, og = geoms(c)
    ct = torch.from_numpy(c["coords"]).to(DEV)
    layers = [ff.LayerWeights(p, ff.FF_BF16, DEV) for p in c["layer_params"]]
    x = to_dev_feats(c["feats"], ff.FF_BF16)
    pe_d = to_dev_feats(_pe(c["feats"].shape, 13, True), ff.FF_BF16)
    out = ff.ff_fwa_block(ct, g, c["G"], layers, ff.FF_BF16, x, pos_embed=pe_d)
    cur = x
    for l, key in enumerate(c["schedule"]):
        perm, goff, ng, _ = ff.ff_flatten(ct, g, key[0], key[1], c["G"])
        cur = ff.ff_group_attention(cur, perm, goff, ng, -(-c["n"] // c["G"]) + c["B"], layers[l], c["G"], ff.FF_BF16,
                                    pos_embed=pe_d)
    torch.cuda.synchronize()
    assert torch.equal(out, cur)
    assert not torch.equal(out, ff.ff_fwa_block(ct, g, c["G"], layers, ff.FF_BF16, x))
