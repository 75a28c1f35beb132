"""GPU: ff_fwa_block in the configuration the benchmark times (bf16, masked tails, weights re-tiled
inside the call, layers chained in sorted order) equals its own layers called one by one through
ff_flatten + ff_group_attention, bit for bit, at every benchmark size; those per-layer calls are
the ones test_gpu_layer.py holds against the oracle teacher-forced.  At the headline size the
block is also compared end to end with the oracle's stack run on bf16-rounded activations."""
import numpy as np
import pytest
import torch

import ffsynth
import oracle
import paper_2301_08739_amd as ff
from gpu_util import DEV, bf16_half_ulp, geoms, to_dev_feats, to_host

pytestmark = pytest.mark.gpu


def _layer_calls(c, ct, g, layers, x):
    cur = x
    for l, key in enumerate(c["schedule"]):
        perm, goff, ng, _ = ff.ff_flatten(ct, g, key[0], key[1], c["G"])
        cur = ff.ff_group_attention(cur, perm, goff, ng, -(-c["n"] // c["G"]) + c["B"], layers[l], c["G"], ff.FF_BF16)
    return cur


@pytest.mark.parametrize("i", [2, 3, 4, 5])
def test_block_equals_its_layer_calls(cfg, i):
    c = cfg(i)
    g, _ = geoms(c)
    print(f"block cfg{i}: n={c['n']} B={c['B']} G={c['G']} C={c['C']} layers={len(c['schedule'])}", flush=True)
    ct = torch.from_numpy(c["coords"]).to(DEV)
    layers = [ff.LayerWeights(p, ff.FF_BF16, DEV) for p in c["layer_params"]]      # not packed: the call re-tiles
    x = to_dev_feats(c["feats"], ff.FF_BF16)
    keep = x.clone()
    out = ff.ff_fwa_block(ct, g, c["G"], layers, ff.FF_BF16, x)
    want = _layer_calls(c, ct, g, layers, x)
    torch.cuda.synchronize()
    assert torch.equal(x, keep)                                                    # the input is not touched
    assert torch.isfinite(out.float()).all()
    assert torch.equal(out, want)
    packed = [ff.LayerWeights(p, ff.FF_BF16, DEV).pack() for p in c["layer_params"]]
    out2 = ff.ff_fwa_block(ct, g, c["G"], packed, ff.FF_BF16, x)                   # weights re-tiled once, ahead of time
    torch.cuda.synchronize()
    assert torch.equal(out2, want)


def test_headline_block_end_to_end_against_the_oracle(cfg):
    """Four layers with a bf16 buffer between them: the oracle rounds each layer's output to bf16 as
    the buffer does.  The per-layer bound is 2e-2 + storage rounding; through four layers the error
    of one layer is carried on by the next (the residual path passes it through with gain one), so
    the bound taken is four times the per-layer one."""
    c = cfg(2)
    g, og = geoms(c)
    cur = c["feats"]
    for l, key in enumerate(c["schedule"]):
        perm, off, _ = oracle.flatten(c["coords"], og, key[0], key[1], c["G"])
        cur = ffsynth.bf16_round(oracle.layer(cur, perm, off, c["layer_params"][l])).astype(np.float64)
    layers = [ff.LayerWeights(p, ff.FF_BF16, DEV) for p in c["layer_params"]]
    out = ff.ff_fwa_block(torch.from_numpy(c["coords"]).to(DEV), g, c["G"], layers, ff.FF_BF16,
                          to_dev_feats(c["feats"], ff.FF_BF16))
    torch.cuda.synchronize()
    got = to_host(out)
    err = np.abs(got - cur)
    bound = 4 * (2e-2 + bf16_half_ulp(cur))
    print(f"cfg2 block end to end: max abs err {err.max():.4e}, mean {err.mean():.3e}, max |ref| {np.abs(cur).max():.2f}",
          flush=True)
    assert np.all(err <= bound)


@pytest.mark.parametrize("num_layers", [1, 2, 3, 5, 9, 17])
def test_layer_counts(cfg, num_layers):
    """One layer (no chaining), fewer layers than sort configurations, counts that are no multiple of
    four, and more layers than one weight re-tiling launch takes (16)."""
    c = cfg(2, num_layers)
    n = 5000
    coords = np.ascontiguousarray(c["coords"][:n])
    g, _ = geoms(c)
    ct = torch.from_numpy(coords).to(DEV)
    layers = [ff.LayerWeights(p, ff.FF_BF16, DEV) for p in c["layer_params"]]
    assert len(layers) == num_layers
    x = to_dev_feats(c["feats"][:n], ff.FF_BF16)
    out = ff.ff_fwa_block(ct, g, c["G"], layers, ff.FF_BF16, x)
    cur = x
    for l, key in enumerate(ffsynth.layer_schedule(num_layers)):
        perm, goff, ng, _ = ff.ff_flatten(ct, g, key[0], key[1], c["G"])
        cur = ff.ff_group_attention(cur, perm, goff, ng, -(-n // c["G"]) + c["B"], layers[l], c["G"], ff.FF_BF16)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    assert torch.equal(out, cur)
