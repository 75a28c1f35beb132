"""GPU parity of EVERY layer of configurations 3, 4 and 5 against the oracle's own chain.

The oracle sorts the cloud itself (explicit tuple sort) and runs its layers one after the other in
float64; between two layers its output is rounded to bf16 once, which is what the bf16 buffer between two
layers holds.  Layer l of the GPU path (Eq. (2) through ff_group_attention, on the perm / group list that
ff_flatten wrote on the device, which must equal the oracle's bit for bit) runs on that same bf16 input and
is compared with the oracle's un-rounded output of layer l on ALL rows: the result before storage rounding
(FF_FLAG_OUT_F32) within 2e-2 everywhere, and the bf16 buffer bit for bit its round-to-nearest-even.
Nothing the oracle consumes comes from the GPU.  ff_fwa_block is then compared end to end with the chain's
last activation.

The chain of a configuration is computed once and extended layer by layer as the tests ask for it (config 5:
about ten seconds of numpy per layer)."""
import numpy as np
import pytest
import torch

import ffsynth
import oracle
import paper_2301_08739_amd as ff
from gpu_util import DEV, assert_bf16_bar, bf16_half_ulp, geoms, to_dev_feats, to_host

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

_CHAINS = {}


class _Chain:
    """acts[l]: input of layer l (bf16-representable, float32); want(l): the oracle's output of layer l."""

    def __init__(self, c):
        self.c = c
        _, og = geoms(c)
        self.perms, self.offs = {}, {}
        for key in dict.fromkeys(c["schedule"]):
            self.perms[key], self.offs[key], _ = oracle.flatten(c["coords"], og, key[0], key[1], c["G"])
        self.acts = [np.asarray(c["feats"], dtype=np.float32)]
        self._last = (-1, None)

    def want(self, l):
        while len(self.acts) <= l + 1:
            k = len(self.acts) - 1
            key = self.c["schedule"][k]
            w = oracle.layer(self.acts[k], self.perms[key], self.offs[key], self.c["layer_params"][k])
            self._last = (k, w)
            self.acts.append(ffsynth.bf16_round(w).astype(np.float32))
        if self._last[0] != l:
            key = self.c["schedule"][l]
            self._last = (l, oracle.layer(self.acts[l], self.perms[key], self.offs[key], self.c["layer_params"][l]))
        return self._last[1]


def _chain(cfg, i):
    if i not in _CHAINS:
        _CHAINS.clear()                      # one configuration's chain at a time (config 5's is 2.5 GB)
        _CHAINS[i] = _Chain(cfg(i))
    return _CHAINS[i]


@pytest.mark.parametrize("i,l", [(i, l) for i in (3, 4, 5) for l in range(8)])
def test_layer_on_the_oracles_chain(cfg, i, l):
    ch = _chain(cfg, i)
    c = ch.c
    assert len(c["schedule"]) == 8
    key = c["schedule"][l]
    g, _ = geoms(c)
    n, G = c["n"], c["G"]
    want = ch.want(l)
    ct = torch.from_numpy(c["coords"]).to(DEV)
    perm, goff, ng, _ = ff.ff_flatten(ct, g, key[0], key[1], G)
    torch.cuda.synchronize()
    k = int(ng.item())
    assert np.array_equal(perm.cpu().numpy(), ch.perms[key])                  # the device sort is the oracle's
    assert np.array_equal(goff.cpu().numpy()[:k + 1], ch.offs[key])
    lw = ff.LayerWeights(c["layer_params"][l], ff.FF_BF16, DEV)
    x = to_dev_feats(ch.acts[l], ff.FF_BF16)
    mg = -(-n // G) + c["B"]
    wide = to_host(ff.ff_group_attention(x, perm, goff, ng, mg, lw, G, ff.FF_BF16, ff.FF_FLAG_OUT_F32))
    narrow = to_host(ff.ff_group_attention(x, perm, goff, ng, mg, lw, G, ff.FF_BF16, 0))
    assert np.array_equal(ffsynth.bf16_round(wide.astype(np.float32)).astype(np.float64), narrow)
    ew, en = assert_bf16_bar(wide, narrow, want)
    sizes = np.diff(ch.offs[key])
    print(f"cfg{i} layer {l} sort {key}: all {n} rows, {k} groups ({int((sizes < G).sum())} short); max abs err "
          f"f32-store {ew:.4e}, bf16-store {en:.4e}; max |ref| {np.abs(want).max():.3f}", flush=True)


@pytest.mark.parametrize("i", [3, 4, 5])
def test_block_end_to_end_on_the_oracles_chain(cfg, i):
    """ff_fwa_block (8 layers, bf16 buffers between them, weights re-tiled inside the call) against the last
    activation of the oracle's chain.  A layer's own error is at most 2e-2 plus the storage rounding of its
    output (half an ulp); the residual path hands the error of the layers before it on with gain one, so the
    bound for L layers is L times the per-layer one: here 8 x (2e-2 + half an ulp of |y|)."""
    ch = _chain(cfg, i)
    c = ch.c
    L = len(c["schedule"])
    ch.want(L - 1)
    ref = ch.acts[L].astype(np.float64)
    g, _ = geoms(c)
    layers = [ff.LayerWeights(p, ff.FF_BF16, DEV) for p in c["layer_params"]]
    out = ff.ff_fwa_block(torch.from_numpy(c["coords"]).to(DEV), g, c["G"], layers, ff.FF_BF16,
                          to_dev_feats(c["feats"], ff.FF_BF16))
    torch.cuda.synchronize()
    err = np.abs(to_host(out) - ref)
    bound = L * (2e-2 + bf16_half_ulp(ref))
    print(f"cfg{i} block end to end, {L} layers: max abs err {err.max():.4e}, mean {err.mean():.3e}, "
          f"max |ref| {np.abs(ref).max():.2f}, worst err/bound {float((err / bound).max()):.3f}", flush=True)
    assert np.all(err <= bound)
