"""GPU: ff_fwa_block allocates nothing, never synchronises and launches on the caller's stream, so it
can be captured into a HIP graph.  Every replay must reproduce the eager result bit for bit, with
eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import paper_2301_08739_amd as ff
from gpu_util import DEV, geoms, to_dev_feats

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("i,kw", [(2, {}), (2, {"tail": ff.FF_TAIL_DROP}), (1, {})])
def test_block_in_a_graph(cfg, i, kw):
    c = cfg(i)
    g, og = geoms(c)
    dt = ff.FF_F32 if c["dtype"] == "f32" else ff.FF_BF16
    coords = torch.from_numpy(c["coords"]).to(DEV)
    layers = [ff.LayerWeights(p, dt, DEV) for p in c["layer_params"]]
    x = to_dev_feats(c["feats"], dt)
    ws = torch.empty(ff.ff_fwa_block_workspace_bytes(c["n"], g, c["G"], layers, dt) + 512, dtype=torch.uint8, device=DEV)
    eager = ff.ff_fwa_block(coords, g, c["G"], layers, dt, x, workspace=ws, **kw).clone()   # also the warm-up call
    out = torch.zeros_like(x)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            ff.ff_fwa_block(coords, g, c["G"], layers, dt, x, out=out, workspace=ws, **kw)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        out.fill_(7.0)                                       # eager work between the replays
        ws.random_(0, 255)                                   # the workspace carries nothing from call to call
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
    # new inputs in the same buffers: the graph reads them at replay time
    x2 = to_dev_feats(np.roll(c["feats"], 1, axis=0), dt)
    want = ff.ff_fwa_block(coords, g, c["G"], layers, dt, x2, **kw)
    x.copy_(x2)
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, want)
