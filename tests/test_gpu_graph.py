"""A captured HIP graph of the hot path replays to the eager result, every time."""
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu
dsvt = pytest.importorskip("paper_2301_06051_amd")
from gpu_util import dev_coords, dev_feats  # noqa: E402


def test_graph_replays_match_eager():
    cfg = synth.CONFIGS[2]
    coords = synth.make_frame(2, n=4000)
    n = len(coords)
    print("[case] graph capture of 2 partitions + 1 block, 4000 pillars", flush=True)
    cd = dev_coords(coords)
    x0 = dev_feats(synth.make_features(41, n, cfg["C"], "bf16"), "bf16")
    layers = [dsvt.LayerWeights(synth.make_layer_weights(42 + a, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], "bf16"))
              for a in (0, 1)]
    pcs = [dsvt.part_cfg(cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], 1, a) for a in (0, 1)]
    maps = [dsvt.SetMaps(pc, n) for pc in pcs]
    out = torch.empty_like(x0)

    def step():
        for pc, mp in zip(pcs, maps):
            dsvt.dsvt_partition(pc, cd, out=mp)
        dsvt.dsvt_block(layers, maps, cd, x0, x_out=out)

    step()
    torch.cuda.synchronize()
    want, want_inds = out.clone(), [m.set_inds.clone() for m in maps]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        out.zero_()                               # eager work between the replays
        for m in maps:
            m.set_inds.fill_(-1)
            m.n_sets.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), rep
        for m, w in zip(maps, want_inds):
            assert torch.equal(m.set_inds, w), rep
