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


def test_graph_of_points_to_bev_map():
    """The whole chain either side of the backbone in one captured graph: points -> voxel rows (dsvt_vfe) -> both
    rotated partitions -> one block -> dense bird's-eye-view map; every replay reproduces the eager result bit for
    bit (the encoder's sorted runs come out in a different order from call to call, its maxima do not)."""
    grid, lo, hi, size, C = (96, 96, 1), (-15.36, -15.36, -2.0), (15.36, 15.36, 4.0), (0.32, 0.32, 6.0), 192
    pts, _ = synth.make_points(61, 30000, lo, hi, f_in=5, clusters=60)
    w, b = synth.make_vfe_weights(62, C, 5)
    print("[case] graph capture of vfe + partition_xy + block + bev scatter, 30000 points", flush=True)
    pd = torch.as_tensor(pts).cuda()
    vfe = dsvt.Vfe(grid, 1, lo, size, 5, C, "bf16", len(pts), 9216, torch.as_tensor(w).cuda(), torch.as_tensor(b).cuda(), True)
    dsvt.dsvt_vfe(vfe, pd)
    torch.cuda.synchronize()
    n = int(vfe.n_voxels.item())                   # the host sizes the later calls with it: fixed for this input
    assert 0 < n <= 9216 and int(vfe.status.item()) == 0
    layers = [dsvt.LayerWeights(synth.make_layer_weights(63 + a, C, 8, 384, (12, 12, 1), "bf16")) for a in (0, 1)]
    pc = dsvt.part_cfg(grid, (12, 12, 1), (6, 6, 0), 36, 1, 0)
    maps = dsvt.SetMapsXY(pc, n)
    feats = torch.empty((n, C), dtype=torch.bfloat16, device="cuda")
    bev = torch.empty((1, *grid, C), dtype=torch.bfloat16, device="cuda")
    bev_status = []

    def step():
        dsvt.dsvt_vfe(vfe, pd)
        dsvt.dsvt_partition_xy(pc, vfe.coords[:n], out=maps)
        dsvt.dsvt_block(layers, maps, vfe.coords[:n], vfe.x[:n], x_out=feats)
        bev_status.append(dsvt.dsvt_bev_scatter(vfe.coords[:n], feats, 1, grid, out=bev)[1])

    step()
    torch.cuda.synchronize()
    assert int(maps.x.status.item()) == 0 and int(bev_status[-1].item()) == 0
    want_feats, want_bev, want_coords = feats.clone(), bev.clone(), vfe.coords[:n].clone()
    assert int((want_bev.float().abs().sum(-1) > 0).sum().item()) == n           # one occupied cell per voxel
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
        feats.zero_(); bev.fill_(1.0); vfe.x.zero_(); vfe.coords.zero_(); vfe.n_voxels.zero_()   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(vfe.n_voxels.item()) == n and torch.equal(vfe.coords[:n], want_coords), rep
        assert torch.equal(feats, want_feats) and torch.equal(bev, want_bev), rep
