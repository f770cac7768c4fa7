"""GPU parity of dsvt_vfe (Sec. 3.1 overview: points -> sparse voxels) against the CPU oracle: voxel
coordinates and counts bit for bit, features bit for bit where the encoder only selects values
(no linear map, float32), else to the tolerance of the arithmetic."""
import numpy as np
import pytest
import torch

import synth
from oracle import dsvt_oracle as orc

pytestmark = pytest.mark.gpu

dsvt = pytest.importorskip("paper_2301_06051_amd")
from gpu_util import assert_maps_equal, rel_err  # noqa: E402

WAYMO_LO, WAYMO_HI = (-74.88, -74.88, -2.0), (74.88, 74.88, 4.0)


def _say(msg):
    print(f"[case] {msg}", flush=True)


def _run(grid, batch, lo, size, pts, pb, C, dtype, w=None, b=None, relu=False, max_voxels=None, vfe=None):
    wd = None if w is None else torch.as_tensor(w).cuda()
    bd = None if b is None else torch.as_tensor(b).cuda()
    if vfe is None:
        vfe = dsvt.Vfe(grid, batch, lo, size, pts.shape[1], C, dtype, len(pts), max_voxels or len(pts), wd, bd, relu)
    dsvt.dsvt_vfe(vfe, torch.as_tensor(pts).cuda(), None if pb is None else torch.as_tensor(pb).cuda())
    torch.cuda.synchronize()
    return vfe


def _check(vfe, ref_coords, ref_x, tol):
    n = int(vfe.n_voxels.item())
    assert n == len(ref_coords) and int(vfe.status.item()) == 0
    assert np.array_equal(vfe.coords[:n].cpu().numpy(), ref_coords)
    if tol == 0:
        assert np.array_equal(vfe.x[:n].double().cpu().numpy(), ref_x)
    else:
        e = rel_err(vfe.x[:n], ref_x)
        _say(f"  rel err {e:.2e}")
        assert e <= tol


@pytest.mark.parametrize("grid,batch,n_points,f_in", [((16, 16, 1), 2, 3000, 5), ((40, 24, 6), 3, 20000, 4), ((7, 5, 3), 1, 1, 3)])
def test_vfe_plain_max_bit_exact(grid, batch, n_points, f_in):
    lo, hi = (-4.0, -2.0, -1.0), (4.0, 2.0, 1.0)
    size = tuple((h - l) / g for l, h, g in zip(lo, hi, grid))
    pts, pb = synth.make_points(21, n_points, lo, hi, f_in=f_in, batch=batch)
    if n_points == 1:
        pts[0, :3] = 0.1
    _say(f"vfe plain max grid={grid} batch={batch} points={n_points}")
    rc, rx = orc.voxel_max_vfe(pts, pb, lo, size, grid, batch)
    vfe = _run(grid, batch, lo, size, pts, pb, f_in, "f32")
    _check(vfe, rc, rx, 0)
    # the same buffers again with fewer points, in another order: nothing of the first call may remain
    perm = np.random.default_rng(1).permutation(n_points)[: max(n_points // 3, 1)]
    rc2, rx2 = orc.voxel_max_vfe(pts[perm], pb[perm], lo, size, grid, batch)
    _check(_run(grid, batch, lo, size, pts[perm], pb[perm], f_in, "f32", vfe=vfe), rc2, rx2, 0)


@pytest.mark.parametrize("dt,C,f_in,relu", [("f32", 64, 5, False), ("f32", 64, 5, True), ("bf16", 192, 5, True), ("bf16", 128, 16, False)])
def test_vfe_linear_map(dt, C, f_in, relu):
    grid, batch = (64, 48, 4), 2
    lo, hi = (-8.0, -6.0, -1.0), (8.0, 6.0, 1.0)
    size = (0.25, 0.25, 0.5)
    pts, pb = synth.make_points(22, 40000, lo, hi, f_in=f_in, batch=batch)
    w, b = synth.make_vfe_weights(23, C, f_in)
    _say(f"vfe linear {dt} C={C} f_in={f_in} relu={relu}")
    rc, rx = orc.voxel_max_vfe(pts, pb, lo, size, grid, batch, w, b, relu)
    _check(_run(grid, batch, lo, size, pts, pb, C, dt, w, b, relu), rc, rx, 1e-5 if dt == "f32" else 4e-3)


@pytest.mark.parametrize("grid_z,n_points", [(1, 180000), (32, 180000)])
def test_vfe_lidar_frame_feeds_the_partition(grid_z, n_points):
    """A frame of the benchmark's shape (468 x 468 cells of 0.32 m; one pillar or 32 layers of 0.1875 m), C = 192
    bf16; the voxel rows it writes are what the set partition takes."""
    grid = (468, 468, grid_z)
    size = (0.32, 0.32, 6.0 / grid_z)
    pts, _ = synth.make_points(24, n_points, WAYMO_LO, WAYMO_HI, f_in=5)
    w, b = synth.make_vfe_weights(25, 192, 5)
    _say(f"vfe lidar frame grid={grid} points={n_points}")
    rc, rx = orc.voxel_max_vfe(pts, None, WAYMO_LO, size, grid, 1, w, b, True)
    vfe = _run(grid, 1, WAYMO_LO, size, pts, None, 192, "bf16", w, b, True)
    _check(vfe, rc, rx, 4e-3)
    n = len(rc)
    win, tau = (12, 12, 8 if grid_z > 1 else 1), 36
    pc = dsvt.part_cfg(grid, win, (6, 6, 0), tau, 1, 0)
    pair = dsvt.dsvt_partition_xy(pc, vfe.coords[:n])
    for axis in (0, 1):
        assert_maps_equal(pair[axis], orc.partition(rc, grid, win, (6, 6, 0), tau, axis))


@pytest.mark.parametrize("n_vox", [16384, 16385, 32768, 40000])
def test_vfe_voxel_counts_at_the_scan_chunk_edges(n_vox):
    """The two scans of the encoder work in chunks of 16,384 elements (a workgroup per chunk): voxel counts of exactly
    one chunk, one more, exactly two, and a bitmap of exactly one chunk of words (1024 x 512 cells)."""
    grid, lo, size = (1024, 512, 1), (0.0, 0.0, 0.0), (1.0, 1.0, 1.0)
    rng = np.random.default_rng(27)
    cells = rng.choice(grid[0] * grid[1], n_vox, replace=False)
    reps = rng.integers(1, 4, n_vox)
    cell_of = np.repeat(cells, reps)
    rng.shuffle(cell_of)
    pts = np.empty((len(cell_of), 4), dtype=np.float32)
    pts[:, 0] = cell_of // grid[1] + rng.uniform(0.1, 0.9, len(cell_of))
    pts[:, 1] = cell_of % grid[1] + rng.uniform(0.1, 0.9, len(cell_of))
    pts[:, 2] = 0.5
    pts[:, 3] = rng.random(len(cell_of))
    _say(f"vfe scan edges voxels={n_vox} points={len(pts)}")
    rc, rx = orc.voxel_max_vfe(pts, None, lo, size, grid, 1)
    assert len(rc) == n_vox
    _check(_run(grid, 1, lo, size, pts, None, 4, "f32", max_voxels=n_vox + 7), rc, rx, 0)


def test_vfe_capacity_and_host_errors():
    grid, lo, size = (16, 16, 1), (-4.0, -2.0, -1.0), (0.5, 0.25, 2.0)
    pts, _ = synth.make_points(26, 3000, lo, (4.0, 2.0, 1.0), f_in=5)
    rc, rx = orc.voxel_max_vfe(pts, None, lo, size, grid, 1)
    cap = len(rc) // 2
    _say(f"vfe capacity {cap} of {len(rc)} voxels")
    vfe = _run(grid, 1, lo, size, pts, None, 5, "f32", max_voxels=cap)
    assert int(vfe.status.item()) == dsvt.binding.ST_VOXEL_OVERFLOW and int(vfe.n_voxels.item()) == len(rc)
    assert np.array_equal(vfe.coords.cpu().numpy(), rc[:cap])
    assert np.array_equal(vfe.x.double().cpu().numpy(), rx[:cap])
    import ctypes as C
    L, B = dsvt.lib(), dsvt.binding
    good = vfe.cfg
    sz = C.c_size_t(0)
    def cfg(**kw):
        c = B.VfeCfg.from_buffer_copy(good)
        for k, v in kw.items():
            setattr(c, k, v)
        return c
    for bad in (cfg(f_in=2), cfg(f_in=17), cfg(C=7), cfg(batch=0), cfg(dtype=5), cfg(voxel_size=B.F32x3(0.5, 0.0, 2.0)),
                cfg(grid=B.I32x3(65536, 65536, 1))):
        assert L.dsvt_vfe_workspace_size(C.byref(bad), 3000, cap, C.byref(sz)) < 0
    p = torch.as_tensor(pts).cuda()
    args = lambda c, ws_bytes, pbatch=None: (C.byref(c), p.data_ptr(), pbatch, 3000, vfe.coords.data_ptr(), vfe.x.data_ptr(),
                                             vfe.n_voxels.data_ptr(), cap, vfe.ws.data_ptr(), ws_bytes, vfe.status.data_ptr(), None)
    assert L.dsvt_vfe(*args(good, vfe.ws.numel() - 1)) == B.DSVT_ENOSPC
    assert L.dsvt_vfe(*args(cfg(batch=2), vfe.ws.numel())) == B.DSVT_EINVAL          # several frames need point_batch
    torch.cuda.synchronize()
