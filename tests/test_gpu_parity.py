"""GPU parity: the HIP path through the C ABI against the CPU oracle on the same seeded inputs.

Index maps must match bit for bit; features to TOL (1e-4 fp32, 2e-2 bf16) as
max |gpu - oracle| / max |oracle| per output tensor.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import dsvt_oracle as orc

pytestmark = pytest.mark.gpu

dsvt = pytest.importorskip("paper_2301_06051_amd")
from gpu_util import TOL, assert_maps_equal, assert_tiles_valid, dev_coords, dev_feats, gpu_maps, rel_err  # noqa: E402


def _say(msg):
    print(f"[case] {msg}", flush=True)


# ------------------------------------------------------------------ partition
@pytest.mark.parametrize("cid,n", [(1, None), (2, None), (3, None), (5, None), (2, 777), (3, 5000)])
@pytest.mark.parametrize("axis", [0, 1])
def test_partition_bit_exact(cid, n, axis):
    cfg = synth.CONFIGS[cid]
    coords = synth.make_frame(cid, n=n)
    shift = cfg["shifts"][-1]
    _say(f"partition cfg{cid} n={len(coords)} axis={axis} shift={shift}")
    om = orc.partition(coords, cfg["grid"], cfg["win"], shift, cfg["tau"], axis)
    gm = gpu_maps(dev_coords(coords), cfg["grid"], cfg["win"], shift, cfg["tau"], cfg["batch"], axis)
    assert_maps_equal(gm, om)


@pytest.mark.parametrize("cid,n", [(1, None), (2, None), (3, None), (2, 777), (3, 5000), (5, 30000)])
def test_partition_xy_bit_exact(cid, n):
    """Both rotated partitions from one call: each equals the oracle's partition of its axis, and the
    Y-axis maps share the set counts, window keys and tile boundaries of the X-axis maps."""
    cfg = synth.CONFIGS[cid]
    coords = synth.make_frame(cid, n=n)
    shift = cfg["shifts"][-1]
    _say(f"partition_xy cfg{cid} n={len(coords)} shift={shift}")
    pc = dsvt.part_cfg(cfg["grid"], cfg["win"], shift, cfg["tau"], cfg["batch"], 0)
    pair = dsvt.dsvt_partition_xy(pc, dev_coords(coords))
    for axis in (0, 1):
        assert_maps_equal(pair[axis], orc.partition(coords, cfg["grid"], cfg["win"], shift, cfg["tau"], axis))
    assert pair[1].n_sets.data_ptr() == pair[0].n_sets.data_ptr()
    # a second call into the same buffers (nothing left over from the first may matter)
    coords2 = synth.make_frame(cid, n=max(len(coords) // 2, 1))
    pair2 = dsvt.SetMapsXY(pc, len(coords2))
    for m in (pair2.x, pair2.y):
        m.tile_desc.fill_(12345)                      # descriptors are not cleared by the caller
    dsvt.dsvt_partition_xy(pc, dev_coords(coords2), out=pair2)
    dsvt.dsvt_partition_xy(pc, dev_coords(coords2), out=pair2)
    for axis in (0, 1):
        om = orc.partition(coords2, cfg["grid"], cfg["win"], shift, cfg["tau"], axis)
        torch.cuda.synchronize()
        n_sets = int(pair2[axis].n_sets.item())
        assert n_sets == om["n_sets"]
        assert np.array_equal(pair2[axis].set_inds[:n_sets].cpu().numpy(), om["set_inds"])
        assert_tiles_valid(pair2[axis], om)


@pytest.mark.parametrize("cid,n", [(2, None), (1, None), (3, 20000)])
def test_partition_xy_multi_bit_exact(cid, n):
    """A stage's window configurations (unshifted, shifted, and a second tau) partitioned by one call."""
    cfg = synth.CONFIGS[cid]
    coords = synth.make_frame(cid, n=n)
    half = tuple(w // 2 for w in cfg["win"][:2]) + (0,)
    variants = [((0, 0, 0), cfg["tau"]), (half, cfg["tau"]), (half, cfg["tau"] // 2 + 1)]
    _say(f"partition_xy_multi cfg{cid} n={len(coords)}")
    pcs = [dsvt.part_cfg(cfg["grid"], cfg["win"], sh, tau, cfg["batch"], 0) for sh, tau in variants]
    outs = [dsvt.SetMapsXY(pc, len(coords)) for pc in pcs]
    cd = dev_coords(coords)
    for _ in range(2):                                 # twice: the second call finds what the first left behind
        dsvt.dsvt_partition_xy_multi(pcs, cd, outs)
    for (sh, tau), out in zip(variants, outs):
        for axis in (0, 1):
            assert_maps_equal(out[axis], orc.partition(coords, cfg["grid"], cfg["win"], sh, tau, axis))

def test_partition_xy_multi_mixed_front_ends():
    """One call whose window configurations take different front ends: 12 x 12 windows (a frame's tables fit one
    workgroup's LDS), 3 x 3 windows (24,000 windows: the general chain), and 24 x 24 windows with a large set."""
    cfg = synth.CONFIGS[2]
    coords = synth.make_frame(2, n=20000)
    variants = [((12, 12, 1), (6, 6, 0), 36), ((3, 3, 1), (1, 2, 0), 4), ((24, 24, 1), (12, 12, 0), 90), ((3, 3, 1), (0, 0, 0), 5)]
    _say("partition_xy_multi with mixed front ends")
    pcs = [dsvt.part_cfg(cfg["grid"], win, sh, tau, 1, 0) for win, sh, tau in variants]
    outs = [dsvt.SetMapsXY(pc, len(coords)) for pc in pcs]
    cd = dev_coords(coords)
    for _ in range(2):
        dsvt.dsvt_partition_xy_multi(pcs, cd, outs)
    for (win, sh, tau), out in zip(variants, outs):
        for axis in (0, 1):
            assert_maps_equal(out[axis], orc.partition(coords, cfg["grid"], win, sh, tau, axis))


@pytest.mark.parametrize("n", [300, 3000, 12000, 20000])
def test_small_frames_spread_over_the_compute_units(n):
    """A frame whose 64-row tiles would not fill the 256 compute units once is cut into more, shorter tiles (at
    most 256, of 16 rows or more between cuts); larger frames keep the 64-row cut or get filled tiles when that saves
    a round.  The work list stays valid."""
    cfg = synth.CONFIGS[2]
    coords = synth.make_frame(2, n=n)
    _say(f"tile spread n={len(coords)}")
    om = orc.partition(coords, cfg["grid"], cfg["win"], (0, 0, 0), cfg["tau"], 0)
    pair = dsvt.dsvt_partition_xy(dsvt.part_cfg(cfg["grid"], cfg["win"], (0, 0, 0), cfg["tau"], 1, 0), dev_coords(coords))
    assert_maps_equal(pair[0], om)
    si = om["set_inds"]
    first = np.ones(si.shape, bool)
    first[:, 1:] = np.diff(si, axis=1) != 0
    rows = int(((first.sum(1) + 3) // 4 * 4).sum())
    nt = int(pair[0].n_tiles.item())
    _say(f"  rows {rows}, tiles {nt}")
    if rows <= 64 * 256:
        cut = min(max((-(-rows // 256) + 3) // 4 * 4, 16), 64)
        assert nt <= min(256, rows // cut + 1) and nt >= 0.8 * min(256, rows // cut)
    else:
        assert nt <= rows / 64 + 2                         # (20,000 voxels: filled tiles, one round instead of two)
        if n == 20000:
            assert nt <= 256


@pytest.mark.parametrize("cid,n", [(2, 45000), (2, 64000), (3, None), (5, None)])
def test_large_frames_get_filled_tiles(cid, n):
    """Frames of several rounds over the compute units: a set starts a tile only when it no longer fits the tile before,
    so tiles hold more than the 64 rows a fixed cut gives; for a frame of a few rounds the tile count ends just under a
    whole number of rounds.  The work list stays valid (both kernels' paths)."""
    cfg = synth.CONFIGS[cid]
    coords = synth.make_frame(cid, n=n)
    _say(f"filled tiles cfg{cid} n={len(coords)}")
    om = orc.partition(coords, cfg["grid"], cfg["win"], (0, 0, 0), cfg["tau"], 0)
    pair = dsvt.dsvt_partition_xy(dsvt.part_cfg(cfg["grid"], cfg["win"], (0, 0, 0), cfg["tau"], cfg["batch"], 0), dev_coords(coords))
    assert_maps_equal(pair[0], om)
    assert_maps_equal(pair[1], orc.partition(coords, cfg["grid"], cfg["win"], (0, 0, 0), cfg["tau"], 1))
    si = om["set_inds"]
    first = np.ones(si.shape, bool)
    first[:, 1:] = np.diff(si, axis=1) != 0
    rows = int(((first.sum(1) + 3) // 4 * 4).sum())
    nt = int(pair[0].n_tiles.item())
    _say(f"  rows {rows}, tiles {nt}, rows per tile {rows / nt:.1f}")
    if nt > 4 * 256:
        # frames of more than four rounds: tiles of up to 96 rows, filled greedily inside pieces of 4,096 rows (the
        # first set that begins in a piece starts a tile); a frame of more than 16,384 sets is taken 4,096 sets at a
        # time, each such run with rows counted from its own start; the count follows from the sets' padded rows alone
        per_set = (first.sum(1) + 3) // 4 * 4
        runs = [per_set] if len(per_set) <= 16384 else [per_set[i:i + 4096] for i in range(0, len(per_set), 4096)]
        want = 0
        for run in runs:
            before = np.concatenate([[0], np.cumsum(run)])
            s = 0
            while s < len(run):
                want += 1
                t = s + 1
                while t < len(run) and before[t + 1] - before[s] <= 96 and before[t] >> 12 == before[s] >> 12:
                    t += 1
                s = t
        assert nt == want
        assert rows / nt > 75                              # (an unbroken greedy fill of the skewed batch's sets gives 76.2)
    else:
        assert rows / nt > 66 and 0.88 < (nt / 256) / np.ceil(nt / 256) <= 1.0


def test_partition_buffers_reused_across_frame_sizes():
    """A stream of frames with different voxel counts through one set of buffers (sized for the largest): the
    scratch buffer's bitmap is left clean by every call whatever the frame's size."""
    cfg = synth.CONFIGS[2]
    grid, win, tau, shift = cfg["grid"], cfg["win"], cfg["tau"], (6, 6, 0)
    pc = dsvt.part_cfg(grid, win, shift, tau, 1, 0)
    cap = 30000
    pair = dsvt.SetMapsXY(pc, cap)
    lib, C = dsvt.lib(), dsvt.binding.C
    ptr = lambda t: C.c_void_p(t.data_ptr())
    for n in (30000, 9000, 21000, 500):
        coords = synth.make_frame(2, n=n)
        _say(f"partition_xy stream n={len(coords)}")
        cd = dev_coords(coords)
        for m in (pair.x, pair.y):
            m.set_inds.fill_(-1)
        rc = lib.dsvt_partition_xy(C.byref(pc), ptr(cd), len(coords), ptr(pair.x.set_inds), ptr(pair.y.set_inds),
                                   ptr(pair.x.voxel_slot), ptr(pair.y.voxel_slot), ptr(pair.x.n_sets), pair.x.max_sets,
                                   ptr(pair.x.set_win), C.byref(pair.x.tile_list), ptr(pair.y.tile_desc), ptr(pair.x.ws),
                                   pair.x.ws.numel(), ptr(pair.x.status), None)
        assert rc == 0
        torch.cuda.synchronize()
        assert int(pair.x.status.item()) == 0
        for axis in (0, 1):
            om = orc.partition(coords, grid, win, shift, tau, axis)
            k = int(pair[axis].n_sets.item())
            assert k == om["n_sets"]
            assert np.array_equal(pair[axis].set_inds[:k].cpu().numpy(), om["set_inds"])
            assert np.array_equal(pair[axis].voxel_slot[:len(coords)].cpu().numpy(), om["voxel_slot"])
            assert_tiles_valid(pair[axis], om)


def test_partition_xy_odd_geometry_and_batch():
    grid, win, shift, tau = (29, 17, 9), (5, 7, 3), (2, 6, 1), 11
    coords = np.concatenate([np.concatenate([np.full((900, 1), b), synth.frame_uniform(60 + b, grid, 900)], 1)
                             for b in range(3)]).astype(np.int32)
    _say("partition_xy odd geometry")
    pair = dsvt.dsvt_partition_xy(dsvt.part_cfg(grid, win, shift, tau, 3, 0), dev_coords(coords))
    for axis in (0, 1):
        assert_maps_equal(pair[axis], orc.partition(coords, grid, win, shift, tau, axis))


@pytest.mark.parametrize("n", [1, 35, 36, 37, 72, 73])
def test_partition_single_window_edges(n):
    """One window holding n voxels around the multiples of tau, including a lone voxel."""
    _say(f"partition one window n={n}")
    grid, win, tau = (12, 12, 1), (12, 12, 1), 36
    coords = np.concatenate([np.zeros((n, 1), np.int64), synth.frame_uniform(3, grid, n)], 1).astype(np.int32)
    for axis in (0, 1):
        om = orc.partition(coords, grid, win, (0, 0, 0), tau, axis)
        gm = gpu_maps(dev_coords(coords), grid, win, (0, 0, 0), tau, 1, axis)
        assert_maps_equal(gm, om)


def test_partition_odd_geometry_and_batch():
    """Window volume not a multiple of 32, grid not a multiple of the window, 3 frames, shift on all axes."""
    grid, win, shift, tau = (29, 17, 9), (5, 7, 3), (2, 6, 1), 11
    coords = np.concatenate([np.concatenate([np.full((900, 1), b), synth.frame_uniform(50 + b, grid, 900)], 1)
                             for b in range(3)]).astype(np.int32)
    _say("partition odd geometry")
    for axis in (0, 1):
        om = orc.partition(coords, grid, win, shift, tau, axis)
        gm = gpu_maps(dev_coords(coords), grid, win, shift, tau, 3, axis)
        assert_maps_equal(gm, om)


def test_partition_reports_bad_input_without_faulting():
    grid, win, tau = (24, 24, 1), (12, 12, 1), 36
    coords = np.concatenate([np.zeros((200, 1), np.int64), synth.frame_uniform(4, grid, 200)], 1).astype(np.int32)
    cfg = dsvt.part_cfg(grid, win, (0, 0, 0), tau, 1, 0)
    _say("partition status bits")
    bad = coords.copy(); bad[5, 1] = 24                           # outside the grid
    gm = dsvt.dsvt_partition(cfg, dev_coords(bad)); torch.cuda.synchronize()
    assert int(gm.status.item()) & dsvt.binding.ST_COORD_RANGE
    rep = coords.copy(); rep[7] = rep[8]                          # repeated cell
    gm = dsvt.dsvt_partition(cfg, dev_coords(rep)); torch.cuda.synchronize()
    assert int(gm.status.item()) & dsvt.binding.ST_COORD_REPEAT
    small = dsvt.SetMaps(cfg, 200, max_sets=3)                    # too few set rows
    gm = dsvt.dsvt_partition(cfg, dev_coords(coords), out=small); torch.cuda.synchronize()
    assert int(gm.status.item()) & dsvt.binding.ST_SET_OVERFLOW
    assert int(gm.n_sets.item()) == orc.partition(coords, grid, win, (0, 0, 0), tau, 0)["n_sets"]
    with pytest.raises(dsvt.DsvtError) as e:
        dsvt.dsvt_partition(dsvt.part_cfg(grid, win, (12, 0, 0), tau, 1, 0), dev_coords(coords), out=gm)
    assert e.value.rc == dsvt.binding.DSVT_EINVAL
    # host-side argument errors of the paired and the multi-configuration entry points
    pair = dsvt.SetMapsXY(cfg, 200)
    with pytest.raises(dsvt.DsvtError) as e:
        dsvt.dsvt_partition_xy_multi([cfg] * 5, dev_coords(coords), [pair] * 5)
    assert e.value.rc == dsvt.binding.DSVT_EINVAL
    lib, C = dsvt.lib(), dsvt.binding.C
    cd = dev_coords(coords)
    ptr = lambda t: C.c_void_p(t.data_ptr())
    rc = lib.dsvt_partition_xy(C.byref(cfg), ptr(cd), 200, ptr(pair.x.set_inds), ptr(pair.y.set_inds), ptr(pair.x.voxel_slot),
                               ptr(pair.y.voxel_slot), ptr(pair.x.n_sets), pair.x.max_sets, None, None, None, ptr(pair.x.ws), 64,
                               ptr(pair.x.status), None)
    assert rc == dsvt.binding.DSVT_ENOSPC                          # scratch too small
    rc = lib.dsvt_partition_xy(C.byref(cfg), ptr(cd), 200, ptr(pair.x.set_inds), None, ptr(pair.x.voxel_slot),
                               ptr(pair.y.voxel_slot), ptr(pair.x.n_sets), pair.x.max_sets, None, None, None, ptr(pair.x.ws),
                               pair.x.ws.numel(), ptr(pair.x.status), None)
    assert rc == dsvt.binding.DSVT_EINVAL                          # an output of the second axis missing
    rc = lib.dsvt_partition_xy(C.byref(cfg), ptr(cd), 200, ptr(pair.x.set_inds), ptr(pair.y.set_inds), ptr(pair.x.voxel_slot),
                               ptr(pair.y.voxel_slot), ptr(pair.x.n_sets), pair.x.max_sets, None, C.byref(pair.x.tile_list), None,
                               ptr(pair.x.ws), pair.x.ws.numel(), ptr(pair.x.status), None)
    assert rc == dsvt.binding.DSVT_EINVAL                          # a work list without the second axis's descriptors
    assert lib.dsvt_partition_ws_init(C.byref(cfg), 200, ptr(pair.x.ws), 64, None) == dsvt.binding.DSVT_ENOSPC
    # no work list and no set_win: the maps alone
    plain = dsvt.SetMapsXY(cfg, 200, tiles=False)
    dsvt.dsvt_partition_xy(cfg, cd, out=plain)
    for axis in (0, 1):
        assert_maps_equal(plain[axis], orc.partition(coords, grid, win, (0, 0, 0), tau, axis))
    # a scratch buffer that dsvt_partition_ws_init has not prepared: no sets, and the status says why
    for maker, call in ((dsvt.SetMaps, dsvt.dsvt_partition), (dsvt.SetMapsXY, dsvt.dsvt_partition_xy)):
        raw = maker(cfg, 200)
        first = raw if maker is dsvt.SetMaps else raw.x
        first.ws[:64].fill_(0x5A)
        call(cfg, dev_coords(coords), out=raw); torch.cuda.synchronize()
        assert int(first.status.item()) & dsvt.binding.ST_WS_STATE and int(first.n_sets.item()) == 0
        assert torch.all(first.voxel_slot == -1)


@pytest.mark.parametrize("cid,n", [(2, 5000), (3, 20000)])
def test_partition_buffer_survives_calls_that_report_errors(cid, n):
    """The partition's scratch buffer carries an occupancy bitmap from call to call (every call finds it zero and
    leaves it zero).  One buffer through: a good frame, a frame with a voxel outside the grid, a frame with a
    repeated cell, a call with too few set rows, a call with too short a work list -- each reports its status bit
    -- and then the good frame again, whose maps must be bit-exact with status 0.  Both front ends (the
    single-workgroup one for the pillar frame, the general chain for the voxel grid)."""
    cfg = synth.CONFIGS[cid]
    coords = synth.make_frame(cid, n=n)
    shift = cfg["shifts"][-1]
    B = dsvt.binding
    pc = dsvt.part_cfg(cfg["grid"], cfg["win"], shift, cfg["tau"], cfg["batch"], 0)
    pair = dsvt.SetMapsXY(pc, len(coords))
    oms = [orc.partition(coords, cfg["grid"], cfg["win"], shift, cfg["tau"], a) for a in (0, 1)]

    def share_ws(other):
        other.x.ws = other.y.ws = pair.x.ws
        return other

    def call(c, out, want_bit):
        out.x.status.zero_()
        dsvt.dsvt_partition_xy(pc, dev_coords(c), out=out)
        torch.cuda.synchronize()
        st = int(out.x.status.item())
        _say(f"  status {st} (expected bit {want_bit})")
        assert (st & want_bit) == want_bit and (want_bit != 0 or st == 0)

    _say(f"partition buffer through error-reporting calls, cfg{cid} n={len(coords)}")
    call(coords, pair, 0)
    for axis in (0, 1):
        assert_maps_equal(pair[axis], oms[axis])
    bad = coords.copy(); bad[5, 1] = cfg["grid"][0]; bad[9, 0] = cfg["batch"]     # outside the grid, outside the batch
    call(bad, pair, B.ST_COORD_RANGE)
    rep = coords.copy(); rep[7] = rep[8]; rep[100] = rep[8]                      # one cell three times
    call(rep, pair, B.ST_COORD_REPEAT)
    call(coords, share_ws(dsvt.SetMapsXY(pc, len(coords), max_sets=3)), B.ST_SET_OVERFLOW)
    call(coords, share_ws(dsvt.SetMapsXY(pc, len(coords), max_tiles=2)), B.ST_TILE_OVERFLOW)
    for m in (pair.x, pair.y):
        m.set_inds.fill_(-1); m.voxel_slot.fill_(-1)
    call(coords, pair, 0)
    for axis in (0, 1):
        assert_maps_equal(pair[axis], oms[axis])


@pytest.mark.parametrize("seed", [2, 5, 8])
def test_large_random_frames_through_the_general_front_end(seed):
    """Seeded random geometries (odd window sizes, shifts on every axis, two to four frames, 190,000-520,000 voxels):
    bounds of 15,000-25,000 sets, i.e. work lists built by the window scan itself, by one workgroup, or piece by piece."""
    rng = np.random.Generator(np.random.Philox(9900 + seed))
    win = (int(rng.integers(6, 25)), int(rng.integers(6, 25)), int(rng.choice([1, 2, 4, 8, 16])))
    grid = (int(rng.integers(200, 470)), int(rng.integers(200, 470)), int(win[2] * rng.integers(1, 5)))
    shift = tuple(int(rng.integers(0, w)) for w in win)
    tau = int(rng.choice([24, 36, 48, 60]))
    batch = int(rng.choice([1, 1, 2, 4]))
    n = int(min(rng.integers(40000, 160000), max(grid[0] * grid[1] * grid[2] // 3, 1)))
    frames = []
    for b in range(batch):
        c = synth.frame_radial(9950 + 16 * seed + b, grid, n)
        frames.append(np.concatenate([np.full((len(c), 1), b, np.int64), c], 1))
    coords = np.concatenate(frames).astype(np.int32)
    pc = dsvt.part_cfg(grid, win, shift, tau, batch, 0)
    oms = [orc.partition(coords, grid, win, shift, tau, a) for a in (0, 1)]
    _say(f"general front end seed={seed} grid={grid} win={win} shift={shift} tau={tau} batch={batch} n={len(coords)} "
         f"bound={dsvt.binding.dsvt_partition_bound(pc, len(coords))[0]} sets={oms[0]['n_sets']}")
    pair = dsvt.dsvt_partition_xy(pc, dev_coords(coords))
    for axis in (0, 1):
        assert_maps_equal(pair[axis], oms[axis])


def test_work_list_of_a_frame_whose_bound_exceeds_the_tables_but_whose_sets_do_not():
    """Two uniformly filled frames of 150,000 voxels: the bound on their sets (voxels / tau + windows = 20,501) is above
    the 16,384 sets one workgroup's tables hold, so the host prepares the piece-wise launches, but the 12,317 sets
    there are fit, and the first workgroup builds the whole list."""
    grid, win, tau, batch, n = (468, 468, 32), (12, 12, 8), 36, 2, 150000
    frames = []
    for b in range(batch):
        c = synth.frame_uniform(700 + b, grid, n)
        frames.append(np.concatenate([np.full((len(c), 1), b, np.int64), c], 1))
    coords = np.concatenate(frames).astype(np.int32)
    pc = dsvt.part_cfg(grid, win, (0, 0, 0), tau, batch, 0)
    bound = dsvt.binding.dsvt_partition_bound(pc, len(coords))[0]
    oms = [orc.partition(coords, grid, win, (0, 0, 0), tau, a) for a in (0, 1)]
    _say(f"work list, bound {bound} sets, {oms[0]['n_sets']} sets")
    assert bound > 16384 >= oms[0]["n_sets"]
    pair = dsvt.dsvt_partition_xy(pc, dev_coords(coords))
    for axis in (0, 1):
        assert_maps_equal(pair[axis], oms[axis])


def test_short_tile_list_on_a_frame_built_in_pieces():
    """The skewed batch has more sets than one workgroup's tables hold, so its work list is built piece by piece; with
    a tile list shorter than it needs, the call reports DSVT_ST_TILE_OVERFLOW, leaves the list empty (the maps are
    still exact) and a block over it runs without touching a row; the same buffers then take the full list."""
    cfg = synth.CONFIGS[5]
    coords = synth.make_frame(5, n=None)
    shift = cfg["shifts"][0]
    pc = dsvt.part_cfg(cfg["grid"], cfg["win"], shift, cfg["tau"], cfg["batch"], 0)
    _say(f"short tile list, cfg5 n={len(coords)}")
    cd = dev_coords(coords)
    oms = [orc.partition(coords, cfg["grid"], cfg["win"], shift, cfg["tau"], a) for a in (0, 1)]
    assert oms[0]["n_sets"] > 16384
    short = dsvt.SetMapsXY(pc, len(coords), max_tiles=1000)
    dsvt.dsvt_partition_xy(pc, cd, out=short)
    torch.cuda.synchronize()
    assert int(short.x.status.item()) == dsvt.binding.ST_TILE_OVERFLOW and int(short.x.n_tiles.item()) == 0
    for axis in (0, 1):
        ns = oms[axis]["n_sets"]
        assert int(short[axis].n_sets.item()) == ns
        assert np.array_equal(short[axis].set_inds[:ns].cpu().numpy(), oms[axis]["set_inds"])
        assert np.array_equal(short[axis].voxel_slot.cpu().numpy(), oms[axis]["voxel_slot"])
    x = dev_feats(synth.make_features(35, len(coords), cfg["C"], cfg["dtype"]), cfg["dtype"])
    mk = lambda sd: synth.make_layer_weights(sd, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], cfg["dtype"], True)
    out = torch.full_like(x, 7.0)
    dsvt.dsvt_block([dsvt.LayerWeights(mk(66)), dsvt.LayerWeights(mk(67))], short, cd, x, x_out=out)
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)
    full = dsvt.SetMapsXY(pc, len(coords))
    full.x.ws = full.y.ws = short.x.ws
    dsvt.dsvt_partition_xy(pc, cd, out=full)
    torch.cuda.synchronize()
    assert int(full.x.status.item()) == 0
    for axis in (0, 1):
        assert_maps_equal(full[axis], oms[axis])


# ------------------------------------------------------------------ set attention / block
def _layer_case(cid, n, seed, rel_bias=True, shift=None):
    cfg = synth.CONFIGS[cid]
    coords = synth.make_frame(cid, n=n)
    x = synth.make_features(seed, len(coords), cfg["C"], cfg["dtype"])
    shift = cfg["shifts"][-1] if shift is None else shift
    mk = lambda s: synth.make_layer_weights(s, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], cfg["dtype"], rel_bias)
    return cfg, coords, x, shift, mk


@pytest.mark.parametrize("cid,n", [(1, None), (2, 5000), (3, 8000), (5, 12000)])
@pytest.mark.parametrize("dup_mode", [0, 1])
@pytest.mark.parametrize("rel_bias", [True, False])
def test_set_attention_parity(cid, n, dup_mode, rel_bias):
    cfg, coords, x, shift, mk = _layer_case(cid, n, 31, rel_bias)
    w = mk(61)
    _say(f"set_attention cfg{cid} n={len(coords)} dup={dup_mode} pe={rel_bias}")
    om = orc.partition(coords, cfg["grid"], cfg["win"], shift, cfg["tau"], 1)
    ref = orc.set_attention(w, om, coords, x, dup_mode)
    cd = dev_coords(coords)
    gm = gpu_maps(cd, cfg["grid"], cfg["win"], shift, cfg["tau"], cfg["batch"], 1)
    y = dsvt.dsvt_set_attention(dsvt.LayerWeights(w, dup_mode), gm, cd, dev_feats(x, cfg["dtype"]))
    torch.cuda.synchronize()
    err = rel_err(y, ref)
    _say(f"  rel err {err:.3e}")
    assert err < TOL[cfg["dtype"]]


@pytest.mark.parametrize("tiles", [True, False])
@pytest.mark.parametrize("cid,n", [(1, None), (2, 5000), (3, 8000), (5, 30000)])
def test_block_parity(cid, n, tiles):
    cfg, coords, x, shift, mk = _layer_case(cid, n, 32)
    ws = [mk(71), mk(72)]
    _say(f"block cfg{cid} n={len(coords)} tiles={tiles}")
    oms = [orc.partition(coords, cfg["grid"], cfg["win"], shift, cfg["tau"], a) for a in (0, 1)]
    ref = orc.block(ws, oms, coords, x)
    cd = dev_coords(coords)
    gms = [gpu_maps(cd, cfg["grid"], cfg["win"], shift, cfg["tau"], cfg["batch"], a, tiles) for a in (0, 1)]
    xd = dev_feats(x, cfg["dtype"])
    out = dsvt.dsvt_block([dsvt.LayerWeights(w) for w in ws], gms, cd, xd)
    torch.cuda.synchronize()
    err = rel_err(out, ref)
    _say(f"  rel err {err:.3e}")
    assert err < TOL[cfg["dtype"]]
    # in place gives the same bits
    again = dsvt.dsvt_block([dsvt.LayerWeights(w) for w in ws], gms, cd, xd, x_out=xd)
    torch.cuda.synchronize()
    assert again.data_ptr() == xd.data_ptr() and torch.equal(again, out)


@pytest.mark.timeout(400)                     # (the oracle needs most of a minute for the voxel frame)
@pytest.mark.parametrize("cid,launch", [(2, "eager"), (2, "hip_graph"), (3, "hip_graph")])
def test_stack_parity_full_pillar_frame(cid, launch):
    """The benchmark workloads in the launch configuration the benchmark times: the 30,000-pillar frame (4 blocks x
    2 layers) and the 120,000-voxel frame (2 blocks, filled tiles from the general front end), both window shifts
    partitioned by one call, everything on one stream, eagerly and as a replayed HIP graph."""
    cfg, coords, x, _, _ = _layer_case(cid, None, 33)
    ws = [[synth.make_layer_weights(200 + 2 * b + a, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], cfg["dtype"])
           for a in (0, 1)] for b in range(cfg["blocks"])]
    _say(f"stack cfg{cid} full frame, {launch}")
    ref = orc.stack(ws, coords, x, cfg["grid"], cfg["win"], cfg["shifts"], cfg["tau"])
    cd = dev_coords(coords)
    shifts = list(cfg["shifts"])
    pcs = [dsvt.part_cfg(cfg["grid"], cfg["win"], sh, cfg["tau"], 1, 0) for sh in shifts]
    maps = [dsvt.SetMapsXY(pc, len(coords)) for pc in pcs]
    layers = [[dsvt.LayerWeights(w) for w in pair] for pair in ws]
    x0 = dev_feats(x, cfg["dtype"])
    buf = torch.empty_like(x0)
    wsb = torch.empty((max(dsvt.dsvt_block_workspace_size(layers[0][0], len(coords)), 1),), dtype=torch.uint8, device="cuda")

    def step():
        dsvt.dsvt_partition_xy_multi(pcs, cd, maps)
        src = x0
        for b, pair in enumerate(layers):
            dsvt.dsvt_block(pair, maps[b % len(shifts)], cd, src, x_out=buf, ws=wsb)
            src = buf

    if launch == "eager":
        step()
    else:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(3):
            buf.zero_()
            graph.replay()
    torch.cuda.synchronize()
    for m, sh in zip(maps, shifts):
        for axis in (0, 1):
            assert_maps_equal(m[axis], orc.partition(coords, cfg["grid"], cfg["win"], sh, cfg["tau"], axis))
    err = rel_err(buf, ref)
    _say(f"  rel err after {2 * cfg['blocks']} layers {err:.3e}")
    assert err < TOL["bf16"]


@pytest.mark.timeout(900)
def test_stack_parity_full_skewed_batch(capsys):
    """The 4 x 200,000-voxel skewed batch (windows 12 x 12 x 32 holding 1 to ~1,850 voxels, tau 36) through the full
    4-block rotated stack at full size, in the launch configuration the benchmark times: both window shifts
    partitioned by one dsvt_partition_xy_multi call, four dsvt_block calls on one stream, eagerly and as a replayed
    HIP graph.  All four maps bit-exact, all 800,000 rows of the output against the oracle.  The oracle takes about
    two minutes here; it reports after every block so that the run is seen to be alive."""
    cfg, coords, x, _, _ = _layer_case(5, None, 33)
    ws = [[synth.make_layer_weights(200 + 2 * b + a, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], cfg["dtype"])
           for a in (0, 1)] for b in range(cfg["blocks"])]

    def progress(msg):
        with capsys.disabled():
            print(f"[case] {msg}", flush=True)

    progress(f"stack cfg5 full batch: {len(coords)} voxels, {cfg['blocks']} blocks")
    cd = dev_coords(coords)
    shifts = list(cfg["shifts"])
    pcs = [dsvt.part_cfg(cfg["grid"], cfg["win"], sh, cfg["tau"], cfg["batch"], 0) for sh in shifts]
    maps = [dsvt.SetMapsXY(pc, len(coords)) for pc in pcs]
    layers = [[dsvt.LayerWeights(w) for w in pair] for pair in ws]
    x0 = dev_feats(x, cfg["dtype"])
    buf = torch.empty_like(x0)

    def step():
        dsvt.dsvt_partition_xy_multi(pcs, cd, maps)
        src = x0
        for b, pair in enumerate(layers):
            dsvt.dsvt_block(pair, maps[b % len(shifts)], cd, src, x_out=buf)
            src = buf

    step()
    torch.cuda.synchronize()
    eager = buf.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(3):
        buf.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(buf, eager)
    progress("  GPU: eager and three graph replays agree bit for bit")
    omaps = []
    for m, sh in zip(maps, shifts):
        oms = [orc.partition(coords, cfg["grid"], cfg["win"], sh, cfg["tau"], axis) for axis in (0, 1)]
        for axis in (0, 1):
            assert_maps_equal(m[axis], oms[axis])
        omaps.append(oms)
        progress(f"  maps of shift {sh} bit-exact ({oms[0]['n_sets']} sets, largest window {int(oms[0]['win_counts'].max())} voxels)")
    ref = x
    for b, pair in enumerate(ws):                 # blocks alternate between the shifts (orc.stack does the same; pinned on the CPU)
        ref = orc.block(pair, omaps[b % len(shifts)], coords, ref)
        progress(f"  oracle block {b} done")
    err = rel_err(eager, ref)
    progress(f"  rel err after {2 * cfg['blocks']} layers {err:.3e}")
    assert err < TOL["bf16"]


def test_layer_argument_errors():
    cfg, coords, x, shift, mk = _layer_case(1, 300, 34)
    cd = dev_coords(coords)
    gm = gpu_maps(cd, cfg["grid"], cfg["win"], shift, cfg["tau"], 1, 0)
    w = mk(81)
    w_bad = dict(w); w_bad["C"], w_bad["heads"] = 96, 4
    lw = dsvt.LayerWeights(w)
    lw.struct.C = 96
    lw.C = 96
    with pytest.raises(dsvt.DsvtError) as e:
        dsvt.dsvt_set_attention(lw, gm, cd, torch.zeros((300, 96), device="cuda"))
    assert e.value.rc == dsvt.binding.DSVT_EUNSUPPORTED


# ------------------------------------------------------------------ attention-style pooling
@pytest.mark.parametrize("cid,n,pool", [(1, None, (2, 2, 1)), (4, 20000, (1, 1, 4)), (4, 6000, (2, 2, 2)),
                                        (4, None, (1, 1, 4))])
@pytest.mark.parametrize("mask_empty", [1, 0])
def test_attn_pool_parity(cid, n, pool, mask_empty):
    cfg = synth.CONFIGS[cid]
    coords = synth.make_frame(cid, n=n)
    x = synth.make_features(35, len(coords), cfg["C"], cfg["dtype"])
    w = synth.make_pool_weights(91, cfg["C"], cfg["heads"], cfg["dtype"])
    _say(f"attn_pool cfg{cid} n={len(coords)} pool={pool} mask_empty={mask_empty}")
    ref_c, ref = orc.attn_pool(w, coords, x, cfg["grid"], pool, mask_empty)
    pw = dsvt.PoolWeights(w, cfg["grid"], pool, cfg["batch"], mask_empty)
    oc, out, n_out, status = dsvt.dsvt_attn_pool(pw, dev_coords(coords), dev_feats(x, cfg["dtype"]))
    torch.cuda.synchronize()
    m = int(n_out.item())
    assert int(status.item()) == 0 and m == len(ref_c) < len(coords)
    assert np.array_equal(oc[:m].cpu().numpy(), ref_c)            # coordinates and order bit-exact
    err = rel_err(out[:m], ref)
    _say(f"  regions {m}, rel err {err:.3e}")
    assert err < TOL[cfg["dtype"]]
    assert torch.all(out[m:] == 0) and torch.all(oc[m:] == 0)     # rows past n_out untouched


@pytest.mark.parametrize("pool,fill", [((2, 2, 2), 1.0), ((2, 2, 2), 0.7), ((1, 1, 4), 1.0), ((2, 1, 1), 0.9)])
def test_attn_pool_dense_regions(pool, fill):
    """Regions that are (nearly) full: a workgroup's 48 regions then hold several 96-row tiles of occupied cells
    and are processed in several passes."""
    grid, C, heads = (16, 16, 8), 64, 4
    rng = np.random.Generator(np.random.Philox(77))
    cells = np.argwhere(rng.random(grid) < fill)
    coords = np.concatenate([np.zeros((len(cells), 1), np.int64), cells], 1).astype(np.int32)
    coords = coords[rng.permutation(len(coords))]
    x = synth.make_features(36, len(coords), C, "f32")
    w = synth.make_pool_weights(92, C, heads, "f32")
    _say(f"attn_pool dense pool={pool} fill={fill} n={len(coords)}")
    for mask_empty in (0, 1):
        ref_c, ref = orc.attn_pool(w, coords, x, grid, pool, mask_empty)
        pw = dsvt.PoolWeights(w, grid, pool, 1, mask_empty)
        oc, out, n_out, status = dsvt.dsvt_attn_pool(pw, dev_coords(coords), dev_feats(x, "f32"))
        torch.cuda.synchronize()
        m = int(n_out.item())
        assert int(status.item()) == 0 and m == len(ref_c)
        assert np.array_equal(oc[:m].cpu().numpy(), ref_c)
        err = rel_err(out[:m], ref)
        _say(f"  mask_empty {mask_empty}: regions {m}, rel err {err:.3e}")
        assert err < TOL["f32"]


@pytest.mark.timeout(400)
@pytest.mark.parametrize("n", [30000, None])
def test_attn_pool_then_block(n):
    """The pooled voxels feed a rotated layer pair on the pooled grid (window 12 x 12 x 8, tau 48); n = None is the
    workload's full 120,000-voxel frame (107,564 pooled voxels)."""
    cfg = synth.CONFIGS[4]
    coords = synth.make_frame(4, n=n)
    x = synth.make_features(36, len(coords), cfg["C"], cfg["dtype"])
    w = synth.make_pool_weights(92, cfg["C"], cfg["heads"], cfg["dtype"])
    ws = [synth.make_layer_weights(93 + a, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], cfg["dtype"]) for a in (0, 1)]
    pgrid = (468, 468, 8)
    _say(f"attn_pool + block on the pooled grid, {len(coords)} voxels")
    ref_c, ref_p = orc.attn_pool(w, coords, x, cfg["grid"], cfg["pool"], 1)
    ref_p16 = synth.round_bf16(ref_p.astype(np.float32))          # the GPU hands bf16 features to the block
    oms = [orc.partition(ref_c, pgrid, cfg["win"], (0, 0, 0), cfg["tau"], a) for a in (0, 1)]
    ref = orc.block(ws, oms, ref_c, ref_p16)
    pw = dsvt.PoolWeights(w, cfg["grid"], cfg["pool"], 1, 1)
    oc, out, n_out, _ = dsvt.dsvt_attn_pool(pw, dev_coords(coords), dev_feats(x, "bf16"))
    m = int(n_out.item())
    pc, px = oc[:m].contiguous(), out[:m].contiguous()
    gms = [gpu_maps(pc, pgrid, cfg["win"], (0, 0, 0), cfg["tau"], 1, a) for a in (0, 1)]
    for gm, om in zip(gms, oms):
        assert_maps_equal(gm, om)
    y = dsvt.dsvt_block([dsvt.LayerWeights(v) for v in ws], gms, pc, px)
    torch.cuda.synchronize()
    err = rel_err(y, ref)
    _say(f"  rel err {err:.3e}")
    assert err < TOL["bf16"]


# ------------------------------------------------------------------ edge cases and wider shapes
@pytest.mark.parametrize("n", [1, 2, 36, 37])
def test_block_on_tiny_inputs(n):
    """A lone voxel (softmax over one key), a pair, exactly tau and tau + 1 voxels in one window."""
    cfg = synth.CONFIGS[1]
    coords = np.concatenate([np.zeros((n, 1), np.int64), synth.frame_uniform(5, (12, 12, 1), n)], 1).astype(np.int32)
    x = synth.make_features(51, n, cfg["C"], "f32")
    ws = [synth.make_layer_weights(52 + a, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], "f32") for a in (0, 1)]
    _say(f"block on {n} voxels")
    oms = [orc.partition(coords, (12, 12, 1), cfg["win"], (0, 0, 0), cfg["tau"], a) for a in (0, 1)]
    ref = orc.block(ws, oms, coords, x)
    cd = dev_coords(coords)
    gms = [gpu_maps(cd, (12, 12, 1), cfg["win"], (0, 0, 0), cfg["tau"], 1, a) for a in (0, 1)]
    for gm, om in zip(gms, oms):
        assert_maps_equal(gm, om)
    out = dsvt.dsvt_block([dsvt.LayerWeights(w) for w in ws], gms, cd, dev_feats(x, "f32"))
    torch.cuda.synchronize()
    assert rel_err(out, ref) < TOL["f32"]


def test_crowded_window_many_sets():
    """One 12x12x32 window holding 1,700 voxels: 48 sets from a single window, plus lone voxels elsewhere."""
    cfg = synth.CONFIGS[5]
    grid = (24, 24, 32)
    dense = synth.frame_uniform(61, (12, 12, 32), 1700)
    lone = np.array([[13, 2, 5], [20, 20, 31], [2, 23, 0]])
    coords = np.concatenate([np.zeros((1703, 1), np.int64), np.concatenate([dense, lone])], 1).astype(np.int32)
    coords = coords[np.random.Generator(np.random.Philox(3)).permutation(len(coords))]
    x = synth.make_features(62, len(coords), cfg["C"], "bf16")
    w = synth.make_layer_weights(63, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], "bf16")
    _say("crowded window: 1700 voxels, tau 36")
    for dup_mode in (0, 1):
        om = orc.partition(coords, grid, cfg["win"], (0, 0, 0), 36, 0)
        assert om["n_sets"] == 48 + 3
        ref = orc.set_attention(w, om, coords, x, dup_mode)
        cd = dev_coords(coords)
        gm = gpu_maps(cd, grid, cfg["win"], (0, 0, 0), 36, 1, 0)
        assert_maps_equal(gm, om)
        y = dsvt.dsvt_set_attention(dsvt.LayerWeights(w, dup_mode), gm, cd, dev_feats(x, "bf16"))
        torch.cuda.synchronize()
        assert rel_err(y, ref) < TOL["bf16"]


@pytest.mark.parametrize("second", [24, 36])
def test_hybrid_window_sizes(second):
    """Blocks alternating window (12,12,1) and a shifted larger window: (24,24,1), the paper's default
    hybrid partition ("Hybrid window partition"; DSVT-P uses (12,12,1) and (24,24,1)), and (36,36,1), the
    third row of its hybrid-window ablation."""
    cfg = synth.CONFIGS[2]
    coords = synth.make_frame(2, n=6000)
    x = synth.make_features(71, len(coords), cfg["C"], "bf16")
    wins = [((12, 12, 1), (0, 0, 0)), ((second, second, 1), (second // 2, second // 2, 0))]
    ws = [[synth.make_layer_weights(72 + 2 * b + a, cfg["C"], cfg["heads"], cfg["hidden"], wins[b][0], "bf16")
           for a in (0, 1)] for b in range(2)]
    _say(f"hybrid window sizes 12x12 / shifted {second}x{second}")
    cd = dev_coords(coords)
    ref, xd = x, dev_feats(x, "bf16")
    for b, (win, shift) in enumerate(wins):
        oms = [orc.partition(coords, cfg["grid"], win, shift, cfg["tau"], a) for a in (0, 1)]
        ref = orc.block(ws[b], oms, coords, ref)
        gms = [gpu_maps(cd, cfg["grid"], win, shift, cfg["tau"], 1, a) for a in (0, 1)]
        for gm, om in zip(gms, oms):
            assert_maps_equal(gm, om)
        xd = dsvt.dsvt_block([dsvt.LayerWeights(w) for w in ws[b]], gms, cd, xd)
    torch.cuda.synchronize()
    err = rel_err(xd, ref)
    _say(f"  rel err {err:.3e}")
    assert err < TOL["bf16"]


def test_gpu_path_is_permutation_invariant():
    """Permuting the input voxels permutes the outputs, bit for bit (no arrival-order dependence)."""
    cfg = synth.CONFIGS[2]
    coords = synth.make_frame(2, n=5000)
    x = synth.make_features(81, len(coords), cfg["C"], "bf16")
    ws = [synth.make_layer_weights(82 + a, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], "bf16") for a in (0, 1)]
    perm = np.random.Generator(np.random.Philox(8)).permutation(len(coords))
    outs = []
    for c, f in ((coords, x), (coords[perm], x[perm])):
        cd = dev_coords(c)
        gms = [gpu_maps(cd, cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], 1, a) for a in (0, 1)]
        outs.append(dsvt.dsvt_block([dsvt.LayerWeights(w) for w in ws], gms, cd, dev_feats(f, "bf16")))
    torch.cuda.synchronize()
    assert torch.equal(outs[1], outs[0][torch.as_tensor(perm).cuda()])


def test_full_size_skewed_batch_sampled():
    """The 4 x 200,000-voxel skewed batch at full size: maps bit-exact, one layer checked on the voxels of
    sampled sets (the oracle evaluates only the sets that hold them)."""
    cfg = synth.CONFIGS[5]
    coords = synth.make_frame(5)
    x = synth.make_features(91, len(coords), cfg["C"], "bf16")
    w = synth.make_layer_weights(92, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], "bf16")
    _say("skewed batch, full size, sampled sets")
    om = orc.partition(coords, cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], 1)
    cd = dev_coords(coords)
    gm = gpu_maps(cd, cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], cfg["batch"], 1)
    assert_maps_equal(gm, om)
    y = dsvt.dsvt_set_attention(dsvt.LayerWeights(w), gm, cd, dev_feats(x, "bf16"))
    torch.cuda.synchronize()
    pick = np.random.Generator(np.random.Philox(9)).choice(om["n_sets"], 400, replace=False)
    sub = dict(om, set_inds=om["set_inds"][pick], n_sets=len(pick))
    members = np.unique(sub["set_inds"])
    slot = {int(v): int(i) for i, v in reversed(list(enumerate(sub["set_inds"].reshape(-1))))}
    sub["voxel_slot"] = np.array([slot[int(v)] for v in members], np.int32)
    ref = orc.set_attention(w, sub, coords, x)
    err = rel_err(y[torch.as_tensor(members).cuda()], ref)
    _say(f"  {len(members)} sampled voxels, rel err {err:.3e}")
    assert err < TOL["bf16"]


def test_width_128_large_window():
    """The nuScenes variant's widths (128 channels, 8 heads, hidden 256, window 30 x 30 x 1; appendix
    "3D Perception on nuScenes") at the largest supported set size, tau = 48."""
    C, heads, hidden, win, tau, grid = 128, 8, 256, (30, 30, 1), 48, (360, 360, 1)
    coords = np.concatenate([np.zeros((9000, 1), np.int64), synth.frame_radial(95, grid, 9000)], 1).astype(np.int32)
    x = synth.make_features(96, len(coords), C, "bf16")
    ws = [synth.make_layer_weights(97 + a, C, heads, hidden, win, "bf16") for a in (0, 1)]
    _say("C=128 window 30x30 tau=48")
    oms = [orc.partition(coords, grid, win, (15, 15, 0), tau, a) for a in (0, 1)]
    ref = orc.block(ws, oms, coords, x)
    cd = dev_coords(coords)
    gms = [gpu_maps(cd, grid, win, (15, 15, 0), tau, 1, a) for a in (0, 1)]
    for gm, om in zip(gms, oms):
        assert_maps_equal(gm, om)
    out = dsvt.dsvt_block([dsvt.LayerWeights(w) for w in ws], gms, cd, dev_feats(x, "bf16"))
    pw = synth.make_pool_weights(98, C, heads, "bf16")
    rc_, rp = orc.attn_pool(pw, coords, x, grid, (2, 2, 1), 0)
    oc, po, n_out, _ = dsvt.dsvt_attn_pool(dsvt.PoolWeights(pw, grid, (2, 2, 1), 1, 0), cd, dev_feats(x, "bf16"))
    torch.cuda.synchronize()
    err, m = rel_err(out, ref), int(n_out.item())
    _say(f"  block rel err {err:.3e}")
    assert err < TOL["bf16"]
    assert m == len(rc_) and np.array_equal(oc[:m].cpu().numpy(), rc_) and rel_err(po[:m], rp) < TOL["bf16"]


@pytest.mark.timeout(600)
@pytest.mark.parametrize("xy,n", [(96, 5000), (468, 120000)])
def test_dsvt_v_four_stages(xy, n):
    """The voxel variant's stage layout (appendix "Network Architecture": four stages, one block each here,
    windows 12 x 12 x {32, 8, 2, 1}, tau = 48, attention-style pooling by {4, 4, 2} along z between stages),
    chained end to end: every stage's maps and pooled coordinates bit-exact, the last stage's features in
    tolerance.  The oracle rounds the features to bf16 where the GPU path stores them (after each call).  Once on a
    small grid, once at frame size (468 x 468 x 32, 120,000 voxels)."""
    C, heads, hidden, tau = 192, 8, 384, 48
    grid0 = (xy, xy, 32)
    coords = np.concatenate([np.zeros((n, 1), np.int64), synth.frame_radial(311, grid0, n)], 1).astype(np.int32)
    x = synth.make_features(312, len(coords), C, "bf16")
    zs, strides = [32, 8, 2, 1], [4, 4, 2]
    _say(f"DSVT-V stage chain: 4 blocks, 3 poolings, {n} voxels on {grid0}")
    ref_c, ref_x = coords, x
    cd, xd = dev_coords(coords), dev_feats(x, "bf16")
    for st, z in enumerate(zs):
        grid, win, shift = (xy, xy, z), (12, 12, z), ((0, 0, 0) if st % 2 == 0 else (6, 6, 0))
        ws = [synth.make_layer_weights(320 + 2 * st + a, C, heads, hidden, win, "bf16") for a in (0, 1)]
        oms = [orc.partition(ref_c, grid, win, shift, tau, a) for a in (0, 1)]
        ref_x = synth.round_bf16(orc.block(ws, oms, ref_c, ref_x).astype(np.float32))
        gms = [gpu_maps(cd, grid, win, shift, tau, 1, a) for a in (0, 1)]
        for gm, om in zip(gms, oms):
            assert_maps_equal(gm, om)
        xd = dsvt.dsvt_block([dsvt.LayerWeights(w) for w in ws], gms, cd, xd)
        torch.cuda.synchronize()
        err = rel_err(xd, ref_x)
        _say(f"  stage {st} (z = {z}, {len(ref_c)} voxels): block rel err {err:.3e}")
        assert err < TOL["bf16"]
        if st < len(strides):
            pool = (1, 1, strides[st])
            pw = synth.make_pool_weights(340 + st, C, heads, "bf16")
            ref_c, ref_p = orc.attn_pool(pw, ref_c, ref_x, grid, pool, 1)
            ref_x = synth.round_bf16(ref_p.astype(np.float32))
            oc, po, n_out, _ = dsvt.dsvt_attn_pool(dsvt.PoolWeights(pw, grid, pool, 1, 1), cd, xd)
            m = int(n_out.item())
            assert m == len(ref_c) and np.array_equal(oc[:m].cpu().numpy(), ref_c)
            cd, xd = oc[:m].contiguous(), po[:m].contiguous()
            assert rel_err(xd, ref_x) < TOL["bf16"]


@pytest.mark.parametrize("C,heads,hidden,win,tau,n", [(128, 8, 256, (30, 30, 1), 90, 9000), (192, 8, 384, (12, 12, 1), 60, 9000),
                                                      (64, 4, 128, (12, 12, 1), 96, 9000)])
def test_large_sets(C, heads, hidden, win, tau, n):
    """Sets of more than 48 voxels (the nuScenes variant uses tau = 90 with 30 x 30 windows, appendix "3D
    Perception on nuScenes"; the ablation on set size goes up to 60): a set then spans four to six key
    tiles and is attended one head per work item."""
    grid = (360, 360, 1) if win[0] == 30 else (96, 96, 1)
    shift = (win[0] // 2, win[1] // 2, 0)
    coords = np.concatenate([np.zeros((n, 1), np.int64), synth.frame_radial(400 + tau, grid, n)], 1).astype(np.int32)
    x = synth.make_features(401 + tau, len(coords), C, "bf16")
    ws = [synth.make_layer_weights(402 + a, C, heads, hidden, win, "bf16") for a in (0, 1)]
    _say(f"C={C} window {win} tau={tau}")
    oms = [orc.partition(coords, grid, win, shift, tau, a) for a in (0, 1)]
    ref = orc.block(ws, oms, coords, x)
    cd = dev_coords(coords)
    gms = [gpu_maps(cd, grid, win, shift, tau, 1, a) for a in (0, 1)]
    for gm, om in zip(gms, oms):
        assert_maps_equal(gm, om)
    out = dsvt.dsvt_block([dsvt.LayerWeights(w) for w in ws], gms, cd, dev_feats(x, "bf16"))
    torch.cuda.synchronize()
    err = rel_err(out, ref)
    nu_max = max(int((np.diff(np.r_[om["set_inds"][s], -7]) != 0).sum()) for om in oms for s in range(0, om["n_sets"], 7))
    _say(f"  rel err {err:.3e}; largest sampled set {nu_max} voxels")
    assert err < TOL["bf16"]


@pytest.mark.parametrize("tau", [24, 36, 48, 60])
def test_set_size_sweep(tau):
    """The set sizes of the paper's set-size ablation (24, 36, 48 for pillars; 36, 48, 60 for voxels) on the pillar
    shape, maps from the paired partition call."""
    C, heads, hidden, grid, win, n = 192, 8, 384, (144, 144, 1), (12, 12, 1), 7000
    shift = (6, 6, 0)
    coords = np.concatenate([np.zeros((n, 1), np.int64), synth.frame_radial(500 + tau, grid, n)], 1).astype(np.int32)
    x = synth.make_features(501 + tau, len(coords), C, "bf16")
    ws = [synth.make_layer_weights(502 + a, C, heads, hidden, win, "bf16") for a in (0, 1)]
    _say(f"set size tau={tau}")
    oms = [orc.partition(coords, grid, win, shift, tau, a) for a in (0, 1)]
    ref = orc.block(ws, oms, coords, x)
    cd = dev_coords(coords)
    gms = dsvt.dsvt_partition_xy(dsvt.part_cfg(grid, win, shift, tau, 1, 0), cd)
    for gm, om in zip(gms, oms):
        assert_maps_equal(gm, om)
    out = dsvt.dsvt_block([dsvt.LayerWeights(w) for w in ws], gms, cd, dev_feats(x, "bf16"))
    torch.cuda.synchronize()
    err = rel_err(out, ref)
    _say(f"  sets {oms[0]['n_sets']}, rel err {err:.3e}")
    assert err < TOL["bf16"]


@pytest.mark.parametrize("dt,C,grid,batch,n", [("bf16", 192, (468, 468, 1), 1, 30000), ("f32", 64, (48, 48, 1), 1, 2000),
                                               ("bf16", 128, (37, 29, 3), 2, 1500)])
def test_bev_scatter_bit_exact(dt, C, grid, batch, n):
    """Sec. 3.1 overview: sparse voxel rows -> dense channels-last bird's-eye-view map; a copy, so bit-exact."""
    coords = np.concatenate([np.concatenate([np.full((n, 1), b, np.int64), synth.frame_uniform(500 + b, grid, n)], 1)
                             for b in range(batch)]).astype(np.int32)
    x = synth.make_features(501, len(coords), C, dt)
    _say(f"bev scatter {dt} C={C} grid={grid} batch={batch}")
    ref = orc.bev_scatter(coords, x, batch, grid)
    out, status = dsvt.dsvt_bev_scatter(dev_coords(coords), dev_feats(x, dt), batch, grid)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    assert np.array_equal(out.float().cpu().numpy(), ref.astype(np.float32))
    bad = coords.copy(); bad[3, 1] = grid[0]                     # out of range: reported, skipped, nothing else disturbed
    out2, status2 = dsvt.dsvt_bev_scatter(dev_coords(bad), dev_feats(x, dt), batch, grid)
    torch.cuda.synchronize()
    assert int(status2.item()) & 1
    ref2 = ref.copy(); ref2[tuple(coords[3])] = 0
    assert np.array_equal(out2.float().cpu().numpy(), ref2.astype(np.float32))


# ------------------------------------------------- set-partition baselines of the ablation (Sec. 4.4)
@pytest.mark.parametrize("cid,n", [(1, None), (2, 9000), (3, 20000), (5, 30000)])
@pytest.mark.parametrize("axis", [2, 3, 4, 5])
def test_partition_variants_bit_exact(cid, n, axis):
    """Random (2, 3) and Sparse (4, 5) inner-window orders: single-map call, through the small-frame and the
    general front end (cfg 5's windows hold up to 1,800 voxels)."""
    cfg = synth.CONFIGS[cid]
    coords = synth.make_frame(cid, n=n)
    shift = cfg["shifts"][-1]
    _say(f"partition variant axis={axis} cfg{cid} n={len(coords)}")
    om = orc.partition(coords, cfg["grid"], cfg["win"], shift, cfg["tau"], axis)
    assert_maps_equal(gpu_maps(dev_coords(coords), cfg["grid"], cfg["win"], shift, cfg["tau"], cfg["batch"], axis), om)


@pytest.mark.parametrize("axis0", [2, 4])
def test_partition_variant_pairs_and_block(axis0):
    """The pair call yields (axis0, axis0 + 1); a block run on those maps matches the oracle's block on its own.
    Regional = the X-axis order in both layers."""
    cfg = synth.CONFIGS[2]
    coords = synth.make_frame(2, n=6000)
    x = synth.make_features(91, len(coords), cfg["C"], "bf16")
    ws = [synth.make_layer_weights(92 + a, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], "bf16") for a in (0, 1)]
    _say(f"variant pair axis0={axis0} + block; regional block")
    cd = dev_coords(coords)
    pair = dsvt.dsvt_partition_xy(dsvt.part_cfg(cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], 1, axis0), cd)
    oms = [orc.partition(coords, cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], axis0 + k) for k in (0, 1)]
    for k in (0, 1):
        assert_maps_equal(pair[k], oms[k])
    lw = [dsvt.LayerWeights(w) for w in ws]
    out = dsvt.dsvt_block(lw, pair, cd, dev_feats(x, "bf16"))
    err = rel_err(out, orc.block(ws, oms, coords, x))
    _say(f"  rel err {err:.3e}")
    assert err < TOL["bf16"]
    if axis0 == 2:
        om0 = orc.partition(coords, cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], 0)
        gm0 = gpu_maps(cd, cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], 1, 0)
        err = rel_err(dsvt.dsvt_block(lw, [gm0, gm0], cd, dev_feats(x, "bf16")), orc.block(ws, [om0, om0], coords, x))
        _say(f"  regional rel err {err:.3e}")
        assert err < TOL["bf16"]
    # an odd first order has no pair
    import ctypes as C
    bad = dsvt.part_cfg(cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], 1, 1)
    with pytest.raises(dsvt.DsvtError):
        dsvt.dsvt_partition_xy(bad, cd)


@pytest.mark.parametrize("seed", list(range(16)))
def test_partition_seeded_random_geometries(seed):
    """Seeded draws of grid, window, shift, set size, frame count and voxel count (all valid inputs): the paired
    call's maps equal the oracle's bit for bit and the work list is a valid tiling, whatever front end and tile
    policy the sizes select."""
    rng = np.random.Generator(np.random.Philox(7000 + seed))
    win = (int(rng.integers(2, 25)), int(rng.integers(2, 25)), int(rng.choice([1, 1, 2, 4, 8])))
    grid = (int(rng.integers(win[0], 300)), int(rng.integers(win[1], 300)), int(win[2] * rng.integers(1, 4)))
    shift = tuple(int(rng.integers(0, w)) for w in win)
    tau = int(rng.choice([4, 7, 12, 24, 36, 48, 60, 90]))
    batch = int(rng.choice([1, 1, 2, 3]))
    cells = grid[0] * grid[1] * grid[2]
    n = int(min(rng.integers(1, 40000), max(cells // 3, 1)))
    kind = int(rng.integers(0, 2))
    frames = []
    for b in range(batch):
        c = synth.frame_radial(7100 + 16 * seed + b, grid, n) if kind else synth.frame_uniform(7100 + 16 * seed + b, grid, n)
        frames.append(np.concatenate([np.full((len(c), 1), b, np.int64), c], 1))
    coords = np.concatenate(frames).astype(np.int32)
    _say(f"random geometry seed={seed} grid={grid} win={win} shift={shift} tau={tau} batch={batch} n={len(coords)}")
    pair = dsvt.dsvt_partition_xy(dsvt.part_cfg(grid, win, shift, tau, batch, 0), dev_coords(coords))
    for axis in (0, 1):
        assert_maps_equal(pair[axis], orc.partition(coords, grid, win, shift, tau, axis))


@pytest.mark.parametrize("seed", list(range(10)))
def test_block_seeded_random_shapes(seed):
    """Seeded draws of channel width, set size, window, shift and voxel count among the supported shapes: one block
    (paired partition call, both layers) against the oracle."""
    rng = np.random.Generator(np.random.Philox(7500 + seed))
    C, heads, hidden, dt = [(64, 4, 128, "f32"), (64, 4, 128, "bf16"), (128, 8, 256, "bf16"), (192, 8, 384, "bf16")][int(rng.integers(0, 4))]
    win = (int(rng.integers(3, 20)), int(rng.integers(3, 20)), int(rng.choice([1, 1, 2, 4])))
    grid = (int(rng.integers(win[0], 160)), int(rng.integers(win[1], 160)), int(win[2] * rng.integers(1, 3)))
    shift = tuple(int(rng.integers(0, w)) for w in win)
    tau = int(rng.choice([8, 20, 36, 48, 64, 90]))
    n = int(min(rng.integers(50, 9000), max(grid[0] * grid[1] * grid[2] // 3, 1)))
    coords = np.concatenate([np.zeros((n, 1), np.int64), synth.frame_radial(7600 + seed, grid, n)], 1).astype(np.int32)
    x = synth.make_features(7700 + seed, len(coords), C, dt)
    ws = [synth.make_layer_weights(7800 + 2 * seed + a, C, heads, hidden, win, dt) for a in (0, 1)]
    _say(f"random block seed={seed} C={C} {dt} grid={grid} win={win} shift={shift} tau={tau} n={n}")
    oms = [orc.partition(coords, grid, win, shift, tau, a) for a in (0, 1)]
    ref = orc.block(ws, oms, coords, x)
    cd = dev_coords(coords)
    gms = dsvt.dsvt_partition_xy(dsvt.part_cfg(grid, win, shift, tau, 1, 0), cd)
    for gm, om in zip(gms, oms):
        assert_maps_equal(gm, om)
    out = dsvt.dsvt_block([dsvt.LayerWeights(w) for w in ws], gms, cd, dev_feats(x, dt))
    torch.cuda.synchronize()
    err = rel_err(out, ref)
    _say(f"  rel err {err:.3e}")
    assert err < TOL[dt]
