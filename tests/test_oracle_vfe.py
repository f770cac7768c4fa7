"""Pins for the oracle's voxel feature encoding (Sec. 3.1 overview: points -> sparse voxels): the cell rule on
hand-placed points, special cases that reduce to a library routine, and invariants a wrong index, a dropped
bias or a min-for-max would break."""
import numpy as np

from oracle import dsvt_oracle as orc
from synth import frames

LO, SZ, GRID = (-4.0, -2.0, -1.0), (0.5, 0.25, 2.0), (16, 16, 1)


def test_cells_of_hand_placed_points():
    pts = np.array([[-4.0, -2.0, -1.0],        # range corner: cell (0, 0, 0)
                    [-3.5, -1.75, 0.99],       # exactly on a cell boundary: the higher cell (1, 1, 0)
                    [-3.5001, -1.7501, 0.0],   # just below it: (0, 0, 0)
                    [3.99, 1.99, 0.5],         # last cell (15, 15, 0)
                    [4.0, 0.0, 0.0],           # upper edge of the range: outside
                    [-4.01, 0.0, 0.0],         # below the range
                    [0.0, 0.0, 1.0],           # z at its upper edge: outside
                    [np.nan, 0.0, 0.0],
                    [0.0, 0.1, 0.0]], np.float32)
    cell, inside = orc.point_cells(pts, None, LO, SZ, GRID, 1)
    assert inside.tolist() == [True, True, True, True, False, False, False, False, True]
    assert cell[inside].tolist() == [[0, 0, 0, 0], [0, 1, 1, 0], [0, 0, 0, 0], [0, 15, 15, 0], [0, 8, 8, 0]]
    _, inside_b = orc.point_cells(pts[:2], np.array([1, 2]), LO, SZ, GRID, 2)
    assert inside_b.tolist() == [True, False]


def test_one_point_per_voxel_is_the_linear_map():
    rng = np.random.default_rng(3)
    cells = rng.permutation(256)[:40]
    pts = np.zeros((40, 5), np.float32)
    pts[:, 0] = LO[0] + (cells // 16 + 0.5) * SZ[0]
    pts[:, 1] = LO[1] + (cells % 16 + 0.5) * SZ[1]
    pts[:, 3:] = rng.random((40, 2))
    w, b = rng.normal(size=(7, 5)), rng.normal(size=7)
    coords, out = orc.voxel_max_vfe(pts, None, LO, SZ, GRID, 1, w, b)
    order = np.argsort(cells)
    assert coords[:, 1].tolist() == (cells[order] // 16).tolist() and coords[:, 2].tolist() == (cells[order] % 16).tolist()
    np.testing.assert_allclose(out, pts[order].astype(np.float64) @ w.T + b, rtol=1e-13)


def test_identity_map_is_a_segmented_maximum():
    pts, pb = frames.make_points(11, 3000, (-4, -2, -1), (4, 2, 1), f_in=5, batch=2)
    coords, out = orc.voxel_max_vfe(pts, pb, LO, SZ, GRID, 2)
    cell, inside = orc.point_cells(pts, pb, LO, SZ, GRID, 2)
    key = ((cell[:, 0] * 16 + cell[:, 1]) * 16 + cell[:, 2])[inside]
    order = np.argsort(key, kind="stable")
    ukeys, first = np.unique(key[order], return_index=True)
    want = np.maximum.reduceat(pts[inside][order].astype(np.float64), first, axis=0)     # library segmented max
    assert 0 < inside.sum() < len(pts)
    assert ((coords[:, 0] * 16 + coords[:, 1]) * 16 + coords[:, 2]).tolist() == ukeys.tolist()
    np.testing.assert_array_equal(out, want)
    # every voxel's position channels lie inside its own cell
    for a in range(3):
        t = (out[:, a] - LO[a]) / SZ[a]
        assert np.all(np.floor(t + 1e-4) >= coords[:, 1 + a] - 0) and np.all(t < coords[:, 1 + a] + 1 + 1e-4)


def test_point_order_and_relu_do_not_matter_the_way_they_should_not():
    pts, pb = frames.make_points(12, 2000, (-4, -2, -1), (4, 2, 1), f_in=4)
    rng = np.random.default_rng(5)
    w, b = rng.normal(size=(6, 4)), rng.normal(size=6)
    c0, y0 = orc.voxel_max_vfe(pts, pb, LO, SZ, GRID, 1, w, b)
    perm = rng.permutation(len(pts))
    c1, y1 = orc.voxel_max_vfe(pts[perm], pb[perm], LO, SZ, GRID, 1, w, b)
    np.testing.assert_array_equal(c0, c1)
    np.testing.assert_array_equal(y0, y1)
    _, yr = orc.voxel_max_vfe(pts, pb, LO, SZ, GRID, 1, w, b, relu=True)
    np.testing.assert_array_equal(yr, np.maximum(y0, 0.0))                  # max commutes with a monotone map
    assert (y0 < 0).any() and (yr == 0).any()
    # a max, not a min or a mean: adding a dominated copy of every point changes nothing, a dominating one does
    lower = pts.copy(); lower[:, 3] -= 1.0
    _, y2 = orc.voxel_max_vfe(np.concatenate([pts, lower]), np.concatenate([pb, pb]), LO, SZ, GRID, 1)
    _, y3 = orc.voxel_max_vfe(pts, pb, LO, SZ, GRID, 1)
    np.testing.assert_array_equal(y2, y3)
