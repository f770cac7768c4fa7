"""Synthetic LiDAR-shaped sparse voxel frames.

The paper evaluates on Waymo Open frames (about 150 m x 150 m at 0.32 m
pillars = 468 x 468 cells, 32 z-layers of 0.1875 m for the voxel variant;
"Implementation Details" and appendix "Network Architecture").  That data is
not available here, so every frame is a seeded stand-in with the same grid
shapes: occupied cells are drawn from a radial 1/r density around the grid
centre plus uniform clutter, with a height profile concentrated near the
ground.  Coordinates are unique integer cells, rows are (b, x, y, z) int32.
"""
import numpy as np

# Workloads: grid (X, Y, Z), voxel count, channel width, heads, FFN width,
# set size tau, window (L, W, H), the two window shifts used by alternating
# blocks, number of blocks, feature dtype, frames per call.
CONFIGS = {
    1: dict(name="tiny_pillar", grid=(48, 48, 1), n=2000, C=64, heads=4, hidden=128, tau=36,
            win=(12, 12, 1), shifts=((0, 0, 0),), blocks=1, dtype="f32", batch=1, kind="uniform"),
    2: dict(name="pillar_frame", grid=(468, 468, 1), n=30000, C=192, heads=8, hidden=384, tau=36,
            win=(12, 12, 1), shifts=((0, 0, 0), (6, 6, 0)), blocks=4, dtype="bf16", batch=1, kind="radial"),
    3: dict(name="voxel_frame", grid=(468, 468, 32), n=120000, C=192, heads=8, hidden=384, tau=48,
            win=(12, 12, 8), shifts=((0, 0, 0), (6, 6, 0)), blocks=2, dtype="bf16", batch=1, kind="radial3d"),
    4: dict(name="pooled_voxel_frame", grid=(468, 468, 32), n=120000, C=192, heads=8, hidden=384, tau=48,
            win=(12, 12, 8), shifts=((0, 0, 0),), blocks=1, dtype="bf16", batch=1, kind="radial3d",
            pool=(1, 1, 4)),
    5: dict(name="skewed_batch", grid=(468, 468, 32), n=200000, C=192, heads=8, hidden=384, tau=36,
            win=(12, 12, 32), shifts=((0, 0, 0), (6, 6, 0)), blocks=4, dtype="bf16", batch=4, kind="skewed"),
    # the nuScenes variant's shape (appendix "3D Perception on nuScenes": 0.3 m pillars over +-54 m, windows of
    # 30 x 30 pillars, set size 90, 128 channels)
    6: dict(name="nuscenes_pillar_frame", grid=(360, 360, 1), n=20000, C=128, heads=8, hidden=256, tau=90,
            win=(30, 30, 1), shifts=((0, 0, 0), (15, 15, 0)), blocks=4, dtype="bf16", batch=1, kind="radial"),
}


def _rng(seed):
    return np.random.Generator(np.random.Philox(int(seed)))


def bf16_bits(a):
    """Round fp32 values to bfloat16 (nearest, ties to even); return the uint16 patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def round_bf16(a):
    """fp32 array whose every value is exactly representable in bfloat16."""
    b = bf16_bits(a).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).reshape(np.shape(a))


def _unique_cells(draw, n, grid, rng):
    """Call draw(m) -> int64 [m,3] candidate cells until n distinct in-grid cells are collected."""
    X, Y, Z = grid
    seen = np.zeros(X * Y * Z, dtype=bool)
    out = []
    have = 0
    while have < n:
        c = draw(max(2 * (n - have), 1024))
        ok = (c[:, 0] >= 0) & (c[:, 0] < X) & (c[:, 1] >= 0) & (c[:, 1] < Y) & (c[:, 2] >= 0) & (c[:, 2] < Z)
        c = c[ok]
        lin = (c[:, 0] * Y + c[:, 1]) * Z + c[:, 2]
        _, first = np.unique(lin, return_index=True)
        first.sort()
        c, lin = c[first], lin[first]
        fresh = ~seen[lin]
        c, lin = c[fresh][: n - have], lin[fresh][: n - have]
        seen[lin] = True
        out.append(c)
        have += len(c)
    return np.concatenate(out, axis=0)


def frame_uniform(seed, grid, n):
    """n distinct cells drawn uniformly over the grid."""
    rng = _rng(seed)
    X, Y, Z = grid
    draw = lambda m: np.stack([rng.integers(0, X, m), rng.integers(0, Y, m), rng.integers(0, Z, m)], 1)
    return _unique_cells(draw, n, grid, rng)


def _radial_xy(rng, m, X, Y):
    r = rng.uniform(2.0, min(X, Y) / 2.0, m)          # area density ~ 1/r  <=>  r uniform
    th = rng.uniform(0.0, 2.0 * np.pi, m)
    return np.floor(X / 2.0 + r * np.cos(th)).astype(np.int64), np.floor(Y / 2.0 + r * np.sin(th)).astype(np.int64)


def frame_radial(seed, grid, n, clutter=0.2, ground_layers=12):
    """80 % radial 1/r around the centre, 20 % uniform clutter; for Z > 1 the height is
    a clipped Gaussian over the lowest `ground_layers` cells for ~90 % of draws."""
    rng = _rng(seed)
    X, Y, Z = grid

    def draw_z(m):
        if Z == 1:
            return np.zeros(m, dtype=np.int64)
        zg = np.clip(np.rint(rng.normal(5.0, 3.0, m)), 0, min(ground_layers, Z) - 1).astype(np.int64)
        zu = rng.integers(0, Z, m)
        return np.where(rng.random(m) < 0.9, zg, zu)

    def draw(m):
        xr, yr = _radial_xy(rng, m, X, Y)
        xu, yu = rng.integers(0, X, m), rng.integers(0, Y, m)
        pick = rng.random(m) < clutter
        return np.stack([np.where(pick, xu, xr), np.where(pick, yu, yr), draw_z(m)], 1)

    return _unique_cells(draw, n, grid, rng)


def frame_skewed(seed, grid, n, win, hot_frac=0.05, hot_share=0.7, cold_frac=0.02):
    """hot_share of the voxels packed into hot_frac of the (unshifted) windows, cold_frac of the
    windows left with exactly one voxel, the rest uniform elsewhere, so that per-window counts
    span 1 ... >1,500."""
    rng = _rng(seed)
    X, Y, Z = grid
    L, W, H = win
    nwx, nwy, nwz = -(-X // L), -(-Y // W), -(-Z // H)
    nw = nwx * nwy * nwz
    perm = rng.permutation(nw)
    n_hot, n_cold = max(1, int(round(hot_frac * nw))), max(1, int(round(cold_frac * nw)))
    hot, cold = perm[:n_hot], perm[n_hot:n_hot + n_cold]
    is_cold = np.zeros(nw, dtype=bool)
    is_cold[cold] = True

    def cell_in(w, m):
        wz, wy, wx = w % nwz, (w // nwz) % nwy, w // (nwz * nwy)
        return np.stack([wx * L + rng.integers(0, L, m), wy * W + rng.integers(0, W, m),
                         wz * H + rng.integers(0, H, m)], 1)

    lone = cell_in(cold, n_cold)
    lone = lone[(lone[:, 0] < X) & (lone[:, 1] < Y) & (lone[:, 2] < Z)]

    def draw(m):
        u = np.stack([rng.integers(0, X, m), rng.integers(0, Y, m), rng.integers(0, Z, m)], 1)
        c = np.where((rng.random(m) < hot_share)[:, None], cell_in(hot[rng.integers(0, n_hot, m)], m), u)
        w = ((c[:, 0] // L) * nwy + c[:, 1] // W) * nwz + c[:, 2] // H
        return c[~is_cold[w]]

    body = _unique_cells(draw, n - len(lone), grid, rng)
    return np.concatenate([body, lone], 0)[rng.permutation(n)]


def make_frame(cfg_id, n=None, seed=None):
    """coords int32 [N,4] = (b, x, y, z) for workload `cfg_id`; `n` overrides voxels per frame."""
    cfg = CONFIGS[cfg_id]
    n = cfg["n"] if n is None else int(n)
    seed = 1000 + cfg_id if seed is None else seed
    frames = []
    for b in range(cfg["batch"]):
        s = seed * 16 + b
        if cfg["kind"] == "uniform":
            c = frame_uniform(s, cfg["grid"], n)
        elif cfg["kind"] in ("radial", "radial3d"):
            c = frame_radial(s, cfg["grid"], n)
        else:
            c = frame_skewed(s, cfg["grid"], n, cfg["win"])
        frames.append(np.concatenate([np.full((len(c), 1), b, np.int64), c], 1))
    return np.ascontiguousarray(np.concatenate(frames, 0), dtype=np.int32)


def make_features(seed, n, C, dtype):
    """N(0,1) features, fp32; rounded to bf16-representable values when dtype == 'bf16'."""
    x = _rng(seed).standard_normal((n, C)).astype(np.float32)
    return round_bf16(x) if dtype == "bf16" else x


def make_points(seed, n_points, range_min, range_max, f_in=5, batch=1, clusters=600, share=0.95, sigma=0.45):
    """LiDAR-shaped point rows [n_points, f_in] float32 (x, y, z in metres, then f_in - 3 attributes in
    [0, 1)) and a frame index per point.  A share of the points falls into Gaussian blobs (objects and
    ground patches, centres at uniform range from the sensor, so dense near it), the rest is spread with
    an area density ~ 1/r out to 7 % beyond the range, so that some points lie outside on purpose: at
    180,000 points over 150 m x 150 m and 0.32 m pillars about 30,000 pillars are hit, from single points
    to several dozen per pillar.  The first 64 rows are put exactly on the range's x edges.  sigma scales
    with the x extent (0.45 at 150 m)."""
    rng = _rng(seed)
    lo, hi = np.asarray(range_min, dtype=np.float64), np.asarray(range_max, dtype=np.float64)
    centre, half = (lo + hi) / 2.0, (hi - lo) / 2.0
    R = min(half[0], half[1])
    sig = sigma * (hi[0] - lo[0]) / 149.76
    cr, cth = rng.uniform(0.0, R, clusters), rng.uniform(0.0, 2.0 * np.pi, clusters)
    cx, cy = centre[0] + cr * np.cos(cth), centre[1] + cr * np.sin(cth)
    pick = rng.integers(0, clusters, n_points)
    blob = rng.random(n_points) < share
    r, th = rng.uniform(0.0, 1.07 * R, n_points), rng.uniform(0.0, 2.0 * np.pi, n_points)
    pts = np.empty((n_points, f_in), dtype=np.float64)
    pts[:, 0] = np.where(blob, cx[pick] + rng.normal(0.0, sig, n_points), centre[0] + r * np.cos(th))
    pts[:, 1] = np.where(blob, cy[pick] + rng.normal(0.0, sig, n_points), centre[1] + r * np.sin(th))
    pts[:, 2] = lo[2] + np.abs(rng.normal(0.25, 0.2, n_points)) * (hi[2] - lo[2])
    pts[:, 3:] = rng.random((n_points, f_in - 3))
    m = min(n_points, 64)
    pts[:m, 0] = np.where(rng.random(m) < 0.5, lo[0], hi[0])
    pb = rng.integers(0, batch, n_points).astype(np.int32)
    return pts.astype(np.float32), pb
