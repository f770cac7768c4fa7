"""CPU oracle for DSVT's Dynamic Sparse Window Attention (arXiv 2301.06051).

TEST INFRASTRUCTURE ONLY.  A plain, slow, float64 numpy statement of what the
paper defines, written to be checked against the paper by eye.  It shares no
code with the HIP path and must never be imported by it: only the tests, the
smoke check and the benchmark's CPU-baseline leg call into this file.

What each function follows:
  partition      Sec. 3.2 "Dynamic set partition": window split, Eq. (2) set
                 count, Eq. (3) slot index, Eq. (4) INDEX; "Rotated set
                 attention": X-/Y-axis main order; "Hybrid window partition":
                 window shift.  axis 2-5: the Random and Sparse baselines of
                 the set-partition ablation (Sec. 4.4), each of them another
                 numbering of the voxels inside a window, which is how the paper
                 says it built them; the Regional baseline is axis 0 in both
                 layers of a block.
  set_attention  Eq. (5): MHSA over every set in one batch, PE added to the
                 logits, duplicated slots masked as keys (sentence after Eq. 3).
  layer / block  Appendix "Network Architecture", DSVT-P paragraph: MHSA,
                 residual, LN, 2-layer MLP with GELU, residual, LN; a block is
                 an X-axis layer followed by a Y-axis layer (Eq. 5, Fig. 3).
  attn_pool      Sec. 3.3, Eq. (6) max-pool query and Eq. (7) attention over
                 the densified pooling region.
  bev_scatter    Sec. 3.1 overview: the voxel features projected to a dense
                 bird's-eye-view map (a definition: out[cell of voxel i] = x[i]).
  voxel_max_vfe  Sec. 3.1 overview: points become sparse voxels through a voxel
                 feature encoding module.  The paper names the step and cites
                 earlier pillar encoders for it; the reading taken is the
                 simplest member of that family: an optional per-point linear
                 map, then the channel-wise maximum over a voxel's points.

Readings taken where the paper is silent (each listed in the design notes):
0-based ranks; Eq. (3) evaluated as an exact integer floor; x (resp. y) most
significant in the inner-window order, z least; windows shifted without wrap,
windows and sets numbered in ascending window key; PE = a learned relative
position bias table per head indexed by the coordinate difference query-key;
LN eps 1e-5, exact (erf) GELU, logit scale 1/sqrt(d); pooling output =
LN(P + Attn(P, region)); voxel feature encoding = max over the voxel's points
of (W f + b), voxels in ascending cell key, the cell of a point decided in
float32 (subtract, divide, compare) so that both sides take the same decision.
Parity unpinned by the paper itself: the PE form, the pooling wrapper
(residual + LN), LN eps / GELU form, the voxel feature encoder's form and the
Random / Sparse partition baselines (one sentence each in the paper) -- they
are pinned only to the stated reading (library LN / GELU / MHSA routines,
numpy's segmented maximum, brute force).
"""
import numpy as np
from scipy.special import erf

F64 = np.float64


# ----------------------------------------------------------------------------
# Partition (Sec. 3.2, Eq. 2-4)
# ----------------------------------------------------------------------------
def windows_per_axis(grid, win, shift):
    """Windows needed to cover cells 0..grid-1 once they are moved by +shift."""
    return tuple((g + s + w - 1) // w for g, s, w in zip(grid, shift, win))


def window_and_inner_keys(coords, grid, win, shift, axis):
    """Step 1-2: window key (batch most significant) and inner-window sort key."""
    c = np.asarray(coords, dtype=np.int64)
    b, x, y, z = c[:, 0], c[:, 1] + shift[0], c[:, 2] + shift[1], c[:, 3] + shift[2]
    L, W, H = win
    nwx, nwy, nwz = windows_per_axis(grid, win, shift)
    win_key = ((b * nwx + x // L) * nwy + y // W) * nwz + z // H
    xi, yi, zi = x % L, y % W, z % H
    if axis % 2 == 0:                   # X-axis main order: x, then y, then z
        inner = (xi * W + yi) * H + zi
    else:                               # Y-axis main order: y, then x, then z
        inner = (yi * L + xi) * H + zi
    if axis in (2, 3):                  # "Random" baseline of the set-partition ablation: a fixed shuffle of the cells
        mul, add = shuffle_constants(L * W * H, axis)
        inner = (inner * mul + add) % (L * W * H)
    return win_key, inner


def shuffle_constants(volume, axis):
    """The inner-window voxel ID of the 'Random' partition baseline is taken as a fixed shuffle of the window's
    V cells, key -> (key * mul + add) mod V: mul = the smallest integer >= floor(0.618 V) + (axis odd) that has
    no common factor with V (so the map is one-to-one), add = floor(V / 3) + (axis odd)."""
    odd = axis % 2
    mul = max(int(0.618 * volume), 1) + odd
    while np.gcd(mul, volume) != 1:
        mul += 1
    return mul, volume // 3 + odd


def partition(coords, grid, win, shift, tau, axis):
    """Rotated dynamic set partition of sparse voxels.

    coords int [N,4] rows (b,x,y,z).  Returns a dict with
      set_inds   int32 [S,tau]  voxel index held by every slot (Eq. 3-4)
      voxel_slot int32 [N]      first flat slot s*tau+k holding each voxel
      set_win    int32 [S]      window key of every set
      n_sets     S = sum over non-empty windows of Eq. (2)
      win_keys / win_counts     the non-empty windows and their N
    """
    n = len(coords)
    win_key, inner = window_and_inner_keys(coords, grid, win, shift, axis)
    order = np.lexsort((inner, win_key))            # sort voxel ids by (window, inner key)
    keys, starts, counts = np.unique(win_key[order], return_index=True, return_counts=True)
    rows, set_win = [], []
    for wk, base, N in zip(keys, starts, counts):
        N = int(N)
        S = N // tau + (1 if N % tau > 0 else 0)                    # Eq. (2)
        t = np.arange(S * tau, dtype=np.int64)                      # t = j*tau + k
        q = (t * N) // (S * tau)                                    # Eq. (3), exact floor
        members = order[base:base + N]
        if axis in (4, 5):              # "Sparse" baseline: every subset spread over the whole window -- the voxel
            d = np.arange(N)            # of rank d goes behind all voxels of a smaller rank residue d mod S
            members = members[np.lexsort((d // S, d % S))]
        rows.append(members[q].reshape(S, tau))                     # Eq. (4): INDEX by inner-window rank
        set_win += [wk] * S
    set_inds = np.concatenate(rows, 0) if rows else np.zeros((0, tau), np.int64)
    flat = set_inds.reshape(-1)
    voxel_slot = np.full(n, -1, dtype=np.int64)
    u, first = np.unique(flat, return_index=True)
    voxel_slot[u] = first
    return dict(set_inds=set_inds.astype(np.int32), voxel_slot=voxel_slot.astype(np.int32),
                set_win=np.asarray(set_win, dtype=np.int32), n_sets=len(set_inds), tau=tau,
                win_keys=keys, win_counts=counts)


# ----------------------------------------------------------------------------
# Layer pieces (appendix "Network Architecture")
# ----------------------------------------------------------------------------
def layer_norm(x, g, b, eps):
    mu = x.mean(-1, keepdims=True)
    var = ((x - mu) ** 2).mean(-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def gelu(x):
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def softmax_rows(logits):
    m = logits.max(-1, keepdims=True)
    e = np.exp(logits - m)
    return e / e.sum(-1, keepdims=True)


def rel_index(o_query, o_key, win):
    """Index into a head's relative-position table for coordinate difference query - key."""
    L, W, H = win
    d = o_query - o_key
    return ((d[..., 0] + L - 1) * (2 * W - 1) + (d[..., 1] + W - 1)) * (2 * H - 1) + (d[..., 2] + H - 1)


def set_attention(w, maps, coords, x, dup_mode=0, chunk=1024):
    """y[N,C] = per-set multi-head self-attention (Eq. 5), out-projected and returned per voxel.

    dup_mode 0: a slot that repeats the previous slot's voxel is masked as a key, so every
    set member counts once.  dup_mode 1: repeats stay as keys.
    """
    x = np.asarray(x, F64)
    C, h = w["C"], w["heads"]
    d = C // h
    set_inds = maps["set_inds"].astype(np.int64)
    S, tau = set_inds.shape
    wqkv, bqkv = np.asarray(w["w_qkv"], F64), np.asarray(w["b_qkv"], F64)
    wo, bo = np.asarray(w["w_o"], F64), np.asarray(w["b_o"], F64)
    table = None if w.get("rel_bias") is None else np.asarray(w["rel_bias"], F64)
    xyz = np.asarray(coords, np.int64)[:, 1:4]
    Y = np.empty((S, tau, C), F64)
    for s0 in range(0, S, chunk):                       # sets are independent: chunks only bound memory
        inds = set_inds[s0:s0 + chunk]
        F = x[inds]                                     # INDEX, Eq. (4): [s,tau,C]
        O = xyz[inds]                                   #                  [s,tau,3]
        qkv = F @ wqkv.T + bqkv
        q, k, v = (qkv[..., i * C:(i + 1) * C].reshape(-1, tau, h, d).transpose(0, 2, 1, 3) for i in range(3))
        logits = q @ k.transpose(0, 1, 3, 2) / np.sqrt(d)          # [s,h,tau(query),tau(key)]
        if table is not None:
            idx = rel_index(O[:, :, None, :], O[:, None, :, :], w["win"])     # [s,query,key]
            logits = logits + table[:, idx].transpose(1, 0, 2, 3)
        if dup_mode == 0:
            dup = np.zeros(inds.shape, bool)
            dup[:, 1:] = inds[:, 1:] == inds[:, :-1]
            logits = np.where(dup[:, None, None, :], -np.inf, logits)
        p = softmax_rows(logits)
        o = (p @ v).transpose(0, 2, 1, 3).reshape(-1, tau, C)
        Y[s0:s0 + chunk] = o @ wo.T + bo
    return Y.reshape(S * tau, C)[maps["voxel_slot"].astype(np.int64)]


def layer(w, maps, coords, x, dup_mode=0):
    """One DSVT layer: x1 = LN(x + MHSA(x)); x2 = LN(x1 + MLP(x1))."""
    x = np.asarray(x, F64)
    x1 = layer_norm(x + set_attention(w, maps, coords, x, dup_mode),
                    np.asarray(w["ln1_g"], F64), np.asarray(w["ln1_b"], F64), w["ln_eps"])
    hid = gelu(x1 @ np.asarray(w["w_1"], F64).T + np.asarray(w["b_1"], F64))
    mlp = hid @ np.asarray(w["w_2"], F64).T + np.asarray(w["b_2"], F64)
    return layer_norm(x1 + mlp, np.asarray(w["ln2_g"], F64), np.asarray(w["ln2_b"], F64), w["ln_eps"])


def block(w_pair, maps_pair, coords, x, dup_mode=0):
    """One DSVT block: X-axis layer then Y-axis layer (Eq. 5)."""
    x = layer(w_pair[0], maps_pair[0], coords, x, dup_mode)
    return layer(w_pair[1], maps_pair[1], coords, x, dup_mode)


def stack(weights, coords, x, grid, win, shifts, tau, dup_mode=0):
    """Backbone of len(weights) blocks; block b uses window shift shifts[b % len(shifts)]."""
    maps = {}
    for b, w_pair in enumerate(weights):
        sh = tuple(shifts[b % len(shifts)])
        if sh not in maps:
            maps[sh] = [partition(coords, grid, win, sh, tau, axis) for axis in (0, 1)]
        x = block(w_pair, maps[sh], coords, x, dup_mode)
    return x


# ----------------------------------------------------------------------------
# Attention-style 3D pooling (Sec. 3.3, Eq. 6-7)
# ----------------------------------------------------------------------------
def attn_pool(w, coords, x, grid, pool, mask_empty=1):
    """Pool every non-empty l x w x h region to one voxel.

    Returns (out_coords int32 [M,4] in ascending region key, out float64 [M,C]).
    Query = channel-wise max over the region's occupied voxels (Eq. 6); keys/values = the
    densified region (Eq. 7): occupied slots only when mask_empty == 1, all l*w*h slots with
    zero features in the holes when mask_empty == 0.
    """
    x = np.asarray(x, F64)
    c = np.asarray(coords, np.int64)
    C, h = w["C"], w["heads"]
    d = C // h
    pl, pw, ph = pool
    Xp, Yp, Zp = (grid[0] + pl - 1) // pl, (grid[1] + pw - 1) // pw, (grid[2] + ph - 1) // ph
    rx, ry, rz = c[:, 1] // pl, c[:, 2] // pw, c[:, 3] // ph
    key = ((c[:, 0] * Xp + rx) * Yp + ry) * Zp + rz
    slot = ((c[:, 1] % pl) * pw + (c[:, 2] % pw)) * ph + (c[:, 3] % ph)
    ukeys, region = np.unique(key, return_inverse=True)
    M, P = len(ukeys), pl * pw * ph
    dense = np.zeros((M, P, C), F64)                    # region padded to dense
    occ = np.zeros((M, P), bool)
    dense[region, slot] = x
    occ[region, slot] = True
    pooled = np.where(occ[:, :, None], dense, -np.inf).max(1)          # Eq. (6)
    g = lambda name: np.asarray(w[name], F64)
    q = (pooled @ g("w_q").T + g("b_q")).reshape(M, h, 1, d)
    k = (dense @ g("w_k").T + g("b_k")).reshape(M, P, h, d).transpose(0, 2, 1, 3)
    v = (dense @ g("w_v").T + g("b_v")).reshape(M, P, h, d).transpose(0, 2, 1, 3)
    logits = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(d)                # [M,h,1,P]
    if mask_empty:
        logits = np.where(occ[:, None, None, :], logits, -np.inf)
    o = (softmax_rows(logits) @ v).reshape(M, C)                       # Eq. (7)
    out = layer_norm(pooled + o @ g("w_o").T + g("b_o"), g("ln_g"), g("ln_b"), w["ln_eps"])
    out_coords = np.stack([ukeys // (Xp * Yp * Zp), (ukeys // (Yp * Zp)) % Xp, (ukeys // Zp) % Yp, ukeys % Zp], 1)
    return out_coords.astype(np.int32), out


# ----------------------------------------------------------------------------
# Bird's-eye-view map (Sec. 3.1, overview)
# ----------------------------------------------------------------------------
def bev_scatter(coords, x, batch, grid):
    """Dense [batch, X, Y, Z, C] map: voxel i's feature row at cell coords[i] = (b, x, y, z), zeros at
    every empty cell.  One voxel at a time, as the definition reads."""
    coords = np.asarray(coords)
    x = np.asarray(x)
    out = np.zeros((batch, grid[0], grid[1], grid[2], x.shape[1]), dtype=x.dtype)
    for i in range(len(coords)):
        b, cx, cy, cz = (int(v) for v in coords[i])
        out[b, cx, cy, cz, :] = x[i]
    return out


# ----------------------------------------------------------------------------
# Voxel feature encoding (Sec. 3.1, overview: point cloud -> sparse voxels)
# ----------------------------------------------------------------------------
def point_cells(points, point_batch, range_min, voxel_size, grid, batch):
    """Cell (b, x, y, z) of every point and whether it lies inside the grid.  The decision is taken in
    float32, one operation at a time: t = (p - range_min) / voxel_size, inside iff 0 <= t < cells,
    cell = t truncated.  Points with a NaN coordinate or a batch index outside [0, batch) are outside."""
    p = np.asarray(points, dtype=np.float32)
    lo = np.asarray(range_min, dtype=np.float32)
    sz = np.asarray(voxel_size, dtype=np.float32)
    n = len(p)
    b = np.zeros(n, dtype=np.int64) if point_batch is None else np.asarray(point_batch, dtype=np.int64)
    inside = (b >= 0) & (b < batch)
    cell = np.zeros((n, 4), dtype=np.int64)
    cell[:, 0] = b
    for a in range(3):
        with np.errstate(invalid="ignore"):
            t = ((p[:, a] - lo[a]).astype(np.float32) / sz[a]).astype(np.float32)
            ok = (t >= np.float32(0)) & (t < np.float32(grid[a]))      # False for NaN
        inside &= ok
        cell[:, 1 + a] = np.where(ok, t, 0).astype(np.int64)            # truncation = floor for t >= 0
    return cell, inside


def voxel_max_vfe(points, point_batch, range_min, voxel_size, grid, batch, w=None, b=None, relu=False):
    """Non-empty voxels in ascending key ((b*X + x)*Y + y)*Z + z and, for each, the channel-wise maximum
    over its points of h = W f + b (f = the point's feature row, its first three entries the position;
    w None: h = f), followed by max(., 0) if relu.  One voxel at a time, one point at a time."""
    pts = np.asarray(points, dtype=np.float32)
    cell, inside = point_cells(pts, point_batch, range_min, voxel_size, grid, batch)
    X, Y, Z = (int(g) for g in grid)
    members = {}
    for i in range(len(pts)):
        if inside[i]:
            bb, cx, cy, cz = (int(v) for v in cell[i])
            members.setdefault(((bb * X + cx) * Y + cy) * Z + cz, []).append(i)
    keys = sorted(members)
    C = pts.shape[1] if w is None else np.shape(w)[0]
    coords = np.zeros((len(keys), 4), dtype=np.int32)
    out = np.zeros((len(keys), C), dtype=F64)
    W = None if w is None else np.asarray(w, dtype=F64)
    B = np.zeros(C, dtype=F64) if b is None else np.asarray(b, dtype=F64)
    for v, key in enumerate(keys):
        coords[v] = (key // (X * Y * Z), (key // (Y * Z)) % X, (key // Z) % Y, key % Z)
        best = np.full(C, -np.inf, dtype=F64)
        for i in members[key]:
            f = pts[i].astype(F64)
            h = f + B if W is None else W @ f + B
            best = np.maximum(best, h)
        out[v] = np.maximum(best, 0.0) if relu else best
    return coords, out
