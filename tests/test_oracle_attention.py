"""Pins for the oracle's set attention, layer, block and pooling.

Expectations come from: brute-force Python loops restricted to each voxel's set-mates,
torch's library MHSA / LayerNorm / GELU in float64 on special cases, closed forms and
invariants (permutation of the voxel order, translation by whole windows).
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import synth
from oracle import dsvt_oracle as orc

GRID, WIN, TAU = (12, 10, 4), (6, 5, 2), 7
C, HEADS, HIDDEN = 8, 2, 16


def _tiny(seed=3, n=64, rel_bias=True, batch=1):
    coords = np.concatenate([np.concatenate([np.full((n, 1), b), synth.frame_uniform(seed + b, GRID, n)], 1)
                             for b in range(batch)]).astype(np.int32)
    x = synth.make_features(seed + 10, len(coords), C, "f32")
    w = synth.make_layer_weights(seed + 20, C, HEADS, HIDDEN, WIN, "f32", rel_bias=rel_bias)
    return coords, x, w


def _brute_set_attention(w, maps, coords, x, dup_mode):
    """For every voxel: dense softmax attention over the member list of the set that holds it."""
    n = len(coords)
    d = C // HEADS
    wq, wk, wv = (np.asarray(w["w_qkv"], np.float64)[i * C:(i + 1) * C] for i in range(3))
    bq, bk, bv = (np.asarray(w["b_qkv"], np.float64)[i * C:(i + 1) * C] for i in range(3))
    L, W, H = w["win"]
    out = np.zeros((n, C))
    for i in range(n):
        rows = [r for r in maps["set_inds"].tolist() if i in r]
        assert len(rows) == 1                        # sets are disjoint and complete
        members = rows[0] if dup_mode == 1 else sorted(set(rows[0]), key=rows[0].index)
        qi = wq @ x[i] + bq
        o = np.zeros(C)
        for hd in range(HEADS):
            sl = slice(hd * d, (hd + 1) * d)
            logit = []
            for m in members:
                km = wk @ x[m] + bk
                s = float(qi[sl] @ km[sl]) / math.sqrt(d)
                if w["rel_bias"] is not None:
                    dx, dy, dz = (int(coords[i][a]) - int(coords[m][a]) for a in (1, 2, 3))
                    s += float(w["rel_bias"][hd][((dx + L - 1) * (2 * W - 1) + dy + W - 1) * (2 * H - 1) + dz + H - 1])
                logit.append(s)
            mx = max(logit)
            e = [math.exp(v - mx) for v in logit]
            z = sum(e)
            for m, em in zip(members, e):
                o[sl] += (em / z) * (wv @ x[m] + bv)[sl]
        out[i] = np.asarray(w["w_o"], np.float64) @ o + np.asarray(w["b_o"], np.float64)
    return out


@pytest.mark.parametrize("dup_mode", [0, 1])
@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("rel_bias", [True, False])
def test_set_attention_matches_brute_force(dup_mode, axis, rel_bias):
    coords, x, w = _tiny(rel_bias=rel_bias, batch=2)
    maps = orc.partition(coords, GRID, WIN, (3, 2, 1), TAU, axis)
    got = orc.set_attention(w, maps, coords, x, dup_mode)
    want = _brute_set_attention(w, maps, coords, x.astype(np.float64), dup_mode)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)
    if dup_mode == 0:                                 # duplicates do change the answer when kept
        other = orc.set_attention(w, maps, coords, x, 1)
        assert np.abs(other - got).max() > 1e-6


def test_set_attention_reduces_to_library_mhsa():
    """Windows holding exactly tau voxels: no duplicates; without PE a set is textbook MHSA."""
    tau, win, grid = 8, (2, 2, 2), (4, 4, 4)
    xs, ys, zs = np.meshgrid(range(4), range(4), range(4), indexing="ij")
    coords = np.stack([np.zeros(64, int), xs.ravel(), ys.ravel(), zs.ravel()], 1).astype(np.int32)
    coords = coords[np.random.Generator(np.random.Philox(1)).permutation(64)]
    x = synth.make_features(2, 64, C, "f32")
    w = synth.make_layer_weights(4, C, HEADS, HIDDEN, win, "f32", rel_bias=False)
    maps = orc.partition(coords, grid, win, (0, 0, 0), tau, 0)
    assert maps["n_sets"] == 8 and sorted(maps["set_inds"].reshape(-1).tolist()) == list(range(64))
    got = orc.set_attention(w, maps, coords, x)
    t = lambda a: torch.tensor(np.asarray(a, np.float64))
    tiles = t(x)[torch.tensor(maps["set_inds"].astype(np.int64))].transpose(0, 1)      # [tau, S, C]
    lib, _ = TF.multi_head_attention_forward(
        tiles, tiles, tiles, C, HEADS, t(w["w_qkv"]), t(w["b_qkv"]), None, None, False, 0.0,
        t(w["w_o"]), t(w["b_o"]), training=False, need_weights=False)
    lib = lib.transpose(0, 1).reshape(-1, C).numpy()
    np.testing.assert_allclose(got, lib[maps["voxel_slot"]], rtol=1e-11, atol=1e-12)


def test_equal_features_give_value_row():
    """All voxels identical and no PE: every softmax is uniform over copies of one V row."""
    coords, x, w = _tiny(rel_bias=False)
    x[:] = x[0]
    maps = orc.partition(coords, GRID, WIN, (0, 0, 0), TAU, 0)
    v = np.asarray(w["w_qkv"], np.float64)[2 * C:] @ x[0] + np.asarray(w["b_qkv"], np.float64)[2 * C:]
    want = np.asarray(w["w_o"], np.float64) @ v + np.asarray(w["b_o"], np.float64)
    for mode in (0, 1):
        np.testing.assert_allclose(orc.set_attention(w, maps, coords, x, mode), np.tile(want, (len(x), 1)),
                                   rtol=1e-11, atol=1e-12)


def test_layer_matches_library_ln_gelu_mlp():
    coords, x, w = _tiny()
    maps = orc.partition(coords, GRID, WIN, (0, 0, 0), TAU, 1)
    got = orc.layer(w, maps, coords, x)
    t = lambda a: torch.tensor(np.asarray(a, np.float64))
    y = t(_brute_set_attention(w, maps, coords, x.astype(np.float64), 0))
    x1 = TF.layer_norm(t(x) + y, (C,), t(w["ln1_g"]), t(w["ln1_b"]), w["ln_eps"])
    mlp = TF.linear(TF.gelu(TF.linear(x1, t(w["w_1"]), t(w["b_1"]))), t(w["w_2"]), t(w["b_2"]))
    want = TF.layer_norm(x1 + mlp, (C,), t(w["ln2_g"]), t(w["ln2_b"]), w["ln_eps"]).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-11)


def test_ln_gelu_softmax_closed_forms():
    r = np.random.Generator(np.random.Philox(9))
    a = r.standard_normal((5, 32)) * 3 + 1
    out = orc.layer_norm(a, np.ones(32), np.zeros(32), 1e-5)
    np.testing.assert_allclose(out.mean(-1), 0, atol=1e-13)
    np.testing.assert_allclose(out.var(-1), a.var(-1) / (a.var(-1) + 1e-5), rtol=1e-12)
    assert orc.gelu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(orc.gelu(np.array([30.0, -30.0])), [30.0, 0.0], atol=1e-12)
    for v in (-2.5, -0.3, 0.7, 1.9):                  # x * Phi(x) against math.erf
        assert abs(orc.gelu(np.array([v]))[0] - v * 0.5 * (1 + math.erf(v / math.sqrt(2)))) < 1e-15
    p = orc.softmax_rows(np.array([[1.0, 2.0, -np.inf, 3.0]]))
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-15)
    assert p[0, 2] == 0.0
    np.testing.assert_allclose(p[0, 3] / p[0, 0], math.exp(2.0), rtol=1e-14)


def test_block_and_stack_invariances():
    """Outputs follow a permutation of the input voxels, and do not move when every
    coordinate is translated by a whole number of windows."""
    coords, x, _ = _tiny(n=96)
    grid = (GRID[0] + 2 * WIN[0], GRID[1] + WIN[1], GRID[2])
    ws = [[synth.make_layer_weights(40 + 2 * b + a, C, HEADS, HIDDEN, WIN, "f32") for a in (0, 1)] for b in range(2)]
    shifts = ((0, 0, 0), (3, 2, 1))
    base = orc.stack(ws, coords, x, grid, WIN, shifts, TAU)
    perm = np.random.Generator(np.random.Philox(11)).permutation(len(coords))
    permuted = orc.stack(ws, coords[perm], x[perm], grid, WIN, shifts, TAU)
    np.testing.assert_allclose(permuted, base[perm], rtol=1e-11, atol=1e-12)
    moved = coords + np.array([0, 2 * WIN[0], WIN[1], 0], np.int32)
    np.testing.assert_allclose(orc.stack(ws, moved, x, grid, WIN, shifts, TAU), base, rtol=1e-11, atol=1e-12)
    # a block is its two layers in X-then-Y order, and the order matters
    mx, my = (orc.partition(coords, grid, WIN, (0, 0, 0), TAU, a) for a in (0, 1))
    one = orc.block(ws[0], [mx, my], coords, x)
    np.testing.assert_allclose(one, orc.layer(ws[0][1], my, coords, orc.layer(ws[0][0], mx, coords, x)), rtol=1e-12)
    assert np.abs(one - orc.block(ws[0], [my, mx], coords, x)).max() > 1e-6


def test_stack_alternates_the_window_shifts():
    """A backbone's blocks take the window shifts in turn ("Hybrid window partition": the shift changes between
    consecutive blocks): stack() must equal the composition written out block by block with shifts 0, 1, 0, and
    must not equal the composition that keeps the first shift throughout, nor the one that starts with the second."""
    coords, x, _ = _tiny(n=96)
    ws = [[synth.make_layer_weights(60 + 2 * b + a, C, HEADS, HIDDEN, WIN, "f32") for a in (0, 1)] for b in range(3)]
    shifts = ((0, 0, 0), (3, 2, 1))
    got = orc.stack(ws, coords, x, GRID, WIN, shifts, TAU)

    def compose(order):
        y = x
        for w_pair, k in zip(ws, order):
            maps = [orc.partition(coords, GRID, WIN, shifts[k], TAU, axis) for axis in (0, 1)]
            y = orc.layer(w_pair[1], maps[1], coords, orc.layer(w_pair[0], maps[0], coords, y))
        return y

    np.testing.assert_allclose(got, compose((0, 1, 0)), rtol=1e-12, atol=1e-13)
    for wrong in ((0, 0, 0), (1, 0, 1), (0, 1, 1)):
        assert np.abs(got - compose(wrong)).max() > 1e-6, wrong
    # a single shift in the list: every block uses it
    one = orc.stack(ws, coords, x, GRID, WIN, (shifts[1],), TAU)
    np.testing.assert_allclose(one, compose((1, 1, 1)), rtol=1e-12, atol=1e-13)


# ------------------------------ pooling (Sec. 3.3) ------------------------------
def _brute_pool(w, coords, x, grid, pool, mask_empty):
    d = C // HEADS
    g = lambda k: np.asarray(w[k], np.float64)
    pl, pw, ph = pool
    regions = {}
    for i, (b, cx, cy, cz) in enumerate(coords.tolist()):
        regions.setdefault((b, cx // pl, cy // pw, cz // ph), {})[((cx % pl) * pw + cy % pw) * ph + cz % ph] = i
    out_c, out = [], []
    for key in sorted(regions):
        mem = regions[key]
        pooled = np.max(np.stack([x[i] for i in mem.values()]), 0)
        q = g("w_q") @ pooled + g("b_q")
        slots = sorted(mem) if mask_empty else range(pl * pw * ph)
        feats = [x[mem[s]] if s in mem else np.zeros(C) for s in slots]
        o = np.zeros(C)
        for hd in range(HEADS):
            sl = slice(hd * d, (hd + 1) * d)
            logit = [float(q[sl] @ (g("w_k") @ f + g("b_k"))[sl]) / math.sqrt(d) for f in feats]
            e = [math.exp(v - max(logit)) for v in logit]
            for f, ev in zip(feats, e):
                o[sl] += ev / sum(e) * (g("w_v") @ f + g("b_v"))[sl]
        r = pooled + g("w_o") @ o + g("b_o")
        r = (r - r.mean()) / math.sqrt(r.var() + w["ln_eps"]) * g("ln_g") + g("ln_b")
        out_c.append(list(key))
        out.append(r)
    return np.array(out_c), np.array(out)


@pytest.mark.parametrize("mask_empty", [0, 1])
@pytest.mark.parametrize("pool", [(1, 1, 4), (2, 2, 2)])
def test_pool_matches_brute_force(mask_empty, pool):
    coords, x, _ = _tiny(n=90, batch=2)
    w = synth.make_pool_weights(77, C, HEADS, "f32")
    oc, out = orc.attn_pool(w, coords, x, GRID, pool, mask_empty)
    bc, bout = _brute_pool(w, coords, x.astype(np.float64), GRID, pool, mask_empty)
    assert np.array_equal(oc, bc)
    np.testing.assert_allclose(out, bout, rtol=1e-11, atol=1e-12)
    assert len(oc) < len(coords)                       # it does pool something


def test_pool_single_voxel_region_is_value_path():
    """One occupied voxel and masked holes: softmax over one key is 1."""
    w = synth.make_pool_weights(78, C, HEADS, "f32")
    coords = np.array([[0, 1, 2, 3], [0, 5, 5, 0]], np.int32)
    x = synth.make_features(79, 2, C, "f32")
    oc, out = orc.attn_pool(w, coords, x, GRID, (1, 1, 4), 1)
    g = lambda k: np.asarray(w[k], np.float64)
    assert oc.tolist() == [[0, 1, 2, 0], [0, 5, 5, 0]]
    for i in range(2):
        p = x[i].astype(np.float64)
        r = p + g("w_o") @ (g("w_v") @ p + g("b_v")) + g("b_o")
        want = TF.layer_norm(torch.tensor(r), (C,), torch.tensor(g("ln_g")), torch.tensor(g("ln_b")), w["ln_eps"])
        np.testing.assert_allclose(out[i], want.numpy(), rtol=1e-11, atol=1e-12)


def test_bev_scatter_definition():
    """Sec. 3.1 overview (BEV projection): the dense map holds every voxel's row at its cell and zeros
    elsewhere -- checked against an independent gather: reading the map back at the voxels' cells returns
    the rows, the number of non-zero cells equals the number of voxels, and the map's sum is the rows' sum."""
    import synth
    from oracle import dsvt_oracle as orc
    grid = (9, 7, 2)
    coords = np.concatenate([np.repeat(np.arange(2), 20)[:, None], np.concatenate([synth.frame_uniform(5 + b, grid, 20) for b in range(2)])], 1)
    x = synth.make_features(6, len(coords), 8, "f32") + 3.0      # no zero rows
    m = orc.bev_scatter(coords, x, 2, grid)
    assert m.shape == (2, 9, 7, 2, 8)
    assert np.array_equal(m[coords[:, 0], coords[:, 1], coords[:, 2], coords[:, 3]], x)
    assert int((np.abs(m).sum(-1) > 0).sum()) == len(coords)
    assert np.isclose(m.sum(dtype=np.float64), x.sum(dtype=np.float64))
