"""Pins for the oracle's set partition (Sec. 3.2, Eq. 2-4; appendix Thm A.2-A.4).

Nothing here calls the oracle to produce its own expectation: expectations come from
hand-worked fixtures, exact rational arithmetic, the theorems' statements and
brute-force loops over tiny inputs.
"""
from fractions import Fraction
from math import floor
import math
import os

import numpy as np
import pytest

import synth
from oracle import dsvt_oracle as orc


def _one_window(N, tau, axis=0):
    """N voxels laid along x inside one large window so that inner rank == voxel index."""
    coords = np.array([[0, i, 0, 0] for i in range(N)], dtype=np.int32)
    return orc.partition(coords, grid=(max(N, 1), 1, 1), win=(max(N, 1), 1, 1), shift=(0, 0, 0), tau=tau, axis=axis)


def test_eq3_hand_worked_fixtures(golden_dir):
    n_cases = 0
    for line in open(os.path.join(golden_dir, "eq3_slots.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, body = line.split("|")
        N, tau = map(int, head.split())
        want = [list(map(int, s.split())) for s in body.split(";")]
        got = _one_window(N, tau)["set_inds"].tolist()
        assert got == want, (N, tau)
        n_cases += 1
    assert n_cases >= 8


@pytest.mark.parametrize("tau", [4, 36, 48])
def test_eq2_eq3_exact_rational_and_theorems(tau):
    """Eq. (2) closed form, Eq. (3) as an exact rational floor, Thm A.2 (disjoint),
    A.3 (complete) and A.4 (balanced) for every N in a range spanning many multiples of tau."""
    for N in list(range(1, 200)) + [tau * 7, tau * 7 + 1, 699, 1536, 1849]:
        m = _one_window(N, tau)
        S = -(-N // tau)
        assert m["n_sets"] == S == N // tau + (1 if N % tau else 0)
        si = m["set_inds"]
        assert si.shape == (S, tau)                      # every set has exactly tau slots
        want = [[floor(Fraction(j * tau + k, S * tau) * N) for k in range(tau)] for j in range(S)]
        assert si.tolist() == want
        members = [set(r.tolist()) for r in si]
        union = set()
        for a in members:
            assert not (union & a)                       # Thm A.2
            union |= a
            assert N // S <= len(a) <= N // S + 1        # Thm A.4
        assert union == set(range(N))                    # Thm A.3
        flat = si.reshape(-1)
        assert np.all(np.diff(flat) >= 0) and np.all(np.diff(flat) <= 1)   # duplicates are adjacent
        if N == S * tau:                                 # "the case N = S x tau is trivial"
            assert flat.tolist() == list(range(N))
        # first flat slot of every voxel
        for i in (0, N // 2, N - 1):
            assert m["voxel_slot"][i] == flat.tolist().index(i)


def _brute_partition(coords, grid, win, shift, tau, axis):
    """Pure-Python statement of the partition: tuples, sorted(), Fractions."""
    L, W, H = win
    per_window = {}
    for i, (b, x, y, z) in enumerate(coords.tolist()):
        x, y, z = x + shift[0], y + shift[1], z + shift[2]
        wkey = (b, x // L, y // W, z // H)
        xi, yi, zi = x % L, y % W, z % H
        inner = (xi, yi, zi) if axis == 0 else (yi, xi, zi)
        per_window.setdefault(wkey, []).append((inner, i))
    set_inds = []
    for wkey in sorted(per_window):
        ranked = [i for _, i in sorted(per_window[wkey])]
        N = len(ranked)
        S = N // tau + (1 if N % tau else 0)
        for j in range(S):
            set_inds.append([ranked[floor(Fraction(j * tau + k, S * tau) * N)] for k in range(tau)])
    return set_inds, per_window


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("shift", [(0, 0, 0), (2, 3, 1)])
def test_partition_matches_brute_force(axis, shift):
    grid, win, tau = (13, 11, 5), (4, 6, 2), 5
    coords = np.concatenate([np.concatenate([np.full((150, 1), b), synth.frame_uniform(7 + b, grid, 150)], 1)
                             for b in range(2)]).astype(np.int32)
    m = orc.partition(coords, grid, win, shift, tau, axis)
    want, per_window = _brute_partition(coords, grid, win, shift, tau, axis)
    assert m["set_inds"].tolist() == want
    assert m["n_sets"] == sum(-(-len(v) // tau) for v in per_window.values())
    flat = m["set_inds"].reshape(-1).tolist()
    assert m["voxel_slot"].tolist() == [flat.index(i) for i in range(len(coords))]
    # every set lies inside one window and set_win names it, in ascending order
    nw = orc.windows_per_axis(grid, win, shift)
    for s, row in enumerate(m["set_inds"]):
        keys = set()
        for i in row:
            b, x, y, z = coords[i]
            keys.add(((b * nw[0] + (x + shift[0]) // win[0]) * nw[1] + (y + shift[1]) // win[1]) * nw[2]
                     + (z + shift[2]) // win[2])
        assert keys == {int(m["set_win"][s])}
    assert np.all(np.diff(m["set_win"]) >= 0)


def test_axes_share_windows_but_not_order():
    """X- and Y-axis layers see the same windows (same N, same S); only the inner order differs."""
    cfg = synth.CONFIGS[1]
    coords = synth.make_frame(1)
    mx = orc.partition(coords, cfg["grid"], cfg["win"], (0, 0, 0), cfg["tau"], 0)
    my = orc.partition(coords, cfg["grid"], cfg["win"], (0, 0, 0), cfg["tau"], 1)
    assert mx["n_sets"] == my["n_sets"]
    assert np.array_equal(mx["win_counts"], my["win_counts"]) and np.array_equal(mx["set_win"], my["set_win"])
    assert not np.array_equal(mx["set_inds"], my["set_inds"])
    # inside a set of the X partition x never decreases along the slots; same for y in the Y partition
    assert np.all(np.diff(coords[mx["set_inds"], 1], axis=1) >= 0)
    assert np.all(np.diff(coords[my["set_inds"], 2], axis=1) >= 0)
    assert not np.all(np.diff(coords[mx["set_inds"], 2], axis=1) >= 0)


def test_partition_permutation_and_completeness_full_frame():
    """Every voxel in at least one set; maps of a permuted input are the permuted maps."""
    cfg = synth.CONFIGS[2]
    coords = synth.make_frame(2, n=6000)
    m = orc.partition(coords, cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], 1)
    assert set(m["set_inds"].reshape(-1).tolist()) == set(range(len(coords)))
    assert np.array_equal(m["set_inds"].reshape(-1)[m["voxel_slot"]], np.arange(len(coords)))
    assert m["n_sets"] == int(np.sum(-(-m["win_counts"] // cfg["tau"])))
    perm = np.random.Generator(np.random.Philox(5)).permutation(len(coords))
    mp = orc.partition(coords[perm], cfg["grid"], cfg["win"], (6, 6, 0), cfg["tau"], 1)
    assert np.array_equal(perm[mp["set_inds"]], m["set_inds"])


def test_float_evaluation_of_eq3_is_not_exact():
    """Why Eq. (3) is taken as an integer floor: the literal float form misplaces slots."""
    tau, bad = 36, 0
    for N in range(1, 1600):
        S = -(-N // tau)
        t = np.arange(S * tau)
        lit = np.floor(t.astype(np.float64) / (S * tau) * N).astype(np.int64)
        bad += int(np.any(lit != (t * N) // (S * tau)))
    assert bad > 0


# ---------------------------------------------------------------- Random / Sparse / Regional baselines (Sec. 4.4)
def _golden_shuffle_constants():
    """{(V, axis): (mul, add)} worked by hand from the stated rule (tests/golden/shuffle_constants.txt)."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "shuffle_constants.txt")
    table = {}
    for line in open(path):
        body = line.split("#")[0].split()
        if body:
            V, axis, mul, add = map(int, body)
            table[(V, axis)] = (mul, add)
    return table


def test_shuffle_constants_match_hand_worked_values():
    """The constants of the Random baseline's cell shuffle against values worked by hand from the rule, for the
    window volumes of the workloads (12x12x1, 12x12x8, 12x12x32, 30x30x1) and of the brute-force case below."""
    golden = _golden_shuffle_constants()
    assert {v for v, _ in golden} >= {48, 144, 900, 1152, 4608}
    for (V, axis), want in golden.items():
        assert orc.shuffle_constants(V, axis) == want, (V, axis)
        mul, add = want                                  # what the rule promises, checked on the literals themselves
        assert math.gcd(mul, V) == 1 and mul >= int(0.618 * V) + axis % 2 and add == V // 3 + axis % 2
        assert all(math.gcd(m, V) != 1 for m in range(int(0.618 * V) + axis % 2, mul))   # no smaller candidate


def _brute_variant(coords, grid, win, shift, tau, axis):
    """The variants written out in plain Python: an explicit shuffle table for axis 2/3 (its constants are the
    hand-worked literals, not the oracle's), an explicit round-robin deal of the ranked voxels for axis 4/5."""
    L, W, H = win
    V = L * W * H
    mul, add = _golden_shuffle_constants()[(V, 2 + axis % 2)]
    table = [(k * mul + add) % V for k in range(V)]
    per_window = {}
    for i, (b, x, y, z) in enumerate(coords.tolist()):
        x, y, z = x + shift[0], y + shift[1], z + shift[2]
        xi, yi, zi = x % L, y % W, z % H
        inner = (xi * W + yi) * H + zi if axis % 2 == 0 else (yi * L + xi) * H + zi
        if axis in (2, 3):
            inner = table[inner]
        per_window.setdefault((b, x // L, y // W, z // H), []).append((inner, i))
    set_inds = []
    for wkey in sorted(per_window):
        ranked = [i for _, i in sorted(per_window[wkey])]
        N = len(ranked)
        S = N // tau + (1 if N % tau else 0)
        if axis in (4, 5):
            piles = [[] for _ in range(S)]
            for d, i in enumerate(ranked):            # deal the ranked voxels round-robin onto S piles ...
                piles[d % S].append(i)
            ranked = [i for pile in piles for i in pile]   # ... and lay the piles end to end
        for j in range(S):
            set_inds.append([ranked[floor(Fraction(j * tau + k, S * tau) * N)] for k in range(tau)])
    return set_inds


@pytest.mark.parametrize("volume", [1, 2, 7, 36, 144, 1152, 4608, 900])
def test_shuffle_is_one_to_one(volume):
    for axis in (2, 3):
        mul, add = orc.shuffle_constants(volume, axis)
        image = sorted((k * mul + add) % volume for k in range(volume))
        assert image == list(range(volume))
    if volume > 7:
        assert orc.shuffle_constants(volume, 2) != orc.shuffle_constants(volume, 3)


@pytest.mark.parametrize("axis", [2, 3, 4, 5])
def test_partition_variants_match_brute_force(axis):
    grid, win, tau, shift = (13, 11, 5), (4, 6, 2), 5, (2, 3, 1)
    coords = np.concatenate([np.concatenate([np.full((150, 1), b), synth.frame_uniform(7 + b, grid, 150)], 1)
                             for b in range(2)]).astype(np.int32)
    m = orc.partition(coords, grid, win, shift, tau, axis)
    assert m["set_inds"].tolist() == _brute_variant(coords, grid, win, shift, tau, axis)
    base = orc.partition(coords, grid, win, shift, tau, axis % 2)
    # the same windows, set counts and voxels per window as the rotated partition; another order inside
    assert m["n_sets"] == base["n_sets"] and np.array_equal(m["set_win"], base["set_win"])
    assert not np.array_equal(m["set_inds"], base["set_inds"])
    assert np.array_equal(m["set_inds"].reshape(-1)[m["voxel_slot"]], np.arange(len(coords)))
    # Thm A.2-A.4 still hold (they only use the ranks): per window every voxel in exactly one set, sizes within 1
    for wk in np.unique(m["set_win"]):
        rows = m["set_inds"][m["set_win"] == wk]
        members = [set(r.tolist()) for r in rows]
        assert sum(len(s) for s in members) == len(set().union(*members))
        assert max(len(s) for s in members) - min(len(s) for s in members) <= 1


def test_sparse_sets_span_the_window_and_regional_sets_do_not():
    """What the names say: along the main axis a Sparse subset reaches across (nearly) the whole window's voxels,
    a Regional one (the rotated partition's X-axis order) covers a slab."""
    cfg = synth.CONFIGS[2]
    coords = synth.make_frame(2, n=20000)
    reg = orc.partition(coords, cfg["grid"], cfg["win"], (0, 0, 0), cfg["tau"], 0)
    spr = orc.partition(coords, cfg["grid"], cfg["win"], (0, 0, 0), cfg["tau"], 4)
    counts = dict(zip(reg["win_keys"].tolist(), reg["win_counts"].tolist()))
    big = np.array([counts[int(w)] >= 2 * cfg["tau"] for w in reg["set_win"]])          # windows of three sets or more
    assert big.sum() > 20
    span = lambda m: np.ptp(coords[m["set_inds"][big], 1], axis=1)          # extent in x of every set
    assert np.median(span(spr)) >= 9 and np.median(span(reg)) <= 5
