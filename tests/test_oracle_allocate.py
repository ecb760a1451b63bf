"""Pins for the oracle's allocation, top-k and compaction steps, CPU only.

Hand-worked hull / greedy case (tests/golden), unit-level PAVA on the marginal
decreases (the paper's own construction of the surrogate, Sec. 4.2), exhaustive
search and dynamic programming over integer budgets, and invariants.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import lukv_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hull_greedy_handworked.txt")


def _golden():
    out = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if line:
            key, val = [t.strip() for t in line.split("=")]
            out[key] = val.split()
    return out


def _curves():
    g = _golden()
    U = np.array([[float(Fraction(t)) for t in g["U0"]], [float(Fraction(t)) for t in g["U1"]]],
                 dtype=np.float32)
    knots = np.tile(np.arange(5, dtype=np.int32), (2, 1))
    return g, U, knots


def test_handworked_hull_and_gains():
    g, U, knots = _curves()
    for h in range(2):
        assert O.concave_hull(knots[h], U[h]) == [int(t) for t in g["hull%d" % h]]
        per_unit = [O._gain_of_unit(O.marginal_gains(knots[h], U[h]), u) for u in range(1, 5)]
        assert per_unit == [float(Fraction(t)) for t in g["gain%d" % h]]


def test_handworked_budgets_all_B():
    g, U, knots = _curves()
    zero, four = np.zeros(2, np.int32), np.full(2, 4, np.int32)
    for B, want in enumerate(g["budgets"]):
        b, st = O.allocate(U, knots, zero, four, B)
        assert st == 0 and b.tolist() == [int(t) for t in want.split(",")]
    b, st = O.allocate(U, knots, np.ones(2, np.int32), four, 3)
    assert st == 0 and b.tolist() == [int(t) for t in g["bmin11_B3"][0].split(",")]
    b, st = O.allocate(U, knots, np.array([0, 3], np.int32), four, 4)
    assert st == 0 and b.tolist() == [int(t) for t in g["bmin03_B4"][0].split(",")]


def test_infeasible_budgets_flagged():
    _, U, knots = _curves()
    zero, four = np.zeros(2, np.int32), np.full(2, 4, np.int32)
    assert O.allocate(U, knots, zero, four, 9)[1] == 1
    b, st = O.allocate(U, knots, np.full(2, 3, np.int32), four, 5)
    assert st == 1 and b.tolist() == [3, 3]
    # a negative minimum retention is no retention count: flagged, handed back unchanged
    b, st = O.allocate(U, knots, np.array([-1, 0], np.int32), four, 3)
    assert st == 1 and b.tolist() == [-1, 0]


# --- the hull by the definition of a strict vertex: a second, order-free construction ---------

def _vertices_by_chords(knots, U):
    """Knot g is a vertex of the upper concave hull iff every chord from an earlier knot to g is
    strictly steeper than every chord from g to a later knot (the end knots always are).  Same
    fp64 chord expression as the oracle's gain (one subtract, one divide), but no scan order."""
    G = len(knots)
    n = np.asarray(knots, dtype=np.int64).astype(np.float64)
    u = np.asarray(U, dtype=np.float32).astype(np.float64)
    out = []
    for g in range(G):
        if g == 0 or g == G - 1:
            out.append(g)
            continue
        steep_in = min((u[g] - u[a]) / (n[g] - n[a]) for a in range(g))
        steep_out = max((u[c] - u[g]) / (n[c] - n[g]) for c in range(g + 1, G))
        if steep_in > steep_out:
            out.append(g)
    return out


@pytest.mark.parametrize("seed", range(10))
def test_scan_equals_vertex_definition(seed):
    rng = np.random.default_rng(700 + seed)
    Gp = int(rng.integers(2, 40))
    L = int(rng.integers(Gp, 4000))
    if seed % 2:
        inc = rng.integers(0, 4, size=Gp).astype(np.float32) / 8     # many collinear runs
    else:
        z = rng.standard_normal(Gp)
        inc = (0.5 * z * z).astype(np.float32)
    inc[0] = 0
    U = np.cumsum(inc).astype(np.float32)
    knots = ((np.arange(Gp) * L) // (Gp - 1)).astype(np.int32) if Gp > 1 else np.zeros(1, np.int32)
    assert O.concave_hull(knots, U) == _vertices_by_chords(knots, U)


def _near_collinear_curve(rng):
    """A curve whose knots lie on (or within a few float32 ulps of) one or two straight lines:
    the case in which rounding of the fp64 chords could make two constructions disagree."""
    Gp = int(rng.integers(3, 24))
    top = int(rng.choice([Gp + 5, 300, 4096, 1 << 17, 1 << 20]))
    knots = np.unique(np.concatenate([[0], rng.integers(1, top, size=Gp - 2), [top]])).astype(np.int64)
    Gp = knots.size
    kind = int(rng.integers(0, 4))
    slope = float(rng.choice([1.0, 1 / 3, 0.1, 7.0, 1e-3])) * float(rng.uniform(0.5, 2.0))
    exact = knots.astype(np.float64) * slope
    if kind == 1:                                   # a second, slightly flatter line after a break
        brk = int(rng.integers(1, Gp - 1))
        exact[brk:] = exact[brk] + (knots[brk:] - knots[brk]) * slope * (1.0 - float(rng.choice([1e-7, 1e-5, 1e-3])))
    U = exact.astype(np.float32)                    # rounded exact line(s)
    if kind >= 2:                                   # plus or minus a few ulps of noise
        bits = U.view(np.int32) + rng.integers(-2, 3, size=Gp).astype(np.int32)
        U = np.maximum(bits, 0).view(np.float32)
    U = np.maximum.accumulate(U)
    U[0] = 0.0
    return knots.astype(np.int32), U.astype(np.float32)


def test_scan_equals_vertex_definition_on_near_collinear_curves():
    """10 000 seeded curves of rounded straight lines with knots up to 2^20: the sequential scan
    and the order-free vertex definition must name the same vertices even where chords differ
    only in their last bits."""
    rng = np.random.default_rng(20260208)
    n_nontrivial = 0
    for _ in range(10000):
        knots, U = _near_collinear_curve(rng)
        a, b = O.concave_hull(knots, U), _vertices_by_chords(knots, U)
        assert a == b, (knots.tolist(), U.tolist())
        n_nontrivial += len(a) > 2
    assert n_nontrivial > 1000          # the family is not all straight lines


def test_collinear_knots_are_not_vertices():
    # slopes 2, 2, 1, 1, 0 by hand: only the knots where the slope drops are vertices
    knots = np.arange(6, dtype=np.int32)
    U = np.array([0, 2, 4, 5, 6, 6], dtype=np.float32)
    assert O.concave_hull(knots, U) == [0, 2, 4, 5]
    assert O.marginal_gains(knots, U) == [(0, 2, 2.0), (2, 4, 1.0), (4, 5, 0.0)]
    assert _vertices_by_chords(knots, U) == [0, 2, 4, 5]
    # a straight line has only its end points
    assert O.concave_hull(knots, np.arange(6, dtype=np.float32)) == [0, 5]


def test_pooling_cascades_and_uses_the_pooled_blocks_own_chord():
    """Hand-worked: unequal knot spacing and a late steep interval that pools three blocks.
    knots 0 1 4 6 7, U 0 3 6 7 12: interval gains 3, 1, 1/2, 5.  The last interval (gain 5) pools
    with (4,6] -> chord over (4,7] = 2 > 1, pools with (1,4] -> chord over (1,7] = 3/2 < 3: stop.
    Vertices 0, 1, 4(end); gains 3 and 3/2.  (An unweighted mean of pooled gains, or a single
    pooling step, gives something else.)"""
    knots = np.array([0, 1, 4, 6, 7], np.int32)
    U = np.array([0, 3, 6, 7, 12], np.float32)
    assert O.concave_hull(knots, U) == [0, 1, 4]
    assert O.marginal_gains(knots, U) == [(0, 1, 3.0), (1, 7, 1.5)]
    assert _vertices_by_chords(knots, U) == [0, 1, 4]


# --- unit-level PAVA (textbook pool-adjacent-violators on the marginal decreases) ----------

def _pava_nonincreasing(d):
    """Isotonic regression of d onto non-increasing sequences, equal weights, exact rationals."""
    blocks = []  # (sum, count)
    for x in d:
        blocks.append((Fraction(x), 1))
        while len(blocks) >= 2 and blocks[-2][0] / blocks[-2][1] < blocks[-1][0] / blocks[-1][1]:
            s2, c2 = blocks.pop()
            s1, c1 = blocks.pop()
            blocks.append((s1 + s2, c1 + c2))
    out = []
    for s, c in blocks:
        out += [s / c] * c
    return out


@pytest.mark.parametrize("seed", range(8))
def test_pava_equals_hull_slopes(seed):
    rng = np.random.default_rng(100 + seed)
    T = int(rng.integers(4, 24))
    dec = rng.integers(0, 9, size=T)                    # per-token importance, integers
    U = np.concatenate([[0], np.cumsum(dec)]).astype(np.float32)
    knots = np.arange(T + 1, dtype=np.int32)
    want = _pava_nonincreasing([int(x) for x in dec])
    segs = O.marginal_gains(knots, U)
    got = [O._gain_of_unit(segs, u) for u in range(1, T + 1)]
    assert all(w >= 0 for w in want)
    assert all(a >= b for a, b in zip(want, want[1:]))
    assert got == pytest.approx([float(w) for w in want], rel=1e-15)


# --- exhaustive search / DP --------------------------------------------------------------

def _interp(knots, U, b):
    return float(np.interp(b, knots.astype(np.float64), U.astype(np.float64)))


def _hull_value(knots, U, b):
    st = O.concave_hull(knots, U)
    return float(np.interp(b, knots[st].astype(np.float64), U[st].astype(np.float64)))


def _dp(value, NH, b_min, b_max, B):
    """Exact optimum of sum_h value(h, b_h) s.t. sum b_h = B, b_min <= b_h <= b_max."""
    NEG = -1e300
    best = [NEG] * (B + 1)
    best[0] = 0.0
    for h in range(NH):
        new = [NEG] * (B + 1)
        for tot in range(B + 1):
            if best[tot] == NEG:
                continue
            for b in range(int(b_min[h]), int(b_max[h]) + 1):
                if tot + b > B:
                    break
                new[tot + b] = max(new[tot + b], best[tot] + value(h, b))
        best = new
    return best[B]


def _random_problem(seed, NH, Gp, L):
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((NH, Gp))
    U = np.cumsum(0.5 * z * z, axis=1)
    U[:, 0] = 0
    U = (np.round(U * 64) / 64).astype(np.float32)       # dyadic values: sums are exact
    knots = np.tile(((np.arange(Gp) * L) // (Gp - 1)).astype(np.int32), (NH, 1))
    b_min = rng.integers(0, 3, size=NH).astype(np.int32)
    b_max = np.full(NH, L, np.int32) - rng.integers(0, 3, size=NH).astype(np.int32)
    return U, knots, b_min, b_max


@pytest.mark.parametrize("seed", range(6))
def test_greedy_matches_dp_on_relaxed_curves(seed):
    NH, Gp, L = 4, 6, 15
    U, knots, b_min, b_max = _random_problem(200 + seed, NH, Gp, L)
    for B in range(int(b_min.sum()), int(b_max.sum()) + 1, 3):
        b, st = O.allocate(U, knots, b_min, b_max, B)
        assert st == 0 and int(b.sum()) == B
        assert np.all(b >= b_min) and np.all(b <= b_max)
        relaxed = sum(_hull_value(knots[h], U[h], b[h]) for h in range(NH))
        dp_relaxed = _dp(lambda h, x: _hull_value(knots[h], U[h], x), NH, b_min, b_max, B)
        assert relaxed == pytest.approx(dp_relaxed, rel=1e-12, abs=1e-12)
        raw = sum(_interp(knots[h], U[h], b[h]) for h in range(NH))
        dp_raw = _dp(lambda h, x: _interp(knots[h], U[h], x), NH, b_min, b_max, B)
        assert raw <= dp_raw + 1e-12 and dp_raw <= relaxed + 1e-12


def test_exhaustive_two_heads_matches_greedy_objective():
    g, U, knots = _curves()
    zero, four = np.zeros(2, np.int32), np.full(2, 4, np.int32)
    for B in range(9):
        b, _ = O.allocate(U, knots, zero, four, B)
        got = sum(_hull_value(knots[h], U[h], b[h]) for h in range(2))
        best = max(_hull_value(knots[0], U[0], x) + _hull_value(knots[1], U[1], B - x)
                   for x in range(5) if 0 <= B - x <= 4)
        assert got == pytest.approx(best, rel=1e-14)
    raw3, dp3, rel3 = [float(Fraction(t)) for t in g["raw_B3"]]
    b, _ = O.allocate(U, knots, zero, four, 3)
    assert sum(_interp(knots[h], U[h], b[h]) for h in range(2)) == raw3
    assert _dp(lambda h, x: _interp(knots[h], U[h], x), 2, zero, four, 3) == dp3
    assert sum(_hull_value(knots[h], U[h], b[h]) for h in range(2)) == pytest.approx(rel3, rel=1e-14)


@pytest.mark.parametrize("seed", range(4))
def test_exhaustive_three_heads(seed):
    NH, Gp, L = 3, 4, 6
    U, knots, b_min, b_max = _random_problem(300 + seed, NH, Gp, L)
    for B in range(int(b_min.sum()), int(b_max.sum()) + 1):
        b, st = O.allocate(U, knots, b_min, b_max, B)
        assert st == 0
        got = sum(_hull_value(knots[h], U[h], b[h]) for h in range(NH))
        best = max(sum(_hull_value(knots[h], U[h], x[h]) for h in range(NH))
                   for x in itertools.product(*[range(int(b_min[h]), int(b_max[h]) + 1) for h in range(NH)])
                   if sum(x) == B)
        assert got == pytest.approx(best, rel=1e-12, abs=1e-12)


# --- invariants -------------------------------------------------------------------------

def test_gains_nonnegative_nonincreasing_and_concave_is_own_hull():
    U, knots, _, _ = _random_problem(400, 5, 12, 40)
    for h in range(5):
        g = [s[2] for s in O.marginal_gains(knots[h], U[h])]
        assert all(x >= 0 for x in g) and all(a > b for a, b in zip(g, g[1:]))
    x = np.arange(9)
    conc = np.sqrt(x).astype(np.float32)
    assert O.concave_hull(x.astype(np.int32), conc) == list(range(9))


def test_power_of_two_scaling_and_uniform_split():
    U, knots, b_min, b_max = _random_problem(401, 5, 12, 40)
    b1, _ = O.allocate(U, knots, b_min, b_max, 77)
    b2, _ = O.allocate(U * np.float32(0.25), knots, b_min, b_max, 77)
    assert b1.tolist() == b2.tolist()
    same = np.tile(U[:1], (5, 1))
    zero, full = np.zeros(5, np.int32), np.full(5, 40, np.int32)
    for B in (3, 17, 101):
        b, _ = O.allocate(same, knots, zero, full, B)
        assert int(b.sum()) == B
        # identical curves: a tied hull segment is filled head by head, lowest index first
        assert all(b[i] >= b[i + 1] for i in range(4))


def test_offsets_are_prefix_sums():
    assert O.offsets_of(np.array([3, 0, 5], np.int32)).tolist() == [0, 3, 3, 8]


# --- profile and look-up --------------------------------------------------------------------

def test_handworked_profile_and_lookup():
    g, U, knots = _curves()
    zero, four = np.zeros((1, 2), np.int32), np.full((1, 2), 4, np.int32)
    rho = [0.0, 0.25, 0.5, 0.75, 1.0]
    phi = O.profile_build(U[None], knots[None], zero, four, 4, rho)
    assert phi.dtype == np.float32 and phi.shape == (5, 2)
    assert phi[:, 0].tolist() == [float(Fraction(t)) for t in g["phi_h0"]]
    assert phi[:, 1].tolist() == [float(Fraction(t)) for t in g["phi_h1"]]
    for key, sigma in (("lookup_3_8", 0.375), ("lookup_5_8", 0.625)):
        b = O.budgets_from_profile(phi, rho, sigma, 4, zero[0], four[0])
        assert b.tolist() == [int(t) for t in g[key][0].split(",")]
    # on a grid ratio the look-up returns that row's budgets; outside the grid, the end rows
    assert O.budgets_from_profile(phi, rho, 0.5, 4, zero[0], four[0]).tolist() == [3, 1]
    assert O.budgets_from_profile(phi, rho, -1.0, 4, zero[0], four[0]).tolist() == [4, 4]
    assert O.budgets_from_profile(phi, rho, 2.0, 4, zero[0], four[0]).tolist() == [0, 0]
    # bounds clip the looked-up budgets
    assert O.budgets_from_profile(phi, rho, 0.625, 4, np.array([3, 0], np.int32), np.array([4, 0], np.int32)).tolist() == [3, 0]
    # two calibration queries: the mean of their local ratios (Eq. 11)
    U2 = np.stack([U, U[::-1]])
    phi2 = O.profile_build(U2, np.stack([knots, knots]), np.zeros((2, 2), np.int32), np.full((2, 2), 4, np.int32), 4, rho)
    assert phi2[2].tolist() == [float(Fraction(t)) for t in g["phi2_rho_1_2"]]


def test_profile_rows_reproduce_the_allocation_on_the_grid():
    """For one query, looking the profile up AT a grid ratio gives back that ratio's budgets
    (1 - b/L is exact in fp32 for these sizes), and the budgets sum to floor((1-rho) L NH)."""
    NH, Gp, L = 5, 9, 64
    U, knots, b_min, b_max = _random_problem(900, NH, Gp, L)
    b_min[:] = 0
    b_max[:] = L
    rho = [i / 8 for i in range(9)]
    phi = O.profile_build(U[None], knots[None], b_min[None], b_max[None], L, rho)
    for i, r in enumerate(rho):
        b = O.budgets_from_profile(phi, rho, r, L, b_min, b_max)
        want, st = O.allocate(U, knots, b_min, b_max, int((1 - r) * L * NH))
        assert st == 0 and b.tolist() == want.tolist()
    assert np.all(np.diff(phi, axis=0) >= 0)        # compressing more never keeps more in a head


def test_handworked_utility_curve_and_properties():
    g = _golden()
    imp = np.array([float(Fraction(t)) for t in g["curve_importance"]], np.float32)
    sc = np.array([float(Fraction(t)) for t in g["curve_scores"]], np.float32)
    assert O.utility_curve(imp, sc, range(5)).tolist() == [float(t) for t in g["curve_full"]]
    assert O.utility_curve(imp, sc, [0, 2, 4]).tolist() == [float(t) for t in g["curve_knots_0_2_4"]]
    rng = np.random.default_rng(31)
    T = 200
    imp = rng.random(T).astype(np.float32)
    sc = rng.integers(0, 20, T).astype(np.float32)          # many ties
    u = O.utility_curve(imp, sc, range(T + 1))
    assert u[0] == 0 and np.all(np.diff(u) >= 0) and u[-1] == pytest.approx(float(imp.astype(np.float64).sum()), rel=1e-6)
    # brute force: U(i) = importance of the i best tokens under (score desc, index asc)
    rank = sorted(range(T), key=lambda j: (-float(sc[j]), j))
    for i in (1, 7, 50, 199):
        assert u[i] == pytest.approx(sum(float(imp[j]) for j in rank[:i]), rel=1e-6)
    # ranking by the importance itself gives a concave curve (its own hull)
    u2 = O.utility_curve(imp, imp, range(T + 1))
    assert np.all(np.diff(u2, 2) <= 1e-6)
    assert np.all(u2 >= u - 1e-5)


# --- top-k and compaction -----------------------------------------------------------------

@pytest.mark.parametrize("seed", range(5))
def test_select_brute_force_with_ties(seed):
    rng = np.random.default_rng(500 + seed)
    n = 60
    s = rng.integers(0, 6, size=n).astype(np.float32) / 4       # many exact ties
    s[rng.integers(0, n, 4)] = np.inf
    s[rng.integers(0, n, 2)] = -0.0
    for k in (0, 1, 7, 30, n):
        got = O.select(s, k)
        # definition: i is kept iff fewer than k positions beat it
        # (strictly larger score, or equal score and lower index)
        want = [i for i in range(n)
                if sum(1 for j in range(n) if s[j] > s[i] or (s[j] == s[i] and j < i)) < k]
        assert got.tolist() == want
        assert got.dtype == np.int32


def test_compact_is_bitwise_gather():
    rng = np.random.default_rng(9)
    x = rng.integers(0, 65536, size=(20, 8)).astype(np.uint16)
    idx = np.array([0, 3, 19], np.int32)
    out = O.compact(x, idx)
    assert out.dtype == x.dtype and np.array_equal(out, x[[0, 3, 19]])
    out[0, 0] ^= 1
    assert x[0, 0] != out[0, 0]
