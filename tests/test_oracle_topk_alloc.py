"""Pins of the oracle's baseline allocation (global top-k over the pooled scores of all heads,
Sec. 4.2 opening / Sec. 5.1 "Baselines"): a hand-worked case, the definition as an exhaustive
search over subsets, the tie rule, and the properties that hold at any size."""
import itertools

import numpy as np
import pytest

from oracle import lukv_oracle as O


def _f32(*rows):
    return [np.asarray(r, dtype=np.float32) for r in rows]


def test_handworked_global_topk():
    """Three heads, scores written down; the five largest of the nine candidates are 9, 8, 7
    (head 0), 6 (head 2), 5 (head 1)."""
    sc = _f32([9, 1, 8, 7], [5, 2], [3, 6, 4])
    b, ok = O.allocate_topk(sc, 5)
    assert ok and b.tolist() == [3, 1, 1] and b.dtype == np.int32
    # one more place: 4 (head 2)
    assert O.allocate_topk(sc, 6)[0].tolist() == [3, 1, 2]
    # floor of one position per head changes nothing here (every head already holds one) ...
    assert O.allocate_topk(sc, 5, floor=1)[0].tolist() == [3, 1, 1]
    # ... a floor of two does: head 1 keeps {5, 2}, head 2 keeps {6, 4}, head 0 keeps {9, 8}; of the
    # five places none is left beyond the six guaranteed ones -> infeasible; with seven places the
    # one free place goes to 7 (head 0)
    b, ok = O.allocate_topk(sc, 5, floor=2)
    assert not ok and b.tolist() == [2, 2, 2]
    b, ok = O.allocate_topk(sc, 7, floor=2)
    assert ok and b.tolist() == [3, 2, 2]
    # the safeguard at work: without it head 1 would get nothing
    assert O.allocate_topk(_f32([9, 8, 7], [1, 0.5]), 3)[0].tolist() == [3, 0]
    assert O.allocate_topk(_f32([9, 8, 7], [1, 0.5]), 3, floor=1)[0].tolist() == [2, 1]
    # the guaranteed positions do not compete again for the free places: 9 and 8 are guaranteed,
    # the one free place goes to the better of {1, 7}
    assert O.allocate_topk(_f32([9, 1], [8, 7]), 3, floor=1)[0].tolist() == [1, 2]


def test_ties_go_to_the_lowest_head_then_the_lowest_position():
    sc = _f32([1, 1, 1, 1], [1, 1, 1, 1], [1, 1, 1, 1])
    assert O.allocate_topk(sc, 6)[0].tolist() == [4, 2, 0]
    assert O.allocate_topk(sc, 6, floor=1)[0].tolist() == [4, 1, 1]
    # a tie at the cut only: 5 > 3 = 3 = 3 > 1
    sc = _f32([1, 3], [3, 5], [3, 0])
    assert O.allocate_topk(sc, 2)[0].tolist() == [1, 1, 0]
    assert O.allocate_topk(sc, 3)[0].tolist() == [1, 2, 0]
    assert O.allocate_topk(sc, 4)[0].tolist() == [1, 2, 1]


def test_forced_positions_come_first():
    """Scores of +inf (sink and observation window) are retained before anything finite."""
    inf = np.inf
    sc = _f32([inf, 0.5, 0.1, inf], [inf, 0.9, 0.8, inf])
    assert O.allocate_topk(sc, 4)[0].tolist() == [2, 2]
    assert O.allocate_topk(sc, 5)[0].tolist() == [2, 3]
    assert O.allocate_topk(sc, 3)[0].tolist() == [2, 1]      # ties among the infinities: lowest head first


def test_infeasible_cases():
    sc = _f32([3, 2, 1], [6, 5])
    for B, floor in ((6, 0), (1, 1), (5, 3), (2, -1)):
        b, ok = O.allocate_topk(sc, B, floor)
        assert not ok and b.tolist() == [floor, floor]
    assert O.allocate_topk(sc, 5)[0].tolist() == [3, 2]
    assert O.allocate_topk(sc, 0)[0].tolist() == [0, 0]


def _best_subset(scores, B, floor):
    """The definition as a search: among all sets of B candidates that hold at least `floor`
    of every head, the one of largest total score (unique when the scores are distinct, and it
    necessarily holds each head's `floor` best)."""
    cands = [(h, j) for h, s in enumerate(scores) for j in range(len(s))]
    best, best_sum = None, -np.inf
    for sub in itertools.combinations(cands, B):
        cnt = np.bincount([h for h, _ in sub], minlength=len(scores))
        if cnt.min() < floor:
            continue
        tot = sum(float(scores[h][j]) for h, j in sub)
        if tot > best_sum:
            best, best_sum = cnt, tot
    return best


@pytest.mark.parametrize("seed", range(6))
def test_equals_exhaustive_search_on_tiny_inputs(seed):
    rng = np.random.default_rng(seed)
    lens = rng.integers(2, 5, size=3)
    vals = rng.permutation(np.arange(1, lens.sum() + 1)).astype(np.float32)      # distinct
    sc, o = [], 0
    for n in lens:
        sc.append(vals[o:o + n])
        o += n
    for floor in (0, 1):
        for B in range(3 * floor, int(lens.sum()) + 1):
            want = _best_subset(sc, B, floor)
            got, ok = O.allocate_topk(sc, B, floor)
            assert ok and got.tolist() == want.tolist(), (seed, B, floor)


@pytest.mark.parametrize("seed", range(4))
def test_properties_at_size(seed):
    rng = np.random.default_rng(100 + seed)
    H = 8
    lens = rng.integers(300, 3000, size=H)
    sc = [np.round(rng.gamma(0.3, 1.0, size=n), 2).astype(np.float32) for n in lens]   # many ties
    for s in sc:
        s[:4] = np.inf
        s[-32:] = np.inf
    floor = 50
    prev = None
    for B in (H * floor, H * floor + 1, 3000, 3001, 3002, int(lens.sum()) - 1, int(lens.sum())):
        b, ok = O.allocate_topk(sc, B, floor)
        assert ok and int(b.sum()) == B and np.all(b >= floor) and np.all(b <= lens)
        # the retained sets, head by head, are exactly the best B of the pooled candidates
        # under the order (score desc, head asc, position asc), floors aside
        kept = [set(O.select(sc[h], int(b[h])).tolist()) for h in range(H)]
        want = [set(O.select(sc[h], floor).tolist()) for h in range(H)]
        free = sorted((-float(sc[h][j]), h, j) for h in range(H) for j in range(lens[h]) if j not in want[h])
        for _, h, j in free[:B - H * floor]:
            want[h].add(j)
        assert kept == want
        if prev is not None and B == prev[0] + 1:
            d = b - prev[1]
            assert d.min() == 0 and d.sum() == 1            # one more place -> exactly one head grows
        prev = (B, b)
    # invariance: a positive scale on every score, or listing the heads in reverse when no two
    # candidates tie across heads, does not change who gets what
    b0 = O.allocate_topk(sc, 3000, floor)[0]
    assert np.array_equal(O.allocate_topk([s * np.float32(4.0) for s in sc], 3000, floor)[0], b0)
    distinct = [(rng.permutation(n) + 10000 * h).astype(np.float32) for h, n in enumerate(lens)]
    bd = O.allocate_topk(distinct, 3000, floor)[0]
    assert np.array_equal(O.allocate_topk(distinct[::-1], 3000, floor)[0], bd[::-1])
    assert O.allocate_topk([sc[0]], 123)[0].tolist() == [123]
