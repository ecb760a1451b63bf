"""CPU oracle for the LU-KV prefill-time eviction path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 statement of what the path computes, written from the paper:
  score    - Eq. 1 (scaled-dot-product softmax) applied to the SnapKV observation
             window (Sec. 2 "Intra-head Eviction Policies", App. D Table 8: window 32,
             kernel 7), with the always-kept sink / recent window of App. E;
  allocate - Sec. 4.2 "Efficient Optimization via Convex Hull Relaxation", Eq. 9-10 and
             App. A.2: convex surrogate, non-increasing marginal gains, unit-by-unit
             greedy until B_total is spent (Eq. 8's equality constraint);
  allocate_topk - the baseline allocation of Sec. 4.2's opening / Sec. 5.1 "Baselines": budgets
             from a global top-k over the pooled surrogate scores of all heads;
  select   - Sec. 3.2 symbol table, M^pi(k): top-k by the metric, descending, with the
             fixed deterministic tie rule App. A.1 assumes (lowest index first);
  compact  - Sec. 3.2 / Eq. 3: the retained index set I_{l,h} as a dense per-head cache;
  profile  - Sec. 4.3, Eq. 11 and "Online Execution": the static table of local ratios over a
             grid of global ratios, and the look-up that turns a target ratio into budgets;
  decode   - Sec. 3.2, Eq. 3: a decode step's attention over the retained entries (the consumer
             of the compacted cache).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module.  It shares no code with the HIP path and never calls it.

Parity pins (tests/test_oracle_*.py): hand-worked softmax/pool and hull/greedy cases,
closed forms, brute-force definitions, unit-level PAVA, exhaustive and DP search.
Not pinned by anything: whether these scores and budgets reach the paper's
LongBench / RULER quality (needs model weights and datasets) - parity unpinned.

Readings of points the paper leaves open are listed next to each function.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np


# ----------------------------------------------------------------------------
# storage decoding (the oracle's own; nothing here is shared with the GPU path)
# ----------------------------------------------------------------------------

def decode(x: np.ndarray) -> np.ndarray:
    """Stored tensor -> float64.  uint16 arrays are bfloat16 bit patterns."""
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


# ----------------------------------------------------------------------------
# step 1: observation-window score (Eq. 1; SnapKV metric)
# ----------------------------------------------------------------------------

def window_attention_sum(q_win: np.ndarray, k: np.ndarray, n_kv_heads: int,
                         scale: float | None = None, lse: np.ndarray | None = None) -> np.ndarray:
    """Unpooled metric: for every KV head, the attention mass each cached position
    receives from the last w queries, summed over the window and averaged over the
    G query heads that share the KV head.

    q_win [H_q, w, d], k [H_kv, L, d] (float64).  Returns [H_kv, L] float64.

    Eq. 1: A = softmax_j(q.k_j / sqrt(d_h)) over the keys visible to the query.
    Readings: window row i sits at position L-w+i and sees keys j <= L-w+i (Eq. 1's
    j <= k); the sum (not mean) over the window ("accumulated attention scores");
    mean over the group's query heads, taken before pooling.

    lse [H_q, w] (optional): the log of Eq. 1's denominator for every window row, as a
    prefill attention kernel leaves it (natural log of the sum over the visible keys of
    exp(scaled logit)).  When given it is used as the normaliser, A = exp(s - lse), instead
    of being recomputed (Sec. 4.3: the scores are a by-product of prefill).
    """
    H_q, w, d = q_win.shape
    H_kv, L, _ = k.shape
    G = H_q // n_kv_heads
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros((H_kv, L), dtype=np.float64)
    j = np.arange(L)[None, :]
    t = (L - w + np.arange(w))[:, None]
    visible = j <= t                                   # [w, L]
    for c in range(H_kv):
        acc = np.zeros(L, dtype=np.float64)
        for g in range(G):
            s = scale * (q_win[c * G + g] @ k[c].T)    # [w, L]
            s = np.where(visible, s, -np.inf)
            if lse is not None:
                p = np.exp(s - np.asarray(lse[c * G + g], dtype=np.float64)[:, None])
            else:
                m = s.max(axis=1, keepdims=True)
                e = np.exp(s - m)
                p = e / e.sum(axis=1, keepdims=True)
            acc += p.sum(axis=0)
        out[c] = acc / G
    return out


def max_pool_1d(r: np.ndarray, kernel: int) -> np.ndarray:
    """Stride-1 max-pool with the window clipped at both ends:
    out[j] = max r[max(0, j-h) .. min(n-1, j+h)], h = kernel // 2 (kernel odd)."""
    n = r.shape[-1]
    h = kernel // 2
    pad = np.full(r.shape[:-1] + (h,), -np.inf)
    padded = np.concatenate([pad, r, pad], axis=-1)
    out = np.full(r.shape, -np.inf)
    for t in range(kernel):
        out = np.maximum(out, padded[..., t:t + n])
    return out


def window_lse(q_win: np.ndarray, k: np.ndarray, n_kv_heads: int,
               scale: float | None = None) -> np.ndarray:
    """log of Eq. 1's denominator for every window row: lse[q, i] = log sum_{j <= L-w+i}
    exp(scale * q_i . k_j), float64 [H_q, w].  What a prefill attention kernel returns
    beside its output; an INPUT of the lse variant of the score step."""
    H_q, w, d = q_win.shape
    H_kv, L, _ = k.shape
    G = H_q // n_kv_heads
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros((H_q, w), dtype=np.float64)
    for qh in range(H_q):
        s = scale * (q_win[qh] @ k[qh // G].T)
        for i in range(w):
            row = s[i, :L - w + i + 1]
            m = row.max()
            out[qh, i] = m + math.log(np.exp(row - m).sum())
    return out


def score(q_win: np.ndarray, k: np.ndarray, n_kv_heads: int, window: int,
          pool_kernel: int, n_sink: int, scale: float | None = None,
          lse: np.ndarray | None = None) -> np.ndarray:
    """Pooled SnapKV score S [H_kv, L] float32.

    The window sum is pooled over the prefix [0, L-w) only; the result is rounded to
    float32; then the recent window (j >= L-w) and the first n_sink positions are
    forced to +inf: they are always kept (App. E) and count against the head's budget.
    """
    L = k.shape[1]
    P = L - window
    if P < 1:
        raise ValueError("context must be longer than the observation window")
    r = window_attention_sum(q_win, k, n_kv_heads, scale, lse)
    s = np.full(r.shape, np.inf, dtype=np.float32)
    s[:, :P] = max_pool_1d(r[:, :P], pool_kernel).astype(np.float32)
    s[:, :min(n_sink, L)] = np.inf
    return s


# ----------------------------------------------------------------------------
# step 2: global head-level budget allocation (Sec. 4.2, Eq. 8-10, App. A.2)
# ----------------------------------------------------------------------------

def _slope(knots: Sequence[int], U: Sequence[float], a: int, b: int) -> float:
    """Canonical gain of one unit on the chord a->b: one fp64 subtract, one fp64 divide."""
    return float((np.float64(U[b]) - np.float64(U[a])) / np.float64(int(knots[b]) - int(knots[a])))


def concave_hull(knots: Sequence[int], U: Sequence[float]) -> List[int]:
    """Indices of the knots that are vertices of the upper concave hull of (knots[g], U[g]).

    The profiled utility U(i) = L(0) - L(i) is the retained importance mass; the
    paper's convex non-increasing surrogate of the loss is obtained by the
    Pool-Adjacent-Violators scan over the marginal decreases (Sec. 4.2, App. A.2),
    which is the least concave majorant of U.  Between grid knots U is taken linear,
    so the hull of the knots is the hull of the curve.

    The scan, left to right over the grid intervals: every interval starts as a block
    of its own whose gain is the mean marginal decrease over the block, i.e. the chord
    between the block's end knots; while the newest block's gain is not strictly below
    the gain of the block before it, the two are pooled into one block (whose gain is
    again the chord between ITS end knots).  The blocks that remain have strictly
    decreasing gains; their end knots are the hull vertices (collinear knots pool away).
    """
    ends: List[int] = [0]                  # ends[i], ends[i+1] = end knots of block i
    for g in range(1, len(knots)):
        ends.append(g)
        while len(ends) >= 3 and _slope(knots, U, ends[-3], ends[-2]) <= _slope(knots, U, ends[-2], ends[-1]):
            del ends[-2]                   # pool the last two blocks
    return ends


def marginal_gains(knots: Sequence[int], U: Sequence[float]) -> List[Tuple[int, int, float]]:
    """Hull segments (n_a, n_b, gain): Eq. 9's g(i) = gain for every unit i in (n_a, n_b]."""
    st = concave_hull(knots, U)
    return [(int(knots[a]), int(knots[b]), _slope(knots, U, a, b)) for a, b in zip(st[:-1], st[1:])]


def _gain_of_unit(segs: List[Tuple[int, int, float]], u: int) -> float:
    for lo, hi, g in segs:
        if lo < u <= hi:
            return g
    return -math.inf


def allocate(curves: np.ndarray, knots: np.ndarray, b_min: np.ndarray, b_max: np.ndarray,
             B: int) -> Tuple[np.ndarray, int]:
    """Greedy allocation on the relaxed curves (App. A.2 "Optimality of greedy allocation").

    curves [NH, Gp] float32, knots [NH, Gp] int (knots[:,0] = 0, strictly increasing),
    b_min/b_max [NH].  Every head first receives b_min units (minimum retention,
    App. E); then one unit at a time goes to the head whose next unit has the largest
    gain, until sum(budgets) = B.  Equal gains: lowest head index first.
    Returns (budgets int32 [NH], status); status 1 = infeasible (budgets = b_min): B outside
    [sum b_min, sum min(b_max, last knot)], or a bound that is no retention count (b_min < 0 or
    b_min above the head's cap).
    """
    NH = curves.shape[0]
    segs = [marginal_gains(knots[h], curves[h]) for h in range(NH)]
    budgets = np.array([int(x) for x in b_min], dtype=np.int64)
    cap = np.minimum(np.array([int(x) for x in b_max], dtype=np.int64), knots[:, -1].astype(np.int64))
    R = int(B) - int(budgets.sum())
    if R < 0 or R > int(np.maximum(cap - budgets, 0).sum()) or np.any(budgets > cap) or np.any(budgets < 0):
        return budgets.astype(np.int32), 1

    def next_gain(h: int) -> float:
        return _gain_of_unit(segs[h], int(budgets[h]) + 1) if budgets[h] < cap[h] else -math.inf

    nxt = np.array([next_gain(h) for h in range(NH)], dtype=np.float64)
    for _ in range(R):
        h = int(np.argmax(nxt))          # first maximum = lowest head index
        budgets[h] += 1
        nxt[h] = next_gain(h)
    return budgets.astype(np.int32), 0


def allocate_topk(scores: Sequence[np.ndarray], B_total: int, floor: int = 0) -> Tuple[np.ndarray, bool]:
    """The baseline allocation Sec. 4.2's opening and Sec. 5.1 "Baselines" describe (global
    top-k): the candidate positions of all heads are pooled and the B_total of largest surrogate
    score are retained; a head's budget is the number of its positions among them.  `floor` is
    the safeguard (App. D Table 8 gives AdaKV a safeguard ratio; the floor in tokens is the
    caller's): the `floor` best positions of every head are retained first, the remaining
    B_total - H * floor places go to the best of all other candidates.

    scores: one float32 vector per head (lengths may differ).  Pooled candidates are ordered by
    (score descending, head ascending, position ascending) - the tie rule of `select`, extended
    by the head index (reading R-T1).  Returns (budgets int32 [H], feasible); infeasible
    (floor beyond a head's length, B_total < H * floor, B_total beyond the number of candidates)
    gives budgets = floor for every head.
    """
    H = len(scores)
    lens = [int(len(s)) for s in scores]
    budgets = np.full(H, floor, dtype=np.int32)
    if floor < 0 or any(floor > n for n in lens) or B_total < H * floor or B_total > sum(lens):
        return budgets, False
    head, pos, val = [], [], []                    # every candidate outside the floors
    for h, s in enumerate(scores):
        outside = np.ones(lens[h], dtype=bool)
        outside[select(np.asarray(s), floor)] = False
        pos.append(np.nonzero(outside)[0])
        head.append(np.full(len(pos[-1]), h, dtype=np.int64))
        val.append(np.asarray(s, dtype=np.float64)[pos[-1]])
    head, pos, val = np.concatenate(head), np.concatenate(pos), np.concatenate(val)
    order = np.lexsort((pos, head, -val))          # last key is the primary one
    taken = order[:B_total - H * floor]
    budgets += np.bincount(head[taken], minlength=H).astype(np.int32)
    return budgets, True


def offsets_of(budgets: np.ndarray) -> np.ndarray:
    """Row offset of every head in the packed outputs: exclusive prefix sum, int64 [NH+1]."""
    return np.concatenate([[0], np.cumsum(budgets.astype(np.int64))]).astype(np.int64)


# ----------------------------------------------------------------------------
# offline profile and online look-up (Sec. 4.3, Eq. 11; "Online Execution" steps 1-2)
# ----------------------------------------------------------------------------

def utility_curve(importance: np.ndarray, scores: np.ndarray, knots: Sequence[int]) -> np.ndarray:
    """Profiled utility of one head on a grid of budgets (Sec. 4.1, Eq. 6 read as R-A1): the
    tokens are ranked by the heuristic metric (descending score, ties to the lowest index, the
    order M^pi takes them in) and U(i) = L(0) - L(M^pi(i)) is the importance mass of the first
    i tokens of that ranking.  importance [T] >= 0, scores [T]; returns U at the knots, float32
    (fp64 running sum in ranking order, rounded once)."""
    order = np.argsort(-np.asarray(scores, dtype=np.float64), kind="stable")
    u = np.concatenate([[0.0], np.cumsum(np.asarray(importance, dtype=np.float64)[order])])
    return u[np.asarray(knots, dtype=np.int64)].astype(np.float32)


def profile_build(curves: np.ndarray, knots: np.ndarray, b_min: np.ndarray, b_max: np.ndarray,
                  L: int, rho: Sequence[float]) -> np.ndarray:
    """Static profile Phi[n_rho, NH] (float32): for every calibration query m and every global
    compression ratio rho on the grid, solve the relaxed allocation (Eq. 10) with
    B = floor((1 - rho) * L * NH) and take the local ratios r* = 1 - b / L; Phi is their mean
    over the queries (Eq. 11).

    curves, knots [M, NH, Gp]; b_min, b_max [M, NH].  Reading: a ratio whose budget is not
    feasible (below the minimum retention) takes allocate()'s documented result, b = b_min.
    The mean is the fp64 sum over m in order, divided by M, rounded to float32.
    """
    M, NH = curves.shape[0], curves.shape[1]
    phi = np.zeros((len(rho), NH), dtype=np.float64)
    for ri, r in enumerate(rho):
        B = int(math.floor((1.0 - float(r)) * float(L) * float(NH)))
        acc = np.zeros(NH, dtype=np.float64)
        for m in range(M):
            b, _ = allocate(curves[m], knots[m], b_min[m], b_max[m], B)
            acc = acc + (1.0 - b.astype(np.float64) / float(L))
        phi[ri] = acc / float(M)
    return phi.astype(np.float32)


def budgets_from_profile(phi: np.ndarray, rho: Sequence[float], sigma: float, L: int,
                         b_min: np.ndarray, b_max: np.ndarray) -> np.ndarray:
    """Online steps 1-2: look the local ratios up at the target global ratio sigma (linear
    between the two neighbouring grid ratios, end values outside the grid) and turn them into
    integer budgets b = floor((1 - r) * L), kept inside [b_min, b_max].  fp64 throughout:
    t = (sigma - rho_i) / (rho_{i+1} - rho_i), r = phi_i + t * (phi_{i+1} - phi_i)."""
    rho = [float(x) for x in rho]
    n = len(rho)
    if n == 1 or sigma <= rho[0]:
        r = phi[0].astype(np.float64)
    elif sigma >= rho[-1]:
        r = phi[-1].astype(np.float64)
    else:
        i = max(j for j in range(n - 1) if rho[j] <= sigma)
        t = (float(sigma) - rho[i]) / (rho[i + 1] - rho[i])
        lo, hi = phi[i].astype(np.float64), phi[i + 1].astype(np.float64)
        r = lo + t * (hi - lo)
    b = np.floor((1.0 - r) * float(L)).astype(np.int64)
    b = np.minimum(np.maximum(b, b_min.astype(np.int64)), b_max.astype(np.int64))
    return b.astype(np.int32)


# ----------------------------------------------------------------------------
# step 3: per-head top-k (M^pi(k)) and step 4: compaction
# ----------------------------------------------------------------------------

def select(s: np.ndarray, k: int) -> np.ndarray:
    """The k positions of largest score, ties to the lowest index, returned ascending."""
    order = np.argsort(-s.astype(np.float64), kind="stable")
    return np.sort(order[:k]).astype(np.int32)


def compact(x: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Rows idx of x [L, d], bit for bit, in the given order."""
    return x[idx].copy()


# ----------------------------------------------------------------------------
# consumer of the compacted cache: one decode step (Sec. 3.2, Eq. 3)
# ----------------------------------------------------------------------------

def decode_attention(q: np.ndarray, k_rows: np.ndarray, v_rows: np.ndarray,
                     scale: float | None = None) -> np.ndarray:
    """Attention of decode queries over the retained entries of one KV head (Eq. 3 restricted to
    the index set I_{l,h}): out[g] = softmax_r(scale * q[g] . k_rows[r]) @ v_rows.

    q [G, d] (the query heads of the group), k_rows, v_rows [n, d], all float64.  Returns
    [G, d] float64.  n = 0 gives zeros (nothing to attend to)."""
    G, d = q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    if k_rows.shape[0] == 0:
        return np.zeros((G, d), dtype=np.float64)
    s = scale * (q @ k_rows.T)                                  # [G, n]
    p = np.exp(s - s.max(axis=1, keepdims=True))
    p = p / p.sum(axis=1, keepdims=True)
    return p @ v_rows


# ----------------------------------------------------------------------------
# whole path
# ----------------------------------------------------------------------------

def evict(q_win: np.ndarray, k: np.ndarray, v: np.ndarray, cu_seqlens: Sequence[int],
          n_kv_heads: int, window: int, pool_kernel: int, n_sink: int,
          curves: np.ndarray, knots: np.ndarray, b_min: np.ndarray, b_max: np.ndarray,
          B: Sequence[int], layers: Sequence[int] | None = None, scale: float | None = None,
          lse: np.ndarray | None = None):
    """score -> allocate -> select -> compact for packed sequences.

    q_win [NL, H_q, n_seqs*w, d], k, v [NL, H_kv, total_len, d] as stored (bf16 bits or
    f32); curves/knots [n_seqs, NL*H_kv, Gp]; b_min/b_max [n_seqs, NL*H_kv]; B [n_seqs].
    Heads are ordered (sequence, layer, kv head).  `layers` restricts scoring/selection to
    some layers (allocation is always global); other layers get empty outputs.
    lse [NL, H_q, n_seqs*w] float32 (optional): the window rows' log-sum-exp, see score().

    Returns dict: budgets [n_seqs*NL*H_kv], offsets [..+1], status [n_seqs],
    pooled {(s, l): [H_kv, L_s] f32}, kept {(s, l, c): int32 idx}, k_out/v_out {(s,l,c): rows}.
    """
    NL, H_q = q_win.shape[0], q_win.shape[1]
    n_seqs = len(cu_seqlens) - 1
    budgets, status = [], []
    for s in range(n_seqs):
        b, st = allocate(curves[s], knots[s], b_min[s], b_max[s], int(B[s]))
        budgets.append(b)
        status.append(st)
    budgets = np.concatenate(budgets)
    offsets = offsets_of(budgets)
    pooled, kept, k_out, v_out = {}, {}, {}, {}
    use_layers = range(NL) if layers is None else layers
    for s in range(n_seqs):
        a, b = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        for l in use_layers:
            q = decode(q_win[l, :, s * window:(s + 1) * window, :])
            kk = decode(k[l, :, a:b, :])
            row_lse = None if lse is None else lse[l, :, s * window:(s + 1) * window]
            S = score(q, kk, n_kv_heads, window, pool_kernel, n_sink, scale, row_lse)
            pooled[(s, l)] = S
            for c in range(n_kv_heads):
                hi = (s * NL + l) * n_kv_heads + c
                idx = select(S[c], int(budgets[hi]))
                kept[(s, l, c)] = idx
                k_out[(s, l, c)] = compact(k[l, c, a:b, :], idx)
                v_out[(s, l, c)] = compact(v[l, c, a:b, :], idx)
    return {"budgets": budgets, "offsets": offsets, "status": np.array(status, dtype=np.int32),
            "pooled": pooled, "kept": kept, "k_out": k_out, "v_out": v_out}
