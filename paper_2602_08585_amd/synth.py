"""Seeded synthetic inputs for the LU-KV eviction path.

This module only *draws inputs*: window queries, cached keys/values, profiled
utility curves, grid knots and per-head bounds.  It holds none of the method's
arithmetic (no softmax, pooling, hull, top-k or gather), so the CPU oracle and
the HIP path may both consume what it returns.

The inputs stand in for the paper's long-context prompts on Llama-3.1-8B-class
GQA attention (Sec. 5.1): shapes are the model's, values mimic an attention
sink plus sparse heavy hitters.  No benchmark item is used or reproduced.

Everything is generated on the host from a counter-based generator
(numpy Philox) keyed by (seed, layer, sequence), rounded to the storage dtype,
and returned as numpy arrays; bf16 tensors are returned as uint16 bit patterns.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import numpy as np

BF16 = "bf16"
F32 = "f32"


@dataclasses.dataclass
class Workload:
    """Shape and recipe of one synthetic eviction problem."""

    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_lens: List[int]            # one entry per packed sequence
    window: int
    pool_kernel: int = 7
    n_sink: int = 4
    dtype: str = BF16
    keep_ratio: float = 0.2
    n_grid: int = 64
    heavy_frac: float = 0.01       # fraction of prefix positions planted as heavy hitters
    heavy_spans: int = 0           # >0: heavy hitters clustered in this many spans ...
    heavy_span_len: int = 256      # ... of this many consecutive tokens
    curve_family: str = "gamma"    # "gamma" | "mixed" | "spread"
    q_gain: float = 1.0            # multiplies Q; 1.0 is the literal recipe
    seed: int = 0x5EED0000

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_seqs(self) -> int:
        return len(self.seq_lens)

    @property
    def total_len(self) -> int:
        return int(sum(self.seq_lens))

    @property
    def cu_seqlens(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seq_lens)]).astype(np.int32)

    @property
    def heads_per_problem(self) -> int:
        """Heads that share one global budget: every (layer, kv head) of a sequence."""
        return self.n_layers * self.n_kv_heads

    def budget_total(self, seq: int) -> int:
        """B = floor(keep_ratio * L * number of heads in the problem)."""
        # the ratio is applied in exact integer arithmetic on a 1e-6 grid so
        # that floor() does not depend on binary rounding of e.g. 0.2
        num = int(round(self.keep_ratio * 1_000_000))
        return (num * self.seq_lens[seq] * self.heads_per_problem) // 1_000_000


def _ragged_lengths(seed: int, n: int, lo: int, hi: int) -> List[int]:
    rng = np.random.Generator(np.random.Philox(key=seed))
    return [int(x) for x in rng.integers(lo, hi + 1, size=n)]


def workload(name: str) -> Workload:
    """The five named configurations (Tiny, 8B/32k layer, full 8B prefill,
    long context, ragged batch)."""
    if name == "tiny":
        return Workload("tiny", 1, 8, 4, 64, [1024], 16, dtype=F32, n_grid=32,
                        heavy_frac=0.02, seed=0x5EED0000 + 1)
    if name == "8b_32k":
        return Workload("8b_32k", 1, 32, 8, 128, [32768], 32, seed=0x5EED0000 + 2)
    if name == "8b_full_20":
        return Workload("8b_full_20", 32, 32, 8, 128, [32768], 32, curve_family="mixed",
                        seed=0x5EED0000 + 3)
    if name == "8b_full_10":
        return Workload("8b_full_10", 32, 32, 8, 128, [32768], 32, keep_ratio=0.1,
                        curve_family="mixed", seed=0x5EED0000 + 3)
    if name == "long_128k":
        return Workload("long_128k", 32, 32, 8, 128, [131072], 64, keep_ratio=0.05,
                        heavy_spans=16, heavy_span_len=256, curve_family="mixed",
                        seed=0x5EED0000 + 4)
    if name == "batched":
        lens = _ragged_lengths(0x5EED0000 + 5, 16, 4096, 65536)
        return Workload("batched", 1, 32, 8, 128, lens, 32, curve_family="spread",
                        seed=0x5EED0000 + 5)
    raise KeyError(name)


# ----------------------------------------------------------------------------
# storage formats
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == BF16:
        return f32_to_bf16_bits(x)
    return np.ascontiguousarray(x, dtype=np.float32)


# ----------------------------------------------------------------------------
# Q / K / V
# ----------------------------------------------------------------------------

def _rng(seed: int, *stream: int) -> np.random.Generator:
    key = seed
    for s in stream:
        key = (key * 1000003 + s + 1) & 0xFFFFFFFFFFFFFFFF
    return np.random.Generator(np.random.Philox(key=key))


def make_layer_qkv(wl: Workload, layer: int) -> Dict[str, np.ndarray]:
    """Window queries and cached K/V of one layer, for every packed sequence.

    Returns float32 *unrounded* construction rounded to the storage dtype:
      q_win [n_q_heads, n_seqs*window, d], k, v [n_kv_heads, total_len, d].
    Per sequence: entries ~ N(0,1)/sqrt(d); key 0 scaled x4 (sink); a fraction of
    prefix positions per KV head replaced by 3*|k_j|*qbar/|qbar| where qbar is the
    mean window query of that KV head's group (heavy hitters).
    """
    d, w, G = wl.head_dim, wl.window, wl.group
    inv = 1.0 / math.sqrt(d)
    q_all = np.empty((wl.n_q_heads, wl.n_seqs * w, d), dtype=np.float32)
    k_all = np.empty((wl.n_kv_heads, wl.total_len, d), dtype=np.float32)
    v_all = np.empty((wl.n_kv_heads, wl.total_len, d), dtype=np.float32)
    cu = wl.cu_seqlens
    for s, L in enumerate(wl.seq_lens):
        rng = _rng(wl.seed, layer, s)
        q = rng.standard_normal((wl.n_q_heads, w, d), dtype=np.float32) * np.float32(inv * wl.q_gain)
        k = rng.standard_normal((wl.n_kv_heads, L, d), dtype=np.float32) * np.float32(inv)
        v = rng.standard_normal((wl.n_kv_heads, L, d), dtype=np.float32) * np.float32(inv)
        k[:, 0, :] *= np.float32(4.0)
        P = L - w
        for c in range(wl.n_kv_heads):
            qbar = q[c * G:(c + 1) * G].reshape(-1, d).mean(axis=0)
            qbar = qbar / np.float32(np.linalg.norm(qbar))
            if wl.heavy_spans > 0:
                starts = rng.integers(1, max(2, P - wl.heavy_span_len), size=wl.heavy_spans)
                pos = np.unique(np.concatenate(
                    [np.arange(st, min(P, st + wl.heavy_span_len)) for st in starts]))
            else:
                n_heavy = int(wl.heavy_frac * P)
                pos = np.sort(rng.choice(np.arange(1, P), size=n_heavy, replace=False)) \
                    if n_heavy > 0 else np.zeros(0, dtype=np.int64)
            if pos.size:
                norms = np.linalg.norm(k[c, pos, :], axis=1, keepdims=True).astype(np.float32)
                k[c, pos, :] = np.float32(3.0) * norms * qbar[None, :]
        q_all[:, s * w:(s + 1) * w, :] = q
        k_all[:, cu[s]:cu[s + 1], :] = k
        v_all[:, cu[s]:cu[s + 1], :] = v
    return {"q_win": _store(q_all, wl.dtype), "k": _store(k_all, wl.dtype),
            "v": _store(v_all, wl.dtype)}


def make_decode_queries(wl: Workload, layers: Optional[List[int]] = None) -> np.ndarray:
    """One decode query per (layer, query head, sequence): entries ~ N(0,1) * q_gain / sqrt(d),
    rounded to the storage dtype; [NL, H_q, n_seqs, d] (the consumer test of the packed cache)."""
    layers = list(range(wl.n_layers)) if layers is None else layers
    d = wl.head_dim
    out = np.empty((len(layers), wl.n_q_heads, wl.n_seqs, d), dtype=np.float32)
    for li, layer in enumerate(layers):
        rng = _rng(wl.seed, 4242, layer)
        out[li] = rng.standard_normal((wl.n_q_heads, wl.n_seqs, d), dtype=np.float32) * \
            np.float32(wl.q_gain / math.sqrt(d))
    return _store(out, wl.dtype)


def make_qkv(wl: Workload, layers: Optional[List[int]] = None, workers: int = 1) -> Dict[str, np.ndarray]:
    """Stack `make_layer_qkv` over layers: q_win [NL, H_q, n_seqs*w, d],
    k, v [NL, H_kv, total_len, d].  workers > 1 draws layers on that many host threads (every
    layer has its own keyed generator, so the result does not depend on it)."""
    layers = list(range(wl.n_layers)) if layers is None else layers
    if workers > 1 and len(layers) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as pool:
            parts = list(pool.map(lambda l: make_layer_qkv(wl, l), layers))
    else:
        parts = [make_layer_qkv(wl, l) for l in layers]
    return {key: np.stack([p[key] for p in parts]) for key in ("q_win", "k", "v")}


# ----------------------------------------------------------------------------
# utility curves, knots, bounds
# ----------------------------------------------------------------------------

def make_knots(L: int, n_grid: int) -> np.ndarray:
    """Integer grid n_g = floor(g*L/(n_grid-1)), g = 0..n_grid-1 (needs L >= n_grid-1)."""
    g = np.arange(n_grid, dtype=np.int64)
    return ((g * L) // (n_grid - 1)).astype(np.int32)


def make_curves(wl: Workload, seq: int = 0) -> np.ndarray:
    """Profiled utility curves U[heads_per_problem, n_grid], float32, non-decreasing,
    U[:,0] = 0, generally non-concave.

    "gamma":  cumulative sums of Gamma(1/2) increments (z^2/2, z ~ N(0,1)).
    "mixed":  per head one of saturating 1-exp(-x/tau), flat-then-steep x^p, or a
              logistic knee, plus small Gamma(1/2) increments, times 10^U(-2,0).
    "spread": "gamma" times 10^U(-4,0), so some heads end at b_min and others near L.
    """
    NH, Gp = wl.heads_per_problem, wl.n_grid
    rng = _rng(wl.seed, 7777, seq)
    z = rng.standard_normal((NH, Gp))
    inc = 0.5 * z * z
    inc[:, 0] = 0.0
    x = np.linspace(0.0, 1.0, Gp)[None, :]
    if wl.curve_family == "gamma":
        U = np.cumsum(inc, axis=1)
    elif wl.curve_family == "spread":
        amp = 10.0 ** rng.uniform(-4.0, 0.0, size=(NH, 1))
        U = np.cumsum(inc, axis=1) * amp
    elif wl.curve_family == "mixed":
        fam = rng.integers(0, 3, size=NH)
        tau = rng.uniform(0.02, 0.2, size=(NH, 1))
        pw = rng.uniform(2.0, 6.0, size=(NH, 1))
        x0 = rng.uniform(0.1, 0.9, size=(NH, 1))
        sat = 1.0 - np.exp(-x / tau)
        steep = x ** pw
        logi = 1.0 / (1.0 + np.exp(-(x - x0) / 0.03))
        logi = logi - logi[:, :1]
        base = np.where((fam == 0)[:, None], sat, np.where((fam == 1)[:, None], steep, logi))
        amp = 10.0 ** rng.uniform(-2.0, 0.0, size=(NH, 1))
        U = (base + 0.02 * np.cumsum(inc, axis=1) / Gp) * amp
    else:
        raise KeyError(wl.curve_family)
    U = np.maximum.accumulate(U, axis=1)
    U[:, 0] = 0.0
    return np.ascontiguousarray(U, dtype=np.float32)


def make_bounds(wl: Workload, seq: int = 0):
    """b_min = max(ceil(0.01*L), window + n_sink), b_max = L, for every head of the problem."""
    L = wl.seq_lens[seq]
    lo = max(-((-L) // 100), wl.window + wl.n_sink)
    NH = wl.heads_per_problem
    return (np.full(NH, lo, dtype=np.int32), np.full(NH, L, dtype=np.int32))


def make_allocation_inputs(wl: Workload):
    """Curves, knots, bounds and budgets for every sequence (one allocation problem each):
    curves [n_seqs, NH, Gp] f32, knots [n_seqs, NH, Gp] i32, b_min/b_max [n_seqs, NH] i32,
    B [n_seqs] i64.  NH is ordered (layer, kv head)."""
    NH, Gp = wl.heads_per_problem, wl.n_grid
    curves = np.empty((wl.n_seqs, NH, Gp), dtype=np.float32)
    knots = np.empty((wl.n_seqs, NH, Gp), dtype=np.int32)
    b_min = np.empty((wl.n_seqs, NH), dtype=np.int32)
    b_max = np.empty((wl.n_seqs, NH), dtype=np.int32)
    B = np.empty(wl.n_seqs, dtype=np.int64)
    for s, L in enumerate(wl.seq_lens):
        curves[s] = make_curves(wl, s)
        knots[s] = make_knots(L, Gp)[None, :]
        b_min[s], b_max[s] = make_bounds(wl, s)
        B[s] = wl.budget_total(s)
    return {"curves": curves, "knots": knots, "b_min": b_min, "b_max": b_max, "B": B}
