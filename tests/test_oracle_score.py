"""Pins for the oracle's score step (Eq. 1 + SnapKV window / pooling), CPU only.

Each test checks the oracle against something other than itself: hand-worked
rationals (tests/golden), closed forms, a brute-force loop written from the
definition, and torch's CPU softmax / max_pool1d as a second opinion.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import lukv_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "softmax_pool_handworked.txt")


def _golden():
    out = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if not line:
            continue
        key, val = [t.strip() for t in line.split("=")]
        out[key] = [float("inf") if t == "inf" else float(Fraction(t)) for t in val.split()]
    return out


def _handworked_inputs():
    g = _golden()
    a = np.array(g["a"])
    q = np.ones((1, 2, 1))
    k = np.log(a)[None, :, None]
    return g, q, k


def test_handworked_unpooled_is_causal():
    g, q, k = _handworked_inputs()
    r = O.window_attention_sum(q, k, 1, scale=1.0)
    assert np.allclose(r[0, :4], g["unpooled"], rtol=0, atol=1e-14)
    assert not np.allclose(r[0, :4], g["noncausal"], atol=1e-3)


@pytest.mark.parametrize("p,key", [(3, "pool3"), (7, "pool7")])
def test_handworked_pooled(p, key):
    g, q, k = _handworked_inputs()
    s = O.score(q, k, 1, window=2, pool_kernel=p, n_sink=0, scale=1.0)
    want = np.array(g[key])
    assert s.dtype == np.float32
    assert np.array_equal(np.isinf(s[0]), np.isinf(want))
    fin = np.isfinite(want)
    assert np.array_equal(s[0][fin], want[fin].astype(np.float32))


def test_handworked_pool_stays_inside_prefix():
    g = _golden()
    k = np.log(np.array(g["a2"]))[None, :, None]
    s = O.score(np.ones((1, 2, 1)), k, 1, window=2, pool_kernel=3, n_sink=0, scale=1.0)
    want = np.array(g["pool3_a2"])
    assert np.array_equal(np.isinf(s[0]), np.isinf(want))
    assert np.array_equal(s[0][:4], want[:4].astype(np.float32))


def test_handworked_lse_variant():
    g, q, k = _handworked_inputs()
    lse = np.log(np.array(g["row_sums"]))[None, :]
    assert np.allclose(O.window_lse(q, k, 1, scale=1.0), lse, rtol=1e-15)
    r = O.window_attention_sum(q, k, 1, scale=1.0, lse=lse)
    assert np.allclose(r[0, :4], g["unpooled"], rtol=0, atol=1e-14)
    # a normaliser that is too large by ln 2 halves every probability
    r2 = O.window_attention_sum(q, k, 1, scale=1.0, lse=lse + math.log(2.0))
    assert np.allclose(r2[0, :4], np.array(g["unpooled"]) / 2, rtol=1e-14)


def test_lse_variant_equals_recomputed_normaliser():
    L, w, d, Hq, Hkv = 77, 6, 8, 6, 3
    rng = np.random.default_rng(11)
    q = rng.standard_normal((Hq, w, d)) * 2
    k = rng.standard_normal((Hkv, L, d))
    lse = O.window_lse(q, k, Hkv)
    # brute-force definition of the log-sum-exp
    for qh in (0, 5):
        for i in (0, w - 1):
            t = L - w + i
            want = math.log(sum(math.exp(sum(q[qh, i, x] * k[qh // 2, j, x] for x in range(d)) / math.sqrt(d))
                                for j in range(t + 1)))
            assert lse[qh, i] == pytest.approx(want, rel=1e-13)
    a = O.score(q, k, Hkv, w, 5, 2)
    b = O.score(q, k, Hkv, w, 5, 2, lse=lse)
    fin = np.isfinite(a)
    assert np.array_equal(fin, np.isfinite(b))
    assert np.allclose(a[fin], b[fin], rtol=1e-6)


def test_handworked_topk_lowest_index_ties():
    g, q, k = _handworked_inputs()
    s = O.score(q, k, 1, window=2, pool_kernel=3, n_sink=0, scale=1.0)
    for kk in (3, 4, 5):
        assert O.select(s[0], kk).tolist() == [int(x) for x in g["top%d" % kk]]


def test_identical_keys_closed_form_and_group_mean():
    # all keys equal => every visible key gets 1/(t+1); R[j] = sum_i 1/(L-w+i+1) for any G
    L, w, d, Hq, Hkv = 40, 5, 8, 6, 2
    rng = np.random.default_rng(3)
    q = rng.standard_normal((Hq, w, d))
    k = np.tile(rng.standard_normal((1, 1, d)), (Hkv, L, 1))
    r = O.window_attention_sum(q, k, Hkv)
    want = sum(Fraction(1, L - w + i + 1) for i in range(w))
    assert np.allclose(r[:, :L - w], float(want), rtol=1e-13)
    assert float(Fraction(11, 30)) == pytest.approx(
        O.window_attention_sum(np.ones((1, 2, 1)), np.ones((1, 6, 1)), 1)[0, 0], rel=1e-14)


def test_total_mass_is_window_size():
    # every softmax row sums to 1 => the unpooled metric over all L columns sums to w
    L, w, d, Hq, Hkv = 97, 8, 16, 8, 4
    rng = np.random.default_rng(4)
    q = rng.standard_normal((Hq, w, d)) * 3
    k = rng.standard_normal((Hkv, L, d))
    r = O.window_attention_sum(q, k, Hkv)
    assert np.allclose(r.sum(axis=1), w, rtol=1e-12)


def test_brute_force_definition():
    """Loop-by-loop restatement of Eq. 1 with math.exp, causal range, GQA mean, clipped pool."""
    L, w, d, Hq, Hkv, p, n_sink = 23, 4, 3, 4, 2, 5, 2
    G = Hq // Hkv
    rng = np.random.default_rng(5)
    q = rng.standard_normal((Hq, w, d)) * 2
    k = rng.standard_normal((Hkv, L, d))
    got = O.score(q, k, Hkv, w, p, n_sink)
    P = L - w
    for c in range(Hkv):
        R = [0.0] * L
        for g in range(G):
            for i in range(w):
                t = L - w + i
                logit = [sum(q[c * G + g, i, x] * k[c, j, x] for x in range(d)) / math.sqrt(d)
                         for j in range(t + 1)]
                mx = max(logit)
                den = sum(math.exp(v - mx) for v in logit)
                for j in range(t + 1):
                    R[j] += math.exp(logit[j] - mx) / den / G
        for j in range(L):
            if j >= P or j < n_sink:
                assert got[c, j] == np.inf
            else:
                want = max(R[max(0, j - p // 2): min(P - 1, j + p // 2) + 1])
                assert got[c, j] == pytest.approx(want, rel=1e-6)


def test_pool_properties_and_library_cross_check():
    rng = np.random.default_rng(6)
    r = rng.random((3, 50))
    assert np.array_equal(O.max_pool_1d(r, 1), r)
    for p in (3, 7, 9):
        got = O.max_pool_1d(r, p)
        assert np.all(got >= r)
        ref = torch.nn.functional.max_pool1d(torch.from_numpy(r)[None], p, stride=1, padding=p // 2)[0]
        assert np.array_equal(got, ref.numpy())


def test_softmax_library_cross_check():
    L, w, d = 64, 6, 8
    rng = np.random.default_rng(7)
    q = rng.standard_normal((2, w, d))
    k = rng.standard_normal((1, L, d))
    r = O.window_attention_sum(q, k, 1)
    qt, kt = torch.from_numpy(q), torch.from_numpy(k[0])
    s = torch.einsum("gid,jd->gij", qt, kt) / math.sqrt(d)
    mask = torch.arange(L)[None, :] > (L - w + torch.arange(w))[:, None]
    s = s.masked_fill(mask[None], float("-inf"))
    ref = torch.softmax(s, dim=-1).sum(dim=1).mean(dim=0)
    assert np.allclose(r[0], ref.numpy(), rtol=1e-12, atol=1e-15)


def test_bf16_decode_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x8000, 0x3DCD], dtype=np.uint16)
    want = [1.0, -1.0, 3.140625, 0.0, -0.0, 0.10009765625]
    assert O.decode(bits).tolist() == want


def test_window_not_longer_than_context():
    with pytest.raises(ValueError):
        O.score(np.ones((1, 4, 2)), np.ones((1, 4, 2)), 1, 4, 3, 0)


# --- decode-step attention over retained entries (Eq. 3) -------------------------------------

def test_decode_attention_handworked_and_special_cases():
    # two retained entries, logits ln 1 and ln 3 (scale 1): weights 1/4 and 3/4
    q = np.array([[1.0, 0.0]])
    k = np.array([[0.0, 5.0], [math.log(3.0), -2.0]])
    v = np.array([[4.0, 0.0], [0.0, 8.0]])
    assert np.allclose(O.decode_attention(q, k, v, scale=1.0), [[1.0, 6.0]], rtol=1e-15)
    # a single retained entry returns its value row; equal keys average the values
    assert np.array_equal(O.decode_attention(q, k[:1], v[:1], scale=1.0), v[:1])
    same = np.tile(k[:1], (5, 1))
    vals = np.arange(10.0).reshape(5, 2)
    assert np.allclose(O.decode_attention(q, same, vals), vals.mean(axis=0)[None], rtol=1e-15)
    assert np.array_equal(O.decode_attention(q, k[:0], v[:0]), np.zeros((1, 2)))


def test_decode_attention_library_cross_check():
    rng = np.random.default_rng(21)
    G, n, d = 4, 37, 16
    q, k, v = rng.standard_normal((G, d)), rng.standard_normal((n, d)), rng.standard_normal((n, d))
    got = O.decode_attention(q, k, v)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[None], torch.from_numpy(k)[None],
                                                           torch.from_numpy(v)[None])[0].numpy()
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-14)
    # every output row is a convex combination of the value rows
    assert np.all(got <= v.max(axis=0) + 1e-12) and np.all(got >= v.min(axis=0) - 1e-12)
