"""Pins of the oracle's patch attention output: exact rational closed forms, scalar brute force,
agreement with the already pinned scoring functions through the normaliser, invariants and planted
mistakes."""
import math
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import epicache_oracle as orc


def _fixture():
    # keys (ln a, ln b), integer queries, scale 1: every exp is an integer a^m b^n
    ctx = [(2, 3), (5, 1), (1, 7)]
    patch = [(3, 2), (4, 4)]
    queries = [(1, 2), (2, 1)]
    vals = [[1, 0, 2], [0, 3, -1], [4, 1, 0], [2, 2, 2], [-3, 0, 5]]      # integer values, d_v = 3 ... see below
    return ctx, patch, queries, vals


def test_exact_rational_outputs():
    ctx, patch, queries, vals = _fixture()
    keys = ctx + patch
    # the oracle uses one head_dim for q, k and v: embed the 2-d keys/queries and the 3-d values in d = 3
    k = np.zeros((1, 1, 5, 3))
    k[0, 0, :, :2] = [[math.log(a), math.log(b)] for a, b in keys]
    q = np.zeros((1, 1, 2, 3))
    q[0, 0, :, :2] = queries
    v = np.array(vals, dtype=np.float64).reshape(1, 1, 5, 3)
    w = lambda key, qu: Fraction(key[0]) ** qu[0] * Fraction(key[1]) ** qu[1]
    for causal in (True, False):
        out, lse = orc.patch_attention(q, k, v, 3, causal, scale=1.0)
        for t, qu in enumerate(queries):
            visible = keys[:3 + (t + 1 if causal else 0)]
            den = sum(w(key, qu) for key in visible)
            want = [sum(w(key, qu) * vals[i][c] for i, key in enumerate(visible)) / den for c in range(3)]
            np.testing.assert_allclose(out[0, 0, t], [float(x) for x in want], rtol=1e-13, atol=1e-15)
            assert abs(lse[0, 0, t] - math.log(den)) < 1e-13
    # hand check: query (1,2), causal: weights 18, 5, 49, 12 over 84 -> O[0] = (18*1 + 5*0 + 49*4 + 12*2)/84
    out, _ = orc.patch_attention(q, k, v, 3, True, scale=1.0)
    assert abs(out[0, 0, 0, 0] - (18 + 196 + 24) / 84) < 1e-13


def test_scalar_brute_force_and_library_softmax():
    rng = np.random.default_rng(0)
    nb, Hq, Hkv, p, d, N = 2, 4, 2, 3, 5, 6
    q = rng.standard_normal((nb, Hq, p, d))
    k = rng.standard_normal((nb, Hkv, N + p + 1, d))
    v = rng.standard_normal((nb, Hkv, N + p + 1, d))
    scale = 1 / math.sqrt(d)
    for causal in (True, False):
        out, lse = orc.patch_attention(q, k, v, N, causal)
        for b in range(nb):
            for hq in range(Hq):
                h = hq // 2                                   # query head hq reads KV head hq // G
                for t in range(p):
                    n = N + (t + 1 if causal else 0)
                    logits = [scale * sum(q[b, hq, t, c] * k[b, h, i, c] for c in range(d)) for i in range(n)]
                    den = sum(math.exp(z) for z in logits)
                    for c in range(d):
                        want = sum(math.exp(logits[i]) / den * v[b, h, i, c] for i in range(n))
                        assert abs(out[b, hq, t, c] - want) < 1e-12
                    w = softmax(np.array(logits))
                    np.testing.assert_allclose(out[b, hq, t], w @ v[b, h, :n], rtol=1e-12, atol=1e-14)
                    assert abs(lse[b, hq, t] - logsumexp(logits)) < 1e-12


def test_normalisers_tie_the_output_pass_to_the_scoring():
    """The lse returned here is exactly what score_given_lse needs to reproduce score_causal_patch / score."""
    rng = np.random.default_rng(1)
    q = rng.standard_normal((2, 4, 3, 6))
    k = rng.standard_normal((2, 2, 12, 6))
    v = rng.standard_normal((2, 2, 12, 6))
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        _, lse = orc.patch_attention(q, k, v, 8, True)
        np.testing.assert_allclose(orc.score_given_lse(q, k, 8, lse, reduce), orc.score_causal_patch(q, k, 8, reduce),
                                   rtol=1e-12)
        _, lse = orc.patch_attention(q, k, v, 8, False)
        np.testing.assert_allclose(orc.score_given_lse(q, k, 8, lse, reduce), orc.score(q, k, 8, reduce), rtol=1e-12)


def test_invariants():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 2, 4, 5))
    k = rng.standard_normal((1, 1, 13, 5))
    v = rng.standard_normal((1, 1, 13, 5))
    out, lse = orc.patch_attention(q, k, v, 7, True)
    # convex combination: inside the bounding box of the visible value rows
    for t in range(4):
        vis = v[0, 0, :7 + t + 1]
        assert (out[0, :, t] <= vis.max(axis=0) + 1e-12).all() and (out[0, :, t] >= vis.min(axis=0) - 1e-12).all()
    # equal value rows come straight through; a constant shift of all values shifts the output
    vc = np.tile(v[0, 0, :1], (13, 1))[None, None]
    np.testing.assert_allclose(orc.patch_attention(q, k, vc, 7, True)[0], np.broadcast_to(v[0, 0, 0], (1, 2, 4, 5)), rtol=1e-12)
    np.testing.assert_allclose(orc.patch_attention(q, k, v + 3.0, 7, True)[0], out + 3.0, rtol=1e-12)
    # causal: patch value j only reaches tokens t >= j; rows past the patch reach nobody
    for j in range(4):
        v2 = v.copy()
        v2[0, 0, 7 + j] += 1.0
        moved = np.abs(orc.patch_attention(q, k, v2, 7, True)[0] - out).max(axis=(0, 1, 3)) > 0
        assert moved.tolist() == [t >= j for t in range(4)]
    v3, k3 = v.copy(), k.copy()
    v3[0, 0, 11:], k3[0, 0, 11:] = np.nan, np.nan
    assert np.isfinite(orc.patch_attention(q, k3, v3, 7, True)[0]).all()
    # a dominant key hands over its value row
    k4 = k.copy()
    k4[0, 0, 2] = 50 * q[0, 0, 1] / np.linalg.norm(q[0, 0, 1])
    o4, _ = orc.patch_attention(q, k4, v, 7, True, scale=1.0)
    np.testing.assert_allclose(o4[0, 0, 1], v[0, 0, 2], atol=1e-8)


@pytest.mark.parametrize("mistake", [None, "values_of_head_zero", "weights_not_normalised", "patch_fully_visible",
                                     "transposed_weights"])
def test_planted_mistakes_fail_the_closed_form(mistake):
    ctx, patch, queries, vals = _fixture()
    keys = np.array([[math.log(a), math.log(b)] for a, b in ctx + patch])
    qs = np.array(queries, dtype=np.float64)
    V = np.array(vals, dtype=np.float64)
    got = []
    for t in range(2):
        n = 5 if mistake == "patch_fully_visible" else 3 + t + 1
        e = np.exp(keys[:n] @ qs[t])
        w = e if mistake == "weights_not_normalised" else e / e.sum()
        if mistake == "transposed_weights":
            w = np.exp(keys[:n] @ qs[1 - t])
            w = w / w.sum()
        vv = np.tile(V[0], (n, 1)) if mistake == "values_of_head_zero" else V[:n]
        got.append(w @ vv)
    want0 = np.array([(18 + 196 + 24) / 84, (15 + 49 + 24) / 84, (36 - 5 + 24) / 84])
    ok = np.allclose(got[0], want0, rtol=1e-12)
    den1 = 4 * 3 + 25 * 1 + 1 * 7 + 9 * 2 + 16 * 4       # query (2,1): a^2 b over ctx + both patch keys
    want1 = np.array([(12 * 1 + 7 * 4 + 18 * 2 - 64 * 3) / den1, (25 * 3 + 7 * 1 + 18 * 2) / den1,
                      (12 * 2 - 25 + 18 * 2 + 64 * 5) / den1])
    ok = ok and np.allclose(got[1], want1, rtol=1e-12)
    assert ok == (mistake is None)


def test_per_head_context_lengths():
    """Heads with their own context length (App. A.2, head-wise non-uniform retention): each head attends to its
    own rows 0 .. n-1 and to the patch rows right behind them.  Pinned by a scalar brute force, by the weights
    read out through identity value rows, and by NaN in every row a head must not touch."""
    rng = np.random.default_rng(11)
    nb, Hq, Hkv, p, d, C = 2, 4, 2, 3, 4, 12
    q = rng.standard_normal((nb, Hq, p, d))
    k = rng.standard_normal((nb, Hkv, C, d))
    v = rng.standard_normal((nb, Hkv, C, d))
    n = np.array([[5, 0], [9, 2]])
    for causal in (True, False):
        kk, vv = k.copy(), v.copy()
        for b in range(nb):
            for h in range(Hkv):
                kk[b, h, n[b, h] + (p if causal else 0):] = np.nan
                vv[b, h, n[b, h] + (p if causal else 0):] = np.nan
        out, lse = orc.patch_attention(q, kk, vv, n, causal, scale=0.7)
        for b in range(nb):
            for hq in range(Hq):
                h = hq // 2
                for t in range(p):
                    vis = list(range(n[b, h])) + ([n[b, h] + j for j in range(t + 1)] if causal else [])
                    if not vis:
                        assert (out[b, hq, t] == 0).all() and lse[b, hq, t] == -np.inf
                        continue
                    zs = [0.7 * sum(q[b, hq, t, c] * k[b, h, i, c] for c in range(d)) for i in vis]
                    den = sum(math.exp(z) for z in zs)
                    want = [sum(math.exp(z) / den * v[b, h, i, c] for z, i in zip(zs, vis)) for c in range(d)]
                    np.testing.assert_allclose(out[b, hq, t], want, rtol=1e-12, atol=1e-14)
                    assert abs(lse[b, hq, t] - math.log(den)) < 1e-12
    # a scalar length and an array filled with it are the same thing
    a = orc.patch_attention(q, k, v, 6, True)
    b_ = orc.patch_attention(q, k, v, np.full((nb, Hkv), 6), True)
    assert (a[0] == b_[0]).all() and (a[1] == b_[1]).all()
    # identity value rows read the weights out: they sum to one over the head's own visible rows only
    eye = np.zeros((nb, Hkv, C, C)); eye[:, :, np.arange(C), np.arange(C)] = 1.0
    w, _ = orc.patch_attention(q, k, eye, n, True, scale=0.7)
    for b in range(nb):
        for hq in range(Hq):
            for t in range(p):
                nv = n[b, hq // 2] + t + 1
                assert abs(w[b, hq, t, :nv].sum() - 1.0) < 1e-12 and (w[b, hq, t, nv:] == 0).all()
