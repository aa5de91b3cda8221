"""Pins of the oracle's scoring with the patch's own causal keys in the denominator: exact
rational closed forms, a scalar brute force, limits that reduce to the pinned plain score, the
causal structure itself, and planted mistakes."""
import math
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import logsumexp

from oracle import epicache_oracle as orc


def _case(rng, nb=2, Hq=4, Hkv=2, p=3, d=6, N=7):
    q = rng.standard_normal((nb, Hq, p, d))
    k = rng.standard_normal((nb, Hkv, N + p + 2, d))
    return q, k, N


def test_exact_rational_weights():
    """Keys (ln a, ln b) and integer queries (m, n) with scale 1 make every exp an integer a^m b^n, so the
    weights are exact fractions.  d = 2, one head, p = 2 patch tokens, N = 3 context keys."""
    ctx = [(2, 3), (5, 1), (1, 7)]
    patch = [(3, 2), (4, 4)]
    queries = [(1, 2), (2, 1)]                      # patch token 0, patch token 1
    k = np.array([[math.log(a), math.log(b)] for a, b in ctx + patch]).reshape(1, 1, 5, 2)
    q = np.array(queries, dtype=np.float64).reshape(1, 1, 2, 2)
    w = lambda key, qu: Fraction(key[0]) ** qu[0] * Fraction(key[1]) ** qu[1]
    rows = []
    for t, qu in enumerate(queries):
        den = sum(w(c, qu) for c in ctx) + sum(w(pk, qu) for pk in patch[:t + 1])   # token t sees patch 0..t
        rows.append([w(c, qu) / den for c in ctx])
    # hand check of one entry: query (1,2): ctx 2*9=18, 5*1=5, 1*49=49; patch0 3*4=12 -> 18/84
    assert rows[0][0] == Fraction(18, 84)
    want_max = [float(max(rows[0][i], rows[1][i])) for i in range(3)]
    want_sum = [float(rows[0][i] + rows[1][i]) for i in range(3)]
    got_max = orc.score_causal_patch(q, k, 3, orc.REDUCE_MAX, scale=1.0)[0, 0]
    got_sum = orc.score_causal_patch(q, k, 3, orc.REDUCE_SUM, scale=1.0)[0, 0]
    np.testing.assert_allclose(got_max, want_max, rtol=1e-13)
    np.testing.assert_allclose(got_sum, want_sum, rtol=1e-13)


def test_scalar_brute_force_with_gqa_groups():
    rng = np.random.default_rng(1)
    q, k, N = _case(rng)
    nb, Hq, p, d = q.shape
    Hkv, G = k.shape[1], 2
    scale = 1.0 / math.sqrt(d)
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        got = orc.score_causal_patch(q, k, N, reduce)
        for b in range(nb):
            for h in range(Hkv):
                for i in range(N):
                    vals = []
                    for hq in range(h * G, (h + 1) * G):       # query head hq votes for KV head hq // G
                        for t in range(p):
                            logit = lambda j: scale * sum(q[b, hq, t, c] * k[b, h, j, c] for c in range(d))
                            den = sum(math.exp(logit(j)) for j in range(N))
                            den += sum(math.exp(logit(N + j)) for j in range(t + 1))
                            vals.append(math.exp(logit(i)) / den)
                    want = max(vals) if reduce == orc.REDUCE_MAX else sum(vals)
                    assert abs(got[b, h, i] - want) <= 1e-12 * want


def test_agrees_with_supplied_normaliser_scoring_and_with_plain_score_in_the_limit():
    rng = np.random.default_rng(2)
    q, k, N = _case(rng)
    nb, Hq, p, d = q.shape
    G, scale = 2, 1.0 / math.sqrt(d)
    lse = np.empty((nb, Hq, p))
    for b in range(nb):
        for hq in range(Hq):
            for t in range(p):
                keys = np.concatenate([k[b, hq // G, :N], k[b, hq // G, N:N + t + 1]])
                lse[b, hq, t] = logsumexp(scale * keys @ q[b, hq, t])
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        np.testing.assert_allclose(orc.score_causal_patch(q, k, N, reduce),
                                   orc.score_given_lse(q, k, N, lse, reduce), rtol=1e-12)
    # patch keys that every query finds hopeless drop out of the denominator: the plain score returns
    far = k.copy()
    qpos = np.abs(q)                                                 # all-positive queries ...
    far[:, :, N:N + p] = -50.0                                       # ... against all-negative patch keys
    np.testing.assert_allclose(orc.score_causal_patch(qpos, far, N, orc.REDUCE_SUM),
                               orc.score(qpos, far, N, orc.REDUCE_SUM), rtol=1e-12)


def test_causal_structure_and_mass():
    rng = np.random.default_rng(3)
    q, k, N = _case(rng, nb=1, Hq=2, Hkv=1, p=4)
    p, d = 4, q.shape[3]
    rows = q[0].reshape(2 * p, d)
    scale = 0.5
    base = orc.attention_weights_causal_patch(rows, k[0, 0, :N], k[0, 0, N:N + p], scale, p)
    plain = orc.attention_weights(rows, k[0, 0, :N], scale)
    assert (base < plain).all()                          # a larger denominator lowers every weight
    assert (base.sum(axis=1) < 1).all()                  # the rest of the mass sits on the patch keys
    for j in range(p):                                   # patch key j is visible to tokens t >= j only
        kp = k[0, 0, N:N + p].copy()
        kp[j] += 1.0
        moved = orc.attention_weights_causal_patch(rows, k[0, 0, :N], kp, scale, p)
        changed = np.abs(moved - base).max(axis=1) > 0
        assert changed.tolist() == [(r % p) >= j for r in range(2 * p)]
    # a patch token whose own key dominates keeps almost nothing for the context
    kp = k[0, 0, N:N + p].copy()
    kp[0] = 100.0 * rows[0] / np.linalg.norm(rows[0])
    w0 = orc.attention_weights_causal_patch(rows, k[0, 0, :N], kp, scale, p)[0]
    assert w0.sum() < 1e-6
    # rows beyond n_ctx + p are never read
    k2 = k.copy()
    k2[:, :, N + p:] = np.nan
    assert np.isfinite(orc.score_causal_patch(q, k2, N)).all()


def _variant(q, k, N, reduce, scale, mistake):
    nb, Hq, p, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    out = np.empty((nb, Hkv, N))
    for b in range(nb):
        for h in range(Hkv):
            rows = q[b, h * G:(h + 1) * G].reshape(G * p, d)
            w = np.empty((G * p, N))
            for r in range(G * p):
                t = r % p
                if mistake == "row_index_not_token_index":
                    t = r
                visible = t + 1
                if mistake == "strictly_before":
                    visible = t
                if mistake == "whole_patch_visible":
                    visible = p
                keys = np.concatenate([k[b, h, :N], k[b, h, N:N + min(visible, p)]])
                if mistake == "patch_from_row_zero":
                    keys = np.concatenate([k[b, h, :N], k[b, h, :min(visible, p)]])
                z = scale * keys @ rows[r]
                e = np.exp(z - z.max())
                w[r] = e[:N] / e.sum()
            out[b, h] = w.max(axis=0) if reduce == orc.REDUCE_MAX else w.sum(axis=0)
    return out


@pytest.mark.parametrize("mistake", [None, "row_index_not_token_index", "strictly_before",
                                     "whole_patch_visible", "patch_from_row_zero"])
def test_planted_mistakes_are_caught_by_the_closed_form(mistake):
    # the exact-fraction case above, extended to two query heads sharing the KV head (G = 2)
    ctx = [(2, 3), (5, 1), (1, 7)]
    patch = [(3, 2), (4, 4)]
    queries = [[(1, 2), (2, 1)], [(0, 1), (3, 0)]]     # [query head][patch token]
    k = np.array([[math.log(a), math.log(b)] for a, b in ctx + patch]).reshape(1, 1, 5, 2)
    q = np.array(queries, dtype=np.float64).reshape(1, 2, 2, 2)
    w = lambda key, qu: Fraction(key[0]) ** qu[0] * Fraction(key[1]) ** qu[1]
    rows = []
    for g in range(2):
        for t in range(2):
            qu = queries[g][t]
            den = sum(w(c, qu) for c in ctx) + sum(w(pk, qu) for pk in patch[:t + 1])
            rows.append([w(c, qu) / den for c in ctx])
    want = np.array([float(sum(r[i] for r in rows)) for i in range(3)])
    got = _variant(q, k, 3, orc.REDUCE_SUM, 1.0, mistake)[0, 0]
    ok = np.allclose(got, want, rtol=1e-12)
    assert ok == (mistake is None)
    if mistake is None:
        np.testing.assert_allclose(orc.score_causal_patch(q, k, 3, orc.REDUCE_SUM, scale=1.0)[0, 0], want, rtol=1e-13)
