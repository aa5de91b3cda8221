"""Pins of the oracle's baseline scorers of App. A.2 that are Eq. 1 with another patched prompt:
SnapKV (the block's last w tokens are the prompt, attend causally, and are always kept) and KVzip
(the whole block is the prompt: a long patch, evaluated in chunks).  Exact fractions from a hand-worked
fixture, scalar brute force, agreement with separately written and separately pinned oracle functions,
invariants, and planted mistakes that the fixture must reject."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import softmax

from oracle import epicache_oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "snapkv_window_fractions.txt")


def _fixture():
    fx = {"rows": []}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tag, rest = line.split(None, 1)
        if tag in ("a", "b"):
            fx[tag] = [int(x) for x in rest.split()]
        elif tag == "window":
            fx["w"] = int(rest)
        elif tag == "row":
            left, right = rest.split("|")
            hq, t, x, y = (int(v) for v in left.split())
            fx["rows"].append((hq, t, x, y, [Fraction(v) for v in right.split()]))
        elif tag in ("max", "sum"):
            fx[tag] = [Fraction(v) for v in rest.split()]
        elif tag.startswith("keep_"):
            fx[tag] = [int(v) for v in rest.split()]
    return fx


def _fixture_tensors(fx):
    n, w = len(fx["a"]), fx["w"]
    k = np.array([[math.log(a), math.log(b)] for a, b in zip(fx["a"], fx["b"])]).reshape(1, 1, n, 2)
    q = np.zeros((1, 2, w, 2))
    for hq, t, x, y, _ in fx["rows"]:
        q[0, hq, t] = (x, y)
    return q, k, n, w


def test_fixture_rows_are_what_the_definition_gives():
    """The fractions in the fixture, recomputed with exact integer arithmetic from its a, b and queries."""
    fx = _fixture()
    n, w = len(fx["a"]), fx["w"]
    for hq, t, x, y, want in fx["rows"]:
        e = [Fraction(a) ** x * Fraction(b) ** y for a, b in zip(fx["a"], fx["b"])]
        den = sum(e[:n - w + t + 1])                       # window token t sees rows 0 .. n-w+t
        assert [e[i] / den for i in range(n - w)] == want
    assert fx["max"] == [max(r[4][i] for r in fx["rows"]) for i in range(n - w)]
    assert fx["sum"] == [sum(r[4][i] for r in fx["rows"]) for i in range(n - w)]


@pytest.mark.parametrize("reduce,key", [(orc.REDUCE_MAX, "max"), (orc.REDUCE_SUM, "sum")])
def test_snapkv_scores_match_the_hand_worked_fractions(reduce, key):
    fx = _fixture()
    q, k, n, w = _fixture_tensors(fx)
    got = orc.score_snapkv(q, k, n, reduce, scale=1.0)
    assert got.shape == (1, 1, n - w)
    np.testing.assert_allclose(got[0, 0], [float(f) for f in fx[key]], rtol=1e-13)


def test_snapkv_step_keeps_the_window_and_the_best_earlier_rows():
    fx = _fixture()
    q, k, n, w = _fixture_tensors(fx)
    v = np.arange(n * 3, dtype=np.float64).reshape(1, 1, n, 3)
    for reduce, tag in ((orc.REDUCE_MAX, "keep_max_M3"), (orc.REDUCE_SUM, "keep_sum_M3")):
        s, idx, kk, vv = orc.evict_step_snapkv(q, k, v, n, 3, reduce, scale=1.0)
        assert idx[0, 0].tolist() == fx[tag]
        np.testing.assert_array_equal(kk[0, 0], k[0, 0][fx[tag]])
        np.testing.assert_array_equal(vv[0, 0], v[0, 0][fx[tag]])
    assert orc.evict_step_snapkv(q, k, v, n, 4, orc.REDUCE_MAX, scale=1.0)[1][0, 0].tolist() == fx["keep_max_M4"]
    # the budget equals the window: only the window survives; the budget covers everything: nothing is evicted
    assert orc.evict_step_snapkv(q, k, v, n, w, orc.REDUCE_MAX, scale=1.0)[1][0, 0].tolist() == [n - 2, n - 1]
    assert orc.evict_step_snapkv(q, k, v, n, n, orc.REDUCE_MAX, scale=1.0)[1][0, 0].tolist() == list(range(n))
    with pytest.raises(AssertionError):
        orc.evict_step_snapkv(q, k, v, n, w - 1, orc.REDUCE_MAX, scale=1.0)


def test_snapkv_scalar_brute_force_with_gqa_groups():
    rng = np.random.default_rng(5)
    nb, Hq, Hkv, w, d, n = 2, 6, 2, 3, 5, 9
    G = Hq // Hkv
    q = rng.standard_normal((nb, Hq, w, d))
    k = rng.standard_normal((nb, Hkv, n + 2, d))          # two spare rows that must never be read
    scale = 1.0 / math.sqrt(d)
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        got = orc.score_snapkv(q, k, n, reduce)
        for b in range(nb):
            for h in range(Hkv):
                for i in range(n - w):
                    votes = []
                    for hq in range(h * G, (h + 1) * G):
                        for t in range(w):
                            logit = lambda j: scale * sum(q[b, hq, t, c] * k[b, h, j, c] for c in range(d))
                            den = sum(math.exp(logit(j)) for j in range(n - w + t + 1))
                            votes.append(math.exp(logit(i)) / den)
                    want = max(votes) if reduce == orc.REDUCE_MAX else sum(votes)
                    assert got[b, h, i] == pytest.approx(want, rel=1e-12)


def test_snapkv_is_the_causal_patch_score_with_the_window_as_the_patch():
    """score_causal_patch (written and pinned separately) with n_ctx - w context rows and the window rows as
    the patch's own keys is the same quantity."""
    rng = np.random.default_rng(6)
    q = rng.standard_normal((2, 4, 4, 8))
    k = rng.standard_normal((2, 2, 21, 8))
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        np.testing.assert_allclose(orc.score_snapkv(q, k, 21, reduce), orc.score_causal_patch(q, k, 17, reduce),
                                   rtol=1e-12)


def test_snapkv_window_of_one_is_a_single_softmax_row():
    rng = np.random.default_rng(7)
    q = rng.standard_normal((1, 1, 1, 4))
    k = rng.standard_normal((1, 1, 10, 4))
    row = softmax(0.5 * (k[0, 0] @ q[0, 0, 0]))           # all ten rows, the query's own included
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        np.testing.assert_allclose(orc.score_snapkv(q, k, 10, reduce)[0, 0], row[:9], rtol=1e-12)


def test_snapkv_step_invariants_on_random_inputs():
    rng = np.random.default_rng(8)
    nb, Hq, Hkv, w, d, n, M = 2, 4, 2, 4, 8, 40, 17
    q = rng.standard_normal((nb, Hq, w, d))
    k = rng.standard_normal((nb, Hkv, n, d))
    v = rng.standard_normal((nb, Hkv, n, d))
    s, idx, kk, vv = orc.evict_step_snapkv(q, k, v, n, M, orc.REDUCE_SUM)
    assert idx.shape == (nb, Hkv, M) and (np.diff(idx, axis=2) > 0).all()
    assert (idx[:, :, -w:] == np.arange(n - w, n)).all()                  # the window is always retained
    for b in range(nb):
        for h in range(Hkv):
            early = idx[b, h, :M - w]
            assert early.max() < n - w
            assert early.tolist() == orc.topk_by_counting(list(s[b, h].astype(np.float32)), M - w)
            np.testing.assert_array_equal(kk[b, h], k[b, h][idx[b, h]])
            np.testing.assert_array_equal(vv[b, h], v[b, h][idx[b, h]])
    # rows beyond n_ctx are never read: garbage there changes nothing
    k2 = np.concatenate([k, np.full((nb, Hkv, 3, d), 1e6)], axis=2)
    np.testing.assert_array_equal(orc.score_snapkv(q, k2, n, orc.REDUCE_SUM), s)


# ---- planted mistakes: each is a plausible misreading; the hand-worked fixture must reject it

def _snapkv_mutant(q, k, n, reduce, mode):
    nb, Hq, w, d = q.shape
    G = Hq // k.shape[1]
    n_before = n - w
    votes = []
    for g in range(G):
        for t in range(w):
            if mode == "window_sees_all_window_rows":
                visible = k[0, 0, :n]
            elif mode == "token_does_not_see_itself":
                visible = k[0, 0, :n_before + t]
            elif mode == "window_rows_not_in_the_denominator":
                visible = k[0, 0, :n_before]
            else:
                raise ValueError(mode)
            e = np.exp(visible @ q[0, g, t])
            votes.append(e[:n_before] / e.sum())
    votes = np.array(votes)
    return votes.max(axis=0) if reduce == orc.REDUCE_MAX else votes.sum(axis=0)


@pytest.mark.parametrize("mode", ["window_sees_all_window_rows", "token_does_not_see_itself",
                                  "window_rows_not_in_the_denominator"])
def test_planted_mask_mistakes_are_rejected_by_the_fixture(mode):
    fx = _fixture()
    q, k, n, w = _fixture_tensors(fx)
    for reduce, key in ((orc.REDUCE_MAX, "max"), (orc.REDUCE_SUM, "sum")):
        wrong = _snapkv_mutant(q, k, n, reduce, mode)
        assert not np.allclose(wrong, [float(f) for f in fx[key]], rtol=1e-6), (mode, key)


def test_planted_retention_mistakes_are_rejected_by_the_fixture():
    fx = _fixture()
    q, k, n, w = _fixture_tensors(fx)
    s = orc.score_snapkv(q, k, n, orc.REDUCE_MAX, scale=1.0)[0, 0]
    plain_top3_of_the_scored_rows = sorted(np.argsort(-s)[:3].tolist())          # window not retained
    assert plain_top3_of_the_scored_rows != fx["keep_max_M3"]
    budget_not_reduced_by_the_window = sorted(np.argsort(-s)[:3].tolist() + [n - 2, n - 1])
    assert budget_not_reduced_by_the_window != fx["keep_max_M3"]


# ---- KVzip: a long patch evaluated in chunks

@pytest.mark.parametrize("reduce", [orc.REDUCE_MAX, orc.REDUCE_SUM])
@pytest.mark.parametrize("chunk", [1, 2, 3, 5, 7, 64])
def test_long_patch_in_chunks_equals_the_plain_score(reduce, chunk):
    rng = np.random.default_rng(11)
    q = rng.standard_normal((2, 4, 7, 6))
    k = rng.standard_normal((2, 2, 13, 6))
    np.testing.assert_allclose(orc.score_by_patch_chunks(q, k, 13, chunk, reduce), orc.score(q, k, 13, reduce), rtol=1e-13)


def test_long_patch_chunks_against_the_integer_power_fixture():
    """The four rows of tests/golden/softmax_integer_powers.txt as one query head with a patch of four tokens,
    scored two tokens at a time: the reductions printed in that fixture must come out."""
    path = os.path.join(os.path.dirname(GOLDEN), "softmax_integer_powers.txt")
    a = b = None
    rows, want = [], {}
    for line in open(path):
        tag, _, rest = line.strip().partition(" ")
        if tag == "a":
            a = [int(x) for x in rest.split()]
        elif tag == "b":
            b = [int(x) for x in rest.split()]
        elif tag == "row":
            rows.append([int(x) for x in rest.split("|")[0].split()])
        elif tag in ("max", "sum"):
            want[tag] = [float(Fraction(x)) for x in rest.split()]
    k = np.array([[math.log(x), math.log(y)] for x, y in zip(a, b)]).reshape(1, 1, 4, 2)
    q = np.array(rows, dtype=np.float64).reshape(1, 1, 4, 2)
    np.testing.assert_allclose(orc.score_by_patch_chunks(q, k, 4, 2, orc.REDUCE_MAX, scale=1.0)[0, 0], want["max"], rtol=1e-13)
    np.testing.assert_allclose(orc.score_by_patch_chunks(q, k, 4, 3, orc.REDUCE_SUM, scale=1.0)[0, 0], want["sum"], rtol=1e-13)
    # planted mistake: chunks of a max-reduction added up instead of maximised
    added = orc.score(q[:, :, :2], k, 4, orc.REDUCE_MAX, 1.0) + orc.score(q[:, :, 2:], k, 4, orc.REDUCE_MAX, 1.0)
    assert not np.allclose(added[0, 0], want["max"], rtol=1e-6)
