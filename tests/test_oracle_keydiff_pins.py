"""Pins of the oracle's KeyDiff score (App. A.2): hand-worked values, scalar brute force,
invariances, degenerate cases and planted mistakes."""
import math

import numpy as np
import pytest

from oracle import epicache_oracle as orc


def _k(rows):
    return np.array(rows, dtype=np.float64)[None, None]


def test_hand_worked_3_4_5():
    # keys (3,0) and (0,4): anchor (1.5, 2), |anchor| = 2.5 -> cosines 0.6 and 0.8
    np.testing.assert_allclose(orc.score_keydiff(_k([[3, 0], [0, 4]]), 2)[0, 0], [-0.6, -0.8], rtol=1e-15)
    # three keys (1,0), (1,0), (-1,0): anchor (1/3, 0): the odd one out scores +1 and is kept first
    s = orc.score_keydiff(_k([[1, 0], [1, 0], [-1, 0]]), 3)[0, 0]
    np.testing.assert_allclose(s, [-1, -1, 1], rtol=1e-15)
    assert orc.topk_1d(s, 1).tolist() == [2]
    # identical keys: every cosine is 1
    np.testing.assert_allclose(orc.score_keydiff(_k([[2, -1, 5]] * 4), 4)[0, 0], [-1] * 4, rtol=1e-15)


def test_scalar_brute_force_and_prefix_only():
    rng = np.random.default_rng(0)
    k = rng.standard_normal((2, 3, 9, 5))
    n = 6
    got = orc.score_keydiff(k, n)
    assert got.shape == (2, 3, n)
    for b in range(2):
        for h in range(3):
            anchor = [sum(k[b, h, j, c] for j in range(n)) / n for c in range(5)]
            na = math.sqrt(sum(a * a for a in anchor))
            for i in range(n):
                dot = sum(k[b, h, i, c] * anchor[c] for c in range(5))
                ni = math.sqrt(sum(k[b, h, i, c] ** 2 for c in range(5)))
                assert abs(got[b, h, i] + dot / (ni * na)) < 1e-13
    k2 = k.copy()
    k2[:, :, n:] = 1e9                       # rows beyond n_ctx are not part of the anchor
    np.testing.assert_array_equal(orc.score_keydiff(k2, n), got)


def test_invariances_and_bounds():
    rng = np.random.default_rng(1)
    k = rng.standard_normal((1, 2, 12, 6))
    s = orc.score_keydiff(k, 12)
    assert (np.abs(s) <= 1 + 1e-15).all()
    np.testing.assert_allclose(orc.score_keydiff(3.7 * k, 12), s, rtol=1e-13)          # global scale
    perm = rng.permutation(12)
    np.testing.assert_allclose(orc.score_keydiff(k[:, :, perm], 12), s[:, :, perm], rtol=1e-13)
    rot, _ = np.linalg.qr(rng.standard_normal((6, 6)))                                  # rotations
    np.testing.assert_allclose(orc.score_keydiff(k @ rot, 12), s, rtol=1e-12)
    # mean of the cosines weighted by the key norms is |anchor| * n / sum of norms (from the definition)
    keys = k[0, 0]
    anchor = keys.mean(axis=0)
    lhs = (-(s[0, 0]) * np.linalg.norm(keys, axis=1)).sum()
    assert abs(lhs - 12 * np.linalg.norm(anchor)) < 1e-12


def test_degenerate_and_ragged():
    s = orc.score_keydiff(_k([[0, 0], [1, 1], [1, -1]]), 3)[0, 0]     # a zero key has cosine 0
    np.testing.assert_allclose(s, [0, -1 / math.sqrt(2), -1 / math.sqrt(2)], rtol=1e-15)
    s = orc.score_keydiff(_k([[1, 2], [-1, -2]]), 2)[0, 0]            # zero anchor
    assert s.tolist() == [0, 0]
    k = np.random.default_rng(2).standard_normal((2, 2, 8, 4))
    lens = [[8, 3], [0, 1]]
    s = orc.score_keydiff(k, lens)
    assert np.isnan(s[1, 0]).all() and np.isnan(s[0, 1, 3:]).all()
    np.testing.assert_array_equal(s[0, 1, :3], orc.score_keydiff(k[:1, 1:2], 3)[0, 0])
    assert s[1, 1, 0] == -1.0                                          # a single key is its own anchor


def _variant(keys, mistake):
    n = len(keys)
    if mistake == "anchor_of_unit_keys":
        anchor = (keys / np.linalg.norm(keys, axis=1, keepdims=True)).mean(axis=0)
    elif mistake == "anchor_excludes_self":
        return np.array([-(keys[i] @ (keys.sum(0) - keys[i])) /
                         (np.linalg.norm(keys[i]) * np.linalg.norm(keys.sum(0) - keys[i])) for i in range(n)])
    else:
        anchor = keys.mean(axis=0)
    cos = keys @ anchor / (np.linalg.norm(keys, axis=1) * np.linalg.norm(anchor))
    if mistake == "dot_not_cosine":
        cos = keys @ anchor
    return cos if mistake == "similarity_not_dissimilarity" else -cos


@pytest.mark.parametrize("mistake", [None, "anchor_of_unit_keys", "anchor_excludes_self", "dot_not_cosine",
                                     "similarity_not_dissimilarity"])
def test_planted_mistakes_fail_the_hand_worked_case(mistake):
    got = _variant(np.array([[3.0, 0.0], [0.0, 4.0]]), mistake)
    assert np.allclose(got, [-0.6, -0.8], rtol=1e-12) == (mistake is None)
