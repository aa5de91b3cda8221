"""Pins of the CPU oracle against things other than itself (no GPU).

The paper prints no numeric example for the eviction step, so the pins are
closed forms (tests/golden/), textbook special cases computed by library
routines the oracle does not call, algebraic invariants, and brute force.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import epicache_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _load_integer_powers():
    a = b = None
    rows, red = [], {}
    for line in open(os.path.join(GOLDEN, "softmax_integer_powers.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tag, rest = line.split(None, 1)
        if tag == "a":
            a = [int(t) for t in rest.split()]
        elif tag == "b":
            b = [int(t) for t in rest.split()]
        elif tag == "row":
            xy, fr = rest.split("|")
            rows.append(([int(t) for t in xy.split()], [Fraction(t) for t in fr.split()]))
        else:
            red[tag] = [Fraction(t) for t in rest.split()]
    return a, b, rows, red


# ---------------------------------------------------------------- score pins

def test_attention_weights_closed_form_rows():
    a, b, rows, _ = _load_integer_powers()
    keys = np.array([[math.log(x), math.log(y)] for x, y in zip(a, b)])
    for (x, y), expect in rows:
        got = orc.attention_weights(np.array([[float(x), float(y)]]), keys, 1.0)[0]
        np.testing.assert_allclose(got, [float(f) for f in expect], rtol=1e-13)


@pytest.mark.parametrize("reduce,tag", [(orc.REDUCE_MAX, "max"), (orc.REDUCE_SUM, "sum")])
def test_score_closed_form_group_reduction(reduce, tag):
    """One KV head, G = 2 query heads x p = 2 patch tokens = the 4 fixture rows."""
    a, b, rows, red = _load_integer_powers()
    keys = np.array([[math.log(x), math.log(y)] for x, y in zip(a, b)])
    q = np.array([r[0] for r in rows], dtype=np.float64).reshape(1, 2, 2, 2)
    k = keys.reshape(1, 1, 4, 2)
    got = orc.score(q, k, 4, reduce, scale=1.0)[0, 0]
    np.testing.assert_allclose(got, [float(f) for f in red[tag]], rtol=1e-13)


def test_score_gqa_mapping_contiguous_groups():
    """Query head hq votes for KV head hq // G: KV head 0 sees fixture rows 0-1, head 1 rows 2-3."""
    a, b, rows, _ = _load_integer_powers()
    keys = np.array([[math.log(x), math.log(y)] for x, y in zip(a, b)])
    # Hq = 4, Hkv = 2, p = 1
    q = np.array([r[0] for r in rows], dtype=np.float64).reshape(1, 4, 1, 2)
    k = np.stack([keys, keys[::-1]]).reshape(1, 2, 4, 2)
    s = orc.score(q, k, 4, orc.REDUCE_SUM, scale=1.0)
    e0 = [float(rows[0][1][i] + rows[1][1][i]) for i in range(4)]
    e1 = [float(rows[2][1][i] + rows[3][1][i]) for i in range(4)][::-1]
    np.testing.assert_allclose(s[0, 0], e0, rtol=1e-13)
    np.testing.assert_allclose(s[0, 1], e1, rtol=1e-13)


def test_score_default_scale_is_inverse_sqrt_d():
    # d = 4, q = (1,1,1,1), key i = (2 ln n_i, 0, 0, 0): logit = 2 ln n_i / 2 = ln n_i
    n = [1, 2, 5]
    k = np.zeros((1, 1, 3, 4))
    k[0, 0, :, 0] = [2 * math.log(x) for x in n]
    q = np.ones((1, 1, 1, 4))
    s = orc.score(q, k, 3, orc.REDUCE_MAX)[0, 0]
    np.testing.assert_allclose(s, [1 / 8, 2 / 8, 5 / 8], rtol=1e-13)


def test_single_row_equals_library_softmax():
    """G = p = 1: both reductions reduce to one softmax row; check against scipy and torch."""
    rng = np.random.default_rng(7)
    d, N = 16, 50
    q = rng.standard_normal((1, 1, 1, d))
    k = rng.standard_normal((1, 1, N, d))
    z = (k[0, 0] @ q[0, 0, 0]) / math.sqrt(d)
    via_lse = np.exp(z - scipy.special.logsumexp(z))
    via_torch = torch.softmax(torch.from_numpy(z), dim=0).numpy()
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        s = orc.score(q, k, N, reduce)[0, 0]
        np.testing.assert_allclose(s, via_lse, rtol=1e-12)
        np.testing.assert_allclose(s, via_torch, rtol=1e-12)


def test_score_against_elementwise_python_loops():
    """Brute force with scalar Python arithmetic (no matmul, no numpy reductions)."""
    rng = np.random.default_rng(11)
    nb, Hq, Hkv, p, d, N = 2, 4, 2, 3, 5, 7
    q = rng.standard_normal((nb, Hq, p, d))
    k = rng.standard_normal((nb, Hkv, N + 2, d))  # capacity > n_ctx
    G = Hq // Hkv
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        s = orc.score(q, k, N, reduce)
        for b in range(nb):
            for h in range(Hkv):
                acc = [0.0] * N
                for g in range(G):
                    for t in range(p):
                        z = [sum(q[b, h * G + g, t, c] * k[b, h, i, c] for c in range(d)) / math.sqrt(d)
                             for i in range(N)]
                        den = sum(math.exp(x) for x in z)
                        for i in range(N):
                            w = math.exp(z[i]) / den
                            acc[i] = max(acc[i], w) if reduce == orc.REDUCE_MAX else acc[i] + w
                np.testing.assert_allclose(s[b, h], acc, rtol=1e-12)


def test_rows_beyond_n_ctx_are_ignored():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 2, 4, 8))
    k = rng.standard_normal((1, 1, 12, 8))
    k2 = k.copy()
    k2[:, :, 9:] = 100.0
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        np.testing.assert_array_equal(orc.score(q, k, 9, reduce), orc.score(q, k2, 9, reduce))


def test_sum_mode_total_mass_is_R_and_bounds():
    rng = np.random.default_rng(5)
    nb, Hq, Hkv, p, d, N = 2, 6, 2, 5, 8, 33
    q = rng.standard_normal((nb, Hq, p, d)) * 3
    k = rng.standard_normal((nb, Hkv, N, d))
    R = (Hq // Hkv) * p
    ssum = orc.score(q, k, N, orc.REDUCE_SUM)
    smax = orc.score(q, k, N, orc.REDUCE_MAX)
    np.testing.assert_allclose(ssum.sum(axis=2), R, rtol=1e-12)
    assert (smax.max(axis=2) >= 1.0 / N).all()
    assert (smax <= ssum * (1 + 1e-15)).all() and (ssum <= R * smax * (1 + 1e-15)).all()


def test_zero_queries_or_equal_keys_give_uniform_weights():
    N, R = 10, 6
    k = np.random.default_rng(1).standard_normal((1, 1, N, 4))
    q0 = np.zeros((1, 2, 3, 4))
    np.testing.assert_allclose(orc.score(q0, k, N, orc.REDUCE_MAX), 1.0 / N, rtol=1e-15)
    np.testing.assert_allclose(orc.score(q0, k, N, orc.REDUCE_SUM), R / N, rtol=1e-15)
    q = np.random.default_rng(2).standard_normal((1, 2, 3, 4))
    ksame = np.tile(k[:, :, :1], (1, 1, N, 1))
    np.testing.assert_allclose(orc.score(q, ksame, N, orc.REDUCE_MAX), 1.0 / N, rtol=1e-14)


def test_key_shift_invariance_and_permutation_equivariance():
    rng = np.random.default_rng(9)
    q = rng.standard_normal((1, 4, 3, 8))
    k = rng.standard_normal((1, 2, 21, 8))
    u = rng.standard_normal(8)
    perm = rng.permutation(21)
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        s = orc.score(q, k, 21, reduce)
        np.testing.assert_allclose(orc.score(q, k + u, 21, reduce), s, rtol=1e-11)
        np.testing.assert_allclose(orc.score(q, k[:, :, perm], 21, reduce), s[:, :, perm], rtol=1e-12)


def test_dominant_key_takes_all_the_mass():
    d, N = 4, 9
    q = np.ones((1, 2, 2, d))
    k = np.zeros((1, 1, N, d))
    k[0, 0, 4] = 25.0  # logit 4*25/2 = 50 above the rest
    smax = orc.score(q, k, N, orc.REDUCE_MAX)[0, 0]
    ssum = orc.score(q, k, N, orc.REDUCE_SUM)[0, 0]
    assert abs(smax[4] - 1) < 1e-20 + 1e-15 and abs(ssum[4] - 4) < 1e-14
    assert np.delete(smax, 4).max() < 1e-21


def test_score_given_lse_reduces_to_score_and_to_the_closed_form():
    rng = np.random.default_rng(31)
    q = rng.standard_normal((2, 4, 3, 8))
    k = rng.standard_normal((2, 2, 17, 8))
    z = np.einsum("bhtd,bhnd->bhtn", q, np.repeat(k, 2, axis=1)) / math.sqrt(8)
    lse = scipy.special.logsumexp(z, axis=3)                      # normaliser over exactly the context keys
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        np.testing.assert_allclose(orc.score_given_lse(q, k, 17, lse, reduce), orc.score(q, k, 17, reduce), rtol=1e-12)
    a, b, rows, red = _load_integer_powers()
    keys = np.array([[math.log(x), math.log(y)] for x, y in zip(a, b)]).reshape(1, 1, 4, 2)
    qq = np.array([r[0] for r in rows], dtype=np.float64).reshape(1, 2, 2, 2)
    lse = np.log(np.array([10.0, 7.0, 19.0, 113.0 / 6.0])).reshape(1, 2, 2)   # denominators of the fixture rows
    got = orc.score_given_lse(qq, keys, 4, lse, orc.REDUCE_SUM, scale=1.0)[0, 0]
    np.testing.assert_allclose(got, [float(f) for f in red["sum"]], rtol=1e-13)


def test_score_given_lse_with_a_larger_denominator_is_the_restricted_full_softmax():
    """Normaliser taken over context keys plus extra keys (the patch's own keys in a real forward
    pass): the result is the attention weight of the concatenated softmax on the context columns."""
    rng = np.random.default_rng(37)
    d, N, X = 8, 13, 5
    q = rng.standard_normal((1, 1, 4, d))
    k = rng.standard_normal((1, 1, N, d))
    extra = rng.standard_normal((X, d))
    full = orc.attention_weights(q[0, 0], np.concatenate([k[0, 0], extra]), 1 / math.sqrt(d))   # [4, N+X]
    z_all = (q[0, 0] @ np.concatenate([k[0, 0], extra]).T) / math.sqrt(d)
    lse = scipy.special.logsumexp(z_all, axis=1).reshape(1, 1, 4)
    np.testing.assert_allclose(orc.score_given_lse(q, k, N, lse, orc.REDUCE_MAX)[0, 0], full[:, :N].max(axis=0), rtol=1e-12)
    np.testing.assert_allclose(orc.score_given_lse(q, k, N, lse, orc.REDUCE_SUM)[0, 0], full[:, :N].sum(axis=0), rtol=1e-12)


# ----------------------------------------------------------------- topk pins

def test_topk_matches_counting_definition_with_ties():
    rng = np.random.default_rng(13)
    for trial in range(200):
        N = int(rng.integers(1, 65))
        M = int(rng.integers(1, N + 3))
        s = rng.integers(0, 6, N).astype(np.float32)  # many exact ties
        assert orc.topk_1d(s, M).tolist() == orc.topk_by_counting(s.tolist(), M)


def test_topk_exhaustive_small_permutations():
    for N in range(1, 7):
        for perm in itertools.permutations(range(N)):
            s = np.array(perm, dtype=np.float32)
            for M in range(1, N + 1):
                expect = sorted(i for i in range(N) if perm[i] >= N - M)
                assert orc.topk_1d(s, M).tolist() == expect


def test_topk_invariants_random():
    rng = np.random.default_rng(17)
    s = rng.random((3, 2, 500)).astype(np.float32)
    M = 123
    idx = orc.topk(s, M)
    assert idx.shape == (3, 2, M) and idx.dtype == np.int32
    for b in range(3):
        for h in range(2):
            I = idx[b, h]
            assert (np.diff(I) > 0).all() and I[0] >= 0 and I[-1] < 500
            rest = np.setdiff1d(np.arange(500), I)
            assert s[b, h][I].min() >= s[b, h][rest].max()


def test_topk_degenerate_cases():
    s = np.array([0.3, 0.9, 0.1, 0.5], dtype=np.float32)
    assert orc.topk_1d(s, 4).tolist() == [0, 1, 2, 3]      # M = N: identity
    assert orc.topk_1d(s, 9).tolist() == [0, 1, 2, 3]      # M > N: keep everything
    assert orc.topk_1d(s, 1).tolist() == [1]               # Fig. 1b shape: M = 1 of 1 + 3
    assert orc.topk_1d(np.full(7, 0.25, np.float32), 3).tolist() == [0, 1, 2]  # all equal: oldest


# -------------------------------------------------------------- compact pins

def test_compact_is_a_row_gather_of_bit_patterns():
    rng = np.random.default_rng(19)
    x = rng.integers(0, 2 ** 16, (2, 3, 20, 8), dtype=np.uint16)
    idx = np.sort(np.stack([[rng.permutation(20)[:7] for _ in range(3)] for _ in range(2)]), axis=-1)
    out = orc.compact(x, idx.astype(np.int32))
    for b in range(2):
        for h in range(3):
            for j in range(7):
                assert (out[b, h, j] == x[b, h, idx[b, h, j]]).all()
    ident = np.tile(np.arange(20, dtype=np.int32), (2, 3, 1))
    assert (orc.compact(x, ident) == x).all()


# ------------------------------------------------------------ whole-step pins

def test_evict_step_kept_tokens_follow_the_rows_under_permutation():
    rng = np.random.default_rng(23)
    nb, Hq, Hkv, p, d, N, M = 1, 4, 2, 4, 8, 40, 15
    q = rng.standard_normal((nb, Hq, p, d))
    k = rng.standard_normal((nb, Hkv, N, d))
    v = rng.standard_normal((nb, Hkv, N, d))
    perm = rng.permutation(N)
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        _, idx, kk, vv = orc.evict_step(q, k, v, N, M, reduce)
        _, idx_p, _, _ = orc.evict_step(q, k[:, :, perm], v[:, :, perm], N, M, reduce)
        for h in range(Hkv):
            assert set(perm[idx_p[0, h]].tolist()) == set(idx[0, h].tolist())
            assert (kk[0, h] == k[0, h][idx[0, h]]).all() and (vv[0, h] == v[0, h][idx[0, h]]).all()


def test_block_prefill_sweep_keeps_cache_at_budget():
    """Sec. 2.2 / App. A.3: cache is M after every step and never above M + M_block."""
    rng = np.random.default_rng(29)
    Hq, Hkv, p, d, M, B = 2, 1, 3, 4, 6, 4
    cache_k = np.empty((1, Hkv, 0, d))
    cache_v = np.empty((1, Hkv, 0, d))
    for step in range(8):
        cache_k = np.concatenate([cache_k, rng.standard_normal((1, Hkv, B, d))], axis=2)
        cache_v = np.concatenate([cache_v, rng.standard_normal((1, Hkv, B, d))], axis=2)
        n = cache_k.shape[2]
        assert n <= M + B
        q = rng.standard_normal((1, Hq, p, d))
        _, idx, cache_k, cache_v = orc.evict_step(q, cache_k, cache_v, n, M)
        assert cache_k.shape[2] == min(M, n) == idx.shape[2]
    assert cache_k.shape[2] == M
