"""Pins of the oracle's ragged functions (per-head lengths, per-item budgets, pooled head-wise
selection) against things that are not the oracle: the counting definition evaluated by brute
force, hand-worked cases, invariants, and reductions to the already pinned uniform functions.
Planted mistakes (CPU copies of the selection with one plausible error) must fail them."""
import numpy as np
import pytest

from oracle import epicache_oracle as orc


def _rand_heads(rng, H, max_len, levels=None):
    lens = rng.integers(0, max_len + 1, size=H)
    if levels:   # few distinct values: plenty of ties within and across heads
        return [rng.integers(0, levels, size=n).astype(np.float64) for n in lens]
    return [rng.random(n) for n in lens]


# ---- pooled selection: a worked example, by hand -------------------------------------------
def test_pooled_selection_hand_worked_example():
    # Hkv = 3, M = 2 -> 6 of the 9 entries survive.  Sorted pool: 9 8 7 7 6 | 5 5 4 1, the sixth
    # place is a tie at 5 between (h0, i2) and (h2, i0): the lower head wins it.
    heads = [np.array([9.0, 1.0, 5.0]), np.array([7.0, 8.0]), np.array([5.0, 7.0, 4.0, 6.0])]
    keep = orc.select_pooled(heads, 2)
    assert [k.tolist() for k in keep] == [[0, 2], [0, 1], [1, 3]]
    # a head that concentrates on one token keeps few rows, the flat head keeps many
    heads = [np.array([100.0, 0.1, 0.1, 0.1]), np.array([3.0, 3.1, 3.2, 3.3])]
    assert [k.tolist() for k in orc.select_pooled(heads, 2)] == [[0], [1, 2, 3]]


@pytest.mark.parametrize("seed", range(12))
def test_pooled_selection_equals_counting_definition(seed):
    rng = np.random.default_rng(100 + seed)
    H = int(rng.integers(1, 5))
    heads = _rand_heads(rng, H, 9, levels=4 if seed % 2 else None)
    M = int(rng.integers(1, 6))
    got = orc.select_pooled(heads, M)
    want = orc.select_pooled_by_counting(heads, M)
    assert [g.tolist() for g in got] == want


@pytest.mark.parametrize("seed", range(6))
def test_pooled_selection_invariants(seed):
    rng = np.random.default_rng(200 + seed)
    H, M = 4, 7
    heads = _rand_heads(rng, H, 30)
    keep = orc.select_pooled(heads, M)
    total = sum(len(s) for s in heads)
    assert sum(len(k) for k in keep) == min(H * M, total)            # the layer holds Hkv * M rows
    kept_min = min((heads[h][keep[h]].min() for h in range(H) if len(keep[h])), default=np.inf)
    drop_max = max((np.delete(heads[h], keep[h]).max() for h in range(H)
                    if len(heads[h]) > len(keep[h])), default=-np.inf)
    assert kept_min >= drop_max                                      # one threshold for all heads
    for h in range(H):
        assert (np.diff(keep[h]) > 0).all()
    # monotone transforms of the whole pool change nothing; raising one head's scores can only help it
    same = orc.select_pooled([np.exp(3 * s) for s in heads], M)
    assert all((a == b).all() for a, b in zip(keep, same))
    boosted = [s.copy() for s in heads]
    boosted[2] = boosted[2] + 10.0
    kb = orc.select_pooled(boosted, M)
    assert len(kb[2]) == min(len(heads[2]), H * M) and len(kb[2]) >= len(keep[2])


def test_pooled_selection_reduces_to_topk_for_one_head_and_keeps_everything_that_fits():
    rng = np.random.default_rng(5)
    s = rng.integers(0, 6, size=40).astype(np.float64)
    assert (orc.select_pooled([s], 9)[0] == orc.topk_1d(s, 9)).all()
    assert orc.topk_by_counting(list(s), 9) == orc.select_pooled([s], 9)[0].tolist()
    heads = [rng.random(3), rng.random(0), rng.random(5)]
    keep = orc.select_pooled(heads, 3)   # 9 slots, 8 rows
    assert [k.tolist() for k in keep] == [[0, 1, 2], [], [0, 1, 2, 3, 4]]


def test_identical_heads_share_the_budget_evenly_up_to_ties():
    s = np.array([0.5, 0.1, 0.9, 0.3, 0.7, 0.2])
    keep = orc.select_pooled([s, s, s], 2)      # 6 slots; the values 0.9 and 0.7 fill them exactly
    assert [k.tolist() for k in keep] == [[2, 4]] * 3
    keep = orc.select_pooled([s, s, s], 1)      # 3 slots, all for the three copies of 0.9
    assert [k.tolist() for k in keep] == [[2]] * 3
    keep = orc.select_pooled([s, s], 1)[0:2]    # 2 slots
    assert [k.tolist() for k in keep] == [[2], [2]]
    s2 = np.array([0.9, 0.7, 0.7])
    keep = orc.select_pooled([s2, s2], 1)       # slots: both 0.9
    assert [k.tolist() for k in keep] == [[0], [0]]
    keep = orc.select_pooled([s2, s2, s2], 2)   # 6 slots: three 0.9, then 0.7 ties: h0 i1, h0 i2, h1 i1
    assert [k.tolist() for k in keep] == [[0, 1, 2], [0, 1], [0]]


# ---- planted mistakes ------------------------------------------------------------------------
def _pooled_variant(heads, M, mistake):
    H = len(heads)
    lens = [len(s) for s in heads]
    pool = np.concatenate(heads)
    total = len(pool)
    n_keep = min(H * M, total)
    if mistake == "budget_not_scaled_by_heads":
        n_keep = min(M, total)
    pos = np.arange(total)
    if mistake == "ties_to_higher_position":
        pos = -pos
    if mistake == "ties_by_token_then_head":
        pos = np.concatenate([np.arange(n) * H + h for h, n in enumerate(lens)])
    key = pool if mistake == "keeps_smallest" else -pool
    order = np.lexsort((pos, key))[:n_keep]
    if mistake == "per_head_topk":
        return [orc.topk_1d(s, M).tolist() for s in heads]
    kept = np.zeros(total, dtype=bool)
    kept[order] = True
    out, start = [], 0
    for n in lens:
        out.append(np.nonzero(kept[start:start + n])[0].tolist())
        start += n
    return out


@pytest.mark.parametrize("mistake", [None, "budget_not_scaled_by_heads", "ties_to_higher_position",
                                     "ties_by_token_then_head", "keeps_smallest", "per_head_topk"])
def test_planted_mistakes_in_pooled_selection_are_caught(mistake):
    cases = [
        ([np.array([9.0, 1.0, 5.0]), np.array([7.0, 8.0]), np.array([5.0, 7.0, 4.0, 6.0])], 2,
         [[0, 2], [0, 1], [1, 3]]),
        ([np.array([0.9, 0.7, 0.7])] * 3, 2, [[0, 1, 2], [0, 1], [0]]),
        ([np.array([100.0, 0.1, 0.1, 0.1]), np.array([3.0, 3.1, 3.2, 3.3])], 2, [[0], [1, 2, 3]]),
    ]
    agree = all(_pooled_variant(h, M, mistake) == want for h, M, want in cases)
    assert agree == (mistake is None)


# ---- ragged scoring and the whole ragged step ------------------------------------------------
def _tiny_batch(rng, nb=3, Hq=4, Hkv=2, p=3, d=8, C=20):
    q = rng.standard_normal((nb, Hq, p, d))
    k = rng.standard_normal((nb, Hkv, C, d))
    v = rng.standard_normal((nb, Hkv, C, d))
    return q, k, v


def test_score_ragged_is_the_uniform_score_of_each_prefix():
    rng = np.random.default_rng(7)
    q, k, _ = _tiny_batch(rng)
    n_ctx = [[5, 20], [0, 1], [13, 7]]
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        rows = orc.score_ragged(q, k, n_ctx, reduce)
        for b in range(3):
            for h in range(2):
                n = n_ctx[b][h]
                assert rows[b][h].shape == (n,)
                if n:
                    want = orc.score(q[b:b + 1], k[b:b + 1], n, reduce)[0, h]
                    assert np.array_equal(rows[b][h], want)
                if n and reduce == orc.REDUCE_SUM:     # every query row spreads weight 1 over its n keys
                    assert abs(rows[b][h].sum() - 2 * 3) < 1e-12
    assert orc.score_ragged(q, k, n_ctx, orc.REDUCE_MAX)[1][1].tolist() == [1.0]   # a single key takes all


def test_evict_step_ragged_per_head_with_equal_lengths_is_the_uniform_step():
    rng = np.random.default_rng(8)
    q, k, v = _tiny_batch(rng)
    n, M = 17, 6
    s, idx, kk, vv = orc.evict_step(q, k, v, n, M, orc.REDUCE_SUM)
    rows, keep, rk, rv = orc.evict_step_ragged(q, k, v, [[n, n]] * 3, [M] * 3, False, orc.REDUCE_SUM)
    for b in range(3):
        for h in range(2):
            assert np.array_equal(rows[b][h], s[b, h]) and np.array_equal(keep[b][h], idx[b, h])
            assert np.array_equal(rk[b][h], kk[b, h]) and np.array_equal(rv[b][h], vv[b, h])


def test_evict_step_ragged_budgets_and_lengths_are_per_item():
    rng = np.random.default_rng(9)
    q, k, v = _tiny_batch(rng)
    n_ctx = [[20, 11], [4, 0], [9, 16]]
    budgets = [5, 8, 3]
    for pooled in (False, True):
        rows, keep, kk, vv = orc.evict_step_ragged(q, k, v, n_ctx, budgets, pooled)
        for b in range(3):
            counts = [len(x) for x in keep[b]]
            if pooled:
                assert sum(counts) == min(2 * budgets[b], sum(n_ctx[b]))
            else:
                assert counts == [min(budgets[b], n) for n in n_ctx[b]]
            for h in range(2):
                assert (keep[b][h] < n_ctx[b][h]).all()
                assert np.array_equal(kk[b][h], k[b, h][keep[b][h]])      # a gather, nothing else
                assert np.array_equal(vv[b][h], v[b, h][keep[b][h]])
                kept_scores = rows[b][h].astype(np.float32)[keep[b][h]]
                dropped = np.delete(rows[b][h].astype(np.float32), keep[b][h])
                if not pooled and len(dropped) and len(kept_scores):
                    assert kept_scores.min() >= dropped.max()
