"""The pins must be sharp: plausible mistakes planted in a copy of the oracle's scoring
(on the CPU) have to disagree with the closed-form fixture or the invariants."""
import math

import numpy as np
import pytest

from oracle import epicache_oracle as orc
from tests.test_oracle_pins import _load_integer_powers


def _score_variant(q, k, n_ctx, reduce, scale, mistake):
    nb, Hq, p, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    out = np.empty((nb, Hkv, n_ctx))
    for b in range(nb):
        for h in range(Hkv):
            if mistake == "interleaved_heads":      # hq % Hkv instead of hq // G
                rows = np.concatenate([q[b, hq] for hq in range(Hq) if hq % Hkv == h])
            else:
                rows = q[b, h * G:(h + 1) * G].reshape(G * p, d)
            keys = k[b, h, :n_ctx]
            z = rows @ keys.T
            if mistake != "no_scale":
                z = scale * z
            if mistake == "softmax_over_rows":
                z = z - z.max(axis=0, keepdims=True)
                e = np.exp(z)
                w = e / e.sum(axis=0, keepdims=True)
            else:
                z = z - z.max(axis=1, keepdims=True)
                e = np.exp(z)
                w = e / e.sum(axis=1, keepdims=True)
            if mistake == "mean_not_sum" and reduce == orc.REDUCE_SUM:
                out[b, h] = w.mean(axis=0)
            elif mistake == "swap_reductions":
                out[b, h] = w.sum(axis=0) if reduce == orc.REDUCE_MAX else w.max(axis=0)
            else:
                out[b, h] = w.max(axis=0) if reduce == orc.REDUCE_MAX else w.sum(axis=0)
    return out


def _fixture_case():
    a, b, rows, red = _load_integer_powers()
    keys = np.array([[math.log(x), math.log(y)] for x, y in zip(a, b)])
    # Hq = 4, Hkv = 2, p = 1: KV head 0 <- fixture rows 0,1; KV head 1 (keys reversed) <- rows 2,3
    q = np.array([r[0] for r in rows], dtype=np.float64).reshape(1, 4, 1, 2)
    k = np.stack([keys, keys[::-1]]).reshape(1, 2, 4, 2)
    expect = {}
    for tag, fn in (("max", max), ("sum", lambda x: sum(x))):
        e0 = [float(fn([rows[0][1][i], rows[1][1][i]])) for i in range(4)]
        e1 = [float(fn([rows[2][1][i], rows[3][1][i]])) for i in range(4)][::-1]
        expect[tag] = np.array([e0, e1])[None]
    return q, k, expect


def test_correct_variant_matches_fixture_and_oracle():
    q, k, expect = _fixture_case()
    for reduce, tag in ((orc.REDUCE_MAX, "max"), (orc.REDUCE_SUM, "sum")):
        np.testing.assert_allclose(_score_variant(q, k, 4, reduce, 0.5, None), orc.score(q, k, 4, reduce, 0.5), rtol=1e-13)
        np.testing.assert_allclose(orc.score(q, k, 4, reduce, 1.0), expect[tag], rtol=1e-13)


@pytest.mark.parametrize("mistake", ["interleaved_heads", "no_scale", "softmax_over_rows", "mean_not_sum",
                                     "swap_reductions"])
def test_planted_mistake_is_caught(mistake):
    q, k, expect = _fixture_case()
    caught = False
    for reduce, tag in ((orc.REDUCE_MAX, "max"), (orc.REDUCE_SUM, "sum")):
        scale = 0.5 if mistake == "no_scale" else 1.0
        # for "no_scale" the fixture is rescaled: keys doubled so that scale 0.5 gives the printed weights
        kk = k * 2.0 if mistake == "no_scale" else k
        got = _score_variant(q, kk, 4, reduce, scale, mistake)
        if not np.allclose(got, expect[tag], rtol=1e-9):
            caught = True
    assert caught, f"the closed-form pin does not notice '{mistake}'"
