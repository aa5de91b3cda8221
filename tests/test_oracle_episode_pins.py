"""Pins of the oracle's episode geometry (Sec. 3.1 Eq. 3, Stage 3a/3b): hand-worked cases,
library routines that compute the same thing another way, invariants and planted mistakes."""
import numpy as np
import pytest
from scipy.spatial.distance import cdist

from oracle import epicache_oracle as orc


def test_hand_worked_medoids():
    # cluster 0: (1,0), (0,1), (1,1): centroid (2/3, 2/3) -> the diagonal member (index 3) is closest
    # cluster 1: a single member is its own centroid; cluster 2 is empty
    emb = np.array([[1.0, 0.0], [5.0, 5.1], [0.0, 1.0], [1.0, 1.0]])
    cent, med = orc.episode_medoids(emb, [0, 1, 0, 0], 3)
    np.testing.assert_allclose(cent, [[2 / 3, 2 / 3], [5.0, 5.1], [0, 0]], rtol=1e-15)
    assert med.tolist() == [3, 1, -1]
    # two members at the same angle to the centroid: the lower index wins
    _, med = orc.episode_medoids(np.array([[0.0, 2.0], [2.0, 0.0]]), [0, 0], 1)
    assert med.tolist() == [0]


def test_medoids_against_scipy_cosine_distances():
    rng = np.random.default_rng(0)
    emb = rng.standard_normal((60, 16))
    assign = rng.integers(0, 5, size=60)
    cent, med = orc.episode_medoids(emb, assign, 5)
    for e in range(5):
        members = np.nonzero(assign == e)[0]
        np.testing.assert_allclose(cent[e], emb[members].mean(axis=0), rtol=1e-13)
        dist = cdist(emb[members], cent[e][None], metric="cosine")[:, 0]     # 1 - cosine
        assert med[e] == members[np.argmin(dist)]
    # scaling an embedding does not change its cosine, but it moves the centroid towards it
    assert orc.episode_medoids(emb * 3.0, assign, 5)[1].tolist() == med.tolist()


def test_hand_worked_matching_and_threshold():
    cents = np.array([[1.0, 0.0], [0.0, 1.0], [-1.0, 0.0]])
    q = np.array([[2.0, 0.1], [0.3, 4.0], [-1.0, -1.0], [0.0, 0.0], [1.0, 1.0]])
    ep, cs = orc.match_queries(q, cents)
    assert ep.tolist() == [0, 1, 2, 0, 0]           # zero query: all cosines 0 -> lowest index; tie -> lower e
    np.testing.assert_allclose(cs[2], 1 / np.sqrt(2), rtol=1e-15)
    assert cs[3] == 0.0
    ep, _ = orc.match_queries(q, cents, tau=0.9)     # Stage 3b: too far from every centroid -> new episode
    assert ep.tolist() == [0, 1, -1, -1, -1]
    ep, _ = orc.match_queries(q, cents, tau=1 / np.sqrt(2) - 1e-12)
    assert ep.tolist() == [0, 1, 2, -1, 0]


def test_matching_against_scipy_and_invariances():
    rng = np.random.default_rng(1)
    cents, q = rng.standard_normal((7, 12)), rng.standard_normal((40, 12))
    ep, cs = orc.match_queries(q, cents)
    sim = 1 - cdist(q, cents, metric="cosine")
    assert ep.tolist() == sim.argmax(axis=1).tolist()
    np.testing.assert_allclose(cs, sim.max(axis=1), rtol=1e-12)
    scale_q, scale_c = rng.random(40) + 0.1, rng.random(7) + 0.1
    assert orc.match_queries(q * scale_q[:, None], cents * scale_c[:, None])[0].tolist() == ep.tolist()
    # a member's own cluster centroid is not necessarily its match, but a centroid matches itself
    assert orc.match_queries(cents, cents)[0].tolist() == list(range(7))


@pytest.mark.parametrize("mistake", [None, "dot_product", "euclidean", "ties_to_higher"])
def test_planted_mistakes_in_matching(mistake):
    cents = np.array([[1.0, 0.0], [0.0, 10.0], [-1.0, 0.0], [1.0, 0.0], [30.0, 30.0]])
    q = np.array([[2.0, 0.1], [1.0, 1.0]])

    def variant(q, cents):
        if mistake == "dot_product":
            sim = q @ cents.T
        elif mistake == "euclidean":
            sim = -cdist(q, cents)
        else:
            sim = 1 - cdist(q, cents, metric="cosine")
        if mistake == "ties_to_higher":
            return [len(cents) - 1 - int(np.argmax(r[::-1])) for r in sim]
        return [int(np.argmax(r)) for r in sim]

    # q0 is almost parallel to centroids 0 and 3 (a tie: the lower index wins) although the long diagonal
    # centroid 4 has the largest dot product; q1 is parallel to centroid 4, which is far away in distance.
    assert (variant(q, cents) == [0, 4]) == (mistake is None)
    assert orc.match_queries(q, cents)[0].tolist() == [0, 4]
