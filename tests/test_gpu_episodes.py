"""GPU parity of the episode geometry calls (Sec. 3.1 Eq. 3, Stage 3a/3b) against the CPU oracle.
Embeddings are seeded synthetic vectors with cluster structure (the encoder is outside the library)."""
import sys

import numpy as np
import pytest
import torch

from oracle import epicache_oracle as orc
from paper_2509_17396_amd import binding as ep

pytestmark = pytest.mark.gpu

DEV = "cuda"
COS_TOL = 1e-5   # fp32 dot products of up to a few thousand terms against float64


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def clustered(seed, K, D, E):
    """K unit-ish vectors around E random directions, plus the assignment a clustering would return."""
    rng = np.random.default_rng(seed)
    dirs = rng.standard_normal((E, D))
    assign = rng.integers(0, E, size=K).astype(np.int32)
    emb = (dirs[assign] + 0.7 * rng.standard_normal((K, D))).astype(np.float32)
    return emb, assign


def gpu_medoids(emb, assign, E):
    cent = torch.full((E, emb.shape[1]), float("nan"), dtype=torch.float32, device=DEV)
    med = torch.full((E,), -7, dtype=torch.int32, device=DEV)
    ep.epicache_episode_medoids(torch.from_numpy(emb).to(DEV), torch.from_numpy(assign).to(DEV), E, cent, med)
    torch.cuda.synchronize()
    return cent.cpu().numpy(), med.cpu().numpy()


def gpu_match(q, cents, tau):
    out = torch.full((q.shape[0],), -7, dtype=torch.int32, device=DEV)
    cs = torch.full((q.shape[0],), float("nan"), dtype=torch.float32, device=DEV)
    ep.epicache_match_queries(torch.from_numpy(q).to(DEV), torch.from_numpy(cents).to(DEV), tau, out, cs)
    torch.cuda.synchronize()
    return out.cpu().numpy(), cs.cpu().numpy()


@pytest.mark.parametrize("K,D,E", [(500, 384, 4), (1200, 1024, 10), (37, 100, 5), (64, 8192, 3), (9, 1, 2)])
def test_medoids_match_oracle(K, D, E):
    say(f"medoids K={K} D={D} E={E}")
    emb, assign = clustered(K + D, K, D, E)
    assign[assign == E - 1] = 0 if K < 40 else E - 1      # the small cases get an empty last cluster
    cent, med = gpu_medoids(emb, assign, E)
    o_cent, o_med = orc.episode_medoids(emb, assign, E)
    np.testing.assert_allclose(cent, o_cent, rtol=1e-5, atol=1e-6)
    for e in range(E):
        if o_med[e] < 0:
            assert med[e] == -1 and (cent[e] == 0).all()
            continue
        assert assign[med[e]] == e
        if med[e] != o_med[e]:      # allowed only when the two members are equally close within fp32
            gap = orc._cosine(emb[o_med[e]].astype(np.float64), o_cent[e]) - \
                  orc._cosine(emb[med[e]].astype(np.float64), o_cent[e])
            assert 0 <= gap <= COS_TOL, f"cluster {e}: gap {gap}"


def test_medoid_ties_go_to_the_lower_index_and_strays_are_ignored():
    emb = np.array([[0, 2], [2, 0], [5, 5], [2, 0], [0, 2], [1, 0]], dtype=np.float32)
    assign = np.array([0, 0, 7, 0, 0, -1], dtype=np.int32)     # 7 and -1 belong to no cluster
    cent, med = gpu_medoids(emb, assign, 2)
    assert med.tolist() == [0, -1]
    np.testing.assert_array_equal(cent, [[1, 1], [0, 0]])
    assert orc.episode_medoids(emb, assign, 2)[1].tolist() == [0, -1]


@pytest.mark.parametrize("nq,D,E", [(64, 384, 4), (300, 1024, 10), (5, 100, 1), (7, 3000, 130)])
def test_matching_matches_oracle(nq, D, E):
    say(f"match nq={nq} D={D} E={E}")
    rng = np.random.default_rng(nq + D)
    cents = rng.standard_normal((E, D)).astype(np.float32)
    noise = rng.uniform(0.2, 6.0, size=(nq, 1))           # from close to a centroid to unrelated
    q = (cents[rng.integers(0, E, size=nq)] + noise * rng.standard_normal((nq, D))).astype(np.float32)
    q[0] = cents[0] + 0.1 * rng.standard_normal(D)        # one clear match ...
    q[1] = rng.standard_normal(D) * (np.arange(D) % 2) - cents[0] * 0.5   # ... and one clear miss
    tau = 0.3
    got, cs = gpu_match(q, cents, tau)
    want, o_cs = orc.match_queries(q, cents, tau)
    np.testing.assert_allclose(cs, o_cs, atol=COS_TOL)
    free, _ = gpu_match(q, cents, float("-inf"))
    o_free, _ = orc.match_queries(q, cents)
    for i in range(nq):
        if free[i] != o_free[i]:    # two centroids equally close within fp32
            gap = o_cs[i] - orc._cosine(q[i].astype(np.float64), cents[free[i]].astype(np.float64))
            assert 0 <= gap <= COS_TOL
        if abs(o_cs[i] - tau) > COS_TOL:
            assert (got[i] == -1) == (want[i] == -1)
            if got[i] != -1:
                assert got[i] == free[i]
    assert (got == -1).any() and (got != -1).any()     # the threshold really splits this input


def test_matching_ties_zero_vectors_and_threshold_edge():
    cents = np.array([[1, 0], [0, 10], [-1, 0], [1, 0], [30, 30]], dtype=np.float32)
    q = np.array([[2, 0], [1, 1], [0, 0], [0, -3]], dtype=np.float32)
    got, cs = gpu_match(q, cents, float("-inf"))
    assert got.tolist() == [0, 4, 0, 0] and orc.match_queries(q, cents)[0].tolist() == [0, 4, 0, 0]
    assert cs[0] == 1.0 and cs[2] == 0.0 and cs[3] == 0.0
    got, _ = gpu_match(q, cents, 1.0)        # cosine == tau still matches (only "below" opens an episode)
    assert got.tolist() == [0, -1, -1, -1] or got.tolist() == [0, 4, -1, -1]
    assert orc.match_queries(q, cents, 1.0)[0][0] == 0


def test_centroid_depends_on_its_members_only():
    """Eq. 3: a centroid is the mean of its own members.  A non-finite embedding in one cluster must not
    reach the centroids of the others."""
    say("centroids with a non-finite member elsewhere")
    emb, assign = clustered(3, 300, 256, 4)
    bad = int(np.nonzero(assign == 2)[0][0])
    emb[bad, 5], emb[bad, 17] = np.inf, np.nan
    cent, _ = gpu_medoids(emb, assign, 4)
    clean = emb.copy()
    clean[bad] = 0.0
    o_cent, _ = orc.episode_medoids(clean, assign, 4)
    for e in (0, 1, 3):
        assert np.isfinite(cent[e]).all()
        np.testing.assert_allclose(cent[e], o_cent[e], rtol=1e-5, atol=1e-6)
    assert not np.isfinite(cent[2, 5]) and not np.isfinite(cent[2, 17])
