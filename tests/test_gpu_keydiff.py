"""GPU parity of the KeyDiff scorer (App. A.2) and of a KeyDiff eviction step on the shared
select / compact back end, against the CPU oracle."""
import sys

import numpy as np
import pytest
import torch

from oracle import epicache_oracle as orc
from paper_2509_17396_amd import binding as ep
from paper_2509_17396_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda"
# Scores are cosines in [-1, 1] computed with fp32 sums of d products and N keys: the error is absolute
# (a cosine near 0 has no relative accuracy), bounded by a few d * 2^-24.
ATOL_COS = 2e-5


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def wl(name, **kw):
    return synth.WORKLOADS[name].scaled(**kw)


def gpu_keydiff(k, N, n_ctx=None):
    kd = k.to(DEV)
    q = torch.empty((kd.shape[0], kd.shape[1], 1, kd.shape[3]), dtype=kd.dtype, device=DEV)   # geometry only
    prm = ep.make_params(q, kd, n_cached=0, n_block=N, budget=1)
    ws = ep.alloc_workspace(prm)
    scores = torch.full((kd.shape[0], kd.shape[1], N), -7.0, dtype=torch.float32, device=DEV)
    nc = None if n_ctx is None else torch.tensor(np.asarray(n_ctx, dtype=np.int32), device=DEV)
    ep.epicache_score_keydiff(prm, kd, scores, ws, nc)
    torch.cuda.synchronize()
    return scores.cpu().numpy()


KEYDIFF_CASES = [
    ("fp32_d40_ragged_rows", "tiny", dict(E=2, Hq=6, Hkv=2, p=5, d=40), 203, 230),
    ("fp32_d8", "tiny", dict(E=1, Hq=2, Hkv=2, p=1, d=8), 3000, None),
    ("fp32_d256", "tiny", dict(E=1, Hq=2, Hkv=1, p=1, d=256), 700, None),
    ("bf16_d128_outlier_channels", "llama32_3b", dict(E=2, Hq=6, Hkv=2), 4096, None),
    ("bf16_d128_several_chunks_ragged", "llama31_8b", dict(E=1, Hq=8, Hkv=2), 1500 + 37, 1600),
    ("bf16_d64", "llama32_3b", dict(E=2, Hq=4, Hkv=2, d=64), 333, None),
    ("bf16_d96_topics", "qwen25_7b", dict(E=1, Hq=4, Hkv=2, d=96), 1111, None),
    ("bf16_one_key", "llama32_3b", dict(E=1, Hq=2, Hkv=2), 1, 8),
]


@pytest.mark.parametrize("case", KEYDIFF_CASES, ids=[c[0] for c in KEYDIFF_CASES])
def test_keydiff_scores_match_oracle(case):
    name, base, over, N, cap = case
    w = wl(base, **over)
    say(f"keydiff {name}")
    _, k, _ = synth.make_layer(w, layer=0, n_ctx=N, capacity=cap)
    got = gpu_keydiff(k, N)
    want = orc.score_keydiff(synth.to_f64_numpy(k), N)
    err = np.abs(got - want).max()
    assert err <= ATOL_COS, f"{name}: max abs err {err:.3e}"
    say(f"  max abs err {err:.3e}")


def test_keydiff_ragged_lengths_and_degenerate_keys():
    w = wl("llama32_3b", E=2, Hq=6, Hkv=3)
    N = 1300
    _, k, _ = synth.make_layer(w, layer=1, n_ctx=N)
    k[0, 0, 5] = 0                       # a zero key scores 0
    k[1, 2, :4] = 0
    k[1, 2, 0, 0], k[1, 2, 1, 0] = 1.0, -1.0   # ... and so does every key of a head whose anchor is zero
    n_ctx = [[N, 0, 513], [512, 1, 4]]
    got = gpu_keydiff(k, N, n_ctx)
    want = orc.score_keydiff(synth.to_f64_numpy(k), n_ctx)
    for b in range(2):
        for h in range(3):
            n = n_ctx[b][h]
            assert np.abs(got[b, h, :n] - want[b, h, :n]).max(initial=0) <= ATOL_COS
            assert (got[b, h, n:] == -7.0).all()
    assert got[0, 0, 5] == 0.0 and (got[1, 2, :4] == 0.0).all() and got[1, 1, 0] == -1.0


def test_keydiff_eviction_step_on_the_shared_back_end():
    """KeyDiff scores -> epicache_topk -> epicache_compact: the kept set equals the oracle's except for
    tokens within the score tolerance of the threshold; the cache is the bit-exact gather of the kept rows."""
    w = wl("llama32_3b", E=2, Hq=6, Hkv=2, M=512, B=512)
    N = w.M + w.B
    say("keydiff eviction step")
    _, k, v = synth.make_layer(w, layer=4, n_ctx=N)
    kd, vd = k.to(DEV).clone(), v.to(DEV).clone()
    q = torch.empty((w.E, w.Hkv, 1, w.d), dtype=kd.dtype, device=DEV)
    prm = ep.make_params(q, kd, n_cached=w.M, n_block=w.B, budget=w.M)
    ws = ep.alloc_workspace(prm)
    scores = torch.empty((w.E, w.Hkv, N), dtype=torch.float32, device=DEV)
    keep = torch.empty((w.E, w.Hkv, w.M), dtype=torch.int32, device=DEV)
    ep.epicache_score_keydiff(prm, kd, scores, ws)
    ep.epicache_topk(prm, scores, keep)
    ep.epicache_compact(prm, keep, kd, vd)
    torch.cuda.synchronize()
    keep = keep.cpu().numpy()
    o_scores = orc.score_keydiff(synth.to_f64_numpy(k), N)
    o_keep = orc.topk(o_scores.astype(np.float32), w.M)
    differ = 0
    for b in range(w.E):
        for h in range(w.Hkv):
            assert (np.diff(keep[b, h]) > 0).all() and keep[b, h].min() >= 0 and keep[b, h].max() < N
            sym = np.setxor1d(keep[b, h], o_keep[b, h])
            thr = np.sort(o_scores[b, h])[N - w.M]
            assert (np.abs(o_scores[b, h][sym] - thr) <= ATOL_COS).all()
            differ += sym.size
    kb, vb = synth.raw_bits_numpy(k), synth.raw_bits_numpy(v)
    np.testing.assert_array_equal(synth.raw_bits_numpy(kd.cpu())[:, :, :w.M], orc.compact(kb, keep))
    np.testing.assert_array_equal(synth.raw_bits_numpy(vd.cpu())[:, :, :w.M], orc.compact(vb, keep))
    say(f"  tokens differing inside the band: {differ}")
