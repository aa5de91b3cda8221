"""Seeded sweep of valid shapes through the whole eviction step against the oracle: head dims that take the
MFMA kernels (64, 128 in bf16) and the plain ones (any multiple of 8, fp32 or bf16), group sizes, patch
lengths, context lengths around tile boundaries, budgets from 1 to N, both reductions, with and without the
patch's own causal keys, K/V buffers with spare capacity."""
import sys

import numpy as np
import pytest
import torch

from oracle import epicache_oracle as orc
from paper_2509_17396_amd import binding as ep
from paper_2509_17396_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda"
N_CASES = 160


def draw_case(i):
    rng = np.random.default_rng(0xE91C + i)
    bf16 = bool(rng.integers(0, 2))
    d = int(rng.choice([64, 128])) if (bf16 and rng.random() < 0.7) else int(8 * rng.integers(1, 33))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 3, 4, 7]))
    p = int(rng.choice([1, 3, 16, 31, 32, 33, 64, 65, 100]))
    N = int(rng.choice([1, 2, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 511, 513, 700, 1025]))
    M = int(rng.choice([1, max(1, N // 3), max(1, N // 2), max(1, N - 1), N + 5], p=[0.15, 0.3, 0.3, 0.15, 0.1]))
    E = int(rng.integers(1, 4))
    recipe = str(rng.choice(["normal", "outlier_channels", "student_t"]))
    reduce = int(rng.integers(0, 2))
    causal = int(rng.integers(0, 2))
    spare = int(rng.choice([0, 3, 64]))
    return dict(bf16=bf16, d=d, Hkv=Hkv, G=G, p=p, N=N, M=M, E=E, recipe=recipe, reduce=reduce, causal=causal,
                spare=spare, seed=i)


def run_case(c, i, overlapped_chunks=0):
    """overlapped_chunks > 0: through epicache_evict_step_overlapped with that many chunks asked for."""
    w = synth.WORKLOADS["tiny"].scaled(E=c["E"], Hq=c["Hkv"] * c["G"], Hkv=c["Hkv"], d=c["d"], p=c["p"],
                                       dtype="bf16" if c["bf16"] else "f32", M=c["M"], B=1, recipe=c["recipe"],
                                       seed=0xE91C1000 + i)
    N, M = c["N"], c["M"]
    rows = N + (c["p"] if c["causal"] else 0)
    q, k, v = synth.make_layer(w, layer=i, n_ctx=rows, capacity=rows + c["spare"])
    qd, kd, vd = q.to(DEV), k.to(DEV).clone(), v.to(DEV).clone()
    n_cached = min(M, N)
    prm = ep.make_params(qd, kd, n_cached=n_cached, n_block=N - n_cached, budget=M, reduce=c["reduce"],
                         causal_patch=c["causal"])
    n_keep = min(M, N)
    scores = torch.full((w.E, w.Hkv, N), float("nan"), dtype=torch.float32, device=DEV)
    keep = torch.full((w.E, w.Hkv, n_keep), -1, dtype=torch.int32, device=DEV)
    if overlapped_chunks:
        nbytes, used = ep.epicache_overlapped_workspace_size(prm, overlapped_chunks)
        assert used == -(-w.E // -(-w.E // min(overlapped_chunks, w.E)))
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV)
        ep.epicache_evict_step_overlapped(prm, qd, kd, vd, ws, torch.cuda.Stream(), overlapped_chunks, scores, keep)
    else:
        ws = ep.alloc_workspace(prm)
        ep.epicache_evict_step(prm, qd, kd, vd, ws, scores, keep)
    torch.cuda.synchronize()
    scores, keep = scores.cpu().numpy(), keep.cpu().numpy()
    qq, kk = pu.oracle_inputs(q, k)
    want = orc.score_causal_patch(qq, kk, N, c["reduce"]) if c["causal"] else orc.score(qq, kk[:, :, :N], N, c["reduce"])
    rtol = pu.rtol_for(q.dtype)
    pu.assert_scores_close(scores, want, rtol, str(c))
    pu.assert_keep_matches(keep, want, M, rtol, str(c))
    kb, vb = synth.raw_bits_numpy(k), synth.raw_bits_numpy(v)
    got_k, got_v = synth.raw_bits_numpy(kd.cpu()), synth.raw_bits_numpy(vd.cpu())
    if N > M:
        np.testing.assert_array_equal(got_k[:, :, :n_keep], orc.compact(kb, keep))
        np.testing.assert_array_equal(got_v[:, :, :n_keep], orc.compact(vb, keep))
        np.testing.assert_array_equal(got_k[:, :, N:], kb[:, :, N:])     # patch rows and spare capacity untouched
    else:
        np.testing.assert_array_equal(got_k, kb)
        np.testing.assert_array_equal(got_v, vb)


@pytest.mark.parametrize("i", range(N_CASES))
def test_evict_step_random_shape(i):
    c = draw_case(i)
    print(f"[case] {c}", flush=True)
    sys.stdout.flush()
    run_case(c, i)


@pytest.mark.parametrize("i", range(48))
def test_overlapped_step_random_shape(i):
    """The same sweep through the two-stream pipeline: 2-9 batch items cut into 2-9 chunks (equal chunks, a shorter
    last chunk, one item per chunk)."""
    c = draw_case(1000 + i)
    rng = np.random.default_rng(0x0E71 + i)
    c["E"] = int(rng.integers(2, 10))
    chunks = int(rng.integers(2, 10))
    print(f"[case] overlapped, {chunks} chunks asked: {c}", flush=True)
    sys.stdout.flush()
    run_case(c, 1000 + i, overlapped_chunks=chunks)
