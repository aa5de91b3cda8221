"""GPU parity at the full sizes of the five workloads.

Inputs are generated on the GPU by the seeded generator; the oracle gets the very
same bits (copied back) for a sample of (batch item, KV head) pairs, which it can
compute one by one, and the rest is checked through properties that hold at any
size.  The first test is the exact launch configuration that bench.py times."""
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


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def evict_on_gpu(q, k, v, M, N, reduce):
    prm = ep.make_params(q, k, n_cached=min(M, N), n_block=N - min(M, N), budget=M, reduce=reduce)
    ws = ep.alloc_workspace(prm)
    nb, H = q.shape[0], k.shape[1]
    scores = torch.full((nb, H, N), float("nan"), dtype=torch.float32, device=DEV)
    keep = torch.full((nb, H, min(M, N)), -1, dtype=torch.int32, device=DEV)
    ep.epicache_evict_step(prm, q, k, v, ws, scores, keep)
    torch.cuda.synchronize()
    return scores, keep


def check_sampled(q, k0, v0, k, v, scores, keep, M, N, reduce, samples, what):
    """q, k0, v0: inputs (k0/v0 untouched copies); k, v: after the step."""
    rtol = pu.rtol_for(q.dtype)
    nb, H = k0.shape[0], k0.shape[1]
    n_keep = min(M, N)
    # properties over the whole batch, on the device
    assert torch.isfinite(scores).all(), what
    assert (keep[:, :, 1:] > keep[:, :, :-1]).all() and keep.min() >= 0 and keep.max() < N, what
    if reduce == orc.REDUCE_SUM:  # total attention mass of the R rows
        R = (q.shape[1] // H) * q.shape[2]
        torch.testing.assert_close(scores.double().sum(dim=2), torch.full((nb, H), float(R), dtype=torch.float64, device=DEV),
                                   rtol=1e-4, atol=0)
    # no evicted token outscores a kept one (by more than nothing: exact, same fp32 scores)
    kept_min = torch.gather(scores, 2, keep.long()).min(dim=2).values
    mask = torch.ones_like(scores, dtype=torch.bool).scatter_(2, keep.long(), False)
    evicted_max = torch.where(mask, scores, torch.full_like(scores, -1.0)).max(dim=2).values
    assert (kept_min >= evicted_max).all(), what
    # compaction bit exact everywhere: gather with the GPU's own index list, on the device, via torch
    idx = keep.long().unsqueeze(-1).expand(-1, -1, -1, k0.shape[3])
    assert torch.equal(torch.gather(k0, 2, idx).view(torch.int16), k[:, :, :n_keep].view(torch.int16)), what
    assert torch.equal(torch.gather(v0, 2, idx).view(torch.int16), v[:, :, :n_keep].view(torch.int16)), what
    # sampled (b, h): scores and kept set against the oracle
    differ = 0
    for (b, h) in samples:
        say(f"  {what}: oracle on b={b} h={h}")
        o = pu.oracle_score_one_head(q, k0, b, h, N, reduce)
        pu.assert_scores_close(scores[b, h].cpu().numpy(), o, rtol, f"{what} b={b} h={h}")
        differ += pu.assert_keep_matches(keep[b:b + 1, h:h + 1].cpu().numpy(), o[None, None], M, rtol, f"{what} b={b} h={h}")
    return differ


@pytest.mark.parametrize("reduce", [orc.REDUCE_SUM, orc.REDUCE_MAX], ids=["sum", "max"])
def test_config2_all_layers_folded_as_benchmarked(reduce):
    """LLaMA-3.2-3B-shaped: 28 layers x 4 episodes folded into one launch (what bench.py times)."""
    w = synth.WORKLOADS["llama32_3b"]
    say(f"config 2 folded L={w.L} reduce={reduce}")
    q, k0, v0 = synth.make_folded(w, range(w.L), device=DEV)
    k, v = k0.clone(), v0.clone()
    scores, keep = evict_on_gpu(q, k, v, w.M, w.N, reduce)
    nb = w.L * w.E
    samples = [(0, 0), (5, 3), (57, 7), (nb - 1, w.Hkv - 1)]
    differ = check_sampled(q, k0, v0, k, v, scores, keep, w.M, w.N, reduce, samples, "config2")
    say(f"  kept-set differences inside the band: {differ}")


FULL_LAYER_CASES = [
    ("llama31_8b", [(0, 0), (3, 7)]),
    ("qwen25_7b", [(0, 0), (7, 3)]),
    ("stress", [(0, 0), (15, 7)]),
]


@pytest.mark.parametrize("reduce", [orc.REDUCE_SUM, orc.REDUCE_MAX], ids=["sum", "max"])
@pytest.mark.parametrize("name,samples", FULL_LAYER_CASES, ids=[c[0] for c in FULL_LAYER_CASES])
def test_configs_3_to_5_one_layer_full_shape(name, samples, reduce):
    w = synth.WORKLOADS[name]
    say(f"{name} one layer E={w.E} N={w.N} R={w.R} reduce={reduce}")
    q, k0, v0 = synth.make_layer(w, layer=1, device=DEV)
    k, v = k0.clone(), v0.clone()
    scores, keep = evict_on_gpu(q, k, v, w.M, w.N, reduce)
    differ = check_sampled(q, k0, v0, k, v, scores, keep, w.M, w.N, reduce, samples, name)
    say(f"  kept-set differences inside the band: {differ}")


def test_config3_sweep_free_running_invariants():
    """Config 3's sweep at full per-layer shape (M = B = 4096, E = 4), 6 of its 50 steps, free running
    on the GPU: the cache is M after every step once filled and never exceeds M + B rows."""
    w = synth.WORKLOADS["llama31_8b"]
    cap = w.M + w.B
    say("config 3 sweep, free running")
    kbuf = torch.zeros(w.E, w.Hkv, cap, w.d, dtype=torch.bfloat16, device=DEV)
    vbuf = torch.zeros_like(kbuf)
    n_cached = 0
    for step in range(6):
        q, bk, bv = synth.make_layer(w, layer=0, step=step, device=DEV, n_ctx=w.B)
        assert n_cached + w.B <= cap
        kbuf[:, :, n_cached:n_cached + w.B] = bk
        vbuf[:, :, n_cached:n_cached + w.B] = bv
        N = n_cached + w.B
        k0, v0 = kbuf.clone(), vbuf.clone()
        prm = ep.make_params(q, kbuf, n_cached=n_cached, n_block=w.B, budget=w.M, reduce=orc.REDUCE_MAX)
        ws = ep.alloc_workspace(prm)
        keep = torch.full((w.E, w.Hkv, min(w.M, N)), -1, dtype=torch.int32, device=DEV)
        ep.epicache_evict_step(prm, q, kbuf, vbuf, ws, None, keep)
        torch.cuda.synchronize()
        n_keep = min(w.M, N)
        assert (keep[:, :, 1:] > keep[:, :, :-1]).all() and keep.min() >= 0 and keep.max() < N
        idx = keep.long().unsqueeze(-1).expand(-1, -1, -1, w.d)
        assert torch.equal(torch.gather(k0, 2, idx).view(torch.int16), kbuf[:, :, :n_keep].view(torch.int16))
        assert torch.equal(torch.gather(v0, 2, idx).view(torch.int16), vbuf[:, :, :n_keep].view(torch.int16))
        n_cached = n_keep
        assert n_cached == min(w.M, N)
    assert n_cached == w.M
