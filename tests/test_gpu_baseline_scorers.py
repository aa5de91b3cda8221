"""GPU parity of the App. A.2 baselines that are Eq. 1 with another patched prompt: SnapKV (the block's
last w tokens are the prompt, attend causally, and are always kept) and KVzip (a patch as long as the
block, scored in chunks of its tokens).  Scores elementwise against the oracle, kept sets by the band
rule (the window rows exactly), compacted K/V bit for bit."""
import ctypes
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


def _inputs(nb, Hq, Hkv, p, d, C, dtype, seed):
    gen = torch.Generator(device=DEV).manual_seed(seed)
    q = torch.randn((nb, Hq, p, d), device=DEV, generator=gen).to(dtype)
    k = torch.randn((nb, Hkv, C, d), device=DEV, generator=gen).to(dtype)
    v = torch.randn((nb, Hkv, C, d), device=DEV, generator=gen).to(dtype)
    return q, k, v


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


SNAPKV_CASES = [
    # nb, Hq, Hkv, w, d, N, M, dtype
    (2, 8, 2, 64, 128, 1500, 700, torch.bfloat16),     # the paper's window of 64, ragged last tile
    (1, 4, 4, 64, 128, 4096, 2048, torch.bfloat16),    # G = 1
    (3, 12, 4, 16, 64, 333, 100, torch.bfloat16),      # short window, d = 64
    (2, 4, 2, 8, 32, 200, 64, torch.float32),          # fp32 path
    (1, 6, 2, 96, 128, 1000, 97, torch.bfloat16),      # budget one above the window
    (2, 8, 2, 64, 128, 500, 600, torch.bfloat16),      # N <= M: nothing evicted
]


@pytest.mark.parametrize("reduce", [orc.REDUCE_MAX, orc.REDUCE_SUM], ids=["max", "sum"])
@pytest.mark.parametrize("case", SNAPKV_CASES, ids=[f"N{c[5]}_M{c[6]}_w{c[3]}_{str(c[7])[6:]}" for c in SNAPKV_CASES])
def test_snapkv_step_matches_oracle(case, reduce):
    nb, Hq, Hkv, w, d, N, M, dtype = case
    say(f"snapkv {case} reduce={reduce}")
    q, k0, v0 = _inputs(nb, Hq, Hkv, w, d, N + 5, dtype, seed=N + M)   # five spare rows that must not be touched
    k, v = k0.clone(), v0.clone()
    prm = ep.make_params(q, k, n_cached=min(M, N), n_block=N - min(M, N), budget=M, reduce=reduce)
    ws = torch.empty(max(ep.epicache_snapkv_workspace_size(prm), 256), dtype=torch.uint8, device=DEV)
    n_keep = min(M, N)
    scores = torch.full((nb, Hkv, N - w), float("nan"), dtype=torch.float32, device=DEV)
    keep = torch.full((nb, Hkv, n_keep), -1, dtype=torch.int32, device=DEV)
    ep.epicache_evict_step_snapkv(prm, q, k, v, ws, scores, keep)
    torch.cuda.synchronize()
    rtol = pu.rtol_for(dtype)
    o_s, o_idx, o_k, o_v = orc.evict_step_snapkv(synth.to_f64_numpy(q), synth.to_f64_numpy(k0), None, N, M, reduce,
                                                 k_bits=synth.raw_bits_numpy(k0), v_bits=synth.raw_bits_numpy(v0))
    pu.assert_scores_close(scores.cpu().numpy(), o_s, rtol, "snapkv scores")
    g = keep.cpu().numpy()
    pu.assert_keep_valid(g, N, n_keep, "snapkv keep")
    if N > M:
        assert (g[:, :, M - w:] == np.arange(N - w, N)).all(), "the window rows are always retained"
        differ = pu.assert_keep_matches(g[:, :, :M - w], o_s, M - w, rtol, "snapkv earlier rows")
    else:
        assert (g == np.arange(N)).all()
        differ = 0
    # compaction: the bit-exact gather of the GPU's own list; where the lists agree, the oracle's rows
    idx = keep.long().unsqueeze(-1).expand(-1, -1, -1, d)
    assert torch.equal(_bits(torch.gather(k0, 2, idx)), _bits(k[:, :, :n_keep]))
    assert torch.equal(_bits(torch.gather(v0, 2, idx)), _bits(v[:, :, :n_keep]))
    assert torch.equal(_bits(k[:, :, N:]), _bits(k0[:, :, N:])) and torch.equal(_bits(v[:, :, N:]), _bits(v0[:, :, N:]))
    if differ == 0:
        assert (g == o_idx).all()
        assert (synth.raw_bits_numpy(k[:, :, :n_keep]) == o_k).all() and (synth.raw_bits_numpy(v[:, :, :n_keep]) == o_v).all()
    # intermediates inside the workspace give the same cache
    k2, v2 = k0.clone(), v0.clone()
    ep.epicache_evict_step_snapkv(prm, q, k2, v2, ws)
    torch.cuda.synchronize()
    assert torch.equal(_bits(k2), _bits(k)) and torch.equal(_bits(v2), _bits(v))


def test_snapkv_validation():
    q, k, v = _inputs(1, 4, 2, 64, 128, 512, torch.bfloat16, seed=1)
    lib = ep.load()
    out = ctypes.c_size_t(0)
    bad = ep.make_params(q, k, n_cached=64, n_block=448, budget=64, reduce=ep.REDUCE_MAX)      # budget == window, N > M
    assert lib.epicache_snapkv_workspace_size(ctypes.byref(bad), ctypes.byref(out)) == ep.ERR_INVALID_ARG
    bad = ep.make_params(q, k, n_cached=100, n_block=348, budget=100, reduce=ep.REDUCE_MAX, causal_patch=1)
    assert lib.epicache_snapkv_workspace_size(ctypes.byref(bad), ctypes.byref(out)) == ep.ERR_INVALID_ARG
    ok = ep.make_params(q, k, n_cached=100, n_block=412, budget=100, reduce=ep.REDUCE_MAX)
    assert lib.epicache_snapkv_workspace_size(ctypes.byref(ok), ctypes.byref(out)) == ep.OK
    ws = torch.empty(out.value, dtype=torch.uint8, device=DEV)
    st = lib.epicache_evict_step_snapkv(ctypes.byref(ok), q.data_ptr(), k.data_ptr(), v.data_ptr(), None, None,
                                        ws.data_ptr(), out.value - 256, None)
    assert st == ep.ERR_WORKSPACE_TOO_SMALL


KVZIP_CASES = [
    # nb, Hq, Hkv, p, d, N, M, dtype            G * p, chunks of 4096 / G tokens
    (1, 8, 2, 4112, 128, 2048, 1024, torch.bfloat16),   # 16448 rows: beyond the limit of epicache_score; 5 chunks, ragged tail
    (2, 4, 4, 4096 + 24, 128, 700, 300, torch.bfloat16),  # G = 1: a block of 4096 tokens behind a 24-token instruction
    (1, 14, 2, 1200, 64, 900, 256, torch.bfloat16),     # G = 7: chunks of 576 tokens
    (1, 4, 2, 2500, 32, 150, 60, torch.float32),        # fp32 path, 2 chunks
    (2, 8, 2, 100, 128, 300, 100, torch.bfloat16),      # short patch: a single chunk
]


@pytest.mark.parametrize("reduce", [orc.REDUCE_MAX, orc.REDUCE_SUM], ids=["max", "sum"])
@pytest.mark.parametrize("case", KVZIP_CASES, ids=[f"p{c[3]}_G{c[1] // c[2]}_N{c[5]}_{str(c[7])[6:]}" for c in KVZIP_CASES])
def test_kvzip_long_patch_matches_oracle(case, reduce):
    nb, Hq, Hkv, p, d, N, M, dtype = case
    say(f"kvzip {case} reduce={reduce}")
    q, k0, v0 = _inputs(nb, Hq, Hkv, p, d, N + 3, dtype, seed=p + N)
    prm = ep.make_params(q, k0, n_cached=M, n_block=N - M, budget=M, reduce=reduce)
    ws = torch.empty(max(ep.epicache_kvzip_workspace_size(prm), 256), dtype=torch.uint8, device=DEV)
    rtol = pu.rtol_for(dtype)
    o = orc.score(synth.to_f64_numpy(q), synth.to_f64_numpy(k0), N, reduce)
    # scores alone
    scores = torch.full((nb, Hkv, N), float("nan"), dtype=torch.float32, device=DEV)
    ep.epicache_score_kvzip(prm, q, k0, scores, ws)
    torch.cuda.synchronize()
    pu.assert_scores_close(scores.cpu().numpy(), o, rtol, "kvzip scores")
    if (Hq // Hkv) * p <= 16384:   # where the plain call accepts the patch too, the two are the same up to the chunk order
        plain = torch.empty_like(scores)
        ep.epicache_score(prm, q, k0, plain, ep.alloc_workspace(prm))
        torch.cuda.synchronize()
        torch.testing.assert_close(scores, plain, rtol=1e-5, atol=1e-30)
    # the whole step
    k, v = k0.clone(), v0.clone()
    scores2 = torch.full_like(scores, float("nan"))
    keep = torch.full((nb, Hkv, M), -1, dtype=torch.int32, device=DEV)
    ep.epicache_evict_step_kvzip(prm, q, k, v, ws, scores2, keep)
    torch.cuda.synchronize()
    assert torch.equal(scores2.view(torch.int32), scores.view(torch.int32))
    differ = pu.assert_keep_matches(keep.cpu().numpy(), o, M, rtol, "kvzip keep")
    idx = keep.long().unsqueeze(-1).expand(-1, -1, -1, d)
    assert torch.equal(_bits(torch.gather(k0, 2, idx)), _bits(k[:, :, :M]))
    assert torch.equal(_bits(torch.gather(v0, 2, idx)), _bits(v[:, :, :M]))
    if differ == 0:
        assert (synth.raw_bits_numpy(k[:, :, :M]) == orc.compact(synth.raw_bits_numpy(k0), keep.cpu().numpy())).all()
    k2, v2 = k0.clone(), v0.clone()
    ep.epicache_evict_step_kvzip(prm, q, k2, v2, ws)       # intermediates inside the workspace
    torch.cuda.synchronize()
    assert torch.equal(_bits(k2), _bits(k)) and torch.equal(_bits(v2), _bits(v))


def test_kvzip_validation():
    q, k, v = _inputs(1, 8, 2, 5000, 128, 256, torch.bfloat16, seed=2)
    lib = ep.load()
    out = ctypes.c_size_t(0)
    prm = ep.make_params(q, k, n_cached=128, n_block=128, budget=128, reduce=ep.REDUCE_SUM)
    assert lib.epicache_workspace_size(ctypes.byref(prm), ctypes.byref(out)) == ep.ERR_UNSUPPORTED   # 20000 rows
    assert lib.epicache_kvzip_workspace_size(ctypes.byref(prm), ctypes.byref(out)) == ep.OK
    prm.causal_patch = 1
    assert lib.epicache_kvzip_workspace_size(ctypes.byref(prm), ctypes.byref(out)) == ep.ERR_INVALID_ARG
    prm.causal_patch = 0
    prm.q_stride_h = 4000 * 128                                                     # does not hold 5000 tokens
    assert lib.epicache_kvzip_workspace_size(ctypes.byref(prm), ctypes.byref(out)) == ep.ERR_INVALID_ARG
