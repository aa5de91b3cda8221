"""epicache_evict_step_overlapped: the step as a two-stream pipeline over chunks of the batch (scoring of chunk
c + 1 beside the selection and compaction of chunk c).  Every chunking must give what the oracle gives:
scores elementwise, kept sets by the band rule, K/V the bit-exact gather of the kept rows; and what follows the
call on the caller's stream must see the finished caches."""
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


CASES = [
    # nb, Hq, Hkv, p, d, N, M, dtype, n_chunks asked, chunks expected
    (6, 8, 2, 64, 128, 700, 300, torch.bfloat16, 4, 3),      # 4 asked -> chunks of 2 items -> 3 chunks
    (7, 8, 2, 40, 128, 515, 200, torch.bfloat16, 3, 3),      # tail chunk of a single item, ragged last key tile
    (5, 4, 4, 16, 64, 333, 111, torch.bfloat16, 32, 5),      # more chunks asked than items: one item each
    (4, 4, 2, 8, 32, 200, 64, torch.float32, 2, 2),          # fp32 path
    (3, 8, 2, 64, 128, 600, 256, torch.bfloat16, 1, 1),      # one chunk: the plain step
    (64, 16, 4, 64, 128, 512, 256, torch.bfloat16, 0, 1),    # library's choice: 256 heads of 256 rows, but too little work to cut
    (64, 16, 4, 64, 128, 512, 256, torch.bfloat16, 2, 2),    # the same in two chunks of 32 items
    (8, 6, 2, 64, 128, 512, 256, torch.bfloat16, 0, 1),      # library's choice: 192 scoring rows -> plain step
    (4, 8, 2, 64, 128, 256, 300, torch.bfloat16, 2, 2),      # N <= M: nothing evicted
]


@pytest.mark.parametrize("reduce", [orc.REDUCE_MAX, orc.REDUCE_SUM], ids=["max", "sum"])
@pytest.mark.parametrize("case", CASES, ids=[f"nb{c[0]}_R{c[1] // c[2] * c[3]}_N{c[5]}_M{c[6]}_{str(c[7])[6:]}_c{c[8]}"
                                             for c in CASES])
def test_overlapped_step_matches_oracle(case, reduce):
    nb, Hq, Hkv, p, d, N, M, dtype, asked, expected = case
    say(f"overlapped {case} reduce={reduce}")
    q, k0, v0 = _inputs(nb, Hq, Hkv, p, d, N + 3, dtype, seed=1000 * nb + N)
    n_cached = min(M, N)
    prm = ep.make_params(q, k0, n_cached=n_cached, n_block=N - n_cached, budget=M, reduce=reduce)
    nbytes, used = ep.epicache_overlapped_workspace_size(prm, asked)
    assert used == expected
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV)
    n_keep = min(M, N)
    aux = torch.cuda.Stream()
    rtol = pu.rtol_for(dtype)
    o_s = orc.score(synth.to_f64_numpy(q), synth.to_f64_numpy(k0), N, reduce)

    k, v = k0.clone(), v0.clone()
    scores = torch.full((nb, Hkv, N), float("nan"), dtype=torch.float32, device=DEV)
    keep = torch.full((nb, Hkv, n_keep), -1, dtype=torch.int32, device=DEV)
    ep.epicache_evict_step_overlapped(prm, q, k, v, ws, aux, asked, scores, keep)
    # no synchronisation: these copies are enqueued on the caller's stream and must see the finished step
    k_after, v_after = k.clone(), v.clone()
    torch.cuda.synchronize()
    pu.assert_scores_close(scores.cpu().numpy(), o_s, rtol, "overlapped scores")
    g = keep.cpu().numpy()
    if N > M:
        differ = pu.assert_keep_matches(g, o_s, M, rtol, "overlapped keep")
        idx = keep.long().unsqueeze(-1).expand(-1, -1, -1, d)
        assert torch.equal(_bits(torch.gather(k0, 2, idx)), _bits(k_after[:, :, :n_keep]))
        assert torch.equal(_bits(torch.gather(v0, 2, idx)), _bits(v_after[:, :, :n_keep]))
        assert torch.equal(_bits(k_after[:, :, N:]), _bits(k0[:, :, N:]))      # spare rows untouched
        if differ == 0:
            assert (synth.raw_bits_numpy(k_after[:, :, :n_keep]) == orc.compact(synth.raw_bits_numpy(k0), g)).all()
            assert (synth.raw_bits_numpy(v_after[:, :, :n_keep]) == orc.compact(synth.raw_bits_numpy(v0), g)).all()
    else:
        assert (g == np.arange(N)).all()
        assert torch.equal(_bits(k_after), _bits(k0)) and torch.equal(_bits(v_after), _bits(v0))

    # against the plain step: the same scores up to the order of pass 1's key splits, the same caches where the kept
    # sets agree; intermediates inside the workspace and the compactions on the caller's own stream change nothing
    k1, v1 = k0.clone(), v0.clone()
    s1 = torch.empty_like(scores)
    i1 = torch.empty_like(keep)
    ep.epicache_evict_step(prm, q, k1, v1, ep.alloc_workspace(prm), s1, i1)
    k2, v2 = k0.clone(), v0.clone()
    ep.epicache_evict_step_overlapped(prm, q, k2, v2, ws, aux, asked)
    k3, v3 = k0.clone(), v0.clone()
    ep.epicache_evict_step_overlapped(prm, q, k3, v3, ws, torch.cuda.current_stream(), asked)
    torch.cuda.synchronize()
    torch.testing.assert_close(scores, s1, rtol=1e-5, atol=1e-30)
    if torch.equal(keep, i1):
        assert torch.equal(_bits(k_after[:, :, :n_keep]), _bits(k1[:, :, :n_keep]))
        assert torch.equal(_bits(v_after[:, :, :n_keep]), _bits(v1[:, :, :n_keep]))
    for kk, vv in ((k2, v2), (k3, v3)):
        assert torch.equal(_bits(kk[:, :, :n_keep]), _bits(k_after[:, :, :n_keep]))
        assert torch.equal(_bits(vv[:, :, :n_keep]), _bits(v_after[:, :, :n_keep]))


@pytest.mark.parametrize("reduce", [orc.REDUCE_MAX, orc.REDUCE_SUM], ids=["max", "sum"])
def test_overlapped_step_with_supplied_normalisers(reduce):
    """row_lse_opt: the scoring of every chunk is the single pass of epicache_score_lse on that chunk's slice of the
    caller's normalisers.  With normalisers taken over the context keys the result is Eq. 1 itself (the oracle's plain
    score); the caches must be those of epicache_evict_step_lse bit for bit (the single pass has no key splits)."""
    nb, Hq, Hkv, p, d, N, M = 7, 8, 2, 40, 128, 700, 256
    say(f"overlapped with row_lse, 3 chunks, reduce={reduce}")
    q, k0, v0 = _inputs(nb, Hq, Hkv, p, d, N, torch.bfloat16, seed=4242)
    prm = ep.make_params(q, k0, n_cached=M, n_block=N - M, budget=M, reduce=reduce)
    qq, kk = synth.to_f64_numpy(q), synth.to_f64_numpy(k0)
    G = Hq // Hkv
    z = np.einsum("bhgtd,bhnd->bhgtn", qq.reshape(nb, Hkv, G, p, d), kk) / np.sqrt(d)
    zmax = z.max(axis=-1, keepdims=True)
    lse_np = (zmax[..., 0] + np.log(np.exp(z - zmax).sum(axis=-1))).reshape(nb, Hq, p)   # natural log-sum-exp per row
    lse = torch.from_numpy(lse_np.astype(np.float32)).to(DEV)
    o_s = orc.score(qq, kk, N, reduce)
    nbytes, used = ep.epicache_overlapped_workspace_size(prm, 3, with_row_lse=True)
    assert used == 3
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    k, v = k0.clone(), v0.clone()
    scores = torch.full((nb, Hkv, N), float("nan"), dtype=torch.float32, device=DEV)
    keep = torch.full((nb, Hkv, M), -1, dtype=torch.int32, device=DEV)
    ep.epicache_evict_step_overlapped(prm, q, k, v, ws, torch.cuda.Stream(), 3, scores, keep, row_lse=lse)
    k1, v1 = k0.clone(), v0.clone()
    s1, i1 = torch.empty_like(scores), torch.empty_like(keep)
    ep.epicache_evict_step_lse(prm, q, k1, v1, lse, ep.alloc_workspace(prm), s1, i1)
    torch.cuda.synchronize()
    rtol = pu.rtol_for(torch.bfloat16)
    pu.assert_scores_close(scores.cpu().numpy(), o_s, rtol, "overlapped lse scores")
    pu.assert_keep_matches(keep.cpu().numpy(), o_s, M, rtol, "overlapped lse keep")
    assert torch.equal(scores.view(torch.int32), s1.view(torch.int32)) and torch.equal(keep, i1)
    assert torch.equal(_bits(k[:, :, :M]), _bits(k1[:, :, :M])) and torch.equal(_bits(v[:, :, :M]), _bits(v1[:, :, :M]))


def test_overlapped_calls_back_to_back_share_the_event_pool():
    """Three steps of a cache enqueued without a host synchronisation in between (each appends a block to what the
    previous one kept), the same sequence through the plain step: the events of one call are reused by the next
    while it may still be running."""
    nb, Hq, Hkv, p, d, M, B = 6, 8, 2, 64, 128, 256, 256
    say("overlapped: three dependent steps back to back")
    q, k0, v0 = _inputs(nb, Hq, Hkv, p, d, M + B, torch.bfloat16, seed=77)
    blocks = [_inputs(nb, Hq, Hkv, p, d, B, torch.bfloat16, seed=78 + i) for i in range(3)]
    prm = ep.make_params(q, k0, n_cached=M, n_block=B, budget=M, reduce=ep.REDUCE_SUM)
    aux = torch.cuda.Stream()
    nbytes, used = ep.epicache_overlapped_workspace_size(prm, 3)
    assert used == 3
    ws_o = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    ws_p = ep.alloc_workspace(prm)
    results = []
    for overlapped in (False, True):
        k, v = k0.clone(), v0.clone()
        for qb, kb, vb in blocks:
            k[:, :, M:] = kb
            v[:, :, M:] = vb
            if overlapped:
                ep.epicache_evict_step_overlapped(prm, qb, k, v, ws_o, aux, 3)
            else:
                ep.epicache_evict_step(prm, qb, k, v, ws_p)
        torch.cuda.synchronize()
        results.append((k[:, :, :M].clone(), v[:, :, :M].clone()))
    # chunks of 2 items and the whole batch of 6 get the same key splits here (so few workgroups that both take
    # the most splits N = 512 allows), so the scores, and with them the caches, are identical bit for bit
    assert torch.equal(_bits(results[0][0]), _bits(results[1][0]))
    assert torch.equal(_bits(results[0][1]), _bits(results[1][1]))


def test_overlapped_validation():
    q, k, v = _inputs(4, 8, 2, 64, 128, 512, torch.bfloat16, seed=5)
    lib = ep.load()
    prm = ep.make_params(q, k, n_cached=256, n_block=256, budget=256, reduce=ep.REDUCE_SUM)
    out, used = ctypes.c_size_t(0), ctypes.c_int32(0)
    for bad in (-1, 65):
        assert lib.epicache_overlapped_workspace_size(ctypes.byref(prm), bad, 0, ctypes.byref(out),
                                                      ctypes.byref(used)) == ep.ERR_INVALID_ARG
    assert lib.epicache_overlapped_workspace_size(ctypes.byref(prm), 2, 0, ctypes.byref(out), ctypes.byref(used)) == ep.OK
    ws = torch.empty(out.value, dtype=torch.uint8, device=DEV)
    aux = torch.cuda.Stream()
    st = lib.epicache_evict_step_overlapped(ctypes.byref(prm), q.data_ptr(), k.data_ptr(), v.data_ptr(), None, None, None,
                                            2, ws.data_ptr(), out.value - 256, None, ctypes.c_void_p(aux.cuda_stream))
    assert st == ep.ERR_WORKSPACE_TOO_SMALL
    st = lib.epicache_evict_step_overlapped(ctypes.byref(prm), q.data_ptr(), k.data_ptr(), k.data_ptr(), None, None, None,
                                            2, ws.data_ptr(), out.value, None, ctypes.c_void_p(aux.cuda_stream))
    assert st == ep.ERR_INVALID_ARG     # K and V must be distinct buffers
    lse = torch.zeros(4, 8, 64, dtype=torch.float32, device=DEV)
    prm.causal_patch = 1                # a supplied normaliser already fixes the denominator
    st = lib.epicache_evict_step_overlapped(ctypes.byref(prm), q.data_ptr(), k.data_ptr(), v.data_ptr(), lse.data_ptr(),
                                            None, None, 2, ws.data_ptr(), out.value, None,
                                            ctypes.c_void_p(aux.cuda_stream))
    assert st == ep.ERR_INVALID_ARG
    torch.cuda.synchronize()
