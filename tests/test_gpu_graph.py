"""The library only enqueues kernels (no allocation, no memset, no host synchronisation), so a whole
eviction step can be captured into a HIP graph and replayed, as a serving loop would do.  Every replay
is checked against the eager result, with eager work and synchronisations between the replays."""
import sys

import pytest
import torch

from paper_2509_17396_amd import binding as ep
from paper_2509_17396_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("ragged,overlapped", [(False, False), (True, False), (False, True)],
                         ids=["uniform", "ragged_pooled", "overlapped_two_streams"])
def test_evict_step_replays_from_a_graph(ragged, overlapped):
    """overlapped: epicache_evict_step_overlapped in two chunks; its second stream joins the capture through the
    chunk events (fork) and the join event, and the event pool serves eager calls again afterwards."""
    w = synth.WORKLOADS["llama32_3b"].scaled(E=4 if overlapped else 2, M=512, B=512)
    say(f"graph capture, ragged={ragged}, overlapped={overlapped}")
    inputs = [synth.make_layer(w, layer=l, device=DEV) for l in range(3)]
    q, k, v = (t.clone() for t in inputs[0])
    nb, H, N = w.E, w.Hkv, w.N
    prm = ep.make_params(q, k, n_cached=w.M, n_block=w.B, budget=w.M, reduce=ep.REDUCE_SUM)
    if ragged:
        _, cap = ep.epicache_ragged_workspace_size(prm, ep.SELECT_POOLED)
        ws = ep.alloc_ragged_workspace(prm, ep.SELECT_POOLED)
        n_ctx = torch.full((nb, H), N, dtype=torch.int32, device=DEV)
        n_ctx[0, 1], n_ctx[1, 3] = 700, 0
        n_kept = torch.zeros((nb, H), dtype=torch.int32, device=DEV)
    elif overlapped:
        cap = w.M
        nbytes, used = ep.epicache_overlapped_workspace_size(prm, 2)
        assert used == 2
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        aux = torch.cuda.Stream()
    else:
        cap = w.M
        ws = ep.alloc_workspace(prm)
    scores = torch.zeros((nb, H, N), dtype=torch.float32, device=DEV)
    keep = torch.zeros((nb, H, cap), dtype=torch.int32, device=DEV)

    def step():
        if ragged:
            ep.epicache_evict_step_ragged(prm, ep.SELECT_POOLED, q, k, v, n_ctx, None, n_kept, ws, scores, keep)
        elif overlapped:
            ep.epicache_evict_step_overlapped(prm, q, k, v, ws, aux, 2, scores, keep)
        else:
            ep.epicache_evict_step(prm, q, k, v, ws, scores, keep)

    def load(i):
        for dst, src in zip((q, k, v), inputs[i]):
            dst.copy_(src)

    # eager results for the three input sets
    want = []
    for i in range(3):
        load(i)
        step()
        torch.cuda.synchronize()
        want.append([t.clone() for t in (scores, keep, k, v)] + ([n_kept.clone()] if ragged else []))

    load(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for i in (1, 2, 0, 1):           # replays on changing inputs, eager copies and syncs in between
        load(i)
        scores.fill_(-1.0)
        keep.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [scores, keep, k, v] + ([n_kept] if ragged else [])
        valid = None
        for g, e in zip(got, want[i]):
            if g is keep and ragged:   # entries past n_kept are not written
                pos = torch.arange(cap, device=DEV)[None, None, :]
                valid = pos < want[i][4][:, :, None]
                assert torch.equal(torch.where(valid, g, 0), torch.where(valid, e, 0)), f"replay on set {i}: keep"
            elif g is scores and ragged:
                posn = torch.arange(N, device=DEV)[None, None, :]
                m = posn < n_ctx[:, :, None]
                assert torch.equal(torch.where(m, g, 0), torch.where(m, e, 0)), f"replay on set {i}: scores"
            else:
                assert torch.equal(g.view(torch.uint8) if g.dtype == torch.bfloat16 else g,
                                   e.view(torch.uint8) if e.dtype == torch.bfloat16 else e), f"replay on set {i}"
    if overlapped:   # an eager call after the capture: the same events, recorded outside a capture again
        load(2)
        step()
        torch.cuda.synchronize()
        assert torch.equal(k.view(torch.uint8), want[2][2].view(torch.uint8))
