"""epicache_evict_step_static: the entry point for callers that cannot allocate.  Its workspace is an
array inside the library's code object; everything else is epicache_evict_step, so every output must be
bit-identical to that call's on the same inputs.  Two calls in a row share the array, the second with a
smaller input, and a request beyond the array's size is refused before anything is enqueued."""
import ctypes
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


def both_ways(w, reduce, layer, with_outputs):
    q, k0, v0 = synth.make_layer(w, layer=layer, device=DEV)
    prm = ep.make_params(q, k0, n_cached=w.M, n_block=w.B, budget=w.M, reduce=reduce)
    n_keep = min(w.M, w.N)
    out = []
    for static in (False, True):
        k, v = k0.clone(), v0.clone()
        scores = torch.full((w.E, w.Hkv, w.N), float("nan"), dtype=torch.float32, device=DEV) if with_outputs else None
        keep = torch.full((w.E, w.Hkv, n_keep), -1, dtype=torch.int32, device=DEV) if with_outputs else None
        if static:
            ep.epicache_evict_step_static(prm, q, k, v, scores, keep)
        else:
            ws = ep.alloc_workspace(prm)
            ep.epicache_evict_step(prm, q, k, v, ws, scores, keep)
        torch.cuda.synchronize()
        out.append((k, v, scores, keep))
    (k_a, v_a, s_a, i_a), (k_b, v_b, s_b, i_b) = out
    assert torch.equal(k_a[:, :, :n_keep].view(torch.int16), k_b[:, :, :n_keep].view(torch.int16))
    assert torch.equal(v_a[:, :, :n_keep].view(torch.int16), v_b[:, :, :n_keep].view(torch.int16))
    assert not torch.equal(k_a[:, :, :n_keep], k0[:, :, :n_keep])  # the step did move rows
    if with_outputs:
        assert torch.equal(s_a.view(torch.int32), s_b.view(torch.int32))
        assert torch.equal(i_a, i_b)


@pytest.mark.parametrize("reduce", [ep.REDUCE_SUM, ep.REDUCE_MAX], ids=["sum", "max"])
def test_static_scratch_step_equals_workspace_step_twice_in_a_row(reduce):
    big = synth.WORKLOADS["llama32_3b"].scaled(E=3, M=1024, B=1024)
    small = synth.WORKLOADS["llama32_3b"].scaled(E=1, M=300, B=212, p=40)
    say(f"static scratch, first call E={big.E} N={big.N}, reduce={reduce}")
    both_ways(big, reduce, layer=0, with_outputs=True)
    say(f"static scratch, second call on the same array, smaller: E={small.E} N={small.N}")
    both_ways(small, reduce, layer=1, with_outputs=True)
    say("static scratch, intermediates inside the array")
    both_ways(small, reduce, layer=2, with_outputs=False)
    both_ways(big, reduce, layer=3, with_outputs=False)


def test_static_scratch_rejects_what_does_not_fit():
    """Validation only: nothing is enqueued, so the pointers are never touched."""
    q = torch.empty(64, 32, 256, 128, dtype=torch.bfloat16, device="meta")
    k = torch.empty(64, 8, 24576, 128, dtype=torch.bfloat16, device="meta")
    prm = ep.make_params(q, k, n_cached=16384, n_block=8192, budget=16384, reduce=ep.REDUCE_SUM)
    assert ep.epicache_workspace_size(prm) > ep.STATIC_SCRATCH_BYTES
    dummy = ctypes.c_void_p(4096)
    st = ep.load().epicache_evict_step_static(ctypes.byref(prm), dummy, dummy, ctypes.c_void_p(8192), None, None, None)
    assert st == ep.ERR_WORKSPACE_TOO_SMALL
