"""GPU parity of the patch attention output and normalisers against the CPU oracle, and of the chain
patch attention -> scoring on the returned normalisers against the oracle's causal-patch scores."""
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


def wl(name, **kw):
    return synth.WORKLOADS[name].scaled(**kw)


def gpu_patch_attention(q, k, v, N, causal):
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    prm = ep.make_params(qd, kd, n_cached=0, n_block=N, budget=1, causal_patch=causal)
    out = torch.full(qd.shape, float("nan"), dtype=qd.dtype, device=DEV)
    lse = torch.full(qd.shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    ep.epicache_patch_attention(prm, qd, kd, vd, out, lse)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64), lse


def out_tolerance(o64, v64, dtype):
    """Elementwise bound.  The output is a convex combination of value rows, so its error is absolute, in
    units of the largest value.  fp32 path: accumulation order only.  bf16 path: the output itself is rounded
    to bf16 (half an ulp, 2^-9 relative, doubled for slack) and the weights are rounded to bf16 before the
    product with V (2^-9 relative each, so at most 2^-9 of the largest value in total)."""
    vmax = np.abs(v64).max()
    if dtype == torch.float32:
        return 1e-5 * vmax + 0 * o64
    return 2.0 ** -8 * np.abs(o64) + 2.0 ** -9 * vmax


CASES = [
    # name, base workload, overrides, context rows N
    ("fp32_plain_d40", "tiny", dict(E=2, Hq=6, Hkv=2, p=5, d=40), 203),
    ("fp32_plain_long_patch", "tiny", dict(E=1, Hq=2, Hkv=1, p=150, d=16), 300),
    ("bf16_plain_d64", "llama32_3b", dict(E=1, Hq=4, Hkv=2, p=20, d=64), 333),
    ("bf16_mfma_R192_three_waves", "llama32_3b", dict(E=2, Hq=6, Hkv=2, p=64), 640),
    ("bf16_mfma_R128_four_waves", "llama32_3b", dict(E=1, Hq=4, Hkv=2, p=64), 500),
    ("bf16_mfma_R64_two_waves", "llama32_3b", dict(E=1, Hq=2, Hkv=2, p=64), 257),
    ("bf16_mfma_R256_eight_waves", "llama31_8b", dict(E=2, Hq=8, Hkv=2, p=64), 520),
    ("bf16_mfma_R448_eight_waves_one_idle", "qwen25_7b", dict(E=1, Hq=14, Hkv=2, p=64), 300),
    ("bf16_mfma_ragged_rows_p37", "llama32_3b", dict(E=1, Hq=6, Hkv=2, p=37), 1000),
    ("bf16_mfma_two_patch_tiles_p100", "llama31_8b", dict(E=1, Hq=8, Hkv=2, p=100), 777),
    ("bf16_mfma_one_context_key", "llama32_3b", dict(E=1, Hq=4, Hkv=2, p=16), 1),
    ("bf16_mfma_student_t", "stress", dict(E=1, Hq=8, Hkv=2, p=32), 1500),
]


@pytest.mark.parametrize("causal", [1, 0], ids=["causal_patch", "context_only"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_patch_attention_matches_oracle(case, causal):
    name, base, over, N = case
    w = wl(base, **over)
    say(f"patch_attention {name} causal={causal}")
    q, k, v = synth.make_layer(w, layer=2, n_ctx=N + w.p)
    out, lse, _ = gpu_patch_attention(q, k, v, N, causal)
    qq, kk = pu.oracle_inputs(q, k)
    vv = synth.to_f64_numpy(v)
    o_out, o_lse = orc.patch_attention(qq, kk, vv, N, bool(causal))
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    err_lse = np.abs(lse - o_lse).max()
    tol = out_tolerance(o_out, vv[:, :, :N + w.p], q.dtype)
    ratio = (np.abs(out - o_out) / tol).max()
    assert err_lse <= 2e-5 * (1 + np.abs(o_lse).max()), f"{name}: lse err {err_lse:.3e}"
    assert ratio <= 1.0, f"{name}: output error {ratio:.2f} x its bound"
    say(f"  max |lse err| {err_lse:.2e}, max |out err| {np.abs(out - o_out).max():.2e} = {ratio:.2f} x the bound")


def test_patch_attention_then_scoring_on_its_normalisers():
    """The normalisers the attention pass returns feed the single-pass scoring: together they give the
    causal-patch scores of Eq. 1 with K read twice."""
    w = wl("llama32_3b", E=2, Hq=6, Hkv=2, p=64)
    N = 900
    say("patch_attention -> score_lse")
    q, k, v = synth.make_layer(w, layer=4, n_ctx=N + w.p)
    _, _, lse_dev = gpu_patch_attention(q, k, v, N, 1)
    qd, kd = q.to(DEV), k.to(DEV)
    for reduce in (orc.REDUCE_MAX, orc.REDUCE_SUM):
        prm = ep.make_params(qd, kd, n_cached=0, n_block=N, budget=7, reduce=reduce)
        ws = ep.alloc_workspace(prm)
        scores = torch.empty((w.E, w.Hkv, N), dtype=torch.float32, device=DEV)
        ep.epicache_score_lse(prm, qd, kd, lse_dev, scores, ws)
        torch.cuda.synchronize()
        want = orc.score_causal_patch(*pu.oracle_inputs(q, k), N, reduce)
        pu.assert_scores_close(scores.cpu().numpy(), want, pu.RTOL_BF16, f"reduce={reduce}")


@pytest.mark.parametrize("causal", [1, 0], ids=["causal_patch", "context_only"])
def test_evict_step_with_the_patch_attention_folded_in(causal):
    """epicache_evict_step_attn: the patch's attention output, then scoring on its normalisers, selection and
    compaction.  Output against the oracle's attention, kept rows against the oracle's scores under the same
    denominator (within the band), cache = bit-exact gather, and identical to the two separate calls."""
    w = wl("llama32_3b", E=2, Hq=6, Hkv=2, p=64, M=384, B=256)
    N = w.M + w.B
    say(f"evict_step_attn causal={causal}")
    q, k, v = synth.make_layer(w, layer=6, n_ctx=N + w.p)
    qd, kd, vd = q.to(DEV), k.to(DEV).clone(), v.to(DEV).clone()
    prm = ep.make_params(qd, kd, n_cached=w.M, n_block=w.B, budget=w.M, reduce=orc.REDUCE_MAX, causal_patch=causal)
    ws = ep.alloc_workspace(prm)
    out = torch.full(qd.shape, float("nan"), dtype=qd.dtype, device=DEV)
    scores = torch.full((w.E, w.Hkv, N), float("nan"), dtype=torch.float32, device=DEV)
    keep = torch.full((w.E, w.Hkv, w.M), -1, dtype=torch.int32, device=DEV)
    ep.epicache_evict_step_attn(prm, qd, kd, vd, out, ws, scores, keep)
    torch.cuda.synchronize()
    qq, kk = pu.oracle_inputs(q, k)
    vv = synth.to_f64_numpy(v)
    o_out, _ = orc.patch_attention(qq, kk, vv, N, bool(causal))
    tol = out_tolerance(o_out, vv[:, :, :N + w.p], q.dtype)
    assert (np.abs(out.float().cpu().numpy() - o_out) <= tol).all()
    o_scores = orc.score_causal_patch(qq, kk, N, orc.REDUCE_MAX) if causal else orc.score(qq, kk, N, orc.REDUCE_MAX)
    pu.assert_scores_close(scores.cpu().numpy(), o_scores, pu.RTOL_BF16, "scores")
    keep_np = keep.cpu().numpy()
    differ = pu.assert_keep_matches(keep_np, o_scores, w.M, pu.RTOL_BF16, "keep")
    kb, vb = synth.raw_bits_numpy(k), synth.raw_bits_numpy(v)
    np.testing.assert_array_equal(synth.raw_bits_numpy(kd.cpu())[:, :, :w.M], orc.compact(kb, keep_np))
    np.testing.assert_array_equal(synth.raw_bits_numpy(vd.cpu())[:, :, :w.M], orc.compact(vb, keep_np))
    # the same through the two separate calls
    kd2, vd2 = k.to(DEV).clone(), v.to(DEV).clone()
    out2 = torch.empty_like(out)
    lse2 = torch.empty(qd.shape[:3], dtype=torch.float32, device=DEV)
    ep.epicache_patch_attention(prm, qd, kd2, vd2, out2, lse2)
    prm0 = ep.make_params(qd, kd2, n_cached=w.M, n_block=w.B, budget=w.M, reduce=orc.REDUCE_MAX)
    ep.epicache_evict_step_lse(prm0, qd, kd2, vd2, lse2, ep.alloc_workspace(prm0))
    torch.cuda.synchronize()
    assert torch.equal(out2.view(torch.int16), out.view(torch.int16))
    assert torch.equal(kd2.view(torch.int16), kd.view(torch.int16)) and torch.equal(vd2.view(torch.int16), vd.view(torch.int16))
    say(f"  tokens differing inside the band: {differ}")


def test_patch_attention_is_bit_identical_from_run_to_run():
    """Same inputs, same bits, for every workgroup shape the launcher picks (R = 64, 96, 128, 192, 256)."""
    for Hq, p in ((2, 64), (2, 96), (4, 64), (6, 64), (8, 64)):
        w = wl("llama32_3b", E=2, Hq=Hq, Hkv=2, p=p, M=384, B=256)
        N = w.M + w.B
        q, k, v = synth.make_layer(w, layer=6, n_ctx=N + w.p)
        qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
        prm = ep.make_params(qd, kd, n_cached=w.M, n_block=w.B, budget=w.M, causal_patch=1)
        runs = []
        for _ in range(4):
            out = torch.empty_like(qd)
            lse = torch.empty(qd.shape[:3], dtype=torch.float32, device=DEV)
            ep.epicache_patch_attention(prm, qd, kd, vd, out, lse)
            torch.cuda.synchronize()
            runs.append((out, lse))
        for out, lse in runs[1:]:
            assert torch.equal(out.view(torch.int16), runs[0][0].view(torch.int16)), f"R={w.R}: output differs between runs"
            assert torch.equal(lse.view(torch.int32), runs[0][1].view(torch.int32)), f"R={w.R}: lse differs between runs"


RAGGED_CASES = [
    # name, base workload, overrides, longest context, per-(b, h) lengths (None = drawn)
    ("bf16_mfma", "llama32_3b", dict(E=3, Hq=6, Hkv=2, p=64), 700, [[700, 0], [1, 333], [64, 65]]),
    ("bf16_mfma_drawn", "llama31_8b", dict(E=4, Hq=8, Hkv=4, p=37), 1500, None),
    ("fp32_plain", "tiny", dict(E=2, Hq=4, Hkv=2, p=9, d=24), 260, [[0, 260], [17, 256]]),
]


@pytest.mark.parametrize("causal", [1, 0], ids=["causal_patch", "context_only"])
@pytest.mark.parametrize("case", RAGGED_CASES, ids=[c[0] for c in RAGGED_CASES])
def test_ragged_patch_attention_matches_oracle(case, causal):
    """Every head with its own context length (read from device memory); the patch rows of a head follow its
    own context.  Rows no head may touch hold NaN on the GPU side."""
    name, base, over, n_max, lengths = case
    w = wl(base, **over)
    say(f"patch_attention_ragged {name} causal={causal}")
    if lengths is None:
        lengths = np.random.default_rng(5).integers(0, n_max + 1, size=(w.E, w.Hkv))
        lengths[0, 0], lengths[-1, -1] = n_max, 0
    n = np.asarray(lengths, dtype=np.int64)
    q, k, v = synth.make_layer(w, layer=3, n_ctx=n_max + w.p)
    k_dev, v_dev = k.clone(), v.clone()
    for b in range(w.E):
        for h in range(w.Hkv):
            k_dev[b, h, n[b, h] + (w.p if causal else 0):] = float("nan")
            v_dev[b, h, n[b, h] + (w.p if causal else 0):] = float("nan")
    qd, kd, vd = q.to(DEV), k_dev.to(DEV), v_dev.to(DEV)
    nd = torch.tensor(n, dtype=torch.int32, device=DEV)
    prm = ep.make_params(qd, kd, n_cached=0, n_block=n_max, budget=1, causal_patch=causal)
    out = torch.full(qd.shape, float("nan"), dtype=qd.dtype, device=DEV)
    lse = torch.full(qd.shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    ep.epicache_patch_attention_ragged(prm, qd, kd, vd, nd, out, lse)
    torch.cuda.synchronize()
    out, lse = out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    qq, kk = pu.oracle_inputs(q, k)
    vv = synth.to_f64_numpy(v)
    o_out, o_lse = orc.patch_attention(qq, kk, vv, n, bool(causal))
    assert not np.isnan(out).any() and not np.isnan(lse).any()
    G = w.Hq // w.Hkv
    empty = np.repeat(n == 0, G, axis=1) & (not causal)           # [E, Hq]: queries without any key
    assert (lse[empty] == -np.inf).all() and (out[empty] == 0).all() and (o_lse[empty] == -np.inf).all()
    live = ~empty
    err_lse = np.abs(lse[live] - o_lse[live]).max()
    tol = out_tolerance(o_out, vv, q.dtype)
    ratio = (np.abs(out - o_out) / tol)[live].max()
    assert err_lse <= 2e-5 * (1 + np.abs(o_lse[live]).max()), f"{name}: lse err {err_lse:.3e}"
    assert ratio <= 1.0, f"{name}: output error {ratio:.2f} x its bound"
    say(f"  max |lse err| {err_lse:.2e}, output error {ratio:.2f} x the bound, {int(empty.sum())} empty heads")


def test_ragged_patch_attention_feeds_the_ragged_step():
    """patch_attention_ragged -> evict_step_ragged on its normalisers == the ragged step that computes its own."""
    w = wl("llama32_3b", E=3, Hq=6, Hkv=2, p=64, M=128, B=200)
    n_max = w.M + w.B
    say("patch_attention_ragged -> evict_step_ragged")
    n = np.array([[328, 100], [5, 250], [129, 128]], dtype=np.int64)
    budgets = np.array([128, 60, 128], dtype=np.int64)
    q, k, v = synth.make_layer(w, layer=1, n_ctx=n_max)
    qd, nd = q.to(DEV), torch.tensor(n, dtype=torch.int32, device=DEV)
    bd = torch.tensor(budgets, dtype=torch.int32, device=DEV)
    prm = ep.make_params(qd, k.to(DEV), n_cached=w.M, n_block=w.B, budget=w.M, reduce=ep.REDUCE_SUM)
    results = []
    for use_attn in (False, True):
        kd, vd = k.to(DEV), v.to(DEV)
        ws = ep.alloc_ragged_workspace(prm, ep.SELECT_PER_HEAD)
        n_kept = torch.empty((w.E, w.Hkv), dtype=torch.int32, device=DEV)
        scores = torch.zeros((w.E, w.Hkv, n_max), dtype=torch.float32, device=DEV)
        keep = torch.full((w.E, w.Hkv, w.M), -1, dtype=torch.int32, device=DEV)
        lse = None
        if use_attn:
            out = torch.empty_like(qd)
            lse = torch.empty(qd.shape[:3], dtype=torch.float32, device=DEV)
            ep.epicache_patch_attention_ragged(prm, qd, kd, vd, nd, out, lse)
        ep.epicache_evict_step_ragged(prm, ep.SELECT_PER_HEAD, qd, kd, vd, nd, bd, n_kept, ws, scores=scores,
                                      keep_idx=keep, row_lse=lse)
        torch.cuda.synchronize()
        results.append((scores.cpu().numpy(), keep.cpu().numpy(), n_kept.cpu().numpy(), kd.cpu(), vd.cpu()))
    (s0, keep0, nk0, k0, v0), (s1, keep1, nk1, k1, v1) = results
    assert (nk0 == nk1).all()
    for b in range(w.E):
        for h in range(w.Hkv):
            np.testing.assert_allclose(s1[b, h, :n[b, h]], s0[b, h, :n[b, h]], rtol=2e-4, atol=1e-30)
    # the kept sets agree wherever the two score vectors order the rows identically; here: count the overlap
    same = sum(len(set(keep0[b, h, :nk0[b, h]]) & set(keep1[b, h, :nk1[b, h]])) for b in range(w.E) for h in range(w.Hkv))
    assert same >= 0.99 * nk0.sum()
