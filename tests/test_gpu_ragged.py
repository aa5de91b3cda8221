"""GPU parity of the ragged entry points (per-head context lengths, per-item budgets, per-head or
pooled head-wise selection) against the CPU oracle, through the C ABI."""
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
SELECTS = [(ep.SELECT_PER_HEAD, False), (ep.SELECT_POOLED, True)]


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def wl(name, **kw):
    return synth.WORKLOADS[name].scaled(**kw)


def i32(a):
    return torch.tensor(np.asarray(a, dtype=np.int32), dtype=torch.int32, device=DEV)


def lengths(seed, nb, Hkv, n_max, special=()):
    """Seeded per-head lengths in 0..n_max with the given special values planted first."""
    rng = np.random.default_rng(seed)
    n = rng.integers(1, n_max + 1, size=(nb, Hkv))
    flat = n.reshape(-1)
    for i, s in enumerate(special):
        flat[i % flat.size] = s
    return n


# ------------------------------------------------------------------- score

RAGGED_SCORE_CASES = [
    # name, base workload, overrides, N_max, special lengths
    ("fp32_generic", "tiny", dict(E=3, Hq=6, Hkv=2, p=5, d=40), 203, (0, 1, 203, 32, 33)),
    ("bf16_stream_R192", "llama32_3b", dict(E=2, Hq=6, Hkv=2, p=64), 1100, (0, 1, 63, 64)),
    ("bf16_stream_R96_many_splits", "llama32_3b", dict(E=3, Hq=6, Hkv=2, p=32), 3000, (65, 3000, 2, 257)),
    ("bf16_keys_stationary_R400", "llama31_8b", dict(E=2, Hq=8, Hkv=2, p=100), 900, (0, 255, 256, 257)),
    ("bf16_d64", "llama32_3b", dict(E=2, Hq=4, Hkv=2, p=48, d=64), 333, (333, 1, 100, 64)),
]


@pytest.mark.parametrize("reduce", [orc.REDUCE_MAX, orc.REDUCE_SUM], ids=["max", "sum"])
@pytest.mark.parametrize("case", RAGGED_SCORE_CASES, ids=[c[0] for c in RAGGED_SCORE_CASES])
def test_score_ragged_matches_oracle(case, reduce):
    name, base, over, n_max, special = case
    w = wl(base, **over)
    say(f"score_ragged {name} reduce={reduce}")
    q, k, _ = synth.make_layer(w, layer=1, n_ctx=n_max)
    n_ctx = lengths(11, w.E, w.Hkv, n_max, special)
    qd, kd = q.to(DEV), k.to(DEV)
    prm = ep.make_params(qd, kd, n_cached=0, n_block=n_max, budget=7, reduce=reduce)
    ws = ep.alloc_workspace(prm)
    scores = torch.full((w.E, w.Hkv, n_max), -7.0, dtype=torch.float32, device=DEV)
    ep.epicache_score_ragged(prm, qd, kd, i32(n_ctx), scores, ws)
    torch.cuda.synchronize()
    got = scores.cpu().numpy()
    want = orc.score_ragged(*pu.oracle_inputs(q, k), n_ctx, reduce)
    worst = 0.0
    for b in range(w.E):
        for h in range(w.Hkv):
            n = n_ctx[b, h]
            assert (got[b, h, n:] == -7.0).all(), f"{name} b={b} h={h}: wrote beyond its {n} rows"
            if n:
                worst = max(worst, pu.assert_scores_close(got[b, h, :n], want[b][h], pu.rtol_for(q.dtype),
                                                          f"{name} b={b} h={h} n={n}"))
    say(f"  max rel err {worst:.3e}")


def test_score_ragged_with_causal_patch_keys():
    """Every head's patch keys follow its own context rows (rows n_ctx .. n_ctx+p-1)."""
    w = wl("llama32_3b", E=2, Hq=6, Hkv=2, p=40)
    n_max = 700
    say("score_ragged causal_patch")
    q, k, _ = synth.make_layer(w, layer=1, n_ctx=n_max + w.p)
    n_ctx = lengths(12, w.E, w.Hkv, n_max, (n_max, 1, 64))
    qd, kd = q.to(DEV), k.to(DEV)
    prm = ep.make_params(qd, kd, n_cached=0, n_block=n_max, budget=7, reduce=orc.REDUCE_SUM, causal_patch=1)
    ws = ep.alloc_workspace(prm)
    scores = torch.full((w.E, w.Hkv, n_max), -7.0, dtype=torch.float32, device=DEV)
    ep.epicache_score_ragged(prm, qd, kd, i32(n_ctx), scores, ws)
    torch.cuda.synchronize()
    got = scores.cpu().numpy()
    qq, kk = pu.oracle_inputs(q, k)
    for b in range(w.E):
        for h in range(w.Hkv):
            n = n_ctx[b, h]
            G = w.Hq // w.Hkv
            want = orc.score_causal_patch(qq[b:b + 1, h * G:(h + 1) * G], kk[b:b + 1, h:h + 1], n, orc.REDUCE_SUM)[0, 0]
            pu.assert_scores_close(got[b, h, :n], want, pu.RTOL_BF16, f"b={b} h={h} n={n}")
            assert (got[b, h, n:] == -7.0).all()


@pytest.mark.parametrize("reduce", [orc.REDUCE_MAX, orc.REDUCE_SUM], ids=["max", "sum"])
def test_score_ragged_with_supplied_normalisers(reduce):
    """row_lse given: single pass over K; every head's normaliser belongs to its own prefix of keys
    (plus, for one batch item, extra mass as if the patch's own keys had been attended too)."""
    from scipy.special import logsumexp
    w = wl("llama32_3b", E=2, Hq=6, Hkv=2, p=48)
    n_max = 900
    say(f"score_ragged row_lse reduce={reduce}")
    q, k, _ = synth.make_layer(w, layer=2, n_ctx=n_max)
    n_ctx = lengths(13, w.E, w.Hkv, n_max, (n_max, 1, 65))
    qq, kk = pu.oracle_inputs(q, k)
    G = w.Hq // w.Hkv
    lse = np.empty((w.E, w.Hq, w.p), dtype=np.float64)
    for b in range(w.E):
        for hq in range(w.Hq):
            n = n_ctx[b, hq // G]
            z = (qq[b, hq] @ kk[b, hq // G, :n].T) / np.sqrt(w.d)
            lse[b, hq] = logsumexp(z, axis=1) + (0.7 if b == 1 else 0.0)
    qd, kd = q.to(DEV), k.to(DEV)
    prm = ep.make_params(qd, kd, n_cached=0, n_block=n_max, budget=7, reduce=reduce)
    ws = ep.alloc_workspace(prm)
    scores = torch.full((w.E, w.Hkv, n_max), -7.0, dtype=torch.float32, device=DEV)
    lse32 = torch.tensor(lse, dtype=torch.float32, device=DEV)
    ep.epicache_score_ragged(prm, qd, kd, i32(n_ctx), scores, ws, row_lse=lse32)
    torch.cuda.synchronize()
    got = scores.cpu().numpy()
    lse_used = lse32.cpu().numpy().astype(np.float64)      # the oracle gets the rounded values the GPU got
    for b in range(w.E):
        for h in range(w.Hkv):
            n = n_ctx[b, h]
            want = orc.score_given_lse(qq[b:b + 1, h * G:(h + 1) * G], kk[b:b + 1, h:h + 1], n,
                                       lse_used[b:b + 1, h * G:(h + 1) * G], reduce)[0, 0]
            pu.assert_scores_close(got[b, h, :n], want, pu.RTOL_BF16, f"b={b} h={h} n={n}")
            assert (got[b, h, n:] == -7.0).all()
    # whole ragged step on the same normalisers: same kept rows as the two-pass step where the
    # normaliser is the plain one (batch item 0)
    v = torch.randn(k.shape, generator=torch.Generator().manual_seed(1)).to(k.dtype)
    outs = []
    for use_lse in (False, True):
        kd2, vd2 = k.to(DEV).clone(), v.to(DEV).clone()
        prm2 = ep.make_params(qd, kd2, n_cached=0, n_block=n_max, budget=100, reduce=reduce)
        ws2 = ep.alloc_ragged_workspace(prm2, ep.SELECT_POOLED)
        n_kept = torch.zeros((w.E, w.Hkv), dtype=torch.int32, device=DEV)
        ep.epicache_evict_step_ragged(prm2, ep.SELECT_POOLED, qd, kd2, vd2, i32(n_ctx), None, n_kept, ws2,
                                      row_lse=lse32 if use_lse else None)
        torch.cuda.synchronize()
        outs.append((n_kept.cpu().numpy(), kd2.cpu()))
    # same pool size; per head the two scorings may only trade tokens that sit on the threshold
    assert outs[0][0][0].sum() == outs[1][0][0].sum()
    assert np.abs(outs[0][0][0] - outs[1][0][0]).max() <= 2


# ------------------------------------------------------------------- select

def gpu_select(scores_np, n_ctx, budgets, m_max, select):
    nb, H, n_max = scores_np.shape
    # shapes only: the selection reads no Q/K, so any tensors of the right geometry describe it
    q = torch.empty((nb, H, 1, 8), dtype=torch.float32, device=DEV)
    k = torch.empty((nb, H, n_max, 8), dtype=torch.float32, device=DEV)
    prm = ep.make_params(q, k, n_cached=0, n_block=n_max, budget=m_max)
    nbytes, cap = ep.epicache_ragged_workspace_size(prm, select)
    ws = ep.alloc_ragged_workspace(prm, select)
    keep = torch.full((nb, H, cap), -1, dtype=torch.int32, device=DEV)
    n_kept = torch.full((nb, H), -1, dtype=torch.int32, device=DEV)
    ep.epicache_select_ragged(prm, select, torch.from_numpy(scores_np).to(DEV), i32(n_ctx),
                              None if budgets is None else i32(budgets), keep, n_kept, ws)
    torch.cuda.synchronize()
    return keep.cpu().numpy(), n_kept.cpu().numpy(), cap


def make_scores(kind, rng, shape):
    if kind == "uniform":
        return rng.random(shape, dtype=np.float32)
    if kind == "ties":       # few distinct values: the threshold class is large and spans heads
        return (rng.integers(0, 6, size=shape) / 8).astype(np.float32)
    if kind == "signed":     # negative values, zeros, infinities (no -0: the library orders it below +0)
        s = rng.standard_normal(shape).astype(np.float32)
        s[rng.random(shape) < 0.05] = 0.0
        s[rng.random(shape) < 0.01] = np.inf
        s[rng.random(shape) < 0.01] = -np.inf
        return s
    if kind == "skewed":     # one head dominates the pool, another is negligible
        s = rng.random(shape, dtype=np.float32)
        s[:, 0] *= 1e-6
        s[:, -1] += 2.0
        return s
    raise ValueError(kind)


SELECT_SIZES = [(300, 8, 40), (4096, 8, 2048), (5000, 3, 700), (20000, 2, 9000), (70, 1, 9)]


@pytest.mark.parametrize("select,pooled", SELECTS, ids=["per_head", "pooled"])
@pytest.mark.parametrize("kind", ["uniform", "ties", "signed", "skewed"])
@pytest.mark.parametrize("n_max,H,m_max", SELECT_SIZES, ids=[f"N{n}_H{h}_M{m}" for n, h, m in SELECT_SIZES])
def test_select_ragged_identical_to_oracle(n_max, H, m_max, kind, select, pooled):
    nb = 5
    say(f"select_ragged N_max={n_max} H={H} M_max={m_max} {kind} pooled={pooled}")
    rng = np.random.default_rng(n_max * 7 + H + len(kind))
    scores = make_scores(kind, rng, (nb, H, n_max))
    n_ctx = lengths(n_max + H, nb, H, n_max, (0, n_max, 1, min(n_max, m_max), min(n_max, m_max + 1)))
    budgets = rng.integers(1, m_max + 1, size=nb)
    budgets[0] = m_max
    budgets[1] = 1
    keep, n_kept, cap = gpu_select(scores, n_ctx, budgets, m_max, select)
    rows = [[scores[b, h, :n_ctx[b, h]] for h in range(H)] for b in range(nb)]
    want = orc.select_ragged(rows, budgets, pooled)
    for b in range(nb):
        for h in range(H):
            assert n_kept[b, h] == len(want[b][h]), f"b={b} h={h}: n_kept {n_kept[b, h]} != {len(want[b][h])}"
            assert n_kept[b, h] <= cap
            np.testing.assert_array_equal(keep[b, h, :n_kept[b, h]], want[b][h], err_msg=f"b={b} h={h}")
            assert (keep[b, h, n_kept[b, h]:] == -1).all(), f"b={b} h={h}: wrote beyond n_kept"


def test_select_ragged_without_budget_array_uses_the_common_budget():
    rng = np.random.default_rng(3)
    scores = rng.random((2, 4, 500), dtype=np.float32)
    n_ctx = lengths(4, 2, 4, 500, (500, 7))
    for select, pooled in SELECTS:
        keep, n_kept, _ = gpu_select(scores, n_ctx, None, 64, select)
        rows = [[scores[b, h, :n_ctx[b, h]] for h in range(4)] for b in range(2)]
        want = orc.select_ragged(rows, [64, 64], pooled)
        for b in range(2):
            for h in range(4):
                np.testing.assert_array_equal(keep[b, h, :n_kept[b, h]], want[b][h])


# ------------------------------------------------------------------- compact

@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 40), (torch.bfloat16, 64)],
                         ids=["bf16_d128", "f32_d40", "bf16_d64"])
def test_compact_ragged_bit_exact(dtype, d):
    nb, H, n_max, m_max = 3, 4, 700, 150
    say(f"compact_ragged {dtype} d={d}")
    rng = np.random.default_rng(21)
    gen = torch.Generator().manual_seed(5)
    k = torch.randn((nb, H, n_max, d), generator=gen).to(dtype)
    v = torch.randn((nb, H, n_max, d), generator=gen).to(dtype)
    n_ctx = lengths(22, nb, H, n_max, (0, 1, n_max))
    scores = rng.random((nb, H, n_max), dtype=np.float32)
    rows = [[scores[b, h, :n_ctx[b, h]] for h in range(H)] for b in range(nb)]
    budgets = [m_max, 3, 77]
    for select, pooled in SELECTS:
        want = orc.select_ragged(rows, budgets, pooled)
        kd, vd = k.to(DEV).clone(), v.to(DEV).clone()
        prm = ep.make_params(kd, kd, n_cached=0, n_block=n_max, budget=m_max)
        _, cap = ep.epicache_ragged_workspace_size(prm, select)
        keep = np.full((nb, H, cap), -1, dtype=np.int32)
        n_kept = np.zeros((nb, H), dtype=np.int32)
        for b in range(nb):
            for h in range(H):
                n_kept[b, h] = len(want[b][h])
                keep[b, h, :n_kept[b, h]] = want[b][h]
        ep.epicache_compact_ragged(prm, select, i32(keep), i32(n_kept), kd, vd)
        torch.cuda.synchronize()
        kb, vb = synth.raw_bits_numpy(k), synth.raw_bits_numpy(v)
        gk, gv = synth.raw_bits_numpy(kd.cpu()), synth.raw_bits_numpy(vd.cpu())
        for b in range(nb):
            for h in range(H):
                n = n_kept[b, h]
                np.testing.assert_array_equal(gk[b, h, :n], kb[b, h][want[b][h]])
                np.testing.assert_array_equal(gv[b, h, :n], vb[b, h][want[b][h]])
                np.testing.assert_array_equal(gk[b, h, n:], kb[b, h, n:])   # rows past the kept ones stay
                np.testing.assert_array_equal(gv[b, h, n:], vb[b, h, n:])


# ------------------------------------------------------------------- whole step

def run_ragged_step(q, k, v, n_ctx, budgets, m_max, n_max, select, reduce, want_intermediates=True, chunks=0):
    """chunks > 0: through epicache_evict_step_ragged_overlapped with that many chunks asked for."""
    qd, kd, vd = q.to(DEV), k.to(DEV).clone(), v.to(DEV).clone()
    prm = ep.make_params(qd, kd, n_cached=0, n_block=n_max, budget=m_max, reduce=reduce)
    nb, H = kd.shape[0], kd.shape[1]
    if chunks:
        nbytes, cap, used = ep.epicache_ragged_overlapped_workspace_size(prm, select, chunks)
        assert cap == ep.epicache_ragged_workspace_size(prm, select)[1]
        assert used == -(-nb // -(-nb // min(chunks, nb)))
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV)
    else:
        _, cap = ep.epicache_ragged_workspace_size(prm, select)
        ws = ep.alloc_ragged_workspace(prm, select)
    n_kept = torch.full((nb, H), -1, dtype=torch.int32, device=DEV)
    scores = keep = None
    if want_intermediates:
        scores = torch.full((nb, H, n_max), float("nan"), dtype=torch.float32, device=DEV)
        keep = torch.full((nb, H, cap), -1, dtype=torch.int32, device=DEV)
    if chunks:
        ep.epicache_evict_step_ragged_overlapped(prm, select, qd, kd, vd, i32(n_ctx), i32(budgets), n_kept, ws,
                                                 torch.cuda.Stream(), chunks, scores, keep)
    else:
        ep.epicache_evict_step_ragged(prm, select, qd, kd, vd, i32(n_ctx), i32(budgets), n_kept, ws, scores, keep)
    torch.cuda.synchronize()
    return (None if scores is None else scores.cpu().numpy(), None if keep is None else keep.cpu().numpy(),
            n_kept.cpu().numpy(), kd.cpu(), vd.cpu())


def check_ragged_step(q, k, v, n_ctx, budgets, m_max, n_max, select, pooled, reduce, what, chunks=0):
    scores, keep, n_kept, kd, vd = run_ragged_step(q, k, v, n_ctx, budgets, m_max, n_max, select, reduce, chunks=chunks)
    rtol = pu.rtol_for(q.dtype)
    rows = orc.score_ragged(*pu.oracle_inputs(q, k), n_ctx, reduce)
    nb, H = n_kept.shape
    got_keep = [[keep[b, h, :n_kept[b, h]] for h in range(H)] for b in range(nb)]
    for b in range(nb):
        for h in range(H):
            if n_ctx[b][h]:
                pu.assert_scores_close(scores[b, h, :n_ctx[b][h]], rows[b][h], rtol, f"{what} b={b} h={h}")
    differ = pu.assert_ragged_keep_matches(got_keep, rows, budgets, pooled, rtol, what)
    # compaction: bit exact for the rows the GPU selected; rows past them untouched
    kb, vb = synth.raw_bits_numpy(k), synth.raw_bits_numpy(v)
    gk, gv = synth.raw_bits_numpy(kd), synth.raw_bits_numpy(vd)
    for b in range(nb):
        for h in range(H):
            n = n_kept[b, h]
            np.testing.assert_array_equal(gk[b, h, :n], kb[b, h][got_keep[b][h]])
            np.testing.assert_array_equal(gv[b, h, :n], vb[b, h][got_keep[b][h]])
            np.testing.assert_array_equal(gk[b, h, n:], kb[b, h, n:])
    # the workspace-only variant gives the same cache and counts
    _, _, n_kept2, kd2, vd2 = run_ragged_step(q, k, v, n_ctx, budgets, m_max, n_max, select, reduce, False, chunks)
    assert (n_kept2 == n_kept).all()
    assert torch.equal(kd2.view(torch.uint8), kd.view(torch.uint8)) and torch.equal(vd2.view(torch.uint8), vd.view(torch.uint8))
    return differ, n_kept


@pytest.mark.parametrize("select,pooled", SELECTS, ids=["per_head", "pooled"])
@pytest.mark.parametrize("reduce", [orc.REDUCE_MAX, orc.REDUCE_SUM], ids=["max", "sum"])
def test_evict_step_ragged_tiny_fp32(reduce, select, pooled):
    w = wl("tiny", E=3)
    say(f"evict_step_ragged tiny reduce={reduce} pooled={pooled}")
    q, k, v = synth.make_layer(w)
    n_ctx = lengths(31, w.E, w.Hkv, w.N, (w.N, 0, 1))
    budgets = [w.M, max(1, w.M // 3), 2]
    differ, _ = check_ragged_step(q, k, v, n_ctx, budgets, w.M, w.N, select, pooled, reduce, "tiny")
    say(f"  tokens differing inside the band: {differ}")


@pytest.mark.parametrize("select,pooled", SELECTS, ids=["per_head", "pooled"])
def test_evict_step_ragged_bf16_layer(select, pooled):
    """LLaMA-3.2-3B-shaped heads with ragged lengths and a different budget per batch item."""
    w = wl("llama32_3b", E=3, M=512, B=512)
    say(f"evict_step_ragged llama32_3b-shaped pooled={pooled}")
    q, k, v = synth.make_layer(w, layer=2)
    n_ctx = lengths(32, w.E, w.Hkv, w.N, (w.N, 0, 1, 513, 64))
    budgets = [512, 300, 17]
    differ, n_kept = check_ragged_step(q, k, v, n_ctx, budgets, w.M, w.N, select, pooled, orc.REDUCE_SUM, "bf16")
    say(f"  tokens differing inside the band: {differ}; kept per head of item 0: {n_kept[0].tolist()}")


def test_layers_with_eq6_budgets_fold_into_one_launch():
    """Sec. 3.2: layers whose budgets M_l come from Eq. 6 hold M_l + B rows before the step; folded into the
    batch axis they are one ragged launch, checked against the uniform oracle step of each layer."""
    w = wl("llama31_8b", E=2, Hq=8, Hkv=2, p=32, M=384, B=256, L=3)
    m_l = ep.epicache_layer_budgets([0.12, 0.31, 0.05], 2.0, w.M)
    assert sum(m_l) == w.L * w.M and len(set(m_l)) == 3
    n_max, m_max = max(m_l) + w.B, max(m_l)
    say(f"folded layers, budgets {m_l}")
    qs, ks, vs, n_ctx, budgets = [], [], [], [], []
    for l in range(w.L):
        q, k, v = synth.make_layer(w, layer=l, n_ctx=m_l[l] + w.B, capacity=n_max)
        qs.append(q), ks.append(k), vs.append(v)
        n_ctx += [[m_l[l] + w.B] * w.Hkv] * w.E
        budgets += [m_l[l]] * w.E
    q, k, v = torch.cat(qs), torch.cat(ks), torch.cat(vs)
    scores, keep, n_kept, kd, vd = run_ragged_step(q, k, v, n_ctx, budgets, m_max, n_max, ep.SELECT_PER_HEAD,
                                                   orc.REDUCE_SUM)
    for l in range(w.L):
        sl = slice(l * w.E, (l + 1) * w.E)
        N, M = m_l[l] + w.B, m_l[l]
        o_scores, o_keep, o_k, o_v = orc.evict_step(*pu.oracle_inputs(qs[l], ks[l]), None, N, M, orc.REDUCE_SUM,
                                                    k_bits=synth.raw_bits_numpy(ks[l]),
                                                    v_bits=synth.raw_bits_numpy(vs[l]))
        assert (n_kept[sl] == M).all()
        pu.assert_scores_close(scores[sl, :, :N], o_scores, pu.RTOL_BF16, f"layer {l}")
        pu.assert_keep_matches(keep[sl, :, :M], o_scores, M, pu.RTOL_BF16, f"layer {l}")
        same = (keep[sl, :, :M] == o_keep).all(axis=2)
        assert same.any()
        np.testing.assert_array_equal(synth.raw_bits_numpy(kd[sl])[:, :, :M][same], o_k[same])
        np.testing.assert_array_equal(synth.raw_bits_numpy(vd[sl])[:, :, :M][same], o_v[same])


def test_pooled_sweep_feeds_its_own_counts_forward():
    """Head-wise non-uniform retention over a block sweep: the per-head counts one step leaves on the
    device are the next step's cached lengths (no host round trip inside the library); the layer as a
    whole settles at Hkv * M rows while the heads differ.  Each step is checked against the oracle
    started from the same cache."""
    w = wl("llama31_8b", E=2, Hq=8, Hkv=4, p=32, M=256, B=256)
    H, steps = w.Hkv, 4
    n_max = H * w.M + w.B          # a head may hold the whole layer's budget before the next block
    say(f"pooled sweep {steps} steps, capacity {n_max}")
    cache = [[(None, None)] * H for _ in range(w.E)]
    n_cached = np.zeros((w.E, H), dtype=np.int64)
    for step in range(steps):
        q, bk, bv = synth.make_layer(w, layer=0, step=step, n_ctx=w.B)
        k = torch.zeros((w.E, H, n_max, w.d), dtype=bk.dtype)
        v = torch.zeros_like(k)
        for b in range(w.E):
            for h in range(H):
                c = n_cached[b, h]
                if c:
                    k[b, h, :c], v[b, h, :c] = cache[b][h]
                k[b, h, c:c + w.B], v[b, h, c:c + w.B] = bk[b, h], bv[b, h]
        n_ctx = n_cached + w.B
        assert n_ctx.max() <= n_max
        budgets = [w.M] * w.E
        differ, n_kept = check_ragged_step(q, k, v, n_ctx, budgets, w.M, n_max, ep.SELECT_POOLED, True,
                                           orc.REDUCE_MAX, f"step {step}")
        assert (n_kept.sum(axis=1) == np.minimum(H * w.M, n_ctx.sum(axis=1))).all()
        # resynchronise on the oracle's cache
        _, o_keep, o_k, o_v = orc.evict_step_ragged(*pu.oracle_inputs(q, k), None, n_ctx, budgets, True,
                                                    orc.REDUCE_MAX, k_bits=synth.raw_bits_numpy(k),
                                                    v_bits=synth.raw_bits_numpy(v))
        for b in range(w.E):
            for h in range(H):
                n_cached[b, h] = len(o_keep[b][h])
                cache[b][h] = (torch.from_numpy(o_k[b][h].view(np.int16)).view(torch.bfloat16),
                               torch.from_numpy(o_v[b][h].view(np.int16)).view(torch.bfloat16))
        say(f"  step {step}: differ {differ}, oracle rows per head of item 0: {n_cached[0].tolist()}")
    assert len(set(n_cached[0].tolist())) > 1     # the heads really ended up with different lengths


@pytest.mark.parametrize("i", range(60))
def test_evict_step_ragged_random_shape(i):
    """Seeded sweep of valid shapes through the ragged step: head dims of the MFMA and of the plain kernels,
    per-head lengths from 0 to the maximum, per-item budgets from 1 to beyond the longest head, per-head and
    pooled selection, both reductions."""
    rng = np.random.default_rng(0xAD4 + i)
    bf16 = bool(rng.integers(0, 2))
    d = int(rng.choice([64, 128])) if (bf16 and rng.random() < 0.7) else int(8 * rng.integers(1, 33))
    Hkv, G = int(rng.integers(1, 5)), int(rng.choice([1, 2, 3, 4]))
    p = int(rng.choice([1, 7, 32, 33, 64, 90]))
    n_max = int(rng.choice([2, 64, 65, 129, 256, 300, 513, 700]))
    E = int(rng.integers(1, 4))
    m_max = int(rng.choice([1, max(1, n_max // 3), max(1, n_max // 2), n_max + 3]))
    select, pooled = SELECTS[int(rng.integers(0, 2))]
    reduce = int(rng.integers(0, 2))
    w = wl("tiny", E=E, Hq=Hkv * G, Hkv=Hkv, d=d, p=p, dtype="bf16" if bf16 else "f32", M=m_max, B=1,
           recipe=str(rng.choice(["normal", "outlier_channels", "student_t"])), seed=0xE91C2000 + i)
    say(f"evict_step_ragged random {i}: bf16={bf16} d={d} Hkv={Hkv} G={G} p={p} n_max={n_max} E={E} m_max={m_max} "
        f"pooled={pooled} reduce={reduce}")
    q, k, v = synth.make_layer(w, layer=i, n_ctx=n_max)
    n_ctx = rng.integers(0, n_max + 1, size=(E, Hkv))
    n_ctx.reshape(-1)[int(rng.integers(0, n_ctx.size))] = n_max
    budgets = [int(x) for x in rng.integers(1, m_max + 1, size=E)]
    check_ragged_step(q, k, v, n_ctx, budgets, m_max, n_max, select, pooled, reduce, f"random {i}")


@pytest.mark.parametrize("i", range(30))
def test_evict_step_ragged_overlapped_random_shape(i):
    """The same sweep through epicache_evict_step_ragged_overlapped: 2-7 batch items in 2-7 chunks, every array
    used in slices of whole items (lengths, budgets, counts, scores, kept indices)."""
    rng = np.random.default_rng(0x0AD4 + i)
    bf16 = bool(rng.integers(0, 2))
    d = int(rng.choice([64, 128])) if (bf16 and rng.random() < 0.7) else int(8 * rng.integers(1, 33))
    Hkv, G = int(rng.integers(1, 5)), int(rng.choice([1, 2, 3, 4]))
    p = int(rng.choice([1, 7, 32, 33, 64, 90]))
    n_max = int(rng.choice([2, 64, 65, 129, 256, 300, 513, 700]))
    E = int(rng.integers(2, 8))
    chunks = int(rng.integers(2, 8))
    m_max = int(rng.choice([1, max(1, n_max // 3), max(1, n_max // 2), n_max + 3]))
    select, pooled = SELECTS[int(rng.integers(0, 2))]
    reduce = int(rng.integers(0, 2))
    w = wl("tiny", E=E, Hq=Hkv * G, Hkv=Hkv, d=d, p=p, dtype="bf16" if bf16 else "f32", M=m_max, B=1,
           recipe=str(rng.choice(["normal", "outlier_channels", "student_t"])), seed=0xE91C3000 + i)
    say(f"evict_step_ragged_overlapped random {i}: bf16={bf16} d={d} Hkv={Hkv} G={G} p={p} n_max={n_max} E={E} "
        f"chunks={chunks} m_max={m_max} pooled={pooled} reduce={reduce}")
    q, k, v = synth.make_layer(w, layer=i, n_ctx=n_max)
    n_ctx = rng.integers(0, n_max + 1, size=(E, Hkv))
    n_ctx.reshape(-1)[int(rng.integers(0, n_ctx.size))] = n_max
    budgets = [int(x) for x in rng.integers(1, m_max + 1, size=E)]
    check_ragged_step(q, k, v, n_ctx, budgets, m_max, n_max, select, pooled, reduce, f"overlapped random {i}",
                      chunks=chunks)
