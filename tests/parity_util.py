"""Comparison helpers for GPU-vs-oracle parity tests (no method arithmetic here)."""
import numpy as np
import torch

from oracle import epicache_oracle as orc
from paper_2509_17396_amd import synth

# Score tolerances of the benchmark spec: relative error against the float64 oracle.
RTOL_F32 = 1e-5    # fp32 inputs
RTOL_BF16 = 2e-2   # bf16 inputs, fp32 accumulation
# Scores this small are compared absolutely: weights below ~2^-100 may flush to zero on the GPU.
ATOL = 1e-30


def rtol_for(dtype: torch.dtype) -> float:
    return RTOL_F32 if dtype == torch.float32 else RTOL_BF16


def assert_scores_close(gpu_scores: np.ndarray, oracle_scores: np.ndarray, rtol: float, what=""):
    g = np.asarray(gpu_scores, dtype=np.float64)
    o = np.asarray(oracle_scores, dtype=np.float64)
    assert g.shape == o.shape, (g.shape, o.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite GPU score"
    err = np.abs(g - o)
    bound = rtol * np.abs(o) + ATOL
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err / bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} scores out of tolerance; worst at {i}: "
                             f"gpu {g[i]!r} oracle {o[i]!r} rel {err[i] / max(abs(o[i]), 1e-300):.3e}")
    return float((err / (np.abs(o) + ATOL)).max())


def assert_keep_valid(keep: np.ndarray, N: int, n_keep: int, what=""):
    """What is never negotiable: count, range, strictly ascending order."""
    assert keep.shape[-1] == n_keep, f"{what}: kept {keep.shape[-1]} != {n_keep}"
    assert (keep >= 0).all() and (keep < N).all(), f"{what}: index out of range"
    assert (np.diff(keep, axis=-1) > 0).all(), f"{what}: indices not strictly ascending"


def assert_keep_matches(gpu_keep: np.ndarray, oracle_scores: np.ndarray, M: int, rtol: float, what=""):
    """Kept sets must equal the oracle's except for tokens whose oracle score lies within
    the score tolerance of the oracle's M-th largest score.  Returns #tokens that differ."""
    nb, H, N = oracle_scores.shape
    n_keep = min(M, N)
    assert_keep_valid(gpu_keep, N, n_keep, what)
    differ = 0
    for b in range(nb):
        for h in range(H):
            s = oracle_scores[b, h]
            ref = orc.topk_1d(s.astype(np.float32), M)
            got = gpu_keep[b, h]
            sym = np.setxor1d(ref, got)
            if sym.size == 0:
                continue
            thr = np.sort(s)[N - n_keep]
            off = np.abs(s[sym] - thr)
            band = rtol * abs(thr) + ATOL
            assert (off <= band).all(), (
                f"{what} b={b} h={h}: {sym.size} differing tokens, "
                f"{(off > band).sum()} outside the tolerance band (thr {thr!r}, worst {off.max()!r})")
            differ += sym.size
    return differ


def oracle_inputs(q: torch.Tensor, k: torch.Tensor):
    """float64 host copies with exactly the values of the (fp32 / bf16) device tensors."""
    return synth.to_f64_numpy(q), synth.to_f64_numpy(k)


def oracle_score_one_head(q: torch.Tensor, k: torch.Tensor, b: int, h: int, N: int, reduce: int,
                          scale=None) -> np.ndarray:
    """Oracle scores of one (batch item, KV head) of a large tensor: [N] float64."""
    G = q.shape[1] // k.shape[1]
    qq = synth.to_f64_numpy(q[b:b + 1, h * G:(h + 1) * G])
    kk = synth.to_f64_numpy(k[b:b + 1, h:h + 1, :N])
    return orc.score(qq, kk, N, reduce, scale)[0, 0]


def oracle_score_heads(q: torch.Tensor, k: torch.Tensor, heads, N: int, reduce: int, scale=None, workers=None):
    """Oracle scores of several (batch item, KV head) pairs of a large tensor, one oracle call per head,
    the calls spread over host threads (numpy releases the interpreter lock inside its loops).
    Returns {(b, h): [N] float64}."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    G = q.shape[1] // k.shape[1]
    heads = list(heads)
    host = {}
    for (b, h) in heads:  # exact widening of the device bits, done once, serially
        host[(b, h)] = (synth.to_f64_numpy(q[b:b + 1, h * G:(h + 1) * G]), synth.to_f64_numpy(k[b:b + 1, h:h + 1, :N]))
    if workers is None:
        workers = max(1, min(16, os.cpu_count() or 1))

    def one(bh):
        qq, kk = host[bh]
        return bh, orc.score(qq, kk, N, reduce, scale)[0, 0]

    with ThreadPoolExecutor(max_workers=workers) as pool:
        return dict(pool.map(one, heads))


def assert_ragged_keep_matches(gpu_keep, oracle_rows, budgets, pooled: bool, rtol: float, what=""):
    """Ragged counterpart of assert_keep_matches.  gpu_keep[b][h]: kept indices of head (b, h);
    oracle_rows[b][h]: float64 oracle scores of its n_ctx rows.  Counts are exact (per head, or per
    item when pooled); membership may differ from the oracle's only for tokens whose oracle score lies
    within the score tolerance of the oracle's threshold score.  Returns #tokens that differ."""
    differ = 0
    for b, rows in enumerate(oracle_rows):
        H, M = len(rows), int(budgets[b])
        rows32 = [r.astype(np.float32) for r in rows]
        ref = orc.select_pooled(rows32, M) if pooled else [orc.topk_1d(r, M) for r in rows32]
        for h in range(H):
            got = np.asarray(gpu_keep[b][h])
            assert (got >= 0).all() and (got < len(rows[h])).all(), f"{what} b={b} h={h}: index out of range"
            assert (np.diff(got) > 0).all(), f"{what} b={b} h={h}: indices not strictly ascending"
            if not pooled:
                assert len(got) == min(M, len(rows[h])), f"{what} b={b} h={h}: kept {len(got)}"
        total = sum(len(r) for r in rows)
        n_keep = min(H * M, total)
        if pooled:
            assert sum(len(g) for g in gpu_keep[b]) == n_keep, f"{what} b={b}: pooled count"
            pool_thr = np.sort(np.concatenate(rows))[total - n_keep] if 0 < n_keep < total else None
        for h in range(H):
            sym = np.setxor1d(ref[h], np.asarray(gpu_keep[b][h]))
            if sym.size == 0:
                continue
            if pooled:
                assert pool_thr is not None, f"{what} b={b} h={h}: everything fits, yet the sets differ"
                thr = pool_thr
            else:
                thr = np.sort(rows[h])[len(rows[h]) - min(M, len(rows[h]))]
            off = np.abs(rows[h][sym] - thr)
            band = rtol * abs(thr) + ATOL
            assert (off <= band).all(), (
                f"{what} b={b} h={h}: {sym.size} differing tokens, {(off > band).sum()} outside the band "
                f"(thr {thr!r}, worst {off.max()!r})")
            differ += sym.size
    return differ
