"""CPU oracle for the EpiCache eviction step.  TEST INFRASTRUCTURE ONLY.

This is the plain definition of what one eviction step of block-wise prefill
computes, written from the paper and evaluated in float64 with numpy.  It is
slow on purpose, shares no code with the HIP path and must never be imported by
the product package: only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may use it.

What the paper fixes and what is a reading of it:
  * importance of context token i = attention weight it receives from the
    patched-prompt queries, reduced over the query tokens with max (Sec. 2.3,
    Eq. 1).  REDUCE_SUM (sum of the weights, "attention mass") is the variant
    the benchmark spec asks for next to it.
  * the top M tokens are kept (Sec. 3.1 Stage 2; Alg. 1 phase A3), so that the
    cache returns to size M after growing to M + M_block (Sec. 2.2, App. A.3).
  * readings where the paper is silent: the G query heads of a GQA group vote
    for their KV head with the same operator as the query tokens; the softmax
    is over the N context keys only; logits are scaled by 1/sqrt(d); ties go to
    the lower index; kept rows stay in their original order.
Which reduction and softmax denominator the authors' own runs used cannot be
checked against anything (no code, no numbers in the paper): parity unpinned
for that choice; both reductions are implemented.
"""
from __future__ import annotations

import math

import numpy as np

REDUCE_MAX = 0  # Eq. 1
REDUCE_SUM = 1


def attention_weights(q_rows: np.ndarray, k_ctx: np.ndarray, scale: float) -> np.ndarray:
    """Attn(x_t -> x_i) for every query row t and context key i (Sec. 2.3).

    q_rows [R, d], k_ctx [N, d] float64.  Row-wise softmax of scale * q.k over
    the N context keys.  Returns [R, N].
    """
    z = scale * (q_rows @ k_ctx.T)
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def score(q: np.ndarray, k: np.ndarray, n_ctx: int, reduce: int = REDUCE_MAX,
          scale: float | None = None) -> np.ndarray:
    """Importance s[b, h, i] of context token i for KV head h of batch item b.

    q [nb, Hq, p, d], k [nb, Hkv, C >= n_ctx, d] (any float dtype, widened to
    float64).  Query head hq votes for KV head hq // G, G = Hq / Hkv.
    Eq. 1 with the reduction taken over the G * p rows of the group.
    Returns float64 [nb, Hkv, n_ctx].
    """
    nb, Hq, p, d = q.shape
    Hkv = k.shape[1]
    assert Hq % Hkv == 0 and k.shape[0] == nb and k.shape[3] == d and k.shape[2] >= n_ctx
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty((nb, Hkv, n_ctx), dtype=np.float64)
    for b in range(nb):
        for h in range(Hkv):
            rows = np.asarray(q[b, h * G:(h + 1) * G], dtype=np.float64).reshape(G * p, d)
            keys = np.asarray(k[b, h, :n_ctx], dtype=np.float64)
            attn = attention_weights(rows, keys, scale)
            out[b, h] = attn.max(axis=0) if reduce == REDUCE_MAX else attn.sum(axis=0)
    return out


def score_given_lse(q: np.ndarray, k: np.ndarray, n_ctx: int, row_lse: np.ndarray, reduce: int = REDUCE_MAX,
                    scale: float | None = None) -> np.ndarray:
    """Eq. 1 when every scoring query's softmax normaliser is supplied from outside.

    row_lse [nb, Hq, p]: natural log of the sum of exp(scale * q.k) over all keys that query attends
    to.  If that set is the N context keys this equals score(); if it is larger (in a real forward
    pass patch token t also attends to the patch tokens up to t, Sec. 2.3) the result is the
    attention weight under that larger denominator, restricted to the context columns.
    """
    nb, Hq, p, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty((nb, Hkv, n_ctx), dtype=np.float64)
    for b in range(nb):
        for h in range(Hkv):
            rows = np.asarray(q[b, h * G:(h + 1) * G], dtype=np.float64).reshape(G * p, d)
            lse = np.asarray(row_lse[b, h * G:(h + 1) * G], dtype=np.float64).reshape(G * p, 1)
            keys = np.asarray(k[b, h, :n_ctx], dtype=np.float64)
            attn = np.exp(scale * (rows @ keys.T) - lse)
            out[b, h] = attn.max(axis=0) if reduce == REDUCE_MAX else attn.sum(axis=0)
    return out


def topk_1d(s: np.ndarray, M: int) -> np.ndarray:
    """Indices of the min(M, N) largest entries of s, ascending; ties -> lower index."""
    N = s.shape[0]
    keep = min(M, N)
    order = np.lexsort((np.arange(N), -s))  # primary: score descending, secondary: index
    return np.sort(order[:keep]).astype(np.int32)


def topk(scores: np.ndarray, M: int) -> np.ndarray:
    """Per (b, h) top-M retention (Sec. 3.1 Stage 2).  scores [nb, Hkv, N] -> int32 [nb, Hkv, min(M,N)]."""
    nb, Hkv, N = scores.shape
    out = np.empty((nb, Hkv, min(M, N)), dtype=np.int32)
    for b in range(nb):
        for h in range(Hkv):
            out[b, h] = topk_1d(scores[b, h], M)
    return out


def topk_by_counting(s, M: int):
    """The same set from the counting definition, O(N^2), pure Python, tiny inputs only.

    Token i is kept iff fewer than M tokens beat it, where j beats i when
    s_j > s_i, or s_j == s_i and j < i.
    """
    N = len(s)
    kept = []
    for i in range(N):
        beaten_by = 0
        for j in range(N):
            if s[j] > s[i] or (s[j] == s[i] and j < i):
                beaten_by += 1
        if beaten_by < M:
            kept.append(i)
    return kept


def compact(x: np.ndarray, keep_idx: np.ndarray) -> np.ndarray:
    """Rows keep_idx[b, h, :] of x[b, h] moved to the front, in order (Sec. 2.2, App. A.3).

    x [nb, Hkv, C, d] of any dtype (bit patterns are copied, no arithmetic).
    Returns a new array [nb, Hkv, n_keep, d].
    """
    nb, Hkv = keep_idx.shape[:2]
    out = np.empty((nb, Hkv, keep_idx.shape[2], x.shape[3]), dtype=x.dtype)
    for b in range(nb):
        for h in range(Hkv):
            out[b, h] = x[b, h][keep_idx[b, h]]
    return out


def evict_step(q, k, v, n_ctx: int, M: int, reduce: int = REDUCE_MAX, scale=None,
               k_bits=None, v_bits=None):
    """One eviction step (Alg. 1 phase A3): score, keep top M, compact K and V.

    The selection is taken on the scores rounded to float32, the precision of
    the score buffer that the selection reads.  k_bits / v_bits, if given, are
    the raw bit patterns to gather instead of k / v.
    Returns (scores float64, keep_idx int32, K', V').
    """
    s = score(q, k, n_ctx, reduce, scale)
    idx = topk(s.astype(np.float32), M)
    kk = compact(k if k_bits is None else k_bits, idx)
    vv = compact(v if v_bits is None else v_bits, idx)
    return s, idx, kk, vv


def layer_budgets_real(sensitivity, alpha: float, M: int):
    """Eq. 6 as printed: M_l = s_l^alpha / sum_j s_j^alpha * (L * M), real valued."""
    s = np.asarray(sensitivity, dtype=np.float64)
    w = s ** alpha
    return w / w.sum() * (len(s) * M)


def layer_budgets(sensitivity, alpha: float, M: int):
    """Integer budgets from Eq. 6 (Alg. 1 phase A2, last line).

    Reading where the paper is silent: round by largest remainder (ties to the lower layer) so the
    budgets sum to L * M exactly, then make sure no layer has zero rows by moving one row from the
    currently largest layer; all-zero sensitivities give the uniform split.
    """
    L = len(sensitivity)
    s = [float(x) for x in sensitivity]
    w = [x ** alpha for x in s]
    wsum = 0.0
    for x in w:
        wsum += x
    if not wsum > 0.0:
        return [M] * L
    quota = [x / wsum * float(L * M) for x in w]
    out = [int(math.floor(x)) for x in quota]
    frac = [x - math.floor(x) for x in quota]
    for _ in range(L * M - sum(out)):
        best = max(range(L), key=lambda l: (frac[l], -l))
        out[best] += 1
        frac[best] = -1.0
    for l in range(L):
        if out[l] < 1:
            big = max(range(L), key=lambda j: (out[j], -j))
            out[big] -= 1
            out[l] = 1
    return out


# ---------------------------------------------------------------------------------------------
# Ragged batches: every (batch item, KV head) has its own number of context rows and every
# batch item its own budget.  Needed for head-wise non-uniform retention (App. A.2, last
# paragraph: every method of the paper's experiments selects tokens head-wise non-uniformly in
# the manner of Ada-KV) and for layers with different budgets (Eq. 6) folded into one batch.
#
# Reading (the paper only cites the rule, it does not print it): the scores of the Hkv heads of
# one batch item (one layer of one episode) form one pool; the Hkv * M highest-scoring entries
# of the pool are kept, so a head whose attention is spread over many tokens keeps more rows
# than a head that concentrates on a few, and the layer as a whole still holds Hkv * M rows.
# Ties go to the lower head, then to the lower token index.  No per-head floor is applied.
# Which variant of the cited rule the authors ran cannot be checked: parity unpinned for that
# choice; the pooled top-k itself is pinned by its counting definition.
# ---------------------------------------------------------------------------------------------

def score_ragged(q, k, n_ctx, reduce: int = REDUCE_MAX, scale: float | None = None):
    """Eq. 1 per (b, h) over the first n_ctx[b][h] rows of k[b, h].

    Returns rows[b][h]: float64 array of length n_ctx[b][h] (empty where it is 0).
    """
    nb, Hq, p, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    rows = []
    for b in range(nb):
        per_head = []
        for h in range(Hkv):
            n = int(n_ctx[b][h])
            if n == 0:
                per_head.append(np.empty(0, dtype=np.float64))
                continue
            qr = np.asarray(q[b, h * G:(h + 1) * G], dtype=np.float64).reshape(G * p, d)
            keys = np.asarray(k[b, h, :n], dtype=np.float64)
            attn = attention_weights(qr, keys, scale)
            per_head.append(attn.max(axis=0) if reduce == REDUCE_MAX else attn.sum(axis=0))
        rows.append(per_head)
    return rows


def select_pooled(head_scores, M: int):
    """Head-wise non-uniform retention for one batch item.

    head_scores: list of Hkv 1-D arrays (lengths may differ).  Keeps the min(Hkv * M, total)
    largest entries of the concatenation; ties -> lower head, then lower index.
    Returns a list of Hkv ascending int32 index arrays.
    """
    H = len(head_scores)
    lens = [len(s) for s in head_scores]
    pool = np.concatenate([np.asarray(s) for s in head_scores]) if H else np.empty(0)
    total = pool.shape[0]
    n_keep = min(H * M, total)
    order = np.lexsort((np.arange(total), -pool))[:n_keep]   # score descending, then pool position
    kept = np.zeros(total, dtype=bool)
    kept[order] = True
    out, start = [], 0
    for h in range(H):
        out.append(np.nonzero(kept[start:start + lens[h]])[0].astype(np.int32))
        start += lens[h]
    return out


def select_pooled_by_counting(head_scores, M: int):
    """The same sets from the counting definition, O(total^2), pure Python, tiny inputs only.

    Entry (h, i) is kept iff fewer than Hkv * M entries beat it, where (g, j) beats (h, i) when it
    scores higher, or equally with (g, j) < (h, i) in lexicographic order.
    """
    H = len(head_scores)
    flat = [(float(s), h, i) for h in range(H) for i, s in enumerate(head_scores[h])]
    out = [[] for _ in range(H)]
    for (s, h, i) in flat:
        beaten_by = 0
        for (t, g, j) in flat:
            if t > s or (t == s and (g, j) < (h, i)):
                beaten_by += 1
        if beaten_by < H * M:
            out[h].append(i)
    return out


def select_ragged(rows, budgets, pooled: bool):
    """rows[b][h]: 1-D scores; budgets[b]: M_b.  Returns keep[b][h]: ascending int32 arrays."""
    keep = []
    for b, per_head in enumerate(rows):
        M = int(budgets[b])
        if pooled:
            keep.append(select_pooled(per_head, M))
        else:
            keep.append([topk_1d(np.asarray(s), M) for s in per_head])
    return keep


def evict_step_ragged(q, k, v, n_ctx, budgets, pooled: bool, reduce: int = REDUCE_MAX, scale=None,
                      k_bits=None, v_bits=None):
    """One eviction step on a ragged batch: score, select (per head or pooled), compact.

    As in evict_step the selection reads the scores rounded to float32.
    Returns (rows, keep, K', V') with K'[b][h] = the kept rows of k[b, h] (or of k_bits), in order.
    """
    rows = score_ragged(q, k, n_ctx, reduce, scale)
    rows32 = [[s.astype(np.float32) for s in per_head] for per_head in rows]
    keep = select_ragged(rows32, budgets, pooled)
    ks = k if k_bits is None else k_bits
    vs = v if v_bits is None else v_bits
    kk = [[ks[b, h][idx] for h, idx in enumerate(per_head)] for b, per_head in enumerate(keep)]
    vv = [[vs[b, h][idx] for h, idx in enumerate(per_head)] for b, per_head in enumerate(keep)]
    return rows, keep, kk, vv


# ---------------------------------------------------------------------------------------------
# The patch's own keys in the denominator.  In a forward pass of the model the patch token
# x_{n+1+t} attends causally to the n context tokens and to the patch tokens up to itself, so the
# attention weight of Eq. 1 is normalised over n + t + 1 keys.  (Sec. 2.3 only says that the patch
# queries attend back to the context; score() above takes that literally and normalises over the
# context alone.)  The patch is appended after the context (Sec. 2.3): its keys sit in rows
# [n_ctx, n_ctx + p) of k[b, h], and they are never scored or kept themselves.
# ---------------------------------------------------------------------------------------------

def attention_weights_causal_patch(q_rows, k_ctx, k_patch, scale: float, p: int) -> np.ndarray:
    """Weights on the N context keys for the R = G*p query rows (row r = g*p + t is patch token t).

    Row r's softmax runs over the N context keys and the patch keys 0..t.  Returns [R, N].
    """
    R, N = q_rows.shape[0], k_ctx.shape[0]
    out = np.empty((R, N), dtype=np.float64)
    for r in range(R):
        t = r % p
        keys = np.concatenate([k_ctx, k_patch[:t + 1]])
        z = scale * (keys @ q_rows[r])
        z = z - z.max()
        e = np.exp(z)
        out[r] = e[:N] / e.sum()
    return out


def score_causal_patch(q, k, n_ctx: int, reduce: int = REDUCE_MAX, scale: float | None = None) -> np.ndarray:
    """Eq. 1 with the patch's own causal keys in every softmax denominator.

    q [nb, Hq, p, d]; k [nb, Hkv, C >= n_ctx + p, d] with the patch keys in rows n_ctx .. n_ctx+p-1.
    Returns float64 [nb, Hkv, n_ctx].
    """
    nb, Hq, p, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    assert k.shape[2] >= n_ctx + p
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty((nb, Hkv, n_ctx), dtype=np.float64)
    for b in range(nb):
        for h in range(Hkv):
            rows = np.asarray(q[b, h * G:(h + 1) * G], dtype=np.float64).reshape(G * p, d)
            ctx = np.asarray(k[b, h, :n_ctx], dtype=np.float64)
            patch = np.asarray(k[b, h, n_ctx:n_ctx + p], dtype=np.float64)
            attn = attention_weights_causal_patch(rows, ctx, patch, scale, p)
            out[b, h] = attn.max(axis=0) if reduce == REDUCE_MAX else attn.sum(axis=0)
    return out


# ---------------------------------------------------------------------------------------------
# Attention-based baselines of App. A.2: Eq. 1 with another choice of patched prompt, on the same
# top-M / compaction back end.
#
# KVzip: the patch is a repetition instruction followed by the whole block, so p is about the
# block size (thousands of query tokens per head).  Nothing else changes: its scores are score()
# above with that long patch.  Every scoring row is normalised on its own, so the reduction over
# the rows may be taken over any partition of the patch tokens into chunks and then over the
# chunks; score_by_patch_chunks() writes that out and the pins check it against score().
#
# SnapKV: the patch is the window formed by the last w tokens of the block itself (w = 64 in the
# paper).  Those tokens are part of the context: their keys sit in rows n_ctx-w .. n_ctx-1 of the
# cache, and in the forward pass window token t attends causally to every earlier row and to the
# window rows up to itself.
# Readings where the paper is silent: only the rows before the window are scored (a window token's
# weight on another window token is not an importance vote for itself); the window rows are always
# retained, as in SnapKV's own design, so the M - w best of the earlier rows are kept next to them;
# the budget must therefore be at least w.  If n_ctx <= M nothing is evicted.
# ---------------------------------------------------------------------------------------------

def score_by_patch_chunks(q, k, n_ctx: int, chunk: int, reduce: int = REDUCE_MAX,
                          scale: float | None = None) -> np.ndarray:
    """score() of a long patch (KVzip), evaluated `chunk` patch tokens at a time and combined with
    the same reduction.  q [nb, Hq, p, d].  Returns float64 [nb, Hkv, n_ctx]."""
    p = q.shape[2]
    out = None
    for t0 in range(0, p, chunk):
        part = score(q[:, :, t0:t0 + chunk], k, n_ctx, reduce, scale)
        if out is None:
            out = part
        else:
            out = np.maximum(out, part) if reduce == REDUCE_MAX else out + part
    return out


def score_snapkv(q_window, k, n_ctx: int, reduce: int = REDUCE_MAX, scale: float | None = None) -> np.ndarray:
    """Importance of the rows before the observation window, voted by the window's own queries.

    q_window [nb, Hq, w, d]: query states of the last w context tokens; k [nb, Hkv, C >= n_ctx, d].
    Window token t sits at row n_ctx - w + t and attends to rows 0 .. n_ctx - w + t (itself included).
    Returns float64 [nb, Hkv, n_ctx - w].
    """
    nb, Hq, w, d = q_window.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    n_before = n_ctx - w
    assert n_before >= 0
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty((nb, Hkv, n_before), dtype=np.float64)
    for b in range(nb):
        for h in range(Hkv):
            votes = np.empty((G * w, n_before), dtype=np.float64)
            for g in range(G):
                for t in range(w):
                    visible = np.asarray(k[b, h, :n_before + t + 1], dtype=np.float64)
                    z = scale * (visible @ np.asarray(q_window[b, h * G + g, t], dtype=np.float64))
                    e = np.exp(z - z.max())
                    votes[g * w + t] = e[:n_before] / e.sum()
            if n_before:
                out[b, h] = votes.max(axis=0) if reduce == REDUCE_MAX else votes.sum(axis=0)
    return out


def evict_step_snapkv(q_window, k, v, n_ctx: int, M: int, reduce: int = REDUCE_MAX, scale=None,
                      k_bits=None, v_bits=None):
    """One eviction step with SnapKV's observation window as the patched prompt.

    Keeps the window rows and the M - w best-scoring earlier rows (selection on the scores rounded
    to float32, ties to the lower row), in their original order.
    Returns (scores float64 [nb, Hkv, n_ctx - w], keep_idx int32 [nb, Hkv, min(M, n_ctx)], K', V').
    """
    nb, Hq, w, d = q_window.shape
    Hkv = k.shape[1]
    assert M >= w, "the budget must cover the observation window"
    s = score_snapkv(q_window, k, n_ctx, reduce, scale)
    n_keep = min(M, n_ctx)
    idx = np.empty((nb, Hkv, n_keep), dtype=np.int32)
    window_rows = np.arange(n_ctx - w, n_ctx, dtype=np.int32)
    for b in range(nb):
        for h in range(Hkv):
            if n_ctx <= M:
                idx[b, h] = np.arange(n_ctx, dtype=np.int32)
            else:
                idx[b, h] = np.concatenate([topk_1d(s[b, h].astype(np.float32), M - w), window_rows])
    kk = compact(k if k_bits is None else k_bits, idx)
    vv = compact(v if v_bits is None else v_bits, idx)
    return s, idx, kk, vv


# ---------------------------------------------------------------------------------------------
# KeyDiff scoring (App. A.2, "KeyDiff"): an attention-free baseline that runs on the same
# select / compact back end.  Per KV head the anchor is the average of the key states of all
# context tokens; a token's score is minus the cosine similarity between its key and the anchor,
# so keys that point away from the bulk are kept.
# Reading where the text is silent: a zero key or a zero anchor has cosine 0.
# ---------------------------------------------------------------------------------------------

def score_keydiff(k, n_ctx) -> np.ndarray:
    """k [nb, Hkv, C, d]; n_ctx an int or per-(b, h) lengths.  Returns float64 [nb, Hkv, max n_ctx];
    entries at or beyond a head's own length are NaN."""
    nb, Hkv = k.shape[:2]
    lens = np.broadcast_to(np.asarray(n_ctx), (nb, Hkv))
    out = np.full((nb, Hkv, int(lens.max())), np.nan, dtype=np.float64)
    for b in range(nb):
        for h in range(Hkv):
            n = int(lens[b, h])
            if n == 0:
                continue
            keys = np.asarray(k[b, h, :n], dtype=np.float64)
            anchor = keys.sum(axis=0) / n
            dots = keys @ anchor
            norms = np.sqrt((keys * keys).sum(axis=1)) * math.sqrt(float(anchor @ anchor))
            cos = np.divide(dots, norms, out=np.zeros(n), where=norms > 0)
            out[b, h, :n] = -cos
    return out


# ---------------------------------------------------------------------------------------------
# Episode geometry on segment embeddings (Sec. 3.1): centroid and centroid-closest segment of
# every cluster (Stage 1, Eq. 3) and query-to-episode matching (Stage 3a, with the Stage 3b rule
# that a query too far from every centroid opens a new episode).  The embeddings and the cluster
# assignment are inputs: the encoder and K-Means are outside this library.
# Readings: ties go to the lower index; an empty cluster has a zero centroid and medoid -1; the
# cosine with a zero vector is 0.
# ---------------------------------------------------------------------------------------------

def _cosine(u: np.ndarray, v: np.ndarray) -> float:
    den = math.sqrt(float(u @ u)) * math.sqrt(float(v @ v))
    return float(u @ v) / den if den > 0 else 0.0


def episode_medoids(emb, assign, E: int):
    """Eq. 3.  emb [K, D], assign [K] in 0..E-1.  Returns (centroids float64 [E, D], medoid int32 [E]):
    centroid = mean of the member embeddings, medoid = member with the largest cosine to it."""
    emb = np.asarray(emb, dtype=np.float64)
    K, D = emb.shape
    cent = np.zeros((E, D), dtype=np.float64)
    med = np.full(E, -1, dtype=np.int32)
    for e in range(E):
        members = [k for k in range(K) if assign[k] == e]
        if not members:
            continue
        cent[e] = emb[members].sum(axis=0) / len(members)
        best = -np.inf
        for k in members:                      # ascending k, strict improvement: ties keep the lower k
            c = _cosine(emb[k], cent[e])
            if c > best:
                best, med[e] = c, k
    return cent, med


def match_queries(queries, centroids, tau: float = -np.inf):
    """Stage 3a: e = argmax_e cos(q, c_e) (ties -> lower e); Stage 3b: -1 if that cosine is below tau.
    Returns (episode int32 [nq], cosine float64 [nq])."""
    queries = np.asarray(queries, dtype=np.float64)
    centroids = np.asarray(centroids, dtype=np.float64)
    nq = queries.shape[0]
    ep = np.empty(nq, dtype=np.int32)
    cs = np.empty(nq, dtype=np.float64)
    for i in range(nq):
        best, arg = -np.inf, -1
        for e in range(centroids.shape[0]):
            c = _cosine(queries[i], centroids[e])
            if c > best:
                best, arg = c, e
        cs[i] = best
        ep[i] = arg if best >= tau else -1
    return ep, cs


# ---------------------------------------------------------------------------------------------
# The patch's own attention output.  The patched prompt has to be run through the layer anyway
# (Sec. 2.3: it is appended after the block and attends back to it), so the pass that produces the
# softmax normalisers of Eq. 1 can also produce the patch tokens' attention output
# O_t = sum_i Attn(x_t -> x_i) v_i.  Keys and values of the patch follow the context rows
# (rows n_ctx .. n_ctx + p - 1); with causal_patch they are attended causally, without it the
# softmax runs over the context rows only (the denominators score() uses).
# ---------------------------------------------------------------------------------------------

def patch_attention(q, k, v, n_ctx, causal_patch: bool = True, scale: float | None = None):
    """Returns (O float64 [nb, Hq, p, d], lse float64 [nb, Hq, p]): attention output of every patch
    query and the natural log of its softmax denominator.
    n_ctx: one context length for all heads, or an integer array [nb, Hkv] for caches whose heads hold
    different numbers of tokens (head-wise non-uniform retention, App. A.2): head (b, h) then has its
    context in rows 0 .. n_ctx[b,h]-1 and the patch's keys and values right behind them.  A query with no
    key at all (empty context, no causal patch keys) gets O = 0 and lse = -inf."""
    nb, Hq, p, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    lengths = np.broadcast_to(np.asarray(n_ctx, dtype=np.int64), (nb, Hkv))
    out = np.empty((nb, Hq, p, np.shape(v)[-1]), dtype=np.float64)   # value rows may be wider than d
    lse = np.empty((nb, Hq, p), dtype=np.float64)
    for b in range(nb):
        for hq in range(Hq):
            h = hq // G
            for t in range(p):
                n_keys = int(lengths[b, h]) + (t + 1 if causal_patch else 0)
                if n_keys == 0:
                    out[b, hq, t] = 0.0
                    lse[b, hq, t] = -np.inf
                    continue
                keys = np.asarray(k[b, h, :n_keys], dtype=np.float64)
                vals = np.asarray(v[b, h, :n_keys], dtype=np.float64)
                z = scale * (keys @ np.asarray(q[b, hq, t], dtype=np.float64))
                m = z.max()
                e = np.exp(z - m)
                s = e.sum()
                out[b, hq, t] = (e / s) @ vals
                lse[b, hq, t] = m + math.log(s)
    return out, lse
