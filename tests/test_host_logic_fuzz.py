"""Host-side logic under random parameters (no GPU): the validator never crashes, accepts every
well-formed geometry inside the documented envelope, rejects what lies outside it with the documented
status, and the workspace sizes it reports cover every buffer a step keeps there."""
import ctypes

import torch
from hypothesis import given, settings, strategies as st

from paper_2509_17396_amd import binding as ep


def _dense_params(nb, Hkv, G, p, d, n_cached, n_block, budget, dtype, reduce, causal, extra_rows, pad):
    Hq = Hkv * G
    cap = n_cached + n_block + (p if causal else 0) + extra_rows
    kst = d + 8 * pad
    prm = ep.Params(ctypes.sizeof(ep.Params), nb, Hq, Hkv, d, n_cached, n_block, budget, p, dtype, reduce, 0.0,
                    causal, 0, Hq * p * d, p * d, d, Hkv * cap * kst, cap * kst, kst)
    return prm


geometry = st.tuples(
    st.integers(1, 6), st.integers(1, 8), st.integers(1, 7), st.integers(1, 300),
    st.sampled_from([8, 16, 40, 64, 96, 128, 256]), st.integers(0, 5000), st.integers(0, 5000),
    st.integers(1, 6000), st.sampled_from([ep.DTYPE_F32, ep.DTYPE_BF16]),
    st.sampled_from([ep.REDUCE_MAX, ep.REDUCE_SUM]), st.integers(0, 1), st.integers(0, 50), st.integers(0, 3))


@settings(max_examples=300, deadline=None)
@given(geometry)
def test_well_formed_geometries_are_accepted_and_sized(g):
    nb, Hkv, G, p, d, n_cached, n_block, budget, dtype, reduce, causal, extra, pad = g
    prm = _dense_params(*g)
    lib = ep.load()
    size = ctypes.c_size_t(0)
    status = lib.epicache_workspace_size(ctypes.byref(prm), ctypes.byref(size))
    N, R = n_cached + n_block, G * p
    if N < 1:
        assert status == ep.ERR_INVALID_ARG
        return
    if R > 16384:
        assert status == ep.ERR_UNSUPPORTED
        return
    assert status == ep.OK, (g, status)
    nbh = nb * Hkv
    n_keep = min(budget, N)
    # scores, kept indices and at least one (max, sum) pair per scoring row all live in the workspace
    assert size.value >= nbh * N * 4 + nbh * n_keep * 4 + nbh * R * 8
    assert size.value % 256 == 0
    for select in (ep.SELECT_PER_HEAD, ep.SELECT_POOLED):
        rsize, cap = ctypes.c_size_t(0), ctypes.c_int32(0)
        assert lib.epicache_ragged_workspace_size(ctypes.byref(prm), select, ctypes.byref(rsize),
                                                  ctypes.byref(cap)) == ep.OK
        want_cap = min(N, budget if select == ep.SELECT_PER_HEAD else Hkv * budget)
        assert cap.value == want_cap
        assert rsize.value >= nbh * N * 4 + nbh * want_cap * 4 + nbh * 8


@settings(max_examples=200, deadline=None)
@given(geometry, st.sampled_from(["kv_stride_t", "kv_stride_h", "kv_stride_b", "q_stride_t", "q_stride_h",
                                  "q_stride_b", "n_q_heads", "head_dim", "struct_size", "reserved"]),
       st.integers(1, 7))
def test_broken_geometries_are_rejected(g, field, delta):
    nb, Hkv, G, p, d, n_cached, n_block = g[:7]
    if n_cached + n_block < 1 or G * p > 16384:
        return
    prm = _dense_params(*g)
    if field.endswith("stride_t") or field.endswith("stride_h") or field.endswith("stride_b"):
        setattr(prm, field, getattr(prm, field) - delta)          # no longer a multiple of 8, or rows overlap
        if field.endswith("_b") and nb == 1 and (getattr(prm, field) % 8 == 0):
            return                                                 # the batch stride of a single item is not read
    elif field == "n_q_heads":
        if Hkv == 1:
            return
        prm.n_q_heads = prm.n_q_heads + (1 if (prm.n_q_heads + 1) % Hkv else 2) if Hkv > 2 else prm.n_q_heads + 1
        if prm.n_q_heads % Hkv == 0:
            return
    elif field == "head_dim":
        prm.head_dim = d + delta                                   # not a multiple of 8 (delta < 8)
    elif field == "struct_size":
        prm.struct_size = prm.struct_size - delta
    elif field == "reserved":
        prm.reserved = delta
    size = ctypes.c_size_t(0)
    status = ep.load().epicache_workspace_size(ctypes.byref(prm), ctypes.byref(size))
    assert status in (ep.ERR_INVALID_ARG, ep.ERR_UNSUPPORTED), (g, field, delta, status)


@settings(max_examples=300, deadline=None)
@given(geometry)
def test_snapkv_and_kvzip_plans_never_crash_and_follow_their_rules(g):
    nb, Hkv, G, p, d, n_cached, n_block, budget, dtype, reduce, causal, extra, pad = g
    prm = _dense_params(*g)
    lib = ep.load()
    N, R = n_cached + n_block, G * p
    size = ctypes.c_size_t(0)
    plain = lib.epicache_workspace_size(ctypes.byref(prm), ctypes.byref(size))
    # SnapKV: the window (p rows) is part of the N context rows
    st_s = lib.epicache_snapkv_workspace_size(ctypes.byref(prm), ctypes.byref(size))
    if plain != ep.OK:
        assert st_s == plain
    elif causal:
        assert st_s == ep.ERR_INVALID_ARG          # the call applies the window's mask itself
    elif N > budget and budget <= p:
        assert st_s == ep.ERR_INVALID_ARG          # the window alone would use up the budget
    else:
        # the window rows follow the rows that are scored: the same capacity as the plain step
        assert st_s == ep.OK, (g, st_s)
        assert size.value % 256 == 0 and size.value >= nb * Hkv * min(budget, N) * 4
    # KVzip: any patch length; the same answer as the plain call where that accepts the patch
    st_k = lib.epicache_kvzip_workspace_size(ctypes.byref(prm), ctypes.byref(size))
    if N < 1:
        assert st_k == ep.ERR_INVALID_ARG
    elif causal:
        assert st_k == ep.ERR_INVALID_ARG
    else:
        assert st_k == ep.OK, (g, st_k)
        assert size.value % 256 == 0 and size.value >= 2 * nb * Hkv * N * 4 + nb * Hkv * min(budget, N) * 4


@settings(max_examples=300, deadline=None)
@given(geometry, st.integers(-2, 70))
def test_overlapped_plans_cover_the_batch_and_their_chunks(g, asked):
    nb, Hkv, G, p, d, n_cached, n_block, budget, dtype, reduce, causal, extra, pad = g
    prm = _dense_params(*g)
    lib = ep.load()
    size, plain, used = ctypes.c_size_t(0), ctypes.c_size_t(0), ctypes.c_int32(-1)
    st_plain = lib.epicache_workspace_size(ctypes.byref(prm), ctypes.byref(plain))
    st_o = lib.epicache_overlapped_workspace_size(ctypes.byref(prm), asked, 0, ctypes.byref(size), ctypes.byref(used))
    if st_plain != ep.OK:
        assert st_o == st_plain
        return
    if asked < 0 or asked > 64:
        assert st_o == ep.ERR_INVALID_ARG
        return
    assert st_o == ep.OK, (g, asked, st_o)
    n = used.value
    assert 1 <= n <= min(64, nb)
    if asked:
        # chunks of ceil(nb / asked) batch items each, the last one shorter
        per = -(-nb // min(asked, nb))
        assert n == -(-nb // per)
    per = -(-nb // n)
    # every chunk's slice is the workspace of a step over that chunk
    one = _dense_params(per, *g[1:])
    body = ctypes.c_size_t(0)
    assert lib.epicache_workspace_size(ctypes.byref(one), ctypes.byref(body)) == ep.OK
    tail_nb = nb - (n - 1) * per
    assert 1 <= tail_nb <= per
    tail = ctypes.c_size_t(0)
    assert lib.epicache_workspace_size(ctypes.byref(_dense_params(tail_nb, *g[1:])), ctypes.byref(tail)) == ep.OK
    assert size.value == (n - 1) * body.value + tail.value
    if n == 1:
        assert size.value == plain.value


def test_overlapped_chunk_choice_for_the_benchmarked_workloads():
    """The library's own chunk count (n_chunks = 0): chunks of about 64 (item, head) pairs that still score for a
    tenth of a millisecond each, none where the scoring has fewer than 256 rows per head."""
    from paper_2509_17396_amd import synth
    want = {"tiny": 1, "llama32_3b": 1, "llama31_8b": 16, "qwen25_7b": 14, "stress": 64}
    with_lse = {"tiny": 1, "llama32_3b": 1, "llama31_8b": 8, "qwen25_7b": 8, "stress": 64}
    for name, chunks in want.items():
        w = synth.WORKLOADS[name]
        nb, cap = w.L * w.E, w.M + w.B
        dtype = ep.DTYPE_F32 if w.dtype == "f32" else ep.DTYPE_BF16
        prm = ep.Params(ctypes.sizeof(ep.Params), nb, w.Hq, w.Hkv, w.d, w.M, w.B, w.M, w.p, dtype, ep.REDUCE_SUM, 0.0,
                        0, 0, w.Hq * w.p * w.d, w.p * w.d, w.d, w.Hkv * cap * w.d, cap * w.d, w.d)
        size, used = ctypes.c_size_t(0), ctypes.c_int32(0)
        assert ep.load().epicache_overlapped_workspace_size(ctypes.byref(prm), 0, 0, ctypes.byref(size),
                                                            ctypes.byref(used)) == ep.OK
        assert used.value == chunks, (name, used.value)
        # with the caller's normalisers the scoring is one pass: half the work per chunk
        assert ep.load().epicache_overlapped_workspace_size(ctypes.byref(prm), 0, 1, ctypes.byref(size),
                                                            ctypes.byref(used)) == ep.OK
        assert used.value == with_lse[name], (name, used.value)


@settings(max_examples=200, deadline=None)
@given(geometry, st.integers(1, 64), st.sampled_from([ep.SELECT_PER_HEAD, ep.SELECT_POOLED]))
def test_ragged_overlapped_plans_are_sums_of_ragged_chunk_plans(g, asked, select):
    nb, Hkv, G, p, d, n_cached, n_block, budget, dtype, reduce, causal, extra, pad = g
    prm = _dense_params(*g)
    lib = ep.load()
    plain, cap = ctypes.c_size_t(0), ctypes.c_int32(0)
    st_plain = lib.epicache_ragged_workspace_size(ctypes.byref(prm), select, ctypes.byref(plain), ctypes.byref(cap))
    size, cap_o, used = ctypes.c_size_t(0), ctypes.c_int32(-1), ctypes.c_int32(-1)
    st_o = lib.epicache_ragged_overlapped_workspace_size(ctypes.byref(prm), select, asked, 0, ctypes.byref(size),
                                                         ctypes.byref(cap_o), ctypes.byref(used))
    assert st_o == st_plain
    if st_plain != ep.OK:
        return
    assert cap_o.value == cap.value
    per = -(-nb // min(asked, nb))
    n = -(-nb // per)
    assert used.value == n
    body, tail, c2 = ctypes.c_size_t(0), ctypes.c_size_t(0), ctypes.c_int32(0)
    assert lib.epicache_ragged_workspace_size(ctypes.byref(_dense_params(per, *g[1:])), select, ctypes.byref(body),
                                              ctypes.byref(c2)) == ep.OK
    assert lib.epicache_ragged_workspace_size(ctypes.byref(_dense_params(nb - (n - 1) * per, *g[1:])), select,
                                              ctypes.byref(tail), ctypes.byref(c2)) == ep.OK
    assert size.value == (n - 1) * body.value + tail.value
