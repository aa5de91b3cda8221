"""ctypes binding of libepicache.so: argument marshalling only.

Every function mirrors the C entry point of the same name in include/epicache.h
and takes torch tensors that live on the GPU; the tensors supply device
pointers and strides, torch supplies the current HIP stream.  Nothing is
computed here and there is no fallback: if the library is missing, loading
fails with an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libepicache.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE_TOO_SMALL, ERR_DEVICE = range(5)
DTYPE_F32, DTYPE_BF16 = 0, 1
REDUCE_MAX, REDUCE_SUM = 0, 1
SELECT_PER_HEAD, SELECT_POOLED = 0, 1

ENTRY_POINTS = (
    "epicache_workspace_size", "epicache_score", "epicache_score_lse", "epicache_topk", "epicache_compact",
    "epicache_evict_step", "epicache_evict_step_static", "epicache_evict_step_lse", "epicache_layer_budgets",
    "epicache_overlapped_workspace_size", "epicache_evict_step_overlapped",
    "epicache_ragged_overlapped_workspace_size", "epicache_evict_step_ragged_overlapped",
    "epicache_ragged_workspace_size", "epicache_score_ragged", "epicache_select_ragged", "epicache_compact_ragged",
    "epicache_evict_step_ragged", "epicache_snapkv_workspace_size", "epicache_evict_step_snapkv",
    "epicache_kvzip_workspace_size", "epicache_score_kvzip", "epicache_evict_step_kvzip", "epicache_score_keydiff", "epicache_patch_attention",
    "epicache_patch_attention_ragged",
    "epicache_evict_step_attn",
    "epicache_episode_medoids", "epicache_match_queries", "epicache_status_string", "epicache_version",
)
_INT_RETURNING = ENTRY_POINTS[:-2]


class Params(ctypes.Structure):
    """struct epicache_params"""
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("n_batch", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("n_cached", ctypes.c_int32),
        ("n_block", ctypes.c_int32),
        ("budget", ctypes.c_int32),
        ("patch_len", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("reduce", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float),
        ("causal_patch", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("q_stride_b", ctypes.c_int64),
        ("q_stride_h", ctypes.c_int64),
        ("q_stride_t", ctypes.c_int64),
        ("kv_stride_b", ctypes.c_int64),
        ("kv_stride_h", ctypes.c_int64),
        ("kv_stride_t", ctypes.c_int64),
    ]


class EpicacheError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load the HIP library built in-tree.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2509_17396_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    pp = ctypes.POINTER(Params)
    lib.epicache_workspace_size.argtypes = [pp, ctypes.POINTER(sz)]
    lib.epicache_score.argtypes = [pp, vp, vp, vp, vp, sz, vp]
    lib.epicache_score_lse.argtypes = [pp, vp, vp, vp, vp, vp, sz, vp]
    lib.epicache_topk.argtypes = [pp, vp, vp, vp, sz, vp]
    lib.epicache_compact.argtypes = [pp, vp, vp, vp, vp, sz, vp]
    lib.epicache_evict_step.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.epicache_evict_step_static.argtypes = [pp, vp, vp, vp, vp, vp, vp]
    lib.epicache_evict_step_lse.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.epicache_overlapped_workspace_size.argtypes = [pp, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(sz),
                                                       ctypes.POINTER(ctypes.c_int32)]
    lib.epicache_evict_step_overlapped.argtypes = [pp, vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp, sz, vp, vp]
    lib.epicache_layer_budgets.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int32, ctypes.c_double,
                                           ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    i32c = ctypes.c_int32
    lib.epicache_ragged_workspace_size.argtypes = [pp, i32c, ctypes.POINTER(sz), ctypes.POINTER(i32c)]
    lib.epicache_score_ragged.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.epicache_select_ragged.argtypes = [pp, i32c, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.epicache_compact_ragged.argtypes = [pp, i32c, vp, vp, vp, vp, vp, sz, vp]
    lib.epicache_evict_step_ragged.argtypes = [pp, i32c, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.epicache_ragged_overlapped_workspace_size.argtypes = [pp, i32c, i32c, i32c, ctypes.POINTER(sz),
                                                              ctypes.POINTER(i32c), ctypes.POINTER(i32c)]
    lib.epicache_evict_step_ragged_overlapped.argtypes = [pp, i32c, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32c, vp, sz,
                                                          vp, vp]
    lib.epicache_snapkv_workspace_size.argtypes = [pp, ctypes.POINTER(sz)]
    lib.epicache_evict_step_snapkv.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.epicache_kvzip_workspace_size.argtypes = [pp, ctypes.POINTER(sz)]
    lib.epicache_score_kvzip.argtypes = [pp, vp, vp, vp, vp, sz, vp]
    lib.epicache_evict_step_kvzip.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.epicache_score_keydiff.argtypes = [pp, vp, vp, vp, vp, sz, vp]
    lib.epicache_patch_attention.argtypes = [pp, vp, vp, vp, vp, vp, vp]
    lib.epicache_patch_attention_ragged.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp]
    lib.epicache_evict_step_attn.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.epicache_episode_medoids.argtypes = [vp, vp, i32c, i32c, i32c, vp, vp, vp]
    lib.epicache_match_queries.argtypes = [vp, vp, i32c, i32c, i32c, ctypes.c_float, vp, vp, vp]
    for name in _INT_RETURNING:
        getattr(lib, name).restype = i32
    lib.epicache_status_string.argtypes = [i32]
    lib.epicache_status_string.restype = ctypes.c_char_p
    lib.epicache_version.argtypes = []
    lib.epicache_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().epicache_status_string(int(status)).decode()


def version() -> str:
    return load().epicache_version().decode()


def make_params(q: torch.Tensor, k: torch.Tensor, n_cached: int, n_block: int, budget: int,
                reduce: int = REDUCE_MAX, softmax_scale: float = 0.0, causal_patch: int = 0) -> Params:
    """Fill epicache_params from Q [nb,Hq,p,d] and K [nb,Hkv,C,d] (shapes and strides only)."""
    nb, Hq, p, d = q.shape
    assert q.dtype == k.dtype and q.stride(3) == 1 and k.stride(3) == 1
    dtype = {torch.float32: DTYPE_F32, torch.bfloat16: DTYPE_BF16}[q.dtype]
    return Params(ctypes.sizeof(Params), nb, Hq, k.shape[1], d, n_cached, n_block, budget, p, dtype,
                  reduce, softmax_scale, causal_patch, 0, q.stride(0), q.stride(1), q.stride(2),
                  k.stride(0), k.stride(1), k.stride(2))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != OK:
        raise EpicacheError(status, where)


def epicache_workspace_size(params: Params) -> int:
    out = ctypes.c_size_t(0)
    _check(load().epicache_workspace_size(ctypes.byref(params), ctypes.byref(out)),
           "epicache_workspace_size")
    return out.value


def alloc_workspace(params: Params, device="cuda") -> torch.Tensor:
    return torch.empty(max(epicache_workspace_size(params), 256), dtype=torch.uint8, device=device)


def epicache_score(params: Params, q, k, scores, workspace) -> None:
    _check(load().epicache_score(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(scores),
                                 _ptr(workspace), workspace.numel(), _stream()), "epicache_score")


def epicache_score_lse(params: Params, q, k, row_lse, scores, workspace) -> None:
    _check(load().epicache_score_lse(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(row_lse), _ptr(scores),
                                     _ptr(workspace), workspace.numel(), _stream()), "epicache_score_lse")


def epicache_topk(params: Params, scores, keep_idx, workspace=None) -> None:
    _check(load().epicache_topk(ctypes.byref(params), _ptr(scores), _ptr(keep_idx), _ptr(workspace),
                                0 if workspace is None else workspace.numel(), _stream()),
           "epicache_topk")


def epicache_compact(params: Params, keep_idx, k, v, workspace=None) -> None:
    _check(load().epicache_compact(ctypes.byref(params), _ptr(keep_idx), _ptr(k), _ptr(v),
                                   _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                   _stream()), "epicache_compact")


def epicache_evict_step(params: Params, q, k, v, workspace, scores=None, keep_idx=None) -> None:
    _check(load().epicache_evict_step(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(scores),
                                      _ptr(keep_idx), _ptr(workspace), workspace.numel(), _stream()),
           "epicache_evict_step")


STATIC_SCRATCH_BYTES = 64 << 20


def epicache_evict_step_static(params: Params, q, k, v, scores=None, keep_idx=None) -> None:
    _check(load().epicache_evict_step_static(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(scores),
                                             _ptr(keep_idx), _stream()), "epicache_evict_step_static")


def epicache_overlapped_workspace_size(params: Params, n_chunks: int = 0, with_row_lse: bool = False):
    """(bytes, number of chunks the step will use)"""
    out, used = ctypes.c_size_t(0), ctypes.c_int32(0)
    _check(load().epicache_overlapped_workspace_size(ctypes.byref(params), n_chunks, int(with_row_lse),
                                                     ctypes.byref(out), ctypes.byref(used)),
           "epicache_overlapped_workspace_size")
    return out.value, used.value


def epicache_evict_step_overlapped(params: Params, q, k, v, workspace, aux_stream, n_chunks: int = 0, scores=None,
                                   keep_idx=None, row_lse=None) -> None:
    """aux_stream: a torch.cuda.Stream of the same device (selection and compaction run there)."""
    _check(load().epicache_evict_step_overlapped(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(row_lse),
                                                 _ptr(scores), _ptr(keep_idx), n_chunks, _ptr(workspace),
                                                 workspace.numel(), _stream(),
                                                 ctypes.c_void_p(aux_stream.cuda_stream)),
           "epicache_evict_step_overlapped")


def epicache_evict_step_lse(params: Params, q, k, v, row_lse, workspace, scores=None, keep_idx=None) -> None:
    _check(load().epicache_evict_step_lse(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(row_lse),
                                          _ptr(scores), _ptr(keep_idx), _ptr(workspace), workspace.numel(),
                                          _stream()), "epicache_evict_step_lse")


def epicache_ragged_workspace_size(params: Params, select: int):
    """-> (workspace bytes, keep_capacity)"""
    out, cap = ctypes.c_size_t(0), ctypes.c_int32(0)
    _check(load().epicache_ragged_workspace_size(ctypes.byref(params), int(select), ctypes.byref(out),
                                                 ctypes.byref(cap)), "epicache_ragged_workspace_size")
    return out.value, cap.value


def alloc_ragged_workspace(params: Params, select: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(epicache_ragged_workspace_size(params, select)[0], 256), dtype=torch.uint8,
                       device=device)


def epicache_score_ragged(params: Params, q, k, n_ctx, scores, workspace, row_lse=None) -> None:
    _check(load().epicache_score_ragged(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(n_ctx), _ptr(row_lse),
                                        _ptr(scores), _ptr(workspace), workspace.numel(), _stream()),
           "epicache_score_ragged")


def epicache_select_ragged(params: Params, select: int, scores, n_ctx, budgets, keep_idx, n_kept,
                           workspace) -> None:
    _check(load().epicache_select_ragged(ctypes.byref(params), int(select), _ptr(scores), _ptr(n_ctx),
                                         _ptr(budgets), _ptr(keep_idx), _ptr(n_kept), _ptr(workspace),
                                         workspace.numel(), _stream()), "epicache_select_ragged")


def epicache_compact_ragged(params: Params, select: int, keep_idx, n_kept, k, v, workspace=None) -> None:
    _check(load().epicache_compact_ragged(ctypes.byref(params), int(select), _ptr(keep_idx), _ptr(n_kept),
                                          _ptr(k), _ptr(v), _ptr(workspace),
                                          0 if workspace is None else workspace.numel(), _stream()),
           "epicache_compact_ragged")


def epicache_evict_step_ragged(params: Params, select: int, q, k, v, n_ctx, budgets, n_kept, workspace,
                               scores=None, keep_idx=None, row_lse=None) -> None:
    _check(load().epicache_evict_step_ragged(ctypes.byref(params), int(select), _ptr(q), _ptr(k), _ptr(v),
                                             _ptr(n_ctx), _ptr(budgets), _ptr(row_lse), _ptr(n_kept), _ptr(scores),
                                             _ptr(keep_idx), _ptr(workspace), workspace.numel(), _stream()),
           "epicache_evict_step_ragged")


def epicache_ragged_overlapped_workspace_size(params: Params, select: int, n_chunks: int = 0,
                                              with_row_lse: bool = False):
    """(bytes, keep capacity, number of chunks the step will use)"""
    out, cap, used = ctypes.c_size_t(0), ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load().epicache_ragged_overlapped_workspace_size(ctypes.byref(params), int(select), n_chunks,
                                                            int(with_row_lse), ctypes.byref(out), ctypes.byref(cap),
                                                            ctypes.byref(used)),
           "epicache_ragged_overlapped_workspace_size")
    return out.value, cap.value, used.value


def epicache_evict_step_ragged_overlapped(params: Params, select: int, q, k, v, n_ctx, budgets, n_kept, workspace,
                                          aux_stream, n_chunks: int = 0, scores=None, keep_idx=None,
                                          row_lse=None) -> None:
    _check(load().epicache_evict_step_ragged_overlapped(ctypes.byref(params), int(select), _ptr(q), _ptr(k), _ptr(v),
                                                        _ptr(n_ctx), _ptr(budgets), _ptr(row_lse), _ptr(n_kept),
                                                        _ptr(scores), _ptr(keep_idx), n_chunks, _ptr(workspace),
                                                        workspace.numel(), _stream(),
                                                        ctypes.c_void_p(aux_stream.cuda_stream)),
           "epicache_evict_step_ragged_overlapped")


def epicache_patch_attention(params: Params, q, k, v, out, lse_out) -> None:
    _check(load().epicache_patch_attention(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse_out),
                                           _stream()), "epicache_patch_attention")


def epicache_patch_attention_ragged(params: Params, q, k, v, n_ctx, out, lse_out) -> None:
    _check(load().epicache_patch_attention_ragged(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(n_ctx),
                                                  _ptr(out), _ptr(lse_out), _stream()),
           "epicache_patch_attention_ragged")


def epicache_evict_step_attn(params: Params, q, k, v, out, workspace, scores=None, keep_idx=None) -> None:
    _check(load().epicache_evict_step_attn(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(scores),
                                           _ptr(keep_idx), _ptr(workspace), workspace.numel(), _stream()),
           "epicache_evict_step_attn")


def epicache_snapkv_workspace_size(params: Params) -> int:
    out = ctypes.c_size_t(0)
    _check(load().epicache_snapkv_workspace_size(ctypes.byref(params), ctypes.byref(out)), "epicache_snapkv_workspace_size")
    return out.value


def epicache_evict_step_snapkv(params: Params, q_window, k, v, workspace, scores=None, keep_idx=None) -> None:
    _check(load().epicache_evict_step_snapkv(ctypes.byref(params), _ptr(q_window), _ptr(k), _ptr(v), _ptr(scores),
                                             _ptr(keep_idx), _ptr(workspace), workspace.numel(), _stream()),
           "epicache_evict_step_snapkv")


def epicache_kvzip_workspace_size(params: Params) -> int:
    out = ctypes.c_size_t(0)
    _check(load().epicache_kvzip_workspace_size(ctypes.byref(params), ctypes.byref(out)), "epicache_kvzip_workspace_size")
    return out.value


def epicache_score_kvzip(params: Params, q, k, scores, workspace) -> None:
    _check(load().epicache_score_kvzip(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(scores), _ptr(workspace),
                                       workspace.numel(), _stream()), "epicache_score_kvzip")


def epicache_evict_step_kvzip(params: Params, q, k, v, workspace, scores=None, keep_idx=None) -> None:
    _check(load().epicache_evict_step_kvzip(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(scores),
                                            _ptr(keep_idx), _ptr(workspace), workspace.numel(), _stream()),
           "epicache_evict_step_kvzip")


def epicache_score_keydiff(params: Params, k, scores, workspace, n_ctx=None) -> None:
    _check(load().epicache_score_keydiff(ctypes.byref(params), _ptr(k), _ptr(n_ctx), _ptr(scores),
                                         _ptr(workspace), workspace.numel(), _stream()), "epicache_score_keydiff")


def epicache_episode_medoids(embeddings, assignment, n_episodes: int, centroids, medoid) -> None:
    K, D = embeddings.shape
    assert embeddings.dtype == torch.float32 and embeddings.is_contiguous() and assignment.dtype == torch.int32
    _check(load().epicache_episode_medoids(_ptr(embeddings), _ptr(assignment), K, int(n_episodes), D,
                                           _ptr(centroids), _ptr(medoid), _stream()), "epicache_episode_medoids")


def epicache_match_queries(queries, centroids, tau: float, episode, cosine=None) -> None:
    nq, D = queries.shape
    assert queries.dtype == torch.float32 and queries.is_contiguous() and centroids.is_contiguous()
    _check(load().epicache_match_queries(_ptr(queries), _ptr(centroids), nq, centroids.shape[0], D, float(tau),
                                         _ptr(episode), _ptr(cosine), _stream()), "epicache_match_queries")


def epicache_layer_budgets(sensitivity, alpha: float, budget: int):
    """Eq. 6 on the host: integer per-layer budgets that sum to len(sensitivity) * budget."""
    n = len(sensitivity)
    sens = (ctypes.c_double * n)(*[float(x) for x in sensitivity])
    out = (ctypes.c_int32 * n)()
    _check(load().epicache_layer_budgets(sens, n, float(alpha), int(budget), out), "epicache_layer_budgets")
    return list(out)
