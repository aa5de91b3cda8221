"""The C-ABI library: it loads, exports what include/epicache.h declares, and its
host-side validation returns the documented status codes.  No GPU needed: every
call here fails validation before anything is enqueued (or is pure host code)."""
import ctypes
import os
import re

import pytest
import torch

from paper_2509_17396_amd import binding as ep

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _params(**kw):
    q = torch.empty(2, 8, 16, 128, dtype=torch.bfloat16)
    k = torch.empty(2, 2, 640, 128, dtype=torch.bfloat16)
    prm = ep.make_params(q, k, n_cached=512, n_block=128, budget=512, reduce=ep.REDUCE_SUM)
    for name, val in kw.items():
        setattr(prm, name, val)
    return prm


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "epicache.h")).read()
    declared = re.findall(r"EPICACHE_API\s+[\w\s\*]+?\b(epicache_\w+)\s*\(", header)
    assert set(declared) == set(ep.ENTRY_POINTS) and len(declared) == len(ep.ENTRY_POINTS)
    lib = ep.load()
    for name in declared:
        assert getattr(lib, name) is not None
    assert re.fullmatch(r"\d+\.\d+\.\d+", ep.version())


def test_header_is_plain_c(tmp_path):
    """include/epicache.h compiles as C99 and as C++ with warnings on, and the struct layout the ctypes
    binding assumes is the one a C compiler produces."""
    import subprocess
    src = tmp_path / "abi_check.c"
    src.write_text(
        '#include <stddef.h>\n#include <stdio.h>\n#include "epicache.h"\n'
        "int main(void) {\n"
        "  epicache_params p; (void)p;\n"
        '  printf("%zu %zu %zu\\n", sizeof(epicache_params), offsetof(epicache_params, q_stride_b),\n'
        "         offsetof(epicache_params, causal_patch));\n"
        "  return (int)(EPICACHE_SELECT_POOLED - 1 + EPICACHE_REDUCE_SUM - 1 + EPICACHE_DTYPE_BF16 - 1);\n"
        "}\n")
    inc = os.path.join(ROOT, "include")
    exe = tmp_path / "abi_check"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, str(src), "-o", str(exe)],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(x) for x in out] == [ctypes.sizeof(ep.Params), ep.Params.q_stride_b.offset,
                                     ep.Params.causal_patch.offset]
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc,
                    str(src)], check=True)


def test_params_struct_matches_header_layout():
    assert ctypes.sizeof(ep.Params) == 4 * 14 + 8 * 6
    assert ep.Params.q_stride_b.offset == 56


def test_status_strings():
    seen = {ep.status_string(s) for s in range(5)}
    assert len(seen) == 5 and ep.status_string(99) == "unknown status"


def test_workspace_size_is_host_only_and_monotone():
    small = ep.epicache_workspace_size(_params())
    assert small > 0 and small % 256 == 0
    assert ep.epicache_workspace_size(_params(patch_len=8, q_stride_h=8 * 128)) <= small


@pytest.mark.parametrize("field,value,status", [
    ("struct_size", 4, ep.ERR_INVALID_ARG),
    ("n_batch", 0, ep.ERR_INVALID_ARG),
    ("budget", 0, ep.ERR_INVALID_ARG),
    ("patch_len", 0, ep.ERR_INVALID_ARG),
    ("n_kv_heads", 3, ep.ERR_INVALID_ARG),       # 8 % 3 != 0
    ("dtype", 7, ep.ERR_INVALID_ARG),
    ("reduce", 2, ep.ERR_INVALID_ARG),
    ("softmax_scale", -1.0, ep.ERR_INVALID_ARG),
    ("softmax_scale", float("nan"), ep.ERR_INVALID_ARG),
    ("softmax_scale", 2.0e6, ep.ERR_UNSUPPORTED),
    ("causal_patch", 2, ep.ERR_INVALID_ARG),
    ("causal_patch", 1, ep.ERR_INVALID_ARG),      # capacity 640 = N: no room for the 16 patch keys
    ("reserved", 1, ep.ERR_INVALID_ARG),
    ("n_block", -600, ep.ERR_INVALID_ARG),
    ("kv_stride_t", 64, ep.ERR_INVALID_ARG),     # rows would overlap
    ("kv_stride_t", 132, ep.ERR_INVALID_ARG),    # not a multiple of 8
    ("kv_stride_h", 1000, ep.ERR_INVALID_ARG),   # capacity below N
    ("head_dim", 12, ep.ERR_UNSUPPORTED),
    ("patch_len", 2048, ep.ERR_INVALID_ARG),     # the Q strides of the fixture do not hold 2048 rows per head
    ("kv_stride_t", 1 << 21, ep.ERR_UNSUPPORTED),  # token stride beyond the 32-bit row offsets of the kernels
    ("n_cached", (1 << 24) + 8, ep.ERR_INVALID_ARG),  # exceeds the capacity the strides imply
])
def test_bad_params_are_rejected_before_any_launch(field, value, status):
    prm = _params(**{field: value})
    out = ctypes.c_size_t(0)
    lib = ep.load()
    assert lib.epicache_workspace_size(ctypes.byref(prm), ctypes.byref(out)) == status
    # the compute entry points validate params first, with the same result
    dummy = ctypes.c_void_p(4096)
    assert lib.epicache_score(ctypes.byref(prm), dummy, dummy, dummy, dummy, 1 << 30, None) == status
    assert lib.epicache_score_lse(ctypes.byref(prm), dummy, dummy, dummy, dummy, dummy, 1 << 30, None) == status
    assert lib.epicache_topk(ctypes.byref(prm), dummy, dummy, None, 0, None) == status
    assert lib.epicache_compact(ctypes.byref(prm), dummy, dummy, ctypes.c_void_p(8192), None, 0, None) == status
    assert lib.epicache_evict_step(ctypes.byref(prm), dummy, dummy, ctypes.c_void_p(8192), None, None,
                                   dummy, 1 << 30, None) == status


def test_static_scratch_entry_point_refuses_oversized_requests_on_the_host():
    q = torch.empty(64, 32, 256, 128, dtype=torch.bfloat16, device="meta")
    k = torch.empty(64, 8, 24576, 128, dtype=torch.bfloat16, device="meta")
    prm = ep.make_params(q, k, n_cached=16384, n_block=8192, budget=16384, reduce=ep.REDUCE_SUM)
    assert ep.epicache_workspace_size(prm) > ep.STATIC_SCRATCH_BYTES
    a, b = ctypes.c_void_p(4096), ctypes.c_void_p(8192)
    lib = ep.load()
    assert lib.epicache_evict_step_static(ctypes.byref(prm), a, a, b, None, None, None) == ep.ERR_WORKSPACE_TOO_SMALL
    assert lib.epicache_evict_step_static(ctypes.byref(_params(budget=0)), a, a, b, None, None, None) == ep.ERR_INVALID_ARG


def test_null_misaligned_and_small_workspace_are_rejected():
    prm = _params()
    lib = ep.load()
    a, b, c = ctypes.c_void_p(4096), ctypes.c_void_p(8192), ctypes.c_void_p(4100)
    need = ep.epicache_workspace_size(prm)
    assert lib.epicache_workspace_size(ctypes.byref(prm), None) == ep.ERR_INVALID_ARG
    assert lib.epicache_workspace_size(None, ctypes.byref(ctypes.c_size_t())) == ep.ERR_INVALID_ARG
    assert lib.epicache_score(ctypes.byref(prm), None, a, a, a, need, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_score(ctypes.byref(prm), a, c, a, a, need, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_score(ctypes.byref(prm), a, a, a, a, 16, None) == ep.ERR_WORKSPACE_TOO_SMALL
    assert lib.epicache_score_lse(ctypes.byref(prm), a, a, None, a, a, need, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_score_lse(ctypes.byref(prm), a, a, a, a, a, 16, None) == ep.ERR_WORKSPACE_TOO_SMALL
    assert lib.epicache_topk(ctypes.byref(prm), a, None, None, 0, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_compact(ctypes.byref(prm), a, a, a, None, 0, None) == ep.ERR_INVALID_ARG  # K is V
    assert lib.epicache_compact(ctypes.byref(prm), a, a, None, None, 0, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_evict_step(ctypes.byref(prm), a, a, b, None, None, a, need - 1, None) == \
        ep.ERR_WORKSPACE_TOO_SMALL
    assert lib.epicache_evict_step(ctypes.byref(prm), a, a, a, None, None, a, need, None) == ep.ERR_INVALID_ARG


def test_ragged_calls_validate_on_the_host():
    prm = _params()
    lib = ep.load()
    a, b = ctypes.c_void_p(4096), ctypes.c_void_p(8192)
    for select, cap in ((ep.SELECT_PER_HEAD, 512), (ep.SELECT_POOLED, 640)):   # min(M, N) and min(Hkv*M, N)
        need, got_cap = ep.epicache_ragged_workspace_size(prm, select)
        assert got_cap == cap and need % 256 == 0 and need > ep.epicache_workspace_size(prm) - 256
    need, _ = ep.epicache_ragged_workspace_size(prm, ep.SELECT_POOLED)
    sz, cap = ctypes.c_size_t(), ctypes.c_int32()
    assert lib.epicache_ragged_workspace_size(ctypes.byref(prm), 2, ctypes.byref(sz), ctypes.byref(cap)) == \
        ep.ERR_INVALID_ARG                                                      # unknown selection rule
    assert lib.epicache_ragged_workspace_size(ctypes.byref(prm), 0, None, ctypes.byref(cap)) == ep.ERR_INVALID_ARG
    assert lib.epicache_score_ragged(ctypes.byref(prm), a, a, None, None, a, a, need, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_score_ragged(ctypes.byref(prm), a, a, a, None, a, a, 16, None) == ep.ERR_WORKSPACE_TOO_SMALL
    assert lib.epicache_select_ragged(ctypes.byref(prm), 1, a, a, None, a, None, a, need, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_select_ragged(ctypes.byref(prm), 1, a, a, None, a, a, a, need - 1, None) == \
        ep.ERR_WORKSPACE_TOO_SMALL
    assert lib.epicache_select_ragged(ctypes.byref(prm), 5, a, a, None, a, a, a, need, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_compact_ragged(ctypes.byref(prm), 0, a, a, a, a, None, 0, None) == ep.ERR_INVALID_ARG  # K is V
    assert lib.epicache_compact_ragged(ctypes.byref(prm), 0, a, None, a, b, None, 0, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_evict_step_ragged(ctypes.byref(prm), 1, a, a, b, a, None, None, None, None, None, a, need,
                                          None) == ep.ERR_INVALID_ARG          # n_kept is required
    assert lib.epicache_evict_step_ragged(ctypes.byref(prm), 1, a, a, b, a, None, None, a, None, None, a, need - 1,
                                          None) == ep.ERR_WORKSPACE_TOO_SMALL
    bad = _params(budget=0)
    assert lib.epicache_evict_step_ragged(ctypes.byref(bad), 1, a, a, b, a, None, None, a, None, None, a, need,
                                          None) == ep.ERR_INVALID_ARG
    # pooled selection keeps its per-head counters on chip: at most 1024 KV heads
    q = torch.empty(1, 2048, 1, 8, dtype=torch.float32)
    k = torch.empty(1, 2048, 16, 8, dtype=torch.float32)
    wide = ep.make_params(q, k, n_cached=0, n_block=16, budget=4)
    assert ep.epicache_ragged_workspace_size(wide, ep.SELECT_PER_HEAD)[1] == 4
    with pytest.raises(ep.EpicacheError) as ei:
        ep.epicache_ragged_workspace_size(wide, ep.SELECT_POOLED)
    assert ei.value.status == ep.ERR_UNSUPPORTED


def test_keydiff_and_episode_calls_validate_on_the_host():
    prm = _params()
    lib = ep.load()
    a = ctypes.c_void_p(4096)
    need = ep.epicache_workspace_size(prm)
    assert lib.epicache_score_keydiff(ctypes.byref(prm), None, None, a, a, need, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_score_keydiff(ctypes.byref(prm), a, None, a, a, 16, None) == ep.ERR_WORKSPACE_TOO_SMALL
    assert lib.epicache_score_keydiff(ctypes.byref(prm), a, ctypes.c_void_p(4100), a, a, need, None) == \
        ep.ERR_INVALID_ARG
    b = ctypes.c_void_p(8192)
    assert lib.epicache_patch_attention(ctypes.byref(prm), a, a, a, None, a, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_patch_attention(ctypes.byref(prm), a, a, a, a, b, None) == ep.ERR_INVALID_ARG   # out is q
    assert lib.epicache_patch_attention(ctypes.byref(_params(budget=0)), a, a, a, b, b, None) == ep.ERR_INVALID_ARG
    ragged = lib.epicache_patch_attention_ragged
    assert ragged(ctypes.byref(prm), a, a, a, None, b, b, None) == ep.ERR_INVALID_ARG                   # no lengths
    assert ragged(ctypes.byref(prm), a, a, a, ctypes.c_void_p(4100), b, b, None) == ep.ERR_INVALID_ARG  # alignment
    assert ragged(ctypes.byref(prm), a, a, a, a, a, b, None) == ep.ERR_INVALID_ARG                      # out is q
    c, d = ctypes.c_void_p(12288), ctypes.c_void_p(16384)
    step = lib.epicache_evict_step_attn
    assert step(ctypes.byref(prm), a, b, c, None, None, None, d, need, None) == ep.ERR_INVALID_ARG     # no out
    assert step(ctypes.byref(prm), a, b, b, d, None, None, d, need, None) == ep.ERR_INVALID_ARG        # k is v
    assert step(ctypes.byref(prm), a, b, c, b, None, None, d, need, None) == ep.ERR_INVALID_ARG        # out is k
    assert step(ctypes.byref(prm), a, b, c, ctypes.c_void_p(20480), None, None, d, 16, None) == \
        ep.ERR_WORKSPACE_TOO_SMALL
    assert step(ctypes.byref(prm), a, b, c, ctypes.c_void_p(20484), None, None, d, need, None) == \
        ep.ERR_INVALID_ARG                                                                             # alignment
    assert lib.epicache_episode_medoids(a, a, 10, 0, 8, a, a, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_episode_medoids(a, None, 10, 2, 8, a, a, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_episode_medoids(a, a, 10, 2, 10000, a, a, None) == ep.ERR_UNSUPPORTED
    assert lib.epicache_match_queries(a, a, 0, 2, 8, 0.5, a, None, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_match_queries(a, a, 3, 2, 8, float("nan"), a, None, None) == ep.ERR_INVALID_ARG
    assert lib.epicache_match_queries(a, a, 3, 2, 8, 0.5, None, None, None) == ep.ERR_INVALID_ARG


def test_binding_raises_with_status():
    with pytest.raises(ep.EpicacheError) as ei:
        ep.epicache_workspace_size(_params(budget=-3))
    assert ei.value.status == ep.ERR_INVALID_ARG


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No CPU fallback: without the built HIP library the binding raises."""
    monkeypatch.setattr(ep, "_lib", None)
    monkeypatch.setattr(ep, "_LIB_PATH", str(tmp_path / "libepicache.so"))
    with pytest.raises(FileNotFoundError):
        ep.load()
    with pytest.raises(FileNotFoundError):
        ep.epicache_workspace_size(_params())


def test_product_package_never_imports_the_oracle():
    import pathlib
    pkg = pathlib.Path(ROOT) / "paper_2509_17396_amd"
    for path in list(pkg.rglob("*.py")) + list(pkg.rglob("*.hip")) + list(pkg.rglob("*.h")):
        text = path.read_text()
        assert "oracle" not in text.lower() or path.name == "synth.py", path
