"""The hand-written VALU instructions of the MFMA kernels against the wait states the hardware needs.

The compiler inserts the wait states that gfx950 requires between an MFMA and the first vector ALU instruction
that reads its result, and between a transcendental and a reader of its result, but only for instructions it
generated itself: an inline-assembly `v_max3_f32` placed straight behind an MFMA reads the accumulator before
the matrix core has written it.  This test compiles the two MFMA sources to ISA (device side only, a few
seconds each) and walks every control-flow path from each MFMA / transcendental to the inline-assembly
instructions behind it."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2509_17396_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
MFMA_8_PASS_WAIT_STATES = 12   # passes + 3, + 1 on gfx950
TRANS_WAIT_STATES = 1


def _regs(tok):
    tok = tok.strip()
    m = re.match(r"([va])\[(\d+):(\d+)\]", tok)
    if m:
        return {(m.group(1), r) for r in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = re.match(r"([va])(\d+)$", tok)
    return {(m.group(1), int(m.group(2)))} if m else set()


def _kernels(text):
    """Yields (name, instructions, labels); an instruction is (text, written_by_hand)."""
    name, ins, labels, by_hand = None, [], {}, False
    for line in text.splitlines():
        s = line.strip()
        if re.match(r"^_Z\w+:", s):
            name, ins, labels = s[:-1], [], {}
        elif s.startswith(";;#ASMSTART"):
            by_hand = True
        elif s.startswith(";;#ASMEND"):
            by_hand = False
        elif re.match(r"^\.LBB\w+:", s):
            labels[s.split(":")[0]] = len(ins)
        elif s.startswith(".Lfunc_end"):     # a kernel can hold several s_endpgm; this closes it
            if ins:
                yield name, ins, labels
            ins, labels = [], {}
        elif s and not s.startswith((".", ";", "//")) and not s.endswith(":"):
            ins.append((s.split(";")[0].strip(), by_hand))


def _sources(text):
    ops = text.split(None, 1)[1].split(",")
    return set().union(*[_regs(o) for o in ops[1:]]) if len(ops) > 1 else set()


def exposed_readers(ins, labels, is_producer, need):
    """Inline-assembly VALU instructions that read a producer's result fewer than `need` wait states behind it
    on some path.  A compiler-generated VALU reader ends a path: the compiler has put the wait states in front
    of it."""
    found = []
    for i, (text, _) in enumerate(ins):
        if not is_producer(text):
            continue
        dst = _regs(text.split(None, 1)[1].split(",")[0])
        seen, work = set(), [(i + 1, 0)]
        while work:
            j, ws = work.pop()
            while j < len(ins) and ws < need and (j, ws) not in seen:
                seen.add((j, ws))
                u, by_hand = ins[j]
                op = u.split()[0]
                if op.startswith("v_") and "mfma" not in op and _sources(u) & dst:
                    if by_hand:
                        found.append((ws, text, u))
                    break
                if op == "s_endpgm":
                    break
                m = re.match(r"s_nop (\d+)", u)
                ws_next = ws + (int(m.group(1)) + 1 if m else 1)
                if op.startswith("s_cbranch") or op == "s_branch":
                    target = u.split()[1]
                    if target in labels:
                        work.append((labels[target], ws_next))
                    if op == "s_branch":
                        break
                j, ws = j + 1, ws_next
    return found


def _sregs(tok):
    tok = tok.strip()
    m = re.match(r"s\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"s(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def hand_written_sgpr_readers_behind_valu(ins, need):
    """Hand-written instructions (the direct global->LDS loads and the s_mov to M0 in front of them) that read
    an SGPR a vector instruction (v_readfirstlane and the like) wrote fewer than `need` wait states before, in
    straight-line order: the hardware needs 5 between a VALU write of an SGPR and a memory instruction reading it."""
    found = []
    for i, (text, by_hand) in enumerate(ins):
        parts = text.split(None, 1)
        if not by_hand or len(parts) < 2 or parts[0].startswith("v_"):
            continue
        ops = parts[1].split(",")
        use = set().union(*[_sregs(o) for o in (ops[1:] if parts[0].startswith("s_mov") else ops)])
        ws = 0
        for j in range(i - 1, -1, -1):
            if ws >= need or not use:
                break
            u = ins[j][0].split(None, 1)
            if u[0].startswith("v_") and len(u) > 1 and _sregs(u[1].split(",")[0]) & use:
                found.append((ws, ins[j][0], text))
                break
            m = re.match(r"s_nop (\d+)", ins[j][0])
            ws += int(m.group(1)) + 1 if m else 1
    return found


def _isa(source):
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only", "-S", "-o", "-",
           os.path.join(CSRC, source)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    return res.stdout


def test_the_checker_finds_a_planted_exposure():
    ins = [("v_mfma_f32_32x32x16_bf16 v[68:83], v[236:239], v[108:111], v[68:83]", False),
           ("s_cbranch_scc1 .LBB0_1", False),
           ("v_mov_b32_e32 v1, v68", False),       # the compiler's own reader: covered
           ("s_endpgm", False),
           ("v_max3_f32 v236, v68, v69, v70", True),
           ("s_endpgm", False)]
    hits = exposed_readers(ins, {".LBB0_1": 4}, lambda t: "v_mfma" in t, MFMA_8_PASS_WAIT_STATES)
    assert [h[0] for h in hits] == [1]
    sg = [("v_readfirstlane_b32 s7, v3", False), ("s_add_i32 s8, s8, 1", False), ("s_mov_b32 m0, s7", True),
          ("s_nop 0", True), ("global_load_lds_dwordx4 v[2:3], off", True)]
    assert [h[0] for h in hand_written_sgpr_readers_behind_valu(sg, 5)] == [1]
    assert hand_written_sgpr_readers_behind_valu([sg[0]] + [("s_nop 4", False)] + sg[1:], 5) == []
    padded = ins[:4] + [("s_nop 7", False), ("s_nop 3", False)] + ins[4:]
    assert exposed_readers(padded, {".LBB0_1": 4}, lambda t: "v_mfma" in t, MFMA_8_PASS_WAIT_STATES) == []


@pytest.mark.parametrize("source", ["score_mfma.hip", "patch_attn.hip"])
def test_no_hand_written_valu_reads_an_unfinished_result(source):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not present")
    n_mfma_kernels = 0
    for name, ins, labels in _kernels(_isa(source)):
        if not any("v_mfma" in t for t, _ in ins):
            continue
        n_mfma_kernels += 1
        after_mfma = exposed_readers(ins, labels, lambda t: "v_mfma" in t, MFMA_8_PASS_WAIT_STATES)
        assert not after_mfma, (name, after_mfma[:3])
        after_trans = exposed_readers(ins, labels, lambda t: t.startswith(("v_exp_f32", "v_log_f32", "v_rcp_f32")),
                                      TRANS_WAIT_STATES)
        assert not after_trans, (name, after_trans[:3])
        sgpr = hand_written_sgpr_readers_behind_valu(ins, 5)
        assert not sgpr, (name, sgpr[:3])
    assert n_mfma_kernels >= 3
