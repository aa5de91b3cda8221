#!/usr/bin/env python3
"""Eviction-step throughput on one MI355X.

One step = one pass of the whole hot path (score -> top-M -> in-place compaction,
one epicache_evict_step_overlapped call: the step with the selection and compaction
of one part of the batch on a second stream beside the scoring of the next, where the library
finds that worthwhile, else the plain epicache_evict_step) over one batch of
synthetic input: all L layers x
E episodes of a workload folded into the batch axis.  The default workload is the
largest one, "stress": 32 layers x 16 episodes = 512 caches of 8 KV heads,
M = 16384 cached + 8192 block rows per head, 256 patch queries per query head,
bf16 (48 GiB of K and V).  Inputs are resident in HBM before the clock starts.
Compaction is destructive, so every timed step starts from a pristine copy of
K and V: for the small workloads each step has its own freshly generated set and
the K steps run back to back inside one bracket; for workloads whose sets do not
fit that way, one working set is restored from a master copy before each step,
outside the timed interval, and each step is bracketed on its own.

Prints ONE JSON line: whole-job tokens/s (token = one context position of one
episode in one layer), per-stage times measured with HIP events on the launch
stream, the roofline of the dominant stage, the same figures for the other four
workloads (`configs`), and the CPU oracle timed on a bounded sample of the same
workload.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_FP32_VALU_TFLOPS = 157.3    # MI355X fp32 vector (the fp32 workload runs plain FMAs)
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
# What the chip sustains, chip-wide, for v_mfma_f32_32x32x16_bf16 with Eq. 1's softmax arithmetic (two multiply-add /
# exp2 / add triples) behind each, all operands in registers: profiles/microbench_mfma_softmax_ceiling.txt
SUSTAINED_MFMA_SOFTMAX_TFLOPS = 1417.0
DISTINCT_SETS_BUDGET = 100e9     # bytes of K+V that may be spent on one set per step


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="stress")
    ap.add_argument("--reduce", default="sum", choices=["sum", "max"])
    ap.add_argument("--stage-reps", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--no-other-configs", action="store_true", help="skip the `configs` block")
    ap.add_argument("--no-extras", action="store_true", help="skip the entry points outside the timed step")
    return ap.parse_args()


def cpu_baseline(w, reduce, budget_s):
    """The oracle as it stands, on the host cores, head by head on the first layer(s) of the same workload."""
    from oracle import epicache_oracle as orc
    from paper_2509_17396_amd import synth
    blas_threads = None
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        pass
    heads, spent, layer = 0, 0.0, 0
    one = w.scaled(E=1)   # one episode's cache per generated layer keeps the host-side generation short
    while spent < budget_s:
        q, k, v = synth.make_layer(one, layer=layer % w.L, step=layer // w.L)
        for b in range(one.E):
            for h in range(w.Hkv):
                qq = synth.to_f64_numpy(q[b:b + 1, h * w.G:(h + 1) * w.G])
                kk = synth.to_f64_numpy(k[b:b + 1, h:h + 1])
                kb, vb = synth.raw_bits_numpy(k[b:b + 1, h:h + 1]), synth.raw_bits_numpy(v[b:b + 1, h:h + 1])
                t0 = time.perf_counter()
                orc.evict_step(qq, kk, None, w.N, w.M, reduce, k_bits=kb, v_bits=vb)
                spent += time.perf_counter() - t0
                heads += 1
                if spent >= budget_s:
                    break
            if spent >= budget_s:
                break
        layer += 1
    tokens = heads * w.N / w.Hkv   # a token is one context position over all Hkv heads of a cache
    return {"value": tokens / spent, "unit": "tokens/s", "cores": int(os.cpu_count() or 1),
            "blas_threads": blas_threads, "kind": "oracle",
            "sample": f"{heads} (episode, KV head) pairs of the same workload (one episode per layer), one after another "
                      f"(a full step has {w.L * w.E * w.Hkv}), each scored, selected and compacted by the "
                      f"numpy float64 oracle; {spent:.1f} s; the matrix product inside uses the BLAS threads, "
                      f"the rest of the oracle one core"}


def profiled_traffic(workload, key):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if there is one.
    Returns (bytes or None, source description or None)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        data = open(path, "rb").read()
    except OSError:
        return None, None
    for line in data.decode().splitlines():
        parts = line.split()
        if len(parts) == 3 and parts[0] == "traffic_bytes" and parts[1] == key:
            return float(parts[2]), f"profiles/hbm_traffic_{workload}.txt sha256:{hashlib.sha256(data).hexdigest()[:12]}"
    return None, None


def events(n, k):
    import torch
    return [[torch.cuda.Event(enable_timing=True) for _ in range(k)] for _ in range(n)]


def mean_ms(ev, i):
    return sum(e[i].elapsed_time(e[i + 1]) for e in ev) / len(ev)


def measure(w, reduce_name, steps, warmup, stage_reps, extras, aux):
    """One workload, all layers folded into one launch.  Returns the figures of the timed step and its stages."""
    import torch
    from paper_2509_17396_amd import binding as ep
    from paper_2509_17396_amd import synth

    dev = "cuda"
    reduce = ep.REDUCE_SUM if reduce_name == "sum" else ep.REDUCE_MAX
    layers = list(range(w.L))
    nb, nbh = w.L * w.E, w.L * w.E * w.Hkv
    elem = 4 if w.dtype == "f32" else 2
    bytes_per_set = 2 * nbh * w.N * w.d * elem
    n_sets = steps + warmup
    distinct = n_sets * bytes_per_set <= DISTINCT_SETS_BUDGET
    tokens_per_step = nb * w.N

    # ---- inputs, resident in HBM before anything is timed
    if distinct:
        sets = [synth.make_folded(w, layers, step=s, device=dev) for s in range(n_sets)]
        q0, k0, v0 = sets[0]
    else:
        q0, kmaster, vmaster = synth.make_folded(w, layers, step=0, device=dev)
        k0, v0 = torch.empty_like(kmaster), torch.empty_like(vmaster)
    prm = ep.make_params(q0, k0, n_cached=w.M, n_block=w.B, budget=w.M, reduce=reduce)
    ws = ep.alloc_workspace(prm)
    # The timed step is epicache_evict_step_overlapped with the library's own choice of chunks: scoring of chunk
    # c + 1 on the launch stream beside the selection and compaction of chunk c on a second stream (one chunk, i.e.
    # the plain epicache_evict_step, where that does not pay).
    ws_bytes, n_chunks = ep.epicache_overlapped_workspace_size(prm, 0)
    ws_step = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def step(q, k, v):
        ep.epicache_evict_step_overlapped(prm, q, k, v, ws_step, aux, 0)

    torch.cuda.synchronize()

    # ---- whole-step timing: W warm-up steps, then exactly K timed steps
    if distinct:
        for s in range(warmup):
            step(*sets[s])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(warmup, n_sets):
            step(*sets[s])
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        timing = "K steps back to back in one bracket, each on its own input set"
        kfresh, vfresh = synth.make_folded(w, layers, step=0, device=dev)[1:]
        del sets[1:]
    else:
        elapsed = 0.0
        for s in range(n_sets):
            k0.copy_(kmaster), v0.copy_(vmaster)     # restore, outside the timed interval
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            step(q0, k0, v0)
            torch.cuda.synchronize()
            if s >= warmup:
                elapsed += time.perf_counter() - t0
        timing = "each step bracketed on its own; K and V restored from a master copy between steps, untimed"
        kfresh, vfresh = kmaster, vmaster
    ms_per_step = elapsed / steps * 1e3

    # ---- the same step with the stages one after the other on one stream (epicache_evict_step)
    kp, vp = k0, v0
    ev = events(stage_reps + 1, 2)
    for e in ev:
        kp.copy_(kfresh), vp.copy_(vfresh)
        e[0].record()
        ep.epicache_evict_step(prm, q0, kp, vp, ws)
        e[1].record()
    torch.cuda.synchronize()
    t_step_serial = mean_ms(ev[1:], 0) * 1e-3

    # ---- per-stage timing with HIP events on the launch stream (whole batch per launch, the launch configuration
    # of epicache_evict_step, which enqueues exactly these three calls; the overlapped step launches the same
    # kernels once per chunk)
    scores = torch.empty(nb, w.Hkv, w.N, dtype=torch.float32, device=dev)
    keep = torch.empty(nb, w.Hkv, w.M, dtype=torch.int32, device=dev)
    ev = events(stage_reps + 1, 4)
    for e in ev:
        kp.copy_(kfresh), vp.copy_(vfresh)
        e[0].record()
        ep.epicache_score(prm, q0, kp, scores, ws)
        e[1].record()
        ep.epicache_topk(prm, scores, keep)
        e[2].record()
        ep.epicache_compact(prm, keep, kp, vp)
        e[3].record()
    torch.cuda.synchronize()
    t_score, t_topk, t_compact = (mean_ms(ev[1:], i) * 1e-3 for i in range(3))

    # ---- the other reduction over the scoring rows (Eq. 1 takes the maximum; the headline is quoted on the
    # column sum): same data flow, timed beside it
    other = ep.REDUCE_MAX if reduce == ep.REDUCE_SUM else ep.REDUCE_SUM
    prm_other = ep.make_params(q0, k0, n_cached=w.M, n_block=w.B, budget=w.M, reduce=other)
    ev = events(stage_reps + 1, 3)
    for e in ev:
        kp.copy_(kfresh), vp.copy_(vfresh)
        e[0].record()
        ep.epicache_score(prm_other, q0, kp, scores, ws)
        e[1].record()
        ep.epicache_evict_step(prm_other, q0, kp, vp, ws)
        e[2].record()
    torch.cuda.synchronize()
    t_score_other, t_step_other = (mean_ms(ev[1:], i) * 1e-3 for i in range(2))
    ev = events(stage_reps + 1, 2)
    for e in ev:
        kp.copy_(kfresh), vp.copy_(vfresh)
        e[0].record()
        ep.epicache_evict_step_overlapped(prm_other, q0, kp, vp, ws_step, aux, 0)
        e[1].record()
    torch.cuda.synchronize()
    t_step_other_overlapped = mean_ms(ev[1:], 0) * 1e-3

    # ---- the step for callers whose prefill attention kernel already returned the patch rows' normalisers
    # (here they come, untimed, from epicache_patch_attention): one pass over K, then the same selection and compaction
    attn_out = torch.empty_like(q0)
    lse = torch.empty(nb, w.Hq, w.p, dtype=torch.float32, device=dev)
    ep.epicache_patch_attention(prm, q0, kfresh, vfresh, attn_out, lse)
    del attn_out
    ev = events(stage_reps + 1, 3)
    for e in ev:
        kp.copy_(kfresh), vp.copy_(vfresh)
        e[0].record()
        ep.epicache_score_lse(prm, q0, kp, lse, scores, ws)
        e[1].record()
        ep.epicache_evict_step_lse(prm, q0, kp, vp, lse, ws)
        e[2].record()
    torch.cuda.synchronize()
    t_score_lse, t_step_lse = (mean_ms(ev[1:], i) * 1e-3 for i in range(2))
    # ... and the same step over chunks on two streams (epicache_evict_step_overlapped with row_lse_opt)
    lse_bytes, lse_chunks = ep.epicache_overlapped_workspace_size(prm, 0, with_row_lse=True)
    ws_lse = torch.empty(max(lse_bytes, 256), dtype=torch.uint8, device=dev)
    ev = events(stage_reps + 1, 2)
    for e in ev:
        kp.copy_(kfresh), vp.copy_(vfresh)
        e[0].record()
        ep.epicache_evict_step_overlapped(prm, q0, kp, vp, ws_lse, aux, 0, row_lse=lse)
        e[1].record()
    torch.cuda.synchronize()
    t_step_lse_overlapped = mean_ms(ev[1:], 0) * 1e-3
    del ws_lse

    bf16 = w.dtype == "bf16"
    flops_score = 2.0 * w.R * w.N * w.d * nbh                        # one Q.K^T (algorithmic)
    peak_score = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_FP32_VALU_TFLOPS
    bytes_score = nbh * (w.N * w.d * elem + w.R * w.d * elem + 4.0 * w.N)   # K once + Q + scores
    bytes_topk = nbh * (4.0 * w.N + 4.0 * w.M)
    bytes_compact = nbh * (4.0 * w.M * w.d * elem + 4.0 * w.M)      # read+write of kept K and V rows + indices
    res = {
        "workload": f"{w.name}: L={w.L} layers x E={w.E} episodes folded into one launch, "
                    f"Hq/Hkv={w.Hq}/{w.Hkv}, d={w.d}, {w.dtype}, M={w.M}, block={w.B}, patch={w.p}, reduce={reduce_name}",
        "tokens_per_step": tokens_per_step, "ms_per_step": ms_per_step, "tokens_per_s": tokens_per_step / (elapsed / steps),
        "timing": timing, "bytes_per_input_set": bytes_per_set,
        "step_entry_point": f"epicache_evict_step_overlapped, {n_chunks} chunk(s)" +
                            (": the plain step" if n_chunks == 1 else
                             ", selection and compaction of a chunk on a second stream beside the scoring of the next"),
        "serial_step_ms": t_step_serial * 1e3,
        "score_ms": t_score * 1e3, "topk_ms": t_topk * 1e3, "compact_ms": t_compact * 1e3,
        "score_tflops_algorithmic": flops_score / t_score / 1e12,
        "score_frac_peak_algorithmic": flops_score / t_score / 1e12 / peak_score,
        "score_frac_peak_executed": 2 * flops_score / t_score / 1e12 / peak_score,
        "score_peak_tflops": peak_score, "score_peak_kind": "bf16 MFMA" if bf16 else "fp32 vector ALU",
        "compact_gbs": bytes_compact / t_compact / 1e9,
        "compact_frac_hbm_peak": bytes_compact / t_compact / 1e9 / PEAK_HBM_GBS,
        "select_plus_compact_ms": (t_topk + t_compact) * 1e3,
        "select_plus_compact_frac_hbm_peak": (bytes_topk + bytes_compact) / (t_topk + t_compact) / 1e9 / PEAK_HBM_GBS,
        "normalisers_supplied": {"score_ms": t_score_lse * 1e3, "evict_step_ms": t_step_lse * 1e3,
                                 "evict_step_overlapped_ms": t_step_lse_overlapped * 1e3,
                                 "overlapped_chunks": lse_chunks,
                                 "tokens_per_s": tokens_per_step / min(t_step_lse, t_step_lse_overlapped),
                                 "score_frac_peak_algorithmic": flops_score / t_score_lse / 1e12 / peak_score,
                                 "note": "epicache_evict_step_lse, and epicache_evict_step_overlapped with row_lse_opt: the "
                                         "patch rows' log-sum-exp supplied by the caller (its own attention pass returns them), "
                                         "scoring is one pass over K; not the timed step"},
        "other_reduce": {"reduce": "max" if other == ep.REDUCE_MAX else "sum", "score_ms": t_score_other * 1e3,
                         "evict_step_ms": t_step_other * 1e3, "evict_step_overlapped_ms": t_step_other_overlapped * 1e3,
                         "tokens_per_s": tokens_per_step / min(t_step_other, t_step_other_overlapped)},
        "_bytes": {"score": bytes_score, "topk": bytes_topk, "compact": bytes_compact, "flops_score": flops_score},
    }
    if not extras:
        return res

    stages = {}
    # ---- the patch's own attention output and normalisers (context keys only here: the bench tensors
    # have no spare rows for the patch's keys), the pass that makes the single-pass scoring possible
    attn_out = torch.empty_like(q0)
    ev = events(stage_reps + 1, 2)
    for e in ev:
        e[0].record()
        ep.epicache_patch_attention(prm, q0, kfresh, vfresh, attn_out, lse)
        e[1].record()
    torch.cuda.synchronize()
    t_attn = mean_ms(ev[1:], 0) * 1e-3
    stages["patch_attention"] = {
        "ms": t_attn * 1e3, "tflops": 2 * flops_score / t_attn / 1e12,
        "frac_mfma_peak": 2 * flops_score / t_attn / 1e12 / PEAK_BF16_MFMA_TFLOPS,
        "note": "epicache_patch_attention (Q.K^T and P.V, K and V read once); its normalisers feed "
                "normalisers_supplied; not part of the timed step"}

    # ---- the step with the patch's forward pass folded in (attention output, then scoring on its
    # normalisers, selection, compaction) in one call
    ev = events(stage_reps + 1, 2)
    for e in ev:
        kp.copy_(kfresh), vp.copy_(vfresh)
        e[0].record()
        ep.epicache_evict_step_attn(prm, q0, kp, vp, attn_out, ws)
        e[1].record()
    torch.cuda.synchronize()
    stages["evict_step_attn"] = {
        "ms": mean_ms(ev[1:], 0),
        "note": "epicache_evict_step_attn: patch_attention + single-pass scoring + topk + compact in one call; "
                "not part of the timed step"}
    del attn_out

    # ---- the ragged entry point on the same inputs (every head holds N rows before the step):
    # lengths and budgets are read from device memory; pooled = head-wise non-uniform retention
    n_ctx = torch.full((nb, w.Hkv), w.N, dtype=torch.int32, device=dev)
    budgets = torch.full((nb,), w.M, dtype=torch.int32, device=dev)
    n_kept = torch.empty((nb, w.Hkv), dtype=torch.int32, device=dev)
    t_ragged = {}
    for tag, select in (("per_head", ep.SELECT_PER_HEAD), ("pooled", ep.SELECT_POOLED)):
        wsr = ep.alloc_ragged_workspace(prm, select)
        ev = events(stage_reps + 1, 2)
        for e in ev:
            kp.copy_(kfresh), vp.copy_(vfresh)
            e[0].record()
            ep.epicache_evict_step_ragged(prm, select, q0, kp, vp, n_ctx, budgets, n_kept, wsr)
            e[1].record()
        torch.cuda.synchronize()
        t_ragged[tag] = mean_ms(ev[1:], 0)
        del wsr
        # the same over chunks on two streams
        rbytes, _, rchunks = ep.epicache_ragged_overlapped_workspace_size(prm, select, 0)
        wsr = torch.empty(max(rbytes, 256), dtype=torch.uint8, device=dev)
        ev = events(stage_reps + 1, 2)
        for e in ev:
            kp.copy_(kfresh), vp.copy_(vfresh)
            e[0].record()
            ep.epicache_evict_step_ragged_overlapped(prm, select, q0, kp, vp, n_ctx, budgets, n_kept, wsr, aux, 0)
            e[1].record()
        torch.cuda.synchronize()
        t_ragged[tag + "_overlapped"] = mean_ms(ev[1:], 0)
        del wsr
    stages["evict_step_ragged"] = {
        "ms_per_head": t_ragged["per_head"], "ms_pooled": t_ragged["pooled"],
        "overlapped_ms_per_head": t_ragged["per_head_overlapped"], "overlapped_ms_pooled": t_ragged["pooled_overlapped"],
        "overlapped_chunks": rchunks,
        "note": "epicache_evict_step_ragged / epicache_evict_step_ragged_overlapped on the same inputs, lengths and "
                "budgets read from device memory; not part of the timed step"}

    # ---- the attention-free KeyDiff scorer on the same K (second workload of the same back end)
    ev = events(stage_reps + 1, 2)
    for e in ev:
        e[0].record()
        ep.epicache_score_keydiff(prm, kfresh, scores, ws)
        e[1].record()
    torch.cuda.synchronize()
    t_keydiff = mean_ms(ev[1:], 0) * 1e-3
    bytes_keydiff = nbh * w.N * (w.d * elem + 4.0)
    stages["score_keydiff"] = {
        "ms": t_keydiff * 1e3, "gbs": bytes_keydiff / t_keydiff / 1e9,
        "frac_hbm_peak": bytes_keydiff / t_keydiff / 1e9 / PEAK_HBM_GBS,
        "note": "epicache_score_keydiff: K read once + scores written as algorithmic bytes; not part of the timed step"}

    # ---- Stage-3a matching (Sec. 3.1) at the scale of one long conversation: 256 queries against E centroids
    gen = torch.Generator(device=dev).manual_seed(7)
    cents = torch.randn(w.E, 1024, device=dev, generator=gen)
    qs = torch.randn(256, 1024, device=dev, generator=gen)
    matched = torch.empty(256, dtype=torch.int32, device=dev)
    ev = events(stage_reps + 1, 2)
    for e in ev:
        e[0].record()
        ep.epicache_match_queries(qs, cents, 0.0, matched)
        e[1].record()
    torch.cuda.synchronize()
    stages["match_queries"] = {"ms": mean_ms(ev[1:], 0),
                               "note": "256 queries x 1024 dims against E centroids; latency-bound, not part of the timed step"}
    res["extras"] = stages
    return res


def free_gpu():
    import gc
    import torch
    gc.collect()
    torch.cuda.empty_cache()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the eviction step shards by episode / "
              "KV head / layer with no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_17396_amd import binding as ep
    from paper_2509_17396_amd import synth

    ep.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    w = synth.WORKLOADS[args.workload]

    # The second stream of the overlapped step, one for the whole run: HIP multiplexes streams onto a few hardware
    # queues, and a stream that lands on the launch stream's queue would serialise the two.
    aux = torch.cuda.Stream()
    m = measure(w, args.reduce, args.steps, args.warmup, args.stage_reps, extras=not args.no_extras, aux=aux)
    free_gpu()
    by = m.pop("_bytes")
    t_score, t_topk, t_compact = m["score_ms"] * 1e-3, m["topk_ms"] * 1e-3, m["compact_ms"] * 1e-3

    stages = {
        "score": {"ms": m["score_ms"], "tflops_algorithmic": m["score_tflops_algorithmic"],
                  "tflops_executed": 2 * m["score_tflops_algorithmic"],
                  "frac_mfma_peak_algorithmic": m["score_frac_peak_algorithmic"],
                  "frac_mfma_peak_executed": m["score_frac_peak_executed"],
                  "algorithmic_gbs": by["score"] / t_score / 1e9},
        "topk": {"ms": m["topk_ms"], "gbs": by["topk"] / t_topk / 1e9},
        "compact": {"ms": m["compact_ms"], "gbs": m["compact_gbs"], "frac_hbm_peak": m["compact_frac_hbm_peak"]},
        "select_plus_compact": {"ms": m["select_plus_compact_ms"], "frac_hbm_peak": m["select_plus_compact_frac_hbm_peak"]},
        "other_reduce": m["other_reduce"],
        "normalisers_supplied": m["normalisers_supplied"],
    }
    stages.update(m.pop("extras", {}))
    score_traffic, score_src = profiled_traffic(w.name, "score")
    if score_traffic:   # HBM bytes the two passes moved per launch when the committed profile was taken, over the live time
        stages["score"]["hbm_gbs_profiled_traffic"] = score_traffic / t_score / 1e9
        stages["score"]["frac_hbm_peak_profiled_traffic"] = score_traffic / t_score / 1e9 / PEAK_HBM_GBS
    if t_score >= t_compact + t_topk:
        a = m["score_tflops_algorithmic"]
        roofline = {"kernel": "score (score_stats + score_reduce)", "bound": "mfma", "achieved": a,
                    "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": a / PEAK_BF16_MFMA_TFLOPS,
                    "traffic": score_traffic, "traffic_source": score_src,
                    "launch": "whole batch per launch, timed with HIP events on the launch stream; the overlapped step "
                              "launches the same kernels once per chunk beside the previous chunk's selection and "
                              "compaction (per-chunk durations: profiles/kernels_<workload>_folded.txt, '@grid' rows)",
                    "executed": {"tflops": 2 * a, "frac_of_peak": 2 * a / PEAK_BF16_MFMA_TFLOPS,
                                 "sustained_tflops_for_this_instruction_mix": SUSTAINED_MFMA_SOFTMAX_TFLOPS,
                                 "frac_of_sustained": 2 * a / SUSTAINED_MFMA_SOFTMAX_TFLOPS,
                                 "note": "the step evaluates Q.K^T twice (row normalisers, then column reduction); "
                                         "the sustained figure is a microbenchmark of the same MFMA + softmax "
                                         "instruction mix with nothing else going on"}}
    else:
        traffic, src = profiled_traffic(w.name, "compact")
        roofline = {"kernel": "compact_rows", "bound": "hbm", "achieved": m["compact_gbs"], "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": m["compact_frac_hbm_peak"], "traffic": traffic, "traffic_source": src}

    out = {
        "metric": "evict-step tokens scored+compacted/sec",
        "value": m["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": m["workload"], "tokens_per_step": m["tokens_per_step"], "timing": m["timing"],
                   "step_entry_point": m["step_entry_point"]},
        "serial_step_ms": m["serial_step_ms"],
        "roofline": roofline,
        "stages": stages,
    }

    if not args.no_other_configs:
        # the same figures for the other workloads, each with all its layers folded into one launch
        configs = {w.name: {k: m[k] for k in ("ms_per_step", "serial_step_ms", "step_entry_point", "tokens_per_s", "score_ms",
                                              "score_frac_peak_algorithmic",
                                              "score_frac_peak_executed", "score_peak_kind", "compact_ms",
                                              "select_plus_compact_frac_hbm_peak")}}
        for name, ow in synth.WORKLOADS.items():
            if name == w.name:
                continue
            steps = 20 if ow.L * ow.E * ow.Hkv * ow.N * ow.d < 6e9 else 10
            om = measure(ow, args.reduce, steps, 2, args.stage_reps, extras=False, aux=aux)
            free_gpu()
            configs[name] = {k: om[k] for k in ("ms_per_step", "serial_step_ms", "step_entry_point", "tokens_per_s", "score_ms",
                                                "score_frac_peak_algorithmic",
                                                "score_frac_peak_executed", "score_peak_kind", "compact_ms",
                                                "select_plus_compact_frac_hbm_peak")}
            configs[name]["workload"] = om["workload"]
            configs[name]["other_reduce_evict_step_ms"] = om["other_reduce"]["evict_step_ms"]
            configs[name]["other_reduce_evict_step_overlapped_ms"] = om["other_reduce"]["evict_step_overlapped_ms"]
            configs[name]["normalisers_supplied"] = {k: om["normalisers_supplied"][k] for k in
                                                     ("score_ms", "evict_step_ms", "evict_step_overlapped_ms",
                                                      "score_frac_peak_algorithmic")}
        out["configs"] = configs

    if not args.no_cpu_baseline:
        reduce = ep.REDUCE_SUM if args.reduce == "sum" else ep.REDUCE_MAX
        out["cpu_baseline"] = cpu_baseline(w, reduce, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
