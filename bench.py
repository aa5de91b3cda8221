#!/usr/bin/env python3
"""Eviction-step throughput on one MI355X.

One step = one pass of the whole hot path (score -> top-M -> in-place compaction,
one epicache_evict_step call) over one batch of synthetic input: all L layers x
E episodes of the LLaMA-3.2-3B-shaped workload folded into the batch axis
(28 x 4 caches of 8 KV heads, M = 2048 cached + 2048 block rows, 64 patch
queries per query head, bf16).  Every step runs on its own freshly generated
Q/K/V, resident in HBM before the clock starts.

Prints ONE JSON line: whole-job tokens/s (token = one context position of one
episode in one layer), per-stage times measured with HIP events on the launch
stream, the roofline of the dominant stage, and the CPU oracle timed on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama32_3b")
    ap.add_argument("--reduce", default="sum", choices=["sum", "max"])
    ap.add_argument("--stage-reps", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    return ap.parse_args()


def cpu_baseline(w, reduce, budget_s):
    """The oracle as it stands, on the host cores, on whole layers of the same workload."""
    import numpy as np
    from oracle import epicache_oracle as orc
    from paper_2509_17396_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = 1
    tokens, spent, layers = 0, 0.0, 0
    while spent < budget_s:
        q, k, v = synth.make_layer(w, layer=layers % w.L, step=layers // w.L)
        qq, kk = synth.to_f64_numpy(q), synth.to_f64_numpy(k)
        kb, vb = synth.raw_bits_numpy(k), synth.raw_bits_numpy(v)
        t0 = time.perf_counter()
        orc.evict_step(qq, kk, None, w.N, w.M, reduce, k_bits=kb, v_bits=vb)
        spent += time.perf_counter() - t0
        tokens += w.E * w.N
        layers += 1
    return {"value": tokens / spent, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{layers} whole layers of the same workload (each all {w.E} episodes x "
                      f"{w.Hkv} KV heads; a full step has {w.L}), numpy float64, {spent:.1f} s"}


def measured_traffic(workload, key):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic_bytes" and parts[1] == key:
                return float(parts[2])
    except OSError:
        pass
    return None


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
    dev = "cuda"
    w = synth.WORKLOADS[args.workload]
    reduce = ep.REDUCE_SUM if args.reduce == "sum" else ep.REDUCE_MAX
    layers = list(range(w.L))
    nb = w.L * w.E
    n_sets = args.steps + args.warmup
    bytes_per_set = 2 * nb * w.Hkv * w.N * w.d * 2
    if n_sets * bytes_per_set > 200e9:
        print(f"bench.py: {n_sets} input sets of {bytes_per_set / 2**30:.2f} GiB do not fit; lower --steps",
              file=sys.stderr)
        sys.exit(2)

    # ---- inputs, resident in HBM before anything is timed
    sets = [synth.make_folded(w, layers, step=s, device=dev) for s in range(n_sets)]
    q0, k0, v0 = sets[0]
    prm = ep.make_params(q0, k0, n_cached=w.M, n_block=w.B, budget=w.M, reduce=reduce)
    ws = ep.alloc_workspace(prm)
    torch.cuda.synchronize()

    # ---- whole-step timing: W warm-up steps, then exactly K timed steps
    for s in range(args.warmup):
        q, k, v = sets[s]
        ep.epicache_evict_step(prm, q, k, v, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.warmup, n_sets):
        q, k, v = sets[s]
        ep.epicache_evict_step(prm, q, k, v, ws)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_step = nb * w.N
    value = tokens_per_step / (elapsed / args.steps)

    # ---- per-stage timing with HIP events on the launch stream (same launch configuration:
    # epicache_evict_step enqueues exactly these three calls)
    del sets[1:]
    kp, vp = k0.clone(), v0.clone()   # set 0 was compacted by the warm-up; rebuild it
    q0, kfresh, vfresh = synth.make_folded(w, layers, step=0, device=dev)
    scores = torch.empty(nb, w.Hkv, w.N, dtype=torch.float32, device=dev)
    keep = torch.empty(nb, w.Hkv, w.M, dtype=torch.int32, device=dev)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.stage_reps)]
    for rep in range(args.stage_reps + 1):
        kp.copy_(kfresh), vp.copy_(vfresh)
        e = ev[rep - 1] if rep > 0 else [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        e[0].record()
        ep.epicache_score(prm, q0, kp, scores, ws)
        e[1].record()
        ep.epicache_topk(prm, scores, keep)
        e[2].record()
        ep.epicache_compact(prm, keep, kp, vp)
        e[3].record()
    torch.cuda.synchronize()
    t_score, t_topk, t_compact = (
        sum(e[i].elapsed_time(e[i + 1]) for e in ev) / len(ev) * 1e-3 for i in range(3))

    # ---- the single-pass variant for callers that already hold the row normalisers (their prefill
    # attention kernel returns them): same scores, K read once.  Normalisers come from torch here.
    G = w.Hq // w.Hkv
    lse = torch.empty(nb, w.Hq, w.p, dtype=torch.float32, device=dev)
    for b0 in range(0, nb, 8):
        kk = kfresh[b0:b0 + 8].float().repeat_interleave(G, dim=1)          # [8, Hq, N, d]
        z = torch.matmul(q0[b0:b0 + 8].float(), kk.transpose(2, 3)) / w.d ** 0.5
        lse[b0:b0 + 8] = torch.logsumexp(z, dim=3)
        del kk, z
    ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.stage_reps)]
    for rep in range(args.stage_reps + 1):
        e = ev2[rep - 1] if rep > 0 else [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record()
        ep.epicache_score_lse(prm, q0, kfresh, lse, scores, ws)
        e[1].record()
    torch.cuda.synchronize()
    t_score_lse = sum(e[0].elapsed_time(e[1]) for e in ev2) / len(ev2) * 1e-3

    # ---- the ragged entry point on the same inputs (every head holds N rows before the step):
    # lengths and budgets are read from device memory; pooled = head-wise non-uniform retention
    n_ctx = torch.full((nb, w.Hkv), w.N, dtype=torch.int32, device=dev)
    budgets = torch.full((nb,), w.M, dtype=torch.int32, device=dev)
    n_kept = torch.empty((nb, w.Hkv), dtype=torch.int32, device=dev)
    t_ragged = {}
    for tag, select in (("per_head", ep.SELECT_PER_HEAD), ("pooled", ep.SELECT_POOLED)):
        wsr = ep.alloc_ragged_workspace(prm, select)
        ev3 = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.stage_reps)]
        for rep in range(args.stage_reps + 1):
            kp.copy_(kfresh), vp.copy_(vfresh)
            e = ev3[rep - 1] if rep > 0 else [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            e[0].record()
            ep.epicache_evict_step_ragged(prm, select, q0, kp, vp, n_ctx, budgets, n_kept, wsr)
            e[1].record()
        torch.cuda.synchronize()
        t_ragged[tag] = sum(e[0].elapsed_time(e[1]) for e in ev3) / len(ev3) * 1e-3
        del wsr

    # ---- the patch's own attention output and normalisers (context keys only here: the bench tensors
    # have no spare rows for the patch's keys), the pass that makes the single-pass scoring possible
    attn_out = torch.empty_like(q0)
    attn_lse = torch.empty(nb, w.Hq, w.p, dtype=torch.float32, device=dev)
    ev6 = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.stage_reps)]
    for rep in range(args.stage_reps + 1):
        e = ev6[rep - 1] if rep > 0 else [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record()
        ep.epicache_patch_attention(prm, q0, kfresh, vfresh, attn_out, attn_lse)
        e[1].record()
    torch.cuda.synchronize()
    t_attn = sum(e[0].elapsed_time(e[1]) for e in ev6) / len(ev6) * 1e-3

    # ---- the step with the patch's forward pass folded in (attention output, then scoring on its
    # normalisers, selection, compaction) in one call
    ev7 = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.stage_reps)]
    for rep in range(args.stage_reps + 1):
        kp.copy_(kfresh), vp.copy_(vfresh)
        e = ev7[rep - 1] if rep > 0 else [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record()
        ep.epicache_evict_step_attn(prm, q0, kp, vp, attn_out, ws)
        e[1].record()
    torch.cuda.synchronize()
    t_step_attn = sum(e[0].elapsed_time(e[1]) for e in ev7) / len(ev7) * 1e-3

    # ---- the other reduction over the scoring rows (Eq. 1 takes the maximum; the headline line is quoted on
    # the column sum): same data flow, timed beside it
    other = ep.REDUCE_MAX if reduce == ep.REDUCE_SUM else ep.REDUCE_SUM
    prm_other = ep.make_params(q0, k0, n_cached=w.M, n_block=w.B, budget=w.M, reduce=other)
    ev8 = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.stage_reps)]
    for rep in range(args.stage_reps + 1):
        kp.copy_(kfresh), vp.copy_(vfresh)
        e = ev8[rep - 1] if rep > 0 else [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record()
        ep.epicache_score(prm_other, q0, kp, scores, ws)
        e[1].record()
        ep.epicache_evict_step(prm_other, q0, kp, vp, ws)
        e[2].record()
    torch.cuda.synchronize()
    t_score_other, t_step_other = (sum(e[i].elapsed_time(e[i + 1]) for e in ev8) / len(ev8) * 1e-3 for i in range(2))

    # ---- the attention-free KeyDiff scorer on the same K (second workload of the same back end)
    ev4 = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.stage_reps)]
    for rep in range(args.stage_reps + 1):
        e = ev4[rep - 1] if rep > 0 else [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record()
        ep.epicache_score_keydiff(prm, kfresh, scores, ws)
        e[1].record()
    torch.cuda.synchronize()
    t_keydiff = sum(e[0].elapsed_time(e[1]) for e in ev4) / len(ev4) * 1e-3

    # ---- episode geometry (Sec. 3.1 Eq. 3 and Stage 3a) at the scale of one long conversation:
    # 2048 segment embeddings of dimension 1024 in E clusters, 256 queries to match
    gen = torch.Generator(device=dev).manual_seed(7)
    emb = torch.randn(2048, 1024, device=dev, generator=gen)
    assign = torch.randint(0, w.E, (2048,), device=dev, generator=gen, dtype=torch.int32)
    cents = torch.empty(w.E, 1024, device=dev)
    med = torch.empty(w.E, dtype=torch.int32, device=dev)
    qs = torch.randn(256, 1024, device=dev, generator=gen)
    matched = torch.empty(256, dtype=torch.int32, device=dev)
    ev5 = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.stage_reps)]
    for rep in range(args.stage_reps + 1):
        e = ev5[rep - 1] if rep > 0 else [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record()
        ep.epicache_episode_medoids(emb, assign, w.E, cents, med)
        e[1].record()
        ep.epicache_match_queries(qs, cents, 0.0, matched)
        e[2].record()
    torch.cuda.synchronize()
    t_medoids, t_match = (sum(e[i].elapsed_time(e[i + 1]) for e in ev5) / len(ev5) * 1e-3 for i in range(2))

    nbh = nb * w.Hkv
    flops_score = 2.0 * w.R * w.N * w.d * nbh                      # one Q.K^T (algorithmic)
    bytes_topk = nbh * (4.0 * w.N + 4.0 * w.M)
    bytes_compact = nbh * (4.0 * w.M * w.d * 2 + 4.0 * w.M)        # read+write of K and V rows + indices
    stages = {
        "score": {"ms": t_score * 1e3, "tflops_algorithmic": flops_score / t_score / 1e12,
                  "tflops_executed": 2 * flops_score / t_score / 1e12,
                  "frac_mfma_peak_algorithmic": flops_score / t_score / 1e12 / PEAK_BF16_MFMA_TFLOPS},
        "score_given_lse": {"ms": t_score_lse * 1e3, "tflops_algorithmic": flops_score / t_score_lse / 1e12,
                            "frac_mfma_peak_algorithmic": flops_score / t_score_lse / 1e12 / PEAK_BF16_MFMA_TFLOPS,
                            "note": "epicache_score_lse: row normalisers supplied by the caller, not part of the timed step"},
        "topk": {"ms": t_topk * 1e3, "gbs": bytes_topk / t_topk / 1e9},
        "compact": {"ms": t_compact * 1e3, "gbs": bytes_compact / t_compact / 1e9,
                    "frac_hbm_peak": bytes_compact / t_compact / 1e9 / PEAK_HBM_GBS},
        "evict_step_ragged": {"ms_per_head": t_ragged["per_head"] * 1e3, "ms_pooled": t_ragged["pooled"] * 1e3,
                              "note": "epicache_evict_step_ragged on the same inputs, lengths and budgets read "
                                      "from device memory; not part of the timed step"},
        "patch_attention": {"ms": t_attn * 1e3, "tflops": 2 * flops_score / t_attn / 1e12,
                            "frac_mfma_peak": 2 * flops_score / t_attn / 1e12 / PEAK_BF16_MFMA_TFLOPS,
                            "note": "epicache_patch_attention (Q.K^T and P.V, K and V read once); its normalisers "
                                    "feed score_given_lse; not part of the timed step"},
        "evict_step_attn": {"ms": t_step_attn * 1e3,
                            "note": "epicache_evict_step_attn: patch_attention + score_given_lse + topk + compact in one "
                                    "call; not part of the timed step"},
        "other_reduce": {"reduce": "max" if other == ep.REDUCE_MAX else "sum", "score_ms": t_score_other * 1e3,
                         "evict_step_ms": t_step_other * 1e3,
                         "tokens_per_s": tokens_per_step / t_step_other,
                         "note": "the same step with the other reduction over the scoring rows, HIP events around one call"},
        "score_keydiff": {"ms": t_keydiff * 1e3, "gbs": (nbh * w.N * (w.d * 2.0 + 4.0)) / t_keydiff / 1e9,
                          "frac_hbm_peak": (nbh * w.N * (w.d * 2.0 + 4.0)) / t_keydiff / 1e9 / PEAK_HBM_GBS,
                          "note": "epicache_score_keydiff: K read once + scores written as algorithmic bytes "
                                  "(the kernels read K twice); not part of the timed step"},
        "episode_geometry": {"medoids_ms": t_medoids * 1e3, "match_ms": t_match * 1e3,
                             "note": "2048 segments x 1024 dims in E clusters; 256 queries; latency-bound, "
                                     "not part of the timed step"},
        "select_plus_compact": {"ms": (t_topk + t_compact) * 1e3,
                                "gbs": (bytes_topk + bytes_compact) / (t_topk + t_compact) / 1e9,
                                "frac_hbm_peak": (bytes_topk + bytes_compact) / (t_topk + t_compact) / 1e9 / PEAK_HBM_GBS},
    }
    score_traffic = measured_traffic(w.name, "score")
    if score_traffic:   # HBM bytes the two passes move per launch (rocprofv3 counters, profiles/), over the live time
        stages["score"]["hbm_gbs_measured_traffic"] = score_traffic / t_score / 1e9
        stages["score"]["frac_hbm_peak_measured_traffic"] = score_traffic / t_score / 1e9 / PEAK_HBM_GBS
    if t_score >= t_compact + t_topk:
        a = flops_score / t_score / 1e12
        roofline = {"kernel": "score (score_stats + score_reduce)", "bound": "mfma", "achieved": a,
                    "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": a / PEAK_BF16_MFMA_TFLOPS,
                    "traffic": measured_traffic(w.name, "score")}
    else:
        a = bytes_compact / t_compact / 1e9
        roofline = {"kernel": "compact_rows", "bound": "hbm", "achieved": a, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": a / PEAK_HBM_GBS, "traffic": measured_traffic(w.name, "compact")}

    out = {
        "metric": "evict-step tokens scored+compacted/sec",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: L={w.L} layers x E={w.E} episodes folded into one launch, "
                               f"Hq/Hkv={w.Hq}/{w.Hkv}, d={w.d}, M={w.M}, block={w.B}, patch={w.p}, "
                               f"reduce={args.reduce}",
                   "tokens_per_step": tokens_per_step},
        "roofline": roofline,
        "stages": stages,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, reduce, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
