#!/usr/bin/env python3
"""Benchmark of the MISA indexer hot path on one MI355X.

A step is one pass of the whole indexer (pool -> route -> score -> top-k, plus
the dense re-rank for the MISA-dagger workload) over one batch of seeded
synthetic inputs that are already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3]

The default run times the long-decode workload c3 (the HBM half of the metric:
`value`, `roofline`) and then, in the same process, the MISA-dagger prefill
workload c4 at the same L = 131072 (the matrix-core half: object `prefill`)
and the single-stage prefill chunk c2 (object `prefill_single_stage`), each
once as separate calls and once with scoring and top-k fused, and c4 once more with
fp8 queries on the fp8 matrix instruction (object `prefill_fp8_queries`).  Every number in the
line is measured by this run except where a field says otherwise.
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

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "fp8": 5000.0}   # MI355X dense matrix rates

# HBM bytes per launch of the decode score kernel, NOT measured by this run: rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE of the same launch, scaled by a plain device copy of known size
# (the summaries under profiles/ named below).
PROFILED_TRAFFIC = {"c1": (548.8e6, "profiles/score_stream_c1_hbm_traffic.md"),
                    "c3": (571.0e6, "profiles/score_stream_c3_hbm_traffic.md")}

DESCRIPTIONS = {
    "c0": "tiny decode: 1 seq x 1 query, L=4096, H=64, h=8, B=64, k=256, fp32",
    "c1": "batched decode: 64 seqs x 1 query, L=32768, H=64, h=8, B=64, k=2048, bf16 keys",
    "c2": "prefill chunk (DeepSeek-V3.2-shaped): 4096 causal queries, L=65536, H=64, h=8, B=64, k=2048, bf16 keys",
    "c3": "long decode (GLM-5-shaped): 32 seqs x 1 query, L=131072, H=32, h=8, B=128, k=2048, fp8-e4m3 keys + per-token scale",
    "c4": "MISA-dagger prefill: 2048 causal queries, L=131072, H=64, h=8, B=64, k'=8192 -> k=2048, fp8-e4m3 keys",
}


def key_bytes_per_pair(wl) -> int:
    """Algorithmic bytes the score stage must move per query-key pair in decode:
    one key row (d values at storage width) plus, for fp8, its fp32 scale."""
    return {"f32": 512, "bf16": 256, "e4m3": 132}[wl.k_dtype]


def arithmetic_dtype(wl, native_fp8: bool) -> str:
    """What the scoring path computes in (not a precision claim)."""
    if wl.k_dtype == "f32" or wl.q_dtype == "f32":
        return "f32"
    k = {"bf16": "bf16", "e4m3": "fp8-e4m3"}[wl.k_dtype]
    q = {"bf16": "bf16", "e4m3": "fp8-e4m3"}[wl.q_dtype]
    mm = "fp8 MFMA" if native_fp8 else "bf16 MFMA"
    return f"{k} keys x {q} queries, {mm}, f32 accumulate"


def cpu_baseline(wl, inp, budget_s: float = 20.0) -> dict:
    """Time the fp64 oracle as it stands on a bounded sample of the same workload."""
    import numpy as np
    from oracle import misa_oracle as O
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import oracle_view
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        blas_threads = 1
    rng = np.random.default_rng(0)
    rows = [(s, t) for s in range(wl.n_seq) for t in range(wl.n_q)]
    order = rng.permutation(len(rows))
    pairs, done, t0 = 0, 0, time.perf_counter()
    c0 = time.process_time()
    for i in order:
        s, t = rows[i]
        K, q, w, n = oracle_view(inp, s, t)
        if wl.k_cand:
            O.misa_dagger(q, w, K, wl.B, wl.h, wl.k_cand, wl.k, n)
        else:
            O.misa(q, w, K, wl.B, wl.h, wl.k, n)
        pairs += n
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    busy = (time.process_time() - c0) / dt     # average number of cores kept busy
    return {"value": pairs / dt, "unit": "pairs/s", "cores": max(1, round(busy)), "kind": "oracle",
            "cores_available": len(os.sched_getaffinity(0)), "blas_threads": blas_threads,
            "avg_busy_cores": round(busy, 2),
            "sample": f"{done} of {len(rows)} query rows of {wl.name} (whole pipeline incl. de-quantisation and "
                      f"pooling per row; a serial per-row numpy loop, threads only inside BLAS calls), {dt:.1f} s"}


def measure(args, name: str, fused: bool, main_line: bool) -> dict:
    """Runs workload `name` (steps, per-stage events, graph replays, dense comparison) and
    returns everything measured.  main_line: honour the decode-only / variant options."""
    import torch
    from dataclasses import replace
    from paper_2605_07363_amd import misa, workloads as WL
    from paper_2605_07363_amd.recall_sweep import overlap_stats

    wl = WL.WORKLOADS[name]
    override = {k: v for k, v in (("B", args.block), ("h", args.active_heads),
                                  ("q_dtype", "e4m3" if args.fp8_queries else None)) if v}
    if override:
        wl = WL.scaled(wl, **override)
    inp = WL.make_inputs(wl)
    dv = misa.to_device(inp)
    key_bytes = dv["K"].numel() * dv["K"].element_size()
    if args.paged:
        dv = misa.paginate(dv, args.paged, seed=1)
    p = dv["problem"]
    Q, W = dv["Q"], dv["W"]
    # fp8 queries: a step widens them to bf16 once; prefill workloads with fp8 keys score and re-rank
    # on the codes themselves (fp8 matrix instruction), routing uses the widened copy
    native_fp8 = bool(args.fp8_queries) and wl.k_dtype == "e4m3" and not wl.decode and misa.HAS_FP8_MFMA
    Q8, p8 = None, None
    widen = bool(args.fp8_queries)
    if widen:
        Q8, p8 = Q, (replace(p, q_dtype=misa.FP8_E4M3_MATRIX) if native_fp8 else p)
        Q = torch.empty(Q8.shape, dtype=torch.bfloat16, device="cuda")
        p = replace(p, q_dtype=misa.BF16)
    Qs = Q8 if native_fp8 else Q
    # Decode caches are far larger than the 256 MB last-level cache; rotating
    # copies keeps every step's key reads cold.  Prefill caches are small and
    # are re-read by every query tile, so one copy is the workload.
    n_rot = max(1, args.rotate) if wl.decode else 1
    Ks = [dv["K"]] + [dv["K"].clone() for _ in range(n_rot - 1)]
    scales = [dv["kscale"]] + [None if dv["kscale"] is None else dv["kscale"].clone() for _ in range(n_rot - 1)]
    ix = misa.Indexer(p, wl.k, wl.k_cand, fused=fused)
    if native_fp8:
        ix.p_score = p8
    incremental = args.incremental_pool and main_line
    newest = torch.full((wl.n_seq,), wl.L - 1, dtype=torch.int32, device="cuda")
    if incremental:
        for r in range(n_rot):                       # all copies hold the same keys: pool once
            ix.pool(Ks[r], scales[r])

    stage_names = (["widen"] if widen else []) + ["pool", "route"] + \
        (["select"] if fused else ["score", "topk"]) + (["rerank"] if wl.k_cand else [])

    def step(i, ev=None):
        K, ks = Ks[i % n_rot], scales[i % n_rot]
        mid = [lambda: ix.select_fused(Qs, W, K, ks)] if fused else [lambda: ix.score(Qs, W, K, ks), ix.select]
        pool = (lambda: ix.pool_update(K, ks, newest, 1)) if incremental else (lambda: ix.pool(K, ks))
        calls = ([lambda: misa.convert_queries(p8, Q8, Q)] if widen else []) + \
            [pool, lambda: ix.route(Q, W, K, ks)] + mid + \
            ([lambda: ix.refine(Qs, W, K, ks)] if wl.k_cand else [])
        for j, c in enumerate(calls):
            if ev is not None:
                ev[j][0].record()
            c()
            if ev is not None:
                ev[j][1].record()

    if args.copy_calibration and main_line:
        scratch = torch.empty_like(dv["K"])
        for _ in range(3):
            scratch.copy_(dv["K"])          # reads and writes key_bytes each
        torch.cuda.synchronize()
        del scratch

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # Per-stage durations: eager steps with events around every call.  The library
    # launches on torch's current stream, so torch events bracket its kernels.
    events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in stage_names] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    eager_ms = dt / args.steps * 1e3

    # The per-stage durations reported below come from a second pass of the same eager steps,
    # enqueued behind a run of plain read kernels: the host has then queued every event and
    # launch before the GPU reaches them, so an event pair brackets its kernels back to back and
    # not the host's launch latency on an idle stream (which added 2-8 us to a 97 us kernel,
    # depending on the machine's host).
    blocker = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    blocker_sink = torch.zeros(8 * 1024 * 256, dtype=torch.float32, device="cuda")
    events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in stage_names] for _ in range(args.steps)]
    torch.cuda.synchronize()
    for _ in range(int(1.5 * args.steps * eager_ms / 0.085) + 8):     # one read of 512 MiB takes about 0.085 ms
        misa.probe_hbm_read(blocker, blocker_sink)
    for i in range(args.steps):
        step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    del blocker, blocker_sink

    # Timed region proper: the same step (all calls, same buffers) captured once per
    # key-cache copy into a HIP graph and replayed, which removes the launch gaps
    # between the 5-10 short kernels of a step.  Every replay is checked against
    # the eager result.
    use_graph = not args.no_graph
    if use_graph:
        expect = ix.idx.clone()
        graphs = []
        for r in range(n_rot):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(r)
            graphs.append(g)
        for r in range(n_rot):                      # untimed: first replays + correctness of each graph
            ix.idx.fill_(-7)
            graphs[r].replay()
            torch.cuda.synchronize()
            assert torch.equal(ix.idx, expect), "graph replay differs from the eager step"
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[(args.warmup + i) % n_rot].replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        assert torch.equal(ix.idx, expect), "graph replay differs from the eager step"
        del graphs

    ms_per_step = dt / args.steps * 1e3
    pairs = wl.pairs()
    stage_ms = {n: sum(e[j][0].elapsed_time(e[j][1]) for e in events) / args.steps
                for j, n in enumerate(stage_names)}

    # The dense all-head indexer (Eq. dsa_score + Eq. dsa_topk) on the same inputs, by the same
    # library: ground truth for recall / IoU of the routed selection, and timed next to it (the
    # comparison of the kernel-speed experiment: the dense indexer needs no pooling or routing).
    pd = replace(p, h=p.H)
    dense = misa.Indexer(pd, wl.k)
    dense_reps = 3 if wl.decode else 2
    dev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(dense_reps)]
    dense.score(Q, W, Ks[0], scales[0], dense=True)
    dense.select()
    torch.cuda.synchronize()
    for r in range(dense_reps):
        K, ks = Ks[(r + 1) % n_rot], scales[(r + 1) % n_rot]
        dev[r][0].record()
        dense.score(Q, W, K, ks, dense=True)
        dense.select()
        dev[r][1].record()
    torch.cuda.synchronize()
    dense_ms = min(a.elapsed_time(b) for a, b in dev)
    rows = wl.n_seq * wl.n_q
    rec, iou = overlap_stats(ix.idx.view(rows, -1), dense.idx.view(rows, -1))
    del dense

    # pooling is a one-off per key cache in a serving loop (it is redone in every step here): the
    # timed step without the pool call's own duration
    misa_ms_excl_pool = ms_per_step - stage_ms["pool"]
    out = {
        "workload": f"{wl.name}: {DESCRIPTIONS[wl.name]}"
                    + (f" [overridden: {override}]" if override else "")
                    + (f" [key cache in pages of {args.paged} tokens]" if args.paged else ""),
        "wl": wl, "inp": inp, "fused": fused, "incremental": incremental, "use_graph": use_graph,
        "pairs": pairs, "key_bytes": key_bytes, "n_rot": n_rot,
        "ms_per_step": ms_per_step, "eager_ms": eager_ms, "stage_ms": stage_ms,
        "ms_per_step_excl_pool": misa_ms_excl_pool,
        "dense_dsa_ms": dense_ms,
        "speedup_vs_dense": dense_ms / ms_per_step,
        "speedup_vs_dense_excl_pool": dense_ms / misa_ms_excl_pool,
        "recall": float(rec.mean()), "iou": float(iou.mean()), "iou_min_row": float(iou.min()),
        "dtype": arithmetic_dtype(wl, native_fp8), "native_fp8": native_fp8,
    }
    del ix, Ks, scales
    torch.cuda.empty_cache()
    return out


def roofline_of(m: dict, peaks: dict) -> dict:
    """Roofline object of the dominant (scoring) kernel of a measured workload."""
    wl, stage_ms, pairs = m["wl"], m["stage_ms"], m["pairs"]
    score_s = stage_ms["select" if m["fused"] else "score"] * 1e-3
    if wl.decode:
        algo = pairs * key_bytes_per_pair(wl)
        prof = PROFILED_TRAFFIC.get(wl.name)
        roof = {"kernel": "score_stream_kernel", "bound": "hbm", "achieved": algo / score_s / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": algo / score_s / 1e9 / HBM_PEAK_GBS,
                "traffic": None,
                "traffic_from_profile": None if prof is None else
                {"bytes": prof[0], "source": prof[1], "note": "recorded constant (rocprofv3 --pmc FETCH_SIZE + "
                 "WRITE_SIZE, copy-calibrated), not measured by this run"},
                "algorithmic_bytes": algo, "avg_launch_ms": stage_ms["score"]}
        roof["measured_peak"] = peaks["hbm_read_GBps"]
    else:
        flops = 2.0 * pairs * wl.h * wl.d
        kind = "fp8" if m["native_fp8"] else "bf16"
        peak = MFMA_PEAK_TFLOPS[kind]
        # the fused call scores 17/16 of the pairs (the 1/16 sample and the full pass); only the
        # algorithmic flops are counted, so its fraction understates the matrix work done
        roof = {"kernel": "misa_select_tokens (sample + filter scoring passes + list top-k)" if m["fused"]
                else "score_tile_kernel", "bound": "mfma", "achieved": flops / score_s / 1e12,
                "peak": peak, "unit": "TFLOP/s", "frac": flops / score_s / 1e12 / peak, "traffic": None,
                "algorithmic_flops": flops, "avg_launch_ms": score_s * 1e3, "matrix_dtype": kind}
        roof["measured_peak"] = peaks["mfma_bf16_TFLOPs"] * (2.0 if kind == "fp8" else 1.0)
        if kind == "bf16":
            # the same probe on Gaussian bf16 operands of the workloads' scale: the rate the matrix pipe
            # sustains on such data with nothing else in the kernel (the clock the chip holds depends
            # on the operand values)
            roof["measured_peak_gaussian_operands"] = peaks["mfma_bf16_gaussian_operands_TFLOPs"]
            roof["frac_of_measured_gaussian_operands"] = roof["achieved"] / peaks["mfma_bf16_gaussian_operands_TFLOPs"]
        if kind == "fp8":
            roof["measured_peak_note"] = "2 x the measured bf16 matrix rate (the probe issues bf16 instructions)"
    roof["frac_of_measured"] = roof["achieved"] / roof["measured_peak"]
    return roof


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, choices=sorted(DESCRIPTIONS),
                    help="default: c3, followed by the prefill companion c4 (object `prefill`)")
    ap.add_argument("--no-prefill", action="store_true", help="default run: skip the prefill companion workload")
    ap.add_argument("--block", type=int, default=0, help="override the router block size B of the workload")
    ap.add_argument("--active-heads", type=int, default=0, help="override the number of active heads h")
    ap.add_argument("--fused", action="store_true",
                    help="stages 3+4 as one misa_select_tokens call (no score matrix); prefill workloads")
    ap.add_argument("--incremental-pool", action="store_true",
                    help="decode workloads: the pooled keys of earlier tokens are kept and a step only re-pools "
                         "the block of the newest token (misa_pool_keys_update), as a serving loop would")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE_SIZE",
                    help="keep the key cache as a pool of scattered pages of PAGE_SIZE tokens (misa_problem.page_table)")
    ap.add_argument("--fp8-queries", action="store_true",
                    help="queries stored as e4m3 codes (scale folded into the gates).  Prefill workloads with fp8 "
                         "keys then score on the fp8 matrix instruction; elsewhere a step starts with "
                         "misa_convert_queries and the stages run on the widened queries")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rotate", type=int, default=3, help="key-cache copies rotated between steps (cold reads)")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every kernel eagerly in the timed steps instead of replaying a HIP graph of the step")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain device copies of the key cache (known size), as the reference "
                         "reading for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the indexer shards by sequence / query rows "
              "without communication); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2605_07363_amd import misa, workloads as WL

    default_run = args.workload is None
    name = args.workload or "c3"
    wl0 = WL.WORKLOADS[name]
    if args.fused and wl0.decode:
        print("bench.py: --fused applies to the prefill workloads (c2, c4)", file=sys.stderr)
        return 2
    if args.incremental_pool and not wl0.decode:
        print("bench.py: --incremental-pool applies to the decode workloads (c0, c1, c3)", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    # What this GPU delivers (outside every timed region): the library's read and matrix-instruction
    # probes, so that achieved rates can be read against the measured as well as the published peak.
    peaks = misa.measured_peaks()

    m = measure(args, name, args.fused, True)
    wl = m["wl"]
    roof = roofline_of(m, peaks)
    out = {
        "metric": "indexer query-key pairs/s (whole pass: pool+route+score+top-k" + ("+re-rank)" if wl.k_cand else ")")
                  + (" [score+top-k fused]" if m["fused"] else "")
                  + (" [pool: newest block only]" if m["incremental"] else ""),
        "value": m["pairs"] / (m["ms_per_step"] * 1e-3), "unit": "pairs/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": m["dtype"], "data": "synthetic",
        "config": {"workload": m["workload"], "pairs_per_step": m["pairs"],
                   "key_cache_bytes": m["key_bytes"], "key_buffers_rotated": m["n_rot"]},
        "launch": "hip-graph replay of the whole step" if m["use_graph"] else "eager",
        "eager_ms_per_step": m["eager_ms"],
        "stage_timing": "HIP events around every call of eager steps that were queued behind plain read kernels "
                        "(the GPU never waits for the host between an event and the launch it brackets)",
        "stage_ms": m["stage_ms"],
        "ms_per_step_excl_pool": m["ms_per_step_excl_pool"],
        "score_stage_pairs_per_s": m["pairs"] / (m["stage_ms"]["select" if m["fused"] else "score"] * 1e-3),
        "roofline": roof,
        "measured_peaks": peaks,
        "recall_of_dense_topk": m["recall"],
        "iou_with_dense_topk": m["iou"],
        # the dense all-head indexer (score + top-k, no pooling or routing) timed by the same run
        "dense_dsa_ms": m["dense_dsa_ms"],
        "speedup_vs_dense": m["speedup_vs_dense"],
        "speedup_vs_dense_excl_pool": m["speedup_vs_dense_excl_pool"],
    }

    if default_run and not args.no_prefill:
        # The matrix-core half of the metric: the MISA-dagger prefill workload at the same L (c4) and
        # the single-stage DeepSeek-V3.2-shaped chunk (c2), each as separate calls
        # (score_tile_kernel writes the score matrix) and with scoring + top-k fused.
        import copy
        pargs = copy.copy(args)
        pargs.steps, pargs.warmup = min(args.steps, 10), min(args.warmup, 2)

        def prefill_object(name, fp8_queries=False):
            margs = copy.copy(pargs)
            margs.fp8_queries = fp8_queries
            two = measure(margs, name, False, False)
            one = measure(margs, name, True, False)
            r2, r1 = roofline_of(two, peaks), roofline_of(one, peaks)
            w = two["wl"]
            obj = {
                "workload": two["workload"], "pairs_per_step": two["pairs"], "dtype": two["dtype"],
                "steps": pargs.steps, "warmup": pargs.warmup,
                "ms_per_step": two["ms_per_step"], "value_pairs_per_s": two["pairs"] / (two["ms_per_step"] * 1e-3),
                "stage_ms": two["stage_ms"], "ms_per_step_excl_pool": two["ms_per_step_excl_pool"],
                "roofline": r2,
                "score_tile_ms": two["stage_ms"]["score"],
                "fused": {"ms_per_step": one["ms_per_step"], "stage_ms": one["stage_ms"],
                          "fused_select_ms": one["stage_ms"]["select"], "roofline": r1,
                          "value_pairs_per_s": one["pairs"] / (one["ms_per_step"] * 1e-3)},
                "recall_of_dense_topk": two["recall"], "iou_with_dense_topk": two["iou"],
                "dense_dsa_ms": two["dense_dsa_ms"],
                "speedup_vs_dense": two["speedup_vs_dense"],
                "speedup_vs_dense_fused": one["speedup_vs_dense"],
            }
            if w.k_cand:
                flops = 2.0 * w.n_seq * w.n_q * w.k_cand * w.H * w.d
                obj["rerank_ms"] = two["stage_ms"]["rerank"]
                obj["rerank_TFLOPs"] = flops / (obj["rerank_ms"] * 1e-3) / 1e12
                obj["rerank_frac_of_bf16_peak"] = obj["rerank_TFLOPs"] / MFMA_PEAK_TFLOPS["bf16"]
            return obj

        out["prefill"] = prefill_object("c4")
        out["prefill_single_stage"] = prefill_object("c2")
        # the same MISA-dagger prefill with the queries quantised to e4m3 as well (the paper notes that
        # DSA runs its indexer in FP8): both operands stay fp8 codes, products on the fp8 matrix
        # instruction, priced against the fp8 peak
        out["prefill_fp8_queries"] = prefill_object("c4", fp8_queries=True)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, m["inp"])
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
