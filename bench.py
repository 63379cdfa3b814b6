#!/usr/bin/env python3
"""Benchmark of the MISA indexer hot path on one MI355X.

A step is one pass of the whole indexer (pool -> route -> score -> top-k, plus
the dense re-rank for the MISA-dagger workload) over one batch of seeded
synthetic inputs that are already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3]
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16

# HBM bytes per launch of the score kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a
# plain device copy of known size in the same run (profiles/score_stream_*_hbm_traffic.md).
MEASURED_TRAFFIC_BYTES = {"c1": 548.8e6, "c3": 571.0e6}

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


def cpu_baseline(wl, inp, budget_s: float = 20.0) -> dict:
    """Time the fp64 oracle as it stands on a bounded sample of the same workload."""
    import numpy as np
    from oracle import misa_oracle as O
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import oracle_view
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = 1
    rng = np.random.default_rng(0)
    rows = [(s, t) for s in range(wl.n_seq) for t in range(wl.n_q)]
    order = rng.permutation(len(rows))
    pairs, done, t0 = 0, 0, time.perf_counter()
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
    return {"value": pairs / dt, "unit": "pairs/s", "cores": threads, "kind": "oracle",
            "sample": f"{done} of {len(rows)} query rows of {wl.name} (whole pipeline incl. de-quantisation and "
                      f"pooling per row), {dt:.1f} s"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=sorted(DESCRIPTIONS))
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
                    help="queries stored as e4m3 codes (scale folded into the gates); a step then starts with "
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

    wl = WL.WORKLOADS[args.workload]
    override = {k: v for k, v in (("B", args.block), ("h", args.active_heads),
                                  ("q_dtype", "e4m3" if args.fp8_queries else None)) if v}
    if override:
        wl = WL.scaled(wl, **override)
    torch.cuda.set_device(0)
    inp = WL.make_inputs(wl)
    dv = misa.to_device(inp)
    key_bytes = dv["K"].numel() * dv["K"].element_size()
    if args.paged:
        dv = misa.paginate(dv, args.paged, seed=1)
    p = dv["problem"]
    Q, W = dv["Q"], dv["W"]
    Q8, p8 = None, None
    if args.fp8_queries:
        from dataclasses import replace as _replace
        Q8, p8 = Q, p
        Q = torch.empty(Q8.shape, dtype=torch.bfloat16, device="cuda")
        p = _replace(p, q_dtype=misa.BF16)
    # Decode caches are far larger than the 256 MB last-level cache; rotating
    # copies keeps every step's key reads cold.  Prefill caches are small and
    # are re-read by every query tile, so one copy is the workload.
    n_rot = max(1, args.rotate) if wl.decode else 1
    Ks = [dv["K"]] + [dv["K"].clone() for _ in range(n_rot - 1)]
    scales = [dv["kscale"]] + [None if dv["kscale"] is None else dv["kscale"].clone() for _ in range(n_rot - 1)]
    if args.fused and wl.decode:
        print("bench.py: --fused applies to the prefill workloads (c2, c4)", file=sys.stderr)
        return 2
    ix = misa.Indexer(p, wl.k, wl.k_cand, fused=args.fused)

    if args.incremental_pool and not wl.decode:
        print("bench.py: --incremental-pool applies to the decode workloads (c0, c1, c3)", file=sys.stderr)
        return 2
    newest = torch.full((wl.n_seq,), wl.L - 1, dtype=torch.int32, device="cuda")
    if args.incremental_pool:
        for r in range(n_rot):                       # all copies hold the same keys: pool once
            ix.pool(Ks[r], scales[r])

    stage_names = (["widen"] if args.fp8_queries else []) + ["pool", "route"] + \
        (["select"] if args.fused else ["score", "topk"]) + (["rerank"] if wl.k_cand else [])

    def step(i, ev=None):
        K, ks = Ks[i % n_rot], scales[i % n_rot]
        mid = [lambda: ix.select_fused(Q, W, K, ks)] if args.fused else [lambda: ix.score(Q, W, K, ks), ix.select]
        pool = (lambda: ix.pool_update(K, ks, newest, 1)) if args.incremental_pool else (lambda: ix.pool(K, ks))
        calls = ([lambda: misa.convert_queries(p8, Q8, Q)] if args.fp8_queries else []) + \
            [pool, lambda: ix.route(Q, W, K, ks)] + mid + \
            ([lambda: ix.refine(Q, W, K, ks)] if wl.k_cand else [])
        for j, c in enumerate(calls):
            if ev is not None:
                ev[j][0].record()
            c()
            if ev is not None:
                ev[j][1].record()

    if args.copy_calibration:
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

    # Outside the timed region: which fraction of the dense all-head selection (Eq. dsa_topk)
    # the routed selection recovered, both computed by the library on the same inputs.
    from dataclasses import replace
    from paper_2605_07363_amd.recall_sweep import overlap
    dense = misa.Indexer(replace(p, h=p.H), wl.k)
    dense.score(Q, W, Ks[0], scales[0], dense=True)
    dense.select()
    rows = wl.n_seq * wl.n_q
    recall = overlap(ix.idx.view(rows, -1), dense.idx.view(rows, -1))
    del dense

    ms_per_step = dt / args.steps * 1e3
    pairs = wl.pairs()
    stage_ms = {n: sum(e[j][0].elapsed_time(e[j][1]) for e in events) / args.steps
                for j, n in enumerate(stage_names)}

    # the scoring work: the score call, or the fused call (which scores 17/16 of the pairs:
    # the 1/16 sample and the full pass; only the algorithmic flops are counted)
    score_s = stage_ms["select" if args.fused else "score"] * 1e-3
    if wl.decode:
        algo = pairs * key_bytes_per_pair(wl)
        roof = {"kernel": "score_stream_kernel", "bound": "hbm", "achieved": algo / score_s / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": algo / score_s / 1e9 / HBM_PEAK_GBS,
                "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name), "algorithmic_bytes": algo,
                "avg_launch_ms": stage_ms["score"]}
    else:
        flops = 2.0 * pairs * wl.h * wl.d
        roof = {"kernel": "misa_select_tokens (sample + filter scoring passes + list top-k)" if args.fused
                else "score_tile_kernel", "bound": "mfma", "achieved": flops / score_s / 1e12,
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": flops / score_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                "algorithmic_flops": flops, "avg_launch_ms": score_s * 1e3}

    # What this GPU delivers (outside the timed region): the library's read and matrix-instruction
    # probes, so that the achieved rate can be read against the measured as well as the published peak.
    peaks = misa.measured_peaks()
    roof["measured_peak"] = peaks["hbm_read_GBps" if wl.decode else "mfma_bf16_TFLOPs"]
    roof["frac_of_measured"] = roof["achieved"] / roof["measured_peak"]

    out = {
        "metric": "indexer query-key pairs/s (whole pass: pool+route+score+top-k" + ("+re-rank)" if wl.k_cand else ")")
                  + (" [score+top-k fused]" if args.fused else "")
                  + (" [pool: newest block only]" if args.incremental_pool else ""),
        "value": pairs / (dt / args.steps), "unit": "pairs/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if wl.k_dtype == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {DESCRIPTIONS[wl.name]}"
                               + (f" [overridden: {override}]" if override else "")
                               + (f" [key cache in pages of {args.paged} tokens]" if args.paged else ""),
                   "pairs_per_step": pairs,
                   "key_cache_bytes": key_bytes, "key_buffers_rotated": n_rot},
        "launch": "hip-graph replay of the whole step" if use_graph else "eager",
        "eager_ms_per_step": eager_ms,
        "stage_ms": stage_ms,
        "score_stage_pairs_per_s": pairs / score_s,
        "roofline": roof,
        "measured_peaks": peaks,
        "recall_of_dense_topk": recall,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, inp)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
