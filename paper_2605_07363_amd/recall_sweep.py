#!/usr/bin/env python3
"""Overlap of the routed selection with the dense one over (h, B) on synthetic keys.

For a decode workload this runs the whole indexer on the GPU for every
combination of active heads h and router block size B (the two
hyper-parameters of the method; Experimental results, "Default MISA
hyperparameters", and the ablations on B and h), once single-stage (MISA,
Eq. misa_topk) and once with the dense re-rank of k' = 4k candidates (Eq.
misa_final_topk), and reports which fraction of the dense all-head top-k set
(Eq. dsa_topk) each selection recovers; the same for the two content-free
router scores of the appendix "Ablation: routing score" (gate alone, query
norm) and for the HISA and Block-Sparse comparison indexers at B = 128.  The inputs are the seeded synthetic
caches of workloads.py, so the figures describe those inputs, not a trained
model.

    python -m paper_2605_07363_amd.recall_sweep [--workload c3] [--n-seq 8]
"""
from __future__ import annotations

import argparse
import json
import sys


def _membership(a, b):
    import torch
    n = int(max(a.max(), b.max())) + 2
    rows = a.shape[0]
    ma = torch.zeros((rows, n), dtype=torch.bool, device=a.device)
    mb = torch.zeros_like(ma)
    ma.scatter_(1, (a.long() + 1), True)
    mb.scatter_(1, (b.long() + 1), True)
    ma[:, 0] = False          # column 0 collects the -1 entries (no token)
    mb[:, 0] = False
    return ma, mb


def overlap_stats(a, b):
    """Per row of two index tensors [rows, ka], [rows, kb] (entries -1 = none): the fraction of
    b's tokens that a holds as well (recall of b; 1 for an empty b) and the intersection over
    union of the two sets (Eq. iou; 1 when both are empty).  Returns two float tensors [rows]."""
    ma, mb = _membership(a, b)
    inter = (ma & mb).sum(1).double()
    nb = mb.sum(1).double()
    union = (ma | mb).sum(1).double()
    one = inter.new_ones(())
    recall = (inter / nb.clamp(min=1)).where(nb > 0, one)
    iou = (inter / union.clamp(min=1)).where(union > 0, one)
    return recall, iou


def overlap(a, b):
    """Mean over rows of |a_row ∩ b_row| / |b_row| for index tensors [rows, k] (entries -1 = none)."""
    return float(overlap_stats(a, b)[0].mean())


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c3", choices=["c1", "c3"])
    ap.add_argument("--n-seq", type=int, default=8)
    ap.add_argument("--heads", default="1,2,4,8,16")
    ap.add_argument("--blocks", default="64,128,1024,0", help="router block sizes; 0 = one block for the whole prefix")
    args = ap.parse_args()

    import torch
    from dataclasses import replace
    from . import misa, workloads as WL

    base = WL.scaled(WL.WORKLOADS[args.workload], n_seq=args.n_seq)
    inp = WL.make_inputs(base)
    dv = misa.to_device(inp)
    K, ks, Q, W = dv["K"], dv["kscale"], dv["Q"], dv["W"]
    rows = base.n_seq * base.n_q

    def problem(h, B):
        p = dv["problem"]
        return replace(p, h=h, B=B)

    # dense reference: every head active
    dense = misa.Indexer(problem(base.H, base.B), base.k)
    dense.score(Q, W, K, ks, dense=True)
    dense.select()
    ref = dense.idx.view(rows, -1).clone()

    out = []
    for B in [int(x) or base.L for x in args.blocks.split(",")]:
        for h in [int(x) for x in args.heads.split(",") if int(x) <= base.H]:
            p = problem(h, B)
            one = misa.Indexer(p, base.k)
            r1 = overlap(one.run(K, ks, Q, W).view(rows, -1), ref)
            two = misa.Indexer(p, base.k, 4 * base.k)
            r2 = overlap(two.run(K, ks, Q, W).view(rows, -1), ref)
            out.append({"B": B, "h": h, "misa_recall": round(r1, 4), "misa_dagger_recall": round(r2, 4)})
            print(f"B={B:7d} h={h:3d}  MISA {r1:.4f}  MISA-dagger(k'=4k) {r2:.4f}", file=sys.stderr, flush=True)
    # the two content-free router scores of the appendix "Ablation: routing score" (no block size)
    proxy = []
    for h in [int(x) for x in args.heads.split(",") if int(x) <= base.H]:
        row = {"h": h}
        for name, kind in (("gate", misa.ROUTER_GATE), ("query_norm", misa.ROUTER_QUERY_NORM)):
            ix = misa.Indexer(problem(h, base.B), base.k)
            misa.route_heads_proxy(ix.p, Q, W, kind, ix.heads)
            ix.score(Q, W, K, ks)
            ix.select()
            row[name + "_recall"] = round(overlap(ix.idx.view(rows, -1), ref), 4)
        proxy.append(row)
        print(f"router ablation h={h:3d}  gate {row['gate_recall']:.4f}  query norm {row['query_norm_recall']:.4f}",
              file=sys.stderr, flush=True)
    # comparison indexers with the paper's baseline block size B = 128 and the same token budget
    bp = problem(base.h, 128)
    Kp = torch.empty((base.n_seq, bp.M, base.d), dtype=torch.float32, device="cuda")
    misa.pool_keys(bp, K, ks, Kp, misa.alloc_workspace(bp, misa.OP_POOL))
    baselines = {}
    m_hisa = 4 * base.k // 128                      # candidate tokens = 4k, as MISA-dagger's k'
    idx = torch.empty((base.n_seq, base.n_q, base.k), dtype=torch.int32, device="cuda")
    misa.hisa_select(bp, Q, W, Kp, K, ks, m_hisa, base.k, idx, None, None, misa.alloc_workspace(bp, misa.OP_HISA, m_hisa))
    baselines["hisa_B128_m%d_recall" % m_hisa] = round(overlap(idx.view(rows, -1), ref), 4)
    m_bs = base.k // 128                            # m = k / B blocks
    bidx = torch.empty((base.n_seq, base.n_q, m_bs * 128), dtype=torch.int32, device="cuda")
    misa.block_sparse_select(bp, Q, W, Kp, m_bs, bidx, None, misa.alloc_workspace(bp, misa.OP_HISA, m_bs))
    baselines["block_sparse_B128_m%d_recall" % m_bs] = round(overlap(bidx.view(rows, -1), ref), 4)
    print("comparison indexers:", baselines, file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    print(json.dumps({"workload": base.name, "n_seq": base.n_seq, "L": base.L, "H": base.H, "k": base.k,
                      "rows": out, "router_ablation": proxy, "baselines": baselines}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
