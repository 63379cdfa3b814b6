"""fp8 (e4m3) queries: every call that takes queries is compared with the oracle on the decoded
codes, and with the same call on the queries widened to bf16 (which must agree bit for bit)."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import misa_oracle as O
from paper_2605_07363_amd import workloads as WL
from helpers import assert_scores_close, check_index_set, oracle_view

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def misa():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2605_07363_amd import misa as m
    return m


CASES = {
    "decode_fp8_keys": WL.scaled(WL.WORKLOADS["c3"], n_seq=3, L=4133, B=128, k=300, needles=16, q_dtype="e4m3"),
    "decode_bf16_keys": WL.scaled(WL.WORKLOADS["c1"], n_seq=2, L=3000, B=64, k=200, q_dtype="e4m3"),
    "prefill_fp8_keys": WL.scaled(WL.WORKLOADS["c4"], L=4500, n_q=40, B=64, k=128, k_cand=512, needles=16,
                                  q_dtype="e4m3"),
    "prefill_bf16_keys": WL.scaled(WL.WORKLOADS["c2"], L=3000, n_q=70, B=64, k=200, q_dtype="e4m3"),
    "f32_keys": WL.scaled(WL.WORKLOADS["c0"], L=1500, B=64, q_dtype="e4m3"),
}


def stages(misa, wl, p, K, ks, Q, W):
    out = {}
    Kp = torch.empty((wl.n_seq, p.M, wl.d), dtype=torch.float32, device="cuda")
    misa.pool_keys(p, K, ks, Kp, misa.alloc_workspace(p, misa.OP_POOL))
    heads = torch.empty((wl.n_seq, wl.n_q, wl.h), dtype=torch.int32, device="cuda")
    E = torch.empty((wl.n_seq, wl.n_q, wl.H), dtype=torch.float32, device="cuda")
    misa.route_heads(p, Q, W, Kp, K, ks, heads, E, misa.alloc_workspace(p, misa.OP_ROUTE))
    out["heads"], out["E"] = heads, E
    S = torch.empty((wl.n_seq, wl.n_q, wl.L), dtype=torch.float32, device="cuda")
    misa.score_tokens(p, Q, W, heads, K, ks, S, misa.alloc_workspace(p, misa.OP_SCORE))
    out["S"] = S
    k1 = min(wl.k_cand or wl.k, wl.L)
    idx = torch.empty((wl.n_seq, wl.n_q, k1), dtype=torch.int32, device="cuda")
    misa.topk(p, S, k1, idx, None, misa.alloc_workspace(p, misa.OP_TOPK, k1))
    out["idx"] = idx
    k2 = min(wl.k, k1)
    fin = torch.empty((wl.n_seq, wl.n_q, k2), dtype=torch.int32, device="cuda")
    val = torch.empty((wl.n_seq, wl.n_q, k2), dtype=torch.float32, device="cuda")
    misa.rerank(p, Q, W, K, ks, idx, k1, k2, fin, val, misa.alloc_workspace(p, misa.OP_RERANK, k1))
    out["rerank_idx"], out["rerank_val"] = fin, val
    ph = torch.empty_like(heads)
    misa.route_heads_proxy(p, Q, W, misa.ROUTER_QUERY_NORM, ph)
    out["proxy_heads"] = ph
    return out


@pytest.mark.parametrize("name", list(CASES))
def test_fp8_queries_against_oracle_and_widened_queries(misa, name):
    wl = CASES[name]
    inp = WL.make_inputs(wl, seed=321 + sum(map(ord, name)))
    dv = misa.to_device(inp)
    p = dv["problem"]
    assert p.q_dtype == misa.FP8_E4M3 and dv["Q"].dtype == torch.uint8
    got = stages(misa, wl, p, dv["K"], dv["kscale"], dv["Q"], dv["W"])
    # (a) bit-identical to the same calls on the widened queries
    q16 = torch.empty(dv["Q"].shape, dtype=torch.bfloat16, device="cuda")
    misa.convert_queries(p, dv["Q"], q16)
    table = O.e4m3fn_decode_table()
    np.testing.assert_array_equal(q16.float().cpu().numpy().astype(np.float64), table[inp["Q"]])
    same = stages(misa, wl, replace(p, q_dtype=misa.BF16), dv["K"], dv["kscale"], q16, dv["W"])
    for key in got:
        assert torch.equal(got[key], same[key]), key
    # (b) the oracle on the decoded codes: router scores, token scores with the GPU's heads, dense re-rank values
    E, heads, S = got["E"].cpu().numpy(), got["heads"].cpu().numpy(), got["S"].cpu().numpy()
    fin, val = got["rerank_idx"].cpu().numpy(), got["rerank_val"].cpu().numpy()
    for s in range(wl.n_seq):
        for t in sorted({0, wl.n_q // 2, wl.n_q - 1}):
            K, q, w, n = oracle_view(inp, s, t)
            _, ref_E = O.route_heads(q, w, K, wl.B, wl.h, n)
            assert_scores_close(E[s, t], ref_E, f"E {name} {s},{t}")
            check_index_set(heads[s, t], ref_E, wl.h, f"heads {name} {s},{t}")
            ref_S = O.score_tokens(q, w, heads[s, t], K, n)
            assert_scores_close(S[s, t, :n], ref_S, f"S {name} {s},{t}")
            assert np.all(np.isneginf(S[s, t, n:]))
            dense = O.score_tokens(q, w, np.arange(wl.H), K, n)
            keep = fin[s, t][fin[s, t] >= 0]
            assert_scores_close(val[s, t, :keep.shape[0]], dense[keep], f"re-rank values {name} {s},{t}")


def test_fp8_queries_whole_pipeline_and_fused_call(misa):
    wl = WL.scaled(WL.WORKLOADS["c2"], L=8192, n_q=256, B=128, k=256, q_dtype="e4m3")
    inp = WL.make_inputs(wl, seed=11)
    dv = misa.to_device(inp)
    p = dv["problem"]
    ia = misa.Indexer(p, wl.k)
    a = ia.run(dv["K"], dv["kscale"], dv["Q"], dv["W"]).clone()
    ia.idx.fill_(-3)
    assert torch.equal(ia.run(dv["K"], dv["kscale"], dv["Q"], dv["W"]), a)     # and again on the same object
    b = misa.Indexer(p, wl.k, fused=True).run(dv["K"], dv["kscale"], dv["Q"], dv["W"]).clone()
    assert torch.equal(a, b)
    # the fused call on the codes themselves (widening inside the call)
    ix = misa.Indexer(p, wl.k, fused=True)
    ix.pool(dv["K"], dv["kscale"]); ix.route(dv["Q"], dv["W"], dv["K"], dv["kscale"])
    ix.select_fused(dv["Q"], dv["W"], dv["K"], dv["kscale"])
    assert torch.equal(ix.idx, a)
    got = a.cpu().numpy()
    for t in (0, 100, 255):
        K, q, w, n = oracle_view(inp, 0, t)
        ref = O.misa(q, w, K, wl.B, wl.h, wl.k, n)
        # a legal head flip inside the tolerance would change the set; at these sizes none occurs
        np.testing.assert_array_equal(got[0, t], ref["tokens"])
