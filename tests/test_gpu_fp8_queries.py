"""fp8 (e4m3) queries: every call that takes queries is compared with the oracle on the decoded
codes, and with the same call on the queries widened to bf16 (which must agree bit for bit)."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import misa_oracle as O
from paper_2605_07363_amd import workloads as WL
from helpers import ABS_FRAC_FP8_MATRIX, assert_scores_close, check_index_set, oracle_view

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


# ---------------------------------------------------------------- fp8 matrix instruction
MATRIX_CASES = {
    # head-slot widths 8, 16, 32 and 64 of the tile kernel, ragged tails, several key ranges
    "h8": WL.scaled(WL.WORKLOADS["c4"], L=9000, n_q=70, B=64, k=128, k_cand=512, needles=16, q_dtype="e4m3"),
    "h16": WL.scaled(WL.WORKLOADS["c4"], L=2500, n_q=21, h=16, B=64, k=100, k_cand=300, needles=8, q_dtype="e4m3"),
    "h32_H32": WL.scaled(WL.WORKLOADS["c4"], L=1100, n_q=13, H=32, h=32, B=32, k=64, k_cand=256, needles=8, q_dtype="e4m3"),
    "h3": WL.scaled(WL.WORKLOADS["c4"], L=900, n_q=33, h=3, B=16, k=50, k_cand=200, needles=4, q_dtype="e4m3"),
}


@pytest.mark.parametrize("name", list(MATRIX_CASES))
@pytest.mark.parametrize("paged", [0, 64])
def test_fp8_matrix_instruction_scores_against_oracle(misa, name, paged):
    # q_dtype FP8_E4M3_MATRIX with fp8 keys: routed and dense (all heads) scores of the tile kernel
    # against the oracle on the decoded codes, element by element, under the tolerance of that path
    wl = MATRIX_CASES[name]
    inp = WL.make_inputs(wl, seed=77 + sum(map(ord, name)))
    dv = misa.to_device(inp)
    if paged:
        dv = misa.paginate(dv, paged, seed=2)
    p = replace(dv["problem"], q_dtype=misa.FP8_E4M3_MATRIX)
    ref_heads = np.zeros((wl.n_seq, wl.n_q, wl.h), dtype=np.int32)
    views = {}
    for t in range(wl.n_q):
        K, q, w, n = views[t] = oracle_view(inp, 0, t)
        ref_heads[0, t] = O.route_heads(q, w, K, wl.B, wl.h, n)[0]
    S = torch.full((1, wl.n_q, wl.L), 3.0, dtype=torch.float32, device="cuda")
    ws = misa.alloc_workspace(p, misa.OP_SCORE)
    misa.score_tokens(p, dv["Q"], dv["W"], torch.from_numpy(ref_heads).cuda(), dv["K"], dv["kscale"], S, ws)
    D = torch.empty_like(S)
    misa.score_tokens(p, dv["Q"], dv["W"], None, dv["K"], dv["kscale"], D, ws)
    got, dense = S.cpu().numpy(), D.cpu().numpy()
    for t in range(wl.n_q):
        K, q, w, n = views[t]
        assert_scores_close(got[0, t, :n], O.score_tokens(q, w, ref_heads[0, t], K, n), f"S {name} {t}",
                            abs_frac=ABS_FRAC_FP8_MATRIX)
        assert_scores_close(dense[0, t, :n], O.dsa_scores(q, w, K, n), f"dense S {name} {t}",
                            abs_frac=ABS_FRAC_FP8_MATRIX)
        assert np.all(np.isneginf(got[0, t, n:])) and np.all(np.isneginf(dense[0, t, n:]))


def test_fp8_matrix_instruction_pipeline_and_fused_call(misa):
    # whole MISA-dagger pass with the scoring stage on the codes: fused call = two calls bit for bit,
    # candidates valid under the margin rule of that path, re-rank against the dense oracle scores
    wl = WL.scaled(WL.WORKLOADS["c4"], L=16384, n_q=128, B=64, k=256, k_cand=1024, needles=16, q_dtype="e4m3")
    inp = WL.make_inputs(wl, seed=12)
    dv = misa.to_device(inp)
    p = replace(dv["problem"], q_dtype=misa.FP8_E4M3_MATRIX)
    two = misa.Indexer(p, wl.k, wl.k_cand, want_val=True)
    a = two.run(dv["K"], dv["kscale"], dv["Q"], dv["W"]).clone()
    one = misa.Indexer(p, wl.k, wl.k_cand, fused=True, want_val=True)
    b = one.run(dv["K"], dv["kscale"], dv["Q"], dv["W"]).clone()
    assert torch.equal(two.idx1, one.idx1) and torch.equal(a, b)
    assert torch.equal(two.heads, one.heads)
    heads, cand, fin = two.heads.cpu().numpy(), two.idx1.cpu().numpy(), a.cpu().numpy()
    S = two.S.cpu().numpy()
    for t in (0, 1, 63, 64, 127):
        K, q, w, n = oracle_view(inp, 0, t)
        ref_S = O.score_tokens(q, w, heads[0, t], K, n)
        assert_scores_close(S[0, t, :n], ref_S, f"scores {t}", abs_frac=ABS_FRAC_FP8_MATRIX)
        check_index_set(cand[0, t], ref_S, wl.k_cand, f"candidates {t}", abs_frac=ABS_FRAC_FP8_MATRIX)
        dense = O.dsa_scores(q, w, K, n)
        c = cand[0, t][cand[0, t] >= 0]
        f = fin[0, t][fin[0, t] >= 0]
        pos = np.searchsorted(c, f)
        check_index_set(np.concatenate([pos, np.full(wl.k - pos.shape[0], -1, dtype=pos.dtype)]), dense[c], wl.k,
                        f"re-rank {t}", abs_frac=ABS_FRAC_FP8_MATRIX)
        assert_scores_close(two.val.cpu().numpy()[0, t, :f.shape[0]], dense[f], f"re-rank values {t}",
                            abs_frac=ABS_FRAC_FP8_MATRIX)


@pytest.mark.parametrize("name", ["prefill_fp8_keys", "decode_fp8_keys"])
def test_fp8_matrix_rerank_against_oracle(misa, name):
    # misa_rerank on fp8 codes (H = 64 and H = 32 row tiles, one query and many): dense scores of the
    # listed candidates against Eq. dsa_score, selection by the margin rule of that path
    wl = CASES[name]
    inp = WL.make_inputs(wl, seed=55)
    dv = misa.to_device(inp)
    p = replace(dv["problem"], q_dtype=misa.FP8_E4M3_MATRIX)
    rng = np.random.default_rng(8)
    kc, k = 700, 128
    cand = np.full((wl.n_seq, wl.n_q, kc), -1, dtype=np.int32)
    for s in range(wl.n_seq):
        for t in range(wl.n_q):
            n = oracle_view(inp, s, t)[3]
            m = min(kc - 5, n)
            cand[s, t, :m] = np.sort(rng.choice(n, m, replace=False))
    idx = torch.empty((wl.n_seq, wl.n_q, k), dtype=torch.int32, device="cuda")
    val = torch.empty((wl.n_seq, wl.n_q, k), dtype=torch.float32, device="cuda")
    misa.rerank(p, dv["Q"], dv["W"], dv["K"], dv["kscale"], torch.from_numpy(cand).cuda(), kc, k, idx, val,
                misa.alloc_workspace(p, misa.OP_RERANK, kc))
    got, gv = idx.cpu().numpy(), val.cpu().numpy()
    for s in range(wl.n_seq):
        for t in sorted({0, wl.n_q // 2, wl.n_q - 1}):
            K, q, w, n = oracle_view(inp, s, t)
            dense = O.dsa_scores(q, w, K, n)
            c = cand[s, t][cand[s, t] >= 0]
            f = got[s, t][got[s, t] >= 0]
            pos = np.searchsorted(c, f)
            check_index_set(np.concatenate([pos, np.full(k - pos.shape[0], -1, dtype=pos.dtype)]), dense[c], k,
                            f"re-rank {name} {s},{t}", abs_frac=ABS_FRAC_FP8_MATRIX)
            assert_scores_close(gv[s, t, :f.shape[0]], dense[f], f"re-rank values {name} {s},{t}",
                                abs_frac=ABS_FRAC_FP8_MATRIX)


def test_fp8_matrix_dtype_elsewhere_is_plain_fp8(misa):
    # decode-shaped problems and bf16 keys do not take the fp8 instruction: results equal those of
    # q_dtype FP8_E4M3 bit for bit
    for name in ("decode_fp8_keys", "prefill_bf16_keys"):
        wl = CASES[name]
        dv = misa.to_device(WL.make_inputs(wl, seed=5))
        p = dv["problem"]
        a = stages(misa, wl, p, dv["K"], dv["kscale"], dv["Q"], dv["W"])
        b = stages(misa, wl, replace(p, q_dtype=misa.FP8_E4M3_MATRIX), dv["K"], dv["kscale"], dv["Q"], dv["W"])
        for key in a:
            if name == "decode_fp8_keys" and key.startswith("rerank"):
                continue                      # the candidate gather does take the codes (tested above)
            assert torch.equal(a[key], b[key]), (name, key)


@pytest.mark.parametrize("sampled_are", ["high", "low"])
def test_fp8_matrix_fused_call_repairs_rows_with_misleading_samples(misa, sampled_are):
    # As for bf16 queries: the keys at the sampled positions are made 64x larger (or smaller) than the
    # others through their per-token scale and all gates positive, so the sampled threshold is far too
    # high or far too low; the fused call must repair every row (its store-mode pass runs on query
    # tiles of 64 here, the filter pass on tiles of 32) and equal the two calls bit for bit.
    wl = WL.scaled(WL.WORKLOADS["c4"], L=40000, n_q=70, k=1024, k_cand=0, needles=0, q_dtype="e4m3")
    inp = WL.make_inputs(wl, seed=9)
    pos = np.array([16 * j + (((j * 2654435761) & 0xFFFFFFFF) >> 28) for j in range(wl.L // 16)])
    factor = np.full(wl.L, 1.0 if sampled_are == "high" else 64.0, dtype=np.float32)
    factor[pos] = 64.0 if sampled_are == "high" else 1.0
    inp["kscale"] = (inp["kscale"] * factor[None, :]).astype(np.float32)
    inp["W"] = np.abs(inp["W"]) + 0.01
    dv = misa.to_device(inp)
    p = replace(dv["problem"], q_dtype=misa.FP8_E4M3_MATRIX)
    rng = np.random.default_rng(3)
    heads = torch.from_numpy(np.stack([np.sort(rng.choice(wl.H, wl.h, replace=False)) for _ in range(wl.n_q)])
                             .reshape(1, wl.n_q, wl.h).astype(np.int32)).cuda()
    rows = (1, wl.n_q)
    S = torch.empty(rows + (wl.L,), dtype=torch.float32, device="cuda")
    ref_idx = torch.full(rows + (wl.k,), -9, dtype=torch.int32, device="cuda")
    ref_val = torch.full(rows + (wl.k,), 9.0, dtype=torch.float32, device="cuda")
    misa.score_tokens(p, dv["Q"], dv["W"], heads, dv["K"], dv["kscale"], S, misa.alloc_workspace(p, misa.OP_SCORE))
    misa.topk(p, S, wl.k, ref_idx, ref_val, misa.alloc_workspace(p, misa.OP_TOPK, wl.k))
    idx, val = torch.full_like(ref_idx, -9), torch.full_like(ref_val, 9.0)
    ws = misa.alloc_workspace(p, misa.OP_SELECT, wl.k)
    ws.fill_(0xA5)
    misa.select_tokens(p, dv["Q"], dv["W"], heads, dv["K"], dv["kscale"], wl.k, idx, val, ws)
    assert torch.equal(idx, ref_idx) and torch.equal(val, ref_val)
    assert int(misa.select_repaired_rows(p, True, wl.k, ws).sum()) == wl.n_q
    got, hs = idx.cpu().numpy(), heads.cpu().numpy()
    for t in (0, 63, 64, 69):
        K, q, w, n = oracle_view(inp, 0, t)
        check_index_set(got[0, t], O.score_tokens(q, w, hs[0, t], K, n), wl.k, f"repaired row {t}",
                        abs_frac=ABS_FRAC_FP8_MATRIX)
