"""GPU parity tests of misa_select_tokens (scoring and top-k in one call).

The call must write what misa_score_tokens followed by misa_topk writes
(Eq. misa_score then Eq. misa_topk; all heads: Eq. dsa_score then Eq. dsa_topk).
It is checked (a) against the fp64 oracle with the margin rule and (b) bit for
bit against the two-call GPU path, on inputs that take each of its internal
routes: the sampled-threshold route, rows short enough to keep every key, rows
whose threshold comes out too high or too low (repaired inside the call), and
problems it hands to the two-call path.
"""
import numpy as np
import pytest
import torch

from oracle import misa_oracle as O
from paper_2605_07363_amd import workloads as WL
from helpers import oracle_view, assert_scores_close, check_index_set

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def misa():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2605_07363_amd import misa as m
    return m


def small(base, **kw):
    return WL.scaled(WL.WORKLOADS[base], **kw)


CASES = {
    # name: (workload, routed?)
    "bf16_h8": (small("c2", L=6000, n_q=70, k=200), True),
    "fp8_h8": (small("c4", L=5003, n_q=45, k=300, k_cand=0, needles=16), True),
    "bf16_h16": (small("c2", L=4500, n_q=21, h=16, k=100), True),
    "fp8_dense64": (small("c4", L=4200, n_q=19, k=128, k_cand=0, needles=8), False),
    "bf16_bigk": (small("c2", L=20000, n_q=33, k=8192), True),
    "bf16_k1": (small("c2", L=4100, n_q=9, k=1), True),
    # few long rows: the two-call reference takes the split top-k path here
    "fp8_fewrows": (small("c4", L=40000, n_q=16, k=700, k_cand=0, needles=16), True),
    "fp8_h32": (small("c4", L=4800, n_q=11, h=32, k=150, k_cand=0, needles=8), True),
    "bf16_h3": (small("c2", L=4300, n_q=33, h=3, k=90), True),
    # handed to the two-call path: few queries, short cache, fp32, k above the list limit
    "bf16_decode": (small("c1", n_seq=3, L=5000, k=300), True),
    "bf16_shortL": (small("c2", L=3000, n_q=40, k=200), True),
    "f32_prefill": (WL.scaled(WL.WORKLOADS["c0"], L=5000, n_q=9, decode=False, k=64, needles=4), True),
    "bf16_k9000": (small("c2", L=12000, n_q=16, k=9000), True),
}


def two_call(misa, p, dv, heads, k):
    rows = (p.n_seq, p.n_q)
    S = torch.empty(rows + (p.L,), dtype=torch.float32, device="cuda")
    idx = torch.full(rows + (k,), -9, dtype=torch.int32, device="cuda")
    val = torch.full(rows + (k,), 9.0, dtype=torch.float32, device="cuda")
    misa.score_tokens(p, dv["Q"], dv["W"], heads, dv["K"], dv["kscale"], S)
    misa.topk(p, S, k, idx, val, misa.alloc_workspace(p, misa.OP_TOPK, k))
    return idx, val


def one_call(misa, p, dv, heads, k):
    rows = (p.n_seq, p.n_q)
    idx = torch.full(rows + (k,), -9, dtype=torch.int32, device="cuda")
    val = torch.full(rows + (k,), 9.0, dtype=torch.float32, device="cuda")
    ws = misa.alloc_workspace(p, misa.OP_SELECT, k)
    ws.fill_(0xA5)            # the call may not rely on the workspace contents
    misa.select_tokens(p, dv["Q"], dv["W"], heads, dv["K"], dv["kscale"], k, idx, val, ws)
    one_call.repaired = misa.select_repaired_rows(p, heads is not None, k, ws)
    return idx, val


def random_heads(wl, seed=11):
    rng = np.random.default_rng(seed)
    h = np.stack([np.sort(rng.choice(wl.H, wl.h, replace=False)) for _ in range(wl.n_seq * wl.n_q)])
    return torch.from_numpy(h.reshape(wl.n_seq, wl.n_q, wl.h).astype(np.int32)).cuda()


def check_against_oracle(inp, heads, idx, val, k, rows):
    wl = inp["wl"]
    heads_np = None if heads is None else heads.cpu().numpy()
    idx, val = idx.cpu().numpy(), val.cpu().numpy()
    for s, t in rows:
        K, q, w, n = oracle_view(inp, s, t)
        hs = np.arange(wl.H) if heads_np is None else heads_np[s, t]
        ref = O.score_tokens(q, w, hs, K, n)
        what = f"{wl.name} row {s},{t} (n={n})"
        check_index_set(idx[s, t], ref, k, what)
        ke = min(k, n)
        assert_scores_close(val[s, t, :ke], ref[idx[s, t, :ke]], "values " + what)
        assert np.all(np.isneginf(val[s, t, ke:]))


@pytest.mark.parametrize("name", list(CASES))
def test_select_matches_oracle_and_two_call_path(misa, name):
    wl, routed = CASES[name]
    inp = WL.make_inputs(wl, seed=77 + sum(map(ord, name)))
    dv = misa.to_device(inp)
    p = dv["problem"]
    heads = random_heads(wl) if routed else None
    idx, val = one_call(misa, p, dv, heads, wl.k)
    ref_idx, ref_val = two_call(misa, p, dv, heads, wl.k)
    torch.cuda.synchronize()
    assert torch.equal(idx, ref_idx), name
    assert torch.equal(val, ref_val), name
    two_call_route = name in ("bf16_decode", "bf16_shortL", "f32_prefill", "bf16_k9000")
    assert (one_call.repaired is None) == two_call_route
    if not two_call_route:
        assert int(one_call.repaired.sum()) == 0      # the sampled thresholds were good for every row
    rows = [(s, t) for s in range(wl.n_seq) for t in range(wl.n_q)]
    rng = np.random.default_rng(1)
    pick = sorted({0, len(rows) - 1} | set(rng.choice(len(rows), min(6, len(rows)), replace=False).tolist()))
    check_against_oracle(inp, heads, idx, val, wl.k, [rows[i] for i in pick])


@pytest.mark.parametrize("where", ["one_range", "range_edges", "every_other_range"])
def test_select_with_hits_concentrated_in_few_key_ranges(misa, where):
    # The candidate list of a row is cut into one segment per key range, sized from the sampled
    # scores of that range.  Here all gates are positive and the keys of a few stretches are eight
    # times larger than the rest, so nearly all scores above the threshold fall into one range,
    # into the first and last keys of every range, or into every other range; the segments must
    # adapt (no row may need the repair pass) and the result must equal the two calls bit for bit.
    wl = small("c2", L=32768, n_q=40, k=1024)
    inp = WL.make_inputs(wl, seed=21)
    K = O.bf16_bits_to_f64(inp["K"]).astype(np.float32)
    boost = np.ones(wl.L, dtype=np.float32)
    if where == "one_range":
        boost[9000:11500] = 8.0
    elif where == "range_edges":
        for start in range(0, wl.L, 2048):
            boost[start:start + 70] = 8.0
            boost[start + 2048 - 70:start + 2048] = 8.0
    else:
        for start in range(0, wl.L, 4096):
            boost[start:start + 2048] = 8.0
    inp["K"] = WL.f32_to_bf16_bits(K * boost[None, :, None])
    inp["W"] = np.abs(inp["W"]) + 0.01
    dv = misa.to_device(inp)
    p = dv["problem"]
    heads = random_heads(wl)
    idx, val = one_call(misa, p, dv, heads, wl.k)
    ref_idx, ref_val = two_call(misa, p, dv, heads, wl.k)
    assert torch.equal(idx, ref_idx)
    assert torch.equal(val, ref_val)
    assert int(one_call.repaired.sum()) == 0
    check_against_oracle(inp, heads, idx, val, wl.k, [(0, 0), (0, 39)])


def test_select_rows_of_every_length(misa):
    # Causal queries from the very first position on, and ragged sequences: rows with no visible key,
    # fewer than k, few enough to keep every key, and long ones, in the same call.
    wl = small("c2", n_seq=3, L=9000, n_q=48, k=512)
    inp = WL.make_inputs(wl, seed=5, seq_len=np.array([9000, 0, 4500], dtype=np.int32))
    inp["q_pos"] = np.array(sorted([0, 1, 5, 100, 511, 512, 513, 3000, 4499, 4500, 4501] +
                                   list(range(8963, 9000))), dtype=np.int32)
    assert inp["q_pos"].shape[0] == wl.n_q
    dv = misa.to_device(inp)
    p = dv["problem"]
    heads = random_heads(wl)
    idx, val = one_call(misa, p, dv, heads, wl.k)
    ref_idx, ref_val = two_call(misa, p, dv, heads, wl.k)
    assert torch.equal(idx, ref_idx)
    assert torch.equal(val, ref_val)
    assert int(one_call.repaired.sum()) == 0
    check_against_oracle(inp, heads, idx, val, wl.k, [(0, 0), (0, 3), (0, 5), (0, 47), (1, 20), (2, 9), (2, 30)])


def sampled_position(j):
    """Key that the sampling pass scores in group j of 16 consecutive keys (multiplicative hash, top 4 bits)."""
    return 16 * j + (((j * 2654435761) & 0xFFFFFFFF) >> 28)


@pytest.mark.parametrize("sampled_are", ["high", "low"])
def test_select_repairs_rows_with_misleading_samples(misa, sampled_are):
    # Keys at the sampled positions are made 64x larger (or smaller) than all others and all gates
    # positive, so the sampled threshold is far too high (fewer than k keys reach it) or far too
    # low (the candidate list overflows).  The call must notice and still return the exact top-k.
    wl = small("c2", L=40000, n_q=20, k=1024)
    inp = WL.make_inputs(wl, seed=9)
    K = O.bf16_bits_to_f64(inp["K"]).astype(np.float32)
    pos = np.array([sampled_position(j) for j in range(wl.L // 16)])
    scale = np.full(wl.L, 1.0 if sampled_are == "high" else 64.0, dtype=np.float32)
    scale[pos] = 64.0 if sampled_are == "high" else 1.0
    inp["K"] = WL.f32_to_bf16_bits(K * scale[None, :, None])
    inp["W"] = np.abs(inp["W"]) + 0.01
    dv = misa.to_device(inp)
    p = dv["problem"]
    heads = random_heads(wl)
    idx, val = one_call(misa, p, dv, heads, wl.k)
    ref_idx, ref_val = two_call(misa, p, dv, heads, wl.k)
    assert torch.equal(idx, ref_idx)
    assert torch.equal(val, ref_val)
    assert int(one_call.repaired.sum()) == wl.n_seq * wl.n_q     # every row took the repair pass
    check_against_oracle(inp, heads, idx, val, wl.k, [(0, 0), (0, 19)])


def test_select_longest_rows(misa):
    # the longest supported cache: bitmap and prefix arrays of the row kernel at their largest
    wl = small("c2", L=524288, n_q=8, k=1000, needles=8)
    inp = WL.make_inputs(wl, seed=8)
    dv = misa.to_device(inp)
    p = dv["problem"]
    heads = random_heads(wl)
    idx, val = one_call(misa, p, dv, heads, wl.k)
    ref_idx, ref_val = two_call(misa, p, dv, heads, wl.k)
    assert torch.equal(idx, ref_idx)
    assert torch.equal(val, ref_val)
    assert int(one_call.repaired.sum()) == 0
    check_against_oracle(inp, heads, idx, val, wl.k, [(0, 7)])


@pytest.mark.parametrize("name", ["c2", "c4"])
def test_select_full_size_workloads(misa, name):
    # The prefill workloads at their full size, as bench.py --fused runs them: every row of the
    # fused call equals the two-call path bit for bit and no row needed the repair pass; a few
    # rows are also checked against the oracle.
    wl = WL.WORKLOADS[name]
    k = wl.k_cand if wl.k_cand else wl.k
    inp = WL.make_inputs(wl)
    dv = misa.to_device(inp)
    p = dv["problem"]
    ix = misa.Indexer(p, k)
    ix.pool(dv["K"], dv["kscale"])
    ix.route(dv["Q"], dv["W"], dv["K"], dv["kscale"])
    idx, val = one_call(misa, p, dv, ix.heads, k)
    ref_idx, ref_val = two_call(misa, p, dv, ix.heads, k)
    assert torch.equal(idx, ref_idx)
    assert torch.equal(val, ref_val)
    assert int(one_call.repaired.sum()) == 0
    del ref_idx, ref_val
    check_against_oracle(inp, ix.heads, idx, val, k, [(0, 0), (0, wl.n_q // 2), (0, wl.n_q - 1)])


def test_select_ties_take_the_lower_index(misa):
    # Many identical keys: equal scores everywhere, so the choice is decided by the index rule alone.
    wl = small("c2", L=8192, n_q=16, k=700)
    inp = WL.make_inputs(wl, seed=3)
    inp["K"][:, 1000:7000] = inp["K"][:, 1000:1001]
    dv = misa.to_device(inp)
    p = dv["problem"]
    heads = random_heads(wl)
    idx, val = one_call(misa, p, dv, heads, wl.k)
    ref_idx, ref_val = two_call(misa, p, dv, heads, wl.k)
    assert torch.equal(idx, ref_idx)
    assert torch.equal(val, ref_val)
    check_against_oracle(inp, heads, idx, val, wl.k, [(0, 0), (0, 15)])


def test_select_is_repeatable_and_graph_safe(misa):
    wl = small("c4", L=16384, n_q=64, k=512, k_cand=0, needles=16)
    inp = WL.make_inputs(wl, seed=21)
    dv = misa.to_device(inp)
    p = dv["problem"]
    heads = random_heads(wl)
    ref_idx, _ = two_call(misa, p, dv, heads, wl.k)
    rows = (p.n_seq, p.n_q)
    idx = torch.empty(rows + (wl.k,), dtype=torch.int32, device="cuda")
    ws = misa.alloc_workspace(p, misa.OP_SELECT, wl.k)
    for _ in range(2):
        idx.fill_(-9)
        misa.select_tokens(p, dv["Q"], dv["W"], heads, dv["K"], dv["kscale"], wl.k, idx, None, ws)
        assert torch.equal(idx, ref_idx)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        misa.select_tokens(p, dv["Q"], dv["W"], heads, dv["K"], dv["kscale"], wl.k, idx, None, ws)
    for _ in range(3):
        idx.fill_(-9)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(idx, ref_idx)


def test_select_workspace_is_checked(misa):
    wl = small("c2", L=6000, n_q=16, k=100)
    dv = misa.to_device(WL.make_inputs(wl, seed=2))
    p = dv["problem"]
    idx = torch.empty((1, 16, 100), dtype=torch.int32, device="cuda")
    with pytest.raises(misa.MisaError):
        misa.select_tokens(p, dv["Q"], dv["W"], None, dv["K"], dv["kscale"], 100, idx, None, None)
    small_ws = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(misa.MisaError):
        misa.select_tokens(p, dv["Q"], dv["W"], None, dv["K"], dv["kscale"], 100, idx, None, small_ws)
