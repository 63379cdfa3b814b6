"""Re-rank of many queries with short candidate lists (Eq. misa_final_topk on Eq. dsa_score of
the candidates): the library takes the dense scores and their top-k in one kernel there.  Checked
against the oracle and, bit for bit, against the same rows re-ranked as sub-problems too small
for that kernel (dense scores through the workspace, then the row top-k)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import misa_oracle as O
from paper_2605_07363_amd import workloads as WL
from helpers import ABS_FRAC, ABS_FRAC_FP8_MATRIX, assert_scores_close, check_index_set, oracle_view

pytestmark = pytest.mark.gpu

@pytest.fixture(scope="module")
def misa():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2605_07363_amd import misa as m
    return m


ROWS = 1100          # above the library's threshold for the one-kernel path (1024 rows)


def _problem(seed, k_dtype, q_dtype, H, L):
    wl = WL.scaled(WL.WORKLOADS["c2"], n_seq=1, L=L, n_q=ROWS, H=H, h=1, B=64, k=1, k_cand=0,
                   k_dtype=k_dtype, q_dtype=q_dtype, needles=6, name=f"rrf{seed}")
    return wl, WL.make_inputs(wl, seed=seed)


def _candidates(rng, rows, L, kc, full=False):
    cand = np.full((1, rows, kc), -1, dtype=np.int32)
    for t in range(rows):
        m = kc if full else int(rng.integers(0, kc + 1))
        c = np.sort(rng.choice(L, size=min(m, L), replace=False)).astype(np.int32)
        if not full:
            c[rng.random(c.shape[0]) < 0.03] = -1                 # holes
        cand[0, t, :c.shape[0]] = c
    return cand


def _rerank(misa, p, dv, cand, kc, k, Q=None):
    rows = p.n_q
    idx = torch.full((1, rows, k), -9, dtype=torch.int32, device="cuda")
    val = torch.full((1, rows, k), 7.0, dtype=torch.float32, device="cuda")
    misa.rerank(p, dv["Q"] if Q is None else Q, dv["W"], dv["K"], dv["kscale"], cand, kc, k, idx, val,
                misa.alloc_workspace(p, misa.OP_RERANK, kc))
    torch.cuda.synchronize()
    return idx, val


def _rerank_in_pieces(misa, p, dv, cand, kc, k, piece=500):
    """The same rows as sub-problems of `piece` queries: below the one-kernel threshold."""
    idx, val = [], []
    for a in range(0, p.n_q, piece):
        b = min(a + piece, p.n_q)
        pp = replace(p, n_q=b - a, q_pos=p.q_pos[a:b].contiguous())
        part = dict(dv, Q=dv["Q"][:, a:b].contiguous(), W=dv["W"][:, a:b].contiguous())
        i, v = _rerank(misa, pp, part, cand[:, a:b].contiguous(), kc, k)
        idx.append(i); val.append(v)
    return torch.cat(idx, dim=1), torch.cat(val, dim=1)


def _check_rows_against_oracle(inp, cand, idx, val, k, rows, what, abs_frac=ABS_FRAC):
    for t in rows:
        K, q, w, n = oracle_view(inp, 0, t)
        dense = O.dsa_scores(q, w, K, n) if n else np.zeros(0)
        valid = np.array(sorted(c for c in cand[0, t] if 0 <= c < n), dtype=np.int64)
        ke = min(k, valid.shape[0])
        got = idx[0, t]
        assert np.all(got[ke:] == -1) and np.all(np.diff(got[:ke]) > 0), f"{what} row {t}"
        assert set(got[:ke].tolist()) <= set(valid.tolist()), f"{what} row {t}"
        pos = np.searchsorted(valid, got[:ke])
        padded = np.concatenate([pos, np.full(k - ke, -1, dtype=pos.dtype)])
        check_index_set(padded, dense[valid], k, f"{what} row {t}", abs_frac=abs_frac)
        assert_scores_close(val[0, t, :ke], dense[got[:ke]], f"{what} values row {t}", abs_frac=abs_frac)
        assert np.all(np.isneginf(val[0, t, ke:]))


@pytest.mark.parametrize("k_dtype,q_dtype,H,kc,k", [
    ("bf16", "bf16", 64, 700, 100),      # list length not a multiple of the 128-candidate step
    ("e4m3", "bf16", 64, 1024, 1024),    # k = k': everything that is valid is kept
    ("e4m3", "bf16", 17, 333, 50),       # one row tile, odd head count
    ("bf16", "bf16", 32, 2500, 640),
])
def test_many_query_rerank_against_the_oracle(misa, k_dtype, q_dtype, H, kc, k):
    seed = 9900 + kc
    rng = np.random.default_rng(seed)
    L = 3000
    wl, inp = _problem(seed, k_dtype, q_dtype, H, L)
    dv = misa.to_device(inp)
    p = dv["problem"]
    cand = _candidates(rng, ROWS, L, kc)
    cand[0, 5, kc // 2] = L + 7                           # beyond the cache: skipped
    dcand = torch.from_numpy(cand).cuda()
    idx, val = _rerank(misa, p, dv, dcand, kc, k)
    sample = [0, 1, 5, ROWS - 1] + rng.choice(ROWS, size=36, replace=False).tolist()
    _check_rows_against_oracle(inp, cand, idx.cpu().numpy(), val.cpu().numpy(), k, sample, f"fused rerank {k_dtype}")
    # all rows, bit for bit, against the path that keeps the dense scores
    idx2, val2 = _rerank_in_pieces(misa, p, dv, dcand, kc, k)
    assert torch.equal(idx, idx2)
    assert torch.equal(val, val2)


def test_many_query_rerank_on_the_fp8_matrix_instruction(misa):
    if not misa.HAS_FP8_MFMA:
        pytest.skip("library built without the fp8 matrix path")
    seed, L, kc, k = 9931, 3000, 900, 128
    rng = np.random.default_rng(seed)
    wl, inp = _problem(seed, "e4m3", "e4m3", 64, L)
    dv = misa.to_device(inp)
    p = replace(dv["problem"], q_dtype=misa.FP8_E4M3_MATRIX)
    cand = _candidates(rng, ROWS, L, kc)
    dcand = torch.from_numpy(cand).cuda()
    idx, val = _rerank(misa, p, dv, dcand, kc, k)
    sample = [0, ROWS - 1] + rng.choice(ROWS, size=30, replace=False).tolist()
    _check_rows_against_oracle(inp, cand, idx.cpu().numpy(), val.cpu().numpy(), k, sample, "fused rerank fp8 x fp8",
                               abs_frac=ABS_FRAC_FP8_MATRIX)
    idx2, val2 = _rerank_in_pieces(misa, p, dv, dcand, kc, k)
    assert torch.equal(idx, idx2)
    assert torch.equal(val, val2)


def _times_power_of_two(bits, e):
    """bf16 bit patterns of normal numbers multiplied by 2^e."""
    return (bits.astype(np.int32) + (e << 7)).astype(bits.dtype)


@pytest.mark.parametrize("shape", ["constant", "three_values", "outliers", "tiny_and_huge", "mostly_invalid"])
def test_many_query_rerank_degenerate_score_rows(misa, shape):
    """Rows whose dense scores tie massively, span many binades or are mostly -inf: the selection
    inside the kernel must stay exact (ties to the lower position) on every route it can take."""
    seed, L, kc, k = 9950, 4000, 3000, 700
    rng = np.random.default_rng(seed)
    wl, inp = _problem(seed, "bf16", "bf16", 64, L)
    K = inp["K"]                                           # [1, L, d] bf16 bit patterns
    if shape == "constant":
        K[0, :] = K[0, 17]                                 # every key the same row: all scores of a query equal
    elif shape == "three_values":
        K[0, :] = K[0, rng.integers(0, 3, L)]              # three distinct keys: ~1000 equal scores each
    elif shape == "outliers":
        big = rng.choice(L, size=40, replace=False)
        K[0, big] = _times_power_of_two(K[0, big], 12)     # forty keys 4096 times larger
    elif shape == "tiny_and_huge":
        e = rng.integers(-30, 31, L)                       # keys spread over sixty binades
        K[0] = np.stack([_times_power_of_two(K[0, i], int(e[i])) for i in range(L)])
    dv = misa.to_device(inp)
    p = dv["problem"]
    cand = _candidates(rng, ROWS, L, kc, full=(shape != "mostly_invalid"))
    if shape == "mostly_invalid":
        cand[:, :, 200:] = -1                              # fewer valid candidates than k
        cand[0, 3, :] = -1                                 # none at all
    dcand = torch.from_numpy(cand).cuda()
    idx, val = _rerank(misa, p, dv, dcand, kc, k)
    idx2, val2 = _rerank_in_pieces(misa, p, dv, dcand, kc, k)
    assert torch.equal(idx, idx2)
    assert torch.equal(val, val2)
    sample = [0, 3, ROWS - 1] + rng.choice(ROWS, size=9, replace=False).tolist()
    _check_rows_against_oracle(inp, cand, idx.cpu().numpy(), val.cpu().numpy(), k, sample, f"fused rerank {shape}")


def test_longest_list_the_kernel_takes(misa):
    # k' = 8192 (the limit of the one-kernel path) and k' = 8193 (the first length beyond it) agree
    # with the oracle on sampled rows
    seed, L = 9970, 12000
    rng = np.random.default_rng(seed)
    wl, inp = _problem(seed, "e4m3", "bf16", 64, L)
    dv = misa.to_device(inp)
    p = dv["problem"]
    for kc, k in ((8192, 2048), (8193, 2048)):
        cand = _candidates(rng, ROWS, L, kc, full=True)
        idx, val = _rerank(misa, p, dv, torch.from_numpy(cand).cuda(), kc, k)
        sample = [0, ROWS - 1] + rng.choice(ROWS, size=6, replace=False).tolist()
        _check_rows_against_oracle(inp, cand, idx.cpu().numpy(), val.cpu().numpy(), k, sample, f"rerank k'={kc}")


@pytest.mark.parametrize("paged", [False, True])
def test_many_query_rerank_over_several_ragged_sequences(misa, paged):
    # 3 sequences x 400 queries (1200 rows: the one-kernel path), ragged lengths, optionally a page
    # pool; every sequence alone (400 rows: dense scores + row top-k) must give the same bits
    seed, L, kc, k, n_seq, n_q = 9990, 2500, 1500, 300, 3, 400
    rng = np.random.default_rng(seed)
    wl = WL.scaled(WL.WORKLOADS["c2"], n_seq=n_seq, L=L, n_q=n_q, H=64, h=1, B=64, k=1, k_cand=0,
                   k_dtype="e4m3", q_dtype="bf16", needles=6, name="rrf_multi")
    inp = WL.make_inputs(wl, seed=seed, seq_len=np.array([L, 1700, 900], dtype=np.int32))
    dv = misa.to_device(inp)
    if paged:
        dv = misa.paginate(dv, 64, seed=seed)
    p = dv["problem"]
    cand = np.concatenate([_candidates(rng, n_q, L, kc) for _ in range(n_seq)], axis=0)
    dcand = torch.from_numpy(cand).cuda()
    idx = torch.full((n_seq, n_q, k), -9, dtype=torch.int32, device="cuda")
    val = torch.full((n_seq, n_q, k), 7.0, dtype=torch.float32, device="cuda")
    misa.rerank(p, dv["Q"], dv["W"], dv["K"], dv["kscale"], dcand, kc, k, idx, val,
                misa.alloc_workspace(p, misa.OP_RERANK, kc))
    torch.cuda.synchronize()
    for s in range(n_seq):
        ps = replace(p, n_seq=1, seq_len=p.seq_len[s:s + 1].contiguous(),
                     page_table=None if p.page_table is None else p.page_table[s:s + 1].contiguous())
        Ks, kss = (dv["K"], dv["kscale"]) if paged else (dv["K"][s:s + 1], dv["kscale"][s:s + 1])
        i1 = torch.empty((1, n_q, k), dtype=torch.int32, device="cuda")
        v1 = torch.empty((1, n_q, k), dtype=torch.float32, device="cuda")
        misa.rerank(ps, dv["Q"][s:s + 1], dv["W"][s:s + 1], Ks, kss, dcand[s:s + 1], kc, k, i1, v1,
                    misa.alloc_workspace(ps, misa.OP_RERANK, kc))
        torch.cuda.synchronize()
        assert torch.equal(idx[s:s + 1], i1), f"sequence {s}"
        assert torch.equal(val[s:s + 1], v1), f"sequence {s}"
    ih, vh = idx.cpu().numpy(), val.cpu().numpy()
    for s in range(n_seq):
        for t in [0, n_q - 1] + rng.choice(n_q, size=4, replace=False).tolist():
            K, q, w, n = oracle_view(inp, s, t)
            dense = O.dsa_scores(q, w, K, n) if n else np.zeros(0)
            valid = np.array(sorted(c for c in cand[s, t] if 0 <= c < n), dtype=np.int64)
            ke = min(k, valid.shape[0])
            got = ih[s, t]
            assert np.all(got[ke:] == -1) and np.all(np.diff(got[:ke]) > 0)
            pos = np.searchsorted(valid, got[:ke])
            check_index_set(np.concatenate([pos, np.full(k - ke, -1, dtype=pos.dtype)]), dense[valid], k, f"multi {s},{t}")
            assert_scores_close(vh[s, t, :ke], dense[got[:ke]], f"multi values {s},{t}")


def test_many_query_rerank_writes_only_its_outputs(misa):
    # idx / val are windows of larger buffers filled with a sentinel: nothing outside them changes,
    # and the candidate list (which the kernel overwrites in LDS, not in memory) stays as it was
    seed, L, kc, k = 9995, 2000, 777, 129
    rng = np.random.default_rng(seed)
    wl, inp = _problem(seed, "e4m3", "bf16", 64, L)
    dv = misa.to_device(inp)
    p = dv["problem"]
    cand = torch.from_numpy(_candidates(rng, ROWS, L, kc)).cuda()
    before = cand.clone()
    pad = 4096
    ibuf = torch.full((pad + ROWS * k + pad,), -77, dtype=torch.int32, device="cuda")
    vbuf = torch.full((pad + ROWS * k + pad,), 3.25, dtype=torch.float32, device="cuda")
    idx = ibuf[pad:pad + ROWS * k].view(1, ROWS, k)
    val = vbuf[pad:pad + ROWS * k].view(1, ROWS, k)
    misa.rerank(p, dv["Q"], dv["W"], dv["K"], dv["kscale"], cand, kc, k, idx, val,
                misa.alloc_workspace(p, misa.OP_RERANK, kc))
    torch.cuda.synchronize()
    assert torch.all(ibuf[:pad] == -77) and torch.all(ibuf[pad + ROWS * k:] == -77)
    assert torch.all(vbuf[:pad] == 3.25) and torch.all(vbuf[pad + ROWS * k:] == 3.25)
    assert torch.equal(cand, before)
    assert torch.all(idx >= -1) and torch.all(idx < L)
