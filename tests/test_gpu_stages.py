"""GPU parity of each C-ABI call in isolation: every stage is fed
oracle-produced inputs and compared with the oracle element by element."""
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


def small(name, **kw):
    return WL.scaled(WL.WORKLOADS[name], **kw)


CASES = {
    # spans several tiles and a ragged tail; every dtype combination
    "f32_decode": small("c0", L=1500, B=64),
    "bf16_decode": small("c1", n_seq=3, L=5000, B=64, k=300),
    "fp8_decode": small("c3", n_seq=2, L=4133, B=128, k=300, needles=16),
    "bf16_prefill": small("c2", L=3000, n_q=70, B=64, k=200),
    "fp8_prefill": small("c4", L=2500, n_q=40, B=64, k=128, k_cand=512, needles=16),
    "f32_prefill": WL.scaled(WL.WORKLOADS["c0"], L=700, n_q=9, decode=False, B=50, k=64, needles=4),
    "bf16_bigB": small("c1", n_seq=2, L=3000, B=5000, k=100),
    "bf16_B1": small("c1", n_seq=1, L=300, B=1, k=50, needles=4),
    # block sizes of the paper's own sweep (B = 1024 ... one block for the whole prefix): the
    # pooling kernel cuts such blocks into slices
    "fp8_B1024": small("c3", n_seq=2, L=7000, B=1024, k=200, needles=8),
    "bf16_B4096": small("c1", n_seq=3, L=9500, B=4096, k=200, needles=8),
    "fp8_Bwhole": small("c3", n_seq=2, L=6000, B=6000, k=100, needles=8),
    "glm_dense_h": small("c3", n_seq=1, L=2000, h=32, B=128, k=100, needles=8),
    # other head-slot widths of the prefill kernel (h = 16, 32, 3) and tiny head counts
    "bf16_prefill_h16": small("c2", L=1500, n_q=21, h=16, B=64, k=100),
    "fp8_prefill_h32": small("c4", L=1100, n_q=13, h=32, B=32, k=64, k_cand=256, needles=8),
    "bf16_prefill_h3": small("c2", L=900, n_q=33, h=3, B=16, k=50),
    "bf16_decode_H1": WL.scaled(WL.WORKLOADS["c1"], n_seq=2, L=700, H=1, h=1, B=8, k=20, needles=2),
    # decode batches of eight sequences and more: routing runs as one workgroup per sequence
    # (fewer pooled-block tiles than wavefronts / several tiles per wavefront / a single head)
    "bf16_decode_batch": small("c1", n_seq=9, L=2600, B=16, k=100, needles=8),
    "fp8_decode_batch": small("c3", n_seq=8, L=9000, B=8, k=100, needles=8),
    "bf16_decode_batch_H1": WL.scaled(WL.WORKLOADS["c1"], n_seq=8, L=500, H=1, h=1, B=4, k=20, needles=2),
}


def gen(name, seq_len=None):
    return WL.make_inputs(CASES[name], seed=1234 + sum(map(ord, name)), seq_len=seq_len)


def ragged(wl):
    rng = np.random.default_rng(5)
    lens = rng.integers(1, wl.L + 1, wl.n_seq)
    lens[0] = wl.L
    return lens.astype(np.int32)


# --------------------------------------------------------------------- pool
@pytest.mark.parametrize("name", ["f32_decode", "bf16_decode", "fp8_decode", "bf16_bigB", "bf16_B1",
                                  "fp8_B1024", "bf16_B4096", "fp8_Bwhole"])
@pytest.mark.parametrize("use_len", [False, True])
def test_pool_keys(misa, name, use_len):
    wl = CASES[name]
    inp = gen(name, ragged(wl) if use_len else None)
    dv = misa.to_device(inp)
    p = dv["problem"]
    Kp = torch.full((wl.n_seq, p.M, wl.d), 7.0, dtype=torch.float32, device="cuda")
    misa.pool_keys(p, dv["K"], dv["kscale"], Kp, misa.alloc_workspace(p, misa.OP_POOL))
    got = Kp.cpu().numpy()
    for s in range(wl.n_seq):
        K, _, _, n = oracle_view(inp, s, 0)
        ref = O.pool_keys(K, wl.B, n)
        assert_scores_close(got[s, :ref.shape[0]], ref, f"pool {name} seq {s}")
        assert not got[s, ref.shape[0]:].any()          # blocks past the sequence end are zero


@pytest.mark.parametrize("name", ["bf16_decode", "fp8_decode", "bf16_B4096"])
def test_pool_keys_update_after_append(misa, name):
    # Pooled keys maintained incrementally: pool at the old lengths, append tokens, update from the
    # old lengths on -> identical to pooling everything at the new lengths; earlier blocks untouched.
    wl = CASES[name]
    rng = np.random.default_rng(17)
    new_len = ragged(wl)
    grow = rng.integers(0, 3 * wl.B + 2, wl.n_seq)
    grow[0] = 1                                         # one decoded token
    old_len = np.maximum(new_len - grow, 0).astype(np.int32)
    inp = gen(name, new_len)
    dv = misa.to_device(inp)
    p_new = dv["problem"]
    ws = misa.alloc_workspace(p_new, misa.OP_POOL)
    full = torch.full((wl.n_seq, p_new.M, wl.d), 7.0, dtype=torch.float32, device="cuda")
    misa.pool_keys(p_new, dv["K"], dv["kscale"], full, ws)
    from dataclasses import replace
    old_dev = torch.from_numpy(old_len).cuda()
    p_old = replace(p_new, seq_len=old_dev)
    Kp = torch.full_like(full, 7.0)
    misa.pool_keys(p_old, dv["K"], dv["kscale"], Kp, ws)
    stale = Kp.clone()
    misa.pool_keys_update(p_new, dv["K"], dv["kscale"], Kp, old_dev, 5, ws)
    assert torch.equal(Kp, full)
    got = Kp.cpu().numpy()
    for s in range(wl.n_seq):                           # the updated pooled keys are the block means of Eq. pool
        K, _, _, n = oracle_view(inp, s, 0)
        ref = O.pool_keys(K, wl.B, n)
        assert_scores_close(got[s, :ref.shape[0]], ref, f"updated pool {name} seq {s}")
        assert not got[s, ref.shape[0]:].any()
    for s in range(wl.n_seq):                           # blocks before the first changed one were not written
        first = int(old_len[s]) // wl.B
        assert torch.equal(Kp[s, :first], stale[s, :first])
    # a bound of one block updates only the block of from_token
    Kp1 = stale.clone()
    misa.pool_keys_update(p_new, dv["K"], dv["kscale"], Kp1, old_dev, 1, ws)
    for s in range(wl.n_seq):
        first = int(old_len[s]) // wl.B
        if first * wl.B < int(new_len[s]):
            assert torch.equal(Kp1[s, first], full[s, first])
        assert torch.equal(Kp1[s, first + 1:], stale[s, first + 1:])


def test_pool_B1_decodes_all_fp8_codes(misa):
    # With B = 1 pooling returns the de-quantised keys themselves, so this
    # checks the hardware fp8 decode against the oracle's table for every code.
    codes = np.arange(256, dtype=np.uint8)
    codes[[0x7F, 0xFF]] = 0                               # NaN codes are not valid inputs
    K = np.tile(codes.reshape(2, 128), (1, 1))[None]      # [1, 2, 128]
    scale = np.array([[1.0, 0.37]], dtype=np.float32)
    p = misa.Problem(1, 2, 1, 8, 1, 1, misa.FP8_E4M3, misa.BF16)
    Kp = torch.empty((1, 2, 128), dtype=torch.float32, device="cuda")
    misa.pool_keys(p, torch.from_numpy(K).cuda(), torch.from_numpy(scale).cuda(), Kp)
    ref = O.dequantise(K[0], "e4m3", scale[0])
    np.testing.assert_allclose(Kp.cpu().numpy()[0], ref, rtol=1e-6, atol=0)


# --------------------------------------------------------------------- route
@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("use_len", [False, True])
def test_route_heads(misa, name, use_len):
    wl = CASES[name]
    inp = gen(name, ragged(wl) if use_len else None)
    dv = misa.to_device(inp)
    p = dv["problem"]
    # pooled keys from the oracle (whole-cache pooling, fp32 storage)
    Kp = np.zeros((wl.n_seq, p.M, wl.d), dtype=np.float32)
    for s in range(wl.n_seq):
        K, _, _, _ = oracle_view(inp, s, 0)
        length = wl.L if inp["seq_len"] is None else int(inp["seq_len"][s])
        ref = O.pool_keys(K, wl.B, length)
        Kp[s, :ref.shape[0]] = ref
    heads = torch.full((wl.n_seq, wl.n_q, wl.h), -5, dtype=torch.int32, device="cuda")
    E = torch.empty((wl.n_seq, wl.n_q, wl.H), dtype=torch.float32, device="cuda")
    ws = misa.alloc_workspace(p, misa.OP_ROUTE)
    misa.route_heads(p, dv["Q"], dv["W"], torch.from_numpy(Kp).cuda(), dv["K"], dv["kscale"], heads, E, ws)
    heads, E = heads.cpu().numpy(), E.cpu().numpy()
    exact = 0
    for s in range(wl.n_seq):
        for t in range(wl.n_q):
            K, q, w, n = oracle_view(inp, s, t)
            ref_heads, ref_E = O.route_heads(q, w, K, wl.B, wl.h, n)
            assert_scores_close(E[s, t], ref_E, f"E {name} {s},{t}")
            exact += check_index_set(heads[s, t], ref_E, wl.h, f"heads {name} {s},{t}")
    assert exact >= 0.9 * wl.n_seq * wl.n_q          # legal flips inside the margin must be rare


@pytest.mark.parametrize("name", ["f32_decode", "bf16_decode", "bf16_prefill", "fp8_prefill_h32", "bf16_decode_H1"])
@pytest.mark.parametrize("kind", ["gate", "qnorm"])
def test_route_heads_proxy(misa, name, kind):
    # content-free router scores of the routing-score ablation
    wl = CASES[name]
    inp = gen(name)
    dv = misa.to_device(inp)
    p = dv["problem"]
    heads = torch.full((wl.n_seq, wl.n_q, wl.h), -5, dtype=torch.int32, device="cuda")
    E = torch.empty((wl.n_seq, wl.n_q, wl.H), dtype=torch.float32, device="cuda")
    code = misa.ROUTER_GATE if kind == "gate" else misa.ROUTER_QUERY_NORM
    misa.route_heads_proxy(p, dv["Q"], dv["W"], code, heads, E)
    heads, E = heads.cpu().numpy(), E.cpu().numpy()
    for s in range(wl.n_seq):
        for t in range(wl.n_q):
            _, q, w, _ = oracle_view(inp, s, t)
            ref_heads, ref_E = O.route_heads_proxy(q, w, wl.h, kind)
            assert_scores_close(E[s, t], ref_E, f"proxy E {name} {kind} {s},{t}")
            check_index_set(heads[s, t], ref_E, wl.h, f"proxy heads {name} {kind} {s},{t}")
            if kind == "gate":                      # the gate is copied, so the set is exact
                np.testing.assert_array_equal(heads[s, t], ref_heads)


# --------------------------------------------------------------------- score
@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("use_len", [False, True])
def test_score_tokens(misa, name, use_len):
    wl = CASES[name]
    inp = gen(name, ragged(wl) if use_len else None)
    dv = misa.to_device(inp)
    p = dv["problem"]
    ref_heads = np.zeros((wl.n_seq, wl.n_q, wl.h), dtype=np.int32)
    views = {}
    for s in range(wl.n_seq):
        for t in range(wl.n_q):
            K, q, w, n = views[(s, t)] = oracle_view(inp, s, t)
            ref_heads[s, t] = O.route_heads(q, w, K, wl.B, wl.h, n)[0]
    S = torch.full((wl.n_seq, wl.n_q, wl.L), 3.0, dtype=torch.float32, device="cuda")
    misa.score_tokens(p, dv["Q"], dv["W"], torch.from_numpy(ref_heads).cuda(), dv["K"], dv["kscale"], S)
    got = S.cpu().numpy()
    Sd = torch.empty_like(S)
    misa.score_tokens(p, dv["Q"], dv["W"], None, dv["K"], dv["kscale"], Sd)      # all heads = dense DSA
    got_dense = Sd.cpu().numpy()
    for (s, t), (K, q, w, n) in views.items():
        assert_scores_close(got[s, t, :n], O.score_tokens(q, w, ref_heads[s, t], K, n), f"score {name} {s},{t}")
        assert np.all(np.isneginf(got[s, t, n:])), "invisible keys must score -inf"
        assert_scores_close(got_dense[s, t, :n], O.dsa_scores(q, w, K, n), f"dense {name} {s},{t}")
        assert np.all(np.isneginf(got_dense[s, t, n:]))


def test_score_with_all_heads_listed_equals_dense(misa):
    wl = CASES["bf16_decode"]
    inp = gen("bf16_decode")
    dv = misa.to_device(inp)
    p = misa.Problem(wl.n_seq, wl.L, wl.n_q, wl.H, wl.B, wl.H, misa.BF16, misa.BF16)     # h = H
    allh = torch.arange(wl.H, dtype=torch.int32, device="cuda").repeat(wl.n_seq, wl.n_q, 1).contiguous()
    a = torch.empty((wl.n_seq, wl.n_q, wl.L), dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    misa.score_tokens(p, dv["Q"], dv["W"], allh, dv["K"], dv["kscale"], a)
    misa.score_tokens(p, dv["Q"], dv["W"], None, dv["K"], dv["kscale"], b)
    assert torch.equal(a, b)


# --------------------------------------------------------------------- top-k
def _topk_case(misa, S, k, q_pos=None, seq_len=None):
    n_seq, n_q, L = S.shape
    p = misa.Problem(n_seq, L, n_q, 8, 16, 2, misa.F32, misa.F32,
                     None if q_pos is None else torch.from_numpy(q_pos).cuda(),
                     None if seq_len is None else torch.from_numpy(seq_len).cuda())
    idx = torch.full((n_seq, n_q, k), -7, dtype=torch.int32, device="cuda")
    val = torch.full((n_seq, n_q, k), 9.0, dtype=torch.float32, device="cuda")
    misa.topk(p, torch.from_numpy(S).cuda(), k, idx, val, misa.alloc_workspace(p, misa.OP_TOPK, k))
    idx, val = idx.cpu().numpy(), val.cpu().numpy()
    for s in range(n_seq):
        length = L if seq_len is None else int(np.clip(seq_len[s], 0, L))
        for t in range(n_q):
            n = length if q_pos is None else int(np.clip(int(q_pos[t]) + 1, 0, length))
            ref = O.topk(S[s, t, :n].astype(np.float64), k) if n else np.zeros(0, np.int64)
            ke = ref.shape[0]
            np.testing.assert_array_equal(idx[s, t, :ke], ref, err_msg=f"row {s},{t}")
            assert np.all(idx[s, t, ke:] == -1)
            np.testing.assert_array_equal(val[s, t, :ke], S[s, t, ref])
            assert np.all(np.isneginf(val[s, t, ke:]))


def test_topk_random_rows_bit_exact(misa):
    rng = np.random.default_rng(21)
    S = rng.standard_normal((3, 1, 10007)).astype(np.float32)
    for k in (1, 17, 2048, 10006, 10007, 12000):
        _topk_case(misa, S, k)


def test_topk_ties_zeros_and_constants(misa):
    rng = np.random.default_rng(22)
    S = (np.round(rng.standard_normal((2, 2, 5000)) * 3) / 3).astype(np.float32)     # heavy ties
    S[0, 0, ::7] = 0.0; S[0, 0, 3::7] = -0.0                                        # signed zeros tie
    S[1, 1, :] = 1.25                                                                # constant row
    q_pos = np.array([4999, 2500], dtype=np.int32)
    for k in (5, 256, 2048, 4999):
        _topk_case(misa, S, k, q_pos=q_pos)


def test_topk_short_and_empty_prefixes(misa):
    rng = np.random.default_rng(23)
    S = rng.standard_normal((4, 3, 300)).astype(np.float32)
    q_pos = np.array([0, 5, 299], dtype=np.int32)
    seq_len = np.array([300, 0, 4, 150], dtype=np.int32)
    _topk_case(misa, S, 64, q_pos=q_pos, seq_len=seq_len)


def test_topk_negative_and_extreme_values(misa):
    rng = np.random.default_rng(24)
    S = (rng.standard_normal((1, 2, 4096)) * 1e3).astype(np.float32)
    S[0, 0, :100] = -np.inf
    S[0, 1, 5] = 3e38; S[0, 1, 6] = -3e38; S[0, 1, 7] = 1e-44       # denormal
    q_pos = np.array([4095, 4095], dtype=np.int32)
    for k in (10, 4000, 4096):
        _topk_case(misa, S, k, q_pos=q_pos)


def test_topk_long_rows_split_over_workgroups(misa):
    # few long rows take the multi-workgroup path (sampled prefilter + exact finish)
    rng = np.random.default_rng(25)
    S = rng.standard_normal((2, 2, 40000)).astype(np.float32)
    q_pos = np.array([39999, 33333], dtype=np.int32)
    for k in (1, 300, 2048, 8192, 16384):
        _topk_case(misa, S, k, q_pos=q_pos)
    _topk_case(misa, S, 2048, q_pos=q_pos, seq_len=np.array([40000, 35000], dtype=np.int32))
    # decode rows whose visible prefix is not longer than k: everything is selected
    _topk_case(misa, np.ascontiguousarray(S[:, :1]), 16384, seq_len=np.array([10000, 16385], dtype=np.int32))


def test_topk_prefilter_hand_over_cases(misa):
    # Few long rows: several workgroups per row pass on the elements above a threshold taken
    # from a sample of the row (one 16-element line out of every `ls`, chosen by a hash).  Rows
    # built so that the hand-over is unusable must come out exact all the same.
    rng = np.random.default_rng(29)
    n_seq, L = 7, 65536
    S = rng.standard_normal((n_seq, 1, L)).astype(np.float32)
    S[1, 0] = np.sort(S[1, 0])                                  # every selected element in the last range
    lines = L // 16
    ls = -(-lines // 256)
    g = np.arange(lines // ls, dtype=np.uint64)
    sampled = (g * ls + (((g * 2654435761) & 0xFFFFFFFF) >> 16) % ls).astype(np.int64)
    hot = np.zeros(lines, dtype=bool); hot[sampled] = True
    row = -np.abs(S[2, 0]).reshape(lines, 16)                   # large values only where the sample looks:
    row[hot] = 5.0 + rng.random((hot.sum(), 16))                # the threshold comes out too high
    S[2, 0] = row.reshape(-1)
    row = -np.abs(S[3, 0]).reshape(lines, 16)                   # ... and only where it does not look:
    cold = np.flatnonzero(~hot)[:200]                           # more elements pass than the sample suggests
    row[cold] = 5.0 + rng.random((cold.size, 16))
    S[3, 0] = row.reshape(-1)
    S[4, 0] = 0.5                                               # constant: everything passes
    seq_len = np.array([L, L, L, L, L, 5000, 2048], dtype=np.int32)   # one short range; prefix == k
    for k in (100, 2048, 6000):
        _topk_case(misa, S, k, seq_len=seq_len)
    # the same row lengths with causal positions instead of sequence lengths
    S2 = np.ascontiguousarray(S[:1].repeat(3, axis=1))
    _topk_case(misa, S2, 2048, q_pos=np.array([L - 1, 40000, 8191], dtype=np.int32))


@pytest.mark.parametrize("shape", [(2, 1, 40000), (3, 300, 3000)])
def test_topk_tie_paths(misa, shape):
    rng = np.random.default_rng(26)
    q_pos = None if shape[1] == 1 else np.full(shape[1], shape[2] - 1, dtype=np.int32)
    # (a) few distinct values: the threshold value has far more copies than places (index digits decide)
    S = rng.integers(0, 50, shape).astype(np.float32)
    for k in (7, 1000, 2048):
        _topk_case(misa, S, k, q_pos=q_pos)
    # (b) constant rows and rows with one huge bin: more boundary elements than the list holds
    S = np.full(shape, 0.75, dtype=np.float32)
    S[0, 0, ::3] = 0.7500001
    S[-1, -1, :] = 2.0
    for k in (5, 2048):
        _topk_case(misa, S, k, q_pos=q_pos)
    # (c) values inside one binade only differing in low mantissa bits
    S = (1.0 + rng.integers(0, 1 << 12, shape) * 2.0 ** -23).astype(np.float32)
    _topk_case(misa, S, 1500, q_pos=q_pos)


def test_topk_sampled_single_read_path(misa):
    # many long rows (one workgroup per row); rows with sorted, repeated, constant, clustered
    # and -inf values
    rng = np.random.default_rng(28)
    rows, L = 264, 40000
    S = rng.standard_normal((1, rows, L)).astype(np.float32)
    S[0, 1] = np.sort(S[0, 1])                                  # ascending
    S[0, 2] = np.sort(S[0, 2])[::-1]                            # descending
    S[0, 3] = rng.integers(0, 7, L).astype(np.float32)          # few distinct values
    S[0, 4] = 0.5                                               # constant
    S[0, 5] = -np.abs(S[0, 5]); S[0, 5].reshape(-1, 32)[8::16] = 5.0 + rng.random((L // 32 + 15 - 8) // 16 * 32).reshape(-1, 32)[: len(S[0, 5].reshape(-1, 32)[8::16])]
    S[0, 6] = -np.abs(S[0, 6]); S[0, 6].reshape(-1, 32)[3::16] += 6.0   # large values only in lines the sample skips
    S[0, 7, :20000] = -np.inf                                   # half the row at -inf
    q_pos = np.full(rows, L - 1, dtype=np.int32); q_pos[9] = 33000; q_pos[10] = 32767
    p = misa.Problem(1, L, rows, 8, 16, 2, misa.F32, misa.F32, torch.from_numpy(q_pos).cuda())
    for k in (2048, 100, 9000):
        idx = torch.empty((1, rows, k), dtype=torch.int32, device="cuda")
        val = torch.empty((1, rows, k), dtype=torch.float32, device="cuda")
        misa.topk(p, torch.from_numpy(S).cuda(), k, idx, val, misa.alloc_workspace(p, misa.OP_TOPK, k))
        idx, val = idx.cpu().numpy(), val.cpu().numpy()
        for t in list(range(12)) + [100, rows - 1]:
            n = int(q_pos[t]) + 1
            ref = O.topk(S[0, t, :n].astype(np.float64), k)
            np.testing.assert_array_equal(idx[0, t, :ref.shape[0]], ref, err_msg=f"row {t} k {k}")
            np.testing.assert_array_equal(val[0, t, :ref.shape[0]], S[0, t, ref])


def test_topk_longest_supported_rows(misa):
    # L = 524288 (the documented limit) and k = 16384: split path (one row) and
    # one-workgroup-per-row path (many rows; three of them checked)
    rng = np.random.default_rng(27)
    L = 524288
    S = rng.standard_normal((1, 1, L)).astype(np.float32)
    _topk_case(misa, S, 16384)
    rows = 260
    S = rng.standard_normal((1, rows, L)).astype(np.float32)
    p = misa.Problem(1, L, rows, 8, 16, 2, misa.F32, misa.F32,
                     torch.full((rows,), L - 1, dtype=torch.int32, device="cuda"))
    k = 2048
    idx = torch.empty((1, rows, k), dtype=torch.int32, device="cuda")
    misa.topk(p, torch.from_numpy(S).cuda(), k, idx, None, misa.alloc_workspace(p, misa.OP_TOPK, k))
    idx = idx.cpu().numpy()
    for t in (0, 131, rows - 1):
        ref = np.sort(np.argpartition(-S[0, t], k)[:k])      # no ties in random normals at this size
        assert set(ref.tolist()) == set(O.topk(S[0, t, :].astype(np.float64), k).tolist()) if t == 0 else True
        np.testing.assert_array_equal(idx[0, t], ref)


# --------------------------------------------------------------------- re-rank
@pytest.mark.parametrize("name", ["fp8_prefill", "bf16_decode", "f32_prefill"])
def test_rerank(misa, name):
    wl = CASES[name]
    inp = gen(name)
    dv = misa.to_device(inp)
    p = dv["problem"]
    kc, k = 512, 96
    cand = np.full((wl.n_seq, wl.n_q, kc), -1, dtype=np.int32)
    views = {}
    for s in range(wl.n_seq):
        for t in range(wl.n_q):
            K, q, w, n = views[(s, t)] = oracle_view(inp, s, t)
            c = O.misa(q, w, K, wl.B, wl.h, kc, n)["tokens"]
            cand[s, t, :c.shape[0]] = c
    cand[0, 0, 3] = -1                      # a hole in the middle and an invisible index are skipped
    cand[0, 0, kc - 1] = wl.L + 5
    idx = torch.empty((wl.n_seq, wl.n_q, k), dtype=torch.int32, device="cuda")
    val = torch.empty((wl.n_seq, wl.n_q, k), dtype=torch.float32, device="cuda")
    ws = misa.alloc_workspace(p, misa.OP_RERANK, kc)
    misa.rerank(p, dv["Q"], dv["W"], dv["K"], dv["kscale"], torch.from_numpy(cand).cuda(), kc, k, idx, val, ws)
    idx, val = idx.cpu().numpy(), val.cpu().numpy()
    for (s, t), (K, q, w, n) in views.items():
        dense = O.dsa_scores(q, w, K, n)
        valid = np.array(sorted(c for c in cand[s, t] if 0 <= c < n), dtype=np.int64)
        ke = min(k, valid.shape[0])
        got = idx[s, t]
        assert np.all(got[ke:] == -1) and np.all(np.diff(got[:ke]) > 0)
        assert set(got[:ke].tolist()) <= set(valid.tolist())
        # positions of the chosen tokens inside the candidate list obey the margin rule
        pos = np.searchsorted(valid, got[:ke])
        padded = np.concatenate([pos, np.full(k - ke, -1, dtype=pos.dtype)])
        check_index_set(padded, dense[valid], k, f"rerank {name} {s},{t}")
        assert_scores_close(val[s, t, :ke], dense[got[:ke]], f"rerank values {name} {s},{t}")
        assert np.all(np.isneginf(val[s, t, ke:]))


# --------------------------------------------------------------------- determinism
def test_run_twice_bit_identical(misa):
    wl = CASES["fp8_prefill"]
    inp = gen("fp8_prefill")
    dv = misa.to_device(inp)
    outs = []
    for _ in range(2):
        ix = misa.Indexer(dv["problem"], wl.k, wl.k_cand, want_E=True, want_val=True)
        ix.run(dv["K"], dv["kscale"], dv["Q"], dv["W"])
        torch.cuda.synchronize()
        outs.append([x.clone() for x in (ix.Kp, ix.heads, ix.E, ix.S, ix.idx1, ix.idx, ix.val)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


# --------------------------------------------------------------------- measurement probes
def test_measurement_probes_report_plausible_rates(misa):
    peaks = misa.measured_peaks(repeats=3)
    assert 2000.0 < peaks["hbm_read_GBps"] < 8000.0          # below the published 8 TB/s, above any cache-less floor
    assert 500.0 < peaks["mfma_bf16_TFLOPs"] < 2600.0        # below the published 2.5 PFLOP/s dense bf16
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    flops = misa.probe_mfma_bf16(1, 3, sink)
    torch.cuda.synchronize()
    assert flops == 4 * 3 * 4 * 2 * 32 * 32 * 16
    # operands are 1.0 x {0.5, 1.0}: every accumulator element is 3 iterations x 16 products
    got = sink.cpu().numpy()
    assert set(np.unique(got).tolist()) <= {4 * 16 * 3 * 16 * 0.5, 4 * 16 * 3 * 16 * 1.0, 4 * 16 * 3 * 16 * 0.75}
    # the same loop on supplied operands: a = 2.0, b = 0.25 everywhere, so every product is 0.5
    ops = torch.cat([torch.full((512,), 2.0), torch.full((512,), 0.25)]).to(torch.bfloat16).cuda()
    sink.zero_()
    assert misa.probe_mfma_bf16(1, 3, sink, ops) == flops
    torch.cuda.synchronize()
    assert np.all(sink.cpu().numpy() == 4 * 16 * 3 * 16 * 0.5)
    # Gaussian operands make the chip hold a lower clock: a lower rate than on the constant operands
    assert 500.0 < peaks["mfma_bf16_gaussian_operands_TFLOPs"] < 1.02 * peaks["mfma_bf16_TFLOPs"]


# --------------------------------------------------------------------- random top-k rows
@pytest.mark.parametrize("seed", range(30))
def test_topk_random_distributions(misa, seed):
    # shapes on both sides of every path switch (one workgroup per row / key ranges per row; sampled
    # hand-over usable or not), value distributions with heavy tails, plateaus, ties and -inf
    rng = np.random.default_rng(9000 + seed)
    L = int(rng.choice([int(rng.integers(1, 3000)), int(rng.integers(3000, 40000)), int(rng.integers(32768, 150000))]))
    n_seq = int(rng.integers(1, 4))
    n_q = 1 if rng.integers(0, 2) else int(rng.integers(2, 6))
    k = int(min(rng.choice([1, 7, 100, 1000, 2048, 5000, 9000, 16384]), 16384))
    kind = seed % 6
    shape = (n_seq, n_q, L)
    if kind == 0:
        S = rng.standard_normal(shape)
    elif kind == 1:
        S = rng.standard_cauchy(shape)                                   # heavy tails both ways
    elif kind == 2:
        S = np.round(rng.standard_normal(shape) * 4) / 4                 # many exact ties
    elif kind == 3:
        S = np.maximum(rng.standard_normal(shape), 0.0)                  # half the row exactly zero (ReLU scores)
    elif kind == 4:
        S = rng.standard_normal(shape)
        S[..., : L // 3] += 50.0                                         # a plateau far above the rest
    else:
        S = np.exp(rng.standard_normal(shape) * 3)
        S[rng.random(shape) < 0.3] = -np.inf
    S = S.astype(np.float32)
    q_pos = None if n_q == 1 else rng.integers(0, L, n_q).astype(np.int32)
    seq_len = rng.integers(0, L + 1, n_seq).astype(np.int32) if rng.integers(0, 2) else None
    _topk_case(misa, S, k, q_pos=q_pos, seq_len=seq_len)


# --------------------------------------------------------------------- random re-rank / pooled-key updates
@pytest.mark.parametrize("seed", range(12))
def test_rerank_random_candidate_lists(misa, seed):
    rng = np.random.default_rng(9500 + seed)
    decode = bool(rng.integers(0, 2))
    H = int(rng.choice([1, 8, 17, 32, 64]))
    L = int(rng.integers(30, 3000))
    wl = WL.scaled(WL.WORKLOADS["c3" if decode else "c2"], n_seq=int(rng.integers(1, 4)), L=L,
                   n_q=1 if decode else int(rng.integers(2, 30)), H=H, h=1, B=64, k=1, k_cand=0,
                   k_dtype=["f32", "bf16", "e4m3"][seed % 3], q_dtype=["bf16", "e4m3", "f32"][(seed // 3) % 3],
                   needles=4, name=f"rr{seed}")
    inp = WL.make_inputs(wl, seed=seed, seq_len=rng.integers(0, L + 1, wl.n_seq).astype(np.int32) if seed % 2 else None)
    dv = misa.to_device(inp)
    if seed % 4 == 3:
        dv = misa.paginate(dv, 32, seed=seed)
    p = dv["problem"]
    kc = int(rng.integers(1, min(L, 2500) + 1))
    k = int(rng.integers(1, kc + 1))
    cand = np.full((wl.n_seq, wl.n_q, kc), -1, dtype=np.int32)
    for s in range(wl.n_seq):
        for t in range(wl.n_q):
            c = np.sort(rng.choice(L, size=int(rng.integers(0, kc + 1)), replace=False)).astype(np.int32)
            c[rng.random(c.shape[0]) < 0.05] = -1                 # holes
            cand[s, t, :c.shape[0]] = c
    idx = torch.empty((wl.n_seq, wl.n_q, k), dtype=torch.int32, device="cuda")
    val = torch.empty((wl.n_seq, wl.n_q, k), dtype=torch.float32, device="cuda")
    misa.rerank(p, dv["Q"], dv["W"], dv["K"], dv["kscale"], torch.from_numpy(cand).cuda(), kc, k, idx, val,
                misa.alloc_workspace(p, misa.OP_RERANK, kc))
    idx, val = idx.cpu().numpy(), val.cpu().numpy()
    for s in range(wl.n_seq):
        for t in range(wl.n_q):
            K, q, w, n = oracle_view(inp, s, t)
            dense = O.dsa_scores(q, w, K, n) if n else np.zeros(0)
            valid = np.array(sorted(c for c in cand[s, t] if 0 <= c < n), dtype=np.int64)
            ke = min(k, valid.shape[0])
            got = idx[s, t]
            assert np.all(got[ke:] == -1) and np.all(np.diff(got[:ke]) > 0)
            assert set(got[:ke].tolist()) <= set(valid.tolist())
            pos = np.searchsorted(valid, got[:ke])
            padded = np.concatenate([pos, np.full(k - ke, -1, dtype=pos.dtype)])
            check_index_set(padded, dense[valid], k, f"rerank rr{seed} {s},{t}")
            assert_scores_close(val[s, t, :ke], dense[got[:ke]], f"rerank values rr{seed} {s},{t}")
            assert np.all(np.isneginf(val[s, t, ke:]))


@pytest.mark.parametrize("seed", range(12))
def test_pool_update_random(misa, seed):
    from dataclasses import replace
    rng = np.random.default_rng(9700 + seed)
    L = int(rng.integers(10, 9000))
    B = int(rng.choice([1, 3, 64, 128, 1024, 2500, L + 1]))
    wl = WL.scaled(WL.WORKLOADS["c3"], n_seq=int(rng.integers(1, 5)), L=L, B=B, k=1, needles=0,
                   k_dtype=["f32", "bf16", "e4m3"][seed % 3], name=f"pu{seed}")
    new_len = rng.integers(0, L + 1, wl.n_seq).astype(np.int32)
    old_len = (new_len - rng.integers(0, 3 * B + 2, wl.n_seq)).clip(0).astype(np.int32)
    inp = WL.make_inputs(wl, seed=seed, seq_len=new_len)
    dv = misa.to_device(inp)
    if seed % 3 == 1:
        dv = misa.paginate(dv, 64, seed=seed)
    p_new = dv["problem"]
    ws = misa.alloc_workspace(p_new, misa.OP_POOL)
    full = torch.full((wl.n_seq, p_new.M, wl.d), 7.0, dtype=torch.float32, device="cuda")
    misa.pool_keys(p_new, dv["K"], dv["kscale"], full, ws)
    old_dev = torch.from_numpy(old_len).cuda()
    Kp = torch.full_like(full, 7.0)
    misa.pool_keys(replace(p_new, seq_len=old_dev), dv["K"], dv["kscale"], Kp, ws)
    misa.pool_keys_update(p_new, dv["K"], dv["kscale"], Kp, old_dev, p_new.M, ws)
    assert torch.equal(Kp, full)
    # directly against the block means of Eq. pool (sliced blocks, ragged lengths, paged keys included);
    # entries past a sequence's last block keep what the pooling at the old length left (zeros)
    got = Kp.cpu().numpy()
    for s in range(wl.n_seq):
        K, _, _, n = oracle_view(inp, s, 0)
        ref = O.pool_keys(K, B, n)
        assert_scores_close(got[s, :ref.shape[0]], ref, f"pool update pu{seed} seq {s}")
        assert not got[s, ref.shape[0]:].any()


@pytest.mark.parametrize("seed", range(9))
def test_route_heads_proxy_random(misa, seed):
    rng = np.random.default_rng(9900 + seed)
    H = int(rng.choice([1, 2, 17, 32, 64]))
    wl = WL.scaled(WL.WORKLOADS["c2"], n_seq=int(rng.integers(1, 4)), L=64, n_q=int(rng.integers(1, 50)), H=H,
                   h=int(rng.integers(1, H + 1)), B=16, k=1, needles=0, q_dtype=["bf16", "e4m3", "f32"][seed % 3],
                   k_dtype="bf16", name=f"proxy{seed}")
    inp = WL.make_inputs(wl, seed=seed)
    dv = misa.to_device(inp)
    for kind, code in (("gate", misa.ROUTER_GATE), ("qnorm", misa.ROUTER_QUERY_NORM)):
        heads = torch.full((wl.n_seq, wl.n_q, wl.h), -5, dtype=torch.int32, device="cuda")
        E = torch.empty((wl.n_seq, wl.n_q, wl.H), dtype=torch.float32, device="cuda")
        misa.route_heads_proxy(dv["problem"], dv["Q"], dv["W"], code, heads, E)
        heads, E = heads.cpu().numpy(), E.cpu().numpy()
        for s in range(wl.n_seq):
            for t in range(wl.n_q):
                _, q, w, _ = oracle_view(inp, s, t)
                _, ref_E = O.route_heads_proxy(q, w, wl.h, kind)
                assert_scores_close(E[s, t], ref_E, f"proxy E {kind} {s},{t}")
                check_index_set(heads[s, t], ref_E, wl.h, f"proxy heads {kind} {s},{t}")
