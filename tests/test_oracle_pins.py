"""Pins for the CPU oracle: hand-worked fixture, closed forms, invariants,
special cases that reduce to library routines, exact brute force.

None of these tests touches the GPU or the HIP library.
"""
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import misa_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


# ---------------------------------------------------------------- fixture
@pytest.fixture(scope="module")
def hand():
    with open(os.path.join(HERE, "golden", "hand_example.json")) as f:
        return json.load(f)


@pytest.mark.parametrize("case", [0, 1])
def test_hand_worked_example(hand, case):
    c = hand["cases"][case]
    K = np.array(hand["K"], float); q = np.array(hand["q"], float); w = np.array(hand["w"], float)
    n, B, h, k, kc = c["n"], hand["B"], hand["h"], hand["k"], hand["k_cand"]
    np.testing.assert_allclose(O.pool_keys(K, B, n), c["pooled"], rtol=0, atol=1e-15)
    heads, E = O.route_heads(q, w, K, B, h, n)
    np.testing.assert_allclose(E, c["E"], rtol=1e-15)
    assert heads.tolist() == c["heads"]
    s = O.score_tokens(q, w, heads, K, n)
    np.testing.assert_allclose(s, c["scores"], rtol=0, atol=1e-15)
    assert O.topk(s, k).tolist() == c["tokens"]
    assert O.topk(s, kc).tolist() == c["candidates"]
    np.testing.assert_allclose(O.dsa_scores(q, w, K, n), c["dense_scores"], rtol=0, atol=1e-15)
    assert O.dsa_dense(q, w, K, k, n)["tokens"].tolist() == c["dense_tokens"]
    dag = O.misa_dagger(q, w, K, B, h, kc, k, n)
    assert dag["tokens"].tolist() == c["dagger_tokens"]
    np.testing.assert_allclose(dag["values"], c["dagger_values"], rtol=0, atol=1e-15)
    assert O.misa(q, w, K, B, h, k, n)["tokens"].tolist() == c["tokens"]


# ---------------------------------------------------------------- decoding
def test_e4m3_table_closed_forms():
    t = O.e4m3fn_decode_table()
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and np.signbit(t[0x80])
    assert t[0x01] == 2.0 ** -9            # smallest subnormal
    assert t[0x07] == 7 * 2.0 ** -9        # largest subnormal
    assert t[0x08] == 2.0 ** -6            # smallest normal
    assert t[0x38] == 1.0
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0   # largest finite
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF])  # no infinity in e4m3fn
    finite = t[:0x7F]
    assert np.all(np.diff(finite) > 0)     # codes are monotone in value
    np.testing.assert_array_equal(t[0x80:0xFF], -t[0x00:0x7F])


def test_e4m3_table_matches_torch_cast():
    torch = pytest.importorskip("torch")
    codes = torch.arange(256, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    np.testing.assert_array_equal(np.nan_to_num(O.e4m3fn_decode_table(), nan=-7.0),
                                  np.nan_to_num(ref, nan=-7.0))


def test_bf16_bits_match_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(1)
    bits = rng.integers(0, 1 << 16, 4096).astype(np.uint16)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF]          # skip inf/nan patterns
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.bf16_bits_to_f64(bits), ref)


def test_dequantise_e4m3_scale_per_token():
    codes = np.array([[0x38, 0x40], [0x38, 0xB8]], dtype=np.uint8)   # 1,2 / 1,-1
    scale = np.array([0.5, 3.0], dtype=np.float32)
    np.testing.assert_array_equal(O.dequantise(codes, "e4m3", scale), [[0.5, 1.0], [3.0, -3.0]])


# ---------------------------------------------------------------- pool
def test_pool_special_cases():
    rng = np.random.default_rng(2)
    K = rng.standard_normal((24, 5))
    np.testing.assert_array_equal(O.pool_keys(K, 1), K)                           # B = 1
    np.testing.assert_allclose(O.pool_keys(K, 24)[0], K.mean(0), rtol=1e-14)      # one global mean
    np.testing.assert_allclose(O.pool_keys(K, 100)[0], K.mean(0), rtol=1e-14)     # B > n
    np.testing.assert_allclose(O.pool_keys(K, 6), K.reshape(4, 6, 5).mean(1), rtol=1e-14)
    P = O.pool_keys(K, 7)                                                         # partial last block
    assert P.shape == (4, 5)
    np.testing.assert_allclose(P[3], K[21:24].mean(0), rtol=1e-14)                # mean over 3, not 7
    assert O.pool_keys(K, 4, n=0).shape == (0, 5)
    np.testing.assert_allclose(O.pool_keys(K, 4, n=6)[1], K[4:6].mean(0), rtol=1e-14)   # prefix only


def test_pool_is_weighted_mean_of_means():
    # The count-weighted mean of the pooled keys is the global mean (catches a
    # divisor of B on the partial block).
    rng = np.random.default_rng(3)
    K = rng.standard_normal((23, 4)); B = 5
    P = O.pool_keys(K, B)
    cnt = np.array([5, 5, 5, 5, 3], float)
    np.testing.assert_allclose((P * cnt[:, None]).sum(0) / 23, K.mean(0), rtol=1e-13)


# ---------------------------------------------------------------- brute force (exact)
def _brute(K, q, w, B, h, k, n, k_cand=None):
    """Exact rational arithmetic, scalar loops, straight from the equations."""
    d, H = len(K[0]), len(q)
    K = [[Fraction(x) for x in row] for row in K[:n]]
    q = [[Fraction(x) for x in row] for row in q]
    w = [Fraction(x) for x in w]
    dot = lambda a, b: sum(x * y for x, y in zip(a, b))
    relu = lambda x: x if x > 0 else Fraction(0)
    M = -(-n // B)
    pooled = []
    for b in range(M):
        blk = K[b * B:min((b + 1) * B, n)]
        pooled.append([sum(r[c] for r in blk) / len(blk) for c in range(d)])
    E = []
    for j in range(H):
        E.append(sum(abs(w[j] * relu(dot(q[j], pooled[b]))) for b in range(M)) / M if M else Fraction(0))
    heads = sorted(sorted(range(H), key=lambda j: (-E[j], j))[:h])
    sc = [sum(w[j] * relu(dot(q[j], K[s])) for j in heads) for s in range(n)]
    dense = [sum(w[j] * relu(dot(q[j], K[s])) for j in range(H)) for s in range(n)]
    pick = lambda vals, idxs, c: sorted(sorted(idxs, key=lambda s: (-vals[s], s))[:c])
    tokens = pick(sc, range(n), k)
    out = dict(E=E, heads=heads, scores=sc, dense=dense, tokens=tokens,
               dense_tokens=pick(dense, range(n), k))
    if k_cand is not None:
        cand = pick(sc, range(n), k_cand)
        out["cand"] = cand
        out["dagger"] = pick(dense, cand, k)
    return out


@pytest.mark.parametrize("n,B,H,h,k", [
    (1, 1, 2, 1, 1), (5, 4, 4, 2, 3), (17, 4, 8, 2, 5), (17, 8, 8, 8, 17), (33, 2, 4, 1, 40),
    (64, 16, 8, 2, 9), (40, 64, 4, 2, 7), (30, 1, 2, 2, 30),
])
def test_brute_force_exact_small_integers(n, B, H, h, k):
    # Small-integer inputs and power-of-two B keep every quantity exactly
    # representable, and force many exact ties (duplicated keys, repeated
    # scores), so index sets must agree exactly, ties included.
    rng = np.random.default_rng(100 + n + B + H)
    d = 4
    K = rng.integers(-2, 3, (n, d))
    K[rng.integers(0, n, n // 3 + 1)] = K[0]           # duplicated keys
    q = rng.integers(-2, 3, (H, d)); w = rng.integers(-2, 3, H) / 4.0
    kc = max(k, min(n, 2 * k))
    ref = _brute(K.tolist(), q.tolist(), w.tolist(), B, h, k, n, kc)
    heads, E = O.route_heads(q, w, K, B, h, n)
    assert [Fraction(x) for x in E.tolist()] == ref["E"] or np.allclose(E, [float(x) for x in ref["E"]], rtol=1e-15, atol=0)
    assert heads.tolist() == ref["heads"]
    s = O.score_tokens(q, w, heads, K, n)
    assert s.tolist() == [float(x) for x in ref["scores"]]
    assert O.topk(s, k).tolist() == ref["tokens"]
    assert O.dsa_scores(q, w, K, n).tolist() == [float(x) for x in ref["dense"]]
    assert O.dsa_dense(q, w, K, k, n)["tokens"].tolist() == ref["dense_tokens"]
    dag = O.misa_dagger(q, w, K, B, h, kc, k, n)
    assert dag["candidates"].tolist() == ref["cand"]
    assert dag["tokens"].tolist() == ref["dagger"]


@pytest.mark.parametrize("n,B", [(5, 3), (17, 5), (130, 64), (130, 200), (64, 7)])
def test_brute_force_random_floats(n, B):
    rng = np.random.default_rng(7 * n + B)
    H, d, h, k = 4, 8, 2, max(1, n // 3)
    K = np.round(rng.standard_normal((n, d)) * 64) / 64     # dyadic, exact as Fractions
    q = np.round(rng.standard_normal((H, d)) * 64) / 64
    w = np.round(rng.standard_normal(H) * 64) / 64
    ref = _brute(K.tolist(), q.tolist(), w.tolist(), B, h, k, n, min(n, 2 * k))
    heads, E = O.route_heads(q, w, K, B, h, n)
    np.testing.assert_allclose(E, [float(x) for x in ref["E"]], rtol=1e-13)
    assert heads.tolist() == ref["heads"]
    s = O.score_tokens(q, w, heads, K, n)
    np.testing.assert_allclose(s, [float(x) for x in ref["scores"]], rtol=1e-13, atol=1e-15)
    assert O.topk(s, k).tolist() == ref["tokens"]
    assert O.misa_dagger(q, w, K, B, h, min(n, 2 * k), k, n)["tokens"].tolist() == ref["dagger"]


# ---------------------------------------------------------------- router invariants
def _rand(n=96, H=8, d=16, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n, d)), rng.standard_normal((H, d)), rng.standard_normal(H)


def test_route_all_heads_when_h_equals_H():
    K, q, w = _rand()
    heads, _ = O.route_heads(q, w, K, 8, 8)
    assert heads.tolist() == list(range(8))


def test_route_closed_form_abs_w_times_mean_relu():
    K, q, w = _rand(seed=4)
    _, E = O.route_heads(q, w, K, 8, 3)
    Kp = K.reshape(12, 8, 16).mean(1)
    np.testing.assert_allclose(E, np.abs(w) * np.maximum(q @ Kp.T, 0).mean(1), rtol=1e-13)


def test_route_permutation_and_scale_invariance():
    K, q, w = _rand(seed=5)
    heads, E = O.route_heads(q, w, K, 8, 3)
    perm = np.random.default_rng(9).permutation(8)
    hp, Ep = O.route_heads(q[perm], w[perm], K, 8, 3)
    np.testing.assert_allclose(Ep, E[perm], rtol=1e-14)
    assert sorted(perm[hp].tolist()) == heads.tolist()
    h2, E2 = O.route_heads(q, 3.5 * w, K, 8, 3)             # scaling all gates keeps H_t
    assert h2.tolist() == heads.tolist()
    np.testing.assert_allclose(E2, 3.5 * E, rtol=1e-14)
    h3, _ = O.route_heads(q, -w, K, 8, 3)                   # |A| ignores the gate's sign
    assert h3.tolist() == heads.tolist()


def test_route_hisa_identity_and_dense_link():
    # With non-negative gates, M * sum_j E_j equals the sum over blocks of the
    # HISA block score J_b (Eq. block_score); with B = 1 that is the mean dense
    # DSA score (Eq. dsa_score).
    K, q, w = _rand(seed=6)
    w = np.abs(w)
    _, E = O.route_heads(q, w, K, 8, 3)
    Kp = O.pool_keys(K, 8)
    J = (w[:, None] * np.maximum(q @ Kp.T, 0)).sum(0)
    np.testing.assert_allclose(Kp.shape[0] * E.sum(), J.sum(), rtol=1e-13)
    _, E1 = O.route_heads(q, w, K, 1, 3)
    np.testing.assert_allclose(E1.sum(), O.dsa_scores(q, w, K).mean(), rtol=1e-13)


def test_route_prefix_is_causal():
    # Changing keys after position p must not change the routing of query p.
    K, q, w = _rand(seed=7)
    K2 = K.copy(); K2[50:] += 10.0
    a = O.route_heads(q, w, K, 8, 3, n=50)
    b = O.route_heads(q, w, K2, 8, 3, n=50)
    assert a[0].tolist() == b[0].tolist()
    np.testing.assert_array_equal(a[1], b[1])
    # and equals decode on the truncated cache
    c = O.route_heads(q, w, K[:50], 8, 3)
    np.testing.assert_array_equal(a[1], c[1])


def test_route_empty_prefix():
    K, q, w = _rand()
    heads, E = O.route_heads(q, w, K, 8, 3, n=0)
    assert heads.tolist() == [0, 1, 2] and not E.any()


# ---------------------------------------------------------------- scoring
def test_score_all_heads_is_dense_dsa():
    K, q, w = _rand(seed=8)
    dense = (w[None, :] * np.maximum(K @ q.T, 0)).sum(1)        # Eq. dsa_score via one matmul
    np.testing.assert_allclose(O.score_tokens(q, w, np.arange(8), K), dense, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(O.dsa_scores(q, w, K), dense, rtol=1e-13, atol=1e-15)
    m = O.misa(q, w, K, 8, 8, 10)                               # h = H reproduces DSA
    assert m["tokens"].tolist() == O.dsa_dense(q, w, K, 10)["tokens"].tolist()
    np.testing.assert_array_equal(m["scores"], O.dsa_scores(q, w, K))


def test_score_single_head_is_relu_gemv():
    K, q, w = _rand(seed=9)
    w1 = np.zeros(8); w1[3] = 1.0
    np.testing.assert_allclose(O.score_tokens(q, w1, [3], K), np.maximum(K @ q[3], 0), rtol=1e-14)
    assert np.all(O.score_tokens(q, w1, [3], K)[(K @ q[3]) <= 0] == 0)


def test_score_linear_in_gates_and_head_additive():
    K, q, w = _rand(seed=10)
    a = O.score_tokens(q, w, [1, 4, 6], K)
    np.testing.assert_allclose(O.score_tokens(q, 2.0 * w, [1, 4, 6], K), 2.0 * a, rtol=1e-14)
    parts = sum(O.score_tokens(q, w, [j], K) for j in (1, 4, 6))
    np.testing.assert_allclose(a, parts, rtol=1e-13, atol=1e-15)
    with pytest.raises(ValueError):
        O.score_tokens(q, w, [1, 1], K)


def test_score_fp8_scale_is_homogeneous():
    rng = np.random.default_rng(11)
    codes = rng.integers(0, 0x7F, (40, 16)).astype(np.uint8) | (rng.integers(0, 2, (40, 16)) << 7).astype(np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x10
    sc = rng.uniform(0.01, 0.1, 40).astype(np.float32)
    _, q, w = _rand(d=16, seed=12)
    a = O.score_tokens(q, w, [0, 2], O.dequantise(codes, "e4m3", sc))
    b = O.score_tokens(q, w, [0, 2], O.dequantise(codes, "e4m3", (4 * sc).astype(np.float32)))
    np.testing.assert_allclose(b, 4 * a, rtol=1e-14)


def test_score_respects_prefix():
    K, q, w = _rand(seed=13)
    assert O.score_tokens(q, w, [0, 1], K, n=37).shape == (37,)
    np.testing.assert_array_equal(O.score_tokens(q, w, [0, 1], K, n=37), O.score_tokens(q, w, [0, 1], K)[:37])


# ---------------------------------------------------------------- top-k
def test_topk_definition_by_exhaustive_subsets():
    # The result is the unique k-subset that is maximal under (score desc,
    # index asc): check against every subset on a tiny row with ties.
    s = np.array([1.0, 3.0, 3.0, -0.0, 0.0, 2.0, 3.0])
    for k in range(1, 8):
        best = max(itertools.combinations(range(7), k),
                   key=lambda c: (sum(s[i] for i in c), [-i for i in sorted(c)]))
        # lexicographic: maximise total score, then prefer lower indices among ties
        got = O.topk(s, k).tolist()
        assert len(set(got)) == k and got == sorted(got)
        assert sum(s[i] for i in got) == sum(s[i] for i in best)
        out = [i for i in range(7) if i not in got]
        for i in got:
            for j in out:
                assert s[i] > s[j] or (s[i] == s[j] and i < j)


def test_topk_matches_numpy_stable_sort_and_edge_cases():
    rng = np.random.default_rng(14)
    s = np.round(rng.standard_normal(500) * 4) / 4              # many ties
    for k in (1, 7, 100, 499, 500):
        ref = np.sort(np.argsort(-s, kind="stable")[:k])
        assert O.topk(s, k).tolist() == ref.tolist()
    assert O.topk(s, 900).tolist() == list(range(500))          # k > n: everything
    assert O.topk(np.full(50, 1.5), 8).tolist() == list(range(8))   # constant row
    z = np.array([0.0, -0.0, 0.0, -0.0])
    assert O.topk(z, 2).tolist() == [0, 1]                      # -0.0 ties with +0.0
    with pytest.raises(ValueError):
        O.topk(s, 0)


# ---------------------------------------------------------------- MISA-dagger
def test_dagger_reduces_to_dsa():
    K, q, w = _rand(n=200, seed=15)
    dsa = O.dsa_dense(q, w, K, 20)["tokens"].tolist()
    assert O.misa_dagger(q, w, K, 16, 2, 200, 20)["tokens"].tolist() == dsa     # k' = n
    assert O.misa_dagger(q, w, K, 16, 2, 5000, 20)["tokens"].tolist() == dsa    # k' > n
    assert O.misa_dagger(q, w, K, 16, 8, 40, 20)["tokens"].tolist() == dsa      # h = H


def test_dagger_subset_and_recall_identity():
    K, q, w = _rand(n=300, seed=16)
    dsa = O.dsa_dense(q, w, K, 30)["tokens"]
    prev = -1.0
    for kc in (30, 60, 120, 300):
        r = O.misa_dagger(q, w, K, 16, 2, kc, 30)
        assert set(r["tokens"]) <= set(r["candidates"])
        # members of the dense top-k outrank everything else under I, so the
        # final set keeps exactly those of them that survived stage one
        assert set(r["tokens"]) & set(dsa) == set(dsa) & set(r["candidates"])
        rec = O.recall(r["tokens"], dsa)
        assert rec >= prev; prev = rec
        np.testing.assert_allclose(O.iou(r["tokens"], dsa), rec / (2 - rec), rtol=1e-12)
    assert prev == 1.0


def test_rerank_ignores_padding_and_invisible():
    K, q, w = _rand(n=50, seed=17)
    t, v = O.rerank(q, w, K, [-1, 3, 7, 49, 60, -1], 2, n=40)
    assert set(t) <= {3, 7}
    np.testing.assert_array_equal(v, O.dsa_scores(q, w, K, 40)[t])


# ---------------------------------------------------------------- cost model
def test_cost_model_counts():
    # DSA O(H n); MISA O(h n + H M); dagger adds k' H  (Method; kernel-speed section).
    c = O.head_token_products(131072, 64, 8, 1024)
    assert c == {"dense": 64 * 131072, "misa": 8 * 131072 + 64 * 128}
    c = O.head_token_products(131072, 64, 8, 64, 8192)
    assert c["misa"] == 1048576 + 131072 + 524288
    assert O.head_token_products(131072, 32, 8, 128)["dense"] / O.head_token_products(131072, 32, 8, 128)["misa"] == pytest.approx(3.878, abs=2e-3)


# ---------------------------------------------------------------- router-score ablation variants
def test_proxy_router_scores_closed_forms():
    # Appendix "Ablation: routing score": (a) the gate alone, (b) the query norm.
    rng = np.random.default_rng(41)
    H, d, h = 12, 16, 5
    q = rng.standard_normal((H, d))
    w = rng.standard_normal(H)
    heads, E = O.route_heads_proxy(q, w, h, "gate")
    np.testing.assert_array_equal(E, w)
    np.testing.assert_array_equal(heads, np.sort(np.argsort(-w)[:h]))          # distinct gates: plain sort
    assert w[heads].min() > np.delete(w, heads).max()
    # a negative gate of large magnitude is NOT up-weighted: it ranks last
    w2 = w.copy(); w2[3] = -100.0
    assert 3 not in O.route_heads_proxy(q, w2, H - 1, "gate")[0]
    # (b): axis-aligned queries with known lengths; scaling a head by c scales its score by |c|
    q3 = np.zeros((4, 3)); q3[0, 0] = 3.0; q3[1] = [1.0, 2.0, 2.0]; q3[2, 2] = -5.0; q3[3] = [0.0, 0.6, 0.8]
    heads, E = O.route_heads_proxy(q3, np.ones(4), 2, "qnorm")
    np.testing.assert_allclose(E, [3.0, 3.0, 5.0, 1.0], rtol=1e-15)
    np.testing.assert_array_equal(heads, [0, 2])                              # tie 3.0 == 3.0 -> lower index
    _, E2 = O.route_heads_proxy(-2.5 * q, w, h, "qnorm")
    np.testing.assert_allclose(E2, 2.5 * O.route_heads_proxy(q, w, h, "qnorm")[1], rtol=1e-14)
    np.testing.assert_allclose(O.route_heads_proxy(q, w, h, "qnorm")[1], np.linalg.norm(q, axis=1), rtol=1e-14)
    # neither variant looks at the gates' sign convention of the main router or at the keys
    with pytest.raises(ValueError):
        O.route_heads_proxy(q, w, 0, "gate")
    with pytest.raises(ValueError):
        O.route_heads_proxy(q, w, h, "pooled")


# ---------------------------------------------------------------- HISA / Block-Sparse comparison indexers
def test_block_scores_link_to_router_and_brute_force():
    # Eq. block_score and Eq. misa_route_score are the two marginals of the same affinity
    # matrix: with non-negative gates, sum_b J_b == M * sum_j E_j.
    rng = np.random.default_rng(51)
    H, d, L, B = 6, 8, 37, 5
    q = rng.standard_normal((H, d)); K = rng.standard_normal((L, d)); w = np.abs(rng.standard_normal(H))
    for n in (37, 35, 12, 5, 1):
        J = O.block_scores(q, w, K, B, n)
        _, E = O.route_heads(q, w, K, B, 2, n)
        M = -(-n // B)
        assert J.shape == (M,)
        np.testing.assert_allclose(J.sum(), M * E.sum(), rtol=1e-12)
        # brute force in exact rational arithmetic on a rounded copy
        qf = [[Fraction(float(np.round(x, 3))) for x in row] for row in q]
        Kf = [[Fraction(float(np.round(x, 3))) for x in row] for row in K]
        wf = [Fraction(float(np.round(x, 3))) for x in w]
        Jr = O.block_scores(np.round(q, 3), np.round(w, 3), np.round(K, 3), B, n)
        for b in range(M):
            rows = range(b * B, min((b + 1) * B, n))
            mean = [sum(Kf[s][c] for s in rows) / len(rows) for c in range(d)]
            tot = Fraction(0)
            for j in range(H):
                dot = sum(qf[j][c] * mean[c] for c in range(d))
                tot += wf[j] * max(dot, Fraction(0))
            assert abs(float(tot) - Jr[b]) <= 1e-12 * max(1.0, abs(float(tot)))
    # signed gates: a head with a negative gate lowers the block score
    w2 = w.copy(); w2[0] = -w2[0]
    assert np.all(O.block_scores(q, w2, K, B) <= O.block_scores(q, w, K, B) + 1e-15)


def test_select_blocks_keeps_first_and_last():
    J = np.array([-5.0, 3.0, 9.0, 1.0, 9.0, 2.0, -7.0])
    np.testing.assert_array_equal(O.select_blocks(J, 2), [0, 6])
    np.testing.assert_array_equal(O.select_blocks(J, 3), [0, 2, 6])          # tie 9 == 9 -> lower index
    np.testing.assert_array_equal(O.select_blocks(J, 4), [0, 2, 4, 6])
    np.testing.assert_array_equal(O.select_blocks(J, 5), [0, 1, 2, 4, 6])
    np.testing.assert_array_equal(O.select_blocks(J, 7), np.arange(7))
    np.testing.assert_array_equal(O.select_blocks(J, 50), np.arange(7))
    np.testing.assert_array_equal(O.select_blocks(np.array([1.0]), 2), [0])
    with pytest.raises(ValueError):
        O.select_blocks(J, 1)
    np.testing.assert_array_equal(O.block_tokens(np.array([0, 2]), 4, 10), [0, 1, 2, 3, 8, 9])


def test_hisa_reductions_and_invariants():
    rng = np.random.default_rng(52)
    H, d, L, B, k = 5, 8, 64, 8, 10
    q = rng.standard_normal((H, d)); K = rng.standard_normal((L, d)); w = rng.standard_normal(H)
    for n in (64, 61, 20):
        M = -(-n // B)
        dense = O.dsa_scores(q, w, K, n)
        full = O.hisa(q, w, K, B, M, k, n)                         # every block kept: the dense indexer
        np.testing.assert_array_equal(full["tokens"], O.topk(dense, k))
        r = O.hisa(q, w, K, B, 3, k, n)
        assert r["blocks"][0] == 0 and r["blocks"][-1] == M - 1 and len(r["blocks"]) == min(3, M)
        omega = O.block_tokens(r["blocks"], B, n)
        assert set(r["tokens"].tolist()) <= set(omega.tolist()) and len(r["tokens"]) == min(k, len(omega))
        # the selection is the dense top-k restricted to Omega
        sub = O.topk(dense[omega], k)
        np.testing.assert_array_equal(r["tokens"], omega[sub])
        np.testing.assert_allclose(r["values"], dense[r["tokens"]], rtol=0, atol=0)
        bs = O.block_sparse(q, w, K, B, 3, n)
        np.testing.assert_array_equal(bs["blocks"], r["blocks"])
        np.testing.assert_array_equal(bs["tokens"], omega)
    assert O.hisa(q, w, K, B, 3, k, 0)["tokens"].shape == (0,)


def test_recall_and_iou_hand_values_on_sets_of_different_size():
    # Eq. iou and the recall of a reference set, worked by hand; the two sets differ in size so
    # that dividing by the wrong set's size (or by the union instead of the reference) fails.
    sel, ref = [1, 2, 3, 4, 5, 6], [4, 5, 6, 7]
    assert O.recall(sel, ref) == 3 / 4          # 4, 5, 6 of the four reference tokens
    assert O.recall(ref, sel) == 3 / 6
    assert O.iou(sel, ref) == 3 / 7             # union {1..7}
    assert O.iou(ref, sel) == 3 / 7
    assert O.recall([9], [1, 2, 3]) == 0.0 and O.iou([9], [1, 2, 3]) == 0.0
    assert O.recall([1, 2, 3], [2]) == 1.0 and O.iou([1, 2, 3], [2]) == 1 / 3
    assert O.recall([], []) == 1.0 and O.iou([], []) == 1.0
    assert O.recall([], [5]) == 0.0


def test_overlap_statistics_of_the_report_generator_match_the_oracle_row_by_row():
    # recall / IoU as bench.py and the recall sweep compute them (torch, index rows padded with -1)
    torch = pytest.importorskip("torch")
    from paper_2605_07363_amd.recall_sweep import overlap, overlap_stats
    rng = np.random.default_rng(44)
    rows, ka, kb, n = 40, 24, 16, 60
    a = np.full((rows, ka), -1, dtype=np.int32)
    b = np.full((rows, kb), -1, dtype=np.int32)
    for r in range(rows):
        na, nb = int(rng.integers(0, ka + 1)), int(rng.integers(0, kb + 1))
        if r == 0:
            na, nb = 0, 0
        if r == 1:
            na, nb = ka, 0
        a[r, :na] = np.sort(rng.choice(n, na, replace=False))
        b[r, :nb] = np.sort(rng.choice(n, nb, replace=False))
    rec, iou = overlap_stats(torch.from_numpy(a), torch.from_numpy(b))
    for r in range(rows):
        sa, sb = a[r][a[r] >= 0], b[r][b[r] >= 0]
        assert rec[r].item() == pytest.approx(O.recall(sa, sb), abs=1e-12), r
        assert iou[r].item() == pytest.approx(O.iou(sa, sb), abs=1e-12), r
    assert overlap(torch.from_numpy(a), torch.from_numpy(b)) == pytest.approx(
        np.mean([O.recall(a[r][a[r] >= 0], b[r][b[r] >= 0]) for r in range(rows)]), abs=1e-12)
