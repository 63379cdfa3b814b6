"""Host-side checks of the seeded input generators (no GPU): shapes and storage types of
every configuration, determinism, the storage encodings against independent decoders, and
the planted structure (needles score high for their head, topic segments share a direction).
The generators hold none of the method's arithmetic; the oracle is used here only to decode
and to score."""
import numpy as np
import pytest

from oracle import misa_oracle as O
from paper_2605_07363_amd import workloads as WL

SMALL = {
    "c0": WL.WORKLOADS["c0"],
    "c1": WL.scaled(WL.WORKLOADS["c1"], n_seq=2, L=3000),
    "c2": WL.scaled(WL.WORKLOADS["c2"], L=5000, n_q=600),
    "c3": WL.scaled(WL.WORKLOADS["c3"], n_seq=2, L=5000, needles=16),
    "c4": WL.scaled(WL.WORKLOADS["c4"], L=5000, n_q=40, needles=16),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_shapes_types_and_determinism(name):
    wl = SMALL[name]
    a, b = WL.make_inputs(wl), WL.make_inputs(wl)
    kt = {"f32": np.float32, "bf16": np.uint16, "e4m3": np.uint8}[wl.k_dtype]
    qt = {"f32": np.float32, "bf16": np.uint16}[wl.q_dtype]
    assert a["K"].shape == (wl.n_seq, wl.L, wl.d) and a["K"].dtype == kt
    assert a["Q"].shape == (wl.n_seq, wl.n_q, wl.H, wl.d) and a["Q"].dtype == qt
    assert a["W"].shape == (wl.n_seq, wl.n_q, wl.H) and a["W"].dtype == np.float32
    if wl.k_dtype == "e4m3":
        assert a["kscale"].shape == (wl.n_seq, wl.L) and a["kscale"].dtype == np.float32
        assert np.all(a["kscale"] > 0)
        assert not np.any((a["K"] & 0x7F) == 0x7F)                 # no NaN codes
    else:
        assert a["kscale"] is None
    if wl.decode:
        assert a["q_pos"] is None
    else:
        np.testing.assert_array_equal(a["q_pos"], np.arange(wl.L - wl.n_q, wl.L))
    for key in ("K", "Q", "W"):
        np.testing.assert_array_equal(a[key], b[key])             # same seed, same bytes
    c = WL.make_inputs(wl, seed=1)
    assert not np.array_equal(a["W"], c["W"])
    assert (a["W"] < 0).any() and (a["W"] > 0).any()              # gates of both signs


def test_pairs_count():
    assert WL.WORKLOADS["c1"].pairs() == 64 * 32768
    assert WL.WORKLOADS["c3"].pairs() == 32 * 131072
    wl = WL.WORKLOADS["c2"]
    assert wl.pairs() == sum(range(wl.L - wl.n_q + 1, wl.L + 1))


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -9, -3.1415927, 0.0, -0.0, 1e-40, 65504.0],
                 dtype=np.float32)
    bits = WL.f32_to_bf16_bits(x)
    back = WL.bf16_bits_to_f32(bits)
    np.testing.assert_array_equal(back[:4], np.array([1.0, 1.0, 1.0 + 2 ** -6, 1.0], dtype=np.float32))  # ties to even
    assert np.all(np.abs(back[[4, 8]] - x[[4, 8]]) <= np.abs(x[[4, 8]]) * 2.0 ** -8)
    np.testing.assert_array_equal(O.bf16_bits_to_f64(bits), back.astype(np.float64))  # two decoders agree


def test_fp8_quantisation_round_trips_within_half_a_step():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((50, 128)).astype(np.float32)
    codes, scale = WL.quantise_e4m3(x)
    np.testing.assert_allclose(scale, np.abs(x).max(axis=1) / 448.0, rtol=1e-6)
    back = O.dequantise(codes, "e4m3", scale)
    # e4m3 has 3 mantissa bits: relative step 2^-3 above the subnormal range, absolute step 2^-9 * scale below
    err = np.abs(back - x)
    bound = np.maximum(np.abs(x) * 2.0 ** -4, scale[:, None] * 2.0 ** -10) * 1.0001
    assert np.all(err <= bound)
    assert np.abs(back).max(axis=1) == pytest.approx(np.abs(x).max(axis=1), rel=1e-6)   # the row maximum is exact


def test_needles_and_topics_are_planted():
    wl = SMALL["c3"]
    inp = WL.make_inputs(wl)
    K = O.dequantise(inp["K"][0], "e4m3", inp["kscale"][0])
    norms = np.linalg.norm(K, axis=1)
    needles = np.flatnonzero(np.abs(norms - WL.NEEDLE_GAIN) < 0.15)
    assert needles.shape[0] == wl.needles                          # planted keys have norm 4, all others ~1.1
    q = O.dequantise(inp["Q"][0, 0], "bf16")
    cos = (K[needles] @ q.T) / (norms[needles, None] * np.linalg.norm(q, axis=1)[None, :])
    assert np.all(cos.max(axis=1) > 0.97)                          # each needle is aligned with one query head
    # keys of one topic segment share a direction: their mean is far from zero, and segment means
    # of the same topic agree
    seg = K[:WL.TOPIC_SEGMENT]
    seg = seg[np.abs(np.linalg.norm(seg, axis=1) - WL.NEEDLE_GAIN) > 0.15]
    assert np.linalg.norm(seg.mean(axis=0)) == pytest.approx(WL.TOPIC_KEY_AMPL, abs=0.08)


def test_fp8_queries_fold_their_scale_into_the_gates():
    # q_dtype = "e4m3": the generator stores codes only and multiplies the gates by the
    # per-(query, head) scale.  Because ReLU is positively homogeneous, scoring the codes with the
    # folded gates equals scoring the de-quantised queries (codes x scale) with the original
    # gates (Eq. misa_score / Eq. dsa_score): checked with the oracle on every head.
    wl8 = WL.scaled(WL.WORKLOADS["c1"], n_seq=1, L=400, q_dtype="e4m3", needles=0)
    wl16 = WL.scaled(wl8, q_dtype="bf16")
    a, b = WL.make_inputs(wl8, seed=3), WL.make_inputs(wl16, seed=3)
    assert a["Q"].dtype == np.uint8 and a["Q"].shape == b["Q"].shape
    np.testing.assert_array_equal(a["K"], b["K"])                   # same random stream otherwise
    codes = O.e4m3fn_decode_table()[a["Q"][0, 0]]                    # [H, d] values of the codes
    w_folded = a["W"][0, 0].astype(np.float64)
    w_plain = b["W"][0, 0].astype(np.float64)
    scale = w_folded / w_plain                                       # what the generator folded in
    assert np.all(scale > 0)
    K = O.dequantise(a["K"][0], wl8.k_dtype)
    heads = np.arange(wl8.H)
    s_codes = O.score_tokens(codes, w_folded, heads, K)
    s_values = O.score_tokens(codes * scale[:, None], w_plain, heads, K)
    np.testing.assert_allclose(s_codes, s_values, rtol=1e-6, atol=1e-9)
    # and the codes times their scale reproduce the bf16-free original queries to fp8 precision
    q_orig = O.dequantise(b["Q"][0, 0], "bf16")
    amax = np.abs(q_orig).max(axis=-1, keepdims=True)
    assert np.all(np.abs(codes * scale[:, None] - q_orig) <= amax * (2.0 ** -4 + 2.0 ** -8))
