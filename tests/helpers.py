"""Shared helpers of the GPU parity tests: oracle views of generated inputs,
the score tolerance and the margin rule for index sets."""
import numpy as np

from oracle import misa_oracle as O

REL_TOL = 1e-3      # relative score tolerance fixed by the benchmark spec
ABS_FRAC = 1e-5     # absolute term as a fraction of the largest |score| of the row
# The same for scores contracted on the fp8 matrix instruction (q_dtype FP8_E4M3_MATRIX with fp8
# keys): that instruction adds its 64 exact products in a format narrower than fp32; measured on
# MI355X a 128-term dot product is within 2^-15 of the sum of its absolute products (fp32
# accumulation: 2^-22), which for the score magnitudes of a row comes to a few 1e-5 of the largest.
ABS_FRAC_FP8_MATRIX = 4e-5


def oracle_view(inp, seq, t):
    """(K float64 [L,d], q [H,d], w [H], n) of one query as the oracle sees it."""
    wl = inp["wl"]
    K = O.dequantise(inp["K"][seq], wl.k_dtype, None if inp["kscale"] is None else inp["kscale"][seq])
    qs = inp["Q"][seq, t]
    # fp8 query codes carry no scale (it is folded into W by the generator)
    q = O.dequantise(qs, wl.q_dtype, np.ones(qs.shape[:-1], np.float32) if wl.q_dtype == "e4m3" else None)
    w = inp["W"][seq, t].astype(np.float64)
    length = wl.L if inp["seq_len"] is None else int(np.clip(inp["seq_len"][seq], 0, wl.L))
    n = length if inp["q_pos"] is None else int(np.clip(int(inp["q_pos"][t]) + 1, 0, length))
    return K, q, w, n


def assert_scores_close(got, ref, what="", abs_frac=ABS_FRAC):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return
    tol = REL_TOL * np.abs(ref) + abs_frac * np.max(np.abs(ref))
    bad = np.abs(got - ref) > tol
    assert not bad.any(), (f"{what}: {bad.sum()} of {ref.size} outside tolerance; worst "
                           f"|d|={np.abs(got - ref).max():.3e} at {int(np.argmax(np.abs(got - ref)))}")


def delta_at(ref_row, value, abs_frac=ABS_FRAC):
    return REL_TOL * abs(value) + abs_frac * float(np.max(np.abs(ref_row))) if len(ref_row) else 0.0


def check_index_set(got, ref_scores, k, what="", abs_frac=ABS_FRAC):
    """Margin rule: `got` (ascending, -1 padded) must be a valid top-k of ref_scores.

    Exactly min(k, n) distinct in-range indices; every index whose reference
    score is clearly above the (k+1)-th largest must be present, none clearly
    below the k-th largest may be.  Returns True if the set equals the
    oracle's own choice exactly.
    """
    ref_scores = np.asarray(ref_scores, dtype=np.float64)
    n = ref_scores.shape[0]
    ke = min(k, n)
    got = np.asarray(got)
    assert got.shape[0] == k, what
    head, tail = got[:ke], got[ke:]
    assert np.all(tail == -1), f"{what}: padding must be -1"
    assert np.all(np.diff(head) > 0), f"{what}: indices must be strictly ascending"
    if ke == 0:
        return True
    assert head[0] >= 0 and head[-1] < n, f"{what}: index out of the visible prefix"
    exact = O.topk(ref_scores, k)
    if np.array_equal(exact, head):
        return True
    order = np.sort(ref_scores)[::-1]
    tau_in = order[ke - 1]
    tau_out = order[ke] if ke < n else -np.inf
    d_in, d_out = delta_at(ref_scores, tau_in, abs_frac), (delta_at(ref_scores, tau_out, abs_frac) if ke < n else 0.0)
    chosen = np.zeros(n, bool); chosen[head] = True
    must = ref_scores >= tau_out + 2 * d_out if ke < n else np.ones(n, bool)
    never = ref_scores <= tau_in - 2 * d_in
    assert not (must & ~chosen).any(), f"{what}: a clearly-inside index is missing"
    assert not (never & chosen).any(), f"{what}: a clearly-outside index was selected"
    return False
