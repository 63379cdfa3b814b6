"""Plain fp64 CPU oracle of the MISA indexer.  TEST INFRASTRUCTURE ONLY.

This module is the slow, obviously-correct statement of what the indexer
computes.  It is written from the paper's equations, in the paper's order
and notation, in numpy float64.  It shares no code, table or helper with the
HIP path and must never be imported by the product path.

Notation (paper, Preliminaries and Method sections)
    L        causal prefix length of one query (here: ``n``; the query at
             0-based position p sees keys 0..p inclusive, so n = p + 1)
    k_s      indexing key of prefix token s, shape [d]
    q_{t,j}  indexing query of query t, head j (H^I heads; here ``H``)
    w_{t,j}  gate of head j
    B, M     router block size, M = ceil(n / B) pooled keys
    h        number of active heads,  k  token budget,  k' candidate budget

Every function works on ONE query of ONE sequence and takes already
de-quantised float64 arrays (see ``dequantise``); the ``*_batch`` wrappers
only loop.

Readings taken where the paper is silent (each is also listed in the design
notes of the repository):
  * Pool is the arithmetic mean; a partial last block is averaged over the
    tokens it actually holds.
  * The partition into blocks is per query: query p pools exactly its own
    prefix 0..p, so no pooled key ever contains a future token.
  * TopK ties go to the lower index, for heads and for tokens; -0.0 == +0.0.
  * If fewer than k tokens are visible, all of them are returned.
  * FP8 keys are OCP e4m3fn codes with one fp32 scale per token:
    k_s = scale_s * decode(code_s).

Parity status: every function below is pinned by tests/test_oracle_*.py
(hand-worked fixture, closed forms, invariants, library special cases, brute
force).  The *approximation quality* of MISA against the paper's LongBench /
NIAH / IoU numbers is "parity unpinned": those need model weights and
datasets that are not available.
"""
from __future__ import annotations

import math
import numpy as np

__all__ = [
    "e4m3fn_decode_table", "bf16_bits_to_f64", "dequantise",
    "pool_keys", "route_affinity", "route_heads", "route_heads_proxy", "score_tokens", "dsa_scores",
    "topk", "rerank", "misa", "misa_dagger", "dsa_dense", "iou", "recall",
    "head_token_products", "block_scores", "select_blocks", "block_tokens", "hisa", "block_sparse",
]


# --------------------------------------------------------------------------
# Input decoding (not part of the method: turns stored bit patterns into the
# real numbers they stand for, exactly).
# --------------------------------------------------------------------------
def e4m3fn_decode_table() -> np.ndarray:
    """All 256 values of the OCP FP8 E4M3 ("e4m3fn") format as float64.

    1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits.  Exponent field 0
    is subnormal: (m/8) * 2**-6.  There is no infinity; S.1111.111 is NaN, so
    the largest finite magnitude is 1.75 * 2**8 = 448.
    """
    tab = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            tab[code] = math.nan
        elif e == 0:
            tab[code] = sign * (m / 8.0) * 2.0 ** -6
        else:
            tab[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return tab


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64, exactly.

    bfloat16 is the upper half of an IEEE binary32 word.
    """
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def dequantise(x: np.ndarray, dtype: str, scale: np.ndarray | None = None) -> np.ndarray:
    """Stored tensor -> float64 real values.

    dtype 'f32'  : x is float32.
    dtype 'bf16' : x is uint16 bit patterns.
    dtype 'e4m3' : x is uint8 codes [..., d]; scale is float32 [...] (one per
                   token); value = scale * decode(code).
    """
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f64(x)
    if dtype == "e4m3":
        if scale is None:
            raise ValueError("e4m3 keys need a per-token scale")
        vals = e4m3fn_decode_table()[np.asarray(x, dtype=np.uint8)]
        return vals * np.asarray(scale, dtype=np.float32).astype(np.float64)[..., None]
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------
# Stage 1: block mean pooling  (Eq. pool; reused by the MISA router)
# --------------------------------------------------------------------------
def pool_keys(K: np.ndarray, B: int, n: int | None = None) -> np.ndarray:
    """Pooled keys of the prefix K[0:n], shape [ceil(n/B), d].

    Block b holds tokens b*B .. min((b+1)*B, n) - 1 and is summarised by the
    arithmetic mean of its keys (Eq. pool, "mean pooling").
    """
    K = np.asarray(K, dtype=np.float64)
    n = K.shape[0] if n is None else int(n)
    if B < 1 or n < 0 or n > K.shape[0]:
        raise ValueError("bad B or n")
    M = -(-n // B)
    Kp = np.zeros((M, K.shape[1]), dtype=np.float64)
    for b in range(M):
        lo, hi = b * B, min((b + 1) * B, n)
        Kp[b] = K[lo:hi].sum(axis=0) / float(hi - lo)
    return Kp


# --------------------------------------------------------------------------
# Stage 2: block-pooled router  (Eq. misa_route_score, Eq. misa_route)
# --------------------------------------------------------------------------
def route_affinity(q: np.ndarray, w: np.ndarray, Kp: np.ndarray) -> np.ndarray:
    """A[j, b] = w_j * ReLU(q_j . k~_b)   (Eq. misa_route_score, left part)."""
    q = np.asarray(q, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    return w[:, None] * np.maximum(q @ Kp.T, 0.0)


def _top_by_value_then_index(values: np.ndarray, count: int) -> np.ndarray:
    """Indices of the ``count`` largest values; equal values -> lower index.

    Returned in ascending index order (the result is a set).
    """
    values = np.asarray(values, dtype=np.float64) + 0.0  # -0.0 -> +0.0
    n = values.shape[0]
    count = min(int(count), n)
    order = sorted(range(n), key=lambda i: (-values[i], i))
    return np.array(sorted(order[:count]), dtype=np.int64)


def route_heads(q, w, K, B: int, h: int, n: int | None = None):
    """Active head set H_t and head importances E  (Eq. misa_route).

    The visible prefix K[0:n] is pooled into M = ceil(n/B) keys; then
    E_j = (1/M) * sum_b |A[j, b]| and the h heads with the largest E are kept.
    Returns (heads ascending int64 [h], E float64 [H]).  With an empty prefix
    (n = 0) there is no block, E = 0 and the tie rule picks heads 0..h-1.
    """
    q = np.asarray(q, dtype=np.float64)
    H = q.shape[0]
    if not 1 <= h <= H:
        raise ValueError("h must be in 1..H")
    Kp = pool_keys(K, B, n)
    M = Kp.shape[0]
    if M == 0:
        E = np.zeros(H, dtype=np.float64)
    else:
        A = route_affinity(q, w, Kp)
        E = np.abs(A).sum(axis=1) / float(M)
    return _top_by_value_then_index(E, h), E


def route_heads_proxy(q, w, h: int, kind: str):
    """Head sets of the two content-free router scores of the appendix "Ablation: routing
    score": kind 'gate' ranks heads by the gating weight w_j as it is, kind 'qnorm' by the
    Euclidean norm of q_j.  Returns (heads ascending int64 [h], E float64 [H])."""
    q = np.asarray(q, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    if not 1 <= h <= q.shape[0]:
        raise ValueError("h must be in 1..H")
    if kind == "gate":
        E = w.copy()
    elif kind == "qnorm":
        E = np.sqrt((q * q).sum(axis=1))
    else:
        raise ValueError("kind must be 'gate' or 'qnorm'")
    return _top_by_value_then_index(E, h), E


# --------------------------------------------------------------------------
# Stage 3: token scoring with the active heads  (Eq. misa_score; Eq. dsa_score)
# --------------------------------------------------------------------------
def score_tokens(q, w, heads, K, n: int | None = None) -> np.ndarray:
    """I^[s] = sum_{j in heads} w_j * ReLU(q_j . k_s) for s in 0..n-1."""
    q = np.asarray(q, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    n = K.shape[0] if n is None else int(n)
    heads = np.asarray(heads, dtype=np.int64)
    if len(set(heads.tolist())) != heads.shape[0]:
        raise ValueError("heads must be distinct")
    out = np.zeros(n, dtype=np.float64)
    for j in heads:
        out += w[j] * np.maximum(K[:n] @ q[j], 0.0)
    return out


def dsa_scores(q, w, K, n: int | None = None) -> np.ndarray:
    """Dense DSA indexer score I[s] with all H^I heads  (Eq. dsa_score)."""
    return score_tokens(q, w, np.arange(np.asarray(q).shape[0]), K, n)


# --------------------------------------------------------------------------
# Stage 4: top-k  (Eq. dsa_topk, Eq. misa_topk, Eq. misa_candidate)
# --------------------------------------------------------------------------
def topk(scores: np.ndarray, k: int) -> np.ndarray:
    """The min(k, n) best tokens of a score row, ascending index order."""
    if k < 1:
        raise ValueError("k must be >= 1")
    return _top_by_value_then_index(scores, k)


# --------------------------------------------------------------------------
# Stage 5: MISA-dagger fine stage  (Eq. misa_final_topk)
# --------------------------------------------------------------------------
def rerank(q, w, K, cand, k: int, n: int | None = None):
    """Re-score the candidate set with all H^I heads and keep the best k.

    ``cand`` holds distinct visible token indices; entries < 0 (padding) or
    >= n are ignored.  Ties go to the lower token index.  Returns
    (tokens ascending, their dense scores).
    """
    K = np.asarray(K, dtype=np.float64)
    n = K.shape[0] if n is None else int(n)
    cand = np.asarray(cand, dtype=np.int64)
    cand = np.array(sorted(c for c in cand.tolist() if 0 <= c < n), dtype=np.int64)
    if len(set(cand.tolist())) != cand.shape[0]:
        raise ValueError("candidates must be distinct")
    dense = dsa_scores(q, w, K, n)            # I[s] for the whole prefix ...
    sub = dense[cand]                          # ... restricted to Omega_t
    keep = _top_by_value_then_index(sub, k)    # ascending position == ascending token
    return cand[keep], sub[keep]


# --------------------------------------------------------------------------
# Comparison indexers built from the same parts: HISA (preliminaries, "Indexer
# in HISA", Eq. block_score and Eq. final_topk) and the MoBA-style Block-Sparse
# selector (Experimental results, "Baselines")
# --------------------------------------------------------------------------
def block_scores(q, w, K, B: int, n: int | None = None) -> np.ndarray:
    """J[b] = sum over all heads of w_j * ReLU(q_j . k~_b) for the M = ceil(n/B) pooled
    keys of the visible prefix (Eq. block_score, left part)."""
    Kp = pool_keys(K, B, n)
    if Kp.shape[0] == 0:
        return np.zeros(0, dtype=np.float64)
    return route_affinity(q, w, Kp).sum(axis=0)


def select_blocks(J: np.ndarray, m: int) -> np.ndarray:
    """C = the first and the last block plus the best-scoring other blocks, m blocks in
    all (every block if there are at most m); ties to the lower index; ascending
    (Eq. block_score, right part, with the always-included first and last block)."""
    J = np.asarray(J, dtype=np.float64)
    M = J.shape[0]
    if m < 2:
        raise ValueError("m must be >= 2 (the first and the last block are always kept)")
    if M <= m:
        return np.arange(M, dtype=np.int64)
    forced = [0, M - 1]
    rest = [b for b in range(M) if b not in forced]
    best = _top_by_value_then_index(J[rest], m - len(forced))
    return np.array(sorted(forced + [rest[i] for i in best.tolist()]), dtype=np.int64)


def block_tokens(blocks: np.ndarray, B: int, n: int) -> np.ndarray:
    """Omega = the visible tokens of the given blocks, ascending."""
    out = [s for b in np.asarray(blocks).tolist() for s in range(b * B, min((b + 1) * B, n))]
    return np.array(out, dtype=np.int64)


def hisa(q, w, K, B: int, m: int, k: int, n: int | None = None) -> dict:
    """HISA indexer: top-m blocks by the all-head block score, then the dense indexer score
    inside those blocks and its top-k (Eq. block_score, Eq. final_topk)."""
    n = np.asarray(K).shape[0] if n is None else int(n)
    J = block_scores(q, w, K, B, n)
    if n == 0:
        return {"J": J, "blocks": np.zeros(0, np.int64), "tokens": np.zeros(0, np.int64),
                "values": np.zeros(0)}
    C = select_blocks(J, m)
    tokens, vals = rerank(q, w, K, block_tokens(C, B, n), k, n)
    return {"J": J, "blocks": C, "tokens": tokens, "values": vals}


def block_sparse(q, w, K, B: int, m: int, n: int | None = None) -> dict:
    """Block-Sparse selector: the tokens of the m selected blocks are the selection."""
    n = np.asarray(K).shape[0] if n is None else int(n)
    J = block_scores(q, w, K, B, n)
    if n == 0:
        return {"J": J, "blocks": np.zeros(0, np.int64), "tokens": np.zeros(0, np.int64)}
    C = select_blocks(J, m)
    return {"J": J, "blocks": C, "tokens": block_tokens(C, B, n)}


# --------------------------------------------------------------------------
# Whole pipelines for one query
# --------------------------------------------------------------------------
def misa(q, w, K, B: int, h: int, k: int, n: int | None = None) -> dict:
    """Single-stage MISA: route -> score -> top-k."""
    n = np.asarray(K).shape[0] if n is None else int(n)
    heads, E = route_heads(q, w, K, B, h, n)
    s = score_tokens(q, w, heads, K, n)
    return {"heads": heads, "E": E, "scores": s, "tokens": topk(s, k) if n else np.zeros(0, np.int64)}


def misa_dagger(q, w, K, B: int, h: int, k_cand: int, k: int, n: int | None = None) -> dict:
    """Hierarchical MISA: routed pass keeps k' candidates, dense re-rank keeps k."""
    if k_cand < k:
        raise ValueError("k' must be >= k")
    n = np.asarray(K).shape[0] if n is None else int(n)
    first = misa(q, w, K, B, h, k_cand, n)
    tokens, vals = rerank(q, w, K, first["tokens"], k, n)
    return {"heads": first["heads"], "E": first["E"], "scores": first["scores"],
            "candidates": first["tokens"], "tokens": tokens, "values": vals}


def dsa_dense(q, w, K, k: int, n: int | None = None) -> dict:
    """The dense DSA indexer (Eq. dsa_score + Eq. dsa_topk)."""
    s = dsa_scores(q, w, K, n)
    return {"scores": s, "tokens": topk(s, k) if s.shape[0] else np.zeros(0, np.int64)}


# --------------------------------------------------------------------------
# Metrics and the cost model
# --------------------------------------------------------------------------
def iou(a, b) -> float:
    """Intersection over union of two token sets (Eq. iou)."""
    a, b = set(np.asarray(a).tolist()), set(np.asarray(b).tolist())
    return len(a & b) / len(a | b) if (a | b) else 1.0


def recall(selected, reference) -> float:
    """Fraction of the reference set that was selected."""
    s, r = set(np.asarray(selected).tolist()), set(np.asarray(reference).tolist())
    return len(s & r) / len(r) if r else 1.0


def head_token_products(n: int, H: int, h: int, B: int, k_cand: int = 0) -> dict:
    """Head-token products per query: dense H*n, MISA h*n + H*M (+ k'*H)."""
    M = -(-n // B)
    return {"dense": H * n, "misa": h * n + H * M + min(k_cand, n) * H}
