"""Seeded synthetic indexer inputs shaped like the paper's workloads.

This module only *draws inputs*: random keys, queries and gates with the
shapes of the DeepSeek-V3.2 (H^I = 64) and GLM-5 (H^I = 32) indexers
(Experimental results, "Models" and "Default MISA hyperparameters"), rounded
to the storage type of each configuration.  It contains none of the method's
arithmetic (no pooling, routing, scoring or selection) and is used both by the
CPU oracle's tests and by the HIP path's tests and benchmark, so that both see
the same bytes.

Raw storage convention (numpy, host):
    'f32'  -> float32 array
    'bf16' -> uint16 array of bfloat16 bit patterns
    'e4m3' -> uint8 array of OCP FP8 E4M3 codes + one float32 scale per token
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

BASE_SEED = 20260507


@dataclass(frozen=True)
class Workload:
    name: str
    n_seq: int
    L: int            # keys per sequence
    n_q: int          # queries per sequence
    H: int            # indexer heads H^I
    h: int            # active heads
    B: int            # router block size
    k: int            # final token budget
    k_cand: int       # MISA-dagger candidate budget k' (0 = single stage)
    k_dtype: str      # 'f32' | 'bf16' | 'e4m3'
    q_dtype: str      # 'f32' | 'bf16' | 'e4m3' (codes; the per-(query, head) scale is folded into W)
    decode: bool      # True: one query at the last position, q_pos = None
    structure: str    # 'iid' | 'topic'
    needles: int      # planted needle keys per sequence
    d: int = 128
    cfg_id: int = 0

    @property
    def M(self) -> int:
        return -(-self.L // self.B)

    @property
    def q_pos0(self) -> int:
        return self.L - self.n_q

    def pairs(self) -> int:
        """Query-key pairs scored per pass (visible prefix tokens over all queries)."""
        if self.decode:
            return self.n_seq * self.L
        return self.n_seq * sum(self.q_pos0 + t + 1 for t in range(self.n_q))


WORKLOADS = {
    # Tiny decode, all fp32.
    "c0": Workload("c0", 1, 4096, 1, 64, 8, 64, 256, 0, "f32", "f32", True, "iid", 16, cfg_id=0),
    # Batched decode, bf16 keys and queries.
    "c1": Workload("c1", 64, 32768, 1, 64, 8, 64, 2048, 0, "bf16", "bf16", True, "iid", 64, cfg_id=1),
    # Prefill chunk, DeepSeek-V3.2-shaped.
    "c2": Workload("c2", 1, 65536, 4096, 64, 8, 64, 2048, 0, "bf16", "bf16", False, "topic", 0, cfg_id=2),
    # Long decode, GLM-5-shaped, fp8 keys.
    "c3": Workload("c3", 32, 131072, 1, 32, 8, 128, 2048, 0, "e4m3", "bf16", True, "topic", 256, cfg_id=3),
    # MISA-dagger hierarchical prefill, fp8 keys.
    "c4": Workload("c4", 1, 131072, 2048, 64, 8, 64, 2048, 8192, "e4m3", "bf16", False, "topic", 256, cfg_id=4),
}


def scaled(wl: Workload, **kw) -> Workload:
    """A smaller twin of a workload (same structure, other sizes)."""
    return replace(wl, **kw)


# ---------------------------------------------------------------------------
# storage rounding (input preparation only)
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantise_e4m3(x: np.ndarray):
    """Per-token FP8 quantisation: scale = max|x| / 448, codes = RNE(x / scale).

    Returns (uint8 codes [..., d], float32 scale [...]).  Uses torch's
    float8_e4m3fn cast for the rounding.
    """
    import torch
    x = np.ascontiguousarray(x, dtype=np.float32)
    amax = np.abs(x).max(axis=-1)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    y = np.clip(x / scale[..., None], -448.0, 448.0).astype(np.float32)
    codes = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    return codes, scale


def _store(x: np.ndarray, dtype: str):
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32), None
    if dtype == "bf16":
        return f32_to_bf16_bits(x), None
    if dtype == "e4m3":
        return quantise_e4m3(x)
    raise ValueError(dtype)


def stored_to_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    """Stored queries -> the float32 values they represent (used to build needles; fp8 codes
    without their scale, which does not change a direction)."""
    if dtype == "f32":
        return x
    if dtype == "e4m3":
        import torch
        return torch.from_numpy(np.ascontiguousarray(x)).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    return bf16_bits_to_f32(x)


# ---------------------------------------------------------------------------
# generators
# ---------------------------------------------------------------------------
TOPICS = 8
TOPIC_SEGMENT = 2048      # prefix tokens per topic segment
TOPIC_QUERY_RUN = 512     # consecutive queries sharing a topic
TOPIC_KEY_AMPL = 0.5      # a: key = g/sqrt(d) + a * u_topic
TOPIC_QUERY_AMPL = 0.3145  # b: cos(q, u_topic) ~ 0.3 on the matching heads
NEEDLE_GAIN = 4.0


def make_inputs(wl: Workload, seed: int | None = None, seq_len=None) -> dict:
    """Draw one batch of inputs for ``wl``.

    Returns a dict with K, kscale (or None), Q, W, q_pos (int32 [n_q] or None
    for decode), seq_len (int32 [n_seq] or None), and the workload itself.
    """
    seed = BASE_SEED + 1000 * wl.cfg_id if seed is None else seed
    rng = np.random.default_rng(seed)
    d, H, L, nq = wl.d, wl.H, wl.L, wl.n_q
    inv_sqrt_d = np.float32(1.0 / np.sqrt(d))

    topics = None
    if wl.structure == "topic":
        u = rng.standard_normal((TOPICS, d)).astype(np.float32)
        topics = u / np.linalg.norm(u, axis=1, keepdims=True)

    Ks, scales, Qs, Ws = [], [], [], []
    for _ in range(wl.n_seq):
        # queries and gates
        q = rng.standard_normal((nq, H, d), dtype=np.float32) * inv_sqrt_d
        w = (rng.standard_normal((nq, H)) / np.sqrt(H)).astype(np.float32)
        if topics is not None:
            n_runs = -(-nq // TOPIC_QUERY_RUN)
            q_topic = np.repeat(rng.integers(0, TOPICS, n_runs), TOPIC_QUERY_RUN)[:nq]
            home = np.arange(H) % TOPICS
            match = (home[None, :] == q_topic[:, None])             # [nq, H]
            q += (np.float32(TOPIC_QUERY_AMPL) * match[:, :, None]) * topics[q_topic][:, None, :]
        q_st, q_sc = _store(q, wl.q_dtype)
        if wl.q_dtype == "e4m3":
            # fp8 queries carry no scale array: w ReLU((c q).k) = (c w) ReLU(q.k) for c > 0, so the
            # per-(query, head) scale goes into the gate (this product is input data for both sides)
            w = (w * q_sc).astype(np.float32)
        q_val = stored_to_f32(q_st, wl.q_dtype)

        # keys
        k = rng.standard_normal((L, d), dtype=np.float32) * inv_sqrt_d
        if topics is not None:
            n_seg = -(-L // TOPIC_SEGMENT)
            k_topic = np.repeat(rng.integers(0, TOPICS, n_seg), TOPIC_SEGMENT)[:L]
            k += np.float32(TOPIC_KEY_AMPL) * topics[k_topic]
        if wl.needles:
            # 4 needle heads per sequence, taken among the heads whose gate is
            # positive for the last query (a negative gate would push a needle
            # *down* the ranking); needle i is aligned with head J[i % 4] of a
            # random query.
            positive = np.flatnonzero(w[nq - 1] > 0)
            pool = positive if positive.size >= 4 else np.arange(H)
            J = rng.choice(pool, size=min(4, pool.size), replace=False)
            pos = rng.choice(L, size=min(wl.needles, L), replace=False)
            for i, s in enumerate(pos):
                t = int(rng.integers(0, nq))
                v = q_val[t, int(J[i % J.size])]
                k[s] = np.float32(NEEDLE_GAIN) * v / np.linalg.norm(v)
        k_st, k_sc = _store(k, wl.k_dtype)
        Ks.append(k_st); scales.append(k_sc); Qs.append(q_st); Ws.append(w)

    out = {
        "wl": wl,
        "K": np.stack(Ks),
        "kscale": np.stack(scales) if wl.k_dtype == "e4m3" else None,
        "Q": np.stack(Qs),
        "W": np.stack(Ws),
        "q_pos": None if wl.decode else (wl.q_pos0 + np.arange(nq)).astype(np.int32),
        "seq_len": None if seq_len is None else np.asarray(seq_len, dtype=np.int32),
    }
    return out
