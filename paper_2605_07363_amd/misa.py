"""ctypes binding of libmisa.so (see include/misa.h for the contract).

Argument marshalling only: every stage of the indexer runs in the HIP kernels
of the library.  torch is used for device memory and streams.  Importing this
module fails if the library has not been built; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmisa.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2605_07363_amd.build` "
        "(there is no fallback path)")
lib = ctypes.CDLL(LIB_PATH)

F32, BF16, FP8_E4M3, FP8_E4M3_MATRIX = 0, 1, 2, 3
# q_dtype FP8_E4M3_MATRIX: fp8 query codes that the prefill scoring kernels may contract with fp8
# keys on the fp8 matrix instruction (see "fp8 queries" in misa.h); bench.py labels its lines with it.
HAS_FP8_MFMA = True
DTYPE_CODES = {"f32": F32, "bf16": BF16, "e4m3": FP8_E4M3}
OP_POOL, OP_ROUTE, OP_SCORE, OP_TOPK, OP_RERANK, OP_SELECT, OP_HISA = range(7)
STATUS_NAMES = {0: "MISA_OK", 1: "MISA_ERR_INVALID_ARG", 2: "MISA_ERR_UNSUPPORTED",
                3: "MISA_ERR_WORKSPACE", 4: "MISA_ERR_HIP"}


class misa_problem(ctypes.Structure):
    _fields_ = [("n_seq", ctypes.c_int32), ("L", ctypes.c_int32), ("d", ctypes.c_int32),
                ("n_q", ctypes.c_int32), ("H", ctypes.c_int32), ("B", ctypes.c_int32),
                ("h", ctypes.c_int32), ("k_dtype", ctypes.c_int32), ("q_dtype", ctypes.c_int32),
                ("q_pos", ctypes.c_void_p), ("seq_len", ctypes.c_void_p),
                ("page_table", ctypes.c_void_p), ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32)]


_P = ctypes.POINTER(misa_problem)
_V = ctypes.c_void_p
lib.misa_version.restype = ctypes.c_int32
lib.misa_last_error.restype = ctypes.c_char_p
lib.misa_workspace_bytes.restype = ctypes.c_size_t
lib.misa_workspace_bytes.argtypes = [_P, ctypes.c_int32, ctypes.c_int32]
lib.misa_pool_keys.restype = ctypes.c_int
lib.misa_pool_keys.argtypes = [_P, _V, _V, _V, _V, ctypes.c_size_t, _V]
lib.misa_pool_keys_update.restype = ctypes.c_int
lib.misa_pool_keys_update.argtypes = [_P, _V, _V, _V, _V, ctypes.c_int32, _V, ctypes.c_size_t, _V]
lib.misa_route_heads.restype = ctypes.c_int
lib.misa_route_heads.argtypes = [_P, _V, _V, _V, _V, _V, _V, _V, _V, ctypes.c_size_t, _V]
lib.misa_route_heads_static.restype = ctypes.c_int
lib.misa_route_heads_static.argtypes = [_P, _V, _V, _V, _V, _V, _V, _V, _V]
lib.misa_route_heads_proxy.restype = ctypes.c_int
lib.misa_route_heads_proxy.argtypes = [_P, _V, _V, ctypes.c_int32, _V, _V, _V]
lib.misa_score_tokens.restype = ctypes.c_int
lib.misa_score_tokens.argtypes = [_P, _V, _V, _V, _V, _V, _V, _V, ctypes.c_size_t, _V]
lib.misa_topk.restype = ctypes.c_int
lib.misa_topk.argtypes = [_P, _V, ctypes.c_int32, _V, _V, _V, ctypes.c_size_t, _V]
lib.misa_select_tokens.restype = ctypes.c_int
lib.misa_select_tokens.argtypes = [_P, _V, _V, _V, _V, _V, ctypes.c_int32, _V, _V, _V, ctypes.c_size_t, _V]
lib.misa_select_row_flags_offset.restype = ctypes.c_int64
lib.misa_select_row_flags_offset.argtypes = [_P, ctypes.c_int32, ctypes.c_int32]
lib.misa_hisa_select.restype = ctypes.c_int
lib.misa_hisa_select.argtypes = [_P, _V, _V, _V, _V, _V, ctypes.c_int32, ctypes.c_int32, _V, _V, _V, _V,
                                 ctypes.c_size_t, _V]
lib.misa_block_sparse_select.restype = ctypes.c_int
lib.misa_block_sparse_select.argtypes = [_P, _V, _V, _V, ctypes.c_int32, _V, _V, _V, ctypes.c_size_t, _V]
lib.misa_convert_queries.restype = ctypes.c_int
lib.misa_convert_queries.argtypes = [_P, _V, _V, _V]
lib.misa_probe_hbm_read.restype = ctypes.c_int
lib.misa_probe_hbm_read.argtypes = [_V, ctypes.c_size_t, _V, _V]
lib.misa_probe_mfma_bf16.restype = ctypes.c_int
lib.misa_probe_mfma_bf16.argtypes = [ctypes.c_int32, ctypes.c_int32, _V, ctypes.POINTER(ctypes.c_double), _V]
lib.misa_probe_mfma_bf16_operands.restype = ctypes.c_int
lib.misa_probe_mfma_bf16_operands.argtypes = [ctypes.c_int32, ctypes.c_int32, _V, _V, ctypes.POINTER(ctypes.c_double), _V]
lib.misa_rerank.restype = ctypes.c_int
lib.misa_rerank.argtypes = [_P, _V, _V, _V, _V, _V, ctypes.c_int32, ctypes.c_int32, _V, _V, _V,
                            ctypes.c_size_t, _V]


class MisaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def _check(status: int) -> None:
    if status != 0:
        raise MisaError(status, lib.misa_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors passed to the library must be contiguous device tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(ws: Optional[torch.Tensor]):
    if ws is None:
        return None, 0
    return _ptr(ws), ws.numel() * ws.element_size()


@dataclass
class Problem:
    """Host description of one indexer problem (mirrors struct misa_problem)."""
    n_seq: int
    L: int
    n_q: int
    H: int
    B: int
    h: int
    k_dtype: int
    q_dtype: int
    q_pos: Optional[torch.Tensor] = None     # int32 device [n_q] or None (decode)
    seq_len: Optional[torch.Tensor] = None   # int32 device [n_seq] or None
    d: int = 128
    page_table: Optional[torch.Tensor] = None  # int32 device [n_seq, max_pages] or None (contiguous keys)
    page_size: int = 0

    @property
    def M(self) -> int:
        return -(-self.L // self.B)

    def c(self) -> misa_problem:
        for t in (self.q_pos, self.seq_len, self.page_table):
            if t is not None and (t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous()):
                raise ValueError("q_pos / seq_len / page_table must be contiguous int32 device tensors")
        pt = self.page_table
        if pt is not None and (pt.dim() != 2 or pt.shape[0] != self.n_seq):
            raise ValueError("page_table must have shape [n_seq, max_pages]")
        return misa_problem(self.n_seq, self.L, self.d, self.n_q, self.H, self.B, self.h,
                            self.k_dtype, self.q_dtype,
                            self.q_pos.data_ptr() if self.q_pos is not None else None,
                            self.seq_len.data_ptr() if self.seq_len is not None else None,
                            pt.data_ptr() if pt is not None else None,
                            self.page_size if pt is not None else 0,
                            pt.shape[1] if pt is not None else 0)


def version() -> int:
    return lib.misa_version()


def workspace_bytes(p: Problem, op: int, k: int = 0) -> int:
    return lib.misa_workspace_bytes(ctypes.byref(p.c()), op, k)


def alloc_workspace(p: Problem, op: int, k: int = 0, device="cuda") -> Optional[torch.Tensor]:
    n = workspace_bytes(p, op, k)
    return torch.empty(n, dtype=torch.uint8, device=device) if n else None


def pool_keys(p: Problem, K, kscale, Kp, ws=None) -> None:
    w, wb = _ws(ws)
    _check(lib.misa_pool_keys(ctypes.byref(p.c()), _ptr(K), _ptr(kscale), _ptr(Kp), w, wb, _stream()))


def pool_keys_update(p: Problem, K, kscale, Kp, from_token, max_blocks: int, ws=None) -> None:
    w, wb = _ws(ws)
    _check(lib.misa_pool_keys_update(ctypes.byref(p.c()), _ptr(K), _ptr(kscale), _ptr(Kp), _ptr(from_token),
                                     max_blocks, w, wb, _stream()))


def route_heads(p: Problem, Q, W, Kp, K, kscale, heads, E=None, ws=None) -> None:
    w, wb = _ws(ws)
    _check(lib.misa_route_heads(ctypes.byref(p.c()), _ptr(Q), _ptr(W), _ptr(Kp), _ptr(K), _ptr(kscale),
                                _ptr(heads), _ptr(E), w, wb, _stream()))


ROUTE_STATIC_SCRATCH_BYTES = 4 << 20


def route_heads_static(p: Problem, Q, W, Kp, K, kscale, heads, E=None) -> None:
    """route_heads without a workspace: scratch is an array inside the library (no allocation)."""
    _check(lib.misa_route_heads_static(ctypes.byref(p.c()), _ptr(Q), _ptr(W), _ptr(Kp), _ptr(K), _ptr(kscale),
                                       _ptr(heads), _ptr(E), _stream()))


ROUTER_BLOCK_POOLED, ROUTER_GATE, ROUTER_QUERY_NORM = range(3)


def route_heads_proxy(p: Problem, Q, W, kind: int, heads, E=None) -> None:
    _check(lib.misa_route_heads_proxy(ctypes.byref(p.c()), _ptr(Q), _ptr(W), kind, _ptr(heads), _ptr(E),
                                      _stream()))


def score_tokens(p: Problem, Q, W, heads, K, kscale, S, ws=None) -> None:
    w, wb = _ws(ws)
    _check(lib.misa_score_tokens(ctypes.byref(p.c()), _ptr(Q), _ptr(W), _ptr(heads), _ptr(K),
                                 _ptr(kscale), _ptr(S), w, wb, _stream()))


def topk(p: Problem, S, k: int, idx, val=None, ws=None) -> None:
    w, wb = _ws(ws)
    _check(lib.misa_topk(ctypes.byref(p.c()), _ptr(S), k, _ptr(idx), _ptr(val), w, wb, _stream()))


def select_tokens(p: Problem, Q, W, heads, K, kscale, k: int, idx, val=None, ws=None) -> None:
    w, wb = _ws(ws)
    _check(lib.misa_select_tokens(ctypes.byref(p.c()), _ptr(Q), _ptr(W), _ptr(heads), _ptr(K), _ptr(kscale),
                                  k, _ptr(idx), _ptr(val), w, wb, _stream()))


def select_repaired_rows(p: Problem, routed: bool, k: int, ws) -> Optional[torch.Tensor]:
    """Flags [n_seq, n_q] of the rows the last select_tokens call on `ws` recomputed by the
    two-call path, or None when the problem does not take the sampled route."""
    off = lib.misa_select_row_flags_offset(ctypes.byref(p.c()), int(routed), k)
    if off < 0:
        return None
    n = p.n_seq * p.n_q
    return ws[off:off + 4 * n].view(torch.int32).view(p.n_seq, p.n_q)


def rerank(p: Problem, Q, W, K, kscale, cand, k_cand: int, k: int, idx, val=None, ws=None) -> None:
    w, wb = _ws(ws)
    _check(lib.misa_rerank(ctypes.byref(p.c()), _ptr(Q), _ptr(W), _ptr(K), _ptr(kscale), _ptr(cand),
                           k_cand, k, _ptr(idx), _ptr(val), w, wb, _stream()))


def hisa_select(p: Problem, Q, W, Kp, K, kscale, m: int, k: int, idx, val=None, blocks=None, ws=None) -> None:
    w, wb = _ws(ws)
    _check(lib.misa_hisa_select(ctypes.byref(p.c()), _ptr(Q), _ptr(W), _ptr(Kp), _ptr(K), _ptr(kscale), m, k,
                                _ptr(blocks), _ptr(idx), _ptr(val), w, wb, _stream()))


def block_sparse_select(p: Problem, Q, W, Kp, m: int, idx, blocks=None, ws=None) -> None:
    w, wb = _ws(ws)
    _check(lib.misa_block_sparse_select(ctypes.byref(p.c()), _ptr(Q), _ptr(W), _ptr(Kp), m, _ptr(blocks),
                                        _ptr(idx), w, wb, _stream()))


def convert_queries(p: Problem, Q, Q_bf16) -> None:
    """fp8 (e4m3) query codes -> bf16 values (exact); p.q_dtype must be FP8_E4M3."""
    _check(lib.misa_convert_queries(ctypes.byref(p.c()), _ptr(Q), _ptr(Q_bf16), _stream()))


def probe_hbm_read(buf, sink, nbytes: Optional[int] = None) -> int:
    """Enqueues one read of the first nbytes bytes of buf (default: all, rounded down to 8 KiB); returns nbytes."""
    total = buf.numel() * buf.element_size()
    nbytes = (total if nbytes is None else min(nbytes, total)) // 8192 * 8192
    _check(lib.misa_probe_hbm_read(_ptr(buf), nbytes, _ptr(sink), _stream()))
    return nbytes


def probe_mfma_bf16(workgroups: int, iters: int, sink, operands=None) -> float:
    """Enqueues the matrix-instruction probe; returns its floating-point operation count.
    operands: None (constant operands) or a device tensor of 1024 bf16 (fragments a, then b, of the 64 lanes)."""
    if sink.numel() < workgroups * 256 or sink.dtype != torch.float32:
        raise ValueError("sink must hold workgroups * 256 floats")
    flops = ctypes.c_double(0.0)
    if operands is None:
        _check(lib.misa_probe_mfma_bf16(workgroups, iters, _ptr(sink), ctypes.byref(flops), _stream()))
    else:
        if operands.numel() * operands.element_size() < 2048 or not operands.is_contiguous():
            raise ValueError("operands must hold 2048 contiguous bytes")
        _check(lib.misa_probe_mfma_bf16_operands(workgroups, iters, _ptr(operands), _ptr(sink),
                                                 ctypes.byref(flops), _stream()))
    return flops.value


def measured_peaks(device="cuda", repeats: int = 10) -> dict:
    """Achievable HBM read rate (GB/s) and dense bf16 matrix rate (TFLOP/s) of this GPU, each the
    best of `repeats` event-timed bursts of launches of the library's probes (512 MiB read; ~1e13 flop).
    The matrix rate is taken twice: on the probe's constant operands, and on seeded Gaussian bf16
    operands of the workloads' scale (sigma = 1/sqrt(128)), for which the chip holds a lower clock."""
    buf = torch.empty(512 << 20, dtype=torch.uint8, device=device)
    buf.fill_(1)
    sink = torch.zeros(8 * 1024 * 256, dtype=torch.float32, device=device)
    cus = torch.cuda.get_device_properties(device).multi_processor_count
    wgs, iters = cus * 8, 2048
    g = torch.Generator(device="cpu")
    g.manual_seed(20260507)
    gauss = (torch.randn(1024, generator=g) * (128 ** -0.5)).to(torch.bfloat16).to(device)
    out = {}
    for name in ("hbm_read_GBps", "mfma_bf16_TFLOPs", "mfma_bf16_gaussian_operands_TFLOPs"):
        best = float("inf")
        amount = 0.0
        burst = 8 if name.startswith("hbm") else 2   # launches between the two events: gaps and event cost amortised
        for _ in range(repeats + 2):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(burst):
                amount = probe_hbm_read(buf, sink) if name.startswith("hbm") else \
                    probe_mfma_bf16(wgs, iters, sink, gauss if "gaussian" in name else None)
            e1.record()
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1) / burst)
        out[name] = amount / (best * 1e-3) / (1e9 if name.startswith("hbm") else 1e12)
    return out


# ---------------------------------------------------------------------------
# Plumbing helpers: device copies of generated inputs and preallocated buffers.
# ---------------------------------------------------------------------------
def to_device(inp: dict, device="cuda") -> dict:
    """Raw numpy inputs (see workloads.make_inputs) -> device tensors + Problem."""
    import numpy as np
    wl = inp["wl"]

    def dev(x, kind):
        if x is None:
            return None
        if kind == "bf16":
            return torch.from_numpy(x.view(np.int16)).to(device).view(torch.bfloat16)
        return torch.from_numpy(x).to(device)

    out = {
        "K": dev(inp["K"], wl.k_dtype), "kscale": dev(inp["kscale"], "f32"),
        "Q": dev(inp["Q"], wl.q_dtype), "W": dev(inp["W"], "f32"),
        "q_pos": dev(inp["q_pos"], "i32"), "seq_len": dev(inp["seq_len"], "i32"),
    }
    out["problem"] = Problem(wl.n_seq, wl.L, wl.n_q, wl.H, wl.B, wl.h, DTYPE_CODES[wl.k_dtype],
                             DTYPE_CODES[wl.q_dtype], out["q_pos"], out["seq_len"])
    return out


def paginate(dv: dict, page_size: int, seed: int = 0, spare_pages: int = 3) -> dict:
    """The same inputs with the key cache laid out as a page pool.

    Every sequence's keys are cut into pages of page_size tokens that are scattered over a pool
    [n_pages, page_size, d] by a seeded permutation (a few pages of the pool stay unused); pool
    rows that hold no key are filled with a bit pattern no key has.  Returns a copy of dv with K /
    kscale replaced by the pools and problem.page_table / page_size set.
    """
    from dataclasses import replace
    p = dv["problem"]
    K, ks = dv["K"], dv["kscale"]
    per_seq = -(-p.L // page_size)
    n_pages = p.n_seq * per_seq + spare_pages
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    table = torch.randperm(n_pages, generator=g)[: p.n_seq * per_seq].to(torch.int32).view(p.n_seq, per_seq)
    table = table.to(K.device)
    pad = per_seq * page_size - p.L
    fill = {torch.uint8: 0x7E, torch.bfloat16: 1.0e30, torch.float32: 1.0e30}[K.dtype]

    def pool_of(x, fillv):
        tail = x.shape[2:]
        padded = torch.full((p.n_seq, per_seq * page_size) + tail, fillv, dtype=x.dtype, device=x.device)
        padded[:, : p.L] = x
        pool = torch.full((n_pages, page_size) + tail, fillv, dtype=x.dtype, device=x.device)
        pool[table.view(-1).long()] = padded.view((p.n_seq * per_seq, page_size) + tail)
        return pool.contiguous()

    out = dict(dv)
    out["K"] = pool_of(K, fill)
    out["kscale"] = None if ks is None else pool_of(ks, 1.0e30)
    out["problem"] = replace(p, page_table=table.contiguous(), page_size=page_size)
    return out


class Indexer:
    """Preallocated outputs + workspaces for one problem; runs the stages in order."""

    def __init__(self, p: Problem, k: int, k_cand: int = 0, device="cuda", want_E=False, want_val=False,
                 fused=False):
        """fused: stages 3 and 4 run as one select_tokens call and no score matrix is kept."""
        self.p, self.k, self.k_cand, self.fused = p, k, k_cand, fused
        self.p_score = None     # problem description of the scoring calls when it differs from p (fp8 codes)
        rows = (p.n_seq, p.n_q)
        self.Kp = torch.empty((p.n_seq, p.M, p.d), dtype=torch.float32, device=device)
        self.heads = torch.empty(rows + (p.h,), dtype=torch.int32, device=device)
        self.E = torch.empty(rows + (p.H,), dtype=torch.float32, device=device) if want_E else None
        self.S = None if fused else torch.empty(rows + (p.L,), dtype=torch.float32, device=device)
        k1 = k_cand if k_cand else k
        self.idx1 = torch.empty(rows + (k1,), dtype=torch.int32, device=device)
        self.val1 = torch.empty(rows + (k1,), dtype=torch.float32, device=device) if want_val else None
        self.idx = self.idx1
        self.val = self.val1
        if k_cand:
            self.idx = torch.empty(rows + (k,), dtype=torch.int32, device=device)
            self.val = torch.empty(rows + (k,), dtype=torch.float32, device=device) if want_val else None
        self.ws = {op: alloc_workspace(p, op, k1 if op == OP_TOPK else k_cand, device)
                   for op in (OP_POOL, OP_ROUTE, OP_SCORE, OP_TOPK, OP_RERANK)
                   if (op != OP_RERANK or k_cand) and not (fused and op == OP_TOPK)}
        if fused:
            self.ws[OP_SELECT] = alloc_workspace(p, OP_SELECT, k1, device)

    def pool(self, K, kscale):
        pool_keys(self.p, K, kscale, self.Kp, self.ws[OP_POOL])

    def pool_update(self, K, kscale, from_token, max_blocks=1):
        pool_keys_update(self.p, K, kscale, self.Kp, from_token, max_blocks, self.ws[OP_POOL])

    def route(self, Q, W, K, kscale):
        route_heads(self.p, Q, W, self.Kp, K, kscale, self.heads, self.E, self.ws[OP_ROUTE])

    def score(self, Q, W, K, kscale, dense=False):
        score_tokens(self.p_score or self.p, Q, W, None if dense else self.heads, K, kscale, self.S, self.ws[OP_SCORE])

    def select(self):
        topk(self.p, self.S, self.k_cand if self.k_cand else self.k, self.idx1, self.val1,
             self.ws[OP_TOPK])

    def select_fused(self, Q, W, K, kscale, dense=False):
        select_tokens(self.p_score or self.p, Q, W, None if dense else self.heads, K, kscale,
                      self.k_cand if self.k_cand else self.k, self.idx1, self.val1, self.ws[OP_SELECT])

    def refine(self, Q, W, K, kscale):
        rerank(self.p_score or self.p, Q, W, K, kscale, self.idx1, self.k_cand, self.k, self.idx, self.val,
               self.ws[OP_RERANK])

    def run(self, K, kscale, Q, W, pool=True):
        """One pass of the whole indexer; returns the selected token indices.  fp8 queries are
        widened to bf16 once here instead of inside each of the stage calls; with q_dtype
        FP8_E4M3_MATRIX the scoring stage still gets the codes (fp8 matrix instruction)."""
        if self.p.q_dtype not in (FP8_E4M3, FP8_E4M3_MATRIX):
            return self._run(K, kscale, Q, W, Q, pool)
        if getattr(self, "_q16", None) is None:
            from dataclasses import replace
            self._q16 = torch.empty(Q.shape, dtype=torch.bfloat16, device=Q.device)
            self._p16 = replace(self.p, q_dtype=BF16)
        convert_queries(self.p, Q, self._q16)
        p8, self.p = self.p, self._p16          # the stage methods below read self.p
        codes = p8.q_dtype == FP8_E4M3_MATRIX
        self.p_score = p8 if codes else None
        try:
            return self._run(K, kscale, self._q16, W, Q if codes else self._q16, pool)
        finally:
            self.p, self.p_score = p8, None

    def _run(self, K, kscale, Q, W, Q_score, pool):
        if pool:
            self.pool(K, kscale)
        self.route(Q, W, K, kscale)
        if self.fused:
            self.select_fused(Q_score, W, K, kscale)
        else:
            self.score(Q_score, W, K, kscale)
            self.select()
        if self.k_cand:
            self.refine(Q_score, W, K, kscale)
        return self.idx
