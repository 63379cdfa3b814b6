"""Every call must stay inside the workspace size misa_workspace_bytes reports: the workspace is
cut out of a larger buffer whose surroundings are filled with a pattern that must survive."""
import numpy as np
import pytest

from paper_2605_07363_amd import workloads as WL

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
GUARD = 1 << 16


@pytest.fixture(scope="module")
def misa():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2605_07363_amd import misa as m
    return m


class Guarded:
    def __init__(self, misa, p, op, k=0):
        self.n = misa.workspace_bytes(p, op, k)
        self.buf = torch.full((self.n + 2 * GUARD,), 0xA5, dtype=torch.uint8, device="cuda")
        self.ws = self.buf[GUARD:GUARD + self.n] if self.n else None

    def check(self, what):
        torch.cuda.synchronize()
        assert bool((self.buf[:GUARD] == 0xA5).all()), f"{what}: wrote below its workspace"
        assert bool((self.buf[GUARD + self.n:] == 0xA5).all()), f"{what}: wrote past its workspace ({self.n} bytes)"


class Outputs:
    """Output tensors cut out of pattern-filled buffers; check() verifies the surroundings."""

    def __init__(self):
        self.items = []

    def new(self, shape, dtype, what):
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        buf = torch.full((n + 2 * GUARD,), 0xA5, dtype=torch.uint8, device="cuda")
        self.items.append((buf, n, what))
        return buf[GUARD:GUARD + n].view(dtype).view(shape)

    def check(self):
        torch.cuda.synchronize()
        for buf, n, what in self.items:
            assert bool((buf[:GUARD] == 0xA5).all()) and bool((buf[GUARD + n:] == 0xA5).all()), \
                f"a kernel wrote outside the output {what}"


CASES = {
    "decode_long_rows": WL.scaled(WL.WORKLOADS["c3"], n_seq=3, L=70000, k=2048, needles=16),
    "decode_fp8_queries": WL.scaled(WL.WORKLOADS["c1"], n_seq=2, L=40000, k=300, q_dtype="e4m3"),
    "prefill_fused": WL.scaled(WL.WORKLOADS["c4"], L=9000, n_q=70, k=128, k_cand=2048, needles=16),
    "prefill_fp8_queries": WL.scaled(WL.WORKLOADS["c2"], L=8192, n_q=100, k=2048, q_dtype="e4m3"),
    "sliced_pooling": WL.scaled(WL.WORKLOADS["c3"], n_seq=2, L=9000, B=4000, k=64, needles=4),
    "fp32": WL.scaled(WL.WORKLOADS["c0"], L=3000, B=64, k=100),
}


@pytest.mark.parametrize("name", list(CASES))
def test_calls_stay_inside_their_workspace(misa, name):
    wl = CASES[name]
    dv = misa.to_device(WL.make_inputs(wl, seed=3))
    p = dv["problem"]
    K, ks, Q, W = dv["K"], dv["kscale"], dv["Q"], dv["W"]
    rows = (wl.n_seq, wl.n_q)
    out = Outputs()
    Kp = out.new((wl.n_seq, p.M, wl.d), torch.float32, "Kp")
    g = Guarded(misa, p, misa.OP_POOL)
    misa.pool_keys(p, K, ks, Kp, g.ws)
    g.check("pool_keys")
    start = torch.zeros(wl.n_seq, dtype=torch.int32, device="cuda")
    misa.pool_keys_update(p, K, ks, Kp, start, p.M, g.ws)
    g.check("pool_keys_update")
    heads = out.new(rows + (wl.h,), torch.int32, "heads")
    g = Guarded(misa, p, misa.OP_ROUTE)
    misa.route_heads(p, Q, W, Kp, K, ks, heads, None, g.ws)
    g.check("route_heads")
    S = out.new(rows + (wl.L,), torch.float32, "S")
    g = Guarded(misa, p, misa.OP_SCORE)
    misa.score_tokens(p, Q, W, heads, K, ks, S, g.ws)
    g.check("score_tokens")
    k1 = wl.k_cand or wl.k
    idx1 = out.new(rows + (k1,), torch.int32, "idx (topk)")
    g = Guarded(misa, p, misa.OP_TOPK, k1)
    misa.topk(p, S, k1, idx1, None, g.ws)
    g.check("topk")
    g = Guarded(misa, p, misa.OP_SELECT, k1)
    idx2 = out.new(rows + (k1,), torch.int32, "idx (select_tokens)")
    misa.select_tokens(p, Q, W, heads, K, ks, k1, idx2, None, g.ws)
    g.check("select_tokens")
    assert torch.equal(idx1, idx2)
    k2 = min(wl.k, k1)
    fin = out.new(rows + (k2,), torch.int32, "idx (rerank)")
    g = Guarded(misa, p, misa.OP_RERANK, k1)
    misa.rerank(p, Q, W, K, ks, idx1, k1, k2, fin, None, g.ws)
    g.check("rerank")
    m = max(2, min(16384 // wl.B, 12))
    kh = min(wl.k, m * wl.B)
    hidx = out.new(rows + (kh,), torch.int32, "idx (hisa)")
    g = Guarded(misa, p, misa.OP_HISA, m)
    misa.hisa_select(p, Q, W, Kp, K, ks, m, kh, hidx, None, None, g.ws)
    g.check("hisa_select")
    bidx = out.new(rows + (m * wl.B,), torch.int32, "idx (block sparse)")
    misa.block_sparse_select(p, Q, W, Kp, m, bidx, None, g.ws)
    g.check("block_sparse_select")
    out.check()
