"""misa_route_heads_static (the entry point that allocates nothing) against misa_route_heads:
same inputs, same pooled keys, two calls in a row on the shared scratch array, the second
with a smaller problem; then the oracle on the smaller one."""
import ctypes

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


def _route_both(misa, wl, seed):
    inp = WL.make_inputs(wl, seed=seed)
    dv = misa.to_device(inp)
    p = dv["problem"]
    Kp = torch.empty((wl.n_seq, p.M, wl.d), dtype=torch.float32, device="cuda")
    misa.pool_keys(p, dv["K"], dv["kscale"], Kp, misa.alloc_workspace(p, misa.OP_POOL))
    shape = (wl.n_seq, wl.n_q)
    heads_ws = torch.full(shape + (wl.h,), -5, dtype=torch.int32, device="cuda")
    E_ws = torch.full(shape + (wl.H,), -5.0, dtype=torch.float32, device="cuda")
    misa.route_heads(p, dv["Q"], dv["W"], Kp, dv["K"], dv["kscale"], heads_ws, E_ws,
                     misa.alloc_workspace(p, misa.OP_ROUTE))
    heads_st = torch.full_like(heads_ws, -7)
    E_st = torch.full_like(E_ws, -7.0)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    misa.route_heads_static(p, dv["Q"], dv["W"], Kp, dv["K"], dv["kscale"], heads_st, E_st)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(heads_st, heads_ws), f"{wl.name}: head sets differ from misa_route_heads"
    assert torch.equal(E_st, E_ws), f"{wl.name}: importances differ from misa_route_heads"
    return inp, heads_st.cpu().numpy(), E_st.cpu().numpy()


def test_route_heads_static_two_calls_second_smaller(misa):
    # decode batch (per-wavefront router), then a smaller causal prefill chunk with partial last
    # blocks and fp8 queries (tiled router, query staging at the head of the scratch array)
    big = WL.scaled(WL.WORKLOADS["c3"], n_seq=48, L=9000, B=64, k=100, needles=8, name="static_big")
    small = WL.scaled(WL.WORKLOADS["c4"], L=2300, n_q=37, B=48, k=64, k_cand=256, needles=8,
                      q_dtype="e4m3", name="static_small")
    assert misa.workspace_bytes(misa.to_device(WL.make_inputs(small, seed=1))["problem"], misa.OP_ROUTE) \
        < misa.workspace_bytes(misa.to_device(WL.make_inputs(big, seed=1))["problem"], misa.OP_ROUTE) \
        <= misa.ROUTE_STATIC_SCRATCH_BYTES
    _route_both(misa, big, seed=31)
    inp, heads, E = _route_both(misa, small, seed=32)
    for t in range(small.n_q):
        K, q, w, n = oracle_view(inp, 0, t)
        _, ref_E = O.route_heads(q, w, K, small.B, small.h, n)
        assert_scores_close(E[0, t], ref_E, f"static E {t}")
        check_index_set(heads[0, t], ref_E, small.h, f"static heads {t}")


def test_route_heads_static_rejects_oversize_before_launch(misa):
    # 8192 queries x 64 heads need 8 MiB of partial sums: more than the built-in array
    wl = WL.scaled(WL.WORKLOADS["c2"], L=4096, n_q=8192, B=64, k=16, needles=0, name="static_oversize")
    q_pos = torch.arange(wl.n_q, dtype=torch.int32, device="cuda") % wl.L
    p = misa.Problem(1, wl.L, wl.n_q, wl.H, wl.B, wl.h, misa.BF16, misa.BF16, q_pos=q_pos)
    assert misa.workspace_bytes(p, misa.OP_ROUTE) > misa.ROUTE_STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)
    st = misa.lib.misa_route_heads_static(ctypes.byref(p.c()), fake, fake, fake, fake, None, fake, None, None)
    assert st == 2 and b"scratch" in misa.lib.misa_last_error()
