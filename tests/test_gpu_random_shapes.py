"""Seeded random problems through the whole pipeline against the oracle: odd head counts and
block sizes, every storage type of keys and queries, ragged batches, causal chunks that start
anywhere, the paged layout, single-stage and hierarchical selection."""
import os

import numpy as np
import pytest

from paper_2605_07363_amd import workloads as WL
from test_gpu_pipeline import run_and_check

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def misa():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2605_07363_amd import misa as m
    return m


def draw(seed):
    rng = np.random.default_rng(1000 + seed)
    decode = bool(rng.integers(0, 2))
    k_dtype = ["f32", "bf16", "e4m3"][seed % 3]
    q_dtype = ["bf16", "bf16", "e4m3", "f32"][(seed // 3) % 4]
    H = int(rng.choice([1, 3, 8, 17, 32, 64]))
    h = int(rng.integers(1, H + 1))
    L = int(rng.integers(40, 5000))
    n_q = 1 if decode else int(rng.integers(2, 80))
    n_seq = int(rng.integers(1, 10 if decode else 3))
    B = int(rng.choice([1, 7, 16, 64, 128, 1000, L + 3]))
    k = int(rng.integers(1, min(L, 500) + 1))
    k_cand = int(min(L, k * int(rng.integers(2, 5)))) if rng.integers(0, 3) == 0 else 0
    wl = WL.scaled(WL.WORKLOADS["c2" if not decode else "c3"], n_seq=n_seq, L=L, n_q=n_q, H=H, h=h, B=B, k=k,
                   k_cand=k_cand, k_dtype=k_dtype, q_dtype=q_dtype, decode=decode,
                   needles=int(rng.integers(0, 9)), name=f"random{seed}")
    seq_len = None
    if rng.integers(0, 2):
        seq_len = rng.integers(0, L + 1, n_seq).astype(np.int32)
        seq_len[int(rng.integers(0, n_seq))] = L
    page = int(rng.choice([0, 0, 16, 64, 128]))
    # causal chunk anywhere in the prefix, or arbitrary (unsorted, repeated) query positions
    q_pos = None
    if not decode:
        kind = int(rng.integers(0, 3))
        if kind == 1:
            q_pos = (int(rng.integers(0, L - n_q + 1)) + np.arange(n_q)).astype(np.int32)
        elif kind == 2:
            q_pos = rng.integers(0, L, n_q).astype(np.int32)
    return wl, seq_len, page, q_pos


# MISA_RANDOM_SEEDS=200 widens the sweep for a one-off soak of new kernels
@pytest.mark.parametrize("seed", range(int(os.environ.get("MISA_RANDOM_SEEDS", "24"))))
def test_random_problem(misa, seed):
    wl, seq_len, page, q_pos = draw(seed)
    print(wl, seq_len, page, q_pos, flush=True)
    inp = WL.make_inputs(wl, seed=seed, seq_len=seq_len)
    if q_pos is not None:
        inp["q_pos"] = q_pos
    st = run_and_check(misa, wl, inp, page_size=page)
    assert st["rows"] == wl.n_seq * wl.n_q


@pytest.mark.parametrize("seed", range(int(os.environ.get("MISA_RANDOM_FUSED_SEEDS", "12"))))
def test_random_problem_fused_call_equals_two_calls(misa, seed):
    # problems large enough for the threshold-prefilter path of misa_select_tokens
    rng = np.random.default_rng(5000 + seed)
    H = int(rng.choice([8, 32, 64]))
    L = int(rng.integers(4096, 12000))
    n_q = int(rng.integers(64, 200))
    wl = WL.scaled(WL.WORKLOADS["c2"], n_seq=int(rng.integers(1, 3)), L=L, n_q=n_q, H=H,
                   h=min(H, int(rng.choice([1, 3, 8, 16, H]))), B=int(rng.choice([16, 64, 128, 1024])),
                   k=int(rng.integers(1, 2049)), k_dtype=["bf16", "e4m3"][seed % 2],
                   q_dtype=["bf16", "e4m3"][(seed // 2) % 2], needles=int(rng.integers(0, 9)), name=f"fused{seed}")
    seq_len = None
    if rng.integers(0, 2):
        seq_len = rng.integers(0, L + 1, wl.n_seq).astype(np.int32)
    inp = WL.make_inputs(wl, seed=seed, seq_len=seq_len)
    if rng.integers(0, 2):
        inp["q_pos"] = np.sort(rng.integers(0, L, n_q)).astype(np.int32)
    dv = misa.to_device(inp)
    page = int(rng.choice([0, 64, 256]))
    if page:
        dv = misa.paginate(dv, page, seed=seed)
    p = dv["problem"]
    a = misa.Indexer(p, wl.k, want_val=True)
    b = misa.Indexer(p, wl.k, want_val=True, fused=True)
    ia = a.run(dv["K"], dv["kscale"], dv["Q"], dv["W"])
    ib = b.run(dv["K"], dv["kscale"], dv["Q"], dv["W"])
    assert torch.equal(ia, ib)
    assert torch.equal(a.val, b.val)
    if wl.q_dtype == "e4m3":
        # stage by stage on the codes themselves: every call widens them inside its own workspace
        c = misa.Indexer(p, wl.k, want_val=True, fused=True)
        c.pool(dv["K"], dv["kscale"])
        c.route(dv["Q"], dv["W"], dv["K"], dv["kscale"])
        c.select_fused(dv["Q"], dv["W"], dv["K"], dv["kscale"])
        assert torch.equal(c.idx, ia) and torch.equal(c.val, a.val)
        d = misa.Indexer(p, wl.k, want_val=True)
        d.pool(dv["K"], dv["kscale"])
        d.route(dv["Q"], dv["W"], dv["K"], dv["kscale"])
        d.score(dv["Q"], dv["W"], dv["K"], dv["kscale"])
        d.select()
        assert torch.equal(d.idx, ia) and torch.equal(d.S, a.S)
    if wl.q_dtype == "e4m3" and wl.k_dtype == "e4m3":
        # the same on the fp8 matrix instruction: fused call = two calls bit for bit there too
        from dataclasses import replace
        pm = replace(p, q_dtype=misa.FP8_E4M3_MATRIX)
        e = misa.Indexer(pm, wl.k, want_val=True)
        f = misa.Indexer(pm, wl.k, want_val=True, fused=True)
        ie = e.run(dv["K"], dv["kscale"], dv["Q"], dv["W"])
        jf = f.run(dv["K"], dv["kscale"], dv["Q"], dv["W"])
        assert torch.equal(ie, jf) and torch.equal(e.val, f.val)
