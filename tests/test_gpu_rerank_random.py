"""Seeded random many-query re-rank problems (Eq. misa_final_topk): list lengths up to the
8192 the one-kernel path takes and beyond, any k, head counts, storage types, ragged lists."""
import numpy as np
import pytest
import torch

from paper_2605_07363_amd import workloads as WL
from helpers import ABS_FRAC
from test_gpu_rerank_fused import _candidates, _check_rows_against_oracle, _rerank, _rerank_in_pieces

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def misa():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2605_07363_amd import misa as m
    return m


@pytest.mark.parametrize("seed", range(10))
def test_many_query_rerank_random(misa, seed):
    rng = np.random.default_rng(9980 + seed)
    rows = int(rng.integers(1024, 1400))
    H = int(rng.choice([1, 8, 17, 32, 33, 64]))
    L = int(rng.integers(600, 12000))
    kc = int(rng.choice([int(rng.integers(1, 200)), int(rng.integers(200, 3000)), int(rng.integers(3000, 8193)), 8192, 9000]))
    kc = min(kc, 16384)
    k = int(rng.integers(1, kc + 1))
    wl = WL.scaled(WL.WORKLOADS["c2"], n_seq=1, L=L, n_q=rows, H=H, h=1, B=64, k=1, k_cand=0,
                   k_dtype=["bf16", "e4m3"][seed % 2], q_dtype="bf16", needles=8, name=f"rrr{seed}")
    inp = WL.make_inputs(wl, seed=seed)
    dv = misa.to_device(inp)
    p = dv["problem"]
    cand = _candidates(rng, rows, L, kc, full=bool(seed % 3 == 0))
    dcand = torch.from_numpy(cand).cuda()
    idx, val = _rerank(misa, p, dv, dcand, kc, k)
    idx2, val2 = _rerank_in_pieces(misa, p, dv, dcand, kc, k, piece=700)
    assert torch.equal(idx, idx2), (rows, H, L, kc, k)
    assert torch.equal(val, val2), (rows, H, L, kc, k)
    sample = [0, rows - 1] + rng.choice(rows, size=6, replace=False).tolist()
    _check_rows_against_oracle(inp, cand, idx.cpu().numpy(), val.cpu().numpy(), k, sample, f"random rerank {seed}", abs_frac=ABS_FRAC)
