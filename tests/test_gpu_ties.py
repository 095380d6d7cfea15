"""Exact ties in the biased score (Alg. 1 l.5-7 with b = 0 and repeated keys): rows with the same key get
the same score bit for bit on both sides, so the retained lists must be identical, the newest of the
tied rows winning.  Covers the selection's degenerate paths: every score equal, two or three distinct
values over thousands of candidates, a threshold bin that is split between kept and dropped ties."""
import numpy as np
import pytest
import torch

from oracle import OracleStream
from paper_2409_09086_amd import binding as B
from paper_2409_09086_amd.workloads import random_chunk
from _parity import LockStep

pytestmark = pytest.mark.gpu
DT = {"fp32": torch.float32, "bf16": torch.bfloat16}


def coded_chunk(seed, L, heads, kv, d, dtype, n_codes, t0):
    """random q and v; every key row is one of n_codes fixed vectors per kv-head, chosen by a fixed
    pattern of the stream position so that each code recurs through the whole stream."""
    q, k, v = random_chunk(seed, L, heads, kv, d, dtype)
    g = torch.Generator().manual_seed(4242)
    book = torch.randn((n_codes, kv, d), generator=g).to(k.dtype)
    pos = torch.arange(t0, t0 + L)
    code = (pos * 7 + pos // 5) % n_codes
    return q, book[code].contiguous(), v


@pytest.mark.parametrize("heads,kv,d,dtype,impl,budget,recent,lens,n_codes", [
    (4, 2, 128, "bf16", None, 192, 64, [100, 100, 64, 37, 128], 1),      # every score equal: the newest r stay
    (4, 2, 128, "bf16", None, 192, 64, [100, 100, 64, 37, 128], 2),
    (4, 4, 128, "bf16", None, 192, 64, [100, 100, 64, 37, 128], 3),
    (4, 4, 128, "bf16", None, 160, 33, [97, 97, 97, 97], 7),
    (2, 2, 64, "bf16", 0, 128, 32, [64, 64, 50, 64], 3),                 # matrix-core kernels, head_dim 64
    (2, 2, 64, "bf16", 1, 128, 32, [64, 64, 50, 64], 3),                 # plain-arithmetic kernels on a bf16 stream
    (4, 2, 128, "bf16", 1, 192, 64, [100, 100, 64, 37, 128], 2),         # ... grouped heads, head_dim 128
    (2, 2, 64, "fp32", None, 128, 32, [64, 64, 50, 64], 2),
    (2, 2, 128, "bf16", None, 1536, 256, [1024, 1000, 512, 512], 3),     # 16 wavefronts' worth of candidates
    (2, 1, 128, "bf16", None, 3000, 200, [2048, 2048, 1111], 5),         # four keys per thread
])
def test_exact_ties_go_to_the_newer_rows(heads, kv, d, dtype, impl, budget, recent, lens, n_codes):
    gpu = B.Stream(budget, recent, heads, kv, d, dtype=DT[dtype], bias=0.0, max_chunk=max(lens), impl=impl)
    orc = OracleStream(budget, recent, heads, kv, d, bias=0.0)
    ls = LockStep(gpu, orc)
    t0 = 0
    for step, L in enumerate(lens):
        print("ties", (heads, kv, d, dtype, impl, budget, recent, n_codes), "step", step, "L", L, flush=True)
        q, k, v = coded_chunk(900 + step, L, heads, kv, d, dtype, n_codes, t0)
        n = len(orc) + L
        _, I_g = ls.step(q, k, v, check_state=True, strict=True)
        if n_codes == 1 and n > budget:                               # closed form: the newest budget rows
            assert (I_g == np.arange(n - budget, n)).all()
        t0 += L
    assert ls.swaps == 0
