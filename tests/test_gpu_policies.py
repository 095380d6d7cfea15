"""Comparison policies (Sec. 2, Sec. 4.1: window, initial + recent, cumulative score) as scoring modes of
the same HIP kernels, through the C ABI, in lock-step with the fp64 oracle running the same policy."""
import numpy as np
import pytest
import torch

from oracle import OracleStream
from paper_2409_09086_amd import binding as B
from paper_2409_09086_amd.workloads import CONFIGS, ChunkStream, random_chunk
from _parity import LockStep

pytestmark = pytest.mark.gpu
DT = {"fp32": torch.float32, "bf16": torch.bfloat16}


def pair(policy, budget, recent, heads, kv, d, dtype, bias, max_chunk, impl=None, max_decode=None):
    gpu = B.Stream(budget, recent, heads, kv, d, dtype=DT[dtype], bias=bias, max_chunk=max_chunk, impl=impl,
                   policy=policy, max_decode=max_decode)
    orc = OracleStream(budget, recent, heads, kv, d, bias=bias, policy=policy)
    return LockStep(gpu, orc)


def check_accumulated(ls):
    """cumulative policy: the score array the library carries equals the oracle's totals (+inf = none yet)."""
    score = ls.gpu.export()[3].cpu().numpy().astype(np.float64)
    A = ls.oracle.accumulated()
    never = np.isinf(score)
    assert (A[never] == 0).all()
    assert np.allclose(score[~never], A[~never], rtol=2e-5, atol=1e-9), np.abs(score[~never] - A[~never]).max()


SHAPES = [
    (4, 4, 128, "bf16", 0, 192, 64, [64, 64, 64, 64, 64, 64]),
    (8, 2, 128, "bf16", 0, 160, 48, [100, 37, 64, 1, 129, 77, 5, 160]),
    (8, 2, 128, "bf16", 1, 160, 48, [100, 37, 64, 1, 129, 77]),
    (4, 2, 64, "bf16", 0, 128, 0, [64, 64, 64, 64]),
    (4, 4, 64, "fp32", None, 128, 32, [64, 64, 40, 64, 64]),
    (8, 2, 128, "bf16", 0, 256, 128, [128, 128, 128, 128, 128]),      # scoring shares its rows out over workgroups
]


@pytest.mark.parametrize("policy", ["window", "initial_recent", "cumulative"])
@pytest.mark.parametrize("heads,kv,d,dtype,impl,budget,recent,lens", SHAPES)
def test_policy_streams_match_oracle(policy, heads, kv, d, dtype, impl, budget, recent, lens):
    ls = pair(policy, budget, recent, heads, kv, d, dtype, 1e-3, max(lens), impl=impl)
    total = 0
    for step, L in enumerate(lens):
        print(policy, (heads, kv, d, dtype, impl, budget, recent), "step", step, "L", L, flush=True)
        q, k, v = random_chunk(500 + step, L, heads, kv, d, dtype)
        ls.step(q, k, v, check_state=True)
        total += L
        pos = ls.gpu.positions().cpu().numpy()
        if policy == "window":
            assert (pos == np.arange(max(0, total - budget), total)).all()
        if policy == "initial_recent" and total > budget:
            assert (pos == np.concatenate([np.arange(budget - recent), np.arange(total - recent, total)])).all()
        if policy == "cumulative":
            check_accumulated(ls)
    print("max err %.3g swaps %d" % (ls.max_err, ls.swaps))


def test_cumulative_policy_with_decode_steps_between_chunks():
    ls = pair("cumulative", 128, 32, 4, 2, 128, "bf16", 1e-4, 64, max_decode=8)
    for rnd in range(4):
        q, k, v = random_chunk(40 + rnd, 64, 4, 2, 128, "bf16")
        ls.step(q, k, v, check_state=True)
        for tok in range(5):
            q, k, v = random_chunk(900 + 10 * rnd + tok, 1, 4, 2, 128, "bf16")
            ls.decode(q, k, v)
        check_accumulated(ls)


@pytest.mark.parametrize("policy", ["window", "cumulative"])
def test_policies_at_full_shape_cfg2(policy):
    cfg = CONFIGS["cfg2"]
    ls = pair(policy, cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, cfg.dtype, cfg.bias, cfg.max_chunk)
    for step, (q, k, v) in zip(range(8), ChunkStream(cfg)):
        print("cfg2", policy, "step", step, flush=True)
        ls.step(q, k, v, check_state=(step == 7))
    if policy == "cumulative":
        check_accumulated(ls)
    print("max err %.3g swaps %d" % (ls.max_err, ls.swaps))


def test_batched_eviction_with_the_cumulative_policy():
    n_layers, heads, kv, d, budget, recent = 3, 4, 2, 128, 160, 40
    ls = [pair("cumulative", budget, recent, heads, kv, d, "bf16", 1e-4, 96) for _ in range(n_layers)]
    for step, L in enumerate([96, 96, 50, 96, 96]):
        for li, l in enumerate(ls):
            l.attend(*random_chunk(3000 + 100 * li + step, L, heads, kv, d, "bf16"))
        if ls[0].gpu.pending:
            B.evict_batched([l.gpu for l in ls])
            for l in ls:
                l.finish()
        for l in ls:
            l.check_state()
            check_accumulated(l)


def test_unknown_policy_is_refused():
    with pytest.raises(KeyError):
        B.Stream(64, 16, 2, 2, 64, dtype=torch.bfloat16, policy="lru")
    h = B.ctypes.c_void_p()
    L = B.lib()
    assert L.infmllm_stream_create(64, 16, 2, 2, 64, B.BF16, B.ctypes.byref(h)) == 0
    assert L.infmllm_stream_set_param(h, B.PARAM_POLICY, 4.0) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_POLICY, 2.0) == 0
    L.infmllm_stream_destroy(h)
