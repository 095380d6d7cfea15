"""Layer-batched eviction (Alg. 1, note under "Input") through the C ABI: several streams attend
one after the other, then one infmllm_evict_batched call selects and gathers for all of them.
Every stream is compared with its own fp64 oracle, and with a twin stream driven by infmllm_step."""
import numpy as np
import pytest
import torch

from oracle import OracleStream
from paper_2409_09086_amd import binding as B
from paper_2409_09086_amd.workloads import CONFIGS, ChunkStream, random_chunk
from _parity import LockStep

pytestmark = pytest.mark.gpu
DT = {"fp32": torch.float32, "bf16": torch.bfloat16}


def layers(n_layers, budget, recent, heads, kv, d, dtype, bias, max_chunk, impl=None):
    out = []
    for _ in range(n_layers):
        gpu = B.Stream(budget, recent, heads, kv, d, dtype=DT[dtype], bias=bias, max_chunk=max_chunk, impl=impl)
        orc = OracleStream(budget, recent, heads, kv, d, bias=bias)
        out.append(LockStep(gpu, orc))
    return out


def batched_step(ls, chunks):
    """chunks[i] = (q, k, v) of layer i.  Attend layer by layer, evict together."""
    for l, (q, k, v) in zip(ls, chunks):
        l.attend(q, k, v)
    todo = [l for l in ls if l.gpu.pending]
    if todo:
        assert len(todo) == len(ls)
        B.evict_batched([l.gpu for l in todo])
        for l in todo:
            l.finish()


@pytest.mark.parametrize("n_layers,heads,kv,d,dtype,budget,recent,lens", [
    (3, 4, 4, 128, "bf16", 192, 64, [64, 64, 64, 64, 64]),
    (4, 8, 2, 128, "bf16", 160, 48, [100, 37, 64, 1, 129, 77]),      # grouped heads, ragged, L = 1
    (2, 4, 2, 64, "bf16", 96, 96, [32, 64, 50, 50]),                  # r = 0
    (3, 4, 4, 64, "fp32", 128, 32, [64, 64, 40, 64]),
    (18, 2, 2, 64, "bf16", 96, 32, [48, 48, 48, 30]),                 # more streams than one launch takes
    (2, 16, 2, 64, "bf16", 320, 160, [160, 160, 160, 45, 160]),       # scoring shares its rows out over workgroups
])
def test_batched_eviction_matches_oracle(n_layers, heads, kv, d, dtype, budget, recent, lens):
    ls = layers(n_layers, budget, recent, heads, kv, d, dtype, 1e-3, max(lens))
    for step, L in enumerate(lens):
        print("batched", (n_layers, heads, kv, d, dtype, budget, recent), "step", step, "L", L, flush=True)
        chunks = [random_chunk(1000 * li + step, L, heads, kv, d, dtype) for li in range(n_layers)]
        batched_step(ls, chunks)
        for l in ls:
            l.check_state()
    print("max err %.3g swaps %d" % (max(l.max_err for l in ls), sum(l.swaps for l in ls)))


def test_batched_equals_single_stream_steps_bit_for_bit():
    heads, kv, d, budget, recent = 8, 2, 128, 256, 64
    n_layers, lens = 5, [128, 128, 90, 128, 17, 128]
    mk = lambda: B.Stream(budget, recent, heads, kv, d, dtype=torch.bfloat16, bias=1e-3, max_chunk=128)
    a, b = [mk() for _ in range(n_layers)], [mk() for _ in range(n_layers)]
    for step, L in enumerate(lens):
        print("twin step", step, flush=True)
        chunks = [[x.cuda() for x in random_chunk(77 * li + step, L, heads, kv, d, "bf16")] for li in range(n_layers)]
        res_a = [s.step(*c) for s, c in zip(a, chunks)]
        res_b = [s.step_attend(*c) for s, c in zip(b, chunks)]
        if b[0].pending:
            B.evict_batched(b)
        for li in range(n_layers):
            cnt = int(res_a[li][2].item())
            assert cnt == int(res_b[li][2].item())
            assert torch.equal(res_a[li][0], res_b[li][0])
            assert torch.equal(res_a[li][1][:, :cnt], res_b[li][1][:, :cnt])
            for x, y in zip(a[li].export(), b[li].export()):
                assert torch.equal(x, y)
            assert a[li].streamed == b[li].streamed and len(a[li]) == len(b[li])


def test_batched_eviction_at_full_shape_cfg2():
    cfg = CONFIGS["cfg2"]
    n_layers = 3
    ls = layers(n_layers, cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, cfg.dtype, cfg.bias, cfg.max_chunk)
    gens = [iter(ChunkStream(cfg, layer=li)) for li in range(n_layers)]
    for step in range(7):
        print("cfg2 batched step", step, flush=True)
        batched_step(ls, [next(g) for g in gens])
    for l in ls:
        l.check_state()
    print("max err %.3g swaps %d" % (max(l.max_err for l in ls), sum(l.swaps for l in ls)))


def test_pending_state_and_argument_errors():
    mk = lambda **kw: B.Stream(64, 16, 2, 2, 64, dtype=torch.bfloat16, max_chunk=48, **kw)
    s, other = mk(), mk()
    c = lambda seed, L: [x.cuda() for x in random_chunk(seed, L, 2, 2, 64, "bf16")]
    s.step_attend(*c(1, 48))
    assert not s.pending and len(s) == 48
    with pytest.raises(B.InfMLLMError) as e:                       # nothing pending
        B.evict_batched([s])
    assert e.value.code == B.ESTATE
    s.step_attend(*c(2, 48))
    assert s.pending and len(s) == 48 and s.streamed == 48         # counters move with the eviction
    for call in (lambda: s.step(*c(3, 8)), lambda: s.step_attend(*c(3, 8)), s.export, s.positions):
        with pytest.raises(B.InfMLLMError) as e:
            call()
        assert e.value.code == B.ESTATE
    with pytest.raises(B.InfMLLMError) as e:                       # the other stream has nothing pending
        B.evict_batched([s, other])
    assert e.value.code == B.ESTATE and s.pending
    with pytest.raises(B.InfMLLMError) as e:
        B.evict_batched([s, s])
    assert e.value.code == B.EINVAL and s.pending
    odd = B.Stream(64, 8, 2, 2, 64, dtype=torch.bfloat16, max_chunk=48)
    odd.step_attend(*c(4, 48))
    odd.step_attend(*c(5, 48))
    with pytest.raises(B.InfMLLMError) as e:                       # recent differs
        B.evict_batched([s, odd])
    assert e.value.code == B.EINVAL and s.pending and odd.pending
    B.evict_batched([s])
    B.evict_batched([odd])
    assert not s.pending and len(s) == 64 and s.streamed == 96
    torch.cuda.synchronize()
