"""Cache-relative rotary position encoding (Sec. 3.4 length extrapolation) through the C ABI, in lock-step
with the fp64 oracle: once with the oracle storing its rotated q and k in the stream's element type (as a
model stores them; usual 1e-5 band), once with the oracle keeping them exact (band widened by what that
one rounding can do to a score, derived in the test)."""
import numpy as np
import pytest
import torch

from oracle import OracleStream
from paper_2409_09086_amd import binding as B
from paper_2409_09086_amd.workloads import CONFIGS, ChunkStream, random_chunk
from _parity import LockStep

pytestmark = pytest.mark.gpu
DT = {"fp32": torch.float32, "bf16": torch.bfloat16}
BASE = 10000.0


def pair(budget, recent, heads, kv, d, dtype, bias, max_chunk, impl=None, max_decode=None, policy=None, base=BASE,
         exact=False, band=None):
    gpu = B.Stream(budget, recent, heads, kv, d, dtype=DT[dtype], bias=bias, max_chunk=max_chunk, impl=impl,
                   max_decode=max_decode, policy=policy, rope_base=base)
    orc = OracleStream(budget, recent, heads, kv, d, bias=bias, policy=policy or "infmllm",
                       rope_base=base, rope_round=None if exact else dtype)
    return LockStep(gpu, orc) if band is None else LockStep(gpu, orc, band=band)


@pytest.mark.parametrize("heads,kv,d,dtype,impl,budget,recent,lens", [
    (4, 4, 128, "bf16", 0, 192, 64, [64, 64, 64, 64, 64, 64]),
    (8, 2, 128, "bf16", 0, 160, 48, [100, 37, 64, 1, 129, 77, 5, 160]),
    (8, 2, 128, "bf16", 1, 160, 48, [100, 37, 64, 1, 129, 77]),
    (4, 2, 64, "bf16", 0, 128, 32, [64, 64, 50, 64, 64]),
    (4, 4, 64, "fp32", None, 128, 32, [64, 64, 40, 64, 64]),
    (2, 2, 128, "fp32", None, 96, 24, [48, 48, 48, 48]),
])
def test_rope_streams_match_the_unrounded_oracle(heads, kv, d, dtype, impl, budget, recent, lens):
    """Against the oracle that keeps its rotated q and k exact (no rounding to the stream type).
    Outputs: the usual 2e-2 / 1e-4.  Retained sets: storing a rotated element in bf16 moves it by at most
    2^-9 relative, so a logit scale * sum_i q_i k_i moves by at most 2^-8 * scale * sum_i |q_i k_i|; for the
    N(0,1) inputs used here E|q_i k_i| = 2/pi, so that is 2^-8 * (2/pi) * sqrt(d) <= 0.029 for d = 128
    (typically a tenth of it, the errors having random signs), i.e. a weight moves by at most
    exp(0.029) - 1 = 2.9e-2 relative, and so does a column mean.  Band: 3e-2 relative for bf16 streams.
    For fp32 streams the same bound with 2^-24 is 2e-6, inside the ordinary 1e-5 band."""
    band = 3e-2 if dtype == "bf16" else 1e-5
    ls = pair(budget, recent, heads, kv, d, dtype, 1e-3, max(lens), impl=impl, exact=True, band=band)
    for step, L in enumerate(lens):
        print("rope exact", (heads, kv, d, dtype, impl, budget, recent), "step", step, "L", L, flush=True)
        q, k, v = random_chunk(700 + step, L, heads, kv, d, dtype)
        ls.step(q, k, v, check_state=True)
    print("max err %.3g swaps %d" % (ls.max_err, ls.swaps))


@pytest.mark.parametrize("heads,kv,d,dtype,impl,budget,recent,lens", [
    (4, 4, 128, "bf16", 0, 192, 64, [64, 64, 64, 64, 64, 64]),
    (8, 2, 128, "bf16", 0, 160, 48, [100, 37, 64, 1, 129, 77, 5, 160]),       # grouped heads, ragged, L = 1
    (8, 2, 128, "bf16", 1, 160, 48, [100, 37, 64, 1, 129, 77]),               # plain-arithmetic kernels
    (4, 2, 64, "bf16", 0, 128, 32, [64, 64, 50, 64, 64]),
    (4, 4, 64, "fp32", None, 128, 32, [64, 64, 40, 64, 64]),
    (2, 2, 128, "fp32", None, 96, 24, [48, 48, 48, 48]),
])
def test_rope_streams_match_oracle(heads, kv, d, dtype, impl, budget, recent, lens):
    ls = pair(budget, recent, heads, kv, d, dtype, 1e-3, max(lens), impl=impl)
    for step, L in enumerate(lens):
        print("rope", (heads, kv, d, dtype, impl, budget, recent), "step", step, "L", L, flush=True)
        q, k, v = random_chunk(700 + step, L, heads, kv, d, dtype)
        ls.step(q, k, v, check_state=True)                         # the cache itself holds the rows as given
    print("max err %.3g swaps %d" % (ls.max_err, ls.swaps))


def test_rope_changes_the_result():
    """Same inputs with and without the encoding must differ (the option is not a no-op)."""
    q, k, v = [x.cuda() for x in random_chunk(1, 64, 4, 4, 128, "bf16")]
    a = B.Stream(128, 32, 4, 4, 128, dtype=torch.bfloat16, max_chunk=64)
    b = B.Stream(128, 32, 4, 4, 128, dtype=torch.bfloat16, max_chunk=64, rope_base=BASE)
    oa, ob = a.step(q, k, v)[0], b.step(q, k, v)[0]
    assert (oa.float() - ob.float()).abs().max().item() > 1e-2


def test_rope_with_decode_steps_between_chunks():
    ls = pair(128, 32, 4, 2, 128, "bf16", 1e-4, 64, max_decode=8)
    for rnd in range(4):
        q, k, v = random_chunk(40 + rnd, 64, 4, 2, 128, "bf16")
        ls.step(q, k, v, check_state=True)
        for tok in range(5):
            q, k, v = random_chunk(900 + 10 * rnd + tok, 1, 4, 2, 128, "bf16")
            ls.decode(q, k, v)
        ls.check_state()


def test_rope_with_batched_eviction_and_cumulative_policy():
    n_layers, heads, kv, d, budget, recent = 3, 4, 2, 128, 160, 40
    ls = [pair(budget, recent, heads, kv, d, "bf16", 1e-4, 96, policy="cumulative") for _ in range(n_layers)]
    for step, L in enumerate([96, 96, 50, 96, 96]):
        for li, l in enumerate(ls):
            l.attend(*random_chunk(5000 + 100 * li + step, L, heads, kv, d, "bf16"))
        if ls[0].gpu.pending:
            B.evict_batched([l.gpu for l in ls])
            for l in ls:
                l.finish()
        for l in ls:
            l.check_state()


def test_rope_at_full_shape_cfg2():
    cfg = CONFIGS["cfg2"]
    ls = pair(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim, cfg.dtype, cfg.bias, cfg.max_chunk)
    for step, (q, k, v) in zip(range(7), ChunkStream(cfg)):
        print("cfg2 rope step", step, flush=True)
        ls.step(q, k, v, check_state=(step == 6))
    print("max err %.3g swaps %d" % (ls.max_err, ls.swaps))


def test_rope_import_then_step():
    """An imported cache has no turned copies yet: the next step must make them."""
    ls = pair(96, 24, 4, 4, 64, "bf16", 1e-3, 48)
    for step in range(3):
        ls.step(*random_chunk(60 + step, 48, 4, 4, 64, "bf16"))
    K, V, pos, _ = ls.gpu.export()
    twin = pair(96, 24, 4, 4, 64, "bf16", 1e-3, 48)
    twin.gpu.load(K, V, pos, ls.gpu.streamed)
    twin.oracle.load(K.double().cpu().numpy(), V.double().cpu().numpy(), pos.cpu().numpy(), ls.gpu.streamed)
    twin.step(*random_chunk(99, 48, 4, 4, 64, "bf16"), check_state=True)


def test_bad_rope_base_is_refused():
    h = B.ctypes.c_void_p()
    L = B.lib()
    assert L.infmllm_stream_create(64, 16, 2, 2, 64, B.BF16, B.ctypes.byref(h)) == 0
    assert L.infmllm_stream_set_param(h, B.PARAM_ROPE_BASE, 0.5) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_ROPE_BASE, -3.0) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_ROPE_BASE, 10000.0) == 0
    assert L.infmllm_stream_set_param(h, B.PARAM_ROPE_BASE, 0.0) == 0
    L.infmllm_stream_destroy(h)
