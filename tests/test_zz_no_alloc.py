"""infmllm_stream_attach_static (the entry point for callers that cannot allocate device memory): a stream
whose workspace is the library's own per-device array must give exactly what a stream attached to a caller's
workspace gives -- outputs, retained lists and cache contents bit for bit, since the same kernels run on the
same inputs -- and must stay inside the fp64 oracle's bars.  Two holders in a row, the second smaller, so that
the second sees the first one's leftovers in the array."""
import numpy as np
import pytest
import torch

from oracle import OracleStream
from paper_2409_09086_amd import binding as B
from paper_2409_09086_amd.workloads import random_chunk
from _parity import LockStep

pytestmark = pytest.mark.gpu


def run_pair(heads, kv, d, budget, recent, lens, seed, decode=0):
    """The same chunks through a static-workspace stream and a caller-workspace stream; the static one is also
    driven in lock-step with the oracle."""
    a = B.Stream(budget, recent, heads, kv, d, dtype=torch.bfloat16, bias=1e-3, max_chunk=max(lens), max_decode=decode,
                 static_workspace=True)
    b = B.Stream(budget, recent, heads, kv, d, dtype=torch.bfloat16, bias=1e-3, max_chunk=max(lens), max_decode=decode)
    assert a.workspace is None and b.workspace is not None
    ls = LockStep(a, OracleStream(budget, recent, heads, kv, d, bias=1e-3))
    for step, L in enumerate(lens):
        print("static workspace", (heads, kv, d, budget, recent), "step", step, "L", L, flush=True)
        q, k, v = random_chunk(seed + step, L, heads, kv, d, "bf16")
        out_a, I_a = ls.step(q, k, v, check_state=True)
        out_b, ret_b, cnt_b = b.step(q.cuda(), k.cuda(), v.cuda())
        assert torch.equal(out_a, out_b), "outputs differ between the two workspaces"
        assert (ret_b.cpu().numpy()[:, : int(cnt_b.item())] == I_a).all(), "retained lists differ"
        for x, y in zip(a.export(), b.export()):
            assert torch.equal(x, y), "cache contents differ"
        for i in range(decode):
            q1, k1, v1 = random_chunk(seed + 100 * step + i + 50, 1, heads, kv, d, "bf16")
            o_a = ls.decode(q1, k1, v1)
            o_b = b.decode(q1.cuda(), k1.cuda(), v1.cuda())
            assert torch.equal(o_a, o_b)
    torch.cuda.synchronize()
    a.close()
    return ls.max_err


def test_static_workspace_two_holders_in_a_row():
    e1 = run_pair(8, 2, 128, 640, 128, [256, 256, 256, 200, 256, 77], seed=2100, decode=3)
    # a smaller stream takes the array over: everything it relies on must have been cleared at attach
    e2 = run_pair(4, 4, 64, 96, 32, [48, 48, 20, 48, 48], seed=2200)
    print("static workspace: max err %.3g / %.3g" % (e1, e2))


def test_static_workspace_is_exclusive_and_bounded():
    s = B.Stream(64, 16, 2, 2, 64, dtype=torch.bfloat16, max_chunk=32, static_workspace=True)
    with pytest.raises(B.InfMLLMError) as e:                       # the array has a holder
        B.Stream(64, 16, 2, 2, 64, dtype=torch.bfloat16, max_chunk=32, static_workspace=True)
    assert e.value.code == B.ESTATE
    s.close()
    s = B.Stream(64, 16, 2, 2, 64, dtype=torch.bfloat16, max_chunk=32, static_workspace=True)   # released by destroy
    s.close()
    with pytest.raises(B.InfMLLMError) as e:                       # cfg5's layer needs far more than the array holds
        B.Stream(8192, 2048, 32, 32, 128, dtype=torch.bfloat16, max_chunk=2048, static_workspace=True)
    assert e.value.code == B.ENOMEM and "bytes" in str(e.value)
    with pytest.raises(B.InfMLLMError) as e:
        B.Stream(64, 16, 2, 2, 64, dtype=torch.bfloat16, max_chunk=32, rope_base=10000.0, static_workspace=True)
    assert e.value.code == B.EINVAL
