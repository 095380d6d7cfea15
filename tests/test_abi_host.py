"""Host-side checks of the C ABI that need no GPU: the shared library loads, exports every
symbol the header declares, and rejects bad arguments with the documented codes."""
import ctypes
import os
import re

import pytest

from paper_2409_09086_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "infmllm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(infmllm_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_functions()
    assert len(names) >= 13
    for name in names:
        assert hasattr(L, name), name
    assert sorted(B.EXPORTS) == names


def make(budget=16, recent=4, heads=4, kv=2, d=64, dtype=B.BF16):
    h = ctypes.c_void_p()
    rc = B.lib().infmllm_stream_create(budget, recent, heads, kv, d, dtype, ctypes.byref(h))
    return rc, h


@pytest.mark.parametrize("args", [
    dict(budget=0), dict(budget=-3), dict(recent=-1), dict(recent=17), dict(heads=3, kv=2), dict(heads=0),
    dict(kv=0), dict(d=96), dict(d=0), dict(dtype=7),
])
def test_create_rejects_bad_arguments(args):
    rc, h = make(**args)
    assert rc == B.EINVAL and not h.value
    assert B.last_error() != ""


def test_create_null_out_pointer():
    assert B.lib().infmllm_stream_create(16, 4, 4, 2, 64, 0, None) == B.EINVAL


def test_host_state_machine_without_a_device():
    L = B.lib()
    rc, h = make()
    assert rc == B.OK and h.value
    assert L.infmllm_stream_len(h) == 0 and L.infmllm_stream_streamed(h) == 0
    base = L.infmllm_stream_workspace_bytes(h)
    assert base > 2 * 2 * 2 * 32 * 64 * 2                       # two copies of K and V at capacity 2B
    assert L.infmllm_stream_set_param(h, B.PARAM_MAX_CHUNK, 4.0) == B.OK
    assert L.infmllm_stream_workspace_bytes(h) < base          # capacity is budget + max_chunk
    assert L.infmllm_stream_set_param(h, B.PARAM_BIAS, -1.0) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_BIAS, float("nan")) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_SCALE, 0.0) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_MAX_CHUNK, 0.0) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_IMPL, 2.0) == B.EINVAL
    assert L.infmllm_stream_set_param(h, 99, 1.0) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_BIAS, 0.5) == B.OK
    # nothing below reaches a device: every call is refused on the host
    one = ctypes.c_void_p(256)
    assert L.infmllm_step(h, one, one, one, 4, one, None, None) == B.ESTATE
    assert "attach" in B.last_error()
    assert L.infmllm_stream_positions(h, one) == B.ESTATE
    assert L.infmllm_stream_export(h, None, None, None, None) == B.ESTATE
    assert L.infmllm_stream_import(h, None, None, None, 0, 0) == B.ESTATE
    assert L.infmllm_stream_attach(h, None, 1 << 30, None) == B.EINVAL
    assert L.infmllm_stream_attach(h, ctypes.c_void_p(257), 1 << 30, None) == B.EINVAL     # misaligned
    assert L.infmllm_stream_attach(h, ctypes.c_void_p(256), 16, None) == B.ENOMEM
    L.infmllm_stream_destroy(h)
    L.infmllm_stream_destroy(None)
    assert L.infmllm_stream_len(None) == -1 and L.infmllm_stream_workspace_bytes(None) == 0


def test_optional_modes_are_checked_and_sized_on_the_host():
    """decoding room, comparison policies, position encoding, batched eviction: parameter checks and the
    workspace they ask for, all without a device"""
    L = B.lib()
    rc, h = make(budget=64, recent=16, heads=4, kv=2, d=128)
    assert rc == B.OK
    assert L.infmllm_stream_set_param(h, B.PARAM_MAX_CHUNK, 32.0) == B.OK
    base = L.infmllm_stream_workspace_bytes(h)
    assert L.infmllm_stream_max_len(h) == 64
    assert L.infmllm_stream_set_param(h, B.PARAM_MAX_DECODE, -1.0) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_MAX_DECODE, 2.5) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_MAX_DECODE, 8.0) == B.OK
    with_decode = L.infmllm_stream_workspace_bytes(h)
    assert with_decode > base and L.infmllm_stream_max_len(h) == 72           # 8 more rows per head + partials
    for bad in (-1.0, 4.0, 1.5):
        assert L.infmllm_stream_set_param(h, B.PARAM_POLICY, bad) == B.EINVAL
    for ok in (1.0, 2.0, 3.0, 0.0):
        assert L.infmllm_stream_set_param(h, B.PARAM_POLICY, ok) == B.OK
    assert L.infmllm_stream_workspace_bytes(h) == with_decode                 # policies need no memory
    for bad in (1.0, 0.5, -10000.0, float("inf")):
        assert L.infmllm_stream_set_param(h, B.PARAM_ROPE_BASE, bad) == B.EINVAL
    assert L.infmllm_stream_set_param(h, B.PARAM_ROPE_BASE, 10000.0) == B.OK
    with_rope = L.infmllm_stream_workspace_bytes(h)
    cap, d, elt = 64 + 8 + 32, 128, 2
    assert with_rope - with_decode >= 2 * cap * d * elt + cap * (d // 2) * 16   # turned keys of 2 heads + the table
    assert L.infmllm_stream_set_param(h, B.PARAM_ROPE_BASE, 0.0) == B.OK
    assert L.infmllm_stream_workspace_bytes(h) == with_decode
    # calls that need an attached stream are refused on the host
    one = ctypes.c_void_p(256)
    assert L.infmllm_decode(h, one, one, one, one) == B.ESTATE
    assert L.infmllm_decode_n(h, one, one, one, one, 3) == B.ESTATE
    assert L.infmllm_decode_n(None, one, one, one, one, 3) == B.EINVAL
    assert L.infmllm_step_attend(h, one, one, one, 4, one, None, None) == B.ESTATE
    assert L.infmllm_stream_pending(h) == 0 and L.infmllm_stream_pending(None) == -1
    arr = (ctypes.c_void_p * 1)(h)
    assert L.infmllm_evict_batched(arr, 1, None, None) == B.ESTATE
    assert L.infmllm_evict_batched(arr, 0, None, None) == B.EINVAL
    assert L.infmllm_evict_batched(None, 1, None, None) == B.EINVAL
    assert L.infmllm_stream_profile_select(h, 0) == B.EINVAL
    assert L.infmllm_stream_profile_select(h, 1 << 20) == B.EINVAL
    assert L.infmllm_stream_profile_select(h, 0xFF) == B.OK
    L.infmllm_stream_destroy(h)


@pytest.mark.gpu
def test_step_argument_checks_after_attach():
    """host-side checks of step on an attached stream: every call is refused before any launch"""
    import torch
    ws = torch.empty(1 << 22, dtype=torch.uint8, device="cuda:0")
    addr = (ws.data_ptr() + 255) // 256 * 256
    L = B.lib()
    rc, h = make()
    assert L.infmllm_stream_set_param(h, B.PARAM_MAX_CHUNK, 8.0) == B.OK
    need = L.infmllm_stream_workspace_bytes(h)
    assert need < (1 << 22) - 256
    assert L.infmllm_stream_attach(h, ctypes.c_void_p(addr), need, None) == B.OK
    assert L.infmllm_stream_attach(h, ctypes.c_void_p(addr), need, None) == B.ESTATE
    assert L.infmllm_stream_set_param(h, B.PARAM_BIAS, 0.1) == B.ESTATE
    one = ctypes.c_void_p(256)
    assert L.infmllm_step(h, None, one, one, 4, one, None, None) == B.EINVAL
    assert L.infmllm_step(h, one, one, one, 0, one, None, None) == B.EINVAL
    assert L.infmllm_step(h, one, one, one, 9, one, None, None) == B.ECAPACITY
    assert L.infmllm_stream_import(h, None, None, None, 17, 17) == B.EINVAL
    assert L.infmllm_stream_len(h) == 0
    L.infmllm_stream_destroy(h)
