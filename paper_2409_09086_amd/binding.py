"""ctypes binding of libinfmllm.so: same names as include/infmllm.h, argument marshalling only.

PyTorch is used for device memory (the caller's tensors, the workspace) and for the HIP
stream handle; every step of the path runs in the library's kernels.  If the shared library
is missing the import of this module's functions fails loudly -- there is no fallback.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libinfmllm.so")

BF16, FP32 = 0, 1
OK, EINVAL, ENOMEM, ECAPACITY, ESTATE, EHIP = 0, -1, -2, -3, -4, -5
PARAM_BIAS, PARAM_SCALE, PARAM_MAX_CHUNK, PARAM_IMPL, PARAM_MAX_DECODE, PARAM_POLICY, PARAM_ROPE_BASE, PARAM_ATTN_TILE = 0, 1, 2, 3, 4, 5, 6, 7
POLICIES = {"infmllm": 0, "window": 1, "initial_recent": 2, "cumulative": 3}

EXPORTS = [
    "infmllm_stream_create", "infmllm_stream_set_param", "infmllm_stream_workspace_bytes",
    "infmllm_stream_attach", "infmllm_step", "infmllm_stream_len", "infmllm_stream_streamed",
    "infmllm_stream_positions", "infmllm_stream_export", "infmllm_stream_import",
    "infmllm_stream_last_scores", "infmllm_last_error", "infmllm_stream_destroy",
    "infmllm_stream_profile", "infmllm_stream_profile_read", "infmllm_decode", "infmllm_decode_n", "infmllm_stream_max_len",
    "infmllm_step_attend", "infmllm_stream_pending", "infmllm_evict_batched", "infmllm_stream_profile_select",
    "infmllm_stream_attach_static",
]
STATIC_WORKSPACE_BYTES = 64 << 20
KERNELS = ["append", "attn", "score", "select", "compact", "decode", "rope", "evict"]

_lib = None


class InfMLLMError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("infmllm error %d: %s" % (code, msg))
        self.code = code


def lib():
    """Loads libinfmllm.so (built in-tree by paper_2409_09086_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -m paper_2409_09086_amd.build` (hipcc, gfx950)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        P, I, D = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        L.infmllm_stream_create.argtypes = [I, I, I, I, I, I, ctypes.POINTER(P)]
        L.infmllm_stream_set_param.argtypes = [P, I, D]
        L.infmllm_stream_workspace_bytes.argtypes = [P]
        L.infmllm_stream_workspace_bytes.restype = ctypes.c_size_t
        L.infmllm_stream_attach.argtypes = [P, P, ctypes.c_size_t, P]
        L.infmllm_stream_attach_static.argtypes = [P, P]
        L.infmllm_step.argtypes = [P, P, P, P, I, P, P, P]
        L.infmllm_decode.argtypes = [P, P, P, P, P]
        L.infmllm_decode_n.argtypes = [P, P, P, P, P, ctypes.c_int]
        L.infmllm_step_attend.argtypes = [P, P, P, P, I, P, P, P]
        L.infmllm_stream_pending.argtypes = [P]
        L.infmllm_evict_batched.argtypes = [ctypes.POINTER(P), I, ctypes.POINTER(P), ctypes.POINTER(P)]
        L.infmllm_stream_max_len.argtypes = [P]
        L.infmllm_stream_len.argtypes = [P]
        L.infmllm_stream_streamed.argtypes = [P]
        L.infmllm_stream_streamed.restype = ctypes.c_int64
        L.infmllm_stream_positions.argtypes = [P, P]
        L.infmllm_stream_export.argtypes = [P, P, P, P, P]
        L.infmllm_stream_import.argtypes = [P, P, P, P, I, ctypes.c_int64]
        L.infmllm_stream_last_scores.argtypes = [P, P, ctypes.POINTER(I)]
        L.infmllm_stream_profile.argtypes = [P, I]
        L.infmllm_stream_profile_select.argtypes = [P, ctypes.c_uint]
        L.infmllm_stream_profile_read.argtypes = [P, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(I)]
        L.infmllm_last_error.restype = ctypes.c_char_p
        L.infmllm_stream_destroy.argtypes = [P]
        L.infmllm_stream_destroy.restype = None
        _lib = L
    return _lib


def last_error():
    return lib().infmllm_last_error().decode()


def _check(rc):
    if rc != OK:
        raise InfMLLMError(rc, last_error())


def _dev_ptr(t, dtype=None, shape=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous device tensor" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must have dtype %s (got %s)" % (name, dtype, t.dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s (got %s)" % (name, tuple(shape), tuple(t.shape)))
    return ctypes.c_void_p(t.data_ptr())


class Stream:
    """infmllm_stream_t with its workspace: one layer of one sequence on one GPU."""

    def __init__(self, budget, recent, heads, kv_heads, head_dim, dtype=torch.bfloat16, bias=None, scale=None,
                 max_chunk=None, impl=None, max_decode=None, policy=None, rope_base=None, attn_tile=None,
                 device="cuda:0", hip_stream=None, static_workspace=False):
        L = lib()
        self.dtype = dtype
        code = {torch.bfloat16: BF16, torch.float32: FP32}.get(dtype)
        if code is None:
            raise ValueError("dtype must be torch.bfloat16 or torch.float32")
        h = ctypes.c_void_p()
        _check(L.infmllm_stream_create(budget, recent, heads, kv_heads, head_dim, code, ctypes.byref(h)))
        self._h = h
        self.budget, self.recent, self.heads, self.kv_heads, self.head_dim = budget, recent, heads, kv_heads, head_dim
        for which, val in ((PARAM_BIAS, bias), (PARAM_SCALE, scale), (PARAM_MAX_CHUNK, max_chunk), (PARAM_IMPL, impl),
                           (PARAM_MAX_DECODE, max_decode),
                           (PARAM_POLICY, None if policy is None else POLICIES[policy]),
                           (PARAM_ROPE_BASE, rope_base), (PARAM_ATTN_TILE, attn_tile)):
            if val is not None:
                _check(L.infmllm_stream_set_param(self._h, which, float(val)))
        self.device = torch.device(device)
        nbytes = L.infmllm_stream_workspace_bytes(self._h)
        with torch.cuda.device(self.device):
            self.hip_stream = hip_stream if hip_stream is not None else torch.cuda.current_stream(self.device).cuda_stream
            if static_workspace:
                # infmllm_stream_attach_static: the workspace is the library's own per-device array
                self.workspace = None
                rc = L.infmllm_stream_attach_static(self._h, ctypes.c_void_p(self.hip_stream))
            else:
                self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
                base = self.workspace.data_ptr()
                aligned = (base + 255) // 256 * 256
                rc = L.infmllm_stream_attach(self._h, ctypes.c_void_p(aligned), nbytes, ctypes.c_void_p(self.hip_stream))
            if rc != OK:
                h, self._h = self._h, None
                L.infmllm_stream_destroy(h)
                _check(rc)

    def __del__(self):
        self.close()

    def close(self):
        """infmllm_stream_destroy (also releases the library's static workspace if this stream holds it)."""
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.infmllm_stream_destroy(h)

    def __len__(self):
        return lib().infmllm_stream_len(self._h)

    @property
    def streamed(self):
        return lib().infmllm_stream_streamed(self._h)

    def step(self, q, k, v, out=None, retained=None, n_retained=None, report=True):
        """infmllm_step.  Returns (out, retained, n_retained); the last two are device tensors
        (or None with report=False).  Nothing is synchronised."""
        Lc = q.shape[0]
        _dev_ptr(q, self.dtype, (Lc, self.heads, self.head_dim), "q")
        _dev_ptr(k, self.dtype, (Lc, self.kv_heads, self.head_dim), "k")
        _dev_ptr(v, self.dtype, (Lc, self.kv_heads, self.head_dim), "v")
        if out is None:
            out = torch.empty_like(q)
        if report and retained is None:
            retained = torch.empty((self.kv_heads, self.budget), dtype=torch.int32, device=q.device)
        if report and n_retained is None:
            n_retained = torch.empty((1,), dtype=torch.int32, device=q.device)
        _check(lib().infmllm_step(self._h, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v), Lc,
                                  _dev_ptr(out, self.dtype, q.shape, "out"),
                                  _dev_ptr(retained, torch.int32, (self.kv_heads, self.budget), "retained"),
                                  _dev_ptr(n_retained, torch.int32, None, "n_retained")))
        return out, retained, n_retained

    def step_attend(self, q, k, v, out=None, retained=None, n_retained=None, report=True):
        """infmllm_step_attend: the step up to the scores.  If the chunk fits into the budget the step
        is complete and (out, retained, n_retained) are as from step(); otherwise the eviction is
        left pending (self.pending) for evict_batched(), retained / n_retained are returned unwritten,
        and q, k, v are kept alive here until that call."""
        Lc = q.shape[0]
        _dev_ptr(q, self.dtype, (Lc, self.heads, self.head_dim), "q")
        _dev_ptr(k, self.dtype, (Lc, self.kv_heads, self.head_dim), "k")
        _dev_ptr(v, self.dtype, (Lc, self.kv_heads, self.head_dim), "v")
        if out is None:
            out = torch.empty_like(q)
        if report and retained is None:
            retained = torch.empty((self.kv_heads, self.budget), dtype=torch.int32, device=q.device)
        if report and n_retained is None:
            n_retained = torch.empty((1,), dtype=torch.int32, device=q.device)
        _check(lib().infmllm_step_attend(self._h, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v), Lc,
                                         _dev_ptr(out, self.dtype, q.shape, "out"),
                                         _dev_ptr(retained, torch.int32, (self.kv_heads, self.budget), "retained"),
                                         _dev_ptr(n_retained, torch.int32, None, "n_retained")))
        self._held = (q, k, v, retained, n_retained) if self.pending else None
        return out, retained, n_retained

    @property
    def pending(self):
        return lib().infmllm_stream_pending(self._h) == 1

    def decode(self, q, k, v, out=None):
        """infmllm_decode: q [1,heads,d], k/v [1,kv_heads,d].  Returns out [1,heads,d]."""
        _dev_ptr(q, self.dtype, (1, self.heads, self.head_dim), "q")
        _dev_ptr(k, self.dtype, (1, self.kv_heads, self.head_dim), "k")
        _dev_ptr(v, self.dtype, (1, self.kv_heads, self.head_dim), "v")
        if out is None:
            out = torch.empty_like(q)
        _check(lib().infmllm_decode(self._h, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v),
                                    _dev_ptr(out, self.dtype, q.shape, "out")))
        return out

    def decode_n(self, q, k, v, out=None):
        """infmllm_decode_n: q [n,heads,d], k/v [n,kv_heads,d], one decoding step per row.  Returns out [n,heads,d]."""
        n = q.shape[0]
        _dev_ptr(q, self.dtype, (n, self.heads, self.head_dim), "q")
        _dev_ptr(k, self.dtype, (n, self.kv_heads, self.head_dim), "k")
        _dev_ptr(v, self.dtype, (n, self.kv_heads, self.head_dim), "v")
        if out is None:
            out = torch.empty_like(q)
        _check(lib().infmllm_decode_n(self._h, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v),
                                      _dev_ptr(out, self.dtype, q.shape, "out"), n))
        return out

    def decode_ptrs(self, q, k, v, out):
        """infmllm_decode on raw device addresses (ints) of buffers the caller has already checked:
        the per-call tensor checks of decode() cost more than the kernels of one token."""
        _check(lib().infmllm_decode(self._h, q, k, v, out))

    @property
    def max_len(self):
        return lib().infmllm_stream_max_len(self._h)

    def positions(self):
        pos = torch.empty((self.kv_heads, self.max_len), dtype=torch.int32, device=self.device)
        _check(lib().infmllm_stream_positions(self._h, _dev_ptr(pos)))
        return pos[:, : len(self)]

    def export(self):
        n = len(self)
        K = torch.empty((self.kv_heads, n, self.head_dim), dtype=self.dtype, device=self.device)
        V = torch.empty_like(K)
        pos = torch.empty((self.kv_heads, n), dtype=torch.int32, device=self.device)
        score = torch.empty((self.kv_heads, n), dtype=torch.float32, device=self.device)
        _check(lib().infmllm_stream_export(self._h, _dev_ptr(K), _dev_ptr(V), _dev_ptr(pos), _dev_ptr(score)))
        return K, V, pos, score

    def load(self, K, V, pos, streamed):
        n = K.shape[1]
        _check(lib().infmllm_stream_import(
            self._h, _dev_ptr(K, self.dtype, (self.kv_heads, n, self.head_dim), "K"),
            _dev_ptr(V, self.dtype, (self.kv_heads, n, self.head_dim), "V"),
            _dev_ptr(pos, torch.int32, (self.kv_heads, n), "pos"), n, int(streamed)))

    def profile(self, max_steps):
        _check(lib().infmllm_stream_profile(self._h, int(max_steps)))

    def profile_select(self, names):
        """Record events only for these intervals (names from KERNELS) in the steps profiled from now on."""
        mask = 0
        for n in names:
            mask |= 1 << KERNELS.index(n)
        _check(lib().infmllm_stream_profile_select(self._h, mask))

    def profile_read(self):
        """{kernel: (total ms, launches)} of the steps recorded since the last read."""
        ms = (ctypes.c_float * len(KERNELS))()
        cnt = (ctypes.c_int * len(KERNELS))()
        _check(lib().infmllm_stream_profile_read(self._h, ms, cnt))
        return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(KERNELS)}

    def last_scores(self):
        """Biased scores W' [kv_heads, c] of the most recent evicting step, or None."""
        c = ctypes.c_int(0)
        _check(lib().infmllm_stream_last_scores(self._h, None, ctypes.byref(c)))
        if c.value == 0:
            return None
        w = torch.empty((self.kv_heads, c.value), dtype=torch.float32, device=self.device)
        _check(lib().infmllm_stream_last_scores(self._h, _dev_ptr(w), ctypes.byref(c)))
        return w


def evict_batched(streams):
    """infmllm_evict_batched over Stream objects that all have an eviction pending (the layers of a
    model after step_attend).  The retained / n_retained tensors handed to (or made by) each
    stream's step_attend receive the result.  Nothing is synchronised."""
    n = len(streams)
    P = ctypes.c_void_p
    hs = (P * n)(*[s._h for s in streams])
    held = [getattr(s, "_held", None) for s in streams]
    ret = (P * n)(*[(h[3].data_ptr() if h is not None and h[3] is not None else None) for h in held])
    cnt = (P * n)(*[(h[4].data_ptr() if h is not None and h[4] is not None else None) for h in held])
    _check(lib().infmllm_evict_batched(hs, n, ret, cnt))
    # the gather is enqueued: torch's stream-ordered allocator may now recycle the chunk tensors
    for s in streams:
        s._held = None
