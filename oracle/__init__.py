"""fp64 CPU oracle of the Inf-MLLM streaming step (arxiv 2409.09086, Sec. 3.2-3.4, Alg. 1).

TEST INFRASTRUCTURE ONLY: the arithmetic lives in ``infmllm_oracle.c`` (plain C, double
precision); this module compiles it with gcc on first use and wraps it with ctypes.  It is
imported by the tests, by the smoke check and by the benchmark's cpu_baseline leg; the HIP
library and its Python binding never import it and share no code with it.
"""
import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "infmllm_oracle.c")
_LIB = os.path.join(_HERE, "_build", "liboracle.so")
_lock = threading.Lock()
_lib = None


def build(force=False):
    """Compile the C oracle into oracle/_build/liboracle.so (gcc -O2 -fopenmp)."""
    os.makedirs(os.path.dirname(_LIB), exist_ok=True)
    stale = force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            P = ctypes.c_void_p
            lib.oracle_create.restype = P
            lib.oracle_create.argtypes = [ctypes.c_int] * 5 + [ctypes.c_double] * 2
            lib.oracle_destroy.argtypes = [P]
            lib.oracle_len.argtypes = [P]
            lib.oracle_streamed.argtypes = [P]
            lib.oracle_streamed.restype = ctypes.c_int64
            lib.oracle_attend.argtypes = [P, P, P, P, ctypes.c_int, P]
            lib.oracle_decode.argtypes = [P, P, P, P, P]
            lib.oracle_candidates.argtypes = [P]
            lib.oracle_set_policy.argtypes = [P, ctypes.c_int]
            lib.oracle_set_rope.argtypes = [P, ctypes.c_double, ctypes.c_int]
            lib.oracle_accumulated.argtypes = [P, P]
            lib.oracle_scores.argtypes = [P, P, P]
            lib.oracle_select.argtypes = [P, P]
            lib.oracle_commit.argtypes = [P, P, ctypes.c_int]
            lib.oracle_export.argtypes = [P, P, P, P]
            lib.oracle_import.argtypes = [P, P, P, P, ctypes.c_int, ctypes.c_int64]
            _lib = lib
    return _lib


def threads():
    """OpenMP threads the oracle's head-parallel loop uses on this host."""
    return int(_load().oracle_threads())


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


class OracleStream:
    """One layer of one sequence: a size-constrained KV cache fed chunk by chunk.

    budget B = r + R; recent = R (keys always kept); bias = b of Alg. 1; scale = softmax
    scale (default 1/sqrt(head_dim)).
    """

    POLICIES = {"infmllm": 0, "window": 1, "initial_recent": 2, "cumulative": 3}

    ROUND = {None: 0, "bf16": 1, "fp32": 2}

    def __init__(self, budget, recent, heads, kv_heads, head_dim, bias=1e-4, scale=None, policy="infmllm",
                 rope_base=0.0, rope_round=None):
        lib = _load()
        if scale is None:
            scale = 1.0 / np.sqrt(head_dim)
        self._h = lib.oracle_create(budget, recent, heads, kv_heads, head_dim, float(bias), float(scale))
        if not self._h:
            raise ValueError("oracle_create: invalid arguments")
        self.budget, self.recent, self.heads, self.kv_heads, self.head_dim = budget, recent, heads, kv_heads, head_dim
        self.bias, self.scale = float(bias), float(scale)
        self.policy = policy
        if lib.oracle_set_policy(self._h, self.POLICIES[policy]) != 0:
            raise ValueError("oracle_set_policy failed")
        if lib.oracle_set_rope(self._h, float(rope_base), self.ROUND[rope_round]) != 0:
            raise ValueError("oracle_set_rope failed")

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.oracle_destroy(h)

    def __len__(self):
        return _lib.oracle_len(self._h)

    @property
    def streamed(self):
        return _lib.oracle_streamed(self._h)

    # -- the step, in three parts so that a test can adopt another retained set ----------
    def attend(self, q, k, v):
        """Append the chunk, attend, score.  q [L,Hq,d], k/v [L,Hkv,d].  Returns out [L,Hq,d]."""
        q, k, v = _f64(q), _f64(k), _f64(v)
        L = q.shape[0]
        assert q.shape == (L, self.heads, self.head_dim), q.shape
        assert k.shape == (L, self.kv_heads, self.head_dim) and v.shape == k.shape
        out = np.empty_like(q)
        n = _lib.oracle_attend(self._h, _ptr(q), _ptr(k), _ptr(v), L, _ptr(out))
        if n < 0:
            raise RuntimeError("oracle_attend failed: %d" % n)
        self.n = n
        return out

    def scores(self):
        """(S, W') of the step in flight, each [Hkv, c]; None while nothing is evicted."""
        c = _lib.oracle_candidates(self._h)
        if c <= 0:
            return None
        S = np.empty((self.kv_heads, c), dtype=np.float64)
        Wb = np.empty_like(S)
        assert _lib.oracle_scores(self._h, _ptr(S), _ptr(Wb)) == c
        return S, Wb

    def select(self):
        """Alg. 1 l.5-7.  Returns I as an int32 array [Hkv, count]."""
        I = np.empty((self.kv_heads, self.budget), dtype=np.int32)
        count = _lib.oracle_select(self._h, _ptr(I))
        if count < 0:
            raise RuntimeError("oracle_select failed: %d" % count)
        return np.ascontiguousarray(I[:, :count])

    def commit(self, I):
        """Alg. 1 l.8 with the given index lists (normally select()'s)."""
        I = np.asarray(I, dtype=np.int32)
        count = I.shape[1]
        full = np.zeros((self.kv_heads, self.budget), dtype=np.int32)
        full[:, :count] = I
        rc = _lib.oracle_commit(self._h, _ptr(full), count)
        if rc != 0:
            raise RuntimeError("oracle_commit failed: %d" % rc)

    def step(self, q, k, v, force_retained=None):
        """One whole streaming step.  Returns (out, I).  force_retained replaces the selection."""
        out = self.attend(q, k, v)
        I = self.select() if force_retained is None else np.asarray(force_retained, dtype=np.int32)
        self.commit(I)
        return out, I

    def decode(self, q, k, v):
        """One decoding step: append the token's k, v ([1,Hkv,d]), attend with q ([1,Hq,d]); nothing
        is evicted, the cache may exceed the budget until the next chunk arrives.  Returns out [1,Hq,d]."""
        q, k, v = _f64(q), _f64(k), _f64(v)
        assert q.shape == (1, self.heads, self.head_dim) and k.shape == v.shape == (1, self.kv_heads, self.head_dim)
        out = np.empty_like(q)
        n = _lib.oracle_decode(self._h, _ptr(q), _ptr(k), _ptr(v), _ptr(out))
        if n < 0:
            raise RuntimeError("oracle_decode failed: %d" % n)
        return out

    def accumulated(self):
        """[Hkv, t] accumulated scores of the cached rows (cumulative policy; zeros otherwise)."""
        A = np.empty((self.kv_heads, len(self)), dtype=np.float64)
        _lib.oracle_accumulated(self._h, _ptr(A))
        return A

    # -- state ------------------------------------------------------------------------------
    def export(self):
        t = len(self)
        K = np.empty((self.kv_heads, t, self.head_dim), dtype=np.float64)
        V = np.empty_like(K)
        pos = np.empty((self.kv_heads, t), dtype=np.int64)
        _lib.oracle_export(self._h, _ptr(K), _ptr(V), _ptr(pos))
        return K, V, pos

    def load(self, K, V, pos, streamed):
        K, V = _f64(K), _f64(V)
        pos = np.ascontiguousarray(np.asarray(pos, dtype=np.int64))
        rc = _lib.oracle_import(self._h, _ptr(K), _ptr(V), _ptr(pos), K.shape[1], int(streamed))
        if rc != 0:
            raise RuntimeError("oracle_import failed: %d" % rc)
