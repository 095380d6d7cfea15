"""Seeded synthetic streams shaped like the paper's workloads.

This module only draws random inputs; it holds none of the method's arithmetic, so both
the HIP path and the test oracle may be fed from it.  The paper evaluates on text corpora
and video-QA sets (Sec. 4.1-4.4) that are not available here; these streams borrow only
their shapes: a 7B-class layer (32 heads x 128), a 2K-8K cache, chunks of one prompt or one
video frame's visual tokens, streams of up to 4M tokens.

Every tensor is drawn in fp32 and rounded once to the stream's dtype; whoever consumes it
(GPU or CPU) sees the same bits.  Tensors are torch CPU tensors laid out token-major:
q [L, heads, head_dim], k and v [L, kv_heads, head_dim].
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class StreamConfig:
    name: str
    dtype: str            # "fp32" | "bf16"
    layers: int
    heads: int
    kv_heads: int
    head_dim: int
    budget: int
    recent: int
    chunk: int            # tokens per ordinary chunk
    steps: int            # chunks per layer in the full stream
    bias: float
    seed: int
    sigma: float = 1.0                 # std of q/k/v entries
    heavy_frac: float = 0.0            # fraction of tokens whose key gets a shared offset
    heavy_offset: float = 0.0          # offset added to every dimension of such a key
    text_every: int = 0                # every text_every-th chunk carries extra text tokens
    text_len: int = 0
    ar_rho: float = 0.0                # AR(1) coefficient across chunks (video frames)
    recur_period: int = 0              # a fixed bank of keys recurs every recur_period tokens
    recur_len: int = 0

    def chunk_len(self, step: int) -> int:
        if self.text_every and (step + 1) % self.text_every == 0:
            return self.chunk + self.text_len
        return self.chunk

    @property
    def max_chunk(self) -> int:
        return self.chunk + (self.text_len if self.text_every else 0)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16


CONFIGS = {
    # tiny fp32 stream the CPU oracle finishes in seconds
    "cfg1": StreamConfig("cfg1", "fp32", 1, 4, 4, 64, 256, 64, 64, 8, 1e-4, 1),
    # Llama-2-7B-shaped layer, heavy-hitter key columns
    "cfg2": StreamConfig("cfg2", "bf16", 1, 32, 32, 128, 2048, 512, 512, 64, 1e-4, 2,
                         sigma=0.5, heavy_frac=0.01, heavy_offset=1.5),
    # GQA 8B-shaped layer
    "cfg3": StreamConfig("cfg3", "bf16", 1, 32, 8, 128, 4096, 1024, 1024, 256, 1e-4, 3),
    # video stream: one frame of 576 visual tokens per chunk, a 32-token question every 10 frames
    "cfg4": StreamConfig("cfg4", "bf16", 32, 32, 32, 128, 4096, 1152, 576, 3600, 1e-2, 4,
                         text_every=10, text_len=32, ar_rho=0.95),
    # long-text stress: 4M tokens, a bank of keys recurring every 100k tokens
    "cfg5": StreamConfig("cfg5", "bf16", 32, 32, 32, 128, 8192, 2048, 2048, 2048, 1e-4, 5,
                         heavy_offset=1.5, recur_period=100_000, recur_len=128),
}


def _rng(seed, *key):
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, *[int(x) for x in key]])))


def _normal(rng, shape):
    return rng.standard_normal(size=shape, dtype=np.float32)


class ChunkStream:
    """Iterator over the chunks of one layer of a configured stream.

    ``next(stream)`` returns (q, k, v) for the next step.  Chunks depend on (seed, layer,
    step) only, apart from the AR(1) video stream, which carries the previous frame.
    """

    def __init__(self, cfg: StreamConfig, layer: int = 0, start_step: int = 0):
        self.cfg, self.layer, self.step = cfg, layer, start_step
        self.tokens = sum(cfg.chunk_len(s) for s in range(start_step))
        self._prev = None
        if cfg.recur_period:
            rng = _rng(cfg.seed, layer, 1 << 30)
            self._bank = cfg.sigma * _normal(rng, (cfg.recur_len, cfg.kv_heads, cfg.head_dim)) + cfg.heavy_offset
        if cfg.ar_rho and start_step:
            raise ValueError("the AR(1) stream has to be generated from its first frame")

    def __iter__(self):
        return self

    def __next__(self):
        cfg, s = self.cfg, self.step
        L = cfg.chunk_len(s)
        rng = _rng(cfg.seed, self.layer, s)
        shapes = [(cfg.chunk, cfg.heads, cfg.head_dim), (cfg.chunk, cfg.kv_heads, cfg.head_dim),
                  (cfg.chunk, cfg.kv_heads, cfg.head_dim)]
        eps = [_normal(rng, sh) for sh in shapes]
        if cfg.ar_rho:
            # x_f = rho x_{f-1} + sqrt(1 - rho^2) eps_f, elementwise on the frame block
            if self._prev is None:
                cur = eps
            else:
                a, c = np.float32(cfg.ar_rho), np.float32(np.sqrt(1.0 - cfg.ar_rho ** 2))
                cur = [a * p + c * e for p, e in zip(self._prev, eps)]
            self._prev = cur
        else:
            cur = eps
        q, k, v = [cfg.sigma * x for x in cur]
        if L > cfg.chunk:  # trailing text tokens, iid
            extra = L - cfg.chunk
            tq = cfg.sigma * _normal(rng, (extra, cfg.heads, cfg.head_dim))
            tk = cfg.sigma * _normal(rng, (extra, cfg.kv_heads, cfg.head_dim))
            tv = cfg.sigma * _normal(rng, (extra, cfg.kv_heads, cfg.head_dim))
            q, k, v = np.concatenate([q, tq]), np.concatenate([k, tk]), np.concatenate([v, tv])
        planted = np.zeros(L, dtype=bool)                   # tokens whose key was planted (offset or bank)
        if cfg.heavy_frac:
            heavy = rng.random(L) < cfg.heavy_frac          # per token, shared by all heads
            k = k + np.float32(cfg.heavy_offset) * heavy[:, None, None].astype(np.float32)
            planted |= heavy
        if cfg.recur_period:
            pos = self.tokens + np.arange(L)
            off = pos % cfg.recur_period
            hit = (off < cfg.recur_len) & (pos >= 0)
            if hit.any():
                k = k.copy()
                k[hit] = self._bank[off[hit]]
                planted |= hit
        self.last_planted = planted                         # for whoever wants to report what became of them
        self.step += 1
        self.tokens += L
        dt = cfg.torch_dtype
        return tuple(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(dt) for x in (q, k, v))


def random_chunk(seed, L, heads, kv_heads, head_dim, dtype="fp32", sigma=1.0, key=0):
    """A free-standing iid Gaussian chunk for unit tests."""
    rng = _rng(seed, key)
    dt = torch.float32 if dtype == "fp32" else torch.bfloat16
    mk = lambda h: torch.from_numpy(sigma * _normal(rng, (L, h, head_dim))).to(dt)
    return mk(heads), mk(kv_heads), mk(kv_heads)
