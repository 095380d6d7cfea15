"""CPU-only checks of the seeded input generators and of the oracle's stored regression values."""
import dataclasses
import importlib.util
import os

import numpy as np
import torch

from paper_2409_09086_amd.workloads import CONFIGS, ChunkStream, random_chunk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def small(name, **kw):
    return dataclasses.replace(CONFIGS[name], **kw)


def test_chunks_are_deterministic_and_shaped():
    cfg = small("cfg2", heads=4, kv_heads=4, chunk=96)
    a = [next(ChunkStream(cfg)) for _ in range(2)]
    for x, y in zip(a[0], a[1]):
        assert x.dtype == torch.bfloat16 and torch.equal(x, y)
    q, k, v = a[0]
    assert q.shape == (96, 4, 128) and k.shape == v.shape == (96, 4, 128)
    s = ChunkStream(cfg)
    first, second = next(s), next(s)
    assert not torch.equal(first[0], second[0])
    again = ChunkStream(cfg, start_step=1)
    assert torch.equal(next(again)[1], second[1])              # chunks depend on (seed, layer, step) only
    other_layer = next(ChunkStream(cfg, layer=1))
    assert not torch.equal(other_layer[0], first[0])


def test_heavy_hitter_keys_carry_the_shared_offset():
    cfg = small("cfg2", heads=2, kv_heads=2, chunk=4000, heavy_frac=0.05)
    q, k, v = next(ChunkStream(cfg))
    row_mean = k.float().mean(dim=(1, 2))                      # per token over heads and dims
    heavy = row_mean > 0.75
    assert 0.03 < heavy.float().mean() < 0.07
    assert abs(row_mean[heavy].mean() - 1.5) < 0.05 and abs(row_mean[~heavy].mean()) < 0.01
    assert abs(q.float().std() - 0.5) < 0.01 and abs(v.float().std() - 0.5) < 0.01


def test_video_stream_is_ar1_with_text_every_tenth_chunk():
    cfg = small("cfg4", heads=2, kv_heads=2, chunk=64, text_len=8)
    s = ChunkStream(cfg)
    chunks = [next(s) for _ in range(10)]
    assert [c[0].shape[0] for c in chunks] == [64] * 9 + [72]
    a, b = chunks[3][1].float().flatten(), chunks[4][1].float().flatten()
    rho = float(np.corrcoef(a.numpy(), b.numpy())[0, 1])
    assert abs(rho - 0.95) < 0.02
    assert abs(chunks[8][1].float().std() - 1.0) < 0.05        # stationary
    frame, text = chunks[9][1][:64].float().flatten(), chunks[8][1].float().flatten()
    assert abs(float(np.corrcoef(frame.numpy(), text.numpy())[0, 1]) - 0.95) < 0.02


def test_recurring_key_bank_returns_at_every_period():
    cfg = small("cfg5", heads=2, kv_heads=2, chunk=100, recur_period=250, recur_len=16)
    s = ChunkStream(cfg)
    ks = torch.cat([next(s)[1] for _ in range(6)])             # 600 tokens
    bank = ks[0:16]
    assert torch.equal(ks[250:266], bank) and torch.equal(ks[500:516], bank)
    assert not torch.equal(ks[16:32], ks[266:282])
    assert abs(bank.float().mean() - 1.5) < 0.1                # the bank carries the heavy offset


def test_random_chunk_is_seeded():
    a, b = random_chunk(3, 10, 4, 2, 64, "fp32"), random_chunk(3, 10, 4, 2, 64, "fp32")
    assert all(torch.equal(x, y) for x, y in zip(a, b)) and a[0].dtype == torch.float32
    assert a[0].shape == (10, 4, 64) and a[1].shape == (10, 2, 64)


def test_oracle_reproduces_its_stored_cfg1_values():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(ROOT, "tests", "golden", "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    lines = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "cfg1_oracle.txt")) if not l.startswith("#")]
    i = 0
    while i < len(lines):
        assert lines[i][0] == "bias"
        bias = float(lines[i][1])
        sums = np.array([float(x) for x in lines[i + 1][1:]])
        pos = np.array([[int(x) for x in lines[i + 2 + h][2:]] for h in range(4)])
        got_pos, got_sums = mg.compute(bias)
        assert (got_pos == pos).all()
        np.testing.assert_allclose(got_sums, sums, rtol=1e-9)
        i += 6
