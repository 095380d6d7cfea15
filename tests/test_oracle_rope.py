"""Pins for the oracle's cache-relative rotary position encoding (Sec. 3.4 "length extrapolation"; Sec. 4.1:
the evaluated models use rotary embeddings).  The rotation is re-stated here with complex numbers
(a pair (x[i], x[i+d/2]) is the complex number x[i] + 1j x[i+d/2], turned by exp(1j p base^(-2i/d))) and
fed to torch's fp64 attention routine; the rounding to the stream type is done by torch's own conversion.
No GPU needed."""
import numpy as np
import pytest
import torch

from oracle import OracleStream


def rand(rng, *shape):
    return rng.standard_normal(shape)


def rotate(x, pos, base, round_to=None):
    """x [N, H, d], pos [N] -> rotated copy, via complex multiplication."""
    d = x.shape[-1]
    half = d // 2
    z = x[..., :half] + 1j * x[..., half:]
    theta = base ** (-2.0 * np.arange(half) / d)
    z = z * np.exp(1j * np.asarray(pos, dtype=np.float64)[:, None, None] * theta[None, None, :])
    y = np.concatenate([z.real, z.imag], axis=-1)
    if round_to == "bf16":
        y = torch.from_numpy(y).float().bfloat16().double().numpy()
    if round_to == "fp32":
        y = torch.from_numpy(y).float().double().numpy()
    return y


def attend_numpy(q, K, V, t, scale):
    """q [L,Hq,d] (already rotated), K/V [n,Hkv,d] (K already rotated), causal inside the chunk -> [L,Hq,d]."""
    L, Hq, d = q.shape
    n, Hkv = K.shape[0], K.shape[1]
    out = np.zeros_like(q)
    for g in range(Hq):
        h = g // (Hq // Hkv)
        s = scale * q[:, g] @ K[:, h].T
        mask = np.arange(n)[None, :] > (t + np.arange(L))[:, None]
        s[mask] = -np.inf
        w = np.exp(s - s.max(axis=1, keepdims=True))
        w /= w.sum(axis=1, keepdims=True)
        out[:, g] = w @ V[:, h]
    return out


def sdpa_causal(q, k, v, scale):
    Hq, Hkv = q.shape[1], k.shape[1]
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.from_numpy(v).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


@pytest.mark.parametrize("Hq,Hkv,d,chunks", [(4, 2, 16, [5, 7, 1, 12]), (2, 2, 8, [9, 9])])
def test_without_eviction_it_is_ordinary_rotary_attention(Hq, Hkv, d, chunks):
    """While nothing is evicted the cache row of a token is its stream position, so the result is
    one-shot causal attention over rotary-encoded q and k (library routine, fp64)."""
    rng = np.random.default_rng(20)
    N, base, scale = sum(chunks), 10000.0, 0.31
    q, k, v = rand(rng, N, Hq, d), rand(rng, N, Hkv, d), rand(rng, N, Hkv, d)
    want = sdpa_causal(rotate(q, np.arange(N), base), rotate(k, np.arange(N), base), v, scale)
    o = OracleStream(N, N // 2, Hq, Hkv, d, scale=scale, rope_base=base)
    got, at = [], 0
    for L in chunks:
        got.append(o.step(q[at:at + L], k[at:at + L], v[at:at + L])[0])
        at += L
    assert np.allclose(np.concatenate(got), want, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("round_to", [None, "bf16", "fp32"])
def test_after_eviction_positions_are_cache_rows_not_stream_positions(round_to):
    rng = np.random.default_rng(21)
    Hq, Hkv, d, B, R, base, scale = 4, 2, 16, 12, 4, 500.0, 0.4
    o = OracleStream(B, R, Hq, Hkv, d, scale=scale, rope_base=base, rope_round=round_to)
    for L in (8, 8, 5):
        o.step(rand(rng, L, Hq, d), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))
    Kc, Vc, pos = o.export()                                      # [Hkv, t, d], raw (unrotated) rows
    t = Kc.shape[1]
    assert t == B and not (pos[0] == np.arange(t)).all()          # rows have moved: row != stream position
    L = 6
    q, k, v = rand(rng, L, Hq, d), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d)
    got = o.attend(q, k, v)
    K = np.concatenate([Kc.transpose(1, 0, 2), k])                # [n, Hkv, d]
    V = np.concatenate([Vc.transpose(1, 0, 2), v])
    n = t + L
    want = attend_numpy(rotate(q, t + np.arange(L), base, round_to), rotate(K, np.arange(n), base, round_to), V, t, scale)
    tol = dict(rtol=1e-10, atol=1e-12)
    assert np.allclose(got, want, **tol)
    # per-head stream positions would give something else (so the test can tell the two readings apart)
    spos = np.concatenate([pos[0], o.streamed - L + np.arange(L)])
    other = attend_numpy(rotate(q, o.streamed - L + np.arange(L), base, round_to), rotate(K, spos, base, round_to), V, t, scale)
    assert not np.allclose(got, other, rtol=1e-6, atol=1e-8)


def test_rounding_to_bf16_changes_the_result_and_matches_the_library_conversion():
    rng = np.random.default_rng(22)
    a = OracleStream(32, 8, 2, 2, 8, rope_base=10000.0)
    b = OracleStream(32, 8, 2, 2, 8, rope_base=10000.0, rope_round="bf16")
    q, k, v = rand(rng, 10, 2, 8), rand(rng, 10, 2, 8), rand(rng, 10, 2, 8)
    oa, ob = a.step(q, k, v)[0], b.step(q, k, v)[0]
    assert not np.allclose(oa, ob, rtol=1e-6, atol=1e-9)
    want = attend_numpy(rotate(q, np.arange(10), 10000.0, "bf16"), rotate(k, np.arange(10), 10000.0, "bf16"), v, 0, 1 / np.sqrt(8))
    assert np.allclose(ob, want, rtol=1e-10, atol=1e-12)


def test_decode_token_is_rotated_to_its_cache_row():
    rng = np.random.default_rng(23)
    Hq, Hkv, d, base = 2, 1, 8, 100.0
    o = OracleStream(16, 4, Hq, Hkv, d, scale=0.5, rope_base=base)
    q, k, v = rand(rng, 7, Hq, d), rand(rng, 7, Hkv, d), rand(rng, 7, Hkv, d)
    o.step(q, k, v)
    q1, k1, v1 = rand(rng, 1, Hq, d), rand(rng, 1, Hkv, d), rand(rng, 1, Hkv, d)
    got = o.decode(q1, k1, v1)
    K, V = np.concatenate([k, k1]), np.concatenate([v, v1])
    want = attend_numpy(rotate(q1, [7], base), rotate(K, np.arange(8), base), V, 7, 0.5)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)


def test_scores_use_the_rotated_logits():
    """Alg. 1 l.1 column means come from the same weights: re-derived from the numpy attention matrix."""
    rng = np.random.default_rng(24)
    Hq, Hkv, d, B, R, base, scale = 2, 2, 8, 10, 3, 50.0, 0.6
    o = OracleStream(B, R, Hq, Hkv, d, bias=0.0, scale=scale, rope_base=base)
    o.step(rand(rng, 10, Hq, d), rand(rng, 10, Hkv, d), rand(rng, 10, Hkv, d))
    Kc = o.export()[0]
    L = 4
    q, k = rand(rng, L, Hq, d), rand(rng, L, Hkv, d)
    o.attend(q, k, rand(rng, L, Hkv, d))
    S = o.scores()[0]
    n, c = B + L, B + L - R
    K = rotate(np.concatenate([Kc.transpose(1, 0, 2), k]), np.arange(n), base)
    qr = rotate(q, B + np.arange(L), base)
    for h in range(Hkv):
        s = scale * qr[:, h] @ K[:, h].T
        s[np.arange(n)[None, :] > (B + np.arange(L))[:, None]] = -np.inf
        w = np.exp(s - s.max(axis=1, keepdims=True))
        w /= w.sum(axis=1, keepdims=True)
        assert np.allclose(S[h], w[L - min(R, L):, :c].mean(axis=0), rtol=1e-10, atol=1e-14)


def test_rope_arguments_are_checked():
    with pytest.raises(ValueError):
        OracleStream(8, 2, 1, 1, 4, rope_base=0.5)
    with pytest.raises(ValueError):
        OracleStream(8, 2, 1, 1, 5, rope_base=100.0)              # odd head_dim
    OracleStream(8, 2, 1, 1, 4, rope_base=0.0)
