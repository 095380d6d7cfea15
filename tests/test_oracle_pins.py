"""Pins for the fp64 oracle: each test fixes a part of it to something other than itself --
a library routine (torch's scaled_dot_product_attention in fp64), a closed form, an
invariant of Alg. 1, or brute force on tiny inputs.  None of these needs a GPU.

Citations are to the paper (arxiv 2409.09086): Sec. 3.2 (eviction), Sec. 3.3 (bias),
Alg. 1 (the eight lines of the algorithm).
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import OracleStream


def rand(rng, *shape):
    return rng.standard_normal(shape)


def sdpa_causal(q, k, v, scale):
    """One-shot causal attention over a whole stream with torch's fp64 library routine.
    q [N,Hq,d], k/v [N,Hkv,d] -> [N,Hq,d]."""
    Hq, Hkv = q.shape[1], k.shape[1]
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.from_numpy(v).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


# ---------------------------------------------------------------------------------------
# P1  attention (Sec. 3.2: L new queries against t cached keys plus the new keys)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("Hq,Hkv,d,chunks", [(4, 4, 16, [5, 7, 1, 12]), (8, 2, 8, [3, 3, 9]), (2, 1, 32, [16])])
def test_no_eviction_equals_one_shot_causal_attention(Hq, Hkv, d, chunks):
    rng = np.random.default_rng(10)
    N = sum(chunks)
    q, k, v = rand(rng, N, Hq, d), rand(rng, N, Hkv, d), rand(rng, N, Hkv, d)
    scale = 0.37
    s = OracleStream(budget=N, recent=3, heads=Hq, kv_heads=Hkv, head_dim=d, scale=scale)
    outs, a = [], 0
    for L in chunks:
        o, I = s.step(q[a:a + L], k[a:a + L], v[a:a + L])
        a += L
        outs.append(o)
        assert I.shape == (Hkv, a) and (I == np.arange(a)).all()      # nothing evicted while it fits
    ref = sdpa_causal(q, k, v, scale)
    np.testing.assert_allclose(np.concatenate(outs), ref, rtol=0, atol=1e-12)


def test_default_scale_is_inverse_sqrt_head_dim():
    rng = np.random.default_rng(11)
    q, k, v = rand(rng, 6, 2, 16), rand(rng, 6, 2, 16), rand(rng, 6, 2, 16)
    s = OracleStream(16, 4, 2, 2, 16)
    o, _ = s.step(q, k, v)
    np.testing.assert_allclose(o, sdpa_causal(q, k, v, 1 / 4.0), atol=1e-12)


def test_first_row_of_empty_stream_returns_v0():
    rng = np.random.default_rng(12)
    q, k, v = rand(rng, 4, 2, 8), rand(rng, 4, 2, 8), rand(rng, 4, 2, 8)
    o, _ = OracleStream(8, 2, 2, 2, 8).step(q, k, v)
    np.testing.assert_allclose(o[0], v[0], atol=1e-15)


def test_zero_queries_give_running_mean_of_values():
    rng = np.random.default_rng(13)
    Hkv, d = 2, 8
    s = OracleStream(64, 4, 4, Hkv, d)
    vs = []
    for L in (5, 6):
        k, v = rand(rng, L, Hkv, d), rand(rng, L, Hkv, d)
        t = len(s)
        vs.append(v)
        o, _ = s.step(np.zeros((L, 4, d)), k, v)
        allv = np.concatenate(vs)
        for i in range(L):
            mean = allv[: t + i + 1].mean(axis=0)               # [Hkv, d]
            np.testing.assert_allclose(o[i], np.repeat(mean, 2, axis=0), atol=1e-14)


# ---------------------------------------------------------------------------------------
# P2  score and bias (Alg. 1 l.1-4)
# ---------------------------------------------------------------------------------------
def fill(s, rng, t, Hq, Hkv, d):
    """bring an empty stream to t cached tokens without evicting"""
    q, k, v = rand(rng, t, Hq, d), rand(rng, t, Hkv, d), rand(rng, t, Hkv, d)
    s.step(q, k, v)
    return k, v


@pytest.mark.parametrize("R,L", [(4, 4), (3, 6), (7, 4)])      # R = L, R < L, R > L
def test_zero_queries_closed_form_score(R, L):
    """q = 0 makes every visible weight 1/(t+i+1); the column mean over the last
    l_q = min(R, L) rows is then a finite harmonic sum (Alg. 1 l.1)."""
    rng = np.random.default_rng(20)
    Hq, Hkv, d, B = 4, 2, 8, 10
    s = OracleStream(B, R, Hq, Hkv, d, bias=0.0)
    fill(s, rng, B, Hq, Hkv, d)
    t = B
    s.attend(np.zeros((L, Hq, d)), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))
    S, Wb = s.scores()
    n, lq = t + L, min(R, L)
    assert S.shape == (Hkv, n - R)
    expect = sum(1.0 / (t + i + 1) for i in range(L - lq, L)) / lq
    np.testing.assert_allclose(S, expect, rtol=1e-14)
    np.testing.assert_allclose(Wb, S, rtol=0, atol=0)            # b = 0: no bias
    s.commit(s.select())


@pytest.mark.parametrize("R,L", [(4, 5), (7, 4), (5, 5)])
def test_bias_is_the_ramp_of_alg1(R, L):
    """W' - S = D with D_{c-1} = 0, D_0 = -b (1 - 1/c), constant step b/c, c = n - R
    (Alg. 1 l.2-4 with l read as the recent window on the column side)."""
    rng = np.random.default_rng(21)
    Hq, Hkv, d, B, b = 2, 2, 8, 12, 0.3
    s = OracleStream(B, R, Hq, Hkv, d, bias=b)
    fill(s, rng, B, Hq, Hkv, d)
    s.attend(rand(rng, L, Hq, d), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))
    S, Wb = s.scores()
    c = B + L - R
    D = Wb - S
    assert D.shape == (Hkv, c)
    np.testing.assert_allclose(D[:, -1], 0.0, atol=1e-16)
    np.testing.assert_allclose(D[:, 0], -b * (1 - 1 / c), rtol=1e-12)
    np.testing.assert_allclose(np.diff(D, axis=1), b / c, rtol=1e-9)
    s.commit(s.select())


@pytest.mark.parametrize("R,L,G", [(4, 4, 1), (3, 6, 1), (7, 4, 1), (4, 5, 2)])
def test_scores_equal_column_mean_of_library_attention_matrix(R, L, G):
    """With V = identity the library routine's output IS the weight matrix W of Sec. 3.2;
    its last l_q rows, averaged, restricted to the first n - R columns, are S."""
    rng = np.random.default_rng(22)
    Hkv, B = 2, 10
    Hq = Hkv * G
    n = B + L
    d = n                                                         # so that V = I_n fits
    scale = 0.5
    s = OracleStream(B, R, Hq, Hkv, d, bias=0.0, scale=scale)
    q0, k0 = rand(rng, B, Hq, d), rand(rng, B, Hkv, d)
    eye = np.eye(n)
    v_all = np.repeat(eye[:, None, :], Hkv, axis=1)               # v_j = e_j
    s.step(q0, k0, v_all[:B])
    q1, k1 = rand(rng, L, Hq, d), rand(rng, L, Hkv, d)
    out = s.attend(q1, k1, v_all[B:])
    S, _ = s.scores()
    W = sdpa_causal(np.concatenate([q0, q1]), np.concatenate([k0, k1]), v_all, scale)[B:]   # [L,Hq,n]
    np.testing.assert_allclose(out, W, atol=1e-13)
    lq = min(R, L)
    expect = W[L - lq:].mean(axis=0)[:, : n - R]                  # [Hq, c]
    expect = expect.reshape(Hkv, G, n - R).mean(axis=1)           # pooled over the group
    np.testing.assert_allclose(S, expect, atol=1e-13)
    s.commit(s.select())


def test_candidate_mass_plus_recent_mass_is_one():
    """Softmax rows sum to one (Sec. 3.3), so sum_j S_j = 1 - (mean weight on the R recent
    keys).  The recent mass is read off the attention output by giving the recent keys the
    value e_0 and every other key the value 0."""
    rng = np.random.default_rng(23)
    Hq = Hkv = 2
    d, B, R, L = 8, 12, 5, 7
    s = OracleStream(B, R, Hq, Hkv, d, bias=0.0)
    s.step(rand(rng, B, Hq, d), rand(rng, B, Hkv, d), np.zeros((B, Hkv, d)))
    v = np.zeros((L, Hkv, d))
    v[L - R:, :, 0] = 1.0                                         # recent window = last R of n
    out = s.attend(rand(rng, L, Hq, d), rand(rng, L, Hkv, d), v)
    S, _ = s.scores()
    lq = min(R, L)
    recent_mass = out[L - lq:, :, 0].mean(axis=0)                 # [Hq]
    np.testing.assert_allclose(S.sum(axis=1), 1.0 - recent_mass, atol=1e-14)
    s.commit(s.select())


def test_group_with_identical_queries_matches_mha():
    rng = np.random.default_rng(24)
    Hkv, G, d, B, R, L = 2, 3, 8, 10, 4, 5
    a = OracleStream(B, R, Hkv, Hkv, d, bias=0.01)
    g = OracleStream(B, R, Hkv * G, Hkv, d, bias=0.01)
    for L_ in (B, L):
        q, k, v = rand(rng, L_, Hkv, d), rand(rng, L_, Hkv, d), rand(rng, L_, Hkv, d)
        oa = a.attend(q, k, v)
        og = g.attend(np.repeat(q, G, axis=1), k, v)
        np.testing.assert_allclose(og, np.repeat(oa, G, axis=1), atol=1e-14)
        if a.scores() is not None:
            np.testing.assert_allclose(g.scores()[1], a.scores()[1], atol=1e-15)
        Ia, Ig = a.select(), g.select()
        assert (Ia == Ig).all()
        a.commit(Ia)
        g.commit(Ig)


# ---------------------------------------------------------------------------------------
# P3  selection (Alg. 1 l.5-7)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(4))
def test_selected_set_maximises_total_score_exhaustively(seed):
    rng = np.random.default_rng(30 + seed)
    Hq = Hkv = 2
    d, B, R, L = 4, 9, 3, 5                                       # c = 11, r = 6: 462 subsets
    s = OracleStream(B, R, Hq, Hkv, d, bias=0.05)
    fill(s, rng, B, Hq, Hkv, d)
    s.attend(rand(rng, L, Hq, d), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))
    _, Wb = s.scores()
    I = s.select()
    c, r, n = B + L - R, B - R, B + L
    assert I.shape == (Hkv, B)
    for h in range(Hkv):
        best = max(itertools.combinations(range(c), r), key=lambda sub: Wb[h, list(sub)].sum())
        assert tuple(I[h, :r]) == best                            # ascending, and the argmax subset
        assert (I[h, r:] == np.arange(c, n)).all()                # I_l = [n-R, n)
    s.commit(I)


def test_selection_matches_numpy_argpartition():
    rng = np.random.default_rng(35)
    Hq, Hkv, d, B, R, L = 4, 2, 16, 96, 24, 40
    s = OracleStream(B, R, Hq, Hkv, d, bias=1e-3)
    fill(s, rng, B, Hq, Hkv, d)
    for _ in range(3):
        s.attend(rand(rng, L, Hq, d), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))
        _, Wb = s.scores()
        I = s.select()
        r = B - R
        for h in range(Hkv):
            top = np.sort(np.argpartition(-Wb[h], r - 1)[:r])
            assert (I[h, :r] == top).all()
        s.commit(I)


def test_huge_bias_degenerates_to_sliding_window():
    """b >= c makes the bias step b/c >= 1 exceed any gap between mean weights, so the r
    best are the r newest candidates: the cache is the last B tokens (window attention)."""
    rng = np.random.default_rng(31)
    Hq, Hkv, d, B, R, L = 2, 2, 8, 16, 4, 6
    s = OracleStream(B, R, Hq, Hkv, d, bias=4.0 * (B + L))
    total = 0
    for step in range(8):
        s.step(rand(rng, L, Hq, d), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))
        total += L
        _, _, pos = s.export()
        keep = min(total, B)
        assert (pos == np.arange(total - keep, total)).all()


def test_tiny_bias_prefers_newer_on_exact_ties():
    """q = 0 gives all candidates the same S; with b = 0 the tie goes to the newer slots."""
    rng = np.random.default_rng(32)
    Hq, Hkv, d, B, R, L = 2, 2, 4, 8, 2, 4
    s = OracleStream(B, R, Hq, Hkv, d, bias=0.0)
    fill(s, rng, B, Hq, Hkv, d)
    _, I = s.step(np.zeros((L, Hq, d)), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))
    assert (I == np.arange(L, B + L)).all()


def test_planted_key_aligned_with_queries_is_always_retained():
    rng = np.random.default_rng(33)
    Hq, Hkv, d, B, R, L = 2, 2, 16, 24, 6, 8
    u = np.zeros(d)
    u[0] = 1.0
    s = OracleStream(B, R, Hq, Hkv, d, bias=0.0, scale=1.0)
    k0 = 0.1 * rand(rng, L, Hkv, d)
    k0[2] = 6.0 * u                                                # planted at stream position 2
    s.step(0.1 * rand(rng, L, Hq, d) + 3.0 * u, k0, rand(rng, L, Hkv, d))
    for _ in range(12):
        s.step(0.1 * rand(rng, L, Hq, d) + 3.0 * u, 0.1 * rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))
        _, _, pos = s.export()
        assert (pos == 2).any(axis=1).all()


def test_permuting_old_rows_permutes_the_retained_set():
    """Fully visible keys enter attention symmetrically; with b = 0 the retained SET (as
    stream positions) cannot depend on the order of the cached rows."""
    rng = np.random.default_rng(34)
    Hq, Hkv, d, B, R, L = 4, 2, 8, 20, 5, 7
    K, V = rand(rng, Hkv, B, d), rand(rng, Hkv, B, d)
    pos = np.tile(np.arange(B), (Hkv, 1))
    perm = rng.permutation(B)
    q, k, v = rand(rng, L, Hq, d), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d)
    a = OracleStream(B, R, Hq, Hkv, d, bias=0.0)
    b = OracleStream(B, R, Hq, Hkv, d, bias=0.0)
    a.load(K, V, pos, B)
    b.load(K[:, perm], V[:, perm], pos[:, perm], B)
    oa, _ = a.step(q, k, v)
    ob, _ = b.step(q, k, v)
    np.testing.assert_allclose(oa, ob, atol=1e-13)
    pa, pb = a.export()[2], b.export()[2]
    for h in range(Hkv):
        assert set(pa[h]) == set(pb[h])


# ---------------------------------------------------------------------------------------
# P4  invariants of the size-constrained cache (Alg. 1 l.6-8)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("Hq,Hkv,B,R,chunks", [
    (4, 4, 32, 8, [8] * 10),
    (4, 2, 40, 24, [12, 5, 30, 7, 16, 16, 1, 9]),       # R > L, ragged chunk lengths
    (2, 1, 16, 16, [4] * 8),                             # r = 0: pure window
    (2, 2, 16, 0, [4] * 8),                              # R = 0: nothing is pinned
])
def test_cache_invariants_over_a_stream(Hq, Hkv, B, R, chunks):
    rng = np.random.default_rng(40)
    d = 8
    s = OracleStream(B, R, Hq, Hkv, d, bias=1e-2)
    allk, allv = [], []
    prev_pos = np.zeros((Hkv, 0), dtype=np.int64)
    total = 0
    for L in chunks:
        q, k, v = rand(rng, L, Hq, d), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d)
        allk.append(k)
        allv.append(v)
        t = len(s)
        out, I = s.step(q, k, v)
        n = t + L
        total += L
        assert out.shape == (L, Hq, d)
        assert len(s) == min(n, B) <= B and I.shape == (Hkv, min(n, B))
        assert (np.diff(I, axis=1) > 0).all() and I.min() >= 0 and I.max() < n
        keep_recent = min(R, n)
        if keep_recent:
            assert (I[:, -keep_recent:] == np.arange(n - keep_recent, n)).all()
        K, V, pos = s.export()
        assert (np.diff(pos, axis=1) > 0).all()
        before = np.concatenate([prev_pos, np.tile(np.arange(total - L, total), (Hkv, 1))], axis=1)
        for h in range(Hkv):
            assert (pos[h] == before[h, I[h]]).all()             # retained = previous cache U chunk, by index
            ak, av = np.concatenate(allk)[:, h], np.concatenate(allv)[:, h]
            assert (K[h] == ak[pos[h]]).all() and (V[h] == av[pos[h]]).all()   # rows move unchanged
        prev_pos = pos
    assert s.streamed == total


def test_survival_of_a_recurring_early_token_is_monotone_in_bias():
    """Sec. 3.3: a lower bias keeps older tokens longer.  Qualitative only."""
    Hq = Hkv = 1
    d, B, R, L = 8, 24, 6, 6
    life = []
    for b in (0.0, 1e-3, 1e-1, 10.0):
        rng = np.random.default_rng(41)
        s = OracleStream(B, R, Hq, Hkv, d, bias=b, scale=1.0)
        u = np.zeros(d)
        u[1] = 1.0
        k0 = 0.3 * rand(rng, L, Hkv, d)
        k0[0] = 1.5 * u
        s.step(0.3 * rand(rng, L, Hq, d) + 1.0 * u, k0, rand(rng, L, Hkv, d))
        alive = 0
        for step in range(40):
            s.step(0.3 * rand(rng, L, Hq, d) + 1.0 * u, 0.3 * rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))
            if not (s.export()[2] == 0).any():
                break
            alive += 1
        life.append(alive)
    assert all(x >= y for x, y in zip(life, life[1:])), life
    assert life[0] > life[-1]


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        OracleStream(8, 9, 2, 2, 4)
    with pytest.raises(ValueError):
        OracleStream(8, 2, 3, 2, 4)
    s = OracleStream(8, 2, 2, 2, 4)
    rng = np.random.default_rng(0)
    s.attend(rand(rng, 3, 2, 4), rand(rng, 3, 2, 4), rand(rng, 3, 2, 4))
    with pytest.raises(RuntimeError):
        s.commit(np.array([[0, 0, 1], [0, 1, 2]], dtype=np.int32))   # not strictly ascending


# ---------------------------------------------------------------------------------------
# decoding steps (Sec. 3.2: no eviction while tokens are decoded)
# ---------------------------------------------------------------------------------------
def test_decode_tokens_between_chunks_equal_one_shot_causal_attention():
    rng = np.random.default_rng(50)
    Hq, Hkv, d = 4, 2, 16
    plan = [("chunk", 6), ("decode", 3), ("chunk", 5), ("decode", 4)]
    N = sum(n for _, n in plan)
    q, k, v = rand(rng, N, Hq, d), rand(rng, N, Hkv, d), rand(rng, N, Hkv, d)
    s = OracleStream(budget=N, recent=2, heads=Hq, kv_heads=Hkv, head_dim=d, scale=0.4)
    outs, a = [], 0
    for kind, cnt in plan:
        if kind == "chunk":
            outs.append(s.step(q[a:a + cnt], k[a:a + cnt], v[a:a + cnt])[0])
            a += cnt
        else:
            for _ in range(cnt):
                outs.append(s.decode(q[a:a + 1], k[a:a + 1], v[a:a + 1]))
                a += 1
        assert len(s) == a and s.streamed == a
    np.testing.assert_allclose(np.concatenate(outs), sdpa_causal(q, k, v, 0.4), atol=1e-12)
    assert (s.export()[2] == np.arange(N)).all()


def test_decode_grows_past_the_budget_and_the_next_chunk_evicts_back():
    rng = np.random.default_rng(51)
    Hq, Hkv, d, B, R, L = 2, 2, 8, 12, 4, 5
    s = OracleStream(B, R, Hq, Hkv, d, bias=1e-2)
    fill(s, rng, B, Hq, Hkv, d)
    for i in range(3):
        out = s.decode(rand(rng, 1, Hq, d), rand(rng, 1, Hkv, d), rand(rng, 1, Hkv, d))
        assert out.shape == (1, Hq, d) and len(s) == B + i + 1          # no eviction while decoding
    K, V, pos = s.export()
    assert (pos == np.arange(B + 3)).all()
    _, I = s.step(rand(rng, L, Hq, d), rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))
    n = B + 3 + L
    assert len(s) == B and I.shape == (Hkv, B)
    assert (I[:, -R:] == np.arange(n - R, n)).all()                       # recent window of the new n
    assert (np.diff(s.export()[2], axis=1) > 0).all()


def test_decode_with_zero_query_returns_mean_of_all_values():
    rng = np.random.default_rng(52)
    s = OracleStream(8, 2, 2, 1, 4)
    v0 = rand(rng, 5, 1, 4)
    s.step(rand(rng, 5, 2, 4), rand(rng, 5, 1, 4), v0)
    v1 = rand(rng, 1, 1, 4)
    out = s.decode(np.zeros((1, 2, 4)), rand(rng, 1, 1, 4), v1)
    mean = np.concatenate([v0, v1]).mean(axis=0)                          # [1, 4]
    np.testing.assert_allclose(out[0], np.repeat(mean, 2, axis=0), atol=1e-14)
