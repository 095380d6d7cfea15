"""Pins for the oracle's comparison policies (Sec. 2 "KV cache eviction", Sec. 4.1 baselines): window,
initial + recent, and cumulative score.  Each is fixed to a statement that does not go through the
oracle's own arithmetic: which stream positions must be cached, or an exact rational model of the
score bookkeeping under uniform attention.  No GPU needed."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import OracleStream


def rand(rng, *shape):
    return rng.standard_normal(shape)


def drive(o, rng, chunks, Hq, Hkv, d, zero_q=False):
    for L in chunks:
        q = np.zeros((L, Hq, d)) if zero_q else rand(rng, L, Hq, d)
        o.step(q, rand(rng, L, Hkv, d), rand(rng, L, Hkv, d))


@pytest.mark.parametrize("B,R,chunks", [(16, 4, [5, 7, 9, 3, 16, 1, 8]), (10, 10, [4, 4, 4, 4]), (12, 0, [12, 5, 5])])
def test_window_policy_keeps_exactly_the_newest_tokens(B, R, chunks):
    rng = np.random.default_rng(1)
    o = OracleStream(B, R, 4, 2, 8, policy="window")
    total = 0
    for L in chunks:
        drive(o, rng, [L], 4, 2, 8)
        total += L
        pos = o.export()[2]
        want = np.arange(max(0, total - B), total)
        assert (pos == want).all(), (total, pos[0])


@pytest.mark.parametrize("B,R,chunks", [(16, 4, [5, 7, 9, 3, 16, 1, 8]), (12, 3, [20 // 2, 9, 12, 2])])
def test_initial_recent_policy_keeps_the_first_r_and_the_last_R(B, R, chunks):
    rng = np.random.default_rng(2)
    o = OracleStream(B, R, 2, 2, 8, policy="initial_recent")
    total, r = 0, B - R
    for L in chunks:
        drive(o, rng, [L], 2, 2, 8)
        total += L
        pos = o.export()[2]
        if total <= B:
            want = np.arange(total)
        else:
            want = np.concatenate([np.arange(r), np.arange(total - R, total)])
        assert (pos == want).all(), (total, pos[0])


def test_cumulative_policy_first_eviction_equals_unbiased_alg1():
    """With nothing accumulated yet, W' = S: the same set as Alg. 1 with b = 0."""
    rng = np.random.default_rng(3)
    a = OracleStream(24, 6, 4, 2, 8, bias=0.0)
    b = OracleStream(24, 6, 4, 2, 8, bias=0.37, policy="cumulative")         # the bias must be ignored
    for L in (10, 10):
        q, k, v = rand(rng, L, 4, 8), rand(rng, L, 2, 8), rand(rng, L, 2, 8)
        a.step(q, k, v)
        b.step(q, k, v)
    q, k, v = rand(rng, 12, 4, 8), rand(rng, 12, 2, 8), rand(rng, 12, 2, 8)
    _, Ia = a.step(q, k, v)
    b.attend(q, k, v)
    S, Wb = b.scores()
    assert (S == Wb).all()
    Ib = b.select()
    b.commit(Ib)
    assert (Ia == Ib).all()
    A = b.accumulated()
    r = 24 - 6
    assert (A[:, :r] == np.take_along_axis(S, Ib[:, :r], axis=1)).all() and (A[:, r:] == 0).all()


def model_uniform_attention(B, R, chunks):
    """Exact model of the cumulative policy when every query is zero, so that each row spreads its weight
    evenly over the keys it sees: row i of a chunk arriving at t cached keys gives 1 / (t + i + 1) to each.
    Tracks (stream position, accumulated score) per cached row with rationals."""
    cache, T = [], 0                                   # list of [pos, A]
    r = B - R
    for L in chunks:
        t = len(cache)
        rows = cache + [[T + i, Fraction(0)] for i in range(L)]
        n = t + L
        T += L
        if n > B:
            c, lq = n - R, min(R, L)
            W = []
            for j in range(c):
                S = sum(Fraction(1, t + i + 1) for i in range(L - lq, L) if j <= t + i)
                S = S / lq if lq else Fraction(0)
                W.append(rows[j][1] + S)
            order = sorted(range(c), key=lambda j: (W[j], j), reverse=True)[:r]     # ties: newer first
            keep = sorted(order)
            rows = [[rows[j][0], W[j]] for j in keep] + rows[c:]
        cache = rows
    return cache


@pytest.mark.parametrize("B,R,chunks", [(12, 4, [6, 6, 5, 7, 3, 8]), (10, 3, [10, 2, 9, 1, 1, 6]), (9, 5, [4, 4, 4, 4, 4])])
def test_cumulative_policy_matches_exact_model_under_uniform_attention(B, R, chunks):
    rng = np.random.default_rng(4)
    o = OracleStream(B, R, 2, 1, 4, policy="cumulative")
    drive(o, rng, chunks, 2, 1, 4, zero_q=True)
    want = model_uniform_attention(B, R, chunks)
    pos, A = o.export()[2][0], o.accumulated()[0]
    assert pos.tolist() == [p for p, _ in want]
    assert np.allclose(A, [float(a) for _, a in want], rtol=1e-13, atol=0)


def test_cumulative_policy_keeps_a_heavy_hitter_that_alg1_with_large_bias_drops():
    """A key that every query points at gathers score in every step and stays under the cumulative policy,
    while Alg. 1 with a large bias lets it go once it is old."""
    rng = np.random.default_rng(5)
    d, B, R = 8, 16, 4
    hot = np.zeros(d)
    hot[0] = 6.0
    keep = {}
    for name, kw in (("cum", dict(policy="cumulative")), ("biased", dict(bias=50.0))):
        o = OracleStream(B, R, 1, 1, d, scale=1.0, **kw)
        rng = np.random.default_rng(5)
        k0 = rand(rng, 6, 1, d) * 0.1
        k0[2, 0] = hot                                              # stream position 2
        o.step(np.tile(hot, (6, 1, 1)), k0, rand(rng, 6, 1, d))
        for _ in range(8):
            o.step(np.tile(hot, (6, 1, 1)), rand(rng, 6, 1, d) * 0.1, rand(rng, 6, 1, d))
        keep[name] = 2 in o.export()[2][0]
    assert keep == {"cum": True, "biased": False}


def test_policy_can_only_change_between_steps_and_rejects_unknown_values():
    from oracle import _load
    lib = _load()
    o = OracleStream(8, 2, 1, 1, 4)
    assert lib.oracle_set_policy(o._h, 4) != 0 and lib.oracle_set_policy(o._h, -1) != 0
    rng = np.random.default_rng(6)
    o.attend(rand(rng, 3, 1, 4), rand(rng, 3, 1, 4), rand(rng, 3, 1, 4))
    assert lib.oracle_set_policy(o._h, 1) != 0                       # a step is in flight
    o.commit(o.select())
    assert lib.oracle_set_policy(o._h, 1) == 0
