"""Pins for the window-attention oracle (sink tokens + the last `window` tokens) and for its
bounded-cache simulation.  No GPU is needed."""
import math

import numpy as np
import pytest

from oracle import rpart_oracle as O
from oracle import window_oracle as WO
from tests.util import f64, half_bits


def _hist(rng, L, H, d):
    return half_bits(rng.standard_normal((L, H, d))), half_bits(rng.standard_normal((L, H, d)))


def test_token_set_by_hand():
    assert WO.token_set(10, 2, 3) == [0, 1, 7, 8, 9]
    assert WO.token_set(4, 2, 3) == [0, 1, 2, 3]            # everything still fits
    assert WO.token_set(5, 2, 3) == [0, 1, 2, 3, 4]
    assert WO.token_set(6, 2, 3) == [0, 1, 3, 4, 5]          # token 2 is the first to go
    assert WO.token_set(6, 0, 1) == [5]
    assert WO.token_set(0, 2, 3) == []
    assert WO.token_set(3, 5, 0) == [0, 1, 2] and WO.token_set(9, 5, 0) == [0, 1, 2, 3, 4]


def test_window_covering_everything_is_plain_attention():
    rng = np.random.default_rng(0)
    H, d = 2, 16
    K, V = _hist(rng, 40, H, d)
    q = half_bits(rng.standard_normal((1, H, d)))
    full, _, _ = O.rpart_decode([K], [V], np.array([40], np.int32), q)
    assert np.array_equal(WO.rpart_decode_window([K], [V], [40], q, 0, 40), full)
    assert np.array_equal(WO.rpart_decode_window([K], [V], [40], q, 3, 64), full)
    assert np.array_equal(WO.rpart_decode_window([K], [V], [40], q, 40, 0), full)


def test_window_of_one_returns_the_last_value():
    rng = np.random.default_rng(1)
    K, V = _hist(rng, 9, 3, 8)
    q = half_bits(rng.standard_normal((1, 3, 8)))
    out = WO.rpart_decode_window([K], [V], [9], q, 0, 1)
    assert np.array_equal(out[0], f64(V[8]))


def test_against_numpy_softmax_over_the_explicit_set():
    rng = np.random.default_rng(2)
    H, d, L, n_sink, window = 2, 8, 30, 4, 7
    K, V = _hist(rng, L, H, d)
    q = half_bits(rng.standard_normal((1, H, d)))
    out = WO.rpart_decode_window([K], [V], [L], q, n_sink, window)[0]
    keep = [0, 1, 2, 3] + list(range(23, 30))               # written out by hand for these numbers
    k, v = f64(K)[keep], f64(V)[keep]
    s = np.einsum("thd,hd->ht", k, f64(q)[0]) / math.sqrt(d)
    w = np.exp(s)
    w /= w.sum(axis=1, keepdims=True)
    assert np.abs(out - np.einsum("ht,thd->hd", w, v)).max() < 1e-13


def test_tokens_outside_the_set_do_not_matter_and_inside_do():
    rng = np.random.default_rng(3)
    H, d, L, n_sink, window = 2, 8, 50, 2, 10
    K, V = _hist(rng, L, H, d)
    q = half_bits(rng.standard_normal((1, H, d)))
    ref = WO.rpart_decode_window([K], [V], [L], q, n_sink, window)
    K2, V2 = K.copy(), V.copy()
    K2[2:40] = half_bits(rng.standard_normal((38, H, d)) * 5)
    V2[2:40] = half_bits(rng.standard_normal((38, H, d)) * 5)
    assert np.array_equal(WO.rpart_decode_window([K2], [V2], [L], q, n_sink, window), ref)
    for t in (0, 1, 40, 49):                                # boundary members of the set
        V3 = V.copy()
        V3[t] = half_bits(f64(V[t]) + 1.0)
        assert np.abs(WO.rpart_decode_window([K], [V3], [L], q, n_sink, window) - ref).max() > 1e-6
    for t in (2, 39):                                       # first and last excluded token
        V3 = V.copy()
        V3[t] = half_bits(f64(V[t]) + 1.0)
        assert np.array_equal(WO.rpart_decode_window([K], [V3], [L], q, n_sink, window), ref)


@pytest.mark.parametrize("n_sink,window", [(0, 1), (0, 5), (2, 3), (4, 1), (3, 8)])
def test_bounded_cache_always_holds_exactly_the_token_set(n_sink, window):
    c = WO.BoundedCache(n_sink, window)
    for L in range(1, 40):
        r = c.append()
        assert c.rows[r] == L - 1                           # the new token is where append said
        assert sorted(c.rows) == WO.token_set(L, n_sink, window)
        assert c.rows[:min(L, n_sink)] == list(range(min(L, n_sink)))   # sinks never move
        assert len(c.rows) <= n_sink + window


def test_attention_over_the_bounded_cache_rows_equals_the_definition():
    """Rows of the bounded cache are in ring order, not token order; attention must not care."""
    rng = np.random.default_rng(4)
    H, d, n_sink, window = 2, 8, 2, 5
    K, V = _hist(rng, 23, H, d)
    q = half_bits(rng.standard_normal((1, H, d)))
    c = WO.BoundedCache(n_sink, window)
    for L in range(1, 24):
        c.append()
        rows = np.asarray(c.rows)
        got, _, _ = O.rpart_decode([np.ascontiguousarray(K[rows])], [np.ascontiguousarray(V[rows])],
                                   np.array([len(rows)], np.int32), q)
        want = WO.rpart_decode_window([K], [V], [L], q, n_sink, window)
        assert np.abs(got - want).max() < 1e-13
