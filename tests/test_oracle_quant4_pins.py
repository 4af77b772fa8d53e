"""Pins for the oracle's 4-bit KV quantiser and attention over it (FastDecode Section 5.2: 4-bit
storage quarters the bytes of fp16).

The paper leaves the quantiser to the user; the one pinned here is asymmetric per token and
head: zero = min x, scale = (max x - min x) / 15, code = rint((x - zero) / scale) in 0..15, all in
IEEE binary32; value = code * scale + zero.  No GPU is needed.
"""
import math

import numpy as np

from oracle import rpart_oracle as O
from tests.util import f64, half_bits


def _q(x):
    packed, sz = O.quantize_rows_u4(half_bits(x))
    return O.unpack_u4(packed).astype(np.int32), sz


def test_packing_order_low_nibble_first():
    x = np.array([[0.0, 15.0, 1.0, 2.0]])                     # scale 1, zero 0 -> codes are the values
    packed, sz = O.quantize_rows_u4(half_bits(x))
    assert packed.tolist() == [[0x0 | (0xF << 4), 0x1 | (0x2 << 4)]]
    assert sz.tolist() == [[1.0, 0.0]]
    assert O.unpack_u4(packed).tolist() == [[0, 15, 1, 2]]


def test_exact_rows_with_power_of_two_step():
    step, zero = 2.0 ** -4, -0.5
    ints = np.array([[0, 15, 3, 7, 8, 1, 14, 15]])
    codes, sz = _q(ints * step + zero)                        # exact in binary16
    assert sz[0, 0] == np.float32(step) and sz[0, 1] == np.float32(zero)
    assert np.array_equal(codes, ints)


def test_ties_round_to_even_and_extremes_hit_0_and_15():
    # zero = 0, max = 15 -> scale 1; .5 values are ties
    x = np.array([[0.0, 15.0, 0.5, 1.5, 2.5, 3.5, 13.5, 14.5]])
    codes, sz = _q(x)
    assert sz[0].tolist() == [1.0, 0.0]
    assert codes[0].tolist() == [0, 15, 0, 2, 2, 4, 14, 14]


def test_constant_row():
    codes, sz = _q(np.full((1, 8), -2.5))
    assert np.all(codes == 0) and sz[0].tolist() == [0.0, -2.5]
    codes, sz = _q(np.zeros((1, 8)))
    assert np.all(codes == 0) and sz[0].tolist() == [0.0, 0.0]


def test_error_bound_and_range():
    rng = np.random.default_rng(1)
    x = f64(half_bits(rng.standard_normal((200, 128)) * rng.uniform(0.01, 30, size=(200, 1))))
    codes, sz = _q(x)
    assert codes.min() == 0 and codes.max() == 15
    rows = np.arange(x.shape[0])
    assert np.all(codes[rows, x.argmin(axis=1)] == 0) and np.all(codes[rows, x.argmax(axis=1)] == 15)
    s, z = sz[:, 0:1].astype(np.float64), sz[:, 1:2].astype(np.float64)
    assert np.array_equal(z[:, 0], x.min(axis=1))             # zero = min exactly (binary16 -> binary32)
    err = np.abs(x - (codes * s + z))
    # round to nearest: half a step, plus the binary32 roundings of x - zero and of the quotient
    assert np.all(err <= (0.5 + 2.0 ** -19) * s)
    assert np.all(np.abs(s[:, 0] * 15 - (x.max(axis=1) - x.min(axis=1))) <= 2.0 ** -22 * np.abs(x).max(axis=1))


def test_shift_and_scale_covariance():
    rng = np.random.default_rng(2)
    ints = rng.integers(-60, 60, size=(40, 32)).astype(np.float64)      # small integers: sums stay exact
    c1, sz1 = _q(ints)
    c2, sz2 = _q(ints * 2.0)
    assert np.array_equal(c1, c2) and np.array_equal(sz2, sz1 * 2)
    c3, sz3 = _q(ints + 64.0)                                            # exact shift in binary16
    assert np.array_equal(c1, c3) and np.array_equal(sz3[:, 0], sz1[:, 0])
    assert np.array_equal(sz3[:, 1], sz1[:, 1] + 64)


def test_matches_numpy_float32_restatement():
    rng = np.random.default_rng(3)
    xb = half_bits(rng.standard_normal((300, 128)) * 3)
    packed, sz = O.quantize_rows_u4(xb)
    x32 = xb.view(np.float16).astype(np.float32)
    mn, mx = x32.min(axis=1), x32.max(axis=1)
    s = (mx - mn) / np.float32(15.0)
    assert s.dtype == np.float32 and np.array_equal(s, sz[:, 0]) and np.array_equal(mn, sz[:, 1])
    c = np.clip(np.rint((x32 - mn[:, None]) / s[:, None]), 0, 15).astype(np.uint8)
    assert np.array_equal(c, O.unpack_u4(packed))


def test_requantising_dequantised_rows_is_idempotent():
    rng = np.random.default_rng(4)
    codes = rng.integers(0, 16, size=(40, 32))
    codes[:, 0], codes[:, 1] = 0, 15
    step = 2.0 ** rng.integers(-8, 2, size=(40, 1))
    zero = step * rng.integers(-20, 20, size=(40, 1))
    c2, sz = _q(codes * step + zero)
    assert np.array_equal(c2, codes)
    assert np.array_equal(sz[:, 0], step[:, 0].astype(np.float32))
    assert np.array_equal(sz[:, 1], zero[:, 0].astype(np.float32))


def _random_cache(rng, L, H, d, exact):
    Kc = rng.integers(0, 256, size=(L, H, d // 2)).astype(np.uint8)
    Vc = rng.integers(0, 256, size=(L, H, d // 2)).astype(np.uint8)
    if exact:
        s = 2.0 ** rng.integers(-5, -1, size=(L, H, 1))
        z = s * rng.integers(-12, 4, size=(L, H, 1))
    else:
        s = rng.uniform(0.02, 0.3, size=(L, H, 1))
        z = rng.uniform(-2, 0.5, size=(L, H, 1))
    Ksz = np.concatenate([s, z], axis=2).astype(np.float32)
    s2, z2 = (s * 2, z - 0.25) if exact else (s * 1.5, z + 0.3)
    Vsz = np.concatenate([s2, z2], axis=2).astype(np.float32)
    return Kc, Ksz, Vc, Vsz


def _deq(c, sz):
    return O.unpack_u4(c).astype(np.float64) * sz[..., 0:1].astype(np.float64) + sz[..., 1:2].astype(np.float64)


def test_attention_equals_fp16_path_on_exactly_representable_rows():
    rng = np.random.default_rng(5)
    H, d = 3, 16
    Ls = [1, 7, 33]
    q = half_bits(rng.standard_normal((len(Ls), H, d)))
    parts = [_random_cache(rng, L, H, d, True) for L in Ls]
    K16 = [half_bits(_deq(p[0], p[1])) for p in parts]
    V16 = [half_bits(_deq(p[2], p[3])) for p in parts]
    for p, k in zip(parts, K16):
        assert np.array_equal(f64(k), _deq(p[0], p[1]))                   # really exact in binary16
    lens = np.asarray(Ls, dtype=np.int32)
    out_q, lse_q = O.rpartq4_decode([p[0] for p in parts], [p[1] for p in parts],
                                    [p[2] for p in parts], [p[3] for p in parts], lens, q)
    out_h, lse_h, _ = O.rpart_decode(K16, V16, lens, q)
    assert np.abs(out_q - out_h).max() < 1e-13 and np.abs(lse_q - lse_h).max() < 1e-13


def test_attention_against_numpy_definition_and_empty_sequence():
    rng = np.random.default_rng(6)
    H, d, L = 2, 32, 50
    kc, ksz, vc, vsz = _random_cache(rng, L, H, d, False)
    q = half_bits(rng.standard_normal((1, H, d)))
    out, lse = O.rpartq4_decode([kc], [ksz], [vc], [vsz], np.array([L], np.int32), q)
    k, v = _deq(kc, ksz), _deq(vc, vsz)
    s = np.einsum("thd,hd->ht", k, f64(q)[0]) / math.sqrt(d)
    w = np.exp(s - s.max(axis=1, keepdims=True))
    w /= w.sum(axis=1, keepdims=True)
    assert np.abs(out[0] - np.einsum("ht,thd->hd", w, v)).max() < 1e-13
    assert np.abs(lse[0] - (s.max(axis=1) + np.log(np.exp(s - s.max(axis=1, keepdims=True)).sum(axis=1)))).max() < 1e-12
    out0, lse0 = O.rpartq4_decode([kc], [ksz], [vc], [vsz], np.array([0], np.int32), q)
    assert np.all(out0 == 0) and np.all(np.isneginf(lse0))


def test_append_stores_the_quantised_row_only_at_the_new_position():
    rng = np.random.default_rng(7)
    B, H, d = 2, 3, 16
    L = np.array([0, 4], dtype=np.int32)
    Kc = [rng.integers(0, 256, size=(l + 2, H, d // 2)).astype(np.uint8) for l in L]
    Vc = [rng.integers(0, 256, size=(l + 2, H, d // 2)).astype(np.uint8) for l in L]
    Ksz = [rng.uniform(0, 1, size=(l + 2, H, 2)).astype(np.float32) for l in L]
    Vsz = [rng.uniform(0, 1, size=(l + 2, H, 2)).astype(np.float32) for l in L]
    before = [a.copy() for a in Kc + Vc + Ksz + Vsz]
    k_new = half_bits(rng.standard_normal((B, H, d)))
    v_new = half_bits(rng.standard_normal((B, H, d)) * 4)
    lens = L.copy()
    O.kvq4_append(Kc, Ksz, Vc, Vsz, lens, k_new, v_new)
    assert np.array_equal(lens, L + 1)
    kc_ref, ksz_ref = O.quantize_rows_u4(k_new)
    vc_ref, vsz_ref = O.quantize_rows_u4(v_new)
    for b in range(B):
        assert np.array_equal(Kc[b][L[b]], kc_ref[b]) and np.array_equal(Ksz[b][L[b]], ksz_ref[b])
        assert np.array_equal(Vc[b][L[b]], vc_ref[b]) and np.array_equal(Vsz[b][L[b]], vsz_ref[b])
    for idx, (a0, a1) in enumerate(zip(before, Kc + Vc + Ksz + Vsz)):
        keep = np.ones(a0.shape[0], dtype=bool)
        keep[L[idx % B]] = False
        assert np.array_equal(a0[keep], a1[keep])


def test_quantisation_error_of_attention_is_moderate_on_normal_data():
    """Sanity of the scheme: 4-bit rows change the attention output by a few per cent of max|V|
    on N(0,1) data (each element moves by at most scale/2 ~ range/30)."""
    rng = np.random.default_rng(8)
    H, d, L = 4, 128, 400
    K = half_bits(rng.standard_normal((L, H, d)))
    V = half_bits(rng.standard_normal((L, H, d)))
    q = half_bits(rng.standard_normal((1, H, d)))
    lens = np.array([L], np.int32)
    ref, _, _ = O.rpart_decode([K], [V], lens, q)
    kc, ksz = O.quantize_rows_u4(K)
    vc, vsz = O.quantize_rows_u4(V)
    got, _ = O.rpartq4_decode([kc], [ksz], [vc], [vsz], lens, q)
    assert np.abs(got - ref).max() < 0.08 * np.abs(f64(V)).max()
