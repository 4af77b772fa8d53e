"""Pins for the oracle's int8 KV quantiser and quantised attention (FastDecode Section 5.2).

The paper leaves the quantiser to the user; the one pinned here is symmetric per token and
head: scale = max|x| / 127, code = rint(x / scale), both in IEEE binary32, stored as code + 128.
No GPU is needed.
"""
import math

import numpy as np
import pytest

from oracle import rpart_oracle as O
from tests.util import f64, half_bits


def _q(x):
    """float array [..., d] (values exact in binary16) -> (codes int [-127,127], scales float32)."""
    codes, scales = O.quantize_rows_i8(half_bits(x))
    return codes.astype(np.int32) - 128, scales


def test_exact_rows_power_of_two_scale():
    s0 = 2.0 ** -5
    ints = np.array([[127, -64, 3, 0, -127, 1, 100, -1]])
    codes, scales = _q(ints * s0)
    assert scales[0] == np.float32(s0)
    assert np.array_equal(codes, ints)


def test_ties_round_to_even():
    s0 = 2.0 ** -3
    x = np.array([[127.0, 2.5, 3.5, -2.5, -3.5, 0.5, 1.5, -0.5]]) * s0      # x / scale = k + 1/2
    codes, scales = _q(x)
    assert scales[0] == np.float32(s0)
    assert codes[0].tolist() == [127, 2, 4, -2, -4, 0, 2, 0]


def test_zero_row_and_single_value():
    codes, scales = _q(np.zeros((2, 16)))
    assert np.all(codes == 0) and np.all(scales == 0)
    raw, _ = O.quantize_rows_i8(half_bits(np.zeros((1, 16))))
    assert np.all(raw == 128)
    x = np.zeros((1, 16))
    x[0, 5] = -3.0
    codes, scales = _q(x)
    assert codes[0, 5] == -127 and np.count_nonzero(codes) == 1
    assert scales[0] == np.float32(3.0) / np.float32(127.0)


def test_error_bound_and_extreme_codes():
    rng = np.random.default_rng(1)
    x = f64(half_bits(rng.standard_normal((200, 128)) * rng.uniform(0.01, 30, size=(200, 1))))
    codes, scales = _q(x)
    assert codes.min() >= -127 and codes.max() <= 127
    amax_idx = np.abs(x).argmax(axis=1)
    rows = np.arange(x.shape[0])
    assert np.all(np.abs(codes[rows, amax_idx]) == 127)                 # the largest element hits +-127
    xh = codes * scales[:, None].astype(np.float64)
    err = np.abs(x - xh)
    # round to nearest: half a step, plus the rounding of the binary32 quotient (|x/scale| <= 127,
    # so at most 127 * 2^-24 of a step) which can push a value onto a tie
    assert np.all(err <= (0.5 + 127 * 2.0 ** -23) * scales[:, None])
    assert np.all(np.abs(scales.astype(np.float64) * 127 - np.abs(x).max(axis=1))
                  <= np.abs(x).max(axis=1) * 2.0 ** -23)                # scale = amax/127 to 1 ulp


def test_scaling_and_sign_symmetry():
    rng = np.random.default_rng(2)
    x = f64(half_bits(rng.standard_normal((50, 64))))
    c1, s1 = _q(x)
    c2, s2 = _q(2.0 * x)                                                # exact in binary16
    assert np.array_equal(c1, c2) and np.array_equal(s2, 2 * s1)
    c3, s3 = _q(-x)
    assert np.array_equal(c3, -c1) and np.array_equal(s3, s1)


def test_matches_numpy_float32_restatement():
    rng = np.random.default_rng(3)
    xb = half_bits(rng.standard_normal((300, 128)) * 3)
    codes, scales = O.quantize_rows_i8(xb)
    x32 = xb.view(np.float16).astype(np.float32)
    s = np.abs(x32).max(axis=1) / np.float32(127.0)
    assert s.dtype == np.float32 and np.array_equal(s, scales)
    c = np.rint(x32 / s[:, None]).astype(np.int32) + 128                # float32 division, ties to even
    assert np.array_equal(c.astype(np.uint8), codes)


def test_requantising_dequantised_rows_is_idempotent():
    rng = np.random.default_rng(4)
    codes = rng.integers(-127, 128, size=(40, 32))
    codes[:, 0] = 127                                                    # make the scale recoverable
    scale = 2.0 ** rng.integers(-8, 3, size=(40, 1))
    c2, s2 = _q(codes * scale)                                           # exact in binary16 (7-bit ints)
    assert np.array_equal(c2, codes) and np.array_equal(s2, scale[:, 0].astype(np.float32))


def _random_qcache(rng, L, H, d, pow2_scales):
    Kc = rng.integers(1, 256, size=(L, H, d)).astype(np.uint8)
    Vc = rng.integers(1, 256, size=(L, H, d)).astype(np.uint8)
    if pow2_scales:
        Ks = (2.0 ** rng.integers(-7, -3, size=(L, H))).astype(np.float32)
        Vs = (2.0 ** rng.integers(-7, -3, size=(L, H))).astype(np.float32)
    else:
        Ks = rng.uniform(0.005, 0.05, size=(L, H)).astype(np.float32)
        Vs = rng.uniform(0.005, 0.05, size=(L, H)).astype(np.float32)
    return Kc, Ks, Vc, Vs


def test_quantised_attention_equals_fp16_path_on_exact_rows():
    """With power-of-two scales every dequantised value is exact in binary16, so attention over
    the quantised cache must equal the (separately pinned) fp16 path over those values."""
    rng = np.random.default_rng(5)
    H, d = 3, 16
    Ls = [1, 7, 33]
    q = half_bits(rng.standard_normal((len(Ls), H, d)))
    Kc, Ks, Vc, Vs, K16, V16 = [], [], [], [], [], []
    for L in Ls:
        kc, ks, vc, vs = _random_qcache(rng, L, H, d, True)
        Kc.append(kc); Ks.append(ks); Vc.append(vc); Vs.append(vs)
        K16.append(half_bits((kc.astype(np.float64) - 128) * ks[:, :, None]))
        V16.append(half_bits((vc.astype(np.float64) - 128) * vs[:, :, None]))
        assert np.array_equal(f64(K16[-1]), (kc.astype(np.float64) - 128) * ks[:, :, None])
    lens = np.asarray(Ls, dtype=np.int32)
    out_q, lse_q = O.rpartq_decode(Kc, Ks, Vc, Vs, lens, q)
    out_h, lse_h, _ = O.rpart_decode(K16, V16, lens, q)
    assert np.abs(out_q - out_h).max() < 1e-13 and np.abs(lse_q - lse_h).max() < 1e-13


def test_quantised_attention_against_numpy_definition():
    rng = np.random.default_rng(6)
    H, d, L = 2, 32, 50
    kc, ks, vc, vs = _random_qcache(rng, L, H, d, False)
    q = half_bits(rng.standard_normal((1, H, d)))
    out, lse = O.rpartq_decode([kc], [ks], [vc], [vs], np.array([L], np.int32), q)
    k = (kc.astype(np.float64) - 128) * ks.astype(np.float64)[:, :, None]
    v = (vc.astype(np.float64) - 128) * vs.astype(np.float64)[:, :, None]
    s = np.einsum("thd,hd->ht", k, f64(q)[0]) / math.sqrt(d)
    w = np.exp(s - s.max(axis=1, keepdims=True))
    w /= w.sum(axis=1, keepdims=True)
    assert np.abs(out[0] - np.einsum("ht,thd->hd", w, v)).max() < 1e-13
    assert np.abs(lse[0] - (s.max(axis=1) + np.log(np.exp(s - s.max(axis=1, keepdims=True)).sum(axis=1)))).max() < 1e-12
    # empty sequence
    out0, lse0 = O.rpartq_decode([kc], [ks], [vc], [vs], np.array([0], np.int32), q)
    assert np.all(out0 == 0) and np.all(np.isneginf(lse0))


def test_quantised_append_stores_codes_and_scales_at_the_new_row():
    rng = np.random.default_rng(7)
    B, H, d = 2, 3, 16
    L = np.array([0, 4], dtype=np.int32)
    Kc = [rng.integers(0, 256, size=(l + 2, H, d)).astype(np.uint8) for l in L]
    Vc = [rng.integers(0, 256, size=(l + 2, H, d)).astype(np.uint8) for l in L]
    Ks = [rng.uniform(0, 1, size=(l + 2, H)).astype(np.float32) for l in L]
    Vs = [rng.uniform(0, 1, size=(l + 2, H)).astype(np.float32) for l in L]
    before = [a.copy() for a in Kc + Vc + Ks + Vs]
    k_new = half_bits(rng.standard_normal((B, H, d)))
    v_new = half_bits(rng.standard_normal((B, H, d)) * 4)
    lens = L.copy()
    O.kvq_append(Kc, Ks, Vc, Vs, lens, k_new, v_new)
    assert np.array_equal(lens, L + 1)
    kc_ref, ks_ref = O.quantize_rows_i8(k_new)
    vc_ref, vs_ref = O.quantize_rows_i8(v_new)
    for b in range(B):
        assert np.array_equal(Kc[b][L[b]], kc_ref[b]) and np.array_equal(Ks[b][L[b]], ks_ref[b])
        assert np.array_equal(Vc[b][L[b]], vc_ref[b]) and np.array_equal(Vs[b][L[b]], vs_ref[b])
    after = Kc + Vc + Ks + Vs
    for idx, (a0, a1) in enumerate(zip(before, after)):
        b = idx % B
        keep = np.ones(a0.shape[0], dtype=bool)
        keep[L[b]] = False
        assert np.array_equal(a0[keep], a1[keep])


def test_quantisation_error_of_attention_is_small_on_normal_data():
    """Sanity of the scheme itself: int8 storage changes the attention output by well under
    1 % of max|V| on N(0,1) keys and values (each element moves by at most scale/2)."""
    rng = np.random.default_rng(8)
    H, d, L = 4, 128, 400
    K = half_bits(rng.standard_normal((L, H, d)))
    V = half_bits(rng.standard_normal((L, H, d)))
    q = half_bits(rng.standard_normal((1, H, d)))
    lens = np.array([L], np.int32)
    ref, _, _ = O.rpart_decode([K], [V], lens, q)
    kc, ks = O.quantize_rows_i8(K)
    vc, vs = O.quantize_rows_i8(V)
    got, _ = O.rpartq_decode([kc], [ks], [vc], [vs], lens, q)
    assert np.abs(got - ref).max() < 0.01 * np.abs(f64(V)).max()
