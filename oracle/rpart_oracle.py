"""ctypes access to the fp64 reference in ``rpart_oracle.c``.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU
baseline leg may import this; the GPU library and its binding never do.

Layout used on this side: one token-major ``uint16 [cap_b, H, d]`` numpy array
per sequence for K and one for V (binary16 bit patterns).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rpart_oracle.c")
_LIB = os.path.join(_HERE, "librpart_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C reference with gcc (about a second)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
                               "-o", _LIB, _SRC, "-lm", "-lpthread"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.fdo_half_to_double.restype = ctypes.c_double
        lib.fdo_half_to_double.argtypes = [ctypes.c_uint16]
        lib.fdo_kv_append.restype = None
        lib.fdo_kv_append.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 5
        lib.fdo_rpart_decode.restype = ctypes.c_int
        lib.fdo_rpart_decode.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 8 + [ctypes.c_int]
        lib.fdo_quantize_row_i8.restype = None
        lib.fdo_quantize_row_i8.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        lib.fdo_quantize_rows_i8.restype = None
        lib.fdo_quantize_rows_i8.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        lib.fdo_quantize_rows_u4.restype = None
        lib.fdo_quantize_rows_u4.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        lib.fdo_kvq_append.restype = None
        lib.fdo_kvq_append.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 7
        lib.fdo_rpartq_decode.restype = ctypes.c_int
        lib.fdo_rpartq_decode.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 8
        lib.fdo_quantize_row_u4.restype = None
        lib.fdo_quantize_row_u4.argtypes = [ctypes.c_void_p, ctypes.c_int] + [ctypes.c_void_p] * 3
        lib.fdo_kvq4_append.restype = None
        lib.fdo_kvq4_append.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 7
        lib.fdo_rpartq4_decode.restype = ctypes.c_int
        lib.fdo_rpartq4_decode.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 8
        _lib = lib
    return _lib


def half_to_double(bits: int) -> float:
    return _load().fdo_half_to_double(int(bits) & 0xFFFF)


def _ptr_array(arrs: Sequence[np.ndarray]):
    for a in arrs:
        assert a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"]
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def kv_append(K: List[np.ndarray], V: List[np.ndarray], seq_lens: np.ndarray,
              k_new: np.ndarray, v_new: np.ndarray) -> None:
    """In place: store k_new[b], v_new[b] at row seq_lens[b]; seq_lens += 1.

    K[b], V[b]: uint16 [cap_b, H, d] with cap_b > seq_lens[b]; k_new, v_new: uint16 [B, H, d].
    """
    B, H, d = k_new.shape
    assert seq_lens.dtype == np.int32 and len(K) == len(V) == B == len(seq_lens)
    for b in range(B):
        assert K[b].shape[1:] == (H, d) and V[b].shape[1:] == (H, d)
        assert K[b].shape[0] > seq_lens[b] and V[b].shape[0] > seq_lens[b], "cache full"
    k_new = np.ascontiguousarray(k_new, dtype=np.uint16)
    v_new = np.ascontiguousarray(v_new, dtype=np.uint16)
    _load().fdo_kv_append(B, H, d, seq_lens.ctypes.data, _ptr_array(K), _ptr_array(V),
                          k_new.ctypes.data, v_new.ctypes.data)


def rpart_decode(K: List[np.ndarray], V: List[np.ndarray], seq_lens: np.ndarray,
                 q: np.ndarray, want_weights: bool = False, nthreads: int = 1
                 ) -> Tuple[np.ndarray, np.ndarray, Optional[List[np.ndarray]]]:
    """Attention of q[b,h] over rows [0, seq_lens[b]) of sequence b's cache.

    Returns (out float64 [B,H,d], lse float64 [B,H], weights or None) where
    weights[b] is float64 [H, seq_lens[b]].
    """
    B, H, d = q.shape
    assert seq_lens.dtype == np.int32 and len(K) == len(V) == B == len(seq_lens)
    for b in range(B):
        assert K[b].shape[1:] == (H, d) and V[b].shape[1:] == (H, d)
        assert K[b].shape[0] >= seq_lens[b] and V[b].shape[0] >= seq_lens[b]
    q = np.ascontiguousarray(q, dtype=np.uint16)
    out = np.empty((B, H, d), dtype=np.float64)
    lse = np.empty((B, H), dtype=np.float64)
    wbuf = woff = None
    if want_weights:
        sizes = [int(H) * int(L) for L in seq_lens]
        woff = np.zeros(B, dtype=np.int64)
        if B > 1:
            woff[1:] = np.cumsum(sizes)[:-1]
        wbuf = np.zeros(max(1, sum(sizes)), dtype=np.float64)
    rc = _load().fdo_rpart_decode(B, H, d, seq_lens.ctypes.data, _ptr_array(K), _ptr_array(V),
                                  q.ctypes.data, out.ctypes.data, lse.ctypes.data,
                                  wbuf.ctypes.data if want_weights else None,
                                  woff.ctypes.data if want_weights else None, int(nthreads))
    if rc != 0:
        raise ValueError("fdo_rpart_decode: invalid arguments")
    weights = None
    if want_weights:
        weights = [wbuf[woff[b]: woff[b] + H * int(seq_lens[b])].reshape(H, int(seq_lens[b]))
                   for b in range(B)]
    return out, lse, weights


# ---------------------------------------------------------------------------
# quantised KV-cache (Section 5.2): bytes = code + 128, one float32 scale per token and head
# ---------------------------------------------------------------------------
def _ptrs(arrs, dtype):
    for a in arrs:
        assert a.dtype == dtype and a.flags["C_CONTIGUOUS"]
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def quantize_rows_i8(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """x: uint16 [..., d] binary16 patterns -> (codes uint8 [..., d], scales float32 [...])."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    d = x.shape[-1]
    flat = x.reshape(-1, d)
    codes = np.empty(flat.shape, dtype=np.uint8)
    scales = np.empty(flat.shape[0], dtype=np.float32)
    _load().fdo_quantize_rows_i8(flat.ctypes.data, flat.shape[0], d, codes.ctypes.data, scales.ctypes.data)
    return codes.reshape(x.shape), scales.reshape(x.shape[:-1])


def kvq_append(Kc, Ks, Vc, Vs, seq_lens: np.ndarray, k_new: np.ndarray, v_new: np.ndarray) -> None:
    """In place: quantise k_new[b], v_new[b] into row seq_lens[b]; seq_lens += 1.

    Kc[b], Vc[b]: uint8 [cap_b, H, d]; Ks[b], Vs[b]: float32 [cap_b, H]."""
    B, H, d = k_new.shape
    assert seq_lens.dtype == np.int32 and len(Kc) == len(Ks) == len(Vc) == len(Vs) == B
    for b in range(B):
        assert Kc[b].shape[1:] == (H, d) and Ks[b].shape[1:] == (H,)
        assert Kc[b].shape[0] > seq_lens[b], "cache full"
    k_new = np.ascontiguousarray(k_new, dtype=np.uint16)
    v_new = np.ascontiguousarray(v_new, dtype=np.uint16)
    _load().fdo_kvq_append(B, H, d, seq_lens.ctypes.data, _ptrs(Kc, np.uint8), _ptrs(Ks, np.float32),
                           _ptrs(Vc, np.uint8), _ptrs(Vs, np.float32),
                           k_new.ctypes.data, v_new.ctypes.data)


def rpartq_decode(Kc, Ks, Vc, Vs, seq_lens: np.ndarray, q: np.ndarray):
    """Attention of q over the dequantised rows [0, seq_lens[b]).  Returns (out, lse) float64."""
    B, H, d = q.shape
    assert seq_lens.dtype == np.int32
    q = np.ascontiguousarray(q, dtype=np.uint16)
    out = np.empty((B, H, d), dtype=np.float64)
    lse = np.empty((B, H), dtype=np.float64)
    rc = _load().fdo_rpartq_decode(B, H, d, seq_lens.ctypes.data, _ptrs(Kc, np.uint8),
                                   _ptrs(Ks, np.float32), _ptrs(Vc, np.uint8), _ptrs(Vs, np.float32),
                                   q.ctypes.data, out.ctypes.data, lse.ctypes.data)
    if rc != 0:
        raise ValueError("fdo_rpartq_decode: invalid arguments")
    return out, lse


# ---------------------------------------------------------------------------
# 4-bit cache: packed codes (two per byte) and a (scale, zero) pair per token and head
# ---------------------------------------------------------------------------
def quantize_rows_u4(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """x: uint16 [..., d] binary16 patterns -> (packed uint8 [..., d/2], float32 [..., 2] = scale, zero)."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    d = x.shape[-1]
    assert d % 2 == 0
    flat = x.reshape(-1, d)
    packed = np.empty((flat.shape[0], d // 2), dtype=np.uint8)
    sz = np.empty((flat.shape[0], 2), dtype=np.float32)
    _load().fdo_quantize_rows_u4(flat.ctypes.data, flat.shape[0], d, packed.ctypes.data, sz.ctypes.data)
    return packed.reshape(x.shape[:-1] + (d // 2,)), sz.reshape(x.shape[:-1] + (2,))


def unpack_u4(packed: np.ndarray) -> np.ndarray:
    """uint8 [..., d/2] -> codes uint8 [..., d] (element 2j = low nibble of byte j)."""
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = packed & 15
    out[..., 1::2] = packed >> 4
    return out


def kvq4_append(Kc, Ksz, Vc, Vsz, seq_lens: np.ndarray, k_new: np.ndarray, v_new: np.ndarray) -> None:
    """In place.  Kc[b], Vc[b]: uint8 [cap_b, H, d/2]; Ksz[b], Vsz[b]: float32 [cap_b, H, 2]."""
    B, H, d = k_new.shape
    assert seq_lens.dtype == np.int32 and len(Kc) == len(Ksz) == len(Vc) == len(Vsz) == B
    for b in range(B):
        assert Kc[b].shape[1:] == (H, d // 2) and Ksz[b].shape[1:] == (H, 2)
        assert Kc[b].shape[0] > seq_lens[b], "cache full"
    k_new = np.ascontiguousarray(k_new, dtype=np.uint16)
    v_new = np.ascontiguousarray(v_new, dtype=np.uint16)
    _load().fdo_kvq4_append(B, H, d, seq_lens.ctypes.data, _ptrs(Kc, np.uint8), _ptrs(Ksz, np.float32),
                            _ptrs(Vc, np.uint8), _ptrs(Vsz, np.float32),
                            k_new.ctypes.data, v_new.ctypes.data)


def rpartq4_decode(Kc, Ksz, Vc, Vsz, seq_lens: np.ndarray, q: np.ndarray):
    """Attention of q over the dequantised rows (code * scale + zero).  Returns (out, lse) float64."""
    B, H, d = q.shape
    assert seq_lens.dtype == np.int32
    q = np.ascontiguousarray(q, dtype=np.uint16)
    out = np.empty((B, H, d), dtype=np.float64)
    lse = np.empty((B, H), dtype=np.float64)
    rc = _load().fdo_rpartq4_decode(B, H, d, seq_lens.ctypes.data, _ptrs(Kc, np.uint8),
                                    _ptrs(Ksz, np.float32), _ptrs(Vc, np.uint8), _ptrs(Vsz, np.float32),
                                    q.ctypes.data, out.ctypes.data, lse.ctypes.data)
    if rc != 0:
        raise ValueError("fdo_rpartq4_decode: invalid arguments")
    return out, lse
