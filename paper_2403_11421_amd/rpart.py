"""ctypes binding over the C ABI in ``include/fastdecode_rpart.h``.

Argument marshalling only: every step of the path runs in the HIP kernels of
``libfd_rpart.so``.  torch supplies device memory and the current stream.
There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from . import build as _build

FD_OK, FD_EINVAL, FD_EWORKSPACE, FD_EHIP, FD_ETOOBIG = 0, -1, -2, -3, -4
FD_NOALLOC_SCRATCH_BYTES = 64 << 20
FD_ST_CAPACITY, FD_ST_BADLEN, FD_ST_WINDOW, FD_ST_PLAN = 1, 2, 4, 8
FD_SLOT_FREE = -1

_vp = ctypes.c_void_p


class fd_kv_desc(ctypes.Structure):
    _fields_ = [
        ("k_base", _vp), ("v_base", _vp), ("seq_off", _vp), ("seq_cap", _vp),
        ("seq_lens", _vp), ("status", _vp),
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d", ctypes.c_int32),
        ("chunk_tokens", ctypes.c_int32),
        ("seq_seen", _vp), ("n_sink", ctypes.c_int32),
    ]


class fd_kvq_desc(ctypes.Structure):
    _fields_ = [
        ("k_codes", _vp), ("v_codes", _vp), ("k_scale", _vp), ("v_scale", _vp),
        ("seq_off", _vp), ("seq_cap", _vp), ("seq_lens", _vp), ("status", _vp),
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d", ctypes.c_int32),
        ("chunk_tokens", ctypes.c_int32),
        ("seq_seen", _vp), ("n_sink", ctypes.c_int32), ("bits", ctypes.c_int32),
    ]


class FdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def lib_path() -> str:
    return _build.LIB


def load() -> ctypes.CDLL:
    """Load the built library.  It is built first if none exists; a library older than one of
    its sources is rebuilt where a compiler is at hand and refused otherwise, so that a stale
    build is never tested or timed silently."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    elif _build.is_stale():
        if not _build.have_compiler():
            raise RuntimeError(f"{_build.LIB} is older than its sources and no hipcc is available to rebuild it")
        _build.build()
    lib = ctypes.CDLL(_build.LIB)
    P = ctypes.POINTER(fd_kv_desc)
    lib.fd_version.restype = ctypes.c_int
    lib.fd_version.argtypes = []
    lib.fd_desc_size.restype = ctypes.c_size_t
    lib.fd_desc_size.argtypes = [ctypes.c_int]
    if lib.fd_desc_size(0) != ctypes.sizeof(fd_kv_desc) or lib.fd_desc_size(1) != ctypes.sizeof(fd_kvq_desc):
        raise RuntimeError("libfd_rpart.so was built from a different fastdecode_rpart.h than this binding mirrors")
    lib.fd_strerror.restype = ctypes.c_char_p
    lib.fd_strerror.argtypes = [ctypes.c_int]
    lib.fd_workspace_bytes.restype = ctypes.c_size_t
    lib.fd_workspace_bytes.argtypes = [ctypes.c_int32] * 3 + [ctypes.c_int64]
    lib.fd_kv_append.restype = ctypes.c_int
    lib.fd_kv_append.argtypes = [P, _vp, _vp, _vp]
    lib.fd_rpart_decode.restype = ctypes.c_int
    lib.fd_rpart_decode.argtypes = [P, _vp, _vp, _vp, ctypes.c_size_t, _vp]
    lib.fd_kv_append_plan.restype = ctypes.c_int
    lib.fd_kv_append_plan.argtypes = [P, _vp, _vp, _vp, ctypes.c_size_t, _vp]
    lib.fd_rpart_decode_noalloc.restype = ctypes.c_int
    lib.fd_rpart_decode_noalloc.argtypes = [P, _vp, _vp, _vp]
    lib.fd_rpart_plan.restype = ctypes.c_int
    lib.fd_rpart_plan.argtypes = [P, _vp, ctypes.c_size_t, _vp]
    lib.fd_rpart_partial.restype = ctypes.c_int
    lib.fd_rpart_partial.argtypes = [P, _vp, _vp, _vp, ctypes.c_size_t, _vp]
    lib.fd_rpart_merge.restype = ctypes.c_int
    lib.fd_rpart_merge.argtypes = [P, _vp, _vp, ctypes.c_size_t, _vp]
    lib.fd_rpart_step.restype = ctypes.c_int
    lib.fd_rpart_step.argtypes = [P, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
    lib.fd_rpart_layer_step.restype = ctypes.c_int
    lib.fd_rpart_layer_step.argtypes = [P, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, ctypes.c_int, _vp]
    lib.fd_kv_reset.restype = ctypes.c_int
    lib.fd_kv_reset.argtypes = [P, _vp, ctypes.c_int32, _vp]
    lib.fd_kv_release.restype = ctypes.c_int
    lib.fd_kv_release.argtypes = [P, _vp, ctypes.c_int32, _vp]
    lib.fd_read_status.restype = ctypes.c_int
    lib.fd_read_status.argtypes = [P, ctypes.POINTER(ctypes.c_int32), ctypes.c_int, _vp]
    lib.fd_last_device_status.restype = ctypes.c_int
    lib.fd_last_device_status.argtypes = [P, _vp, ctypes.POINTER(ctypes.c_int32), _vp]
    lib.fd_kv_store_rows.restype = ctypes.c_int
    lib.fd_kv_store_rows.argtypes = [P, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _vp, _vp, ctypes.c_int, _vp]
    lib.fd_plan_info.restype = ctypes.c_int
    lib.fd_plan_info.argtypes = [_vp, ctypes.POINTER(ctypes.c_int32), _vp]
    Q = ctypes.POINTER(fd_kvq_desc)
    for name, args in (("fd_kvq_append", [Q, _vp, _vp, _vp]),
                       ("fd_kvq_store_rows", [Q, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _vp, _vp,
                                              ctypes.c_int, _vp]),
                       ("fd_kvq_append_plan", [Q, _vp, _vp, _vp, ctypes.c_size_t, _vp]),
                       ("fd_kvq_reset", [Q, _vp, ctypes.c_int32, _vp]),
                       ("fd_kvq_release", [Q, _vp, ctypes.c_int32, _vp]),
                       ("fd_rpartq_plan", [Q, _vp, ctypes.c_size_t, _vp]),
                       ("fd_rpartq_partial", [Q, _vp, _vp, _vp, ctypes.c_size_t, _vp]),
                       ("fd_rpartq_merge", [Q, _vp, _vp, ctypes.c_size_t, _vp]),
                       ("fd_rpartq_decode", [Q, _vp, _vp, _vp, ctypes.c_size_t, _vp]),
                       ("fd_rpartq_step", [Q, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]),
                       ("fd_rpartq_layer_step", [Q, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t,
                                                 ctypes.c_int, _vp])):
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = args
    lib.fd_fill_pattern.restype = ctypes.c_int
    lib.fd_fill_pattern.argtypes = [_vp, ctypes.c_size_t, ctypes.c_uint32, _vp]
    lib.fd_hbm_read_probe.restype = ctypes.c_int
    lib.fd_hbm_read_probe.argtypes = [_vp, ctypes.c_size_t, _vp, ctypes.POINTER(ctypes.c_size_t), _vp]
    _lib = lib
    return lib


EXPORTS = ("fd_version", "fd_desc_size", "fd_strerror", "fd_workspace_bytes", "fd_kv_append", "fd_rpart_decode",
           "fd_rpart_plan", "fd_rpart_partial", "fd_rpart_merge", "fd_rpart_step", "fd_kv_reset",
           "fd_read_status", "fd_plan_info", "fd_hbm_read_probe",
           "fd_kvq_append", "fd_kvq_reset", "fd_rpartq_plan", "fd_rpartq_partial", "fd_rpartq_merge",
           "fd_rpartq_decode", "fd_rpartq_step", "fd_rpart_layer_step", "fd_rpartq_layer_step",
           "fd_kv_release", "fd_kvq_release", "fd_rpart_decode_noalloc", "fd_last_device_status",
           "fd_kv_store_rows", "fd_kvq_store_rows", "fd_kv_append_plan", "fd_kvq_append_plan", "fd_fill_pattern")


def version() -> int:
    return load().fd_version()


def strerror(code: int) -> str:
    return load().fd_strerror(code).decode()


def workspace_bytes(B: int, H: int, d: int, max_total_tokens: int) -> int:
    return int(load().fd_workspace_bytes(B, H, d, max_total_tokens))


def _stream() -> Optional[int]:
    return torch.cuda.current_stream().cuda_stream or None


def _check(rc: int, where: str) -> None:
    if rc != FD_OK:
        raise FdError(rc, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _ws(ws: torch.Tensor):
    return ws.data_ptr(), ws.numel() * ws.element_size()


def fd_kv_append(desc: fd_kv_desc, k_new: torch.Tensor, v_new: torch.Tensor) -> None:
    _check(load().fd_kv_append(ctypes.byref(desc), _ptr(k_new), _ptr(v_new), _stream()),
           "fd_kv_append")


def fd_kv_append_plan(desc, k_new: torch.Tensor, v_new: torch.Tensor, workspace: torch.Tensor) -> None:
    """Append and plan in one launch (front half of a step); `desc` is an fd_kv_desc or an
    fd_kvq_desc.  The streaming call on the same workspace must follow."""
    p, n = _ws(workspace)
    quant = isinstance(desc, fd_kvq_desc)
    f = load().fd_kvq_append_plan if quant else load().fd_kv_append_plan
    _check(f(ctypes.byref(desc), _ptr(k_new), _ptr(v_new), p, n, _stream()),
           "fd_kvq_append_plan" if quant else "fd_kv_append_plan")


def fd_rpart_decode(desc: fd_kv_desc, q: torch.Tensor, out: torch.Tensor,
                    workspace: torch.Tensor) -> None:
    p, n = _ws(workspace)
    _check(load().fd_rpart_decode(ctypes.byref(desc), _ptr(q), _ptr(out), p, n, _stream()),
           "fd_rpart_decode")


def fd_rpart_decode_noalloc(desc: fd_kv_desc, q: torch.Tensor, out: torch.Tensor) -> None:
    """fd_rpart_decode on the library's built-in scratch array (no workspace, no allocation)."""
    _check(load().fd_rpart_decode_noalloc(ctypes.byref(desc), _ptr(q), _ptr(out), _stream()),
           "fd_rpart_decode_noalloc")


def fd_rpart_plan(desc: fd_kv_desc, workspace: torch.Tensor) -> None:
    p, n = _ws(workspace)
    _check(load().fd_rpart_plan(ctypes.byref(desc), p, n, _stream()), "fd_rpart_plan")


def fd_rpart_partial(desc: fd_kv_desc, q: torch.Tensor, out: torch.Tensor,
                     workspace: torch.Tensor) -> None:
    p, n = _ws(workspace)
    _check(load().fd_rpart_partial(ctypes.byref(desc), _ptr(q), _ptr(out), p, n, _stream()),
           "fd_rpart_partial")


def fd_rpart_merge(desc: fd_kv_desc, out: torch.Tensor, workspace: torch.Tensor) -> None:
    p, n = _ws(workspace)
    _check(load().fd_rpart_merge(ctypes.byref(desc), _ptr(out), p, n, _stream()), "fd_rpart_merge")


def fd_rpart_step(desc: fd_kv_desc, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                  out: torch.Tensor, workspace: torch.Tensor) -> None:
    p, n = _ws(workspace)
    _check(load().fd_rpart_step(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                p, n, _stream()), "fd_rpart_step")


def fd_kv_reset(desc: fd_kv_desc, seq_ids: Optional[torch.Tensor] = None) -> None:
    n = 0 if seq_ids is None else seq_ids.numel()
    _check(load().fd_kv_reset(ctypes.byref(desc), _ptr(seq_ids), n, _stream()), "fd_kv_reset")


def fd_kv_release(desc, seq_ids: Optional[torch.Tensor] = None) -> None:
    """Mark slots free (seq_lens = FD_SLOT_FREE); `desc` is an fd_kv_desc or an fd_kvq_desc."""
    n = 0 if seq_ids is None else seq_ids.numel()
    quant = isinstance(desc, fd_kvq_desc)
    f = load().fd_kvq_release if quant else load().fd_kv_release
    _check(f(ctypes.byref(desc), _ptr(seq_ids), n, _stream()),
           "fd_kvq_release" if quant else "fd_kv_release")


def fd_read_status(desc, clear: bool = False) -> int:
    """Sticky device status of an fp16 or a quantised cache (both keep it in `desc.status`)."""
    probe = fd_kv_desc(status=desc.status)
    v = ctypes.c_int32(0)
    _check(load().fd_read_status(ctypes.byref(probe), ctypes.byref(v), int(clear), _stream()),
           "fd_read_status")
    return v.value


def fd_last_device_status(desc, workspace: torch.Tensor) -> int:
    """Take the sticky device status (read and clear in one atomic step); fp16 or quantised cache."""
    probe = fd_kv_desc(status=desc.status)
    v = ctypes.c_int32(0)
    _check(load().fd_last_device_status(ctypes.byref(probe), workspace.data_ptr(), ctypes.byref(v), _stream()),
           "fd_last_device_status")
    return v.value


def fd_kv_store_rows(desc, b: int, t0: int, k_rows: Optional[torch.Tensor],
                     v_rows: Optional[torch.Tensor], set_len: bool = False) -> None:
    """Store token rows [H, n, d] (fp16, contiguous) at tokens t0.. of sequence b; `desc` is an
    fd_kv_desc (bit copy) or an fd_kvq_desc (quantised as the append does)."""
    rows = k_rows if k_rows is not None else v_rows
    n = 0 if rows is None else int(rows.shape[1])
    for t in (k_rows, v_rows):
        assert t is None or (t.is_contiguous() and t.dtype == torch.float16 and t.shape[1] == n)
    quant = isinstance(desc, fd_kvq_desc)
    f = load().fd_kvq_store_rows if quant else load().fd_kv_store_rows
    _check(f(ctypes.byref(desc), b, t0, n, _ptr(k_rows), _ptr(v_rows), 1 if set_len else 0, _stream()),
           "fd_kvq_store_rows" if quant else "fd_kv_store_rows")


def fd_plan_info(workspace: torch.Tensor) -> dict:
    info = (ctypes.c_int32 * 4)()
    _check(load().fd_plan_info(workspace.data_ptr(), info, _stream()), "fd_plan_info")
    return {"items": info[0], "chunk_tokens": info[1], "total_tokens": info[2], "grid": info[3]}


def fd_hbm_read_probe(buf: torch.Tensor, sink: torch.Tensor) -> int:
    """Enqueue the pure-read probe over `buf`; returns the bytes it reads."""
    n = ctypes.c_size_t(0)
    _check(load().fd_hbm_read_probe(buf.data_ptr(), buf.numel() * buf.element_size(),
                                    sink.data_ptr(), ctypes.byref(n), _stream()),
           "fd_hbm_read_probe")
    return int(n.value)


def fd_fill_pattern(buf: torch.Tensor, seed: int) -> None:
    """Fill a device tensor with the library's seeded bit pattern (no torch kernel involved)."""
    _check(load().fd_fill_pattern(buf.data_ptr(), buf.numel() * buf.element_size(), seed & 0xFFFFFFFF,
                                  _stream()), "fd_fill_pattern")


# ---------------------------------------------------------------------------
# quantised KV-cache (int8 codes + float32 scales)
# ---------------------------------------------------------------------------
def fd_kvq_append(desc: fd_kvq_desc, k_new: torch.Tensor, v_new: torch.Tensor) -> None:
    _check(load().fd_kvq_append(ctypes.byref(desc), _ptr(k_new), _ptr(v_new), _stream()),
           "fd_kvq_append")


def fd_kvq_reset(desc: fd_kvq_desc, seq_ids: Optional[torch.Tensor] = None) -> None:
    n = 0 if seq_ids is None else seq_ids.numel()
    _check(load().fd_kvq_reset(ctypes.byref(desc), _ptr(seq_ids), n, _stream()), "fd_kvq_reset")


def fd_rpartq_plan(desc: fd_kvq_desc, workspace: torch.Tensor) -> None:
    p, n = _ws(workspace)
    _check(load().fd_rpartq_plan(ctypes.byref(desc), p, n, _stream()), "fd_rpartq_plan")


def fd_rpartq_partial(desc: fd_kvq_desc, q: torch.Tensor, out: torch.Tensor,
                      workspace: torch.Tensor) -> None:
    p, n = _ws(workspace)
    _check(load().fd_rpartq_partial(ctypes.byref(desc), _ptr(q), _ptr(out), p, n, _stream()),
           "fd_rpartq_partial")


def fd_rpartq_merge(desc: fd_kvq_desc, out: torch.Tensor, workspace: torch.Tensor) -> None:
    p, n = _ws(workspace)
    _check(load().fd_rpartq_merge(ctypes.byref(desc), _ptr(out), p, n, _stream()), "fd_rpartq_merge")


def fd_rpartq_decode(desc: fd_kvq_desc, q: torch.Tensor, out: torch.Tensor,
                     workspace: torch.Tensor) -> None:
    p, n = _ws(workspace)
    _check(load().fd_rpartq_decode(ctypes.byref(desc), _ptr(q), _ptr(out), p, n, _stream()),
           "fd_rpartq_decode")


def fd_rpartq_step(desc: fd_kvq_desc, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                   out: torch.Tensor, workspace: torch.Tensor) -> None:
    p, n = _ws(workspace)
    _check(load().fd_rpartq_step(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                 p, n, _stream()), "fd_rpartq_step")


def fd_rpart_layer_step(layer, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                        out: torch.Tensor, workspace: torch.Tensor, replan: bool) -> None:
    """One block's append + attend; `layer` is an fd_kv_desc or an fd_kvq_desc."""
    p, n = _ws(workspace)
    quant = isinstance(layer, fd_kvq_desc)
    f = load().fd_rpartq_layer_step if quant else load().fd_rpart_layer_step
    _check(f(ctypes.byref(layer), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), p, n,
             1 if replan else 0, _stream()),
           "fd_rpartq_layer_step" if quant else "fd_rpart_layer_step")
