"""ctypes binding over ``include/fastdecode_sched.h`` (FastDecode Section 4.2, host integer logic)."""
from __future__ import annotations

import ctypes
from typing import List, Sequence, Tuple

from . import rpart

_i64 = ctypes.c_int64
_configured = False


def _lib():
    global _configured
    lib = rpart.load()
    if not _configured:
        P = ctypes.POINTER(_i64)
        lib.fd_sls_microbatch_size.restype = _i64
        lib.fd_sls_microbatch_size.argtypes = [_i64] * 3
        lib.fd_sls_peak_load.restype = _i64
        lib.fd_sls_peak_load.argtypes = [_i64] * 3
        lib.fd_sls_step_loads.restype = ctypes.c_int
        lib.fd_sls_step_loads.argtypes = [_i64] * 4 + [P]
        lib.fd_batch_step_loads.restype = ctypes.c_int
        lib.fd_batch_step_loads.argtypes = [_i64] * 3 + [P]
        lib.fd_lc_create.restype = ctypes.c_void_p
        lib.fd_lc_create.argtypes = [_i64, _i64]
        lib.fd_lc_destroy.restype = None
        lib.fd_lc_destroy.argtypes = [ctypes.c_void_p]
        lib.fd_lc_add_microbatch.restype = ctypes.c_int
        lib.fd_lc_add_microbatch.argtypes = [ctypes.c_void_p, _i64, _i64]
        lib.fd_lc_earliest_step.restype = _i64
        lib.fd_lc_earliest_step.argtypes = [ctypes.c_void_p, _i64, _i64]
        lib.fd_lc_retire.restype = _i64
        lib.fd_lc_retire.argtypes = [ctypes.c_void_p, _i64]
        lib.fd_lc_count.restype = _i64
        lib.fd_lc_count.argtypes = [ctypes.c_void_p]
        lib.fd_lc_snapshot.restype = _i64
        lib.fd_lc_snapshot.argtypes = [ctypes.c_void_p, _i64, P, P, P]
        lib.fd_lc_controlled_starts.restype = _i64
        lib.fd_lc_controlled_starts.argtypes = [_i64] * 6 + [P, _i64]
        lib.fd_slots_create.restype = ctypes.c_void_p
        lib.fd_slots_create.argtypes = [ctypes.c_int32]
        lib.fd_slots_destroy.restype = None
        lib.fd_slots_destroy.argtypes = [ctypes.c_void_p]
        lib.fd_slots_acquire.restype = ctypes.c_int32
        lib.fd_slots_acquire.argtypes = [ctypes.c_void_p]
        lib.fd_slots_release.restype = ctypes.c_int
        lib.fd_slots_release.argtypes = [ctypes.c_void_p, ctypes.c_int32]
        lib.fd_slots_in_use.restype = ctypes.c_int32
        lib.fd_slots_in_use.argtypes = [ctypes.c_void_p]
        _f64 = ctypes.c_double
        lib.fd_model_sequence_latency.restype = _f64
        lib.fd_model_sequence_latency.argtypes = [_i64, _i64, _f64]
        lib.fd_model_max_batch.restype = _i64
        lib.fd_model_max_batch.argtypes = [_i64, _i64, _f64, P, ctypes.POINTER(_f64), _i64]
        lib.fd_model_sworker_throughput.restype = _f64
        lib.fd_model_sworker_throughput.argtypes = [_i64, _f64]
        lib.fd_model_min_rworkers_memory.restype = _i64
        lib.fd_model_min_rworkers_memory.argtypes = [_i64, _i64, _i64]
        lib.fd_model_num_rworkers.restype = _f64
        lib.fd_model_num_rworkers.argtypes = [_i64, _i64, _f64, _f64]
        _configured = True
    return lib


EXPORTS = ("fd_sls_microbatch_size", "fd_sls_peak_load", "fd_sls_step_loads", "fd_batch_step_loads",
           "fd_lc_create", "fd_lc_destroy", "fd_lc_add_microbatch", "fd_lc_earliest_step",
           "fd_lc_retire", "fd_lc_count", "fd_lc_snapshot", "fd_lc_controlled_starts",
           "fd_model_sequence_latency", "fd_model_max_batch", "fd_model_sworker_throughput",
           "fd_model_min_rworkers_memory", "fd_model_num_rworkers",
           "fd_slots_create", "fd_slots_destroy", "fd_slots_acquire", "fd_slots_release",
           "fd_slots_in_use",
           "fd_build_id")


def _ok(v: int, where: str) -> int:
    if v < 0:
        raise rpart.FdError(int(v), where)
    return int(v)


def sls_microbatch_size(B: int, F: int, S: int) -> int:
    return _ok(_lib().fd_sls_microbatch_size(B, F, S), "fd_sls_microbatch_size")


def sls_peak_load(M: int, F: int, S: int) -> int:
    return _ok(_lib().fd_sls_peak_load(M, F, S), "fd_sls_peak_load")


def sls_step_loads(M: int, F: int, S: int, n_steps: int) -> List[int]:
    buf = (_i64 * max(1, n_steps))()
    _ok(_lib().fd_sls_step_loads(M, F, S, n_steps, buf), "fd_sls_step_loads")
    return list(buf)[:n_steps]


def batch_step_loads(B: int, S: int, n_steps: int) -> List[int]:
    buf = (_i64 * max(1, n_steps))()
    _ok(_lib().fd_batch_step_loads(B, S, n_steps, buf), "fd_batch_step_loads")
    return list(buf)[:n_steps]


class LoadControl:
    """Algorithm 1: bookkeeping of the current micro-batches and the earliest start step."""

    def __init__(self, S: int, W_lim: int):
        self._h = _lib().fd_lc_create(S, W_lim)
        if not self._h:
            raise rpart.FdError(rpart.FD_EINVAL, "fd_lc_create")

    def close(self) -> None:
        if self._h:
            _lib().fd_lc_destroy(self._h)
            self._h = None

    __del__ = close

    def add_microbatch(self, t: int, m: int) -> None:
        _ok(_lib().fd_lc_add_microbatch(self._h, t, m), "fd_lc_add_microbatch")

    def earliest_step(self, t: int, m: int) -> int:
        return _ok(_lib().fd_lc_earliest_step(self._h, t, m), "fd_lc_earliest_step")

    def retire(self, t: int) -> int:
        return _ok(_lib().fd_lc_retire(self._h, t), "fd_lc_retire")

    def __len__(self) -> int:
        return _ok(_lib().fd_lc_count(self._h), "fd_lc_count")

    def snapshot(self) -> List[Tuple[int, int, int]]:
        n = len(self)
        M, E, W = ((_i64 * max(1, n))() for _ in range(3))
        c = _ok(_lib().fd_lc_snapshot(self._h, n, M, E, W), "fd_lc_snapshot")
        return [(M[i], E[i], W[i]) for i in range(c)]


def controlled_starts(B: int, S: int, M: int, F: int, W_lim: int, n_steps: int) -> List[int]:
    """Start steps of the micro-batches admitted by Algorithm 1's driver (fd_lc_controlled_starts)."""
    cap = max(1, n_steps)
    buf = (_i64 * cap)()
    n = _ok(_lib().fd_lc_controlled_starts(B, S, M, F, W_lim, n_steps, buf, cap), "fd_lc_controlled_starts")
    return list(buf)[:n]


# ---------------------------------------------------------------------------
# Section 4.3: batch size and number of R-workers from the measured T(B) and R
# ---------------------------------------------------------------------------
def _finite(v: float, where: str) -> float:
    if v != v:
        raise rpart.FdError(rpart.FD_EINVAL, where)
    return float(v)


def model_sequence_latency(N: int, S: int, T_B: float) -> float:
    return _finite(_lib().fd_model_sequence_latency(N, S, T_B), "fd_model_sequence_latency")


def model_max_batch(N: int, S: int, L: float, table: Sequence[Tuple[int, float]]) -> int:
    n = len(table)
    Bs = (_i64 * max(1, n))(*[b for b, _ in table])
    T = (ctypes.c_double * max(1, n))(*[t for _, t in table])
    return _ok(_lib().fd_model_max_batch(N, S, L, Bs, T, n), "fd_model_max_batch")


def model_sworker_throughput(B: int, T_B: float) -> float:
    return _finite(_lib().fd_model_sworker_throughput(B, T_B), "fd_model_sworker_throughput")


def model_min_rworkers_memory(B: int, S: int, C: int) -> int:
    return _ok(_lib().fd_model_min_rworkers_memory(B, S, C), "fd_model_min_rworkers_memory")


def model_num_rworkers(B: int, S: int, R: float, T_B: float) -> float:
    return _finite(_lib().fd_model_num_rworkers(B, S, R, T_B), "fd_model_num_rworkers")


class Slots:
    """Free list of the B sequence slots of an R-worker (Section 4.1: dropped sequences hand
    their slot to later ones)."""

    def __init__(self, B: int):
        self._h = _lib().fd_slots_create(B)
        if not self._h:
            raise rpart.FdError(rpart.FD_EINVAL, "fd_slots_create")

    def close(self) -> None:
        if self._h:
            _lib().fd_slots_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def acquire(self) -> int:
        """A free slot id, or -1 when every slot is taken."""
        return int(_lib().fd_slots_acquire(self._h))

    def release(self, slot: int) -> None:
        _ok(_lib().fd_slots_release(self._h, slot), "fd_slots_release")

    def in_use(self) -> int:
        return _ok(_lib().fd_slots_in_use(self._h), "fd_slots_in_use")
