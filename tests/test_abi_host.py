"""The C-ABI library loads without a GPU, exports every symbol the header declares,
and rejects bad arguments on the host before enqueuing anything."""
import ctypes
import os
import re

import pytest

from paper_2403_11421_amd import rpart

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                      "include", "fastdecode_rpart.h")


SCHED_HEADER = os.path.join(os.path.dirname(HEADER), "fastdecode_sched.h")


def _declared(path=HEADER):
    text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(fd_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = rpart.load()
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(rpart.EXPORTS)
    from paper_2403_11421_amd import sched
    sched_names = _declared(SCHED_HEADER)
    assert len(sched_names) >= 11 and set(sched_names) == set(sched.EXPORTS)
    for n in sched_names:
        assert hasattr(lib, n), n


def test_binding_mirrors_the_descriptor_structs():
    lib = rpart.load()
    assert lib.fd_desc_size(0) == ctypes.sizeof(rpart.fd_kv_desc) == 80
    assert lib.fd_desc_size(1) == ctypes.sizeof(rpart.fd_kvq_desc) == 96
    assert lib.fd_desc_size(2) == 0
    # field offsets the kernels rely on (pointers first, then the 32-bit fields)
    assert rpart.fd_kv_desc.B.offset == 48 and rpart.fd_kv_desc.seq_seen.offset == 64
    assert rpart.fd_kvq_desc.B.offset == 64 and rpart.fd_kvq_desc.bits.offset == 92


def test_version_and_strerror():
    assert rpart.version() >= 100
    assert rpart.strerror(rpart.FD_OK) == "ok"
    for code in (rpart.FD_EINVAL, rpart.FD_EWORKSPACE, rpart.FD_EHIP, -99):
        assert isinstance(rpart.strerror(code), str) and rpart.strerror(code)


def test_workspace_bytes():
    assert rpart.workspace_bytes(256, 32, 96, 10) == 0          # head_dim must be 64 or 128
    assert rpart.workspace_bytes(-1, 32, 128, 10) == 0
    assert rpart.workspace_bytes(1, 0, 128, 10) == 0
    base = rpart.workspace_bytes(256, 32, 128, 0)
    per_item = 16 + 32 * 130 * 4
    assert base >= 256 * per_item and base % 256 == 0
    more = rpart.workspace_bytes(256, 32, 128, 256 * 2049)
    assert more - base >= (256 * 2049 // 256) * per_item
    assert rpart.workspace_bytes(256, 32, 64, 0) < base


def test_host_side_argument_checks_need_no_gpu():
    lib = rpart.load()
    null = ctypes.POINTER(rpart.fd_kv_desc)()
    assert lib.fd_kv_append(null, None, None, None) == rpart.FD_EINVAL
    assert lib.fd_rpart_decode(null, None, None, None, 0, None) == rpart.FD_EINVAL
    assert lib.fd_rpart_step(null, None, None, None, None, None, 0, None) == rpart.FD_EINVAL
    assert lib.fd_kv_reset(null, None, 0, None) == rpart.FD_EINVAL
    assert lib.fd_plan_info(None, None, None) == rpart.FD_EINVAL
    d = rpart.fd_kv_desc(B=2, H=4, d=96)
    assert lib.fd_kv_append(ctypes.byref(d), None, None, None) == rpart.FD_EINVAL
    d = rpart.fd_kv_desc(B=2, H=4, d=128)                      # null cache pointers
    assert lib.fd_rpart_plan(ctypes.byref(d), None, 0, None) == rpart.FD_EINVAL
    d = rpart.fd_kv_desc(B=0, H=4, d=128)                      # empty batch: nothing to do
    assert lib.fd_kv_append(ctypes.byref(d), None, None, None) == rpart.FD_OK
    assert lib.fd_rpart_decode(ctypes.byref(d), None, None, None, 0, None) == rpart.FD_OK
    # fake, aligned, never dereferenced on the host
    d = rpart.fd_kv_desc(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 2, 4, 128, 0)
    assert lib.fd_rpart_decode(ctypes.byref(d), 0x7000, 0x8000, 0x9000, 16, None) == rpart.FD_EWORKSPACE
    assert lib.fd_rpart_decode(ctypes.byref(d), 0x7001, 0x8000, 0x9000, 1 << 30, None) == rpart.FD_EINVAL
    d.chunk_tokens = -5
    assert lib.fd_rpart_decode(ctypes.byref(d), 0x7000, 0x8000, 0x9000, 1 << 30, None) == rpart.FD_EINVAL


def test_new_entry_points_check_their_arguments_on_the_host():
    lib = rpart.load()
    null = ctypes.POINTER(rpart.fd_kv_desc)()
    v = ctypes.c_int32(0)
    assert lib.fd_last_device_status(null, 0x1000, ctypes.byref(v), None) == rpart.FD_EINVAL
    d = rpart.fd_kv_desc(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 2, 4, 128, 0)
    assert lib.fd_last_device_status(ctypes.byref(d), None, ctypes.byref(v), None) == rpart.FD_EINVAL
    assert lib.fd_last_device_status(ctypes.byref(d), 0x1010, ctypes.byref(v), None) == rpart.FD_EINVAL
    assert lib.fd_last_device_status(ctypes.byref(d), 0x1000, None, None) == rpart.FD_EINVAL
    assert lib.fd_kv_store_rows(null, 0, 0, 1, 0x7000, 0x8000, 0, None) == rpart.FD_EINVAL
    for b, t0, n in ((2, 0, 1), (-1, 0, 1), (0, -1, 1), (0, 0, -1), (0, 2 ** 31 - 1, 1)):
        assert lib.fd_kv_store_rows(ctypes.byref(d), b, t0, n, 0x7000, 0x8000, 0, None) == rpart.FD_EINVAL
    assert lib.fd_kv_store_rows(ctypes.byref(d), 0, 0, 1, 0x7001, None, 0, None) == rpart.FD_EINVAL
    assert lib.fd_kv_store_rows(ctypes.byref(d), 0, 5, 0, None, None, 0, None) == rpart.FD_OK   # nothing to do
    q = rpart.fd_kvq_desc(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, 0x8000, 2, 4, 128, 0, None, 0, 8)
    assert lib.fd_kvq_store_rows(ctypes.byref(q), 2, 0, 1, 0x9000, None, 0, None) == rpart.FD_EINVAL
    assert lib.fd_kvq_store_rows(ctypes.byref(q), 0, 0, 0, None, None, 0, None) == rpart.FD_OK
    q.d = 64
    assert lib.fd_kvq_store_rows(ctypes.byref(q), 0, 0, 0, None, None, 0, None) == rpart.FD_OK
    q.d = 96
    assert lib.fd_kvq_store_rows(ctypes.byref(q), 0, 0, 0, None, None, 0, None) == rpart.FD_EINVAL


def test_stale_library_is_detected_by_content(monkeypatch):
    """The library reports the hash of what it was built from; a tree with other sources (here: a
    hash that cannot match) makes it stale, whatever the file times say."""
    from paper_2403_11421_amd import build
    assert build.built_from() == build.source_hash() and not build.is_stale()
    monkeypatch.setattr(build, "source_hash", lambda extra_flags=(): "0" * 64)
    assert build.is_stale()
    monkeypatch.undo()
    assert not build.is_stale() and build.have_compiler()


def test_binding_raises_fd_error():
    with pytest.raises(rpart.FdError) as e:
        rpart._check(rpart.FD_EWORKSPACE, "x")
    assert e.value.code == rpart.FD_EWORKSPACE and "workspace" in str(e.value)
