"""Build the C-ABI library ``libfd_rpart.so`` for gfx950 with hipcc (in-tree)."""
from __future__ import annotations

import os
import subprocess
import sys

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SOURCES = [os.path.join(_PKG, "csrc", "fd_rpart.hip"), os.path.join(_PKG, "csrc", "fd_sched.cpp")]
INCLUDE = os.path.join(_ROOT, "include")
LIB = os.path.join(_PKG, "libfd_rpart.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # hipcc -O3 must not form packed-fp32 instructions in these kernels
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


DEPS = SOURCES + [os.path.join(_PKG, "csrc", "fd_rpartq.h"), os.path.join(INCLUDE, "fastdecode_rpart.h"),
                  os.path.join(INCLUDE, "fastdecode_sched.h")]


def source_hash(extra_flags=()) -> str:
    """sha256 over the sources, the headers they include and the compiler flags."""
    import hashlib
    h = hashlib.sha256(" ".join(HIPCC_FLAGS + list(extra_flags)).encode())
    for p in DEPS:
        with open(p, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source into the shared library; always recompiles.  The library carries
    the hash of what it was built from (fd_build_id)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = ([hipcc] + HIPCC_FLAGS + list(extra_flags) + [f'-DFD_BUILD_ID="{source_hash(extra_flags)}"', "-I", INCLUDE,
                                                        "-o", LIB] + SOURCES)
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def built_from():
    """The build id the library on disk reports, or None if there is none to ask."""
    import ctypes
    try:
        f = ctypes.CDLL(LIB).fd_build_id
    except (OSError, AttributeError):
        return None
    f.restype = ctypes.c_char_p
    f.argtypes = []
    return f().decode()


def have_compiler() -> bool:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return os.path.isfile(hipcc) and os.access(hipcc, os.X_OK)


def is_stale() -> bool:
    """True when the library is missing or was built from other sources than the tree holds now
    (by content, not by file time: a copied tree keeps no reliable times)."""
    return not os.path.exists(LIB) or built_from() != source_hash()


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
