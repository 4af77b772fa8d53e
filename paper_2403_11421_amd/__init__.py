"""MI355X-native R-Part (decode-step attention over the KV-cache) of FastDecode.

The R-Part is the per-sequence, parameter-free half of a decoder block
(FastDecode Section 3.1, Eq. 2 and Eq. 3): append the new token's K/V to the
sequence's cache, then attend its query over the whole cache.

Sub-modules
-----------
workloads : seeded synthetic inputs shaped like the paper's decode workloads
            (holds none of the method's arithmetic).
rpart     : ctypes binding over the C-ABI library built from ``csrc/``.
sched     : ctypes binding over the host scheduler (Section 4.2, 4.3) in the same library.
kvcache   : device-resident KV-cache slabs (fp16, 8-bit, 4-bit; plain or windowed) and their descriptors.
sls_run   : multi-step decode loop under the schedules of Section 4.2.
pipeline  : R-worker for N blocks and two mini-batches on two streams (Section 4.1).
build     : compiles the library in-tree with hipcc for gfx950.

Nothing is imported eagerly so that the workload generators can be used
without the HIP library being present.
"""

__all__ = ["workloads", "rpart", "sched", "kvcache", "sls_run", "pipeline", "build"]
__version__ = "0.1.0"
