"""MI355X-native R-Part (decode-step attention over the KV-cache) of FastDecode.

The R-Part is the per-sequence, parameter-free half of a decoder block
(FastDecode Section 3.1, Eq. 2 and Eq. 3): append the new token's K/V to the
sequence's cache, then attend its query over the whole cache.

Sub-modules
-----------
workloads : seeded synthetic inputs shaped like the paper's decode workloads
            (holds none of the method's arithmetic).
rpart     : ctypes binding over the C-ABI library built from ``csrc/``.
kvcache   : device-resident KV-cache slabs and their descriptor.

Nothing is imported eagerly so that the workload generators can be used
without the HIP library being present.
"""

__all__ = ["workloads", "rpart", "kvcache"]
__version__ = "0.1.0"
