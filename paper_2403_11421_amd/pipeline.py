"""R-worker for a model of N transformer blocks and two mini-batches (FastDecode Section 4.1).

The S-worker sends, block by block, the Q, K, V vectors of mini-batch A and of mini-batch B in
turns; the R-worker appends and attends against that block's cache and returns O.  Here both
mini-batches' caches live on one device and each mini-batch has its own HIP stream and its own
workspace, so the small kernels of one mini-batch's block (append, plan, merge) run under the
streaming kernel of the other.  The streams are left free to overlap the two streaming kernels
as well: holding the second one back with an event until the first has finished was measured
slower than either alternative (the cross-stream wait costs more than the overlap gains).  All blocks of a mini-batch share one ragged plan per token
step (``fd_rpart_layer_step`` with ``replan`` only for block 0).

Plumbing only: which call goes to which stream.  All arithmetic is in the library's kernels.
"""
from __future__ import annotations

from typing import List, Sequence

import torch

from . import rpart
from .kvcache import KVCache, KVCacheQ


class RWorker:
    def __init__(self, H: int, d: int, n_layers: int, capacities: Sequence[Sequence[int]],
                 kv: str = "fp16", n_streams: int = 2, device="cuda", chunk_tokens: int = 0):
        """capacities[m][b]: token capacity of sequence b of mini-batch m (m = 0, 1, ...)."""
        assert kv in ("fp16", "int8", "int4") and n_streams in (1, 2) and n_layers >= 1
        self.H, self.d, self.n_layers, self.kv = H, d, n_layers, kv
        self.device = torch.device(device)
        self.n_mb = len(capacities)

        def cache(caps):
            if kv == "fp16":
                return KVCache(len(caps), H, d, caps, self.device, chunk_tokens)
            return KVCacheQ(len(caps), H, d, caps, self.device, chunk_tokens, bits=4 if kv == "int4" else 8)

        self.caches: List[List] = [[cache(caps) for _ in range(n_layers)] for caps in capacities]
        self.ws = [self.caches[m][0].workspace(sum(capacities[m])) for m in range(self.n_mb)]
        self._own = [torch.cuda.Stream(self.device) for _ in range(self.n_mb)]   # default priority
        self.use_streams(n_streams)

    def use_streams(self, n_streams: int) -> None:
        """2: each mini-batch on its own stream; 1: the mini-batches alternate on the caller's."""
        assert n_streams in (1, 2)
        self.n_streams = n_streams
        self.streams = self._own if n_streams == 2 else \
            [torch.cuda.current_stream(self.device)] * self.n_mb

    def set_lens(self, m: int, lens: Sequence[int]) -> None:
        for c in self.caches[m]:
            c.set_lens(lens)

    def begin_token(self) -> None:
        """Inputs produced on the caller's stream become visible to the mini-batch streams."""
        cur = torch.cuda.current_stream(self.device)
        for s in self.streams:
            if s != cur:
                s.wait_stream(cur)

    def block_step(self, m: int, layer: int, q, k_new, v_new, out, replan=None) -> None:
        """Enqueue block `layer` of mini-batch `m`: append k_new/v_new, attend with q, write out."""
        with torch.cuda.stream(self.streams[m]):
            rpart.fd_rpart_layer_step(self.caches[m][layer].desc, q, k_new, v_new, out, self.ws[m],
                                      layer == 0 if replan is None else replan)

    def end_token(self) -> None:
        """The caller's stream waits for both mini-batches."""
        cur = torch.cuda.current_stream(self.device)
        for s in self.streams:
            if s != cur:
                cur.wait_stream(s)

    def token_step(self, q, k_new, v_new, out) -> None:
        """One generated token for every sequence of every mini-batch.  q[m][layer] etc. are
        device fp16 [B_m, H, d] tensors; blocks are issued A0, B0, A1, B1, ... as in the
        token-level pipeline."""
        self.begin_token()
        for layer in range(self.n_layers):
            for m in range(self.n_mb):
                self.block_step(m, layer, q[m][layer], k_new[m][layer], v_new[m][layer], out[m][layer])
        self.end_token()

    def status(self) -> int:
        st = 0
        for m in range(self.n_mb):
            for c in self.caches[m]:
                st |= rpart.fd_read_status(c.desc)
        return st
