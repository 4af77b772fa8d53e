"""Device-resident KV-cache of one layer in the layout of ``fd_kv_desc``.

Plumbing only: allocates the K and V slabs and the per-sequence arrays with
torch, fills them from tensors the caller supplies, and exposes the descriptor.
Sequence b owns a ``[H][cap_b][d]`` block at element offset ``seq_off[b]``.
"""
from __future__ import annotations

from typing import Sequence

import torch

from . import rpart


class KVCache:
    def __init__(self, B: int, H: int, d: int, capacities: Sequence[int], device="cuda",
                 chunk_tokens: int = 0):
        assert len(capacities) == B and d in (64, 128)
        self.B, self.H, self.d = B, H, d
        self.device = torch.device(device)
        self.caps = [max(1, int(c)) for c in capacities]
        offs, o = [], 0
        for c in self.caps:
            offs.append(o)
            o += H * c * d
            o = (o + 127) // 128 * 128               # 256-byte aligned blocks
        self.total_elems = max(o, 128)
        self.offs = offs
        self.k = torch.zeros(self.total_elems, dtype=torch.float16, device=self.device)
        self.v = torch.zeros(self.total_elems, dtype=torch.float16, device=self.device)
        self.seq_off = torch.tensor(offs, dtype=torch.int64, device=self.device)
        self.seq_cap = torch.tensor(self.caps, dtype=torch.int32, device=self.device)
        self.seq_lens = torch.zeros(B, dtype=torch.int32, device=self.device)
        self.status = torch.zeros(1, dtype=torch.int32, device=self.device)
        self.desc = rpart.fd_kv_desc(
            self.k.data_ptr(), self.v.data_ptr(), self.seq_off.data_ptr(), self.seq_cap.data_ptr(),
            self.seq_lens.data_ptr(), self.status.data_ptr(), B, H, d, chunk_tokens)

    def set_chunk_tokens(self, t: int) -> None:
        self.desc.chunk_tokens = int(t)

    def block(self, which: str, b: int) -> torch.Tensor:
        """View ``[H, cap_b, d]`` of sequence b's K or V block."""
        slab = self.k if which == "K" else self.v
        n = self.H * self.caps[b] * self.d
        return slab[self.offs[b]: self.offs[b] + n].view(self.H, self.caps[b], self.d)

    def fill(self, which: str, b: int, rows: torch.Tensor, t0: int = 0) -> None:
        """Store fp16 ``rows [H, L, d]`` at tokens t0..t0+L-1 of sequence b (no length change)."""
        L = rows.shape[1]
        self.block(which, b)[:, t0:t0 + L, :].copy_(rows)

    def set_lens(self, lens: Sequence[int]) -> None:
        self.seq_lens.copy_(torch.tensor(list(lens), dtype=torch.int32))

    def workspace(self, max_total_tokens: int) -> torch.Tensor:
        n = rpart.workspace_bytes(self.B, self.H, self.d, max_total_tokens)
        return torch.empty(n, dtype=torch.uint8, device=self.device)
