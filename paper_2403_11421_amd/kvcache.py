"""Device-resident KV-cache of one layer in the layout of ``fd_kv_desc`` / ``fd_kvq_desc``.

Plumbing only: allocates the slabs and the per-sequence arrays with torch and exposes the
descriptor.  Rows are written by the library (``fd_kv_store_rows`` / ``fd_kvq_store_rows``, the
same quantiser as the append): no cache arithmetic lives on this side of the C ABI.
Sequence b owns a ``[H][cap_b][d]`` block at element offset ``seq_off[b]``.
"""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import rpart


class KVCache:
    def __init__(self, B: int, H: int, d: int, capacities: Sequence[int], device="cuda",
                 chunk_tokens: int = 0, n_sink: Optional[int] = None, zero_fill: bool = True):
        """n_sink = None: plain cache.  n_sink >= 0: windowed cache, sequence b keeps its first
        n_sink tokens and its last capacities[b] - n_sink tokens.  zero_fill = False leaves the
        slabs as allocated (the caller fills them); the small arrays are then set up by copies
        from the host, so that constructing the cache dispatches no kernel."""
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
        alloc = torch.zeros if zero_fill else torch.empty
        self.k = alloc(self.total_elems, dtype=torch.float16, device=self.device)
        self.v = alloc(self.total_elems, dtype=torch.float16, device=self.device)
        self.seq_off = torch.tensor(offs, dtype=torch.int64).to(self.device)
        self.seq_cap = torch.tensor(self.caps, dtype=torch.int32).to(self.device)
        self.seq_lens = torch.zeros(B, dtype=torch.int32).to(self.device)
        self.status = torch.zeros(1, dtype=torch.int32).to(self.device)
        self.seq_seen = None if n_sink is None else torch.zeros(B, dtype=torch.int32).to(self.device)
        self.desc = rpart.fd_kv_desc(
            self.k.data_ptr(), self.v.data_ptr(), self.seq_off.data_ptr(), self.seq_cap.data_ptr(),
            self.seq_lens.data_ptr(), self.status.data_ptr(), B, H, d, chunk_tokens,
            None if n_sink is None else self.seq_seen.data_ptr(), 0 if n_sink is None else n_sink)

    def set_chunk_tokens(self, t: int) -> None:
        self.desc.chunk_tokens = int(t)

    def slabs(self):
        """The large allocations (for bulk copies or fills)."""
        return [self.k, self.v]

    def block(self, which: str, b: int) -> torch.Tensor:
        """View ``[H, cap_b, d]`` of sequence b's K or V block."""
        slab = self.k if which == "K" else self.v
        n = self.H * self.caps[b] * self.d
        return slab[self.offs[b]: self.offs[b] + n].view(self.H, self.caps[b], self.d)

    def fill(self, which: str, b: int, rows: torch.Tensor, t0: int = 0) -> None:
        """Store fp16 ``rows [H, L, d]`` at tokens t0..t0+L-1 of sequence b (no length change)."""
        rows = rows.to(device=self.device, dtype=torch.float16).contiguous()
        assert rows.shape[0] == self.H and rows.shape[2] == self.d and t0 + rows.shape[1] <= self.caps[b]
        rpart.fd_kv_store_rows(self.desc, b, t0, rows if which == "K" else None,
                               rows if which == "V" else None)

    def set_lens(self, lens: Sequence[int]) -> None:
        """Cached tokens per sequence; a windowed cache is told the tokens seen so far, which
        must not exceed the capacity here (rows 0..L-1 hold tokens 0..L-1)."""
        t = torch.tensor(list(lens), dtype=torch.int32)
        self.seq_lens.copy_(t)
        if self.seq_seen is not None:
            assert all(L <= c for L, c in zip(lens, self.caps))
            self.seq_seen.copy_(t)

    def workspace(self, max_total_tokens: int) -> torch.Tensor:
        n = rpart.workspace_bytes(self.B, self.H, self.d, max_total_tokens)
        return torch.empty(n, dtype=torch.uint8, device=self.device)


class KVCacheQ:
    """Quantised KV-cache of one layer in the layout of ``fd_kvq_desc`` (d = 128 or 64, 8 or 4 bits)."""

    def __init__(self, B: int, H: int, d: int, capacities: Sequence[int], device="cuda",
                 chunk_tokens: int = 0, n_sink: Optional[int] = None, bits: int = 8,
                 zero_fill: bool = True):
        assert len(capacities) == B and d in (64, 128) and bits in (8, 4)
        self.B, self.H, self.d, self.bits = B, H, d, bits
        self.rb = d * bits // 8                         # bytes of codes per row
        self.mw = 1 if bits == 8 else 2                 # floats of parameters per row
        self.device = torch.device(device)
        self.caps = [max(1, int(c)) for c in capacities]
        # rows a head occupies in its sequence's block: 4-bit rows lie in pairs, so their count
        # is padded to even (the library's head_rows)
        self.rows = [c if bits == 8 else (c + 1) & ~1 for c in self.caps]
        offs, o = [], 0
        for r in self.rows:
            offs.append(o)
            o += H * r * self.rb                        # bytes of codes
            o = (o + 255) // 256 * 256
        self.offs = offs
        self.total_bytes = max(o, 256)
        fill = 128 if bits == 8 else 0
        n_meta = self.total_bytes // self.rb * self.mw
        if zero_fill:
            self.k_codes = torch.full((self.total_bytes,), fill, dtype=torch.uint8, device=self.device)
            self.v_codes = torch.full((self.total_bytes,), fill, dtype=torch.uint8, device=self.device)
            self.k_scale = torch.zeros(n_meta, dtype=torch.float32, device=self.device)
            self.v_scale = torch.zeros(n_meta, dtype=torch.float32, device=self.device)
        else:
            self.k_codes = torch.empty(self.total_bytes, dtype=torch.uint8, device=self.device)
            self.v_codes = torch.empty(self.total_bytes, dtype=torch.uint8, device=self.device)
            self.k_scale = torch.empty(n_meta, dtype=torch.float32, device=self.device)
            self.v_scale = torch.empty(n_meta, dtype=torch.float32, device=self.device)
        self.seq_off = torch.tensor(offs, dtype=torch.int64).to(self.device)
        self.seq_cap = torch.tensor(self.caps, dtype=torch.int32).to(self.device)
        self.seq_lens = torch.zeros(B, dtype=torch.int32).to(self.device)
        self.status = torch.zeros(1, dtype=torch.int32).to(self.device)
        self.seq_seen = None if n_sink is None else torch.zeros(B, dtype=torch.int32).to(self.device)
        self.desc = rpart.fd_kvq_desc(
            self.k_codes.data_ptr(), self.v_codes.data_ptr(), self.k_scale.data_ptr(),
            self.v_scale.data_ptr(), self.seq_off.data_ptr(), self.seq_cap.data_ptr(),
            self.seq_lens.data_ptr(), self.status.data_ptr(), B, H, d, chunk_tokens,
            None if n_sink is None else self.seq_seen.data_ptr(), 0 if n_sink is None else n_sink,
            bits)

    def slabs(self):
        """The large allocations (for bulk copies or fills)."""
        return [self.k_codes, self.v_codes, self.k_scale, self.v_scale]

    def codes(self, which: str, b: int) -> torch.Tensor:
        """``[H, cap_b, rb]`` (uint8): sequence b's K or V code bytes, row by row.  8 bit: a view of
        the slab.  4 bit: a copy, taken out of the paired layout (rows 2p and 2p+1 of a head
        alternate in 8-byte pieces)."""
        slab = self.k_codes if which == "K" else self.v_codes
        rows = self.rows[b]
        blk = slab[self.offs[b]: self.offs[b] + self.H * rows * self.rb]
        if self.bits == 8:
            return blk.view(self.H, rows, self.rb)
        pieces = self.rb // 8
        v = blk.view(self.H, rows // 2, pieces, 2, 8).permute(0, 1, 3, 2, 4)
        return v.reshape(self.H, rows, self.rb)[:, : self.caps[b]]

    def scales(self, which: str, b: int) -> torch.Tensor:
        """View ``[H, cap_b]`` (8 bit: scale) or ``[H, cap_b, 2]`` (4 bit: scale, zero), float32."""
        slab = self.k_scale if which == "K" else self.v_scale
        o = self.offs[b] // self.rb * self.mw
        rows = self.rows[b]
        v = slab[o: o + self.H * rows * self.mw]
        return v.view(self.H, rows) if self.mw == 1 else v.view(self.H, rows, 2)[:, : self.caps[b]]

    def fill(self, which: str, b: int, rows: torch.Tensor, t0: int = 0) -> None:
        """Quantise fp16 ``rows [H, L, d]`` into tokens t0..t0+L-1 of sequence b (the library's
        quantiser, the same as the append's; no length change)."""
        rows = rows.to(device=self.device, dtype=torch.float16).contiguous()
        assert rows.shape[0] == self.H and rows.shape[2] == self.d and t0 + rows.shape[1] <= self.caps[b]
        rpart.fd_kv_store_rows(self.desc, b, t0, rows if which == "K" else None,
                               rows if which == "V" else None)

    def set_lens(self, lens: Sequence[int]) -> None:
        """Cached tokens per sequence; a windowed cache is told the tokens seen so far, which
        must not exceed the capacity here (rows 0..L-1 hold tokens 0..L-1)."""
        t = torch.tensor(list(lens), dtype=torch.int32)
        self.seq_lens.copy_(t)
        if self.seq_seen is not None:
            assert all(L <= c for L, c in zip(lens, self.caps))
            self.seq_seen.copy_(t)

    def workspace(self, max_total_tokens: int) -> torch.Tensor:
        n = rpart.workspace_bytes(self.B, self.H, self.d, max_total_tokens)
        return torch.empty(n, dtype=torch.uint8, device=self.device)
