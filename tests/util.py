"""Helpers shared by the tests: turn seeded workload tensors into the oracle's layout."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from paper_2403_11421_amd import workloads as W


def bits(t: torch.Tensor) -> np.ndarray:
    """fp16 tensor -> uint16 numpy array of its bit patterns (host copy)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()


def f64(b: np.ndarray) -> np.ndarray:
    """uint16 binary16 patterns -> float64 (numpy's decoder)."""
    return b.view(np.float16).astype(np.float64)


def half_bits(x) -> np.ndarray:
    """float array -> binary16 bit patterns (numpy's round-to-nearest-even)."""
    return np.asarray(x, dtype=np.float64).astype(np.float16).view(np.uint16)


class OracleCase:
    """Inputs of one decode step in the oracle's layout.

    K[b], V[b]: uint16 [L_b + 1 + extra, H, d] token-major, rows [0, L_b) filled.
    """

    def __init__(self, cfg: W.RPartConfig, lens: Sequence[int], seed: int = W.DEFAULT_SEED,
                 batch: Optional[Sequence[int]] = None, extra_rows: int = 0):
        self.cfg = cfg
        self.batch = list(range(cfg.B)) if batch is None else list(batch)
        self.lens0 = np.asarray([lens[b] for b in self.batch], dtype=np.int32)
        self.seq_lens = self.lens0.copy()
        self.K: List[np.ndarray] = []
        self.V: List[np.ndarray] = []
        for b, L in zip(self.batch, self.lens0):
            L = int(L)
            for which, dst in (("K", self.K), ("V", self.V)):
                blk = np.zeros((L + 1 + extra_rows, cfg.H, cfg.d), dtype=np.uint16)
                if L:
                    blk[:L] = bits(W.gen_cache_block(cfg, which, b, L, seed).permute(1, 0, 2))
                dst.append(blk)
        self.q = bits(W.gen_vectors(cfg, "q", seed, batch=self.batch))
        self.k_new = bits(W.gen_vectors(cfg, "k_new", seed, batch=self.batch))
        self.v_new = bits(W.gen_vectors(cfg, "v_new", seed, batch=self.batch))

    def max_abs_v(self) -> float:
        m = float(np.abs(f64(self.v_new)).max()) if self.v_new.size else 0.0
        for b, L in enumerate(self.seq_lens):
            if L:
                m = max(m, float(np.abs(f64(self.V[b][:L])).max()))
        return m
