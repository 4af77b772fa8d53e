"""Window attention with sink tokens, and the bounded cache that serves it (the variation of
attention that FastDecode's Related Work names as reducing the R-Part's workload: each new token
interacts with fewer cached tokens).

TEST INFRASTRUCTURE ONLY.  Written from the definition, on the full token history:

  * the token set of a sequence that has seen L tokens is
        S(L) = { t : t < n_sink }  united with  { t : t >= L - window },   0 <= t < L;
    attention (Eq. 2 + Eq. 3) runs over exactly the rows of S(L);
  * a cache of n_sink + window rows serves it: while it has free rows a new token takes the
    next one; once full, the new token replaces the OLDEST token that is not a sink.  Attention
    does not depend on the order of the rows, so the rows need not be kept in token order.

The cache side is simulated literally (a list of which token each row holds, eviction by
search for the oldest), not by index arithmetic.  parity pinned: see tests/test_oracle_window_pins.py.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import rpart_oracle as O


def token_set(L: int, n_sink: int, window: int) -> List[int]:
    return [t for t in range(L) if t < n_sink or t >= L - window]


def rpart_decode_window(K_hist: Sequence[np.ndarray], V_hist: Sequence[np.ndarray],
                        seen: Sequence[int], q: np.ndarray, n_sink: int, window: int):
    """K_hist[b], V_hist[b]: uint16 [>= seen[b], H, d], row t = token t (the whole history).
    Returns the fp64 attention output [B, H, d] over S(seen[b]) for every sequence."""
    Ks, Vs, lens = [], [], []
    for Kb, Vb, L in zip(K_hist, V_hist, seen):
        S = token_set(int(L), n_sink, window)
        Ks.append(np.ascontiguousarray(Kb[S]) if S else np.zeros((1,) + Kb.shape[1:], np.uint16))
        Vs.append(np.ascontiguousarray(Vb[S]) if S else np.zeros((1,) + Vb.shape[1:], np.uint16))
        lens.append(len(S))
    out, _, _ = O.rpart_decode(Ks, Vs, np.asarray(lens, np.int32), q)
    return out


class BoundedCache:
    """Which token each cache row holds, by literal simulation of "replace the oldest non-sink"."""

    def __init__(self, n_sink: int, window: int):
        self.n_sink, self.cap = n_sink, n_sink + window
        self.rows: List[int] = []          # rows[r] = token held by row r
        self.seen = 0

    def append(self) -> int:
        """A new token arrives; returns the row it is stored in."""
        t = self.seen
        self.seen += 1
        if len(self.rows) < self.cap:
            self.rows.append(t)
            return len(self.rows) - 1
        victims = [(tok, r) for r, tok in enumerate(self.rows) if tok >= self.n_sink]
        _, r = min(victims)
        self.rows[r] = t
        return r
