"""Brute-force reference for the sequence-level load-stabilising schedule (FastDecode Section 4.2).

TEST INFRASTRUCTURE ONLY.  Everything here is a literal simulation: every sequence is an object
with a start step, and a step's load is the sum of the lengths of the sequences alive at that
step.  It shares no code with the library's scheduler.

Conventions (fixed by the worked example of Figure 7): a sequence started at step t has length
s - t + 1 at step s and lives for S steps (s = t .. t+S-1), so its last step carries length S.

Pins (tests/test_sched.py): `step_loads` against the arrays and peaks printed with Figure 7 and
against Eq. 6's closed form; `earliest_start_brute_force` against cases worked by hand from the
figure's example (tests/golden/alg1_earliest_start.txt); the Section 4.3 functions against
hand-worked numbers and the simulated schedule's mean load.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def step_loads(starts: Sequence[Tuple[int, int]], S: int, n_steps: int) -> List[int]:
    """Total cached length per step for micro-batches given as (start step, size)."""
    loads = [0] * n_steps
    for t0, m in starts:
        for _ in range(m):                       # one sequence at a time, on purpose
            for s in range(max(t0, 0), min(t0 + S, n_steps)):
                loads[s] += s - t0 + 1
    return loads


def large_batch_starts(B: int, S: int, n_steps: int) -> List[Tuple[int, int]]:
    """All B sequences start together, the next batch when they finish."""
    return [(t, B) for t in range(0, n_steps, S)]


def sls_starts(M: int, F: int, n_steps: int) -> List[Tuple[int, int]]:
    """A micro-batch of M sequences every F steps."""
    return [(t, M) for t in range(0, n_steps, F)]


def earliest_start_brute_force(existing: Sequence[Tuple[int, int]], S: int, W_lim: int,
                               t: int, m: int, horizon: int) -> int:
    """Smallest start step >= t for a new micro-batch of m sequences such that the load at the
    last step of every existing micro-batch stays <= W_lim (the quantity Algorithm 1 guards)."""
    for cand in range(t, horizon):
        ok = True
        allmb = list(existing) + [(cand, m)]
        for t0, _ in existing:
            last = t0 + S - 1
            if last < cand:
                continue
            load = sum(mm * (last - tt + 1) for tt, mm in allmb if tt <= last < tt + S)
            if load > W_lim:
                ok = False
                break
        if ok:
            return cand
    return horizon


# ---------------------------------------------------------------------------
# Section 4.3, written out with exact rationals
# ---------------------------------------------------------------------------
def model_sequence_latency(N, S, T_B):
    """Eq. 7, left side: S tokens, N blocks per token, an S-Part and an equally long R-Part each."""
    from fractions import Fraction
    total = Fraction(0)
    for _token in range(S):
        for _block in range(N):
            total += Fraction(T_B) + Fraction(T_B)
    return total


def model_num_rworkers(B, S, R, T_B):
    """Eq. 10 solved for P: B sequences of mean length S/2 spread over P workers take
    (B*S/2/P)*R per block, which is to equal T_B."""
    from fractions import Fraction
    return Fraction(B) * Fraction(S) / 2 * Fraction(R) / Fraction(T_B)


def model_min_rworkers_memory(B, S, C):
    """Eq. 9: smallest integer P with B*S/2 <= C*P, by search."""
    P = 1
    while 2 * C * P < B * S:
        P += 1
    return P
