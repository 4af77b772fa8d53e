"""Multi-step R-worker loop driven by the schedules of FastDecode Section 4.2.

Plays the role of the S-worker for one layer: every step it hands the R-Part one new (q, k, v)
per live sequence, starts micro-batches (dropping the finished sequences' caches first) as the
schedule dictates, and records the time of each ``fd_rpart_step``.  Used by ``bench.py
--schedule`` and by the multi-step parity test.  Plumbing only: all attention work is in the
library's kernels, all schedule arithmetic in its host scheduler (``sched``).
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional

import torch

from . import rpart, sched, workloads as W
from .kvcache import KVCache, KVCacheQ


def _make_cache(kv: str, B: int, H: int, d: int, S: int, dev):
    """A cache of B slots of S rows in the given format and the step / reset calls that go with it."""
    assert kv in ("fp16", "int8", "int4")
    if kv == "fp16":
        return KVCache(B, H, d, [S] * B, dev), rpart.fd_rpart_step, rpart.fd_kv_reset
    return (KVCacheQ(B, H, d, [S] * B, dev, bits=4 if kv == "int4" else 8),
            rpart.fd_rpartq_step, rpart.fd_kvq_reset)


def step_vectors(cfg: W.RPartConfig, which: str, step: int, seed: int, device) -> torch.Tensor:
    """fp16 [B, H, d] vectors of one step (the counter's token field carries the step index)."""
    tid = {"q": W.TID_Q, "k_new": W.TID_KNEW, "v_new": W.TID_VNEW}[which]
    b = torch.arange(cfg.B, dtype=torch.int64, device=device).view(-1, 1, 1)
    h = torch.arange(cfg.H, dtype=torch.int64, device=device).view(1, cfg.H, 1)
    i = torch.arange(cfg.d, dtype=torch.int64, device=device).view(1, 1, cfg.d)
    return (W.normal_from_counter(seed, tid, W._counter(b, step % 16384, h, i)) * cfg.scale).to(torch.float16)


def controlled_starts(B: int, S: int, M: int, F: int, W_lim: int, n_steps: int) -> List[int]:
    """Start steps of micro-batches of M sequences under Algorithm 1's load control: the
    library's admission loop (`fd_lc_controlled_starts`)."""
    return sched.controlled_starts(B, S, M, F, W_lim, n_steps)


def run_schedule(kind: str, B: int, S: int, F: int, n_steps: int, H: int = 32, d: int = 128,
                 seed: int = W.DEFAULT_SEED, device="cuda", timed: bool = True,
                 on_step: Optional[Callable] = None, W_lim: Optional[int] = None,
                 kv: str = "fp16") -> Dict:
    """kind = "sls": micro-batches of M = B*F/S sequences every F steps (Eq. 5);
    kind = "batch": all B sequences together, the next batch when they finish;
    kind = "control": micro-batches of M = B*F/S sequences admitted by Algorithm 1 under the
    load limit W_lim (default: Eq. 6's peak), see `run_controlled`.

    Sequence slots are reused round-robin; a micro-batch's slots are reset when it starts.
    During the cold start only the slots started so far take part (a prefix of the slots).
    on_step(step, cache, q, k_new, v_new, out, n_active) is called after each step (tests).
    kv = "fp16", "int8" or "int4" chooses the cache format (Section 5.2)."""
    if kind == "control":
        return run_controlled(B, S, F, n_steps, H, d, seed, device, timed, on_step, W_lim, kv)
    assert kind in ("sls", "batch")
    cfg = W.RPartConfig(f"{kind}_B{B}_S{S}_F{F}", B, H, d, "const", 0, 0)
    M = sched.sls_microbatch_size(B, F, S) if kind == "sls" else B
    period = F if kind == "sls" else S
    n_groups = B // M                                   # micro-batches in flight at steady state
    assert n_groups * M == B and (kind == "batch" or n_groups * F >= S), "B*F must cover S"
    loads = (sched.sls_step_loads(M, F, S, n_steps) if kind == "sls"
             else sched.batch_step_loads(B, S, n_steps))

    dev = torch.device(device)
    cache, step_fn, reset_fn = _make_cache(kv, B, H, d, S, dev)
    out = torch.zeros(B, H, d, dtype=torch.float16, device=dev)
    ws = cache.workspace(B * S)
    group_ids = [torch.arange(g * M, (g + 1) * M, dtype=torch.int32, device=dev) for g in range(n_groups)]
    events: List = []
    started = 0
    for step in range(n_steps):
        if step % period == 0:                          # a micro-batch starts: recycle its slots
            g = (step // period) % n_groups
            reset_fn(cache.desc, group_ids[g])
            started = min(n_groups, started + 1)
        n_active = started * M
        cache.desc.B = n_active                         # cold start: only a prefix of the slots is live
        q = step_vectors(cfg, "q", step, seed, dev)
        k_new = step_vectors(cfg, "k_new", step, seed, dev)
        v_new = step_vectors(cfg, "v_new", step, seed, dev)
        if timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        step_fn(cache.desc, q, k_new, v_new, out, ws)
        if timed:
            e1.record()
            events.append((e0, e1))
        if on_step is not None:
            torch.cuda.synchronize()
            on_step(step, cache, q, k_new, v_new, out, n_active)
    torch.cuda.synchronize()
    cache.desc.B = B
    assert rpart.fd_read_status(cache.desc) == 0
    ms = [a.elapsed_time(b) for a, b in events]
    return {"kind": kind, "kv": kv, "B": B, "S": S, "F": F, "M": M, "H": H, "d": d, "steps": n_steps,
            "loads": loads, "ms": ms, "final_lens": cache.seq_lens.cpu().tolist()}


def run_controlled(B: int, S: int, F: int, n_steps: int, H: int = 32, d: int = 128,
                   seed: int = W.DEFAULT_SEED, device="cuda", timed: bool = True,
                   on_step: Optional[Callable] = None, W_lim: Optional[int] = None,
                   kv: str = "fp16") -> Dict:
    """Decode loop whose micro-batches are admitted by Algorithm 1.  Slots of finished sequences
    are released (free slots cost nothing) and reused by the next micro-batch.
    on_step(step, cache, q, k_new, v_new, out, live_slots) is called after each step (tests)."""
    cfg = W.RPartConfig(f"control_B{B}_S{S}_F{F}", B, H, d, "const", 0, 0)
    M = sched.sls_microbatch_size(B, F, S)
    if W_lim is None:                                   # Eq. 6's peak: nothing is held back
        W_lim = sched.sls_peak_load(M, F, S)
    starts = controlled_starts(B, S, M, F, W_lim, n_steps)
    dev = torch.device(device)
    cache, step_fn, reset_fn = _make_cache(kv, B, H, d, S, dev)
    out = torch.zeros(B, H, d, dtype=torch.float16, device=dev)
    ws = cache.workspace(B * S)
    n_groups = B // M
    group_ids = [torch.arange(g * M, (g + 1) * M, dtype=torch.int32, device=dev) for g in range(n_groups)]
    rpart.fd_kv_release(cache.desc)                     # every slot starts free
    busy_until = [0] * n_groups                         # group g holds a micro-batch until this step
    live: List[int] = []
    loads, events = [], []
    nxt = 0
    for step in range(n_steps):
        for g in range(n_groups):                       # finished micro-batches free their slots
            if busy_until[g] == step and step > 0:
                rpart.fd_kv_release(cache.desc, group_ids[g])
                live = [s for s in live if not (g * M <= s < (g + 1) * M)]
        if nxt < len(starts) and starts[nxt] == step:
            g = min(range(n_groups), key=lambda i: busy_until[i])
            assert busy_until[g] <= step
            reset_fn(cache.desc, group_ids[g])
            busy_until[g] = step + S
            live += list(range(g * M, (g + 1) * M))
            nxt += 1
        q = step_vectors(cfg, "q", step, seed, dev)
        k_new = step_vectors(cfg, "k_new", step, seed, dev)
        v_new = step_vectors(cfg, "v_new", step, seed, dev)
        if timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        step_fn(cache.desc, q, k_new, v_new, out, ws)
        if timed:
            e1.record()
            events.append((e0, e1))
        loads.append(sum(step - s0 + 1 for s0 in starts[:nxt] if s0 <= step < s0 + S) * M)
        if on_step is not None:
            torch.cuda.synchronize()
            on_step(step, cache, q, k_new, v_new, out, sorted(live))
    torch.cuda.synchronize()
    assert rpart.fd_read_status(cache.desc) == 0
    ms = [a.elapsed_time(b) for a, b in events]
    return {"kind": "control", "kv": kv, "B": B, "S": S, "F": F, "M": M, "H": H, "d": d, "steps": n_steps,
            "W_lim": W_lim, "starts": starts, "loads": loads, "ms": ms,
            "final_lens": cache.seq_lens.cpu().tolist()}
