#!/usr/bin/env python3
"""Throughput of the R-Part decode step on one MI355X.

A step is one pass of the whole hot path over one batch: restore the cached
lengths, append the new k/v rows and plan the ragged split (one launch), stream
K/V (split-K attention with the log-sum-exp merge folded in; the second launch).
Inputs are synthetic, seeded, resident in HBM before the timed region starts.
Prints ONE JSON line: the headline fields are config 2 with the fp16 cache (or
whatever --config / --kv name); unless --extras none, the same line carries the
other configs and cache formats, the schedule loop and the N-block pipeline
under "extras".

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c2_7b_uniform]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "R-Part decode attention: achieved KV HBM GB/s (% of peak) and sequences/sec"
HBM_PEAK_GBPS = 8000.0
EXTRA_WARM_MS = 50.0          # untimed steps before each entry under extras (see measure_step)
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "rpart_partial_hbm_traffic.json")
TRAFFIC_JSON_Q = os.path.join(ROOT, "profiles", "rpartq_partial_hbm_traffic.json")
KERNEL_SRC = os.path.join(ROOT, "paper_2403_11421_amd", "csrc", "fd_rpart.hip")
KERNEL_SRC_Q = os.path.join(ROOT, "paper_2403_11421_amd", "csrc", "fd_rpartq.h")


def kernel_fingerprint(quantised=False):
    """sha256 of the kernels' source with comments and white space removed: it changes when the
    code does, not when a comment is reworded.  The quantised kernels include the fp16 file's
    planner and helpers, so their fingerprint covers both files."""
    import hashlib
    import re
    src = open(KERNEL_SRC, encoding="utf-8").read()
    if quantised:
        src += open(KERNEL_SRC_Q, encoding="utf-8").read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    src = re.sub(r"//[^\n]*", "", src)
    return hashlib.sha256(re.sub(r"\s+", "", src).encode()).hexdigest()


def counter_traffic(config_name, kv="fp16"):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc, or None
    when no counters were taken for this config and cache format or the kernel code changed since."""
    try:
        quantised = kv != "fp16"
        rec = json.load(open(TRAFFIC_JSON_Q if quantised else TRAFFIC_JSON))
        if rec.get("code_sha256") != kernel_fingerprint(quantised):
            return None
        node = rec["configs"][config_name]
        return (node[kv] if quantised else node)["traffic_bytes"]
    except (OSError, KeyError, ValueError):
        return None


def kv_bytes_per_token(cfg, kv):
    """Algorithmic bytes per cached token: K row + V row over all heads (quantised rows: the code
    bytes plus the row's float32 parameters, one scale for 8 bit, scale and zero for 4 bit)."""
    if kv == "fp16":
        return cfg.bytes_per_token()
    return 2 * cfg.H * (cfg.d + 4) if kv == "int8" else 2 * cfg.H * (cfg.d // 2 + 8)


def build_case(cfg, lens, seed, chunk_tokens, growth=8, kv="fp16", window=0, sinks=0, capacity=0,
               fill="values"):
    """window > 0: a windowed cache of sinks + window rows per sequence that has already seen
    lens[b] tokens (its rows hold that many, or all of them when the history is longer).
    capacity > 0: every sequence gets a block of that many rows (equal slots, as a slot allocator
    hands them out) instead of one fitted to its length.
    fill = "values": the seeded generator's rows (torch kernels on the device) go through the
    library's bulk store.  fill = "pattern": no torch kernel is dispatched at all, the slabs are
    filled by the library's pattern kernel and the step vectors come from the host (for runs
    under rocprofv3's counter collection, which has crashed inside torch's kernel dispatches;
    HBM traffic does not depend on the values)."""
    import torch
    from paper_2403_11421_amd import rpart, workloads as W
    from paper_2403_11421_amd.kvcache import KVCache, KVCacheQ

    dev = torch.device("cuda:0")
    kw = {} if kv == "fp16" else {"bits": 4 if kv == "int4" else 8}
    if fill == "pattern":
        kw["zero_fill"] = False
    cls = KVCache if kv == "fp16" else KVCacheQ
    if window > 0:
        cache = cls(cfg.B, cfg.H, cfg.d, [sinks + window] * cfg.B, dev, chunk_tokens, n_sink=sinks, **kw)
        held = [min(L, sinks + window) for L in lens]
    else:
        caps = [capacity] * cfg.B if capacity > 0 else [L + growth for L in lens]
        assert all(c > L for c, L in zip(caps, lens)), "capacity must exceed every cached length"
        cache = cls(cfg.B, cfg.H, cfg.d, caps, dev, chunk_tokens, **kw)
        held = lens
    if fill == "pattern":
        for slab in cache.slabs():
            rpart.fd_fill_pattern(slab, seed)
        vec = {w: W.gen_vectors(cfg, w, seed, "cpu").to(dev) for w in ("q", "k_new", "v_new")}
    else:
        for b, L in enumerate(held):
            if L:
                cache.fill("K", b, W.gen_cache_block(cfg, "K", b, L, seed, dev))
                cache.fill("V", b, W.gen_cache_block(cfg, "V", b, L, seed, dev))
        vec = {w: W.gen_vectors(cfg, w, seed, dev) for w in ("q", "k_new", "v_new")}
    cache.set_lens(held)
    if window > 0:
        cache.seq_seen.copy_(torch.tensor(list(lens), dtype=torch.int32))
    return cache, vec


def cpu_baseline(cfg, cache, vec, lens_after, n_sample):
    """Time the fp64 oracle (as it stands) on a sample of this workload's sequences."""
    import numpy as np
    import torch
    from oracle import rpart_oracle as O

    threads = max(1, min(16, os.cpu_count() or 1))
    n_sample = min(n_sample, cfg.B)
    step = max(1, cfg.B // n_sample)
    batch = list(range(0, cfg.B, step))[:n_sample]

    def host(t):
        return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()

    K = [host(cache.block("K", b).permute(1, 0, 2)) for b in batch]
    V = [host(cache.block("V", b).permute(1, 0, 2)) for b in batch]
    hl = np.asarray([lens_after[b] for b in batch], dtype=np.int32)
    q = host(vec["q"][torch.tensor(batch, device=vec["q"].device)])
    t0 = time.perf_counter()
    O.rpart_decode(K, V, hl, q, nthreads=threads)
    dt = time.perf_counter() - t0
    kv_bytes = cfg.bytes_per_token() * int(hl.sum())
    return {
        "value": kv_bytes / dt / 1e9, "unit": "GB/s", "cores": min(threads, len(batch)),
        "kind": "oracle",
        "sample": f"{len(batch)} of {cfg.B} sequences (a stride of {step}), all {cfg.H} heads, "
                  f"{int(hl.sum())} cached tokens, decode only, {dt:.2f} s wall",
        "seq_per_s": len(batch) / dt, "cpu_model": _cpu_model(),
    }


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo", encoding="utf-8", errors="replace"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def softmax_entropy(cfg, cache, vec, lens_after, n_sample=4):
    """How peaked the attention of a config with per-head key spread really is: mean entropy (bits)
    of softmax(q K^T / sqrt d) per spread class (head h has spread {1, 2, 4, 8}[h % 4]) over a few
    sample sequences, next to log2 of their mean length (the entropy of uniform weights).
    Plain torch on the cached fp16 rows; a description of the input, not part of the path."""
    import math
    import torch
    ent = torch.zeros(4, dtype=torch.float64)
    cnt = torch.zeros(4, dtype=torch.float64)
    picks = list(range(0, cfg.B, max(1, cfg.B // n_sample)))[:n_sample]
    for b in picks:
        L = lens_after[b]
        K = cache.block("K", b)[:, :L, :].float()                   # [H, L, d]
        s = torch.einsum("hld,hd->hl", K, vec["q"][b].float()) / math.sqrt(cfg.d)
        logp = torch.log_softmax(s.double(), dim=1)
        e = -(logp.exp() * logp).sum(dim=1) / math.log(2.0)          # [H] bits
        for c in range(4):
            sel = e[c::4]
            ent[c] += float(sel.sum())
            cnt[c] += sel.numel()
    mean_len = sum(lens_after[b] for b in picks) / len(picks)
    return {"bits_by_spread_1_2_4_8": [float(x) for x in (ent / cnt)],
            "uniform_bits_at_mean_length": math.log2(mean_len), "sequences": picks}


def _pct(sorted_vals, p):
    """p-th percentile (nearest rank) of an ascending list."""
    if not sorted_vals:
        return None
    k = max(0, min(len(sorted_vals) - 1, int(round(p / 100.0 * (len(sorted_vals) - 1)))))
    return sorted_vals[k]


def measure_step(config, kv, steps, warmup, seed=None, chunk_tokens=0, capacity=0, window=0, sinks=4,
                 flush_mib=0, copy_calibration_mib=0, fill="values", keep=False, warm_ms=0.0):
    """One workload, one cache format: whole-step time over exactly `steps` steps (wall clock
    between synchronisations, HIP events around the streaming kernel on every 4th of them), then
    `steps` more steps with events on every launch for the kernel-time percentiles.  warm_ms > 0:
    after the `warmup` steps, further untimed steps until that much time has passed (the device
    takes some 20 ms of continuous work to reach its clocks after an idle spell: a short config
    timed right after five warm-up steps reads up to 10 % low)."""
    import torch
    from paper_2403_11421_amd import rpart, workloads as W

    cfg = W.CONFIGS[config]
    seed = W.DEFAULT_SEED if seed is None else seed
    lens = W.seq_lens(cfg, seed)
    n_tok = W.total_tokens_after_append(lens)
    if window > 0:                                 # rows attended after the append: the bounded buffer's
        n_tok = sum(min(L + 1, sinks + window) for L in lens)
    # algorithmic bytes: every cached K and V row once (quantised: code bytes + the row parameters)
    kv_bytes = kv_bytes_per_token(cfg, kv) * n_tok
    q8 = kv != "fp16"
    f_partial = rpart.fd_rpartq_partial if q8 else rpart.fd_rpart_partial

    cache, vec = build_case(cfg, lens, seed, chunk_tokens, kv=kv, capacity=capacity, window=window,
                            sinks=sinks, fill=fill)
    out = torch.empty_like(vec["q"])
    ws = cache.workspace(n_tok)
    lens0 = cache.seq_lens.clone()
    seen0 = cache.seq_seen.clone() if window > 0 else None
    desc = cache.desc

    def step(pair=None):
        # the two launches of fd_rpart_step, issued separately so that events can bracket the second
        cache.seq_lens.copy_(lens0)                # every step is the quoted config: L cached + 1 appended
        if seen0 is not None:
            cache.seq_seen.copy_(seen0)
        rpart.fd_kv_append_plan(desc, vec["k_new"], vec["v_new"], ws)
        if pair:
            pair[0].record()
        f_partial(desc, vec["q"], out, ws)
        if pair:
            pair[1].record()

    def events():
        return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    if copy_calibration_mib > 0:
        src = torch.empty(copy_calibration_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                             # reads and writes exactly that many bytes
        torch.cuda.synchronize()
        del src, dst

    # HIP events around the dominant kernel on every 4th timed step: each record costs a ~5 us
    # bubble in the stream, so timing every launch would tax the whole-step figure by ~1 %
    ev = [events() if k % 4 == 0 else None for k in range(steps)]
    flush = torch.zeros(flush_mib << 20, dtype=torch.uint8, device="cuda") if flush_mib > 0 else None
    step_ev = []
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t_warm = time.perf_counter()
    while (time.perf_counter() - t_warm) * 1e3 < warm_ms:
        for _ in range(8):
            step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        if flush is not None:                      # cold caches: time the step alone, by events
            flush.add_(1)
            se = events()
            se[0].record()
            step(ev[k])
            se[1].record()
            step_ev.append(se)
        else:
            step(ev[k])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if flush is not None:
        dt = sum(a.elapsed_time(b) for a, b in step_ev) * 1e-3

    st = rpart.fd_last_device_status(desc, ws)
    assert st == 0, st
    plan = rpart.fd_plan_info(ws)
    assert plan["total_tokens"] == n_tok, (plan, n_tok)
    out_host = out.cpu()                            # checked on the host: no torch kernel needed
    assert bool(torch.isfinite(out_host.float()).all())

    # kernel-time distribution: events on every launch, outside the timed region
    every = [events() for _ in range(steps)]
    for p in every:
        step(p)
    torch.cuda.synchronize()
    kms = sorted(a.elapsed_time(b) for a, b in every)
    # the same kernel launched back to back on the step's plan, one pair of events around the lot:
    # the events' own ~10 us, which weigh on a short kernel's single-launch figure, are shared out
    b2b = events()
    b2b[0].record()
    for _ in range(steps):
        f_partial(desc, vec["q"], out, ws)
    b2b[1].record()
    torch.cuda.synchronize()
    b2b_ms = b2b[0].elapsed_time(b2b[1]) / steps

    ms_step = dt / steps * 1e3
    timed = [p for p in ev if p]
    part_ms = sum(a.elapsed_time(b) for a, b in timed) / len(timed)
    value = kv_bytes / (ms_step * 1e-3) / 1e9
    achieved = kv_bytes / (part_ms * 1e-3) / 1e9
    res = {
        "config": config, "kv": kv, "B": cfg.B, "H": cfg.H, "d": cfg.d, "total_tokens": n_tok,
        "kv_bytes_per_step": kv_bytes, "seed": seed, "plan": plan, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_step, "step_gbps": value, "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
        "seq_per_s": cfg.B / (ms_step * 1e-3),
        "seq_per_s_whole_model": cfg.B / (ms_step * 1e-3) / cfg.n_layers,
        "ns_per_cached_token": ms_step * 1e6 / n_tok,
        "kernel": "rpartq_partial_kernel" if q8 else "rpart_partial_kernel",
        "kernel_ms_avg": part_ms, "launches_timed": len(timed), "kernel_gbps": achieved,
        "frac": achieved / HBM_PEAK_GBPS,
        "kernel_ms_p10": _pct(kms, 10), "kernel_ms_p50": _pct(kms, 50), "kernel_ms_p90": _pct(kms, 90),
        "kernel_launches_in_percentiles": len(kms),
        "kernel_gbps_p50": kv_bytes / (_pct(kms, 50) * 1e-3) / 1e9,
        "kernel_ms_back_to_back": b2b_ms, "kernel_gbps_back_to_back": kv_bytes / (b2b_ms * 1e-3) / 1e9,
        "traffic": counter_traffic(cfg.name, kv) if window == 0 else None,
    }
    if keep:
        res["_objects"] = (cfg, cache, vec, lens, out)
    return res


def read_only_ceiling(slab):
    """The device's pure-read rate, GB/s: the library's read probe over `slab`, or over an 8 GiB
    buffer of its own when the slab is smaller than that (a launch over 4 GB lasts 0.6 ms, and its
    ramp and tail then cost the figure 3 %); median of five launches, each between its own events."""
    import torch
    from paper_2403_11421_amd import rpart
    sink = torch.zeros(1, dtype=torch.int32).to("cuda")
    buf = slab if slab.numel() * slab.element_size() >= (8 << 30) else \
        torch.empty(8 << 30, dtype=torch.uint8, device="cuda")
    nread = rpart.fd_hbm_read_probe(buf, sink)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
    for e0, e1 in pairs:
        e0.record()
        rpart.fd_hbm_read_probe(buf, sink)
        e1.record()
    torch.cuda.synchronize()
    ms = sorted(e0.elapsed_time(e1) for e0, e1 in pairs)[2]
    return nread / (ms * 1e-3) / 1e9


def schedule_result(kind, B, S, F, kv="fp16", W_lim=None):
    """Per-step R-Part latency of a decode loop under a schedule of Section 4.2 (one layer,
    Llama-7B head shape), steady state (after the cold start)."""
    from paper_2403_11421_amd import sls_run, workloads as W
    n_steps = 2 * S
    r = sls_run.run_schedule(kind, B, S, F, n_steps, W_lim=W_lim, kv=kv)
    bpt = kv_bytes_per_token(W.RPartConfig("sched", B, r["H"], r["d"], "const", 0, 0), kv)
    ms, loads = r["ms"], r["loads"]
    steady = list(range(S, n_steps))
    tok = sum(loads[i] for i in steady)
    tms = sum(ms[i] for i in steady)
    srt = sorted(ms[i] for i in steady)
    return {"schedule": kind, "kv": kv, "B": B, "S": S, "F": F, "M": r["M"], "H": r["H"], "d": r["d"],
            "steps": n_steps, "steady_steps": len(steady), "W_lim": r.get("W_lim"),
            "peak_load_tokens": max(loads[i] for i in steady), "mean_load_tokens": tok / len(steady),
            "peak_ms": srt[-1], "p50_ms": _pct(srt, 50), "mean_ms": tms / len(steady),
            "steady_kv_gbps": bpt * tok / (tms * 1e-3) / 1e9,
            "steady_frac_of_hbm_peak": bpt * tok / (tms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "tokens_per_s_one_layer": len(steady) * B / (tms * 1e-3)}


def schedule_mode(args) -> int:
    """One JSON line per schedule."""
    for kind in (["batch", "sls"] if args.schedule == "both" else [args.schedule]):
        r = schedule_result(kind, args.sched_B, args.sched_S, args.sched_F, args.kv,
                            args.sched_wlim if args.sched_wlim > 0 else None)
        r.update({"metric": "R-Part latency per decode step under a sequence schedule (Section 4.2)",
                  "unit": "ms", "n_gpus": 1, "data": "synthetic", "dtype": "f32"})
        print(json.dumps(r))
    return 0


# the S-Part latency the paper prints for its S-worker (Table 2: one block of the 7B model at batch
# 1024 on an A10), used as T(B) of Eq. 11 next to the R measured here; context, not a measurement
PAPER_T_B_MS, PAPER_T_B_BATCH = 7.08, 1024


def pipeline_results(config, kv, layers, steps, warmup, modes=("serial", "shared", "overlap")):
    """Token step of an N-block model with two mini-batches (Section 4.1's token-level pipeline
    as the R-worker sees it): blocks A0, B0, A1, B1, ... each append + attend.  Three ways of
    issuing the same work:
      serial   one stream, every block plans for itself (fd_rpart_step)
      shared   one stream, one plan per mini-batch and token (fd_rpart_layer_step)
      overlap  as shared, each mini-batch on its own stream
    Cached lengths grow by one per token step; the bytes are summed exactly."""
    import torch
    from paper_2403_11421_amd import rpart, sched, workloads as W
    from paper_2403_11421_amd.pipeline import RWorker

    cfg = W.CONFIGS[config]
    N, dev = layers, torch.device("cuda:0")
    Bm = cfg.B // 2                                           # the batch split into mini-batches A and B
    lens = W.seq_lens(cfg)
    mb_lens = [lens[:Bm], lens[Bm:2 * Bm]]
    n_tokens = (warmup + steps) * len(modes)
    sub = [W.RPartConfig(f"{cfg.name}_mb{m}", Bm, cfg.H, cfg.d, "const", 0, 0, scale=cfg.scale)
           for m in range(2)]
    bpt = kv_bytes_per_token(cfg, kv)
    rw = RWorker(cfg.H, cfg.d, N, [[L + n_tokens + 1 for L in l] for l in mb_lens],
                 kv=kv, n_streams=2, device=dev)
    for m in range(2):
        c0 = rw.caches[m][0]
        for b, L in enumerate(mb_lens[m]):
            if L:
                c0.fill("K", b, W.gen_cache_block(cfg, "K", m * Bm + b, L, W.DEFAULT_SEED, dev))
                c0.fill("V", b, W.gen_cache_block(cfg, "V", m * Bm + b, L, W.DEFAULT_SEED, dev))
        for c in rw.caches[m][1:]:                         # values do not affect the timing
            for a, b_ in zip(c.slabs(), c0.slabs()):
                a.copy_(b_)
    vec = [[{w: W.gen_vectors(sub[m], w, 100 + l, dev) for w in ("q", "k_new", "v_new")}
            for l in range(N)] for m in range(2)]
    q = [[vec[m][l]["q"] for l in range(N)] for m in range(2)]
    kn = [[vec[m][l]["k_new"] for l in range(N)] for m in range(2)]
    vn = [[vec[m][l]["v_new"] for l in range(N)] for m in range(2)]
    out = [[torch.empty_like(q[m][l]) for l in range(N)] for m in range(2)]
    step_fn = rpart.fd_rpart_step if kv == "fp16" else rpart.fd_rpartq_step
    results = []
    for mode in modes:                                       # same caches for all
        for m in range(2):
            rw.set_lens(m, mb_lens[m])
        rw.use_streams(2 if mode == "overlap" else 1)

        def token():
            if mode == "serial":
                for l in range(N):
                    for m in range(2):
                        step_fn(rw.caches[m][l].desc, q[m][l], kn[m][l], vn[m][l], out[m][l], rw.ws[m])
            else:
                rw.token_step(q, kn, vn, out)

        for _ in range(warmup):
            token()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            token()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        assert rw.status() == 0
        tokens = sum(sum(L + warmup + s + 1 for L in l) for l in mb_lens for s in range(steps))
        kv_bytes = bpt * tokens * N
        ms = dt / steps * 1e3
        value = kv_bytes / dt / 1e9
        R_ns = dt * 1e9 / (tokens * N)                     # Section 4.3's R: per cached token and block
        results.append({
            "issue": mode, "config": config, "kv": kv, "layers": N, "mini_batches": 2, "sequences": 2 * Bm,
            "steps": steps, "ms_per_token_step": ms, "ms_per_block_step": ms / (2 * N),
            "kv_gbps": value, "frac_of_hbm_peak": value / HBM_PEAK_GBPS,
            "tokens_per_s": 2 * Bm / (ms * 1e-3) * N / cfg.n_layers,
            "R_ns_per_cached_token": R_ns,
            # Eq. 11: R-workers of this kind that one S-worker with the paper's T(B) keeps busy
            # at sequences of 1024 tokens
            "eq11_rworkers_for_paper_sworker": sched.model_num_rworkers(
                PAPER_T_B_BATCH, 1024, R_ns * 1e-6, PAPER_T_B_MS),
            "eq11_inputs": {"B": PAPER_T_B_BATCH, "S": 1024, "T_B_ms": PAPER_T_B_MS,
                            "T_B_source": "paper Table 2, S-Part of one 7B block on an A10"}})
    del rw
    torch.cuda.empty_cache()
    return results


def pipeline_mode(args) -> int:
    for r in pipeline_results(args.config, args.kv, args.layers, args.steps, args.warmup):
        line = {"metric": METRIC, "value": r["kv_gbps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
                "warmup": args.warmup, "ms_per_step": r["ms_per_token_step"], "higher_is_better": True,
                "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                "config": {"workload": f"{r['config']} split into two mini-batches, {r['layers']} blocks, "
                                       f"{r['kv']} KV, one token step = {2 * r['layers']} block steps",
                           "issue": r["issue"], "layers": r["layers"]}}
        line.update({k: v for k, v in r.items() if k not in ("config",)})
        print(json.dumps(line), flush=True)
    return 0


def extras(args):
    """The other configs and cache formats, the schedule loop and the pipeline, each with fewer
    steps than the headline; every entry is measured exactly like the headline."""
    import torch
    ex = {"steps_each": args.extra_steps, "untimed_warm_ms_each": EXTRA_WARM_MS}
    t0 = time.time()

    def short(r):
        keys = ("config", "kv", "total_tokens", "kv_bytes_per_step", "plan", "steps", "ms_per_step", "step_gbps",
                "seq_per_s", "kernel_ms_avg", "kernel_gbps", "frac", "kernel_ms_p10", "kernel_ms_p50",
                "kernel_ms_p90", "kernel_ms_back_to_back", "kernel_gbps_back_to_back")
        return {k: r[k] for k in keys}

    ex["configs_fp16"] = {}
    for name in ("c3_7b_ragged", "c4_13b_geometric", "c5_capacity", "t2_batch1024", "t2_batch1", "c1_tiny"):
        ex["configs_fp16"][name] = short(measure_step(name, "fp16", args.extra_steps, args.warmup, warm_ms=EXTRA_WARM_MS))
        torch.cuda.empty_cache()
    ex["quantised_kv"] = {}
    for kv in ("int8", "int4"):
        ex["quantised_kv"][kv] = {name: short(measure_step(name, kv, args.extra_steps, args.warmup, warm_ms=EXTRA_WARM_MS))
                                  for name in ("c2_7b_uniform", "c3_7b_ragged", "c4_13b_geometric", "c5_capacity",
                                               "t2_batch1024")}
        torch.cuda.empty_cache()
    ex["schedule_loop"] = {kind: schedule_result(kind, args.sched_B, args.sched_S, args.sched_F)
                           for kind in ("batch", "sls")}
    torch.cuda.empty_cache()
    ex["pipeline"] = pipeline_results("c2_7b_uniform", "fp16", args.layers, 10, 3, modes=("serial", "overlap"))
    ex["wall_s"] = time.time() - t0
    return ex


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="c2_7b_uniform")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--chunk-tokens", type=int, default=0, help="split-K chunk length, 0 = library's choice")
    ap.add_argument("--flush-mib", type=int, default=0,
                    help="before every step, read-modify-write this many MiB through the caches (other work "
                         "between two steps of a layer, as in a model of many layers); the step time is then "
                         "the sum of HIP-event times around the steps, not the wall clock")
    ap.add_argument("--capacity", type=int, default=0,
                    help="rows of every sequence's cache block (equal slots); 0 = fitted to its length")
    ap.add_argument("--cpu-sample", type=int, default=96, help="sequences timed on the CPU oracle (0 = skip)")
    ap.add_argument("--kv", choices=["fp16", "int8", "int4"], default="fp16",
                    help="KV-cache format: fp16 (the headline path) or a quantised cache (Section 5.2)")
    ap.add_argument("--extras", choices=["auto", "all", "none"], default="auto",
                    help="also measure the other configs, cache formats, the schedule loop and the pipeline and "
                         "carry them in the same JSON line (auto: only for the default config and format)")
    ap.add_argument("--extra-steps", type=int, default=40, help="timed steps of every entry under extras")
    ap.add_argument("--fill", choices=["values", "pattern"], default="values",
                    help="pattern: fill the cache without dispatching a single torch kernel (for runs under "
                         "rocprofv3 --pmc); implies no CPU baseline, no entropy figure and no extras")
    ap.add_argument("--sched-wlim", type=int, default=0,
                    help="--schedule control: load limit W_lim of Algorithm 1 in cached tokens "
                         "(0 = Eq. 6's peak)")
    ap.add_argument("--schedule", choices=["none", "batch", "sls", "control", "both"], default="none",
                    help="instead of the fixed-length step, run a multi-step decode loop under the "
                         "large-batch or the load-stabilising schedule (Section 4.2) and report the "
                         "per-step R-Part latency")
    ap.add_argument("--window", type=int, default=0,
                    help="window attention: every sequence keeps --sinks first tokens and its last "
                         "WINDOW tokens in a bounded cache (0 = attend to everything)")
    ap.add_argument("--sinks", type=int, default=4)
    ap.add_argument("--pipeline", action="store_true",
                    help="instead of the one-layer step, run token steps of an N-block model with "
                         "two mini-batches (Section 4.1) and compare three ways of issuing them")
    ap.add_argument("--layers", type=int, default=8, help="blocks held by --pipeline")
    ap.add_argument("--sched-B", type=int, default=1024)
    ap.add_argument("--sched-S", type=int, default=1024)
    ap.add_argument("--sched-F", type=int, default=16)
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB before the steps, as the "
                         "known-size reference dispatch for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this library runs the R-Part on ONE GPU; sequences are independent, so more "
              "GPUs would each run this same kernel on their share. Use --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2403_11421_amd import rpart

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    rpart.load()                                   # fails loudly when the HIP library is missing
    torch.cuda.set_device(0)
    if args.schedule != "none":
        return schedule_mode(args)
    if args.pipeline:
        return pipeline_mode(args)

    pattern = args.fill == "pattern"
    r = measure_step(args.config, args.kv, args.steps, args.warmup, seed=args.seed,
                     chunk_tokens=args.chunk_tokens, capacity=args.capacity, window=args.window,
                     sinks=args.sinks, flush_mib=args.flush_mib,
                     copy_calibration_mib=args.copy_calibration_mib, fill=args.fill, keep=True)
    cfg, cache, vec, lens, out = r.pop("_objects")
    q8 = args.kv != "fp16"
    res = {
        "metric": METRIC, "value": r["step_gbps"], "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} H={cfg.H} d={cfg.d} {args.kv} KV, "
                               f"{r['total_tokens']} cached tokens after append, 1 layer"
                               + (f", window attention: {args.sinks} sink + last {args.window} tokens"
                                  if args.window > 0 else "")
                               + (", cache filled with a bit pattern (no torch kernels)" if pattern else ""),
                   "B": cfg.B, "H": cfg.H, "d": cfg.d, "total_tokens": r["total_tokens"],
                   "kv_bytes_per_step": r["kv_bytes_per_step"], "seed": r["seed"], "plan": r["plan"],
                   "launches_per_step": 2},
        "flush_mib_between_steps": args.flush_mib,
        "pct_of_hbm_peak": r["pct_of_hbm_peak"],
        "seq_per_s": r["seq_per_s"],
        "seq_per_s_whole_model": r["seq_per_s_whole_model"],
        "ns_per_cached_token": r["ns_per_cached_token"],
        "roofline": {"bound": "hbm", "kernel": r["kernel"],
                     "achieved": r["kernel_gbps"],
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": r["frac"],
                     "avg_kernel_ms": r["kernel_ms_avg"], "launches_timed": r["launches_timed"],
                     "traffic": r["traffic"], "algorithmic_bytes": r["kv_bytes_per_step"]},
        "kernel_ms_p10": r["kernel_ms_p10"], "kernel_ms_p50": r["kernel_ms_p50"],
        "kernel_ms_p90": r["kernel_ms_p90"],
        "kernel_launches_in_percentiles": r["kernel_launches_in_percentiles"],
        "kernel_ms_back_to_back": r["kernel_ms_back_to_back"],
        "kernel_gbps_back_to_back": r["kernel_gbps_back_to_back"],
    }
    # the device's pure-read ceiling, timed beside the kernel over the K slab (context for `frac`)
    res["roofline"]["read_only_ceiling_gbps"] = read_only_ceiling(cache.k_codes if q8 else cache.k)

    plain = not q8 and args.window == 0 and not pattern
    if cfg.peaked_keys and plain:
        res["softmax_entropy"] = softmax_entropy(cfg, cache, vec, [L + 1 for L in lens])
    if args.cpu_sample > 0 and plain:
        res["cpu_baseline"] = cpu_baseline(cfg, cache, vec, [L + 1 for L in lens], args.cpu_sample)
    want_extras = args.extras == "all" or (args.extras == "auto" and args.config == "c2_7b_uniform"
                                           and plain and args.flush_mib == 0 and args.capacity == 0
                                           and args.chunk_tokens == 0 and args.seed is None)
    if want_extras and not pattern:
        del cache, vec, out
        torch.cuda.empty_cache()
        res["extras"] = extras(args)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
