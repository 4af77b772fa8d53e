#!/usr/bin/env python3
"""Throughput of the R-Part decode step on one MI355X.

A step is one pass of the whole hot path over one batch: restore the cached
lengths, append the new k/v rows and plan the ragged split (one launch), stream
K/V (split-K attention with the log-sum-exp merge folded in; the second launch).  Inputs are synthetic, seeded, resident in HBM before
the timed region starts.  Prints ONE JSON line.

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


def build_case(cfg, lens, seed, chunk_tokens, growth=8, kv="fp16", window=0, sinks=0, capacity=0):
    """window > 0: a windowed cache of sinks + window rows per sequence that has already seen
    lens[b] tokens (its rows hold that many, or all of them when the history is longer).
    capacity > 0: every sequence gets a block of that many rows (equal slots, as a slot allocator
    hands them out) instead of one fitted to its length."""
    import torch
    from paper_2403_11421_amd import workloads as W
    from paper_2403_11421_amd.kvcache import KVCache, KVCacheQ

    dev = torch.device("cuda:0")
    kw = {} if kv == "fp16" else {"bits": 4 if kv == "int4" else 8}
    cls = KVCache if kv == "fp16" else KVCacheQ
    if window > 0:
        cache = cls(cfg.B, cfg.H, cfg.d, [sinks + window] * cfg.B, dev, chunk_tokens, n_sink=sinks, **kw)
        held = [min(L, sinks + window) for L in lens]
    else:
        caps = [capacity] * cfg.B if capacity > 0 else [L + growth for L in lens]
        assert all(c > L for c, L in zip(caps, lens)), "capacity must exceed every cached length"
        cache = cls(cfg.B, cfg.H, cfg.d, caps, dev, chunk_tokens, **kw)
        held = lens
    for b, L in enumerate(held):
        if L:
            cache.fill("K", b, W.gen_cache_block(cfg, "K", b, L, seed, dev))
            cache.fill("V", b, W.gen_cache_block(cfg, "V", b, L, seed, dev))
    cache.set_lens(held)
    if window > 0:
        cache.seq_seen.copy_(torch.tensor(list(lens), dtype=torch.int32))
    vec = {w: W.gen_vectors(cfg, w, seed, dev) for w in ("q", "k_new", "v_new")}
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
        "seq_per_s": len(batch) / dt,
    }


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


def schedule_mode(args) -> int:
    """Per-step R-Part latency of a decode loop under the schedules of Section 4.2 (one layer,
    Llama-7B head shape): one JSON line per schedule."""
    from paper_2403_11421_amd import sls_run

    B, S, F = args.sched_B, args.sched_S, args.sched_F
    n_steps = 2 * S
    for kind in (["batch", "sls"] if args.schedule == "both" else [args.schedule]):
        r = sls_run.run_schedule(kind, B, S, F, n_steps,
                                 W_lim=args.sched_wlim if args.sched_wlim > 0 else None, kv=args.kv)
        from paper_2403_11421_amd import workloads as W
        bpt = kv_bytes_per_token(W.RPartConfig("sched", B, r["H"], r["d"], "const", 0, 0), args.kv)
        ms, loads = r["ms"], r["loads"]
        steady = list(range(S, n_steps))                     # after the cold start
        tok = sum(loads[i] for i in steady)
        tms = sum(ms[i] for i in steady)
        srt = sorted(ms[i] for i in steady)
        print(json.dumps({
            "metric": "R-Part latency per decode step under a sequence schedule (Section 4.2)",
            "schedule": kind, "kv": args.kv, "B": B, "S": S, "F": F, "M": r["M"], "H": r["H"], "d": r["d"],
            "steps": n_steps, "steady_steps": len(steady), "W_lim": r.get("W_lim"),
            "peak_load_tokens": max(loads[i] for i in steady),
            "mean_load_tokens": tok / len(steady),
            "peak_ms": srt[-1], "p50_ms": srt[len(srt) // 2], "mean_ms": tms / len(steady),
            "steady_kv_gbps": bpt * tok / (tms * 1e-3) / 1e9,
            "tokens_per_s_one_layer": len(steady) * B / (tms * 1e-3),
            "unit": "ms", "n_gpus": 1, "data": "synthetic", "dtype": "f32"}))
    return 0


def pipeline_mode(args) -> int:
    """Token step of an N-block model with two mini-batches (Section 4.1's token-level pipeline
    as the R-worker sees it): blocks A0, B0, A1, B1, ... each append + attend.  Three ways of
    issuing the same work, one JSON line each:
      serial   one stream, every block plans for itself (fd_rpart_step)
      shared   one stream, one plan per mini-batch and token (fd_rpart_layer_step)
      overlap  as shared, each mini-batch on its own stream
    Cached lengths grow by one per token step; the bytes are summed exactly."""
    import torch
    from paper_2403_11421_amd import rpart, workloads as W
    from paper_2403_11421_amd.pipeline import RWorker

    cfg = W.CONFIGS[args.config]
    N, dev = args.layers, torch.device("cuda:0")
    Bm = cfg.B // 2                                           # the batch split into mini-batches A and B
    lens = W.seq_lens(cfg)
    mb_lens = [lens[:Bm], lens[Bm:2 * Bm]]
    n_tokens = args.warmup + args.steps
    sub = [W.RPartConfig(f"{cfg.name}_mb{m}", Bm, cfg.H, cfg.d, "const", 0, 0, scale=cfg.scale)
           for m in range(2)]
    bpt = kv_bytes_per_token(cfg, args.kv)
    rw = RWorker(cfg.H, cfg.d, N, [[L + n_tokens + 1 for L in l] for l in mb_lens],
                 kv=args.kv, n_streams=2, device=dev)
    for m in range(2):
        c0 = rw.caches[m][0]
        for b, L in enumerate(mb_lens[m]):
            if L:
                c0.fill("K", b, W.gen_cache_block(cfg, "K", m * Bm + b, L, W.DEFAULT_SEED, dev))
                c0.fill("V", b, W.gen_cache_block(cfg, "V", m * Bm + b, L, W.DEFAULT_SEED, dev))
        for c in rw.caches[m][1:]:                         # values do not affect the timing
            for name in (("k", "v") if args.kv == "fp16" else ("k_codes", "v_codes", "k_scale", "v_scale")):
                getattr(c, name).copy_(getattr(c0, name))
    vec = [[{w: W.gen_vectors(sub[m], w, 100 + l, dev) for w in ("q", "k_new", "v_new")}
            for l in range(N)] for m in range(2)]
    q = [[vec[m][l]["q"] for l in range(N)] for m in range(2)]
    kn = [[vec[m][l]["k_new"] for l in range(N)] for m in range(2)]
    vn = [[vec[m][l]["v_new"] for l in range(N)] for m in range(2)]
    out = [[torch.empty_like(q[m][l]) for l in range(N)] for m in range(2)]
    step_fn = rpart.fd_rpart_step if args.kv == "fp16" else rpart.fd_rpartq_step
    for mode in ("serial", "shared", "overlap"):                                 # same caches for all
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

        for _ in range(args.warmup):
            token()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            token()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        assert rw.status() == 0
        tokens = sum(sum(L + args.warmup + s + 1 for L in l) for l in mb_lens for s in range(args.steps))
        kv_bytes = bpt * tokens * N
        ms = dt / args.steps * 1e3
        value = kv_bytes / dt / 1e9
        print(json.dumps({
            "metric": METRIC, "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"{cfg.name} split into two mini-batches of {Bm}, {N} blocks, "
                                   f"{args.kv} KV, one token step = {2 * N} block steps",
                       "issue": mode, "layers": N, "kv_bytes_per_step": kv_bytes // args.steps},
            "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
            "ms_per_block_step": ms / (2 * N),
            "tokens_per_s": 2 * Bm / (ms * 1e-3) * N / cfg.n_layers,
            # Section 4.3's R: latency of this R-worker per cached token and block
            "R_ns_per_cached_token": dt * 1e9 / (tokens * N)}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
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
    from paper_2403_11421_amd import rpart, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    rpart.load()                                   # fails loudly when the HIP library is missing
    torch.cuda.set_device(0)
    if args.schedule != "none":
        return schedule_mode(args)
    if args.pipeline:
        return pipeline_mode(args)
    cfg = W.CONFIGS[args.config]
    seed = W.DEFAULT_SEED if args.seed is None else args.seed
    lens = W.seq_lens(cfg, seed)
    n_tok = W.total_tokens_after_append(lens)
    if args.window > 0:                            # rows attended after the append: the bounded buffer's
        n_tok = sum(min(L + 1, args.sinks + args.window) for L in lens)
    # algorithmic bytes: every cached K and V row once (int8: d code bytes + a 4-byte scale per row)
    bytes_per_token = kv_bytes_per_token(cfg, args.kv)
    kv_bytes = bytes_per_token * n_tok
    q8 = args.kv != "fp16"
    f_partial = rpart.fd_rpartq_partial if q8 else rpart.fd_rpart_partial

    cache, vec = build_case(cfg, lens, seed, args.chunk_tokens, kv=args.kv, capacity=args.capacity, window=args.window,
                            sinks=args.sinks)
    out = torch.empty_like(vec["q"])
    ws = cache.workspace(n_tok)
    lens0 = cache.seq_lens.clone()
    seen0 = cache.seq_seen.clone() if args.window > 0 else None
    desc = cache.desc

    # HIP events around the dominant kernel on every 4th timed step: each record costs a ~5 us
    # bubble in the stream, so timing every launch would tax the whole-step figure by ~1 %
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          if k % 4 == 0 else None for k in range(args.steps)]

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

    if args.copy_calibration_mib > 0:
        src = torch.ones(args.copy_calibration_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                             # reads and writes exactly that many bytes
        torch.cuda.synchronize()
        del src, dst

    flush = torch.zeros(args.flush_mib << 20, dtype=torch.uint8, device="cuda") if args.flush_mib > 0 else None
    step_ev = []
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        if flush is not None:                      # cold caches: time the step alone, by events
            flush.add_(1)
            se = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
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

    assert rpart.fd_read_status(desc) == 0
    plan = rpart.fd_plan_info(ws)
    assert plan["total_tokens"] == n_tok, (plan, n_tok)
    assert bool(torch.isfinite(out.float()).all())

    ms_step = dt / args.steps * 1e3
    timed = [p for p in ev if p]
    part_ms = sum(a.elapsed_time(b) for a, b in timed) / len(timed)
    value = kv_bytes / (ms_step * 1e-3) / 1e9
    achieved = kv_bytes / (part_ms * 1e-3) / 1e9

    res = {
        "metric": METRIC, "value": value, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} H={cfg.H} d={cfg.d} {args.kv} KV, "
                               f"{n_tok} cached tokens after append, 1 layer"
                               + (f", window attention: {args.sinks} sink + last {args.window} tokens"
                                  if args.window > 0 else ""),
                   "B": cfg.B, "H": cfg.H, "d": cfg.d, "total_tokens": n_tok,
                   "kv_bytes_per_step": kv_bytes, "seed": seed, "plan": plan},
        "flush_mib_between_steps": args.flush_mib,
        "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
        "seq_per_s": cfg.B / (ms_step * 1e-3),
        "seq_per_s_whole_model": cfg.B / (ms_step * 1e-3) / cfg.n_layers,
        "ns_per_cached_token": ms_step * 1e6 / n_tok,
        "roofline": {"bound": "hbm", "kernel": "rpartq_partial_kernel" if q8 else "rpart_partial_kernel",
                     "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "avg_kernel_ms": part_ms, "launches_timed": len(timed), "traffic": counter_traffic(cfg.name, args.kv) if args.window == 0 else None,
                     "algorithmic_bytes": kv_bytes},
    }
    # the device's pure-read ceiling, timed beside the kernel over the K slab (context for `frac`)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    slab = cache.k_codes if q8 else cache.k
    buf = slab if slab.numel() * slab.element_size() >= (1 << 30) else \
        torch.zeros(1 << 31, dtype=torch.uint8, device="cuda")     # tiny configs: a 2 GiB stand-in
    nread = rpart.fd_hbm_read_probe(buf, sink)
    e0.record()
    for _ in range(5):
        rpart.fd_hbm_read_probe(buf, sink)
    e1.record()
    torch.cuda.synchronize()
    res["roofline"]["read_only_ceiling_gbps"] = nread * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9

    if cfg.peaked_keys and not q8 and args.window == 0:
        res["softmax_entropy"] = softmax_entropy(cfg, cache, vec, [L + 1 for L in lens])
    if args.cpu_sample > 0 and not q8 and args.window == 0:
        res["cpu_baseline"] = cpu_baseline(cfg, cache, vec, [L + 1 for L in lens], args.cpu_sample)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
