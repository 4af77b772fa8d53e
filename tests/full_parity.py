"""Whole-batch parity of a full-size config against the oracle, in the launch configuration
bench.py times (append + plan launch, streaming launch, library-chosen chunking, workspace
sized for the step's tokens).

Every oracle input comes from the seeded generator, never from the device cache: for each
sequence the cached rows are regenerated, copied to the host, (for a quantised cache) quantised
by the oracle's own quantiser, the step's k/v appended by the oracle's append, and the query
attended by the oracle's decode.  The device cache blocks are then compared with the oracle's
bit for bit (this covers the library's bulk store and its append), the outputs element by
element.  Sequences are handled in groups so that the host never holds more than a few GB.
"""
from __future__ import annotations

import time
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Sequence

import numpy as np
import torch

from oracle import rpart_oracle as O
from paper_2403_11421_amd import rpart, workloads as W
from paper_2403_11421_amd.kvcache import KVCache, KVCacheQ
from tests.util import bits, f64

TOL = 2e-3
THREADS = 16


def stratified(lens: Sequence[int], n: int) -> List[int]:
    """n sequences spread evenly over the length ranks, shortest and longest included."""
    order = np.argsort(np.asarray(lens), kind="stable")
    if n >= len(lens):
        return sorted(int(x) for x in order)
    picks = {int(order[(k * (len(lens) - 1)) // (n - 1)]) for k in range(n)}
    return sorted(picks)


def _token_major(t: torch.Tensor) -> np.ndarray:
    """device [H, L, ...] -> host [L, H, ...] contiguous"""
    return np.ascontiguousarray(t.permute(1, 0, *range(2, t.dim())).contiguous().cpu().numpy())


def _token_major_bits(t: torch.Tensor) -> np.ndarray:
    return bits(t.permute(1, 0, 2))


class FullCase:
    """Device side of one full-size step in the given cache format ("fp16", "int8", "int4")."""

    def __init__(self, name: str, kv: str, seed: int = W.DEFAULT_SEED):
        self.cfg, self.kv, self.seed = W.CONFIGS[name], kv, seed
        cfg = self.cfg
        self.lens = W.seq_lens(cfg, seed)
        self.n_tok = W.total_tokens_after_append(self.lens)
        dev = "cuda"
        caps = [L + 8 for L in self.lens]
        if kv == "fp16":
            self.cache = KVCache(cfg.B, cfg.H, cfg.d, caps, dev)
        else:
            self.cache = KVCacheQ(cfg.B, cfg.H, cfg.d, caps, dev, bits=4 if kv == "int4" else 8)
        for b, L in enumerate(self.lens):
            if L:
                self.cache.fill("K", b, W.gen_cache_block(cfg, "K", b, L, seed, dev))
                self.cache.fill("V", b, W.gen_cache_block(cfg, "V", b, L, seed, dev))
        self.cache.set_lens(self.lens)
        self.q, self.k_new, self.v_new = (W.gen_vectors(cfg, w, seed, dev) for w in ("q", "k_new", "v_new"))
        self.out = torch.full((cfg.B, cfg.H, cfg.d), float("nan"), dtype=torch.float16, device=dev)
        self.ws = self.cache.workspace(self.n_tok)              # as bench.py sizes it

    def step(self):
        """The calls bench.py times, in its order: the two launches of a step."""
        d = self.cache.desc
        rpart.fd_kv_append_plan(d, self.k_new, self.v_new, self.ws)
        if self.kv == "fp16":
            rpart.fd_rpart_partial(d, self.q, self.out, self.ws)
        else:
            rpart.fd_rpartq_partial(d, self.q, self.out, self.ws)
        torch.cuda.synchronize()
        assert rpart.fd_read_status(d) == 0
        self.plan = rpart.fd_plan_info(self.ws)
        assert self.plan["total_tokens"] == self.n_tok
        assert self.cache.seq_lens.cpu().tolist() == [L + 1 for L in self.lens]
        assert bool(torch.isfinite(self.out.float()).all())


def _oracle_group_fp16(case: FullCase, group, q, k_new, v_new):
    cfg = case.cfg
    K, V = [], []
    for b in group:
        L = case.lens[b]
        for which, dst in (("K", K), ("V", V)):
            blk = np.zeros((L + 1, cfg.H, cfg.d), dtype=np.uint16)
            if L:
                blk[:L] = _token_major_bits(W.gen_cache_block(cfg, which, b, L, case.seed, "cuda"))
            dst.append(blk)
    lens = np.asarray([case.lens[b] for b in group], dtype=np.int32)
    O.kv_append(K, V, lens, k_new[group], v_new[group])
    want, _, _ = O.rpart_decode(K, V, lens, q[group], nthreads=THREADS)
    maxv = 0.0
    for i, b in enumerate(group):
        n = int(lens[i])
        assert np.array_equal(_token_major_bits(case.cache.block("K", b)[:, :n]), K[i]), ("K block", b)
        assert np.array_equal(_token_major_bits(case.cache.block("V", b)[:, :n]), V[i]), ("V block", b)
        maxv = max(maxv, float(np.abs(f64(V[i])).max()))
    return want, maxv


def _oracle_group_quant(case: FullCase, group, q, k_new, v_new):
    cfg, four = case.cfg, case.kv == "int4"
    quantise = O.quantize_rows_u4 if four else O.quantize_rows_i8
    append = O.kvq4_append if four else O.kvq_append
    decode = O.rpartq4_decode if four else O.rpartq_decode
    rb = cfg.d // 2 if four else cfg.d

    def one(b):
        L = case.lens[b]
        st = {}
        for which in ("K", "V"):
            codes = np.zeros((L + 1, cfg.H, rb), dtype=np.uint8)
            par = np.zeros((L + 1, cfg.H, 2) if four else (L + 1, cfg.H), dtype=np.float32)
            if L:
                codes[:L], par[:L] = quantise(host_rows[(b, which)])
            st[which] = (codes, par)
        lens = np.asarray([L], dtype=np.int32)
        append([st["K"][0]], [st["K"][1]], [st["V"][0]], [st["V"][1]], lens, k_new[b:b + 1], v_new[b:b + 1])
        want, _ = decode([st["K"][0]], [st["K"][1]], [st["V"][0]], [st["V"][1]], lens, q[b:b + 1])
        vc, vp = st["V"]
        if four:
            deq = O.unpack_u4(vc).astype(np.float64) * vp[..., 0:1] + vp[..., 1:2]
        else:
            deq = (vc.astype(np.float64) - 128.0) * vp[..., None]
        return st, want[0], float(np.abs(deq).max())

    # the generator runs on the device; everything after the host copy is the oracle's
    host_rows = {}
    for b in group:
        for which in ("K", "V"):
            if case.lens[b]:
                host_rows[(b, which)] = _token_major_bits(
                    W.gen_cache_block(cfg, which, b, case.lens[b], case.seed, "cuda"))
    with ThreadPoolExecutor(THREADS) as pool:
        res = list(pool.map(one, group))
    want = np.stack([r[1] for r in res])
    maxv = max(r[2] for r in res)
    for b, (st, _, _) in zip(group, res):
        n = case.lens[b] + 1
        for which in ("K", "V"):
            assert np.array_equal(_token_major(case.cache.codes(which, b)[:, :n]), st[which][0]), (which, "codes", b)
            assert np.array_equal(_token_major(case.cache.scales(which, b)[:, :n]), st[which][1]), (which, "parameters", b)
    return want, maxv


def check_full_config(name: str, kv: str, n_sample: Optional[int] = None, group_tokens: int = 60000):
    """Run the step at full size and put `n_sample` length-stratified sequences (default: every
    sequence) through the oracle.  Returns (max|err|, max|V|, sequences compared)."""
    t0 = time.time()
    case = FullCase(name, kv)
    cfg = case.cfg
    print(f"{name}/{kv}: built cache for {case.n_tok} tokens in {time.time() - t0:.1f} s", flush=True)
    case.step()
    batch = stratified(case.lens, cfg.B if n_sample is None else n_sample)
    q, k_new, v_new = bits(case.q), bits(case.k_new), bits(case.v_new)
    got = case.out.cpu().double().numpy()
    # every sequence, cheap: the appended rows hold the step's k/v (fp16: the same bits)
    if kv == "fp16":
        for b, L in enumerate(case.lens):
            assert torch.equal(case.cache.block("K", b)[:, L].view(torch.int16), case.k_new[b].view(torch.int16))
            assert torch.equal(case.cache.block("V", b)[:, L].view(torch.int16), case.v_new[b].view(torch.int16))
    err, maxv, done, group, tok = 0.0, 0.0, 0, [], 0
    t1 = time.time()
    for i, b in enumerate(batch):
        group.append(b)
        tok += case.lens[b] + 1
        if tok >= group_tokens or i == len(batch) - 1:
            f = _oracle_group_fp16 if kv == "fp16" else _oracle_group_quant
            want, mv = f(case, group, q, k_new, v_new)
            err = max(err, float(np.abs(got[group] - want).max()))
            maxv = max(maxv, mv)
            done += len(group)
            group, tok = [], 0
            if time.time() - t1 > 20:
                print(f"{name}/{kv}: {done}/{len(batch)} sequences through the oracle, max|err| so far {err:.3e}",
                      flush=True)
                t1 = time.time()
    print(f"{name}/{kv}: {done} of {cfg.B} sequences element by element: max|err|={err:.3e} "
          f"bound={TOL * maxv:.3e} (max|V|={maxv:.2f}) plan={case.plan} total {time.time() - t0:.1f} s", flush=True)
    assert err <= TOL * maxv, f"max|err| {err:.3e} > {TOL} * max|V| ({maxv:.3f})"
    return err, maxv, done
