"""Windowed KV-cache (sink tokens + the last `window` tokens in a bounded buffer) and slot
reuse (free slots, release, restart), through the C ABI, against the oracle.

Window: the oracle attends over the token set taken from the FULL history; the device keeps
only n_sink + window rows in ring order.  Outputs must agree to the usual bar, and every row
of the device cache must hold, bit for bit, the token the oracle's literal eviction simulation
puts there."""
import random

import numpy as np
import pytest
import torch

from oracle import rpart_oracle as O
from oracle import window_oracle as WO
from paper_2403_11421_amd import rpart, sched, workloads as W
from paper_2403_11421_amd.kvcache import KVCache, KVCacheQ
from tests.util import bits, f64

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _vec(cfg, which, step):
    return W.gen_vectors(cfg, which, seed=500 + step, device="cuda")


@pytest.mark.parametrize("n_sink,windows,steps", [
    (2, [5, 3, 8], 40),              # wraps many times, tiny tiles
    (4, [60, 130, 33], 300),         # crosses several wave loads and a ragged tail
    (0, [1, 2, 70], 150),            # no sinks; a window of a single token
])
def test_windowed_fp16_cache_every_step(n_sink, windows, steps):
    H, d = 2, 128
    B = len(windows)
    cfg = W.RPartConfig("win", B, H, d, "const", 0, 0)
    caps = [n_sink + w for w in windows]
    cache = KVCache(B, H, d, caps, n_sink=n_sink)
    ws = cache.workspace(sum(caps))
    out = torch.empty(B, H, d, dtype=torch.float16, device="cuda")
    K_hist = [np.zeros((steps, H, d), np.uint16) for _ in range(B)]
    V_hist = [np.zeros((steps, H, d), np.uint16) for _ in range(B)]
    sims = [WO.BoundedCache(n_sink, w) for w in windows]
    for t in range(steps):
        q, kn, vn = _vec(cfg, "q", t), _vec(cfg, "k_new", t), _vec(cfg, "v_new", t)
        rpart.fd_rpart_step(cache.desc, q, kn, vn, out, ws)
        torch.cuda.synchronize()
        kb, vb = bits(kn), bits(vn)
        for b in range(B):
            K_hist[b][t], V_hist[b][t] = kb[b], vb[b]
            sims[b].append()
        # per-sequence windows differ, so the oracle is called once per sequence
        got = out.cpu().double().numpy()
        for b in range(B):
            wb = WO.rpart_decode_window([K_hist[b]], [V_hist[b]], [t + 1], bits(q)[b:b + 1],
                                        n_sink, windows[b])[0]
            S = WO.token_set(t + 1, n_sink, windows[b])
            maxv = float(np.abs(f64(V_hist[b][S])).max())
            assert np.abs(got[b] - wb).max() <= TOL * maxv, (t, b)
            rows = np.asarray(sims[b].rows)
            dev_k = bits(cache.block("K", b).permute(1, 0, 2))[:len(rows)]
            dev_v = bits(cache.block("V", b).permute(1, 0, 2))[:len(rows)]
            assert np.array_equal(dev_k, K_hist[b][rows]) and np.array_equal(dev_v, V_hist[b][rows])
        assert cache.seq_lens.cpu().tolist() == [min(t + 1, c) for c in caps]
        assert cache.seq_seen.cpu().tolist() == [t + 1] * B
    assert rpart.fd_read_status(cache.desc) == 0


@pytest.mark.parametrize("nbits", [8, 4])
def test_windowed_quantised_cache_every_step(nbits):
    H, d, n_sink, windows, steps = 2, 128, 3, [6, 70], 120
    B = len(windows)
    cfg = W.RPartConfig("winq", B, H, d, "const", 0, 0)
    caps = [n_sink + w for w in windows]
    cache = KVCacheQ(B, H, d, caps, n_sink=n_sink, bits=nbits)
    ws = cache.workspace(sum(caps))
    out = torch.empty(B, H, d, dtype=torch.float16, device="cuda")
    cshape = (steps, H, d) if nbits == 8 else (steps, H, d // 2)       # codes; 4 bit: two per byte
    pshape = (steps, H) if nbits == 8 else (steps, H, 2)               # scale; 4 bit: (scale, zero)
    hist = [dict(Kc=np.zeros(cshape, np.uint8), Ks=np.zeros(pshape, np.float32),
                 Vc=np.zeros(cshape, np.uint8), Vs=np.zeros(pshape, np.float32))
            for _ in range(B)]
    quantise = O.quantize_rows_i8 if nbits == 8 else O.quantize_rows_u4
    decode = O.rpartq_decode if nbits == 8 else O.rpartq4_decode

    def dequant(c, p):
        if nbits == 8:
            return (c.astype(np.float64) - 128) * p[:, :, None]
        return O.unpack_u4(c).astype(np.float64) * p[:, :, 0:1] + p[:, :, 1:2]
    sims = [WO.BoundedCache(n_sink, w) for w in windows]

    def tm(t):
        return np.ascontiguousarray(t.permute(1, 0, *range(2, t.dim())).cpu().numpy())

    for t in range(steps):
        q, kn, vn = _vec(cfg, "q", t), _vec(cfg, "k_new", t), _vec(cfg, "v_new", t)
        rpart.fd_rpartq_step(cache.desc, q, kn, vn, out, ws)
        torch.cuda.synchronize()
        kc, ks = quantise(bits(kn))                          # the oracle's quantiser on the inputs
        vc, vs = quantise(bits(vn))
        got = out.cpu().double().numpy()
        for b in range(B):
            h = hist[b]
            h["Kc"][t], h["Ks"][t], h["Vc"][t], h["Vs"][t] = kc[b], ks[b], vc[b], vs[b]
            sims[b].append()
            rows = np.asarray(sims[b].rows)
            for key, dev in (("Kc", cache.codes("K", b)), ("Ks", cache.scales("K", b)),
                             ("Vc", cache.codes("V", b)), ("Vs", cache.scales("V", b))):
                assert np.array_equal(tm(dev)[:len(rows)], h[key][rows]), (t, b, key)
            S = WO.token_set(t + 1, n_sink, windows[b])
            want, _ = decode([np.ascontiguousarray(h["Kc"][S])], [np.ascontiguousarray(h["Ks"][S])],
                             [np.ascontiguousarray(h["Vc"][S])], [np.ascontiguousarray(h["Vs"][S])],
                             np.array([len(S)], np.int32), bits(q)[b:b + 1])
            maxv = float(np.abs(dequant(h["Vc"][S], h["Vs"][S])).max())
            assert np.abs(got[b] - want[0]).max() <= TOL * maxv, (t, b)
    assert rpart.fd_read_status(cache.desc) == 0


def test_window_state_errors_are_reported_and_skip_the_append():
    H, d = 2, 128
    cfg = W.RPartConfig("winerr", 2, H, d, "const", 0, 0)
    cache = KVCache(2, H, d, [4, 4], n_sink=4)               # no window row left
    rpart.fd_kv_append(cache.desc, _vec(cfg, "k_new", 0), _vec(cfg, "v_new", 0))
    torch.cuda.synchronize()
    assert rpart.fd_read_status(cache.desc, clear=True) == rpart.FD_ST_WINDOW
    assert cache.seq_lens.cpu().tolist() == [0, 0] and cache.seq_seen.cpu().tolist() == [0, 0]
    cache = KVCache(2, H, d, [6, 6], n_sink=1)
    cache.seq_lens.copy_(torch.tensor([3, 0], dtype=torch.int32))       # disagrees with seq_seen = 0
    rpart.fd_kv_append(cache.desc, _vec(cfg, "k_new", 0), _vec(cfg, "v_new", 0))
    torch.cuda.synchronize()
    assert rpart.fd_read_status(cache.desc) == rpart.FD_ST_WINDOW
    assert cache.seq_lens.cpu().tolist() == [3, 1] and cache.seq_seen.cpu().tolist() == [0, 1]


@pytest.mark.parametrize("kv", ["fp16", "int8", "int4"])
def test_slots_are_released_and_reused(kv):
    """Sequences of random lengths come and go; a host free list hands out slots, the device
    side is fd_kv_release / fd_kv_reset.  Every step is checked against the oracle."""
    rng = random.Random(11)
    B, H, d, cap, steps = 6, 2, 128, 48, 90
    cfg = W.RPartConfig("slots", B, H, d, "const", 0, 0)
    cache = KVCache(B, H, d, [cap] * B) if kv == "fp16" else \
        KVCacheQ(B, H, d, [cap] * B, bits=4 if kv == "int4" else 8)
    ws = cache.workspace(B * cap)
    out = torch.empty(B, H, d, dtype=torch.float16, device="cuda")
    slots = sched.Slots(B)
    rpart.fd_kv_release(cache.desc)                          # all slots start free
    live = {}                                                # slot -> [remaining steps, history]
    reused = 0
    ever = set()

    def ids(xs):
        return torch.tensor(sorted(xs), dtype=torch.int32, device="cuda")

    for t in range(steps):
        done = [s for s, v in live.items() if v[0] == 0]
        if done:
            rpart.fd_kv_release(cache.desc, ids(done))
            for s in done:
                slots.release(s)
                del live[s]
        started = []
        while len(live) < B and rng.random() < 0.6:
            s = slots.acquire()
            assert s >= 0 and s not in live
            reused += s in ever
            ever.add(s)
            live[s] = [rng.randint(1, cap), []]
            started.append(s)
        if started:
            (rpart.fd_kv_reset if kv == "fp16" else rpart.fd_kvq_reset)(cache.desc, ids(started))
        q, kn, vn = _vec(cfg, "q", t), _vec(cfg, "k_new", t), _vec(cfg, "v_new", t)
        out.fill_(float("nan"))
        (rpart.fd_rpart_step if kv == "fp16" else rpart.fd_rpartq_step)(cache.desc, q, kn, vn, out, ws)
        torch.cuda.synchronize()
        got = out.cpu().double().numpy()
        lens = cache.seq_lens.cpu().tolist()
        kb, vb, qb = bits(kn), bits(vn), bits(q)
        for s in range(B):
            if s not in live:
                assert lens[s] == rpart.FD_SLOT_FREE and np.all(got[s] == 0)
                continue
            live[s][0] -= 1
            live[s][1].append((kb[s], vb[s]))
            Kh = np.stack([k for k, _ in live[s][1]])
            Vh = np.stack([v for _, v in live[s][1]])
            assert lens[s] == len(Kh)
            if kv == "fp16":
                want, _, _ = O.rpart_decode([Kh], [Vh], np.array([len(Kh)], np.int32), qb[s:s + 1])
                maxv = float(np.abs(f64(Vh)).max())
            elif kv == "int8":
                kc, ks = O.quantize_rows_i8(Kh)
                vc, vs = O.quantize_rows_i8(Vh)
                want, _ = O.rpartq_decode([kc], [ks], [vc], [vs], np.array([len(Kh)], np.int32), qb[s:s + 1])
                maxv = float(np.abs((vc.astype(np.float64) - 128) * vs[:, :, None]).max())
            else:
                kc, ks = O.quantize_rows_u4(Kh)
                vc, vs = O.quantize_rows_u4(Vh)
                want, _ = O.rpartq4_decode([kc], [ks], [vc], [vs], np.array([len(Kh)], np.int32), qb[s:s + 1])
                maxv = float(np.abs(O.unpack_u4(vc).astype(np.float64) * vs[:, :, 0:1] + vs[:, :, 1:2]).max())
            assert np.abs(got[s] - want[0]).max() <= TOL * maxv, (t, s)
    assert reused > 5 and rpart.fd_read_status(cache.desc) == 0
    assert slots.in_use() == len(live)
