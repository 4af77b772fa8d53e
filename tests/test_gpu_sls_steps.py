"""Multi-step R-worker loop under the load-stabilising schedule: every step's output, cache
contents and lengths are checked against the oracle, and the cached lengths follow the
scheduler's loads (FastDecode Section 4.1 + 4.2)."""
import numpy as np
import pytest
import torch

from oracle import rpart_oracle as O
from oracle import sls_oracle as SO
from paper_2403_11421_amd import sls_run
from tests.util import bits, f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind,B,S,F", [("sls", 6, 6, 2), ("batch", 6, 6, 2), ("sls", 8, 12, 3)])
def test_every_step_matches_the_oracle(kind, B, S, F):
    H, d = 3, 128
    n_steps = 3 * S + 1
    M = B * F // S if kind == "sls" else B
    period = F if kind == "sls" else S
    n_groups = B // M
    host = {"K": [np.zeros((S, H, d), np.uint16) for _ in range(B)],
            "V": [np.zeros((S, H, d), np.uint16) for _ in range(B)],
            "lens": np.zeros(B, np.int32)}
    starts = SO.sls_starts(M, F, n_steps) if kind == "sls" else SO.large_batch_starts(B, S, n_steps)
    want_loads = SO.step_loads(starts, S, n_steps)
    seen = []

    def on_step(step, cache, q, k_new, v_new, out, n_active):
        if step % period == 0:                              # the oracle side drops the same slots
            g = (step // period) % n_groups
            host["lens"][g * M:(g + 1) * M] = 0
        act = list(range(n_active))
        K = [host["K"][b] for b in act]
        V = [host["V"][b] for b in act]
        lens = host["lens"][:n_active].copy()
        O.kv_append(K, V, lens, bits(k_new.cpu()[:n_active]), bits(v_new.cpu()[:n_active]))
        host["lens"][:n_active] = lens
        want, _, _ = O.rpart_decode(K, V, lens, bits(q.cpu()[:n_active]))
        got_lens = cache.seq_lens.cpu().numpy()
        assert np.array_equal(got_lens[:n_active], lens)
        assert int(lens.sum()) == want_loads[step]
        for b in act:                                       # live rows bit-exact
            L = int(lens[b])
            assert np.array_equal(bits(cache.block("K", b)[:, :L].permute(1, 0, 2)), K[b][:L])
            assert np.array_equal(bits(cache.block("V", b)[:, :L].permute(1, 0, 2)), V[b][:L])
        maxv = max(float(np.abs(f64(V[b][:int(lens[b])])).max()) for b in act)
        err = float(np.abs(out.cpu()[:n_active].double().numpy() - want).max())
        assert err <= 2e-3 * maxv
        seen.append(step)

    res = sls_run.run_schedule(kind, B, S, F, n_steps, H=H, d=d, timed=False, on_step=on_step)
    assert seen == list(range(n_steps)) and res["loads"] == want_loads


@pytest.mark.parametrize("kv", ["int8", "int4"])
def test_every_step_matches_the_oracle_on_quantised_caches(kv):
    """The same loop over a quantised cache (Section 5.2 with Section 4.2): per step, code bytes,
    row parameters and lengths bit-exact, output within tolerance of the oracle's own
    append-and-attend on host copies."""
    kind, B, S, F, H, d = "sls", 8, 12, 3, 3, 128
    n_steps = 3 * S + 1
    M = B * F // S
    n_groups = B // M
    four = kv == "int4"
    host = {"Kc": [np.zeros((S, H, d // 2 if four else d), np.uint8) for _ in range(B)],
            "Vc": [np.zeros((S, H, d // 2 if four else d), np.uint8) for _ in range(B)],
            "Kp": [np.zeros((S, H, 2) if four else (S, H), np.float32) for _ in range(B)],
            "Vp": [np.zeros((S, H, 2) if four else (S, H), np.float32) for _ in range(B)],
            "lens": np.zeros(B, np.int32)}
    append = O.kvq4_append if four else O.kvq_append
    decode = O.rpartq4_decode if four else O.rpartq_decode
    want_loads = SO.step_loads(SO.sls_starts(M, F, n_steps), S, n_steps)
    seen = []

    def tm(t):
        return np.ascontiguousarray(t.permute(1, 0, *range(2, t.dim())).cpu().numpy())

    def dequant(c, p):
        if four:
            return O.unpack_u4(c).astype(np.float64) * p[..., 0:1] + p[..., 1:2]
        return (c.astype(np.float64) - 128) * p[..., None]

    def on_step(step, cache, q, k_new, v_new, out, n_active):
        if step % F == 0:
            g = (step // F) % n_groups
            host["lens"][g * M:(g + 1) * M] = 0
        act = list(range(n_active))
        sel = [[host[k][b] for b in act] for k in ("Kc", "Kp", "Vc", "Vp")]
        lens = host["lens"][:n_active].copy()
        append(sel[0], sel[1], sel[2], sel[3], lens, bits(k_new.cpu()[:n_active]), bits(v_new.cpu()[:n_active]))
        host["lens"][:n_active] = lens
        want, _ = decode(sel[0], sel[1], sel[2], sel[3], lens, bits(q.cpu()[:n_active]))
        assert np.array_equal(cache.seq_lens.cpu().numpy()[:n_active], lens)
        assert int(lens.sum()) == want_loads[step]
        maxv = 0.0
        for b in act:
            L = int(lens[b])
            assert np.array_equal(tm(cache.codes("K", b))[:L], host["Kc"][b][:L])
            assert np.array_equal(tm(cache.scales("K", b))[:L], host["Kp"][b][:L])
            assert np.array_equal(tm(cache.codes("V", b))[:L], host["Vc"][b][:L])
            assert np.array_equal(tm(cache.scales("V", b))[:L], host["Vp"][b][:L])
            maxv = max(maxv, float(np.abs(dequant(host["Vc"][b][:L], host["Vp"][b][:L])).max()))
        err = float(np.abs(out.cpu()[:n_active].double().numpy() - want).max())
        assert err <= 2e-3 * maxv
        seen.append(step)

    res = sls_run.run_schedule(kind, B, S, F, n_steps, H=H, d=d, timed=False, on_step=on_step, kv=kv)
    assert seen == list(range(n_steps)) and res["loads"] == want_loads and res["kv"] == kv


@pytest.mark.parametrize("frac", [None, 0.7])
def test_load_controlled_loop_matches_the_oracle_and_respects_the_limit(frac):
    """Micro-batches admitted by Algorithm 1 (free slots in between, released and reused): every
    step's output and lengths against the oracle, and the total cached length never above W_lim."""
    from paper_2403_11421_amd import rpart, sched
    B, S, F, H, d = 8, 12, 3, 3, 128
    M = B * F // S
    peak = sched.sls_peak_load(M, F, S)
    W_lim = None if frac is None else int(frac * peak)
    n_steps = 4 * S
    hist = {}                                                # slot -> list of (k bits, v bits)
    seen = []

    def on_step(step, cache, q, k_new, v_new, out, live):
        lens = cache.seq_lens.cpu().tolist()
        got = out.cpu().double().numpy()
        kb, vb, qb = bits(k_new), bits(v_new), bits(q)
        for s in range(B):
            if s not in live:
                assert lens[s] == rpart.FD_SLOT_FREE and np.all(got[s] == 0)
                hist.pop(s, None)
                continue
            if lens[s] == 1:
                hist[s] = []                                 # the slot was restarted this step
            hist[s].append((kb[s], vb[s]))
            K = np.stack([k for k, _ in hist[s]])
            V = np.stack([v for _, v in hist[s]])
            assert lens[s] == len(K)
            want, _, _ = O.rpart_decode([K], [V], np.array([len(K)], np.int32), qb[s:s + 1])
            assert np.abs(got[s] - want[0]).max() <= 2e-3 * float(np.abs(f64(V)).max())
        seen.append(sum(l for l in lens if l > 0))

    res = sls_run.run_schedule("control", B, S, F, n_steps, H=H, d=d, timed=False, on_step=on_step,
                               W_lim=W_lim)
    limit = res["W_lim"]
    assert seen == res["loads"] and max(seen) <= limit
    assert seen == SO.step_loads([(t, M) for t in res["starts"]], S, n_steps)
    if frac is None:
        assert res["starts"] == list(range(0, n_steps, F))   # nothing held back
    else:
        assert res["starts"] != list(range(0, n_steps, F))[:len(res["starts"])]
