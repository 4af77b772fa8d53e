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
