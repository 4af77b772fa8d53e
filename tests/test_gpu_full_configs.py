"""Full-size configs in the launch configuration bench.py times (library-chosen
chunking, workspace from fd_workspace_bytes for the step's token count).

The oracle checks sampled sequences (all heads) element by element; properties
that hold at any size are checked on every output: lengths, appended rows
bit-exact for all sequences, finiteness, and |out| <= max|V| (Eq. 3 is a convex
combination of value rows).
"""
import numpy as np
import pytest
import torch

from paper_2403_11421_amd import rpart, workloads as W
from tests.gpu_util import DeviceCase, check_step

pytestmark = pytest.mark.gpu


def _sample(lens, n=8):
    order = np.argsort(lens, kind="stable")
    picks = {int(order[0]), int(order[-1])}                    # shortest and longest
    for k in range(1, n - 1):
        picks.add(int(order[(k * (len(lens) - 1)) // (n - 1)]))
    return sorted(picks)


@pytest.mark.parametrize("name", ["c2_7b_uniform", "c3_7b_ragged", "c4_13b_geometric",
                                  "c5_capacity"])
def test_full_config_sampled_parity_and_global_properties(name):
    cfg = W.CONFIGS[name]
    lens = W.seq_lens(cfg)
    n_tok = W.total_tokens_after_append(lens)
    print(f"{name}: building {cfg.bytes_per_token() * n_tok / 1e9:.1f} GB of KV", flush=True)
    case = DeviceCase(cfg, lens, extra_cap=8)
    case.ws = case.cache.workspace(n_tok)                      # as bench.py sizes it
    batch = _sample(lens)
    print(f"{name}: step + oracle on sequences {batch} (lens {[lens[b] for b in batch]})", flush=True)
    err, maxv = check_step(case, batch=batch, nthreads=16)
    plan = rpart.fd_plan_info(case.ws)
    print(f"{name}: max|err|={err:.3e} max|V|={maxv:.2f} plan={plan}", flush=True)
    assert plan["total_tokens"] == n_tok

    # every sequence: length bumped by one, appended rows equal the new k/v bit for bit
    assert case.cache.seq_lens.cpu().tolist() == [L + 1 for L in lens]
    for b, L in enumerate(lens):
        assert torch.equal(case.cache.block("K", b)[:, L, :].view(torch.int16),
                           case.k_new[b].view(torch.int16))
        assert torch.equal(case.cache.block("V", b)[:, L, :].view(torch.int16),
                           case.v_new[b].view(torch.int16))
    # every output: finite and inside the convex hull bound
    out = case.out.float()
    assert bool(torch.isfinite(out).all())
    vmax = max(float(case.cache.v.abs().max()), float(case.v_new.abs().max()))
    assert float(out.abs().max()) <= vmax * (1 + 2e-3)
    # per-(b,h) bound on a strided subset of sequences (cheap, device side)
    for b in range(0, cfg.B, max(1, cfg.B // 64)):
        v = case.cache.block("V", b)[:, :lens[b] + 1, :].float()
        hi, lo = v.amax(dim=1), v.amin(dim=1)
        span = (hi - lo).clamp_min(1e-3)
        assert bool((out[b] <= hi + 2e-3 * span + 1e-3).all())
        assert bool((out[b] >= lo - 2e-3 * span - 1e-3).all())


def test_long_context_few_sequences():
    """Long-context decoding at small batch: one sequence of 131071 cached tokens (cut into 128
    chunks per head, laid out by the planner's whole workgroup and merged 64 chunk states at a
    time) and, in the same step, two of 40000 and 70001 and a short one; every sequence against
    the oracle, in the library's own chunking."""
    cfg = W.RPartConfig("long_context", 4, 8, 128, "const", 0, 0)
    lens = [131071, 40000, 70001, 300]
    n_tok = W.total_tokens_after_append(lens)
    case = DeviceCase(cfg, lens, extra_cap=8)
    case.ws = case.cache.workspace(n_tok)
    err, maxv = check_step(case, nthreads=16)
    plan = rpart.fd_plan_info(case.ws)
    print(f"long context: max|err|={err:.3e} max|V|={maxv:.2f} plan={plan}", flush=True)
    assert plan["total_tokens"] == n_tok and plan["items"] > 64
    assert case.cache.seq_lens.cpu().tolist() == [L + 1 for L in lens]
