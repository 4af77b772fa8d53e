"""Full-size configs in the launch configuration bench.py times (staged calls, library-chosen
chunking, workspace from fd_workspace_bytes for the step's token count).

Configs 2, 3 and 4: EVERY sequence goes through the oracle, element by element (cache blocks
bit for bit, outputs within 2e-3 * max|V|).  Config 5 (2048 sequences, 52 GB): 256 sequences
spread evenly over the length ranks; for the rest the properties that hold at any size (lengths,
appended rows bit-exact, finite outputs).
"""
import pytest

from paper_2403_11421_amd import rpart, workloads as W
from tests.full_parity import check_full_config
from tests.gpu_util import DeviceCase, check_step

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,n_sample", [("c2_7b_uniform", None), ("c3_7b_ragged", None),
                                           ("c4_13b_geometric", None), ("c5_capacity", 256)])
def test_full_config_whole_batch_parity(name, n_sample):
    err, maxv, done = check_full_config(name, "fp16", n_sample)
    assert done == (W.CONFIGS[name].B if n_sample is None else n_sample)


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
