"""Seeded random shapes through all three cache formats: batch sizes, head counts, both head
sizes, equal / ragged / few-long / partly-empty / tiny length mixes, forced and free chunking,
one-call steps and separate append + decode, each case checked whole against the oracle."""
import random

import pytest
import torch

from paper_2403_11421_amd import workloads as W
from tests import test_gpu_quant_parity as Q8
from tests.gpu_util import DeviceCase, check_step
from tests.test_gpu_quant4_parity import Q4Case, check_q4step

pytestmark = pytest.mark.gpu


def _draw(rng):
    B = rng.choice([1, 2, 3, 5, 8, 17, 40, 130])
    H = rng.choice([1, 2, 3, 5, 8])
    d = rng.choice([64, 128])
    kind = rng.choice(["equal", "ragged", "few_long", "with_empty", "tiny"])
    if kind == "equal":
        lens = [rng.choice([1, 7, 63, 64, 65, 127, 255, 256, 700, 2049])] * B
    elif kind == "ragged":
        lens = [rng.randint(0, rng.choice([20, 300, 3000])) for _ in range(B)]
    elif kind == "few_long":
        lens = [rng.randint(0, 50) for _ in range(B)]
        lens[rng.randrange(B)] = rng.randint(5000, 30000)
    elif kind == "with_empty":
        lens = [rng.choice([0, 0, rng.randint(1, 600)]) for _ in range(B)]
    else:
        lens = [rng.randint(0, 9) for _ in range(B)]
    return B, H, d, kind, lens, rng.choice([0, 0, 0, 64, 128, 320, 1024]), rng.random() < 0.6


@pytest.mark.parametrize("fmt,seed", [("fp16", 11), ("int8", 12), ("int4", 13)])
def test_random_shapes(fmt, seed):
    rng = random.Random(seed)
    for it in range(40):
        B, H, d, kind, lens, chunk, use_step = _draw(rng)
        cfg = W.RPartConfig("random", B, H, d, "const", 0, 0)
        print(f"{fmt} case {it}: B={B} H={H} d={d} {kind} chunk={chunk} step={use_step} lens[:6]={lens[:6]}", flush=True)
        if fmt == "fp16":
            check_step(DeviceCase(cfg, lens, seed=seed * 100 + it, chunk_tokens=chunk), use_step=use_step)
        elif fmt == "int4":
            check_q4step(Q4Case(cfg, lens, seed=seed * 100 + it, chunk_tokens=chunk), use_step=use_step)
        else:
            Q8.check_qstep(Q8.QCase(cfg, lens, seed=seed * 100 + it, chunk_tokens=chunk), use_step=use_step)
        torch.cuda.empty_cache()
