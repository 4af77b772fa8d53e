"""fd_rpart_decode_noalloc (the entry point for callers that cannot allocate) against
fd_rpart_decode on the same inputs: two calls in a row on the library's built-in scratch array,
the second with a smaller batch, each compared with the workspace entry point's output and with
the oracle.  The array keeps the first call's plan and chunk states when the second call starts.
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle import rpart_oracle as O
from paper_2403_11421_amd import rpart, workloads as W
from tests.gpu_util import TOL, DeviceCase
from tests.util import f64


def _both(cfg, lens, chunk_tokens):
    case = DeviceCase(cfg, lens, extra_cap=2, chunk_tokens=chunk_tokens)
    rpart.fd_kv_append(case.cache.desc, case.k_new, case.v_new)
    rpart.fd_rpart_decode(case.cache.desc, case.q, case.out, case.ws)
    torch.cuda.synchronize()
    want_ws = case.out.clone()
    plan_ws = rpart.fd_plan_info(case.ws)
    got = torch.full_like(case.out, float("nan"))
    rpart.fd_rpart_decode_noalloc(case.cache.desc, case.q, got)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(case.cache.desc) == 0
    # oracle on what the device holds after the append
    ref = case.oracle_inputs()
    want, _, _ = O.rpart_decode(ref["K"], ref["V"], ref["seq_lens"], ref["q"], nthreads=8)
    maxv = max(float(np.abs(f64(v[:L])).max()) for v, L in zip(ref["V"], ref["seq_lens"]) if L)
    g = got.cpu().double().numpy()
    assert np.all(np.isfinite(g))
    err_ws = float(np.abs(g - want_ws.cpu().double().numpy()).max())
    err_or = float(np.abs(g - want).max())
    print(f"noalloc B={cfg.B} H={cfg.H} d={cfg.d} chunk={chunk_tokens}: |vs workspace entry|={err_ws:.3e} "
          f"|vs oracle|={err_or:.3e} bound={TOL * maxv:.3e} plan={plan_ws}", flush=True)
    assert err_ws <= TOL * maxv and err_or <= TOL * maxv
    return got, want_ws, plan_ws


@pytest.mark.gpu
def test_noalloc_matches_workspace_entry_point_two_calls_second_smaller():
    # first call: ragged batch with an empty sequence, forced 64-token chunks, so that the
    # scratch array really holds chunk states of split sequences and the merge reads them
    cfg1 = W.RPartConfig("noalloc_a", 7, 8, 128, "const", 0, 0)
    got1, ws1, plan1 = _both(cfg1, [0, 1, 63, 64, 700, 1500, 3001], 64)
    assert plan1["items"] > cfg1.B
    # the forced chunk length makes both entry points cut the sequences alike: same arithmetic
    # in the same order, so the results are the same bits
    assert torch.equal(got1.view(torch.int16), ws1.view(torch.int16))
    # second call, smaller in every dimension, other head size, library-chosen chunking
    cfg2 = W.RPartConfig("noalloc_b", 3, 4, 64, "const", 0, 0)
    got2, ws2, _ = _both(cfg2, [300, 5, 129], 0)
    assert torch.equal(got2.view(torch.int16), ws2.view(torch.int16))
    # and the first shape again: nothing left behind by the smaller call disturbs it
    got3, ws3, _ = _both(cfg1, [0, 1, 63, 64, 700, 1500, 3001], 64)
    assert torch.equal(got3.view(torch.int16), ws3.view(torch.int16))
    assert torch.equal(got3.view(torch.int16), got1.view(torch.int16))


def test_noalloc_rejects_a_batch_beyond_the_scratch_array():
    lib = rpart.load()
    need = rpart.workspace_bytes(4096, 64, 128, 0)
    assert need > rpart.FD_NOALLOC_SCRATCH_BYTES
    # fake, aligned pointers: the size check comes before anything is dereferenced or enqueued
    d = rpart.fd_kv_desc(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 4096, 64, 128, 0)
    assert lib.fd_rpart_decode_noalloc(ctypes.byref(d), 0x7000, 0x8000, None) == rpart.FD_ETOOBIG
    assert "scratch" in rpart.strerror(rpart.FD_ETOOBIG)
    null = ctypes.POINTER(rpart.fd_kv_desc)()
    assert lib.fd_rpart_decode_noalloc(null, None, None, None) == rpart.FD_EINVAL
