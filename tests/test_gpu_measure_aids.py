"""The two measurement aids of the C ABI (the pure-read probe and the pattern fill) and the
pattern-filled bench path that the counter runs use."""
import numpy as np
import pytest
import torch

from paper_2403_11421_amd import rpart

pytestmark = pytest.mark.gpu


def test_fill_pattern_is_seeded_finite_and_stays_inside_the_buffer():
    n = 1 << 16
    buf = torch.zeros(n + 64, dtype=torch.int32, device="cuda")
    body = buf[32: 32 + n]
    rpart.fd_fill_pattern(body, 7)
    torch.cuda.synchronize()
    a = body.cpu().numpy().copy()
    assert not buf[:32].any() and not buf[32 + n:].any()            # guard words untouched
    rpart.fd_fill_pattern(body, 7)
    torch.cuda.synchronize()
    assert np.array_equal(body.cpu().numpy(), a)                      # same seed, same bits
    rpart.fd_fill_pattern(body, 8)
    torch.cuda.synchronize()
    b = body.cpu().numpy()
    assert (a != b).mean() > 0.99
    h = np.abs(a.view(np.float16).astype(np.float64))
    assert np.isfinite(h).all() and h.min() >= 0.25 and h.max() < 1.0
    assert np.isfinite(a.view(np.float32)).all()
    signs = (a.view(np.uint16) >> 15).mean()
    assert 0.45 < signs < 0.55 and len(np.unique(a)) > 0.99 * n
    with pytest.raises(rpart.FdError):
        rpart.fd_fill_pattern(buf.view(torch.uint8)[1:5], 1)          # misaligned
    with pytest.raises(rpart.FdError):
        rpart.fd_fill_pattern(buf.view(torch.uint8)[:6], 1)           # not whole words


def test_read_probe_reports_what_it_reads_and_writes_nothing_else():
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    per_pass = 2 * cus * 256 * 8 * 16                                  # two workgroups per CU, 32 KiB each
    buf = torch.ones(3 * per_pass + 4096, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    n = rpart.fd_hbm_read_probe(buf, sink)
    torch.cuda.synchronize()
    assert n == 3 * per_pass and bool((buf == 1).all())
    with pytest.raises(rpart.FdError):
        rpart.fd_hbm_read_probe(buf[: per_pass - 16], sink)           # not even one pass
    with pytest.raises(rpart.FdError):
        rpart.fd_hbm_read_probe(buf[1:], sink)                        # misaligned


def test_pattern_filled_bench_case_runs_a_step_with_finite_outputs():
    """bench.py --fill pattern: slabs and vectors filled by the library, small arrays copied from
    the host; the step must run clean on such a cache in every format."""
    import bench
    from paper_2403_11421_amd import workloads as W
    cfg = W.RPartConfig("pat", 6, 4, 128, "const", 0, 0)
    lens = [0, 1, 130, 700, 64, 2049]
    for kv in ("fp16", "int8", "int4"):
        cache, vec = bench.build_case(cfg, lens, 11, 0, kv=kv, fill="pattern")
        out = torch.full((cfg.B, cfg.H, cfg.d), float("nan"), dtype=torch.float16, device="cuda")
        ws = cache.workspace(sum(lens) + cfg.B)
        step = rpart.fd_rpartq_step if kv != "fp16" else rpart.fd_rpart_step
        step(cache.desc, vec["q"], vec["k_new"], vec["v_new"], out, ws)
        torch.cuda.synchronize()
        assert rpart.fd_last_device_status(cache.desc, ws) == 0
        assert cache.seq_lens.cpu().tolist() == [L + 1 for L in lens]
        # a convex combination of cached values (below 1 in magnitude, or tiny for the quantised
        # formats' pattern parameters) and the appended row
        bound = 1.01 * max(1.0, float(vec["v_new"].float().abs().max()))
        finite, biggest = bool(torch.isfinite(out.float()).all()), float(out.float().abs().max())
        assert finite and biggest <= bound
