"""Bulk row store (prompt ingestion), the device status calls, and what the plan check refuses."""
import numpy as np
import pytest
import torch

from oracle import rpart_oracle as O
from paper_2403_11421_amd import rpart, workloads as W
from paper_2403_11421_amd.kvcache import KVCache, KVCacheQ
from tests.gpu_util import DeviceCase, check_step
from tests.util import bits, half_bits

pytestmark = pytest.mark.gpu


def _special_rows(H, n, d, seed):
    """fp16 [H, n, d] with ordinary rows and the rows a quantiser can get wrong."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((H, n, d))
    x[0, 0] = 0.0                                   # all-zero row
    x[0, 1 % n] = 3.25                              # constant row
    x[1 % H, 0] = np.arange(d) * (1.0 / 128)        # exact grid
    x[1 % H, 1 % n] = np.where(np.arange(d) % 2 == 0, 127.0, 63.5)   # ties at .5
    x[2 % H, 0] = rng.standard_normal(d) * 6e-6     # fp16 subnormals
    b = half_bits(x)
    b[2 % H, 1 % n, 5] = 0x8000                     # -0
    return torch.from_numpy(b.view(np.int16).copy()).view(torch.float16).cuda()


@pytest.mark.parametrize("d", [64, 128])
def test_fp16_store_rows_copies_bits_and_leaves_the_rest_alone(d):
    H, caps = 3, [40, 9]
    cache = KVCache(2, H, d, caps)
    cache.k.fill_(1.5)
    cache.v.fill_(-2.5)
    k_rows, v_rows = _special_rows(H, 7, d, 1), _special_rows(H, 7, d, 2)
    rpart.fd_kv_store_rows(cache.desc, 0, 11, k_rows, v_rows)
    rpart.fd_kv_store_rows(cache.desc, 1, 2, None, v_rows)            # V side only
    torch.cuda.synchronize()
    assert rpart.fd_read_status(cache.desc) == 0
    assert torch.equal(cache.block("K", 0)[:, 11:18].view(torch.int16), k_rows.view(torch.int16))
    assert torch.equal(cache.block("V", 0)[:, 11:18].view(torch.int16), v_rows.view(torch.int16))
    assert bool((cache.block("K", 0)[:, :11] == 1.5).all()) and bool((cache.block("K", 0)[:, 18:] == 1.5).all())
    assert bool((cache.block("V", 0)[:, :11] == -2.5).all()) and bool((cache.block("V", 0)[:, 18:] == -2.5).all())
    assert bool((cache.block("K", 1) == 1.5).all())
    assert torch.equal(cache.block("V", 1)[:, 2:9].view(torch.int16), v_rows.view(torch.int16))
    assert cache.seq_lens.cpu().tolist() == [0, 0]                     # lengths untouched
    # set_len: the prompt's rows and its length in one call
    rpart.fd_kv_store_rows(cache.desc, 0, 0, k_rows, v_rows, set_len=True)
    torch.cuda.synchronize()
    assert cache.seq_lens.cpu().tolist() == [7, 0]
    # beyond the capacity: nothing is written, the error is reported
    before = cache.k.clone()
    rpart.fd_kv_store_rows(cache.desc, 1, 3, k_rows, v_rows, set_len=True)
    torch.cuda.synchronize()
    assert rpart.fd_last_device_status(cache.desc, cache.workspace(8)) == rpart.FD_ST_CAPACITY
    assert torch.equal(cache.k, before) and cache.seq_lens.cpu().tolist() == [7, 0]
    for bad in ((2, 0), (-1, 0), (0, -1)):
        with pytest.raises(rpart.FdError):
            rpart.fd_kv_store_rows(cache.desc, bad[0], bad[1], k_rows, v_rows)


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("nbits", [8, 4])
def test_quantised_store_rows_matches_the_oracle_quantiser(nbits, d):
    H, n = 5, 19
    cache = KVCacheQ(3, H, d, [64, 30, 19], bits=nbits)
    quantise = O.quantize_rows_i8 if nbits == 8 else O.quantize_rows_u4
    k_rows, v_rows = _special_rows(H, n, d, 3), _special_rows(H, n, d, 4)
    rpart.fd_kv_store_rows(cache.desc, 1, 4, k_rows, v_rows, set_len=True)
    rpart.fd_kv_store_rows(cache.desc, 2, 0, k_rows, None)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(cache.desc) == 0
    assert cache.seq_lens.cpu().tolist() == [0, 23, 0]
    kc, kp = quantise(bits(k_rows))
    vc, vp = quantise(bits(v_rows))
    assert np.array_equal(cache.codes("K", 1)[:, 4:23].cpu().numpy(), kc)
    assert np.array_equal(cache.scales("K", 1)[:, 4:23].cpu().numpy(), kp)
    assert np.array_equal(cache.codes("V", 1)[:, 4:23].cpu().numpy(), vc)
    assert np.array_equal(cache.scales("V", 1)[:, 4:23].cpu().numpy(), vp)
    assert np.array_equal(cache.codes("K", 2).cpu().numpy(), kc)
    blank = 128 if nbits == 8 else 0
    assert bool((cache.codes("V", 2) == blank).all()) and bool((cache.codes("K", 0) == blank).all())
    assert bool((cache.codes("K", 1)[:, :4] == blank).all()) and bool((cache.scales("K", 1)[:, 23:] == 0).all())
    # one row too many for sequence 2
    rpart.fd_kv_store_rows(cache.desc, 2, 1, k_rows, v_rows)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(cache.desc, clear=True) == rpart.FD_ST_CAPACITY
    assert np.array_equal(cache.codes("K", 2).cpu().numpy(), kc)


def test_prompt_store_then_decode_steps_match_the_oracle():
    """A prompt ingested in one call, then ordinary steps: what Section 4.1's worker does."""
    cfg = W.RPartConfig("prompt", 3, 4, 128, "const", 0, 0)
    lens = [257, 0, 33]
    case = DeviceCase(cfg, [0, 0, 0], seed=5, extra_cap=300)
    for b, L in enumerate(lens):
        if L:
            rpart.fd_kv_store_rows(case.cache.desc, b, 0, W.gen_cache_block(cfg, "K", b, L, 5, "cuda"),
                                   W.gen_cache_block(cfg, "V", b, L, 5, "cuda"), set_len=True)
    torch.cuda.synchronize()
    assert case.cache.seq_lens.cpu().tolist() == lens
    check_step(case)
    check_step(case, use_step=True)
    assert case.cache.seq_lens.cpu().tolist() == [L + 2 for L in lens]


def test_status_take_clears_atomically_and_read_clears_only_what_it_reported():
    cfg = W.RPartConfig("status", 2, 2, 128, "const", 0, 0)
    case = DeviceCase(cfg, [3, 4], seed=9, extra_cap=0)                # both caches are full
    rpart.fd_kv_append(case.cache.desc, case.k_new, case.v_new)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(case.cache.desc) == rpart.FD_ST_CAPACITY          # plain read: sticky
    assert rpart.fd_read_status(case.cache.desc) == rpart.FD_ST_CAPACITY
    case.cache.status.fill_(rpart.FD_ST_CAPACITY | rpart.FD_ST_BADLEN)
    assert rpart.fd_last_device_status(case.cache.desc, case.ws) == rpart.FD_ST_CAPACITY | rpart.FD_ST_BADLEN
    assert rpart.fd_last_device_status(case.cache.desc, case.ws) == 0              # taken
    assert int(case.cache.status.item()) == 0
    # taking the status borrows a header word of the workspace and leaves a plan in it usable
    case2 = DeviceCase(cfg, [100, 700], seed=10)
    rpart.fd_kv_append(case2.cache.desc, case2.k_new, case2.v_new)
    rpart.fd_rpart_plan(case2.cache.desc, case2.ws)
    assert rpart.fd_last_device_status(case2.cache.desc, case2.ws) == 0
    rpart.fd_rpart_partial(case2.cache.desc, case2.q, case2.out, case2.ws)
    rpart.fd_rpart_merge(case2.cache.desc, case2.out, case2.ws)
    torch.cuda.synchronize()
    assert rpart.fd_last_device_status(case2.cache.desc, case2.ws) == 0
    assert bool(torch.isfinite(case2.out.float()).all())
    with pytest.raises(rpart.FdError):
        rpart.fd_last_device_status(case2.cache.desc, case2.ws[1:])               # misaligned


def test_a_plan_made_for_another_cache_format_is_refused():
    """The quantised planner deals units to three workgroups per compute unit and cuts on another
    granule; the fp16 streaming kernel must not run such a plan (and the other way round)."""
    cfg = W.RPartConfig("xplan", 3, 2, 128, "const", 0, 0)
    lens = [100, 5, 700]
    case = DeviceCase(cfg, lens, seed=31)
    qcache = KVCacheQ(cfg.B, cfg.H, cfg.d, [L + 1 for L in lens], bits=8)
    qcache.set_lens(lens)
    rpart.fd_rpartq_plan(qcache.desc, case.ws)                # same B, H, d and workspace size
    case.out.fill_(7.0)
    rpart.fd_rpart_partial(case.cache.desc, case.q, case.out, case.ws)
    rpart.fd_rpart_merge(case.cache.desc, case.out, case.ws)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(case.cache.desc, clear=True) == rpart.FD_ST_PLAN
    assert bool((case.out == 7.0).all())
    rpart.fd_rpart_plan(case.cache.desc, case.ws)
    rpart.fd_rpartq_partial(qcache.desc, case.q, case.out, case.ws)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(qcache.desc, clear=True) == rpart.FD_ST_PLAN
    assert bool((case.out == 7.0).all())
    q4 = KVCacheQ(cfg.B, cfg.H, cfg.d, [L + 1 for L in lens], bits=4)
    q4.set_lens(lens)
    rpart.fd_rpartq_plan(qcache.desc, case.ws)                # 8-bit plan, 4-bit kernel
    rpart.fd_rpartq_partial(q4.desc, case.q, case.out, case.ws)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(q4.desc, clear=True) == rpart.FD_ST_PLAN
    check_step(case)                                           # the workspace is still good for a real step


def test_a_plan_made_from_longer_lengths_never_leaves_the_block():
    """Same shape, same workspace, but planned from a cache with longer sequences: the result is
    wrong, yet every token range is clamped to this cache's capacities (no access outside its
    blocks: the neighbouring guard regions stay untouched and nothing faults)."""
    cfg = W.RPartConfig("clamp", 2, 2, 128, "const", 0, 0)
    big = DeviceCase(cfg, [900, 1200], seed=1)
    small = DeviceCase(cfg, [30, 40], seed=2)
    ws = big.ws
    rpart.fd_rpart_plan(big.cache.desc, ws)
    rpart.fd_rpart_partial(small.cache.desc, small.q, small.out, ws)
    rpart.fd_rpart_merge(small.cache.desc, small.out, ws)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(small.cache.desc) == 0
    assert bool(torch.isfinite(small.out.float()).all())
    small.ws = small.cache.workspace(100)
    check_step(small)
