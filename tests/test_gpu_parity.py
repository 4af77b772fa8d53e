"""HIP path vs fp64 oracle through the C ABI (needs an MI355X).

Bar: seq_lens and cache contents bit-exact; out within 2e-3 * max|V|.
"""
import math

import numpy as np
import pytest
import torch

from oracle import rpart_oracle as O
from paper_2403_11421_amd import rpart, workloads as W
from tests.gpu_util import TOL, DeviceCase, check_step
from tests.util import bits, f64

pytestmark = pytest.mark.gpu


def _cfg(name, B, H, d, **kw):
    return W.RPartConfig(name, B, H, d, "const", 0, 0, **kw)


def test_c1_tiny_config():
    cfg = W.CONFIGS["c1_tiny"]
    case = DeviceCase(cfg, W.seq_lens(cfg))
    err, maxv = check_step(case)
    assert case.cache.seq_lens.cpu().tolist() == [129] * 4
    print(f"c1 max|err|={err:.2e} max|V|={maxv:.2f}")


EDGE_LENS = [0, 1, 2, 3, 4, 7, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 640,
             1000, 1023, 1024, 1025, 2500]


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("chunk", [0, 64, 128, 256, 1024, 4096])
def test_edge_lengths_all_chunk_sizes(d, chunk):
    cfg = _cfg("edges", len(EDGE_LENS), 3, d)
    case = DeviceCase(cfg, EDGE_LENS, seed=11 + d, chunk_tokens=chunk)
    check_step(case)
    info = rpart.fd_plan_info(case.ws)
    assert info["total_tokens"] == sum(EDGE_LENS) + len(EDGE_LENS)
    if chunk:
        granule = 32 if d == 128 else 64             # chunk boundaries: one wave load of rows
        T = -(-chunk // granule) * granule
        assert info["chunk_tokens"] == T
        assert info["items"] == sum(math.ceil((L + 1) / T) for L in EDGE_LENS)


@pytest.mark.parametrize("d", [128, 64])
def test_step_entry_point_and_many_heads(d):
    cfg = _cfg("step", 5, 40, d)
    case = DeviceCase(cfg, [300, 17, 2049, 64, 999], seed=5)
    check_step(case, use_step=True)


def test_peaked_keys_small():
    cfg = W.RPartConfig("peaked", 12, 8, 128, "uniform", 1, 1500, peaked_keys=True)
    case = DeviceCase(cfg, W.seq_lens(cfg, seed=3), seed=3)
    check_step(case)


def test_minimal_workspace_forces_long_chunks():
    cfg = _cfg("minws", 6, 4, 128)
    lens = [5000, 100, 3000, 1, 700, 64]
    case = DeviceCase(cfg, lens, seed=9, chunk_tokens=64)
    n = rpart.workspace_bytes(cfg.B, cfg.H, cfg.d, 0)
    case.ws = torch.empty(n, dtype=torch.uint8, device="cuda")
    check_step(case)
    info = rpart.fd_plan_info(case.ws)
    assert info["items"] <= cfg.B + 1 and info["chunk_tokens"] >= 2048
    with pytest.raises(rpart.FdError) as e:
        rpart.fd_rpart_decode(case.cache.desc, case.q, case.out, case.ws[:n - 256])
    assert e.value.code == rpart.FD_EWORKSPACE


def test_sequences_cut_into_many_chunks():
    """A sequence cut into more than 16 chunks is laid out by the planner's whole workgroup and
    merged 64 chunk states at a time: one sequence of 94 chunks next to short ones (64 d = 64
    chunks is the other width), 137 chunks over three merge batches, and more many-chunk
    sequences than the planner's list holds (it then falls back to one thread per sequence)."""
    for d, lens in ((128, [3000, 5, 0, 700, 33]), (64, [4090, 64, 1]), (128, [4380, 100])):
        granule = 32 if d == 128 else 64
        case = DeviceCase(_cfg("manychunks", len(lens), 2, d), lens, seed=41, chunk_tokens=granule)
        check_step(case)
        info = rpart.fd_plan_info(case.ws)
        assert info["chunk_tokens"] == granule
        assert info["items"] == sum(math.ceil((L + 1) / granule) for L in lens)
    lens = [560 + (i % 7) for i in range(131)]
    case = DeviceCase(_cfg("manybig", len(lens), 1, 128), lens, seed=42, chunk_tokens=32)
    check_step(case)
    assert rpart.fd_plan_info(case.ws)["items"] == sum(math.ceil((L + 1) / 32) for L in lens)


def test_more_sequences_than_planner_threads():
    """3001 sequences (three per planner thread, not a power of two), most of them a few tokens
    long or empty, two long ones among them."""
    lens = [(7 * i) % 23 for i in range(3001)]
    lens[1234], lens[3000] = 1500, 700
    case = DeviceCase(_cfg("manyseq", len(lens), 1, 128), lens, seed=43)
    check_step(case)
    assert rpart.fd_plan_info(case.ws)["total_tokens"] == sum(lens) + len(lens)


def test_active_workgroups_follow_the_share_of_short_sequences():
    """When more than a tenth of the cached tokens sits in sequences under 384 tokens two
    workgroups per compute unit take part, otherwise one; both give the same answer as the oracle
    (the fp16 kernel is launched with two per CU either way)."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    cfg = _cfg("grid", 40, 4, 128)
    short = DeviceCase(cfg, [0] * 8 + [100 + 13 * i for i in range(32)], seed=21)
    check_step(short)
    assert rpart.fd_plan_info(short.ws)["grid"] == 2 * cus
    long_ = DeviceCase(cfg, [0] * 8 + [600 + 13 * i for i in range(32)], seed=22)
    check_step(long_)
    assert rpart.fd_plan_info(long_.ws)["grid"] == cus
    mixed = DeviceCase(cfg, [30 * i for i in range(40)], seed=23)       # uniform mix: ~11 % short
    check_step(mixed)
    assert rpart.fd_plan_info(mixed.ws)["grid"] == 2 * cus


def test_decode_without_append_and_empty_sequences():
    cfg = _cfg("empty", 4, 2, 128)
    case = DeviceCase(cfg, [0, 10, 0, 300], seed=2)
    rpart.fd_rpart_decode(case.cache.desc, case.q, case.out, case.ws)
    torch.cuda.synchronize()
    ref = case.oracle_inputs()
    want, _, _ = O.rpart_decode(ref["K"], ref["V"], ref["seq_lens"], ref["q"])
    got = case.out.cpu().double().numpy()
    assert np.all(got[0] == 0) and np.all(got[2] == 0) and np.all(want[0] == 0)
    assert np.abs(got - want).max() <= TOL * 5.0


def test_single_token_is_bit_exact():
    cfg = _cfg("one", 7, 5, 128)
    case = DeviceCase(cfg, [0] * 7, seed=4)
    check_step(case)
    assert torch.equal(case.out, case.v_new)          # softmax over one token: weight 1


def test_equal_keys_give_mean_of_v():
    cfg = _cfg("mean", 2, 2, 128)
    L = 700
    case = DeviceCase(cfg, [L, L], seed=6, chunk_tokens=128)
    for b in range(2):
        blk = case.cache.block("K", b)
        blk[:, :L, :] = blk[:, :1, :]
    case.k_new.copy_(torch.stack([case.cache.block("K", b)[:, 0, :] for b in range(2)]))
    check_step(case)
    for b in range(2):
        mean = case.cache.block("V", b)[:, :L + 1, :].double().mean(dim=1)
        assert (case.out[b].double() - mean).abs().max() < 1e-3


def test_chunk_size_independence_and_determinism():
    cfg = _cfg("sweep", 3, 4, 128)
    lens = [4000, 777, 2048]
    outs = []
    for chunk in (64, 192, 512, 1024, 4096, 0):
        case = DeviceCase(cfg, lens, seed=8, chunk_tokens=chunk)
        check_step(case)
        first = case.out.clone()
        rpart.fd_rpart_decode(case.cache.desc, case.q, case.out, case.ws)   # again, same state
        torch.cuda.synchronize()
        assert torch.equal(first, case.out)
        outs.append(first.float())
    for o in outs[1:]:
        assert (o - outs[0]).abs().max() <= 2e-3     # one fp16 ulp at |out| < 1 is ~1e-3


def test_capacity_overflow_sets_status_and_skips():
    cfg = _cfg("full", 3, 2, 128)
    case = DeviceCase(cfg, [10, 20, 30], seed=1, extra_cap=1)   # capacities 11, 21, 31
    case.cache.seq_lens.copy_(case.cache.seq_cap)             # every cache full
    case.cache.seq_lens[1] = 20                                # ...except sequence 1
    before = (case.cache.k.clone(), case.cache.v.clone())
    rpart.fd_kv_append(case.cache.desc, case.k_new, case.v_new)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(case.cache.desc, clear=True) == rpart.FD_ST_CAPACITY
    assert rpart.fd_read_status(case.cache.desc) == 0
    assert case.cache.seq_lens.cpu().tolist() == [11, 21, 31]
    assert torch.equal(case.cache.block("K", 1)[:, 20, :], case.k_new[1])
    assert torch.equal(case.cache.block("V", 1)[:, 20, :], case.v_new[1])
    for b in (0, 2):
        n = cfg.H * case.cache.caps[b] * cfg.d
        o = case.cache.offs[b]
        assert torch.equal(case.cache.k[o:o + n], before[0][o:o + n])
        assert torch.equal(case.cache.v[o:o + n], before[1][o:o + n])


def test_bad_length_is_clamped_and_flagged():
    cfg = _cfg("bad", 2, 2, 128)
    case = DeviceCase(cfg, [50, 60], seed=1)
    case.cache.seq_lens[0] = 10_000                            # beyond capacity
    rpart.fd_rpart_decode(case.cache.desc, case.q, case.out, case.ws)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(case.cache.desc, clear=True) & rpart.FD_ST_BADLEN
    assert torch.isfinite(case.out.float()).all()


def test_reset_drops_sequences():
    cfg = _cfg("reset", 4, 2, 64)
    case = DeviceCase(cfg, [100, 200, 300, 400], seed=1)
    rpart.fd_kv_reset(case.cache.desc, torch.tensor([2, 0, 99, -1], dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert case.cache.seq_lens.cpu().tolist() == [0, 200, 0, 400]
    check_step(case)                                           # dropped ones restart at 1 token
    assert case.cache.seq_lens.cpu().tolist() == [1, 201, 1, 401]
    rpart.fd_kv_reset(case.cache.desc)
    torch.cuda.synchronize()
    assert case.cache.seq_lens.cpu().tolist() == [0, 0, 0, 0]


def test_append_preserves_special_bit_patterns():
    cfg = _cfg("bits", 2, 2, 64)
    case = DeviceCase(cfg, [3, 0], seed=1)
    pat = torch.tensor([0x8000, 0x0001, 0x7E01, 0x7C00, 0x03FF, 0xFE55, 0xFC00, 0x0000],
                       dtype=torch.int32).to(torch.int16)
    case.k_new.view(torch.int16)[0, 0, :8] = pat.cuda()
    case.v_new.view(torch.int16)[1, 1, 8:16] = pat.cuda()
    rpart.fd_kv_append(case.cache.desc, case.k_new, case.v_new)
    torch.cuda.synchronize()
    assert torch.equal(case.cache.block("K", 0)[:, 3, :].view(torch.int16), case.k_new[0].view(torch.int16))
    assert torch.equal(case.cache.block("V", 1)[:, 0, :].view(torch.int16), case.v_new[1].view(torch.int16))


def test_subnormal_inputs_are_honoured():
    """fp16 subnormals are exact in fp32 and must not be flushed: with every V a
    subnormal, the output (their weighted mean) is non-zero."""
    cfg = _cfg("sub", 1, 1, 128)
    L = 200
    case = DeviceCase(cfg, [L], seed=1)
    case.cache.block("V", 0).view(torch.int16)[:, :L, :] = 0x0200       # 2^-15
    case.v_new.view(torch.int16)[:] = 0x0200
    check_step(case)
    assert torch.all(case.out.view(torch.int16) == 0x0200)


def test_invalid_arguments_enqueue_nothing():
    cfg = _cfg("inval", 2, 2, 128)
    case = DeviceCase(cfg, [5, 6], seed=1)
    with pytest.raises(rpart.FdError):
        rpart.fd_rpart_decode(case.cache.desc, None, case.out, case.ws)
    with pytest.raises(rpart.FdError):
        rpart.fd_rpart_decode(case.cache.desc, case.q.view(-1)[1:], case.out, case.ws)   # misaligned
    with pytest.raises(rpart.FdError):
        rpart.fd_rpart_decode(case.cache.desc, case.q, case.out, case.ws[1:])            # misaligned
    bad = rpart.fd_kv_desc.from_buffer_copy(case.cache.desc)
    bad.d = 96
    with pytest.raises(rpart.FdError):
        rpart.fd_kv_append(bad, case.k_new, case.v_new)
    torch.cuda.synchronize()
    assert case.cache.seq_lens.cpu().tolist() == [5, 6]


def test_partial_and_merge_refuse_a_workspace_without_a_matching_plan():
    cfg = _cfg("noplan", 3, 2, 128)
    case = DeviceCase(cfg, [100, 5, 700], seed=31)
    case.ws.fill_(0x5A)                                       # never planned
    case.out.fill_(7.0)
    rpart.fd_rpart_partial(case.cache.desc, case.q, case.out, case.ws)
    rpart.fd_rpart_merge(case.cache.desc, case.out, case.ws)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(case.cache.desc, clear=True) == rpart.FD_ST_PLAN
    assert bool((case.out == 7.0).all())                      # nothing written
    # a plan made for another batch shape is refused as well
    other = DeviceCase(_cfg("other", 2, 2, 128), [50, 60], seed=32)
    rpart.fd_rpart_plan(other.cache.desc, case.ws)
    rpart.fd_rpart_partial(case.cache.desc, case.q, case.out, case.ws)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(case.cache.desc, clear=True) == rpart.FD_ST_PLAN
    assert bool((case.out == 7.0).all())
    # and the regular sequence still works on the same workspace afterwards
    check_step(case)


def test_step_can_be_captured_in_a_hip_graph_and_replayed():
    """Every entry point only enqueues kernels (no allocation, no synchronisation, no memset
    node), so a whole step can be captured once and replayed; every replay must give what the
    eager call gives, with eager work and synchronisations between the replays."""
    cfg = _cfg("graph", 5, 4, 128)
    lens = [300, 17, 2049, 0, 999]
    case = DeviceCase(cfg, lens, seed=41, extra_cap=8)
    lens0 = case.cache.seq_lens.clone()
    rpart.fd_rpart_step(case.cache.desc, case.q, case.k_new, case.v_new, case.out, case.ws)
    torch.cuda.synchronize()
    eager = case.out.clone()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    case.cache.seq_lens.copy_(lens0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        g.capture_begin()
        rpart.fd_rpart_step(case.cache.desc, case.q, case.k_new, case.v_new, case.out, case.ws)
        g.capture_end()
    torch.cuda.synchronize()
    assert case.cache.seq_lens.cpu().tolist() == lens         # capture itself runs nothing
    for rep in range(4):
        case.cache.seq_lens.copy_(lens0)
        case.out.fill_(float("nan"))
        (case.q.float() * 2).sum().item()                     # unrelated eager work and a sync
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(case.out, eager), rep
        assert case.cache.seq_lens.cpu().tolist() == [L + 1 for L in lens]
    assert rpart.fd_read_status(case.cache.desc) == 0


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_random_length_mixes(seed):
    """Random ragged batches (empty, a few tokens, a few blocks, a few thousand tokens) under a
    random chunk length: whatever mix of whole blocks, ragged rests and split sequences comes up."""
    rng = np.random.default_rng(1000 + seed)
    kinds = rng.integers(0, 4, size=14)
    lens = [int(x) for x in np.where(kinds == 0, rng.integers(0, 3, 14),
                                     np.where(kinds == 1, rng.integers(1, 41, 14),
                                              np.where(kinds == 2, rng.integers(200, 901, 14),
                                                       rng.integers(1000, 3001, 14))))]
    chunk = int(rng.choice([0, 64, 96, 160, 512, 1000]))
    case = DeviceCase(_cfg("rand%d" % seed, len(lens), 2, 128), lens, seed=50 + seed, chunk_tokens=chunk)
    check_step(case)


def test_folded_merge_standalone_merge_and_repeated_streaming_on_one_plan():
    """The streaming kernel merges a split sequence itself (the wave that finishes the last chunk
    of a head does it).  The stand-alone merge recomputes the same outputs from the chunk states,
    bit for bit; running the streaming kernel again on the same plan gives the same bits again
    (the per-head chunk counters are back at zero after every launch)."""
    cfg = _cfg("fold", 6, 5, 128)
    lens = [0, 700, 33, 3001, 64, 1500]
    case = DeviceCase(cfg, lens, seed=61, chunk_tokens=128)
    case.cache.seq_lens[0] = rpart.FD_SLOT_FREE               # stays empty through the append
    rpart.fd_kv_append(case.cache.desc, case.k_new, case.v_new)
    rpart.fd_rpart_plan(case.cache.desc, case.ws)
    rpart.fd_rpart_partial(case.cache.desc, case.q, case.out, case.ws)
    torch.cuda.synchronize()
    first = case.out.clone()
    finite, zero0 = bool(torch.isfinite(first.float()).all()), bool((first[0] == 0).all())
    assert finite and zero0
    again = torch.full_like(first, float("nan"))
    for _ in range(3):
        rpart.fd_rpart_partial(case.cache.desc, case.q, again, case.ws)
    torch.cuda.synchronize()
    assert torch.equal(again.view(torch.int16), first.view(torch.int16))
    alone = torch.full_like(first, float("nan"))
    rpart.fd_rpart_merge(case.cache.desc, alone, case.ws)
    torch.cuda.synchronize()
    split, single = [1, 3, 5], [2, 4]                          # 701, 3002, 1501 tokens; 34 and 65
    for b in split + [0]:                                      # split sequences and the empty one
        assert torch.equal(alone[b].view(torch.int16), first[b].view(torch.int16))
    for b in single:                                           # not the stand-alone merge's business
        untouched = bool(torch.isnan(alone[b].float()).all())
        assert untouched
    assert rpart.fd_read_status(case.cache.desc) == 0


@pytest.mark.parametrize("d", [64, 128])
def test_two_launch_step_equals_append_then_decode(d):
    """fd_rpart_step (append + plan in one launch, lengths stored by the streaming kernel) against
    fd_kv_append followed by fd_rpart_decode: same cache bits, same lengths, same output bits,
    also with a full cache (append refused), a free slot and an empty sequence in the batch."""
    cfg = _cfg("fused", 7, 3, d)
    lens = [5, 0, 300, 129, 2000, 64, 17]
    a = DeviceCase(cfg, lens, seed=71, extra_cap=1)
    b = DeviceCase(cfg, lens, seed=71, extra_cap=1)
    for case in (a, b):
        case.cache.seq_lens[3] = rpart.FD_SLOT_FREE                       # a free slot
    rpart.fd_rpart_step(a.cache.desc, a.q, a.k_new, a.v_new, a.out, a.ws)
    rpart.fd_kv_append(b.cache.desc, b.k_new, b.v_new)
    rpart.fd_rpart_decode(b.cache.desc, b.q, b.out, b.ws)
    torch.cuda.synchronize()
    want_lens = [6, 1, 301, rpart.FD_SLOT_FREE, 2001, 65, 18]
    assert a.cache.seq_lens.cpu().tolist() == want_lens == b.cache.seq_lens.cpu().tolist()
    assert torch.equal(a.cache.k.view(torch.int16), b.cache.k.view(torch.int16))
    assert torch.equal(a.cache.v.view(torch.int16), b.cache.v.view(torch.int16))
    assert torch.equal(a.out.view(torch.int16), b.out.view(torch.int16))
    assert bool((a.out[3] == 0).all())
    # a second step: every cache is full now (capacity L + 1), nothing may change but the output
    k_before = a.cache.k.clone()
    rpart.fd_rpart_step(a.cache.desc, a.q, a.k_new, a.v_new, a.out, a.ws)
    torch.cuda.synchronize()
    assert rpart.fd_last_device_status(a.cache.desc, a.ws) == rpart.FD_ST_CAPACITY
    assert a.cache.seq_lens.cpu().tolist() == want_lens
    assert torch.equal(a.cache.k, k_before)
    assert torch.equal(a.out.view(torch.int16), b.out.view(torch.int16))


@pytest.mark.parametrize("B,H,L,chunk", [(1, 32, 255, 0), (7, 3, 1000, 256), (300, 2, 129, 64), (5000, 1, 17, 0),
                                         (4, 2, 5000, 128)])
def test_equal_lengths_are_planned_without_a_sort(B, H, L, chunk):
    """Batches of equal-length sequences take the planner's short way (no counting, no sort; items
    b n .. b n + n - 1, chunk-major order): one sequence alone, forced chunks, more sequences than
    planner threads and than the threads' length registers, and a cut into more chunks than the
    short way takes (which must fall back to the general one)."""
    cfg = _cfg("equal", B, H, 64)
    case = DeviceCase(cfg, [L] * B, seed=91, chunk_tokens=chunk, extra_cap=2)
    check_step(case, use_step=True)
    info = rpart.fd_plan_info(case.ws)
    T = info["chunk_tokens"]
    assert info["total_tokens"] == B * (L + 1) and info["items"] == B * math.ceil((L + 1) / T)
    check_step(case)                                          # and again, one token longer
