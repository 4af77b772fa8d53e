"""int8 KV-cache path (FastDecode Section 5.2) vs the oracle, through the C ABI.

Bar: lengths, code bytes and scales bit-exact (the quantiser decides integers, both sides
decide them in binary32); out within 2e-3 * max|V_dequantised|.
"""
import numpy as np
import pytest
import torch

from oracle import rpart_oracle as O
from paper_2403_11421_amd import rpart, workloads as W
from paper_2403_11421_amd.kvcache import KVCacheQ
from tests.util import bits

pytestmark = pytest.mark.gpu
TOL = 2e-3


class QCase:
    def __init__(self, cfg, lens, seed=W.DEFAULT_SEED, extra_cap=1, chunk_tokens=0):
        dev = "cuda"
        self.cfg, self.lens0 = cfg, [int(x) for x in lens]
        self.cache = KVCacheQ(cfg.B, cfg.H, cfg.d, [L + extra_cap for L in self.lens0], dev, chunk_tokens)
        for b, L in enumerate(self.lens0):
            if L:
                self.cache.fill("K", b, W.gen_cache_block(cfg, "K", b, L, seed, dev))
                self.cache.fill("V", b, W.gen_cache_block(cfg, "V", b, L, seed, dev))
        self.cache.set_lens(self.lens0)
        self.q = W.gen_vectors(cfg, "q", seed, dev)
        self.k_new = W.gen_vectors(cfg, "k_new", seed, dev)
        self.v_new = W.gen_vectors(cfg, "v_new", seed, dev)
        self.out = torch.full((cfg.B, cfg.H, cfg.d), float("nan"), dtype=torch.float16, device=dev)
        scale = max(1, -(-256 // chunk_tokens)) if chunk_tokens else 2
        self.ws = self.cache.workspace((sum(self.lens0) + cfg.B) * scale)

    def host(self, batch):
        """Token-major host copies (the oracle's layout) of what the device holds now."""
        c = self.cache
        def tm(t):
            return np.ascontiguousarray(t.permute(1, 0, *range(2, t.dim())).cpu().numpy())
        return dict(Kc=[tm(c.codes("K", b)) for b in batch], Ks=[tm(c.scales("K", b)) for b in batch],
                    Vc=[tm(c.codes("V", b)) for b in batch], Vs=[tm(c.scales("V", b)) for b in batch],
                    lens=c.seq_lens.cpu().numpy().astype(np.int32)[batch].copy())


def check_qstep(case, batch=None, use_step=False):
    cfg = case.cfg
    batch = list(range(cfg.B)) if batch is None else list(batch)
    ref = case.host(batch)                                   # snapshot BEFORE the device step
    sel = torch.tensor(batch, dtype=torch.long)
    k_new, v_new, q = (bits(t.cpu()[sel]) for t in (case.k_new, case.v_new, case.q))
    if use_step:
        rpart.fd_rpartq_step(case.cache.desc, case.q, case.k_new, case.v_new, case.out, case.ws)
    else:
        rpart.fd_kvq_append(case.cache.desc, case.k_new, case.v_new)
        rpart.fd_rpartq_decode(case.cache.desc, case.q, case.out, case.ws)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(case.cache.desc) == 0
    O.kvq_append(ref["Kc"], ref["Ks"], ref["Vc"], ref["Vs"], ref["lens"], k_new, v_new)
    want, _ = O.rpartq_decode(ref["Kc"], ref["Ks"], ref["Vc"], ref["Vs"], ref["lens"], q)
    got_state = case.host(batch)
    assert np.array_equal(got_state["lens"], ref["lens"])
    for key in ("Kc", "Ks", "Vc", "Vs"):                     # whole blocks, appended row included
        for a, b_ in zip(got_state[key], ref[key]):
            assert np.array_equal(a, b_), key
    maxv = 0.0
    for vc, vs, L in zip(ref["Vc"], ref["Vs"], ref["lens"]):
        if L:
            maxv = max(maxv, float(np.abs((vc[:L].astype(np.float64) - 128) * vs[:L, :, None]).max()))
    got = case.out.cpu()[sel].double().numpy()
    assert np.all(np.isfinite(got))
    err = float(np.abs(got - want).max())
    assert err <= TOL * maxv, f"max|err| {err:.3e} > {TOL} * max|V| ({maxv:.3f})"
    return err, maxv


def _cfg(name, B, H, d=128, **kw):
    return W.RPartConfig(name, B, H, d, "const", 0, 0, **kw)


def test_bulk_store_quantises_like_the_oracle():
    """Caches are pre-filled through fd_kvq_store_rows (prompt ingestion): the code bytes and
    scales it stores are the oracle quantiser's, bit for bit, rows outside the range untouched."""
    cfg = _cfg("fill", 2, 3)
    case = QCase(cfg, [300, 77], extra_cap=5)
    for b, L in enumerate(case.lens0):
        for which in ("K", "V"):
            rows = W.gen_cache_block(cfg, which, b, L, W.DEFAULT_SEED, "cuda")
            codes, scales = O.quantize_rows_i8(bits(rows))
            assert np.array_equal(case.cache.codes(which, b)[:, :L].cpu().numpy(), codes)
            assert np.array_equal(case.cache.scales(which, b)[:, :L].cpu().numpy(), scales)
            assert bool((case.cache.codes(which, b)[:, L:] == 128).all())       # as allocated
            assert bool((case.cache.scales(which, b)[:, L:] == 0).all())


EDGE_LENS = [0, 1, 2, 7, 8, 9, 31, 32, 33, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1000, 2500]


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("chunk", [0, 64, 256, 1024, 4096])
def test_edge_lengths_all_chunk_sizes(chunk, d):
    cfg = _cfg("qedges", len(EDGE_LENS), 3, d)
    case = QCase(cfg, EDGE_LENS, seed=21, chunk_tokens=chunk)
    check_qstep(case)
    info = rpart.fd_plan_info(case.ws)
    assert info["total_tokens"] == sum(EDGE_LENS) + len(EDGE_LENS)
    # the 8-bit kernel runs three workgroups per compute unit on short sequences (mean ~300 here)
    assert info["grid"] == 3 * torch.cuda.get_device_properties(0).multi_processor_count


def test_more_sequences_than_planner_threads():
    """2001 sequences: the planner's scrambled visiting order must still reach each one once."""
    lens = [(7 * i) % 23 for i in range(2001)]
    lens[1234], lens[2000] = 1500, 700
    case = QCase(_cfg("q8manyseq", len(lens), 1), lens, seed=43)
    check_qstep(case)
    assert rpart.fd_plan_info(case.ws)["total_tokens"] == sum(lens) + len(lens)


@pytest.mark.parametrize("d", [128, 64])
def test_step_entry_point_many_heads_and_peaked_keys(d):
    cfg = W.RPartConfig("qstep", 6, 40, d, "const", 0, 0, peaked_keys=True)
    case = QCase(cfg, [300, 17, 2049, 64, 999, 4100], seed=5)
    check_qstep(case, use_step=True)


def test_append_quantises_bit_exactly_including_special_rows():
    cfg = _cfg("qbits", 3, 2)
    case = QCase(cfg, [3, 0, 9])
    case.k_new[0, 0, :] = 0                                            # all-zero row: scale 0, bytes 128
    case.v_new[1, 1, :] = 0
    case.v_new[1, 1, 5] = -3.0                                          # one non-zero value
    case.k_new.view(torch.int16)[2, 1, :4] = torch.tensor([0x0001, 0x8001, 0x03FF, 0x0400],
                                                           dtype=torch.int32).to(torch.int16).cuda()  # subnormals
    case.k_new[2, 1, 4:] = 0
    case.v_new[2, 0, :] = torch.arange(128, dtype=torch.float16) * 0.125 - 7.0  # ties: x/scale = k + 1/2
    check_qstep(case)
    assert int(case.cache.codes("K", 0)[0, 3].min()) == 128 and float(case.cache.scales("K", 0)[0, 3]) == 0.0


def test_single_token_returns_its_dequantised_value():
    cfg = _cfg("qone", 5, 4)
    case = QCase(cfg, [0] * 5, seed=4)
    check_qstep(case)
    deq = torch.stack([(case.cache.codes("V", b)[:, 0].float() - 128) * case.cache.scales("V", b)[:, 0:1]
                       for b in range(5)])
    # weight 1: out = x_hat up to the kernel's fp32 rounding of scale*u - 128*scale and one fp16 ulp
    assert float((case.out.float() - deq).abs().max()) <= 2.0 ** -10 * float(deq.abs().max())


def test_determinism_and_chunk_independence():
    cfg = _cfg("qsweep", 3, 4)
    outs = []
    for chunk in (256, 512, 4096, 0):
        case = QCase(cfg, [4000, 777, 2048], seed=8, chunk_tokens=chunk)
        check_qstep(case)
        first = case.out.clone()
        rpart.fd_rpartq_decode(case.cache.desc, case.q, case.out, case.ws)
        torch.cuda.synchronize()
        assert torch.equal(first, case.out)
        outs.append(first.float())
    for o in outs[1:]:
        assert (o - outs[0]).abs().max() <= 2e-3


def test_capacity_overflow_and_reset():
    cfg = _cfg("qfull", 2, 2)
    case = QCase(cfg, [10, 20], extra_cap=1)
    case.cache.seq_lens[0] = case.cache.caps[0]
    before = case.cache.k_codes.clone()
    rpart.fd_kvq_append(case.cache.desc, case.k_new, case.v_new)
    torch.cuda.synchronize()
    assert rpart.fd_read_status(case.cache.desc, clear=True) == rpart.FD_ST_CAPACITY
    assert case.cache.seq_lens.cpu().tolist() == [11, 21]
    n = cfg.H * case.cache.caps[0] * cfg.d
    assert torch.equal(case.cache.k_codes[:n], before[:n])
    rpart.fd_kvq_reset(case.cache.desc, torch.tensor([1], dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert case.cache.seq_lens.cpu().tolist() == [11, 0]


def test_invalid_arguments():
    cfg = _cfg("qinval", 2, 2)
    case = QCase(cfg, [5, 6])
    bad = rpart.fd_kvq_desc.from_buffer_copy(case.cache.desc)
    bad.d = 96
    with pytest.raises(rpart.FdError):
        rpart.fd_kvq_append(bad, case.k_new, case.v_new)
    with pytest.raises(rpart.FdError):
        rpart.fd_rpartq_decode(case.cache.desc, None, case.out, case.ws)
    with pytest.raises(rpart.FdError):
        rpart.fd_rpartq_decode(case.cache.desc, case.q, case.out, case.ws[:1024])


@pytest.mark.parametrize("name,n_sample", [("c2_7b_uniform", None), ("c3_7b_ragged", None),
                                           ("c4_13b_geometric", None), ("c5_capacity", 256)])
def test_full_config_whole_batch_parity(name, n_sample):
    """Every sequence of configs 2-4 (256 length-stratified ones of config 5) through the oracle:
    the oracle quantises the generator's rows itself, so the device's code bytes and row
    parameters (written by fd_kvq_store_rows and fd_kvq_append) are compared bit for bit too."""
    from tests.full_parity import check_full_config
    err, maxv, done = check_full_config(name, "int8", n_sample)
    assert done == (W.CONFIGS[name].B if n_sample is None else n_sample)


def test_long_context_few_sequences():
    """One sequence of 100001 cached tokens next to two shorter ones: many chunks per head
    (planner's cooperative lay-out, batched merge), library-chosen chunking."""
    cfg = _cfg("q8long", 3, 8)
    lens = [100001, 30000, 257]
    case = QCase(cfg, lens, seed=77, extra_cap=4)
    case.ws = case.cache.workspace(sum(lens) + len(lens))
    check_qstep(case)
    plan = rpart.fd_plan_info(case.ws)
    print(f"long context: plan={plan}", flush=True)
    assert plan["items"] > 16


def test_config1_shape_with_a_quantised_cache():
    """Config 1's shape (B=4, H=8, d=64, 128 cached tokens + 1) on the 8-bit cache."""
    cfg = W.CONFIGS["c1_tiny"]
    case = QCase(cfg, W.seq_lens(cfg))
    err, maxv = check_qstep(case, use_step=True)
    print(f"c1_tiny/int8: max|err|={err:.3e} bound={TOL * maxv:.3e}", flush=True)


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
    case = QCase(_cfg("rand%d" % seed, len(lens), 2, 64 if seed % 2 else 128), lens, seed=50 + seed,
                 chunk_tokens=chunk)
    check_qstep(case)
