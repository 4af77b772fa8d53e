"""Seeded workload generators and the byte accounting of the metric (no GPU)."""
import math
import os

import numpy as np
import torch

from paper_2403_11421_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "table3_sizes.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()[:2]
        out[k] = float(v)
    return out


def test_bytes_per_token_matches_table3():
    """16 KB per cached token per layer at the 7B shape reproduces Table 3's sizes
    for 256 cached tokens, and 1 flop per KV byte reproduces Table 2's R-Part flops."""
    g = _gold()
    cfg = W.CONFIGS["c2_7b_uniform"]
    bpt = cfg.bytes_per_token()
    assert bpt == 16384
    assert abs(256 * bpt - g["kv_cache_batch1"]) / g["kv_cache_batch1"] < 2e-3
    assert abs(1024 * 256 * bpt - g["kv_cache_batch1024"]) / g["kv_cache_batch1024"] < 2e-3
    vec = 4 * cfg.H * cfg.d * 2                         # q, k, v, o rows in fp16
    assert abs(vec - g["vectors_batch1"]) / g["vectors_batch1"] < 3e-3
    assert abs(1024 * vec - g["vectors_batch1024"]) / g["vectors_batch1024"] < 3e-3
    flops = 1024 * 256 * 4 * cfg.H * cfg.d              # 2d MACs for q.k + 2d for p.v, per head
    for dev in ("gpu", "cpu"):
        printed = g[f"rpart_{dev}_latency_ms_b1024"] * 1e-3 * g[f"rpart_{dev}_tflops_b1024"] * 1e12
        assert abs(flops - printed) / printed < 5e-3


def test_config_shapes():
    c = W.CONFIGS
    assert (c["c1_tiny"].B, c["c1_tiny"].H, c["c1_tiny"].d) == (4, 8, 64)
    assert (c["c2_7b_uniform"].B, c["c2_7b_uniform"].H, c["c2_7b_uniform"].d) == (256, 32, 128)
    assert (c["c3_7b_ragged"].B, c["c3_7b_ragged"].H) == (512, 32)
    assert (c["c4_13b_geometric"].B, c["c4_13b_geometric"].H) == (256, 40)
    assert c["c4_13b_geometric"].bytes_per_token() == 20480
    assert c["c5_capacity"].B == 2048
    assert W.total_tokens_after_append(W.seq_lens(c["c2_7b_uniform"])) == 256 * 2049
    assert 4 * 32 * 128 * 256 * 2049 == 8594128896


def test_seq_lens_rules():
    for name, cfg in W.CONFIGS.items():
        L = W.seq_lens(cfg)
        assert len(L) == cfg.B and L == W.seq_lens(cfg)
        assert min(L) >= cfg.len_lo and max(L) <= cfg.len_hi
    L3 = np.array(W.seq_lens(W.CONFIGS["c3_7b_ragged"]))
    assert abs(L3.mean() - 2048.5) < 150 and L3.min() < 100 and L3.max() > 3990
    L4 = np.array(W.seq_lens(W.CONFIGS["c4_13b_geometric"]))
    assert abs(L4.mean() - 1024) < 150
    L5 = np.array(W.seq_lens(W.CONFIGS["c5_capacity"]))
    assert abs(L5.mean() - 1536) < 30
    assert W.seq_lens(W.CONFIGS["c3_7b_ragged"], seed=1) != list(L3)


def test_values_are_seeded_normal_and_position_addressable():
    cfg = W.CONFIGS["c2_7b_uniform"]
    a = W.gen_cache_block(cfg, "K", 3, 64)
    b = W.gen_cache_block(cfg, "K", 3, 64)
    assert a.dtype == torch.float16 and a.shape == (32, 64, 128) and torch.equal(a, b)
    # a sub-range regenerates the same rows
    c = W.gen_cache_block(cfg, "K", 3, 16, t0=40)
    assert torch.equal(a[:, 40:56], c)
    # distinct tensors / sequences / seeds differ
    assert not torch.equal(a, W.gen_cache_block(cfg, "V", 3, 64))
    assert not torch.equal(a, W.gen_cache_block(cfg, "K", 4, 64))
    assert not torch.equal(a, W.gen_cache_block(cfg, "K", 3, 64, seed=5))
    x = a.double().flatten()
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1 / math.sqrt(2)) < 0.01
    z = x * math.sqrt(2)
    assert abs((z ** 4).mean() - 3.0) < 0.1                    # normal kurtosis
    q = W.gen_vectors(cfg, "q")
    assert q.shape == (256, 32, 128)
    assert torch.equal(q[[5, 9]], W.gen_vectors(cfg, "q", batch=[5, 9]))


def test_peaked_keys_have_per_head_spread_and_offset():
    cfg = W.CONFIGS["c3_7b_ragged"]
    k = W.gen_cache_block(cfg, "K", 0, 512).double()             # [H,L,d]
    std = (k - k.mean(dim=1, keepdim=True)).std(dim=(1, 2))
    for h in range(8):
        assert abs(std[h] / (1.0, 2.0, 4.0, 8.0)[h % 4] - 1) < 0.05
    off = k.mean(dim=1)                                          # [H,d] ~ c_h
    assert 3.0 < off.std() < 5.0
    assert k.abs().max() < 200
    kn = W.gen_vectors(cfg, "k_new", batch=[0]).double()[0]
    assert (kn - off).abs().mean() < 8.0
