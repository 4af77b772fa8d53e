"""Seeded synthetic inputs for the R-Part decode step.

The paper evaluates on Llama-7b/13b generation (FastDecode Section 6.1); the
time of the R-Part depends only on tensor shapes and cached lengths (Section
4.2: latency proportional to total cached length), so random tensors of those
shapes stand in for activations of the trained models.

Every value is a pure function of ``(seed, tensor id, b, t, h, i)`` through a
counter-based generator (SplitMix64 finaliser -> two 24-bit uniforms ->
Box-Muller), written with torch integer/float ops so that it runs unchanged on
the host or on the device that will hold the cache.  Transcendentals may differ
in the last bit between devices, therefore a consumer that needs the exact
values a device holds copies them from that device.

This module contains no attention arithmetic; it is the only code shared by
the CPU oracle's tests and the HIP path's tests.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Sequence

import torch

DEFAULT_SEED = 20240311

# tensor ids (4 bits)
TID_Q, TID_K, TID_V, TID_KNEW, TID_VNEW, TID_LEN, TID_HEAD = 1, 2, 3, 4, 5, 6, 7

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """Two's-complement reinterpretation of an unsigned 64-bit value."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix_t(z: torch.Tensor) -> torch.Tensor:
    """SplitMix64 output function on an int64 tensor (wrapping arithmetic)."""
    z = z + _s64(_GOLDEN)
    z = (z ^ _lsr(z, 30)) * _s64(_M1)
    z = (z ^ _lsr(z, 27)) * _s64(_M2)
    return z ^ _lsr(z, 31)


def _mix_i(z: int) -> int:
    """SplitMix64 output function on a Python int (same bits as ``_mix_t``)."""
    z = (z + _GOLDEN) & _MASK64
    z = ((z ^ (z >> 30)) * _M1) & _MASK64
    z = ((z ^ (z >> 27)) * _M2) & _MASK64
    return z ^ (z >> 31)


def _key(seed: int, tid: int) -> int:
    return _mix_i((seed & _MASK64) ^ (tid * 0xD1B54A32D192ED03 & _MASK64))


def _counter(b, t, h, i):
    """46-bit element counter: b < 4096, t < 16384, h < 256, i < 256."""
    return ((b * 16384 + t) * 256 + h) * 256 + i


def normal_from_counter(seed: int, tid: int, ctr: torch.Tensor) -> torch.Tensor:
    """Standard normal float32 tensor, one value per int64 counter."""
    bits = _mix_t(ctr ^ _s64(_key(seed, tid)))
    u1 = (_lsr(bits, 40) + 1).to(torch.float32) * (1.0 / 16777216.0)        # (0, 1]
    u2 = (_lsr(bits, 16) & 0xFFFFFF).to(torch.float32) * (1.0 / 16777216.0)  # [0, 1)
    r = torch.sqrt(-2.0 * torch.log(u1))
    return r * torch.cos((2.0 * math.pi) * u2)


def uniform_int(seed: int, tid: int, ctr: int, lo: int, hi: int) -> int:
    """Uniform integer in [lo, hi] (host side)."""
    return lo + _mix_i(ctr ^ _key(seed, tid)) % (hi - lo + 1)


def uniform_unit(seed: int, tid: int, ctr: int) -> float:
    """Uniform float64 in [0, 1) with 53 random bits (host side)."""
    return (_mix_i(ctr ^ _key(seed, tid)) >> 11) / 9007199254740992.0


@dataclass(frozen=True)
class RPartConfig:
    """One decode-step workload: shapes, length rule and value rule."""
    name: str
    B: int
    H: int
    d: int
    len_rule: str            # "const", "uniform", "exp"
    len_lo: int
    len_hi: int
    len_mean: int = 0
    scale: float = 1.0       # multiplies N(0,1) for q, K, V and the new k/v
    peaked_keys: bool = False  # K = sigma_h * N(0,1) + c_h (per-head spread and offset)
    n_layers: int = 32       # layers of the model the shape is taken from

    def bytes_per_token(self) -> int:
        """fp16 K row + V row over all heads of one layer."""
        return 4 * self.H * self.d


CONFIGS: Dict[str, RPartConfig] = {
    # tiny parity case: 128 cached tokens + 1 appended
    "c1_tiny": RPartConfig("c1_tiny", 4, 8, 64, "const", 128, 128, n_layers=1),
    # Llama-7B shape, uniform 2048 cached tokens + 1 appended (16 KB per token per layer)
    "c2_7b_uniform": RPartConfig("c2_7b_uniform", 256, 32, 128, "const", 2048, 2048,
                                 scale=1.0 / math.sqrt(2.0)),
    # Llama-7B shape, ragged lengths, keys with per-head spread/offset
    "c3_7b_ragged": RPartConfig("c3_7b_ragged", 512, 32, 128, "uniform", 1, 4096,
                                peaked_keys=True),
    # Llama-13B shape, exponential ("geometric-like") lengths, mean 1024, clipped
    "c4_13b_geometric": RPartConfig("c4_13b_geometric", 256, 40, 128, "exp", 16, 8192,
                                    len_mean=1024, n_layers=40),
    # capacity stress: 2048 sequences of 1024..2048 tokens
    "c5_capacity": RPartConfig("c5_capacity", 2048, 32, 128, "uniform", 1024, 2048),
    # the workload behind the paper's Table 2 (one block of a 7B model, 256 cached tokens per
    # sequence: 4.19 MB of KV per sequence, Table 3), at its two batch sizes -- context only
    "t2_batch1": RPartConfig("t2_batch1", 1, 32, 128, "const", 255, 255),
    "t2_batch1024": RPartConfig("t2_batch1024", 1024, 32, 128, "const", 255, 255),
}


def seq_lens(cfg: RPartConfig, seed: int = DEFAULT_SEED) -> List[int]:
    """Cached tokens per sequence BEFORE the step's append."""
    out = []
    for b in range(cfg.B):
        if cfg.len_rule == "const":
            L = cfg.len_lo
        elif cfg.len_rule == "uniform":
            L = uniform_int(seed, TID_LEN, b, cfg.len_lo, cfg.len_hi)
        elif cfg.len_rule == "exp":
            u = uniform_unit(seed, TID_LEN, b)
            L = int(math.floor(-cfg.len_mean * math.log1p(-u)))
            L = min(max(L, cfg.len_lo), cfg.len_hi)
        else:
            raise ValueError(cfg.len_rule)
        out.append(L)
    return out


_SIGMAS = (1.0, 2.0, 4.0, 8.0)


def _head_sigma(cfg: RPartConfig, device) -> torch.Tensor:
    s = torch.tensor([_SIGMAS[h % 4] for h in range(cfg.H)], dtype=torch.float32, device=device)
    return s.view(cfg.H, 1, 1)


def _head_offset(cfg: RPartConfig, seed: int, device) -> torch.Tensor:
    h = torch.arange(cfg.H, dtype=torch.int64, device=device).view(cfg.H, 1, 1)
    i = torch.arange(cfg.d, dtype=torch.int64, device=device).view(1, 1, cfg.d)
    return 4.0 * normal_from_counter(seed, TID_HEAD, _counter(0, 0, h, i))   # [H,1,d]


def gen_vectors(cfg: RPartConfig, which: str, seed: int = DEFAULT_SEED,
                device="cpu", batch: Sequence[int] | None = None) -> torch.Tensor:
    """fp16 ``[B', H, d]`` step vectors: ``which`` in {"q", "k_new", "v_new"}."""
    tid = {"q": TID_Q, "k_new": TID_KNEW, "v_new": TID_VNEW}[which]
    bs = list(range(cfg.B)) if batch is None else list(batch)
    b = torch.tensor(bs, dtype=torch.int64, device=device).view(-1, 1, 1)
    h = torch.arange(cfg.H, dtype=torch.int64, device=device).view(1, cfg.H, 1)
    i = torch.arange(cfg.d, dtype=torch.int64, device=device).view(1, 1, cfg.d)
    x = normal_from_counter(seed, tid, _counter(b, 0, h, i)) * cfg.scale
    if which == "k_new" and cfg.peaked_keys:
        x = x * _head_sigma(cfg, device).view(1, cfg.H, 1) + \
            _head_offset(cfg, seed, device).view(1, cfg.H, cfg.d)
    return x.to(torch.float16)


def gen_cache_block(cfg: RPartConfig, which: str, b: int, L: int,
                    seed: int = DEFAULT_SEED, device="cpu", t0: int = 0) -> torch.Tensor:
    """fp16 ``[H, L, d]``: cached rows t0..t0+L-1 of sequence ``b``; ``which`` in {"K","V"}."""
    tid = {"K": TID_K, "V": TID_V}[which]
    h = torch.arange(cfg.H, dtype=torch.int64, device=device).view(cfg.H, 1, 1)
    t = torch.arange(t0, t0 + L, dtype=torch.int64, device=device).view(1, L, 1)
    i = torch.arange(cfg.d, dtype=torch.int64, device=device).view(1, 1, cfg.d)
    x = normal_from_counter(seed, tid, _counter(b, t, h, i)) * cfg.scale
    if which == "K" and cfg.peaked_keys:
        x = x * _head_sigma(cfg, device) + _head_offset(cfg, seed, device)
    return x.to(torch.float16)


def total_tokens_after_append(lens: Sequence[int]) -> int:
    return sum(int(L) + 1 for L in lens)
