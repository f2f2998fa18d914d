"""Counter-based, device-independent random inputs.

Every value is a pure function of (seed, stream name, element index), computed
with 64-bit integer arithmetic and a table lookup only, so a tensor drawn on
the CPU and the same tensor drawn on a GPU are bit-identical.  That lets the
GPU tests draw multi-gigabyte weights on the device while the CPU oracle draws
exactly the same numbers layer by layer on the host.
"""
from __future__ import annotations

import hashlib
import math

import numpy as np
import torch

_MASK64 = (1 << 64) - 1


def _to_i64(u: int) -> int:
    u &= _MASK64
    return u - (1 << 64) if u >= (1 << 63) else u


_C1 = _to_i64(0xBF58476D1CE4E5B9)
_C2 = _to_i64(0x94D049BB133111EB)
_GOLD = 0x9E3779B97F4A7C15


def stream_key(seed: int, name: str) -> int:
    """64-bit key for the sub-stream `name` of `seed` (host-side, via sha256)."""
    h = hashlib.sha256(f"{seed}:{name}".encode()).digest()
    return int.from_bytes(h[:8], "little")


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def counter_hash(key: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """splitmix64 finaliser of (key + (start+i)*golden) for i in [0, count).

    Returns int64 lanes holding the 64 mixed bits (two's complement view).
    Integer multiplication wraps identically on CPU and GPU.
    """
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    x = idx * _to_i64(_GOLD) + _to_i64(key)
    x = (x ^ _lsr(x, 30)) * _C1
    x = (x ^ _lsr(x, 27)) * _C2
    x = x ^ _lsr(x, 31)
    return x


_TABLE_CACHE: dict = {}


def normal_table(mean: float, std: float) -> torch.Tensor:
    """65536 bf16 values: the standard-normal quantiles at (i+0.5)/65536,
    scaled to N(mean, std) in fp64 and rounded once to bf16 (host only)."""
    k = (float(mean), float(std))
    if k not in _TABLE_CACHE:
        p = (torch.arange(65536, dtype=torch.float64) + 0.5) / 65536.0
        z = math.sqrt(2.0) * torch.erfinv(2.0 * p - 1.0)
        _TABLE_CACHE[k] = (mean + std * z).to(torch.bfloat16)
    return _TABLE_CACHE[k]


def seeded_normal_bf16(seed: int, name: str, shape, mean: float, std: float,
                       device="cpu", chunk: int = 1 << 26) -> torch.Tensor:
    """bf16 tensor of `shape` ~ N(mean, std) (65536-level quantile table)."""
    n = int(np.prod(shape))
    key = stream_key(seed, name)
    table = normal_table(mean, std).to(device)
    out = torch.empty(n, dtype=torch.bfloat16, device=device)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        bits = counter_hash(key, s, c, device)
        out[s:s + c] = table[_lsr(bits, 48)]
    return out.view(*shape)


def seeded_token_ids(seed: int, name: str, count: int, vocab: int) -> torch.Tensor:
    """int32 token ids uniform in [0, vocab) (host tensor)."""
    bits = counter_hash(stream_key(seed, name), 0, count)
    return (_lsr(bits, 20) % vocab).to(torch.int32)


def seeded_uniform01(seed: int, name: str, count: int) -> np.ndarray:
    """float64 uniforms in [0,1) with 53 random bits (host)."""
    bits = counter_hash(stream_key(seed, name), 0, count)
    return (_lsr(bits, 11).numpy().astype(np.float64)) / float(1 << 53)


def seeded_permutation(seed: int, name: str, n: int) -> np.ndarray:
    """A permutation of [0, n): stable argsort of n hashed keys (host)."""
    bits = counter_hash(stream_key(seed, name), 0, n)
    return np.argsort(_lsr(bits, 1).numpy(), kind="stable").astype(np.int64)


def seeded_fp8_codes(seed: int, name: str, shape, device="cpu", mag_lo: int = 0x48,
                     mag_hi: int = 0x77) -> torch.Tensor:
    """uint8 e4m3fn codes with a random sign and a magnitude field uniform in
    [mag_lo, mag_hi] (default: values 4 .. 240 times the scale, i.e. spread over
    six binades; never the NaN patterns).  Used to synthesise pre-existing FP8
    cache contents."""
    n = int(np.prod(shape))
    bits = counter_hash(stream_key(seed, name), 0, n, device)
    b = _lsr(bits, 40)
    mag = mag_lo + (b & 0xFFFF) % (mag_hi - mag_lo + 1)
    return ((_lsr(bits, 63) << 7) | mag).to(torch.uint8).view(*shape)
