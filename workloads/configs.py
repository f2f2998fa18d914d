"""The five synthetic workloads (shapes, SwiftKV split, batch recipe).

Shapes and recipes are the benchmark's own: a tiny decoder, Llama-3.1-8B and
-70B shaped decoders, fixed-length and log-uniform varlen prompt batches,
identity or shuffled paged block tables.  All values are seeded (see
generators.py).  Nothing here computes any part of the model.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np
import torch

from .generators import (seeded_normal_bf16, seeded_permutation,
                         seeded_token_ids, seeded_uniform01)

BLOCK_SIZE = 16


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_theta: float
    rms_eps: float = 1e-5

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim


TINY = ModelShape(4, 256, 4, 2, 64, 688, 1024, 1e4, 1e-5)
LLAMA_8B = ModelShape(32, 4096, 32, 8, 128, 14336, 128256, 5e5, 1e-5)
LLAMA_70B = ModelShape(80, 8192, 64, 8, 128, 28672, 128256, 5e5, 1e-5)


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    l: int                      # number of full layers run on prompt tokens
    g: int                      # AcrossKV group size (1 = off)
    seed: int
    kv_fp8: bool = False
    # batch recipe
    fixed_lens: Optional[tuple] = None     # explicit prompt lengths
    loguniform: Optional[tuple] = None     # (count, lo, hi)
    n_decode: int = 0                      # extra 1-token sequences ...
    decode_ctx: int = 0                    # ... each with this many cached tokens
    shuffled_tables: bool = False
    prefix_ctx: int = 0                    # tokens already cached in front of every prompt (prefill in chunks)

    @property
    def n_cache_layers(self):
        return self.l + (self.shape.n_layers - self.l) // self.g


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", TINY, l=2, g=1, seed=1001, fixed_lens=(128,)),
    "8b_l16_b8x2048": Workload("8b_l16_b8x2048", LLAMA_8B, l=16, g=1, seed=1002,
                               fixed_lens=(2048,) * 8),
    "8b_l24_g2_varlen16": Workload("8b_l24_g2_varlen16", LLAMA_8B, l=24, g=2, seed=1003,
                                   loguniform=(16, 512, 8192), shuffled_tables=True),
    "70b_l40_b4x8192": Workload("70b_l40_b4x8192", LLAMA_70B, l=40, g=1, seed=1004,
                                fixed_lens=(8192,) * 4),
    "8b_l16_g4_fp8_32k_dec64": Workload("8b_l16_g4_fp8_32k_dec64", LLAMA_8B, l=16, g=4,
                                        seed=1005, kv_fp8=True, fixed_lens=(32768,),
                                        n_decode=64, decode_ctx=4096),
    # beyond the five configurations: the last 2048-token chunk of 8K-token prompts (the paper's serving
    # runs split prompts into 2048-token chunks), and one decode step of 64 sequences at 2K context
    "8b_l16_b8x2048_ctx6144": Workload("8b_l16_b8x2048_ctx6144", LLAMA_8B, l=16, g=1, seed=1002,
                                       fixed_lens=(2048,) * 8, prefix_ctx=6144),
    "8b_l16_dec64_ctx2048": Workload("8b_l16_dec64_ctx2048", LLAMA_8B, l=16, g=1, seed=1002,
                                     fixed_lens=(), n_decode=64, decode_ctx=2048),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


_PER_LAYER = ("norm1", "wq", "wk", "wv", "wo", "norm2", "wgate", "wup", "wdown")


def _weight_spec(shape: ModelShape, name: str):
    d, qd, kvd, f, v = shape.hidden, shape.q_dim, shape.kv_dim, shape.ffn, shape.vocab
    return {
        "embed": ((v, d), "lin"), "lm_head": ((v, d), "lin"), "final_norm": ((d,), "norm"),
        "norm1": ((d,), "norm"), "norm2": ((d,), "norm"),
        "wq": ((qd, d), "lin"), "wk": ((kvd, d), "lin"), "wv": ((kvd, d), "lin"),
        "wo": ((d, qd), "lin"), "wgate": ((f, d), "lin"), "wup": ((f, d), "lin"),
        "wdown": ((d, f), "lin"),
    }[name]


class WeightStore:
    """Lazily drawn bf16 weights: linear ~ N(0, 0.02), norm gains ~ 1 + N(0, 0.02).

    Row-major [out_features, in_features].  `get` draws on the requested device;
    results are bit-identical on every device.  Tensors are cached only when
    `keep=True` (the GPU side keeps them resident, the oracle streams them).
    """

    def __init__(self, shape: ModelShape, seed: int, device="cpu", keep=False):
        self.shape, self.seed, self.device, self.keep = shape, seed, device, keep
        self._cache: Dict[str, torch.Tensor] = {}

    def get(self, name: str, layer: Optional[int] = None) -> torch.Tensor:
        key = name if layer is None else f"{name}.{layer}"
        if key in self._cache:
            return self._cache[key]
        shp, kind = _weight_spec(self.shape, name)
        mean, std = (1.0, 0.02) if kind == "norm" else (0.0, 0.02)
        t = seeded_normal_bf16(self.seed, key, shp, mean, std, self.device)
        if self.keep:
            self._cache[key] = t
        return t

    def materialize(self):
        """Draw every tensor (requires keep=True); returns self."""
        assert self.keep
        for n in ("embed", "final_norm", "lm_head"):
            self.get(n)
        for j in range(self.shape.n_layers):
            for n in _PER_LAYER:
                self.get(n, j)
        return self


def make_weights(w: Workload, device="cpu", keep=False) -> WeightStore:
    return WeightStore(w.shape, w.seed, device, keep)


@dataclass
class Batch:
    """Packed varlen batch + paged-cache geometry (all host tensors)."""
    token_ids: torch.Tensor          # int32 [T] packed, sequence after sequence
    seq_lens: torch.Tensor           # int32 [B] new tokens per sequence
    context_lens: torch.Tensor       # int32 [B] tokens already cached
    block_tables: torch.Tensor       # int32 [B, max_blocks_per_seq]
    n_blocks: int
    max_blocks_per_seq: int

    @property
    def n_seqs(self):
        return int(self.seq_lens.numel())

    @property
    def n_tokens(self):
        return int(self.seq_lens.sum())


def draw_lengths(w: Workload) -> List[int]:
    if w.fixed_lens is not None:
        lens = list(w.fixed_lens)
    else:
        cnt, lo, hi = w.loguniform
        u = seeded_uniform01(w.seed, "lengths", cnt)
        raw = np.floor(np.exp(math.log(lo) + u * (math.log(hi + 1) - math.log(lo))))
        lens = [int(min(max(x, lo), hi)) for x in raw]
    return lens


def build_batch(w: Workload, lens: Optional[List[int]] = None,
                ctx: Optional[List[int]] = None, shuffled: Optional[bool] = None,
                spare_frac: float = 0.10) -> Batch:
    """Sequences = prompts (ctx 0) followed by `n_decode` one-token sequences."""
    if lens is None:
        lens = draw_lengths(w) + [1] * w.n_decode
        ctx = [w.prefix_ctx] * (len(lens) - w.n_decode) + [w.decode_ctx] * w.n_decode
    if ctx is None:
        ctx = [0] * len(lens)
    if shuffled is None:
        shuffled = w.shuffled_tables
    B = len(lens)
    T = sum(lens)
    ids = seeded_token_ids(w.seed, "token_ids", T, w.shape.vocab)
    need = [(c + n + BLOCK_SIZE - 1) // BLOCK_SIZE for c, n in zip(ctx, lens)]
    used = sum(need)
    n_blocks = used + int(math.ceil(used * spare_frac)) if shuffled else used
    order = seeded_permutation(w.seed, "blocks", n_blocks) if shuffled else np.arange(n_blocks)
    maxb = max(need)
    bt = np.zeros((B, maxb), dtype=np.int32)
    pos = 0
    for b in range(B):
        bt[b, :need[b]] = order[pos:pos + need[b]]
        pos += need[b]
    return Batch(ids, torch.tensor(lens, dtype=torch.int32), torch.tensor(ctx, dtype=torch.int32),
                 torch.from_numpy(bt), n_blocks, maxb)
