"""CPU oracle for the SwiftKV prefill forward pass.  TEST INFRASTRUCTURE ONLY.

This file is the plain definition of what the GPU library must compute,
written from the paper for checking, not for speed.  Only the tests, the
smoke check and the benchmark's CPU-baseline leg may import it; the product
(the HIP library and its Python binding) never does, and this file imports
nothing from the product.

What is computed (SwiftKV paper, Sec. 3.1 "Preliminaries", Sec. 3.2 Eq. 2,
Sec. 3.3 "AcrossKV", Sec. 3.5 forward-pass order, and the footnote of
Sec. 3.2 about the last input token):

  * layers 1..l are ordinary pre-norm Llama decoder layers (Q = X W_Q,
    K = X W_K, V = X W_V with grouped-query heads, Sec. 3.1) run on every new
    token; their K/V go to the KV cache;
  * the residual stream after layer l (the paper's x_{l+1}) feeds the K/V
    projections of every later layer j > l (Eq. 2: KV_j = W_KV^j x_{l+1});
    with AcrossKV one layer per group of g consecutive later layers computes
    the K/V the whole group shares (Sec. 3.3);
  * only the last new token of every sequence (and decode tokens, Sec. 3.5)
    continues through layers l+1..L, attending to those caches, to give logits.

Readings where the paper is silent (listed in the design notes of the repo):
RMSNorm with the *later layer's own* input-norm gain before W_KV^j; rotate-half
RoPE without frequency rescaling, K cached after RoPE; the first layer of an
AcrossKV group is the one that projects; softmax scale 1/sqrt(head_dim),
causal mask including self; consecutive query heads share a KV head.

Arithmetic: everything runs in `dtype` (float64 by default; float32 is used at
8B/70B sizes).  RoPE angles are always formed in float64.  torch.matmul and
torch.softmax are the only library primitives; there is no blocking or fusion.

Pins (tests/test_oracle_*.py): l = L against the Hugging Face Llama CPU
implementation; later-layer K/V against that implementation's own modules
applied to its hidden state l; attention against an explicit-loop brute force;
RoPE / RMSNorm / FP8 closed forms; slot indices by enumeration; FLOP counts
against the paper's Table 1.  Parity unpinned by the paper (self-consistent
conventions only): choice of the projecting layer inside an AcrossKV group,
rms_eps for the 8B/70B shapes, FP8 scale granularity.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Sequence

import torch

BLOCK = 16          # tokens per paged-cache block
FP8_MAX = 448.0     # largest finite e4m3fn magnitude


# --------------------------------------------------------------------------
# small pieces
# --------------------------------------------------------------------------
def rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    """x * rsqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = (x * x).mean(dim=-1, keepdim=True)
    return x * torch.rsqrt(ms + eps) * gain


def rope_cos_sin(pos: torch.Tensor, head_dim: int, theta: float):
    """cos/sin of pos * theta^(-2i/head_dim), i < head_dim/2, in float64."""
    i = torch.arange(head_dim // 2, dtype=torch.float64)
    inv_freq = theta ** (-2.0 * i / head_dim)
    ang = pos.to(torch.float64)[:, None] * inv_freq[None, :]
    return torch.cos(ang), torch.sin(ang)


def rope(x: torch.Tensor, pos: torch.Tensor, theta: float) -> torch.Tensor:
    """Rotate-half RoPE.  x: [n, heads, head_dim]; pairs are (i, i + head_dim/2)."""
    hd = x.shape[-1]
    cos, sin = rope_cos_sin(pos, hd, theta)
    cos = cos.to(x.dtype)[:, None, :]
    sin = sin.to(x.dtype)[:, None, :]
    x1, x2 = x[..., : hd // 2], x[..., hd // 2:]
    return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], dim=-1)


def gqa_attention(q: torch.Tensor, q_pos: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                  act_round=None) -> torch.Tensor:
    """Causal grouped-query attention of queries at absolute positions q_pos
    over keys/values at positions 0..n_k-1.

    q: [n_q, Hq, hd]; k, v: [n_k, Hkv, hd].  Query head h uses KV head
    h // (Hq / Hkv).  Key s is visible to a query at position p iff s <= p.
    act_round: see swiftkv_prefill (applied to the softmax weights).
    """
    n_q, Hq, hd = q.shape
    n_k, Hkv, _ = k.shape
    rep = Hq // Hkv
    visible = torch.arange(n_k)[None, :] <= q_pos.to(torch.int64)[:, None]
    out = torch.empty_like(q)
    for h in range(Hq):
        kh, vh = k[:, h // rep, :], v[:, h // rep, :]
        s = (q[:, h, :] @ kh.T) / math.sqrt(hd)
        s = s.masked_fill(~visible, float("-inf"))
        w = torch.softmax(s, dim=-1)
        out[:, h, :] = (w if act_round is None else act_round(w)) @ vh
    return out


def silu(x: torch.Tensor) -> torch.Tensor:
    return x / (1.0 + torch.exp(-x))


ROUND_POINTS = ("a", "qkv", "p", "o", "h", "z")
"""Places where a reduced-precision pipeline stores an activation between
matrix products: "a" normed layer inputs, "qkv" rotated queries and the K/V
rows, "p" softmax weights, "o" attention output, "h" residual stream, "z" the
SwiGLU product.  All but "h" are inputs of a matrix product."""


def _rounder(act_round):
    """R(x, point) from the `act_round` argument of swiftkv_prefill: None (plain
    definition), one function for every point, or a dict point -> function
    (points not named stay exact)."""
    if act_round is None:
        return lambda x, point: x
    if callable(act_round):
        return lambda x, point: act_round(x)
    unknown = set(act_round) - set(ROUND_POINTS)
    if unknown:
        raise ValueError(f"unknown rounding points {sorted(unknown)}")
    return lambda x, point: act_round[point](x) if point in act_round else x


# --------------------------------------------------------------------------
# AcrossKV layer -> cache-layer map (Sec. 3.3) and paged-cache addressing
# --------------------------------------------------------------------------
def n_cache_layers(L: int, l: int, g: int) -> int:
    if not (1 <= l <= L) or g < 1 or (L - l) % g:
        raise ValueError("need 1 <= l <= L and (L - l) divisible by g")
    return l + (L - l) // g


def cache_layer_of(j: int, l: int, g: int) -> int:
    """0-based cache layer that 1-based model layer j reads/writes."""
    return j - 1 if j <= l else l + (j - l - 1) // g


def leader_layers(L: int, l: int, g: int) -> List[int]:
    """1-based layers whose W_K/W_V project x_{l+1}: the first of each group."""
    return [l + 1 + p * g for p in range((L - l) // g)]


def kv_cache_fraction_saved(L: int, l: int, g: int, bytes_ratio: float = 1.0) -> float:
    """Fraction of KV-cache memory saved versus L full-precision layers."""
    return 1.0 - n_cache_layers(L, l, g) * bytes_ratio / L


def slot_index(block_table_row: Sequence[int], pos: int) -> int:
    return int(block_table_row[pos // BLOCK]) * BLOCK + pos % BLOCK


def slot_mapping(block_tables: torch.Tensor, context_lens: Sequence[int],
                 seq_lens: Sequence[int]):
    """Packed-batch integer plan: cu_seqlens[B+1], positions[T], slots[T],
    last_rows[B] (row of each sequence's last new token)."""
    cu, positions, slots, last_rows = [0], [], [], []
    for b, (c, n) in enumerate(zip(context_lens, seq_lens)):
        for i in range(int(n)):
            p = int(c) + i
            positions.append(p)
            slots.append(slot_index(block_tables[b].tolist(), p))
        cu.append(cu[-1] + int(n))
        last_rows.append(cu[-1] - 1)
    return (torch.tensor(cu, dtype=torch.int32), torch.tensor(positions, dtype=torch.int32),
            torch.tensor(slots, dtype=torch.int64), torch.tensor(last_rows, dtype=torch.int32))


# --------------------------------------------------------------------------
# FP8 e4m3fn (OCP): 1 sign, 4 exponent (bias 7), 3 mantissa bits, no inf,
# 0x7F/0xFF are NaN, largest finite 448.
# --------------------------------------------------------------------------
def fp8_e4m3fn_decode_table() -> torch.Tensor:
    """All 256 codes as float64 (NaN for 0x7F and 0xFF)."""
    vals = []
    for code in range(256):
        s = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            vals.append(float("nan"))
        elif e == 0:
            vals.append(s * (m / 8.0) * 2.0 ** -6)
        else:
            vals.append(s * (1.0 + m / 8.0) * 2.0 ** (e - 7))
    return torch.tensor(vals, dtype=torch.float64)


def fp8_e4m3fn_encode(x: torch.Tensor) -> torch.Tensor:
    """Round-to-nearest-even, saturating at +-448, of float32 `x` -> uint8 codes.

    Done by explicit search over the 127 non-negative finite code values: the
    nearest value wins, ties go to the even code.
    """
    x = x.to(torch.float32)
    table = fp8_e4m3fn_decode_table()[:127].to(torch.float64)       # codes 0..126, ascending
    a = x.abs().to(torch.float64).clamp(max=FP8_MAX).reshape(-1)
    hi = torch.searchsorted(table, a).clamp(max=126)                  # first code with value >= a
    lo = (hi - 1).clamp(min=0)
    d_lo, d_hi = a - table[lo], table[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = torch.where(pick_hi, hi, lo).to(torch.uint8)
    sign = (torch.signbit(x).reshape(-1)).to(torch.uint8) << 7
    return (code | sign).reshape(x.shape)


def fp8_scale(amax: torch.Tensor) -> torch.Tensor:
    """float32 scale from an absmax: max(amax, 1e-12) / 448."""
    return (amax.to(torch.float32).clamp(min=1e-12) / torch.tensor(FP8_MAX, dtype=torch.float32))


def fp8_quantize(x: torch.Tensor, scale: torch.Tensor) -> torch.Tensor:
    """codes = encode(clamp(x / scale, +-448)), the division taken in float32."""
    y = (x.to(torch.float32) / scale.to(torch.float32)).clamp(-FP8_MAX, FP8_MAX)
    return fp8_e4m3fn_encode(y)


def fp8_dequantize(codes: torch.Tensor, scale: torch.Tensor, dtype=torch.float32) -> torch.Tensor:
    tab = fp8_e4m3fn_decode_table().to(torch.float32)
    return (tab[codes.long()] * scale.to(torch.float32)).to(dtype)


# --------------------------------------------------------------------------
# paged KV cache
# --------------------------------------------------------------------------
class PagedKVCache:
    """Physical cache [n_cache_layers][2 (K,V)][n_blocks][16][Hkv][hd].

    Float mode stores values in `dtype`.  FP8 mode stores uint8 e4m3fn codes
    plus float32 scales; reads return code * scale.  Scales are either one per
    (cache layer, K|V, KV head), [n_cache_layers][2][Hkv], set by the caller or
    by swiftkv_prefill, or, with `per_token` (the granularity of Appendix B.1),
    one per (cache layer, K|V, token), [n_cache_layers][2][n_blocks*16], taken
    from the token's own absmax over all KV heads when the token is written.
    """

    def __init__(self, n_layers: int, n_blocks: int, n_kv_heads: int, head_dim: int,
                 block_tables: torch.Tensor, dtype=torch.float64, fp8: bool = False, per_token: bool = False):
        self.C, self.NB, self.Hkv, self.hd = n_layers, n_blocks, n_kv_heads, head_dim
        self.block_tables = block_tables.to(torch.int64)
        self.dtype, self.fp8, self.per_token = dtype, fp8, per_token and fp8
        shape = (n_layers, 2, n_blocks * BLOCK, n_kv_heads, head_dim)
        self.data = torch.zeros(shape, dtype=torch.uint8 if fp8 else dtype)
        if self.per_token:
            self.scales = torch.zeros((n_layers, 2, n_blocks * BLOCK), dtype=torch.float32)
        else:
            self.scales = torch.zeros((n_layers, 2, n_kv_heads), dtype=torch.float32) if fp8 else None

    def slots(self, b: int, pos: torch.Tensor) -> torch.Tensor:
        pos = pos.to(torch.int64)
        return self.block_tables[b][pos // BLOCK] * BLOCK + pos % BLOCK

    def write(self, c: int, b: int, pos: torch.Tensor, k: torch.Tensor, v: torch.Tensor):
        s = self.slots(b, pos)
        if self.per_token:
            for t, x in ((0, k), (1, v)):
                sc = fp8_scale(x.abs().amax(dim=(1, 2)))                    # one scale per written token
                self.scales[c, t, s] = sc
                self.data[c, t, s] = fp8_quantize(x, sc[:, None, None])
        elif self.fp8:
            self.data[c, 0, s] = fp8_quantize(k, self.scales[c, 0][None, :, None])
            self.data[c, 1, s] = fp8_quantize(v, self.scales[c, 1][None, :, None])
        else:
            self.data[c, 0, s] = k.to(self.dtype)
            self.data[c, 1, s] = v.to(self.dtype)

    def read(self, c: int, b: int, n: int):
        """K, V of positions 0..n-1 of sequence b in cache layer c (dequantised)."""
        s = self.slots(b, torch.arange(n))
        k, v = self.data[c, 0, s], self.data[c, 1, s]
        if self.per_token:
            k = fp8_dequantize(k, self.scales[c, 0, s][:, None, None], self.dtype)
            v = fp8_dequantize(v, self.scales[c, 1, s][:, None, None], self.dtype)
        elif self.fp8:
            k = fp8_dequantize(k, self.scales[c, 0][None, :, None], self.dtype)
            v = fp8_dequantize(v, self.scales[c, 1][None, :, None], self.dtype)
        return k, v


# --------------------------------------------------------------------------
# the forward pass
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Shape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_theta: float
    rms_eps: float


WeightFn = Callable[[str, Optional[int]], torch.Tensor]
"""weights(name, layer0) -> tensor [out_features, in_features] (or [hidden] for
norm gains); layer0 is the 0-based layer or None for embed/final_norm/lm_head."""


def _attn_and_mlp(sh: Shape, W, j0: int, h: torch.Tensor, q_pos: torch.Tensor,
                  k: torch.Tensor, v: torch.Tensor, a: torch.Tensor, R=lambda x, point: x) -> torch.Tensor:
    """Rest of decoder layer j0 (0-based) after its K/V are known: queries from
    the normed input `a`, attention over (k, v), O-projection, residual,
    second norm, SwiGLU MLP, residual."""
    n = h.shape[0]
    q = (a @ W("wq", j0).T).view(n, sh.n_q_heads, sh.head_dim)
    q = R(rope(q, q_pos, sh.rope_theta), "qkv")
    o = R(gqa_attention(q, q_pos, k, v, lambda w: R(w, "p")).reshape(n, sh.n_q_heads * sh.head_dim), "o")
    u = R(h + o @ W("wo", j0).T, "h")
    m = R(rmsnorm(u, W("norm2", j0), sh.rms_eps), "a")
    z = R(silu(m @ W("wgate", j0).T) * (m @ W("wup", j0).T), "z")
    return R(u + z @ W("wdown", j0).T, "h")


def swiftkv_prefill(sh: Shape, weights: WeightFn, token_ids: torch.Tensor,
                    seq_lens: Sequence[int], context_lens: Sequence[int],
                    l: int, g: int, cache: PagedKVCache,
                    dtype=torch.float64, fp8_compute_scales: bool = True,
                    seq_subset: Optional[Sequence[int]] = None,
                    all_token_tail: bool = False, act_round=None, early_exit=None):
    """SwiftKV prefill of a packed batch.  Returns logits [B, vocab] (rows of
    sequences outside `seq_subset` are NaN) and leaves K/V in `cache`.

    token_ids: int [T] packed; sequence b has context_lens[b] cached tokens in
    `cache` already and seq_lens[b] new ones (one new token = a decode step,
    several = a chunk of a longer prompt: new token i sits at position
    context + i and attends to the cached positions and to new tokens <= i).
    fp8_compute_scales: in FP8 mode with per-head scales, derive each (cache
    layer, K|V, head) scale from the absmax of what this call writes there (over
    the processed sequences); otherwise use the scales already in `cache`.  A
    cache with per-token scales sets each token's scales when it writes it.
    all_token_tail: run layers l+1..L on every new token instead of only the
    last (checking aid); logits are still those of the last token.
    early_exit: None, or (gain [hidden], head [vocab, hidden], threshold): the
    simple early exit of Appendix B.4.  An extra head reads the layer-l output of
    the last new token, logits_ee = head @ RMSNorm(h_l; gain); when its largest
    softmax probability exceeds the threshold these logits are the result and
    layers l+1..L are not needed for that token, otherwise the remaining layers
    run as usual.  The K/V cache is the same either way (every later layer's
    K/V comes from h_l).  With early_exit the function returns a third value,
    the per-sequence exit flags.
    act_round: None gives the plain definition.  A function (e.g. round to
    bfloat16 and back) is applied to every activation a reduced-precision
    pipeline would store between matrix products (the ROUND_POINTS: normed
    inputs, q/k/v, softmax weights, attention output, residual stream, MLP
    product); a dict point -> function rounds only the named points.  The tests
    use it to measure how far such storage alone moves the result on a given
    model: rounding every point but the residual stream is what bf16 matrix
    instructions force on any implementation.  Not part of the method.
    """
    R = _rounder(act_round)
    L = sh.n_layers
    C = n_cache_layers(L, l, g)
    assert cache.C == C
    B = len(seq_lens)
    seqs = list(range(B)) if seq_subset is None else list(seq_subset)
    cu = [0]
    for n in seq_lens:
        cu.append(cu[-1] + int(n))
    def W(name, j0=None):
        return weights(name, j0).to(dtype)

    pos = {b: int(context_lens[b]) + torch.arange(int(seq_lens[b])) for b in seqs}
    E = W("embed")
    h = {b: E[token_ids[cu[b]:cu[b + 1]].long()] for b in seqs}

    def store(c: int, kv: Dict[int, tuple]):
        """Write one cache layer for all processed sequences (FP8: scales first)."""
        if cache.fp8 and fp8_compute_scales and not cache.per_token:
            for t in (0, 1):
                amax = torch.stack([kv[b][t].abs().amax(dim=(0, 2)) for b in seqs]).amax(dim=0)
                cache.scales[c, t] = fp8_scale(amax)
        for b in seqs:
            cache.write(c, b, pos[b], kv[b][0], kv[b][1])

    # ---- layers 1..l on every new token (Sec. 3.1, 3.2) --------------------
    for j0 in range(l):
        a, kv = {}, {}
        for b in seqs:
            n = h[b].shape[0]
            a[b] = R(rmsnorm(h[b], W("norm1", j0), sh.rms_eps), "a")
            k = rope((a[b] @ W("wk", j0).T).view(n, sh.n_kv_heads, sh.head_dim), pos[b], sh.rope_theta)
            v = (a[b] @ W("wv", j0).T).view(n, sh.n_kv_heads, sh.head_dim)
            kv[b] = (R(k, "qkv"), R(v, "qkv"))
        store(j0, kv)
        for b in seqs:
            n_ctx = int(context_lens[b]) + int(seq_lens[b])
            k_all, v_all = cache.read(j0, b, n_ctx)          # as stored (FP8: dequantised)
            h[b] = _attn_and_mlp(sh, W, j0, h[b], pos[b], k_all, v_all, a[b], R)

    # ---- Eq. 2 + AcrossKV: K/V of every later layer from x_{l+1} -----------
    for p, j in enumerate(leader_layers(L, l, g)):
        j0 = j - 1
        kv = {}
        for b in seqs:
            n = h[b].shape[0]
            a_p = R(rmsnorm(h[b], W("norm1", j0), sh.rms_eps), "a")
            k = rope((a_p @ W("wk", j0).T).view(n, sh.n_kv_heads, sh.head_dim), pos[b], sh.rope_theta)
            v = (a_p @ W("wv", j0).T).view(n, sh.n_kv_heads, sh.head_dim)
            kv[b] = (R(k, "qkv"), R(v, "qkv"))
        store(l + p, kv)

    # ---- only the last new token continues (footnote of Sec. 3.2, Sec. 3.5) -
    if all_token_tail:
        t, tpos = dict(h), dict(pos)
    else:
        t = {b: h[b][-1:] for b in seqs}
        tpos = {b: pos[b][-1:] for b in seqs}
    for j in range(l + 1, L + 1):
        j0 = j - 1
        c = cache_layer_of(j, l, g)
        for b in seqs:
            n_ctx = int(context_lens[b]) + int(seq_lens[b])
            k_all, v_all = cache.read(c, b, n_ctx)
            a = R(rmsnorm(t[b], W("norm1", j0), sh.rms_eps), "a")
            t[b] = _attn_and_mlp(sh, W, j0, t[b], tpos[b], k_all, v_all, a, R)

    logits = torch.full((B, sh.vocab), float("nan"), dtype=dtype)
    gf, Wlm = W("final_norm"), W("lm_head")
    for b in seqs:
        logits[b] = R(rmsnorm(t[b][-1], gf, sh.rms_eps), "a") @ Wlm.T
    hidden_l = {b: h[b] for b in seqs}
    if early_exit is not None:
        g_ee, w_ee, thr = early_exit
        g_ee, w_ee = g_ee.to(dtype), w_ee.to(dtype)
        exited = torch.zeros(B, dtype=torch.bool)
        for b in seqs:
            lg = R(rmsnorm(h[b][-1], g_ee, sh.rms_eps), "a") @ w_ee.T
            if float(torch.softmax(lg, dim=-1).max()) > thr:
                exited[b] = True
                logits[b] = lg
        return logits, hidden_l, exited
    return logits, hidden_l


# --------------------------------------------------------------------------
# operation counts (paper's Table 1 accounting: 2 flops per multiply-add)
# --------------------------------------------------------------------------
def gflops_per_prefill_token(sh: Shape, l: int, g: int, attended_keys: float):
    """Per-prefill-token GFLOPs by operation class with SwiftKV split l and
    AcrossKV group g, in the paper's Table 1 columns.  `attended_keys` is the
    average number of keys a token attends to."""
    L, d = sh.n_layers, sh.hidden
    qd, kvd = sh.n_q_heads * sh.head_dim, sh.n_kv_heads * sh.head_dim
    P = (L - l) // g
    out = {
        "vocab": 2 * (2.0 * d * sh.vocab),                    # embedding + LM head, counted alike
        "kv": (l + P) * 2.0 * d * (2 * kvd),
        "qo": l * 2 * (2.0 * d * qd),
        "mlp": l * 3 * (2.0 * d * sh.ffn),
        "attn": l * 4.0 * qd * attended_keys,
    }
    out["total"] = sum(out.values())
    return {k: v / 1e9 for k, v in out.items()}


def executed_flops(sh: Shape, l: int, g: int, seq_lens: Sequence[int],
                   context_lens: Sequence[int]) -> Dict[str, float]:
    """FLOPs one SwiftKV prefill call actually executes (GEMM and attention
    parts), prompt tokens through l layers + fused KV, one tail row per
    sequence through the remaining layers and the LM head."""
    L, d = sh.n_layers, sh.hidden
    qd, kvd = sh.n_q_heads * sh.head_dim, sh.n_kv_heads * sh.head_dim
    P = (L - l) // g
    T = float(sum(int(n) for n in seq_lens))
    B = float(len(seq_lens))
    layer_gemm = 2.0 * d * (qd + 2 * kvd) + 2.0 * d * qd + 6.0 * d * sh.ffn
    gemm = T * (l * layer_gemm + P * 2.0 * d * 2 * kvd)
    gemm += B * ((L - l) * (2 * 2.0 * d * qd + 6.0 * d * sh.ffn) + 2.0 * d * sh.vocab)
    attn = 0.0
    for c, n in zip(context_lens, seq_lens):
        c, n = int(c), int(n)
        pairs = n * c + n * (n + 1) / 2.0           # (query, visible key) pairs of the new tokens
        attn += l * 4.0 * qd * pairs
        attn += (L - l) * 4.0 * qd * (c + n)        # tail row attends to everything
    return {"gemm": gemm, "attn": attn, "total": gemm + attn}
