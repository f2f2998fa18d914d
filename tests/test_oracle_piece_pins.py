"""Pins for the oracle's building blocks: closed forms, brute force on tiny
inputs, library special cases and the numbers the paper prints."""
import math
import os

import pytest
import torch

import workloads as WL
from oracle import swiftkv_oracle as O
from tests.helpers import oracle_shape

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- attention
def _brute_attention(q, q_pos, k, v):
    """Explicit scalar loops, float64, straight from the softmax definition."""
    n_q, Hq, hd = q.shape
    n_k, Hkv, _ = k.shape
    out = torch.zeros_like(q)
    for i in range(n_q):
        for h in range(Hq):
            kh = h // (Hq // Hkv)
            scores = []
            for s in range(n_k):
                if s <= int(q_pos[i]):
                    dot = sum(float(q[i, h, e]) * float(k[s, kh, e]) for e in range(hd))
                    scores.append((s, dot / math.sqrt(hd)))
            mx = max(x for _, x in scores)
            den = sum(math.exp(x - mx) for _, x in scores)
            for s, x in scores:
                w = math.exp(x - mx) / den
                for e in range(hd):
                    out[i, h, e] += w * float(v[s, kh, e])
    return out


def test_attention_matches_brute_force():
    g = torch.Generator().manual_seed(1)
    q = torch.randn(7, 4, 8, generator=g, dtype=torch.float64)
    k = torch.randn(12, 2, 8, generator=g, dtype=torch.float64)
    v = torch.randn(12, 2, 8, generator=g, dtype=torch.float64)
    q_pos = torch.tensor([5, 6, 7, 8, 9, 10, 11])
    ref = _brute_attention(q, q_pos, k, v)
    assert torch.allclose(O.gqa_attention(q, q_pos, k, v), ref, atol=1e-12)


def test_attention_special_cases():
    g = torch.Generator().manual_seed(2)
    q = torch.randn(9, 4, 16, generator=g, dtype=torch.float64)
    k = torch.randn(9, 2, 16, generator=g, dtype=torch.float64)
    v = torch.randn(9, 2, 16, generator=g, dtype=torch.float64)
    pos = torch.arange(9)
    o = O.gqa_attention(q, pos, k, v)
    # position 0 sees only key 0: the output is exactly v_0 of its KV head
    assert torch.allclose(o[0], v[0].repeat_interleave(2, dim=0), atol=1e-14)
    # GQA == MHA on replicated KV heads == torch's own causal attention
    kk, vv = k.repeat_interleave(2, dim=1), v.repeat_interleave(2, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.transpose(0, 1)[None], kk.transpose(0, 1)[None], vv.transpose(0, 1)[None], is_causal=True)
    assert torch.allclose(o, ref[0].transpose(0, 1), atol=1e-12)
    # constant V rows: any convex combination returns that constant
    vc = torch.ones_like(v) * 3.25
    assert torch.allclose(O.gqa_attention(q, pos, k, vc), torch.full_like(q, 3.25), atol=1e-12)


# --------------------------------------------------------------------- RoPE
def test_rope_closed_forms():
    hd, theta = 16, 1e4
    g = torch.Generator().manual_seed(3)
    x = torch.randn(6, 3, hd, generator=g, dtype=torch.float64)
    pos = torch.tensor([0, 1, 2, 7, 100, 4095])
    y = O.rope(x, pos, theta)
    assert torch.equal(y[0], x[0])                                  # position 0 is the identity
    # each pair (i, i + hd/2) is rotated by pos * theta^(-2i/hd): check with complex numbers
    for t in range(6):
        for i in range(hd // 2):
            ang = float(pos[t]) * theta ** (-2.0 * i / hd)
            z = complex(float(x[t, 1, i]), float(x[t, 1, i + hd // 2])) * complex(math.cos(ang), math.sin(ang))
            assert abs(z.real - float(y[t, 1, i])) < 1e-12 and abs(z.imag - float(y[t, 1, i + hd // 2])) < 1e-12
    # pair norms are preserved
    n_in = x[..., : hd // 2] ** 2 + x[..., hd // 2:] ** 2
    n_out = y[..., : hd // 2] ** 2 + y[..., hd // 2:] ** 2
    assert torch.allclose(n_in, n_out, atol=1e-12)


def test_rope_scores_depend_on_relative_position_only():
    hd, theta = 32, 5e5
    g = torch.Generator().manual_seed(4)
    q = torch.randn(1, 1, hd, generator=g, dtype=torch.float64)
    k = torch.randn(1, 1, hd, generator=g, dtype=torch.float64)
    def score(m, n):
        return float((O.rope(q, torch.tensor([m]), theta) * O.rope(k, torch.tensor([n]), theta)).sum())
    assert abs(score(10, 3) - score(1007, 1000)) < 1e-9
    assert abs(score(10, 3) - score(3, 10)) > 1e-6


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_properties():
    g = torch.Generator().manual_seed(5)
    x = torch.randn(5, 64, generator=g, dtype=torch.float64)
    gain = 1 + 0.1 * torch.randn(64, generator=g, dtype=torch.float64)
    y1 = O.rmsnorm(x, torch.ones(64, dtype=torch.float64), 0.0)
    assert torch.allclose((y1 * y1).mean(-1), torch.ones(5, dtype=torch.float64), atol=1e-12)
    assert torch.allclose(O.rmsnorm(3.7 * x, gain, 0.0), O.rmsnorm(x, gain, 0.0), atol=1e-12)
    assert torch.allclose(O.rmsnorm(x, gain, 1e-5), y1 * gain * torch.sqrt((x * x).mean(-1, keepdim=True) / ((x * x).mean(-1, keepdim=True) + 1e-5)), atol=1e-12)
    # against torch's own rms_norm
    assert torch.allclose(O.rmsnorm(x, gain, 1e-5), torch.nn.functional.rms_norm(x, (64,), gain, 1e-5), atol=1e-12)


# ---------------------------------------------------------------------- FP8
def test_fp8_decode_table_closed_form_and_library():
    tab = O.fp8_e4m3fn_decode_table()
    assert math.isnan(tab[0x7F]) and math.isnan(tab[0xFF])
    assert tab[0x7E] == 448.0 and tab[0xFE] == -448.0
    assert tab[0x01] == 2.0 ** -9 and tab[0x08] == 2.0 ** -6 and tab[0x38] == 1.0
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64)
    ok = ~torch.isnan(tab)
    assert torch.equal(tab[ok], lib[ok]) and torch.isnan(lib[~ok]).all()


def test_fp8_encode_rounding():
    tab = O.fp8_e4m3fn_decode_table()
    finite = [c for c in range(256) if not math.isnan(tab[c]) and c != 0x80]
    codes = torch.tensor(finite, dtype=torch.uint8)
    # every representable value encodes to itself
    assert torch.equal(O.fp8_e4m3fn_encode(tab[codes.long()].float()), codes)
    # midpoints go to the even code; just off the midpoint goes to the nearer
    for c in range(0, 126):
        lo, hi = float(tab[c]), float(tab[c + 1])
        mid = torch.tensor([(lo + hi) / 2], dtype=torch.float32)
        assert float(mid) == (lo + hi) / 2
        assert int(O.fp8_e4m3fn_encode(mid)) == (c if c % 2 == 0 else c + 1)
        assert int(O.fp8_e4m3fn_encode(torch.nextafter(mid, torch.tensor(0.0)))) == c
        assert int(O.fp8_e4m3fn_encode(torch.nextafter(mid, torch.tensor(1e9)))) == c + 1
    # saturation and sign
    assert int(O.fp8_e4m3fn_encode(torch.tensor([1e9]))) == 0x7E
    assert int(O.fp8_e4m3fn_encode(torch.tensor([-1e9]))) == 0xFE
    # agrees with torch's own cast on random in-range values
    g = torch.Generator().manual_seed(6)
    x = (torch.randn(20000, generator=g) * 60).clamp(-448, 448)
    assert torch.equal(O.fp8_e4m3fn_encode(x), x.to(torch.float8_e4m3fn).view(torch.uint8))


def test_fp8_scale_and_error_bound():
    g = torch.Generator().manual_seed(7)
    x = torch.randn(4096, generator=g) * 3
    s = O.fp8_scale(x.abs().max())
    codes = O.fp8_quantize(x, s)
    assert int(codes[x.abs().argmax()]) & 0x7F == 0x7E          # the absmax element becomes +-448
    dq = O.fp8_dequantize(codes, s)
    normal = x.abs() / s >= 2.0 ** -6
    assert ((dq - x).abs()[normal] <= 2.0 ** -4 * x.abs()[normal] * (1 + 1e-6)).all()


def test_fp8_per_token_cache_scales():
    """Per-token scales (Appendix B.1): each written token carries its own K and V
    scale = its absmax over all heads / 448; its largest element becomes +-448;
    tokens written in separate calls get the same codes as tokens written
    together; rows differing by a factor keep their codes and scale by it; the
    library's float8 cast of x / scale gives the same codes."""
    bt = torch.tensor([[2, 0, 1]], dtype=torch.int32)
    g = torch.Generator().manual_seed(9)
    n, H, hd = 37, 2, 8
    k = torch.randn(n, H, hd, generator=g) * torch.logspace(-3, 2, n)[:, None, None]   # rows of very different size
    v = torch.randn(n, H, hd, generator=g)
    c1 = O.PagedKVCache(1, 3, H, hd, bt, dtype=torch.float32, fp8=True, per_token=True)
    c1.write(0, 0, torch.arange(n), k, v)
    slots = c1.slots(0, torch.arange(n))
    assert torch.equal(c1.scales[0, 0, slots], k.abs().amax(dim=(1, 2)).float() / 448)
    assert torch.equal(c1.scales[0, 1, slots], v.abs().amax(dim=(1, 2)).float() / 448)
    assert ((c1.data[0, 0, slots].view(n, -1) & 0x7F).amax(dim=1) == 0x7E).all()
    want = (k / c1.scales[0, 0, slots][:, None, None]).to(torch.float8_e4m3fn).view(torch.uint8)
    assert torch.equal(c1.data[0, 0, slots], want)
    kd, vd = c1.read(0, 0, n)
    big = k.abs() >= 2.0 ** -6 * c1.scales[0, 0, slots][:, None, None]
    assert ((kd - k).abs()[big] <= 2.0 ** -4 * k.abs()[big] * (1 + 1e-6)).all()        # every row, small or large
    # written in two calls
    c2 = O.PagedKVCache(1, 3, H, hd, bt, dtype=torch.float32, fp8=True, per_token=True)
    c2.write(0, 0, torch.arange(20), k[:20], v[:20])
    c2.write(0, 0, torch.arange(20, n), k[20:], v[20:])
    assert torch.equal(c1.data, c2.data) and torch.equal(c1.scales, c2.scales)
    # scaling a row by a power of two moves only its scale
    c3 = O.PagedKVCache(1, 3, H, hd, bt, dtype=torch.float32, fp8=True, per_token=True)
    k3 = k.clone()
    k3[5] *= 8.0
    c3.write(0, 0, torch.arange(n), k3, v)
    assert torch.equal(c3.data, c1.data)
    assert c3.scales[0, 0, slots[5]] == 8 * c1.scales[0, 0, slots[5]]


# ------------------------------------------------------------ integer plans
def test_slot_mapping_enumeration():
    bt = torch.tensor([[7, 2, 9, 0], [4, 1, 0, 0]], dtype=torch.int32)
    cu, pos, slots, last = O.slot_mapping(bt, [0, 17], [40, 1])
    assert cu.tolist() == [0, 40, 41] and last.tolist() == [39, 40]
    assert pos.tolist() == list(range(40)) + [17]
    want = [7 * 16 + p for p in range(16)] + [2 * 16 + p for p in range(16)] + [9 * 16 + p for p in range(8)] + [1 * 16 + 1]
    assert slots.tolist() == want


def test_paged_cache_scatter_gather_roundtrip():
    bt = torch.tensor([[3, 0], [1, 2]], dtype=torch.int32)
    cache = O.PagedKVCache(1, 4, 2, 4, bt)
    k = torch.arange(20 * 2 * 4, dtype=torch.float64).view(20, 2, 4)
    cache.write(0, 1, torch.arange(20), k, -k)
    kk, vv = cache.read(0, 1, 20)
    assert torch.equal(kk, k) and torch.equal(vv, -k)
    # physical placement: position 17 of sequence 1 sits in block 2, offset 1
    assert torch.equal(cache.data[0, 0, 2 * 16 + 1], k[17])
    assert cache.data[0, 0, 3 * 16:].abs().sum() == 0            # sequence 0's blocks untouched


# ----------------------------------------------------- numbers in the paper
def test_table1_gflops_per_prefill_token():
    """Paper Table 1 (Llama-3.1-70B).  Attention column: the baseline row fixes
    the average attended keys; the other rows must then follow."""
    sh = oracle_shape(WL.configs.LLAMA_70B)
    rows = {r[0]: [float(x) for x in r[1:]] for r in _rows("paper_table1_gflops.txt")}
    keys = rows["baseline"][4] * 1e9 / (sh.n_layers * 4.0 * sh.n_q_heads * sh.head_dim)
    cases = {"baseline": (80, 1), "swiftkv25": (60, 1), "swiftkv50": (40, 1), "swiftkv50_acrosskv4": (40, 4)}
    base_total = None
    for name, (l, g) in cases.items():
        got = O.gflops_per_prefill_token(sh, l, g, keys)
        vocab, kv, qo, mlp, attn, total, rel = rows[name]
        if name == "swiftkv25":
            # the paper's 25 % row keeps the K,V column at 2.6: all 80 layers still project K/V
            assert got["kv"] == pytest.approx(2.6, abs=0.1)
        assert got["vocab"] == pytest.approx(vocab, abs=0.15)
        assert got["kv"] == pytest.approx(kv, abs=0.1)
        assert got["qo"] == pytest.approx(qo, abs=0.6)
        assert got["mlp"] == pytest.approx(mlp, abs=0.8)
        assert got["attn"] == pytest.approx(attn, abs=0.5)
        assert got["total"] == pytest.approx(total, abs=1.6)
        base_total = base_total or got["total"]
        assert 100 * got["total"] / base_total == pytest.approx(rel, abs=0.3)


def test_kv_cache_reduction_numbers():
    for L, l, g, ratio, pct in _rows("paper_kv_cache_reduction.txt"):
        got = 100 * O.kv_cache_fraction_saved(int(L), int(l), int(g), float(ratio))
        assert got == pytest.approx(float(pct), abs=1e-9)
    with pytest.raises(ValueError):
        O.n_cache_layers(32, 16, 3)
    assert O.leader_layers(32, 24, 2) == [25, 27, 29, 31]
    assert [O.cache_layer_of(j, 24, 2) for j in (1, 24, 25, 26, 27, 32)] == [0, 23, 24, 24, 25, 27]
    assert O.n_cache_layers(32, 32, 1) == 32 and O.leader_layers(32, 32, 1) == []


def test_normalised_throughput_identity():
    """tokens/s x (2 x parameter count) reproduces the paper's normalised TFLOPS
    (Sec. 4.2), which confirms the 2-flops-per-parameter-per-token accounting."""
    for model, tps, ngpu, tflops in _rows("paper_normalised_throughput.txt"):
        ms = WL.configs.LLAMA_8B if model == "8b" else WL.configs.LLAMA_70B
        per_layer = ms.hidden * (ms.q_dim + 2 * ms.kv_dim) + ms.hidden * ms.q_dim + 3 * ms.hidden * ms.ffn
        params = ms.n_layers * per_layer + 2 * ms.vocab * ms.hidden
        got = float(tps) * 2 * params / int(ngpu) / 1e12
        assert got == pytest.approx(float(tflops), rel=0.03)
        # executed_flops with l = L: per token, 2 flops per decoder-layer parameter (the
        # embedding is a gather and the LM head runs once per sequence, not per token)
        sh = oracle_shape(ms)
        f = O.executed_flops(sh, ms.n_layers, 1, [4096], [0])
        assert f["gemm"] / 4096 == pytest.approx(2 * (params - 2 * ms.vocab * ms.hidden), rel=0.01)


def test_executed_flops_headline_config():
    w = WL.get_workload("8b_l16_b8x2048")
    f = O.executed_flops(oracle_shape(w.shape), w.l, w.g, [2048] * 8, [0] * 8)
    assert f["total"] == pytest.approx(1.232e14, rel=0.01)
    assert f["attn"] == pytest.approx(4.40e12, rel=0.02)
