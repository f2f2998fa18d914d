"""Parity with the CPU oracle on two mid-size decoders whose dimensions are
multiples of 256 and whose batches have more than 1024 tokens: the smallest
cases that take the large-GEMM paths (fragment-order weights, 64-column wave
tiles with RoPE inside a wave tile for head_dim 128 and 64, fused KV scatter,
FP8 staging + absmax) and, with the minimal pack buffer, the LDS-staged loop."""
import sys

import pytest
import torch

import workloads as WL
from workloads.configs import ModelShape, Workload
from tests import gpu_helpers as G

pytestmark = pytest.mark.gpu

MID = {
    "hd128": Workload("mid_hd128", ModelShape(3, 512, 4, 2, 128, 1024, 1024, 1e4, 1e-5), l=2, g=1, seed=2101),
    "hd64": Workload("mid_hd64", ModelShape(3, 512, 8, 4, 64, 768, 1024, 1e4, 1e-5), l=1, g=2, seed=2102),
}
LENS = [700, 300, 129, 1]          # 1130 tokens: above the 1024-row threshold, ragged 256-row tiles


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", params=sorted(MID))
def mid(request):
    wl = MID[request.param]
    store = WL.make_weights(wl, "cpu", keep=True)
    return wl, store, G.device_weights(store)


@pytest.mark.parametrize("packed", [True, False])
@pytest.mark.parametrize("fp8", [False, True])
def test_mid_shapes_match_oracle(mid, packed, fp8):
    from paper_2410_03960_amd import binding as B
    wl, store, dev_w = mid
    _say(f"{wl.name} packed={packed} fp8={fp8}")
    ctx = B.Context(wl.shape, dev_w, wl.l, wl.g, packed_weights=packed)
    assert (B.pack_bytes(wl.shape, wl.l, wl.g) > B.pack_bytes(wl.shape, wl.l, wl.g, minimum=True)) and \
        ctx.pack_buf.numel() == B.pack_bytes(wl.shape, wl.l, wl.g, minimum=not packed)
    batch = WL.build_batch(wl, lens=LENS, shuffled=True)
    if fp8:
        logits, cache, ws = G.run_gpu(ctx, batch, fp8=True, scale_mode=B.SWIFTKV_SCALE_COMPUTE_ABSMAX)
        ologits, ocache, _ = G.run_oracle(wl.shape, store, batch, wl.l, wl.g, fp8=True, compute_scales=True)
        assert G.rel_err(cache.scales.cpu(), ocache.scales) <= 2e-2
        rel, cos = G.FP8_REL, G.FP8_COS
    else:
        logits, cache, ws = G.run_gpu(ctx, batch)
        ologits, ocache, _ = G.run_oracle(wl.shape, store, batch, wl.l, wl.g)
        rel, cos = G.BF16_REL, G.BF16_COS
    G.check_plan(ctx, ws, batch)
    wc = G.compare_caches(cache, ocache, batch, rel=rel, cos=cos, label=wl.name)
    wlg = G.compare_logits(logits, ologits, rel=rel, cos=cos, label=wl.name)
    _say(f"  worst cache rel/cos {wc}, logits {wlg}")
    # a repeated call reproduces its bytes exactly
    logits2, cache2, _ = G.run_gpu(ctx, batch, fp8=fp8, scale_mode=B.SWIFTKV_SCALE_COMPUTE_ABSMAX if fp8 else 0)
    assert torch.equal(cache.data, cache2.data) and torch.equal(logits, logits2)


def test_mid_prompt_in_two_chunks(mid):
    """A 1500-token prompt fed as 1100 + 400 tokens next to a fresh prompt and a
    decode token (the second call reads the first call's cache as its prefix);
    compared with the oracle's one-shot prefill of the same sequences."""
    from paper_2410_03960_amd import binding as B
    wl, store, dev_w = mid
    _say(f"{wl.name} prompt in two chunks")
    ctx = B.Context(wl.shape, dev_w, wl.l, wl.g)
    sh = wl.shape
    n0, cut = 1500, 1100
    full = WL.build_batch(wl, lens=[n0, 700, 61], shuffled=True)
    cache = B.KVCache(ctx.n_cache_layers, full.n_blocks, sh.n_kv_heads, sh.head_dim, full.block_tables, [0, 0, 0])
    off1, off2 = n0, n0 + 700
    # call 1: first 1100 tokens of sequence 0, first 60 tokens of sequence 2
    first = WL.build_batch(wl, lens=[cut, 60], shuffled=True)
    first.block_tables, first.n_blocks = full.block_tables[[0, 2]].contiguous(), full.n_blocks
    first.token_ids = torch.cat([full.token_ids[:cut], full.token_ids[off2:off2 + 60]])
    c1 = B.KVCache(ctx.n_cache_layers, full.n_blocks, sh.n_kv_heads, sh.head_dim, first.block_tables, [0, 0])
    c1.data = cache.data
    G.run_gpu(ctx, first, cache=c1)
    # call 2: the rest of sequence 0 over its cached prefix, sequence 1 fresh, sequence 2's last token as a decode token
    second = WL.build_batch(wl, lens=[n0 - cut, 700, 1], ctx=[cut, 0, 60], shuffled=True)
    second.block_tables, second.n_blocks = full.block_tables, full.n_blocks
    second.token_ids = torch.cat([full.token_ids[cut:n0], full.token_ids[off1:off2], full.token_ids[off2 + 60:off2 + 61]])
    cache.set_context_lens([cut, 0, 60])
    logits, cache, ws = G.run_gpu(ctx, second, cache=cache)
    G.check_plan(ctx, ws, second)
    ologits, ocache, _ = G.run_oracle(sh, store, full, wl.l, wl.g)
    wc = G.compare_caches(cache, ocache, full, label=wl.name)
    wlg = G.compare_logits(logits, ologits, label=wl.name)
    _say(f"  worst cache rel/cos {wc}, logits {wlg}")


@pytest.mark.parametrize("n_seqs", [33, 40, 72, 80, 81])
def test_mid_decode_batches_of_33_to_80_rows(mid, n_seqs):
    """One new token for each of 33 .. 81 sequences over cached contexts of 1..90
    tokens (the contexts are the oracle's own prefill of seeded prompts): a batch
    of 3 .. 5 sixteen-row blocks (81: one row more than the weight-streaming GEMM
    takes, the tiled GEMM runs instead), so every projection of the full layers and of the
    tail goes through the weight-streaming GEMM's form for 33..80 rows (K slices
    in sequence; fp32 + consumer-side K-split sums for Q/K/V, residual, SwiGLU
    and bf16 epilogues); the model with ffn 768 keeps the first form for `down`."""
    from oracle import swiftkv_oracle as O
    from paper_2410_03960_amd import binding as B
    wl, store, dev_w = mid
    sh = wl.shape
    _say(f"{wl.name} decode batch of {n_seqs}")
    gen = torch.Generator().manual_seed(100 + n_seqs)
    ctx_lens = torch.randint(1, 91, (n_seqs,), generator=gen).tolist()
    batch = WL.build_batch(wl, lens=[1] * n_seqs, ctx=ctx_lens, shuffled=True)
    C = O.n_cache_layers(sh.n_layers, wl.l, wl.g)
    ocache = O.PagedKVCache(C, batch.n_blocks, sh.n_kv_heads, sh.head_dim, batch.block_tables)
    for b, cl in enumerate(ctx_lens):
        ids = WL.seeded_token_ids(11, f"{wl.name}ctx{b}", cl, sh.vocab)
        sub = O.PagedKVCache(C, batch.n_blocks, sh.n_kv_heads, sh.head_dim, batch.block_tables[b:b + 1])
        O.swiftkv_prefill(G.oracle_shape(sh), G.weight_fn(store), ids, [cl], [0], wl.l, wl.g, sub)
        s = sub.slots(0, torch.arange(cl))
        ocache.data[:, :, s] = sub.data[:, :, s]
    ctx = B.Context(sh, dev_w, wl.l, wl.g)
    cache = B.KVCache(ctx.n_cache_layers, batch.n_blocks, sh.n_kv_heads, sh.head_dim, batch.block_tables, ctx_lens)
    cache.data.copy_(ocache.data.to(torch.bfloat16))
    ocache.data = ocache.data.to(torch.bfloat16).double()     # both sides read the same bf16 contexts
    logits, cache, ws = G.run_gpu(ctx, batch, cache=cache)
    G.check_plan(ctx, ws, batch)
    ologits, ocache, _ = G.run_oracle(sh, store, batch, wl.l, wl.g, cache=ocache)
    wc = G.compare_caches(cache, ocache, batch, label=wl.name)
    wlg = G.compare_logits(logits, ologits, label=wl.name)
    _say(f"  worst cache rel/cos {wc}, logits {wlg}")
    logits2, cache2, _ = G.run_gpu(ctx, batch, cache=cache)
    assert torch.equal(logits, logits2)
