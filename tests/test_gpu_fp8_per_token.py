"""FP8 KV cache with one scale per token (the granularity of Appendix B.1)
against the CPU oracle: fresh prompts, prompt chunks and decode tokens over
cached contexts, small and mid-size decoders."""
import sys

import pytest
import torch

import workloads as WL
from workloads.configs import ModelShape, Workload
from oracle import swiftkv_oracle as O
from tests import gpu_helpers as G

pytestmark = pytest.mark.gpu
TINY = WL.configs.TINY


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _compare_scales(cache, ocache, batch, label):
    """Scales of every stored token.  A token's scale is the absmax of one K (V)
    row, i.e. one activation value of a pipeline whose attention reads FP8
    values: it is held to the bar of the FP8 cache values themselves (max|diff|
    over the tensor against its largest entry), per cache layer and K|V."""
    for b in range(batch.n_seqs):
        n = int(batch.context_lens[b]) + int(batch.seq_lens[b])
        s = ocache.slots(b, torch.arange(n))
        got, want = cache.scales[:, :, s.cuda()].cpu(), ocache.scales[:, :, s]
        assert (want > 0).all() and (got > 0).all()
        err = (got - want).abs().amax(dim=2) / want.amax(dim=2)
        assert (err <= G.FP8_REL).all(), f"{label}: scales of sequence {b}: {err.max():.3e}"


@pytest.mark.parametrize("l,g,lens", [(2, 2, [90, 20, 1]), (3, 1, [40, 20]), (2, 1, [300])])
def test_fresh_prompts(l, g, lens):
    from paper_2410_03960_amd import binding as B
    wl = WL.get_workload("tiny")
    store = WL.make_weights(wl, "cpu", keep=True)
    dev_w = G.device_weights(store)
    _say(f"per-token fp8, fresh prompts l={l} g={g} lens={lens}")
    batch = WL.build_batch(wl, lens=lens, shuffled=True)
    ctx = B.Context(TINY, dev_w, l, g)
    logits, cache, ws = G.run_gpu(ctx, batch, fp8=True, scale_mode=B.SWIFTKV_SCALE_PER_TOKEN)
    G.check_plan(ctx, ws, batch)
    ologits, ocache, _ = G.run_oracle(TINY, store, batch, l, g, fp8=True, per_token=True)
    _compare_scales(cache, ocache, batch, "fresh")
    G.compare_caches(cache, ocache, batch, rel=G.FP8_REL, cos=G.FP8_COS, label="per-token fp8")
    G.compare_logits(logits, ologits, rel=G.FP8_REL, cos=G.FP8_COS, label="per-token fp8")


def test_chunk_and_decode_over_cached_contexts():
    """Contexts (codes and per-token scales) come from an oracle prefill and are
    copied to the GPU cache; the call adds a chunk, a decode token and a prompt."""
    from paper_2410_03960_amd import binding as B
    wl = WL.get_workload("tiny")
    store = WL.make_weights(wl, "cpu", keep=True)
    dev_w = G.device_weights(store)
    l, g = 2, 1
    lens, ctx_lens = [100, 1, 33], [75, 20, 0]
    _say("per-token fp8, chunk + decode over cached contexts")
    batch = WL.build_batch(wl, lens=lens, ctx=ctx_lens, shuffled=True)
    C = O.n_cache_layers(TINY.n_layers, l, g)
    ocache = O.PagedKVCache(C, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables, fp8=True, per_token=True)
    for b, cl in enumerate(ctx_lens):
        if cl:
            ids = WL.seeded_token_ids(7, f"ctx{b}", cl, TINY.vocab)
            sub = O.PagedKVCache(C, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables[b:b + 1], fp8=True, per_token=True)
            O.swiftkv_prefill(G.oracle_shape(TINY), G.weight_fn(store), ids, [cl], [0], l, g, sub)
            s = sub.slots(0, torch.arange(cl))
            ocache.data[:, :, s] = sub.data[:, :, s]
            ocache.scales[:, :, s] = sub.scales[:, :, s]
    ctx = B.Context(TINY, dev_w, l, g)
    cache = B.KVCache(C, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables, ctx_lens,
                      fp8=True, scale_mode=B.SWIFTKV_SCALE_PER_TOKEN)
    cache.data.copy_(ocache.data)
    cache.scales.copy_(ocache.scales)
    logits, cache, ws = G.run_gpu(ctx, batch, fp8=True, cache=cache)
    G.check_plan(ctx, ws, batch)
    ologits, ocache, _ = G.run_oracle(TINY, store, batch, l, g, fp8=True, cache=ocache)
    _compare_scales(cache, ocache, batch, "chunk")
    G.compare_caches(cache, ocache, batch, rel=G.FP8_REL, cos=G.FP8_COS, label="per-token fp8 chunk")
    G.compare_logits(logits, ologits, rel=G.FP8_REL, cos=G.FP8_COS, label="per-token fp8 chunk")


@pytest.mark.parametrize("name,shape,l,g", [
    ("mid_hd128", ModelShape(3, 512, 4, 2, 128, 1024, 1024, 1e4, 1e-5), 2, 1),
    ("mid_hd64", ModelShape(3, 512, 8, 4, 64, 768, 1024, 1e4, 1e-5), 1, 2),
])
def test_mid_size(name, shape, l, g):
    """More than 1024 tokens: the large-GEMM path with FP8 staging of the fused KV output."""
    from paper_2410_03960_amd import binding as B
    wl = Workload(name, shape, l=l, g=g, seed=2201)
    store = WL.make_weights(wl, "cpu", keep=True)
    dev_w = G.device_weights(store)
    _say(f"per-token fp8, {name}")
    batch = WL.build_batch(wl, lens=[700, 300, 129, 1], shuffled=True)
    ctx = B.Context(shape, dev_w, l, g)
    logits, cache, ws = G.run_gpu(ctx, batch, fp8=True, scale_mode=B.SWIFTKV_SCALE_PER_TOKEN)
    G.check_plan(ctx, ws, batch)
    ologits, ocache, _ = G.run_oracle(shape, store, batch, l, g, fp8=True, per_token=True)
    _compare_scales(cache, ocache, batch, name)
    wc = G.compare_caches(cache, ocache, batch, rel=G.FP8_REL, cos=G.FP8_COS, label=name)
    wl_ = G.compare_logits(logits, ologits, rel=G.FP8_REL, cos=G.FP8_COS, label=name)
    _say(f"  worst cache rel/cos {wc}, logits {wl_}")
    logits2, cache2, _ = G.run_gpu(ctx, batch, fp8=True, scale_mode=B.SWIFTKV_SCALE_PER_TOKEN)
    assert torch.equal(cache.data, cache2.data) and torch.equal(cache.scales, cache2.scales) and torch.equal(logits, logits2)
