"""Prompts that continue over a cached prefix (several new tokens on top of a
cached context) and token-by-token generation after a prompt, against the CPU
oracle on the tiny decoder."""
import sys

import pytest
import torch

import workloads as WL
from oracle import swiftkv_oracle as O
from tests import gpu_helpers as G

pytestmark = pytest.mark.gpu
TINY = WL.configs.TINY


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def tiny():
    wl = WL.get_workload("tiny")
    store = WL.make_weights(wl, "cpu", keep=True)
    return wl, store, G.device_weights(store)


def _ctx(dev_w, l, g):
    from paper_2410_03960_amd import binding as B
    return B.Context(TINY, dev_w, l, g)


def _oracle_contexts(store, batch, ctx_lens, l, g, fp8=False, scales=None):
    """Oracle cache whose first ctx_lens[b] positions of sequence b hold the
    K/V of a seeded prompt (prefilled by the oracle itself)."""
    C = O.n_cache_layers(TINY.n_layers, l, g)
    ocache = O.PagedKVCache(C, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables, fp8=fp8)
    if fp8:
        ocache.scales[:] = scales
    for b, cl in enumerate(ctx_lens):
        if cl:
            ids = WL.seeded_token_ids(7, f"ctx{b}", cl, TINY.vocab)
            sub = O.PagedKVCache(C, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables[b:b + 1], fp8=fp8)
            if fp8:
                sub.scales[:] = scales
            O.swiftkv_prefill(G.oracle_shape(TINY), G.weight_fn(store), ids, [cl], [0], l, g, sub,
                              fp8_compute_scales=False)
            s = sub.slots(0, torch.arange(cl))
            ocache.data[:, :, s] = sub.data[:, :, s]
    return ocache


@pytest.mark.parametrize("l,g,lens,ctx_lens", [
    (2, 2, [70, 1, 5, 200], [40, 17, 0, 130]),      # chunk, decode token, fresh prompt, chunk over several tiles
    (3, 1, [129, 64], [63, 64]),                    # query blocks and key tiles off the 64/128 grid, and on it
    (4, 1, [2, 300], [1, 0]),                       # l = L (no later layers), shortest chunk
    (2, 1, [30, 1, 7], [50, 9, 0]),                 # at most 80 tokens: the weight-streaming GEMM path
])
def test_chunk_over_cached_prefix(tiny, l, g, lens, ctx_lens):
    from paper_2410_03960_amd import binding as B
    wl, store, dev_w = tiny
    _say(f"chunk over cached prefix l={l} g={g} lens={lens} ctx={ctx_lens}")
    batch = WL.build_batch(wl, lens=lens, ctx=ctx_lens, shuffled=True)
    ocache = _oracle_contexts(store, batch, ctx_lens, l, g)
    ctx = _ctx(dev_w, l, g)
    cache = B.KVCache(ctx.n_cache_layers, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables, ctx_lens)
    cache.data.copy_(ocache.data.to(torch.bfloat16))
    ocache.data = ocache.data.to(torch.bfloat16).double()      # both sides start from the same bf16 context
    logits, cache, ws = G.run_gpu(ctx, batch, cache=cache)
    G.check_plan(ctx, ws, batch)
    ologits, ocache, _ = G.run_oracle(TINY, store, batch, l, g, cache=ocache)
    G.compare_caches(cache, ocache, batch, label="chunk")
    G.compare_logits(logits, ologits, label="chunk")


def test_chunk_over_cached_prefix_fp8(tiny):
    """FP8 cache with given scales: the prefix is read as code * scale, the new
    rows are stored as codes and read back the same way."""
    from paper_2410_03960_amd import binding as B
    wl, store, dev_w = tiny
    l, g = 2, 1
    lens, ctx_lens = [100, 1, 33], [75, 20, 0]
    _say("chunk over cached prefix, fp8 cache")
    batch = WL.build_batch(wl, lens=lens, ctx=ctx_lens, shuffled=True)
    C = O.n_cache_layers(TINY.n_layers, l, g)
    scales = 0.02 + 0.01 * torch.rand((C, 2, TINY.n_kv_heads), generator=torch.Generator().manual_seed(3))
    ocache = _oracle_contexts(store, batch, ctx_lens, l, g, fp8=True, scales=scales)
    ctx = _ctx(dev_w, l, g)
    cache = B.KVCache(C, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables, ctx_lens,
                      fp8=True, scale_mode=B.SWIFTKV_SCALE_USE_GIVEN)
    cache.data.copy_(ocache.data)
    cache.scales.copy_(ocache.scales)
    logits, cache, ws = G.run_gpu(ctx, batch, fp8=True, cache=cache)
    G.check_plan(ctx, ws, batch)
    ologits, ocache, _ = G.run_oracle(TINY, store, batch, l, g, fp8=True, compute_scales=False, cache=ocache)
    G.compare_caches(cache, ocache, batch, rel=G.FP8_REL, cos=G.FP8_COS, label="chunk fp8")
    G.compare_logits(logits, ologits, rel=G.FP8_REL, cos=G.FP8_COS, label="chunk fp8")


def test_prompt_in_chunks_on_the_gpu_matches_oracle_one_shot(tiny):
    """The whole prompt goes through the HIP path chunk by chunk (each call sees
    what the earlier calls cached); cache and final logits are compared with the
    oracle's one-shot prefill of the same prompt."""
    from paper_2410_03960_amd import binding as B
    wl, store, dev_w = tiny
    l, g, n = 2, 2, 333
    cuts = [0, 100, 228, 229, n]
    _say("prompt in chunks on the gpu")
    full = WL.build_batch(wl, lens=[n], ctx=[0], shuffled=True)
    ctx = _ctx(dev_w, l, g)
    cache = B.KVCache(ctx.n_cache_layers, full.n_blocks, TINY.n_kv_heads, TINY.head_dim, full.block_tables, [0])
    logits = None
    for a, b in zip(cuts[:-1], cuts[1:]):
        part = WL.build_batch(wl, lens=[b - a], ctx=[a], shuffled=True)
        part.block_tables, part.n_blocks = full.block_tables, full.n_blocks
        part.token_ids = full.token_ids[a:b].clone()
        cache.set_context_lens([a])
        logits, cache, ws = G.run_gpu(ctx, part, cache=cache)
        G.check_plan(ctx, ws, part)
    ologits, ocache, _ = G.run_oracle(TINY, store, full, l, g)
    G.compare_caches(cache, ocache, full, label="chunks")
    G.compare_logits(logits, ologits, label="chunks")


def test_workspace_sized_without_prefix_is_rejected(tiny):
    from paper_2410_03960_amd import binding as B
    wl, store, dev_w = tiny
    batch = WL.build_batch(wl, lens=[64], ctx=[4000], shuffled=False)
    ctx = _ctx(dev_w, 2, 2)
    cache = B.KVCache(ctx.n_cache_layers, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables, [4000])
    ws = torch.empty(ctx.workspace_bytes(64, 1), dtype=torch.uint8, device="cuda")
    logits = torch.empty((1, TINY.vocab), dtype=torch.float32, device="cuda")
    with pytest.raises(B.SwiftKVError) as ei:
        ctx.prefill(batch.token_ids.cuda(), [64], cache, logits, ws)
    assert ei.value.code == B.SWIFTKV_ENOSPC


def test_generation_after_prompt(tiny):
    """Autoregressive decoding (Sec. 3.1, 3.5): after the prompt each step feeds
    one token per sequence with everything before it cached.  Both sides are fed
    the oracle's greedy tokens, logits and cache are compared at every step, and
    the HIP path must pick the same token wherever the oracle's margin between
    its two best tokens exceeds the logit tolerance."""
    from paper_2410_03960_amd import binding as B
    wl, store, dev_w = tiny
    l, g, steps = 2, 2, 6
    lens = [37, 80]
    _say("generation after prompt")
    room = WL.build_batch(wl, lens=[n + steps for n in lens], ctx=[0, 0], shuffled=True)   # block tables with room to grow
    batch = WL.build_batch(wl, lens=lens, ctx=[0, 0], shuffled=True)
    batch.block_tables, batch.n_blocks = room.block_tables, room.n_blocks
    ctx = _ctx(dev_w, l, g)
    cache = B.KVCache(ctx.n_cache_layers, room.n_blocks, TINY.n_kv_heads, TINY.head_dim, room.block_tables, [0, 0])
    logits, cache, _ = G.run_gpu(ctx, batch, cache=cache)
    ologits, ocache, _ = G.run_oracle(TINY, store, batch, l, g)
    cur = list(lens)
    for step in range(steps):
        G.compare_logits(logits, ologits, label=f"step {step}")
        top2 = ologits.topk(2, dim=-1)
        nxt = top2.indices[:, 0]
        for b in range(len(lens)):
            margin = float(top2.values[b, 0] - top2.values[b, 1])
            if margin > 2 * G.BF16_REL * float(ologits[b].abs().max()):
                assert int(logits[b].argmax()) == int(nxt[b]), (step, b)
        dec = WL.build_batch(wl, lens=[1, 1], ctx=cur, shuffled=True)
        dec.block_tables, dec.n_blocks = room.block_tables, room.n_blocks
        dec.token_ids = nxt.to(torch.int32)
        cache.set_context_lens(cur)
        logits, cache, ws = G.run_gpu(ctx, dec, cache=cache)
        G.check_plan(ctx, ws, dec)
        ologits, ocache, _ = G.run_oracle(TINY, store, dec, l, g, cache=ocache)
        cur = [c + 1 for c in cur]
        G.compare_caches(cache, ocache, dec, label=f"step {step}")
    G.compare_logits(logits, ologits, label="last step")


def test_early_exit_selects_confident_rows(tiny):
    """Appendix B.4: an extra head on the layer-l output; rows whose largest
    probability exceeds the threshold return its logits, the others the ordinary
    ones; the cache is that of the plain call.  The decision compares a float32
    probability with the threshold on both sides; the head is scaled so that no
    row sits near the threshold."""
    from paper_2410_03960_amd import binding as B
    wl, store, dev_w = tiny
    l, g = 2, 2
    lens, ctx_lens = [19, 7, 30, 1, 64], [0, 0, 0, 12, 0]
    _say("early exit")
    batch = WL.build_batch(wl, lens=lens, ctx=ctx_lens, shuffled=True)
    gen = torch.Generator().manual_seed(5)
    g_ee = (1 + 0.02 * torch.randn(TINY.hidden, generator=gen)).to(torch.bfloat16)
    w_base = (0.02 * torch.randn(TINY.vocab, TINY.hidden, generator=gen))
    ocache = _oracle_contexts(store, batch, ctx_lens, l, g)
    ocache.data = ocache.data.to(torch.bfloat16).double()
    base = ocache.data.clone()
    # pick a scale for which the oracle's row maxima stay clear of the threshold
    for scale in (40.0, 60.0, 90.0, 140.0):
        w_ee = (scale * w_base).to(torch.bfloat16)
        oc = O.PagedKVCache(ocache.C, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables)
        oc.data = base.clone()
        ologits, _, oflags = O.swiftkv_prefill(G.oracle_shape(TINY), G.weight_fn(store), batch.token_ids, lens, ctx_lens, l, g, oc,
                                               early_exit=(g_ee.double(), w_ee.double(), -1.0))
        pm = torch.softmax(ologits, dim=-1).amax(dim=-1)
        if (pm > 0.97).any() and (pm < 0.92).any() and not ((pm >= 0.92) & (pm <= 0.97)).any():
            break
    else:
        pytest.skip("no scale separates the rows")
    oc = O.PagedKVCache(ocache.C, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables)
    oc.data = base.clone()
    ologits, _, oflags = O.swiftkv_prefill(G.oracle_shape(TINY), G.weight_fn(store), batch.token_ids, lens, ctx_lens, l, g, oc,
                                           early_exit=(g_ee.double(), w_ee.double(), 0.95))
    assert oflags.any() and not oflags.all()
    ctx = _ctx(dev_w, l, g)
    ctx.set_early_exit(g_ee.cuda(), w_ee.cuda(), 0.95)
    cache = B.KVCache(ctx.n_cache_layers, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables, ctx_lens)
    cache.data.copy_(base.to(torch.bfloat16))
    logits, cache, ws = G.run_gpu(ctx, batch, cache=cache)
    flags = ctx.export_exit_flags(ws, batch.n_seqs)
    torch.cuda.synchronize()
    assert flags.cpu().bool().tolist() == oflags.tolist()
    G.compare_caches(cache, oc, batch, label="early exit")
    G.compare_logits(logits, ologits, label="early exit")
    # switched off again: plain logits, no flags
    ctx.set_early_exit(None, None)
    logits2, cache2, ws2 = G.run_gpu(ctx, batch, cache=cache)
    assert int(ctx.export_exit_flags(ws2, batch.n_seqs).sum()) == 0
    plain, _, _ = G.run_oracle(TINY, store, batch, l, g, cache=oc)
    G.compare_logits(logits2, plain, label="early exit off")


@pytest.mark.parametrize("hq,hkv,hd", [(4, 4, 64), (16, 2, 64), (2, 2, 128), (8, 1, 128)])
def test_head_groupings(hq, hkv, hd):
    """Query heads per KV head 1 (plain multi-head attention), 8, and a single KV
    head (multi-query attention), with prompts, a chunk over a cached prefix and
    a decode token in one batch."""
    from paper_2410_03960_amd import binding as B
    from workloads.configs import ModelShape, Workload
    shape = ModelShape(3, 256, hq, hkv, hd, 512, 1024, 1e4, 1e-5)
    wl = Workload(f"heads_{hq}_{hkv}_{hd}", shape, l=2, g=1, seed=2301)
    store = WL.make_weights(wl, "cpu", keep=True)
    dev_w = G.device_weights(store)
    lens, ctx_lens = [150, 40, 1, 9], [0, 70, 33, 0]
    _say(f"head grouping Hq={hq} Hkv={hkv} hd={hd}")
    batch = WL.build_batch(wl, lens=lens, ctx=ctx_lens, shuffled=True)
    C = O.n_cache_layers(shape.n_layers, wl.l, wl.g)
    ocache = O.PagedKVCache(C, batch.n_blocks, hkv, hd, batch.block_tables)
    for b, cl in enumerate(ctx_lens):
        if cl:
            ids = WL.seeded_token_ids(7, f"ctx{b}", cl, shape.vocab)
            sub = O.PagedKVCache(C, batch.n_blocks, hkv, hd, batch.block_tables[b:b + 1])
            O.swiftkv_prefill(G.oracle_shape(shape), G.weight_fn(store), ids, [cl], [0], wl.l, wl.g, sub)
            s = sub.slots(0, torch.arange(cl))
            ocache.data[:, :, s] = sub.data[:, :, s]
    ctx = B.Context(shape, dev_w, wl.l, wl.g)
    cache = B.KVCache(C, batch.n_blocks, hkv, hd, batch.block_tables, ctx_lens)
    cache.data.copy_(ocache.data.to(torch.bfloat16))
    ocache.data = ocache.data.to(torch.bfloat16).double()
    logits, cache, ws = G.run_gpu(ctx, batch, cache=cache)
    G.check_plan(ctx, ws, batch)
    ologits, ocache, _ = G.run_oracle(shape, store, batch, wl.l, wl.g, cache=ocache)
    G.compare_caches(cache, ocache, batch, label="heads")
    G.compare_logits(logits, ologits, label="heads")


def test_many_short_sequences(tiny):
    """300 sequences of 1..20 tokens, a third of them over cached contexts: more
    tail rows than the weight-streaming GEMM takes (it switches to the tiled
    one), many single-query rows, most 128-query blocks nearly empty."""
    from paper_2410_03960_amd import binding as B
    wl, store, dev_w = tiny
    l, g = 2, 1
    gen = torch.Generator().manual_seed(17)
    lens = torch.randint(1, 21, (300,), generator=gen).tolist()
    ctx_lens = [int(c) if i % 3 == 0 else 0 for i, c in enumerate(torch.randint(1, 60, (300,), generator=gen).tolist())]
    _say("many short sequences")
    batch = WL.build_batch(wl, lens=lens, ctx=ctx_lens, shuffled=True)
    ocache = _oracle_contexts(store, batch, ctx_lens, l, g)
    ctx = _ctx(dev_w, l, g)
    cache = B.KVCache(ctx.n_cache_layers, batch.n_blocks, TINY.n_kv_heads, TINY.head_dim, batch.block_tables, ctx_lens)
    cache.data.copy_(ocache.data.to(torch.bfloat16))
    ocache.data = ocache.data.to(torch.bfloat16).double()
    logits, cache, ws = G.run_gpu(ctx, batch, cache=cache)
    G.check_plan(ctx, ws, batch)
    ologits, ocache, _ = G.run_oracle(TINY, store, batch, l, g, cache=ocache)
    G.compare_caches(cache, ocache, batch, label="many")
    G.compare_logits(logits, ologits, label="many")
