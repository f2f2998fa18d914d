"""Helpers for the GPU parity tests: run the HIP library and the CPU oracle on
the same seeded inputs and compare per tensor."""
import torch

import workloads as WL
from oracle import swiftkv_oracle as O
from tests.helpers import cosine, oracle_shape, rel_err, weight_fn

BF16_REL, BF16_COS = 2e-2, 0.999      # bf16 K/V caches and logits vs the oracle
FP8_REL, FP8_COS = 1e-1, 0.995        # FP8 KV path


def device_weights(store_cpu_or_shape, seed=None):
    """dict name -> bf16 CUDA tensor for every weight of the model."""
    if isinstance(store_cpu_or_shape, WL.WeightStore):
        shape, seed = store_cpu_or_shape.shape, store_cpu_or_shape.seed
    else:
        shape = store_cpu_or_shape
    st = WL.WeightStore(shape, seed, device="cuda", keep=True).materialize()
    return dict(st._cache)


def run_gpu(ctx, batch, fp8=False, scale_mode=0, cache=None, stream=None):
    from paper_2410_03960_amd import binding as B
    sh = ctx.shape
    if cache is None:
        cache = B.KVCache(ctx.n_cache_layers, batch.n_blocks, sh.n_kv_heads, sh.head_dim,
                          batch.block_tables, batch.context_lens.tolist(), fp8=fp8, scale_mode=scale_mode)
    T, nseq = batch.n_tokens, batch.n_seqs
    prefix = sum(int(c) for c, n in zip(batch.context_lens.tolist(), batch.seq_lens.tolist()) if n > 1)
    nbytes = ctx.workspace_bytes(T, nseq, B.SWIFTKV_KV_FP8_E4M3 if fp8 else B.SWIFTKV_KV_BF16, prefix)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    logits = torch.empty((nseq, sh.vocab), dtype=torch.float32, device="cuda")
    ids = batch.token_ids.cuda()
    ctx.prefill(ids, batch.seq_lens.tolist(), cache, logits, ws, stream)
    torch.cuda.synchronize()
    return logits, cache, ws


def run_oracle(shape, store, batch, l, g, dtype=torch.float64, fp8=False, compute_scales=True,
               cache=None, seq_subset=None, per_token=False):
    C = O.n_cache_layers(shape.n_layers, l, g)
    if cache is None:
        cache = O.PagedKVCache(C, batch.n_blocks, shape.n_kv_heads, shape.head_dim, batch.block_tables,
                               dtype=dtype, fp8=fp8, per_token=per_token)
    logits, hl = O.swiftkv_prefill(oracle_shape(shape), weight_fn(store), batch.token_ids,
                                   batch.seq_lens.tolist(), batch.context_lens.tolist(), l, g, cache,
                                   dtype=dtype, fp8_compute_scales=compute_scales, seq_subset=seq_subset)
    return logits, cache, hl


def gpu_cache_logical(cache, c, kvsel, slots):
    """Values (float32) the GPU cache holds at `slots` of cache layer c."""
    raw = cache.data[c, kvsel][slots.to(cache.data.device)]
    if cache.fp8:
        tab = O.fp8_e4m3fn_decode_table().float().to(raw.device)
        if cache.scales.shape[-1] == cache.data.shape[2]:       # one scale per slot
            return tab[raw.long()] * cache.scales[c, kvsel][slots.to(raw.device)][:, None, None]
        return tab[raw.long()] * cache.scales[c, kvsel][None, :, None]
    return raw.float()


def compare_caches(gpu_cache, ora_cache, batch, seqs=None, rel=BF16_REL, cos=BF16_COS, label=""):
    """Per cache layer and K/V: compare every stored row of the given sequences."""
    seqs = range(batch.n_seqs) if seqs is None else seqs
    worst = (0.0, 1.0)
    for c in range(ora_cache.C):
        for kvsel in (0, 1):
            got, want = [], []
            for b in seqs:
                n = int(batch.context_lens[b]) + int(batch.seq_lens[b])
                s = ora_cache.slots(b, torch.arange(n))
                want.append(ora_cache.read(c, b, n)[kvsel].float())
                got.append(gpu_cache_logical(gpu_cache, c, kvsel, s).cpu())
            got, want = torch.cat(got), torch.cat(want)
            r, cs = rel_err(got, want), cosine(got, want)
            worst = (max(worst[0], r), min(worst[1], cs))
            assert r <= rel and cs >= cos, f"{label} cache layer {c} {'KV'[kvsel]}: rel {r:.3e} cos {cs:.6f}"
    return worst


def compare_logits(gpu_logits, ora_logits, seqs=None, rel=BF16_REL, cos=BF16_COS, label=""):
    seqs = range(ora_logits.shape[0]) if seqs is None else seqs
    worst = (0.0, 1.0)
    for b in seqs:
        r, cs = rel_err(gpu_logits[b].cpu(), ora_logits[b]), cosine(gpu_logits[b].cpu(), ora_logits[b])
        worst = (max(worst[0], r), min(worst[1], cs))
        assert r <= rel and cs >= cos, f"{label} logits of sequence {b}: rel {r:.3e} cos {cs:.6f}"
    return worst


def check_plan(ctx, ws, batch):
    """Integer plan must match the oracle's bit for bit."""
    slots, pos, cu, last = ctx.export_plan(ws, batch.n_tokens, batch.n_seqs)
    ocu, opos, oslots, olast = O.slot_mapping(batch.block_tables, batch.context_lens.tolist(), batch.seq_lens.tolist())
    assert torch.equal(slots.cpu(), oslots) and torch.equal(pos.cpu(), opos)
    assert torch.equal(cu.cpu(), ocu) and torch.equal(last.cpu(), olast)
