"""Pins the oracle's forward pass to an independent implementation: the
Hugging Face Llama model (CPU, float64).  All run on tiny shapes."""
import math

import pytest
import torch

import workloads as WL
from oracle import swiftkv_oracle as O
from tests.helpers import (all_weights_dict, dict_weight_fn, hf_llama, identity_tables,
                           oracle_shape)

MS = WL.configs.TINY
# The library model forms its RMSNorm variance and rotary angles in float32 even
# when run in float64, so agreement is to float32 rounding (values are O(1)).
TOL = 2e-5


@pytest.fixture(scope="module")
def wd():
    return all_weights_dict(WL.WeightStore(MS, 77), torch.float64)


@pytest.fixture(scope="module")
def hf(wd):
    return hf_llama(MS, wd)


def _ids(n, seed=5):
    return WL.seeded_token_ids(seed, "ids", n, MS.vocab)


def _run_oracle(wd, ids, lens, l, g, ctx=None, **kw):
    ctx = ctx or [0] * len(lens)
    bt, nb = identity_tables(lens, ctx)
    C = O.n_cache_layers(MS.n_layers, l, g)
    cache = O.PagedKVCache(C, nb, MS.n_kv_heads, MS.head_dim, bt)
    out = O.swiftkv_prefill(oracle_shape(MS), dict_weight_fn(wd), ids, lens, ctx, l, g, cache, **kw)
    return (out[0], cache, out[1]) + tuple(out[2:])


def _hf_forward(hf, ids):
    with torch.no_grad():
        out = hf(ids.long()[None], output_hidden_states=True, use_cache=True)
    ks = [out.past_key_values.layers[j].keys[0].transpose(0, 1) for j in range(MS.n_layers)]
    vs = [out.past_key_values.layers[j].values[0].transpose(0, 1) for j in range(MS.n_layers)]
    return out.logits[0], out.hidden_states, ks, vs


def test_l_equals_L_is_standard_prefill(wd, hf):
    """With l = L SwiftKV is ordinary prefill: last-token logits and every
    layer's post-RoPE K and V equal the library model's, for a ragged batch."""
    lens = [37, 1, 20]
    ids = _ids(sum(lens))
    logits, cache, _ = _run_oracle(wd, ids, lens, MS.n_layers, 1)
    off = 0
    for b, n in enumerate(lens):
        ref_logits, _, ks, vs = _hf_forward(hf, ids[off:off + n])
        assert torch.allclose(logits[b], ref_logits[-1], atol=TOL, rtol=0)
        for j in range(MS.n_layers):
            k, v = cache.read(j, b, n)
            assert torch.allclose(k, ks[j], atol=TOL, rtol=0)
            assert torch.allclose(v, vs[j], atol=TOL, rtol=0)
        off += n


@pytest.mark.parametrize("l,g", [(2, 1), (2, 2), (1, 3), (3, 1)])
def test_later_layer_kv_come_from_hidden_l(wd, hf, l, g):
    """Eq. 2: cache layer l+p holds W_K/W_V of the group's first layer applied to
    that layer's input RMSNorm of the library model's hidden state after layer
    l, K rotated by the library's rotary embedding; layers <= l equal the
    library model's own cache."""
    from transformers.models.llama.modeling_llama import apply_rotary_pos_emb
    n = 29
    ids = _ids(n, 9)
    _, cache, hl = _run_oracle(wd, ids, [n], l, g)
    _, hs, ks, vs = _hf_forward(hf, ids)
    assert torch.allclose(hl[0], hs[l][0], atol=TOL, rtol=0)
    for j in range(l):
        k, v = cache.read(j, 0, n)
        assert torch.allclose(k, ks[j], atol=TOL) and torch.allclose(v, vs[j], atol=TOL)
    pos = torch.arange(n)[None]
    cos, sin = hf.model.rotary_emb(hs[l], pos)
    P = (MS.n_layers - l) // g
    assert cache.C == l + P
    for p in range(P):
        layer = hf.model.layers[l + p * g]
        with torch.no_grad():
            a = layer.input_layernorm(hs[l])
            kk = layer.self_attn.k_proj(a).view(1, n, MS.n_kv_heads, MS.head_dim).transpose(1, 2)
            vv = layer.self_attn.v_proj(a).view(1, n, MS.n_kv_heads, MS.head_dim).transpose(1, 2)
            _, kk = apply_rotary_pos_emb(kk, kk, cos, sin)
        k, v = cache.read(l + p, 0, n)
        assert torch.allclose(k, kk[0].transpose(0, 1), atol=TOL, rtol=0)
        assert torch.allclose(v, vv[0].transpose(0, 1), atol=TOL, rtol=0)


def test_reduces_to_standard_model_when_later_layers_add_nothing(wd):
    """If W_O and W_down of every layer > l are zero the residual stream stops
    changing after layer l, so every later layer's true input *is* x_{l+1}: the
    SwiftKV caches and logits must then equal the library model's ordinary
    full prefill."""
    l, n = 2, 23
    w2 = dict(wd)
    for j in range(l, MS.n_layers):
        w2[f"wo.{j}"] = torch.zeros_like(wd[f"wo.{j}"])
        w2[f"wdown.{j}"] = torch.zeros_like(wd[f"wdown.{j}"])
    hf2 = hf_llama(MS, w2)
    ids = _ids(n, 3)
    logits, cache, _ = _run_oracle(w2, ids, [n], l, 1)
    ref_logits, _, ks, vs = _hf_forward(hf2, ids)
    for j in range(MS.n_layers):
        k, v = cache.read(j, 0, n)
        assert torch.allclose(k, ks[j], atol=TOL) and torch.allclose(v, vs[j], atol=TOL)
    assert torch.allclose(logits[0], ref_logits[-1], atol=TOL)


@pytest.mark.parametrize("l,g", [(2, 1), (2, 2), (1, 3)])
def test_tail_against_library_modules(wd, hf, l, g):
    """Last-token logits for l < L, rebuilt from the library model's own modules:
    each later layer's norm / q_proj / rotary / o_proj / MLP applied to the last
    row, with torch's scaled_dot_product_attention over the shared cache."""
    from transformers.models.llama.modeling_llama import apply_rotary_pos_emb
    import torch.nn.functional as F
    n = 26
    ids = _ids(n, 11)
    logits, cache, hl = _run_oracle(wd, ids, [n], l, g)
    rep = MS.n_q_heads // MS.n_kv_heads
    with torch.no_grad():
        t = hl[0][-1:][None]                                   # [1, 1, d]
        cos, sin = hf.model.rotary_emb(t, torch.tensor([[n - 1]]))
        for j in range(l + 1, MS.n_layers + 1):
            layer = hf.model.layers[j - 1]
            k, v = cache.read(O.cache_layer_of(j, l, g), 0, n)
            a = layer.input_layernorm(t)
            q = layer.self_attn.q_proj(a).view(1, 1, MS.n_q_heads, MS.head_dim).transpose(1, 2)
            q, _ = apply_rotary_pos_emb(q, q, cos, sin)
            kk = k.transpose(0, 1).repeat_interleave(rep, dim=0)[None]
            vv = v.transpose(0, 1).repeat_interleave(rep, dim=0)[None]
            o = F.scaled_dot_product_attention(q, kk, vv)       # one query sees all n keys
            o = o.transpose(1, 2).reshape(1, 1, -1)
            t = t + layer.self_attn.o_proj(o)
            t = t + layer.mlp(layer.post_attention_layernorm(t))
        ref = hf.lm_head(hf.model.norm(t))[0, 0]
    assert torch.allclose(logits[0], ref, atol=TOL, rtol=0)


def test_tail_on_every_token_selects_same_last_row(wd):
    ids = _ids(19, 2)
    a, ca, _ = _run_oracle(wd, ids, [19], 2, 2)
    b, cb, _ = _run_oracle(wd, ids, [19], 2, 2, all_token_tail=True)
    assert torch.allclose(a, b, atol=1e-12) and torch.equal(ca.data, cb.data)


def test_prefix_prefill_gives_same_cache(wd):
    """Causality: prefilling the first n tokens alone leaves the same K/V in
    every cache layer as the first n positions of the longer prompt."""
    ids = _ids(45, 8)
    _, c_long, _ = _run_oracle(wd, ids, [45], 2, 2)
    _, c_short, _ = _run_oracle(wd, ids[:17], [17], 2, 2)
    for c in range(c_long.C):
        kl, vl = c_long.read(c, 0, 17)
        ks, vs = c_short.read(c, 0, 17)
        assert torch.allclose(kl, ks, atol=1e-12) and torch.allclose(vl, vs, atol=1e-12)


def test_changing_a_token_leaves_earlier_cache_entries(wd):
    ids = _ids(30, 4)
    ids2 = ids.clone()
    ids2[20] = (ids2[20] + 1) % MS.vocab
    _, c1, _ = _run_oracle(wd, ids, [30], 2, 1)
    _, c2, _ = _run_oracle(wd, ids2, [30], 2, 1)
    for c in range(c1.C):
        k1, _ = c1.read(c, 0, 30)
        k2, _ = c2.read(c, 0, 30)
        assert torch.equal(k1[:20], k2[:20]) and not torch.equal(k1[20:], k2[20:])


def test_decode_token_with_context_matches_prefill_of_longer_prompt(wd):
    """A sequence with n-1 cached tokens and one new token must give the logits
    and the new cache row of an n-token prompt prefill (cache rows for the
    context are copied from that prefill)."""
    n, l, g = 21, 2, 2
    ids = _ids(n, 6)
    full_logits, c_full, _ = _run_oracle(wd, ids, [n], l, g)
    bt, nb = identity_tables([1], [n - 1])
    cache = O.PagedKVCache(c_full.C, nb, MS.n_kv_heads, MS.head_dim, bt)
    cache.data[:, :, : n - 1] = c_full.data[:, :, : n - 1]
    logits, _ = O.swiftkv_prefill(oracle_shape(MS), dict_weight_fn(wd), ids[-1:], [1], [n - 1], l, g, cache)
    assert torch.allclose(logits[0], full_logits[0], atol=1e-10)
    assert torch.allclose(cache.data[:, :, :n], c_full.data[:, :, :n], atol=1e-12)


@pytest.mark.parametrize("l,g,cuts", [(2, 2, [17]), (2, 1, [5, 6, 30]), (3, 1, [16, 32]), (4, 1, [1, 20])])
def test_chunked_prefill_matches_one_shot(wd, l, g, cuts):
    """A prompt fed in chunks (each call: what is cached so far as context, the
    next chunk as new tokens) must leave the cache of a one-shot prefill and,
    after the last chunk, its logits: attention is causal and every other step
    acts per token.  The one-shot result is pinned to the library model above."""
    n = 41
    ids = _ids(n, 21)
    full_logits, c_full, _ = _run_oracle(wd, ids, [n], l, g)
    bt, nb = identity_tables([n], [0])
    cache = O.PagedKVCache(c_full.C, nb, MS.n_kv_heads, MS.head_dim, bt)
    bounds = [0] + cuts + [n]
    logits = None
    for a, b in zip(bounds[:-1], bounds[1:]):
        logits, _ = O.swiftkv_prefill(oracle_shape(MS), dict_weight_fn(wd), ids[a:b], [b - a], [a], l, g, cache)
        # positions past the chunk are still untouched
        assert torch.count_nonzero(cache.data[:, :, b:n]) == 0
    assert torch.allclose(logits[0], full_logits[0], atol=1e-10)
    assert torch.allclose(cache.data[:, :, :n], c_full.data[:, :, :n], atol=1e-12)


def test_chunk_and_decode_and_fresh_prompt_in_one_batch(wd):
    """A batch mixing a chunk over a cached prefix, a decode token and a fresh
    prompt gives, per sequence, what each gives alone (sequences never mix)."""
    l, g = 2, 2
    idsA, idsB, idsC = _ids(37, 31), _ids(12, 32), _ids(9, 33)
    sh, wf = oracle_shape(MS), dict_weight_fn(wd)
    fullA, cA, _ = _run_oracle(wd, idsA, [37], l, g)
    fullB, cB, _ = _run_oracle(wd, idsB, [12], l, g)
    fullC, cC, _ = _run_oracle(wd, idsC, [9], l, g)
    lens, ctx = [17, 1, 9], [20, 11, 0]
    bt, nb = identity_tables(lens, ctx)
    cache = O.PagedKVCache(cA.C, nb, MS.n_kv_heads, MS.head_dim, bt)
    for c in range(cA.C):
        kA, vA = cA.read(c, 0, 20)
        kB, vB = cB.read(c, 0, 11)
        cache.write(c, 0, torch.arange(20), kA, vA)
        cache.write(c, 1, torch.arange(11), kB, vB)
    toks = torch.cat([idsA[20:], idsB[11:], idsC])
    logits, _ = O.swiftkv_prefill(sh, wf, toks, lens, ctx, l, g, cache)
    for b, (full, cref, n) in enumerate([(fullA, cA, 37), (fullB, cB, 12), (fullC, cC, 9)]):
        assert torch.allclose(logits[b], full[0], atol=1e-10)
        for c in range(cA.C):
            k, v = cache.read(c, b, n)
            kr, vr = cref.read(c, 0, n)
            assert torch.allclose(k, kr, atol=1e-12) and torch.allclose(v, vr, atol=1e-12)


def test_per_token_fp8_cache_is_independent_of_batching(wd):
    """With per-token scales nothing a token stores depends on what else is in
    the call: a prompt fed in chunks leaves exactly the codes and scales of the
    one-shot prefill, and a batch of two prompts those of each prompt alone."""
    l, g, n = 2, 2, 41
    sh, wf = oracle_shape(MS), dict_weight_fn(wd)
    ids = _ids(n, 21)
    C = O.n_cache_layers(MS.n_layers, l, g)
    bt, nb = identity_tables([n], [0])
    one = O.PagedKVCache(C, nb, MS.n_kv_heads, MS.head_dim, bt, fp8=True, per_token=True)
    full_logits, _ = O.swiftkv_prefill(sh, wf, ids, [n], [0], l, g, one)
    parts = O.PagedKVCache(C, nb, MS.n_kv_heads, MS.head_dim, bt, fp8=True, per_token=True)
    for a, b in ((0, 16), (16, 17), (17, n)):
        logits, _ = O.swiftkv_prefill(sh, wf, ids[a:b], [b - a], [a], l, g, parts)
    assert torch.equal(one.data[:, :, :n], parts.data[:, :, :n]) and torch.equal(one.scales[:, :, :n], parts.scales[:, :, :n])
    assert torch.allclose(logits[0], full_logits[0], atol=1e-10)
    # and close to the unquantised result (relative error of e4m3 is at most 2^-4 per element)
    plain_logits, plain, _ = _run_oracle(wd, ids, [n], l, g)
    for c in range(C):
        kq, vq = one.read(c, 0, n)
        kp, vp = plain.read(c, 0, n)
        assert (kq - kp).abs().max() <= 0.07 * kp.abs().max() and (vq - vp).abs().max() <= 0.07 * vp.abs().max()
    # two prompts in one batch
    ids2 = _ids(13, 22)
    bt2, nb2 = identity_tables([n, 13], [0, 0])
    both = O.PagedKVCache(C, nb2, MS.n_kv_heads, MS.head_dim, bt2, fp8=True, per_token=True)
    O.swiftkv_prefill(sh, wf, torch.cat([ids, ids2]), [n, 13], [0, 0], l, g, both)
    s0 = both.slots(0, torch.arange(n))
    assert torch.equal(both.data[:, :, s0], one.data[:, :, :n]) and torch.equal(both.scales[:, :, s0], one.scales[:, :, :n])


def test_early_exit_rule(wd):
    """Appendix B.4: a threshold nobody reaches changes nothing; a threshold
    everybody passes returns the extra head applied to the normalised layer-l
    output (rebuilt here from the returned hidden state with library ops); a
    peaked head makes exactly the confident rows exit; the cache never changes."""
    l, g = 2, 2
    lens = [19, 7, 30]
    ids = _ids(sum(lens), 41)
    sh, wf = oracle_shape(MS), dict_weight_fn(wd)
    plain, c_plain, hl = _run_oracle(wd, ids, lens, l, g)
    gen = torch.Generator().manual_seed(5)
    g_ee = 1 + 0.02 * torch.randn(MS.hidden, generator=gen, dtype=torch.float64)
    w_ee = 0.02 * torch.randn(MS.vocab, MS.hidden, generator=gen, dtype=torch.float64)
    never, c1, _, ex = _run_oracle(wd, ids, lens, l, g, early_exit=(g_ee, w_ee, 1.0))
    assert not ex.any() and torch.equal(never, plain) and torch.equal(c1.data, c_plain.data)
    always, c2, _, ex = _run_oracle(wd, ids, lens, l, g, early_exit=(g_ee, w_ee, -1.0))
    assert ex.all() and torch.equal(c2.data, c_plain.data)
    for b in range(3):
        x = hl[b][-1]
        want = torch.nn.functional.linear(torch.nn.functional.rms_norm(x, (MS.hidden,), g_ee, MS.rms_eps), w_ee)
        assert torch.allclose(always[b], want, atol=1e-10)
    # a head that is confident on some rows only: scale the logits until the row maxima straddle 0.95
    pm = torch.softmax(always * 60.0, dim=-1).amax(dim=-1)
    assert pm.min() < 0.94 and (pm > 0.96).any() and not ((pm > 0.94) & (pm < 0.96)).any(), pm
    mixed, c3, _, ex = _run_oracle(wd, ids, lens, l, g, early_exit=(g_ee, 60.0 * w_ee, 0.95))
    assert ex.tolist() == (pm > 0.95).tolist() and torch.equal(c3.data, c_plain.data)
    for b in range(3):
        assert torch.allclose(mixed[b], 60.0 * always[b] if ex[b] else plain[b], atol=1e-9)


def test_sequence_order_only_permutes_outputs(wd):
    lens = [9, 14]
    ids = _ids(23, 12)
    la, ca, _ = _run_oracle(wd, ids, lens, 2, 1)
    ids_sw = torch.cat([ids[9:], ids[:9]])
    lb, cb, _ = _run_oracle(wd, ids_sw, [14, 9], 2, 1)
    assert torch.allclose(la[0], lb[1], atol=1e-12) and torch.allclose(la[1], lb[0], atol=1e-12)
    for c in range(ca.C):
        assert torch.allclose(ca.read(c, 0, 9)[0], cb.read(c, 1, 9)[0], atol=1e-12)


def test_one_token_prompt_closed_form(wd):
    """n = 1: softmax over one key is 1, so each attention output is that
    layer's V row (query heads copy their KV head)."""
    l, g = 2, 2
    ids = _ids(1, 13)
    logits, cache, hl = _run_oracle(wd, ids, [1], l, g)
    sh = oracle_shape(MS)
    rep = MS.n_q_heads // MS.n_kv_heads
    t = hl[0]
    for j in range(l + 1, MS.n_layers + 1):
        v = cache.read(O.cache_layer_of(j, l, g), 0, 1)[1]          # [1, Hkv, hd]
        o = v.repeat_interleave(rep, dim=1).reshape(1, -1)
        u = t + o @ wd[f"wo.{j-1}"].T
        m = O.rmsnorm(u, wd[f"norm2.{j-1}"], MS.rms_eps)
        gate = m @ wd[f"wgate.{j-1}"].T
        t = u + (torch.nn.functional.silu(gate) * (m @ wd[f"wup.{j-1}"].T)) @ wd[f"wdown.{j-1}"].T
    ref = O.rmsnorm(t, wd["final_norm"], MS.rms_eps) @ wd["lm_head"].T
    assert torch.allclose(logits[0], ref[0], atol=1e-10)


def test_block_table_permutation_leaves_logical_cache(wd):
    lens = [20, 33]
    ids = _ids(53, 14)
    _, c1, _ = _run_oracle(wd, ids, lens, 2, 1)
    bt, nb = identity_tables(lens)
    perm = torch.from_numpy(WL.seeded_permutation(3, "p", nb + 4)).to(torch.int32)
    bt2 = perm[bt.long()]
    c2 = O.PagedKVCache(c1.C, nb + 4, MS.n_kv_heads, MS.head_dim, bt2)
    O.swiftkv_prefill(oracle_shape(MS), dict_weight_fn(wd), ids, lens, [0, 0], 2, 1, c2)
    for c in range(c1.C):
        for b, n in enumerate(lens):
            assert torch.equal(c1.read(c, b, n)[0], c2.read(c, b, n)[0])
            assert torch.equal(c1.read(c, b, n)[1], c2.read(c, b, n)[1])
