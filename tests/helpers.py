"""Shared test plumbing: adapts the seeded workloads to the oracle's inputs and
builds the Hugging Face Llama CPU model used to pin the oracle."""
import torch

import workloads as WL
from oracle import swiftkv_oracle as O


def oracle_shape(ms) -> O.Shape:
    return O.Shape(ms.n_layers, ms.hidden, ms.n_q_heads, ms.n_kv_heads, ms.head_dim,
                   ms.ffn, ms.vocab, ms.rope_theta, ms.rms_eps)


def weight_fn(store):
    """oracle WeightFn over a WeightStore (bf16 values, upcast by the oracle)."""
    def f(name, layer0=None):
        return store.get(name, layer0)
    return f


def dict_weight_fn(d):
    def f(name, layer0=None):
        return d[name if layer0 is None else f"{name}.{layer0}"]
    return f


def all_weights_dict(store, dtype=torch.float64):
    ms = store.shape
    d = {n: store.get(n).to(dtype) for n in ("embed", "final_norm", "lm_head")}
    for j in range(ms.n_layers):
        for n in ("norm1", "wq", "wk", "wv", "wo", "norm2", "wgate", "wup", "wdown"):
            d[f"{n}.{j}"] = store.get(n, j).to(dtype)
    return d


def hf_llama(ms, wd):
    """Hugging Face LlamaForCausalLM (CPU, float64, eager attention) holding `wd`."""
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=ms.vocab, hidden_size=ms.hidden, intermediate_size=ms.ffn,
                      num_hidden_layers=ms.n_layers, num_attention_heads=ms.n_q_heads,
                      num_key_value_heads=ms.n_kv_heads, head_dim=ms.head_dim,
                      rms_norm_eps=ms.rms_eps, rope_theta=ms.rope_theta, attention_bias=False,
                      mlp_bias=False, tie_word_embeddings=False, max_position_embeddings=65536)
    cfg._attn_implementation = "eager"
    m = LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": wd["embed"], "model.norm.weight": wd["final_norm"],
          "lm_head.weight": wd["lm_head"]}
    names = {"norm1": "input_layernorm", "wq": "self_attn.q_proj", "wk": "self_attn.k_proj",
             "wv": "self_attn.v_proj", "wo": "self_attn.o_proj", "norm2": "post_attention_layernorm",
             "wgate": "mlp.gate_proj", "wup": "mlp.up_proj", "wdown": "mlp.down_proj"}
    for j in range(ms.n_layers):
        for k, v in names.items():
            sd[f"model.layers.{j}.{v}.weight"] = wd[f"{k}.{j}"]
    missing, unexpected = m.load_state_dict({k: v.double() for k, v in sd.items()}, strict=False)
    assert not unexpected and all("rotary" in k or "inv_freq" in k for k in missing), (missing, unexpected)
    return m


def identity_tables(lens, ctx=None):
    ctx = ctx or [0] * len(lens)
    need = [(c + n + 15) // 16 for c, n in zip(ctx, lens)]
    bt = torch.zeros((len(lens), max(need)), dtype=torch.int32)
    p = 0
    for b, nb in enumerate(need):
        bt[b, :nb] = torch.arange(p, p + nb, dtype=torch.int32)
        p += nb
    return bt, p


def rel_err(a, b):
    a, b = a.double().flatten(), b.double().flatten()
    return float((a - b).abs().max() / b.abs().max().clamp(min=1e-30))


def cosine(a, b):
    a, b = a.double().flatten(), b.double().flatten()
    return float((a @ b) / (a.norm() * b.norm()).clamp(min=1e-30))
