"""Independent library decoder used to pin the oracle: Hugging Face `transformers`'
Llama / Qwen2 modules, random-init, in float64, loaded with the same synthetic parameters.
Nothing here is shared with the oracle or with the HIP path."""
from __future__ import annotations

import numpy as np
import torch


def build_hf(cfg: dict, weights: dict):
    from transformers import LlamaConfig, LlamaForCausalLM, Qwen2Config, Qwen2ForCausalLM

    common = dict(hidden_size=cfg["d_model"], num_attention_heads=cfg["n_q_heads"],
                  num_key_value_heads=cfg["n_kv_heads"], intermediate_size=cfg["d_ffn"],
                  rms_norm_eps=cfg["rms_eps"], rope_theta=cfg["rope_theta"], vocab_size=cfg["vocab"],
                  num_hidden_layers=cfg["n_layers"], tie_word_embeddings=False,
                  max_position_embeddings=4096, attn_implementation="eager")
    if cfg["qkv_bias"]:
        assert cfg["d_model"] == cfg["n_q_heads"] * cfg["head_dim"]
        model = Qwen2ForCausalLM(Qwen2Config(**common))
    else:
        model = LlamaForCausalLM(LlamaConfig(head_dim=cfg["head_dim"], attention_bias=False, **common))
    model = model.double().eval()

    def t(a):
        return torch.from_numpy(np.asarray(a, dtype=np.float64))

    sd = {"model.embed_tokens.weight": t(weights["embed"]), "model.norm.weight": t(weights["g_final"]),
          "lm_head.weight": t(weights["lm_head"])}
    names = dict(wq="self_attn.q_proj.weight", wk="self_attn.k_proj.weight", wv="self_attn.v_proj.weight",
                 wo="self_attn.o_proj.weight", wg="mlp.gate_proj.weight", wu="mlp.up_proj.weight",
                 wd="mlp.down_proj.weight", g_attn="input_layernorm.weight",
                 g_mlp="post_attention_layernorm.weight", bq="self_attn.q_proj.bias",
                 bk="self_attn.k_proj.bias", bv="self_attn.v_proj.bias")
    for i, lw in enumerate(weights["layers"]):
        for k, v in lw.items():
            sd[f"model.layers.{i}.{names[k]}"] = t(v)
    missing, unexpected = model.load_state_dict(sd, strict=False)
    assert not unexpected, unexpected
    assert all("rotary" in m or "inv_freq" in m for m in missing), missing
    return model


@torch.no_grad()
def hf_prefill(model, tokens):
    """Full causal forward; returns (logits [n, V], cache)."""
    ids = torch.tensor(np.asarray(tokens, dtype=np.int64))[None]
    out = model(ids, use_cache=True)
    return out.logits[0].numpy(), out.past_key_values


def cache_kv(cache, layer):
    lyr = cache.layers[layer]
    return lyr.keys[0].numpy(), lyr.values[0].numpy()   # [Hkv, n, hd]


@torch.no_grad()
def hf_fuzzy_step(model, cache, token, bounds):
    """Layer-parallel fuzzy forward of one token composed from the library's own blocks:
    within a set every self-attention block (with its input norm) reads the hidden state that
    enters the set; the MLP blocks (with their norm) run in order on the running residual."""
    pos = cache.get_seq_length()
    h = model.model.embed_tokens(torch.tensor([[int(token)]]))
    position_ids = torch.tensor([[pos]])
    pe = model.model.rotary_emb(h, position_ids)
    attn_outs = []
    for j in range(len(bounds) - 1):
        h1 = h
        outs = {}
        for i in range(bounds[j], bounds[j + 1]):
            layer = model.model.layers[i]
            a = layer.self_attn(hidden_states=layer.input_layernorm(h1), position_embeddings=pe,
                                attention_mask=None, past_key_values=cache,
                                cache_position=torch.tensor([pos]))[0]
            outs[i] = a
            attn_outs.append(a[0, 0].numpy())
        for i in range(bounds[j], bounds[j + 1]):
            layer = model.model.layers[i]
            h = h + outs[i]
            h = h + layer.mlp(layer.post_attention_layernorm(h))
    logits = model.lm_head(model.model.norm(h))
    return logits[0, 0].numpy(), np.stack(attn_outs)


@torch.no_grad()
def hf_full_layer_step(model, cache, token, bounds):
    """Full-layer-parallel forward of one token (the ablation of the paper's App. B) composed from the
    library's blocks: within a set every layer, attention and MLP, starts from the hidden state
    that enters the set, and the set's output is that state plus what every layer adds."""
    pos = cache.get_seq_length()
    h = model.model.embed_tokens(torch.tensor([[int(token)]]))
    pe = model.model.rotary_emb(h, torch.tensor([[pos]]))
    for j in range(len(bounds) - 1):
        h1 = h
        for i in range(bounds[j], bounds[j + 1]):
            layer = model.model.layers[i]
            a = layer.self_attn(hidden_states=layer.input_layernorm(h1), position_embeddings=pe,
                                attention_mask=None, past_key_values=cache,
                                cache_position=torch.tensor([pos]))[0]
            m = layer.mlp(layer.post_attention_layernorm(h1 + a))
            h = h + a + m
    logits = model.lm_head(model.model.norm(h))
    return logits[0, 0].numpy(), h[0, 0].numpy()
