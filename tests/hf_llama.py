"""Builds the `transformers` LLaMA implementation with given weights: the independent library
routine the oracle's target stack is pinned against (it is used by CPU tests only)."""
import numpy as np
import torch
from transformers.models.llama.modeling_llama import LlamaConfig, LlamaForCausalLM


def hf_config(shape, n_layers=None):
    return LlamaConfig(
        hidden_size=shape.hidden, intermediate_size=shape.intermediate,
        num_hidden_layers=shape.n_layers if n_layers is None else n_layers,
        num_attention_heads=shape.n_heads, num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim,
        vocab_size=shape.vocab, rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta,
        attention_bias=False, mlp_bias=False, tie_word_embeddings=False, attn_implementation="eager",
        max_position_embeddings=1 << 15)


def hf_model(shape, layers, tg):
    """layers: list of dicts of torch tensors (eagle3_synth.layer_weights); tg: target_globals."""
    m = LlamaForCausalLM(hf_config(shape, len(layers))).double().eval()
    sd = {"model.embed_tokens.weight": tg["embed"], "model.norm.weight": tg["final_norm"],
          "lm_head.weight": tg["lm_head"]}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "w_gate": "mlp.gate_proj", "w_up": "mlp.up_proj",
             "w_down": "mlp.down_proj", "norm_attn": "input_layernorm", "norm_mlp": "post_attention_layernorm"}
    for l, W in enumerate(layers):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}.weight"] = W[k]
    missing = m.load_state_dict({k: v.double() for k, v in sd.items()}, strict=False)
    assert not missing.unexpected_keys and all("rotary" in k for k in missing.missing_keys), missing
    return m


def hf_forward(model, ids, mask_bool=None, position_ids=None):
    """Returns (logits [T,V], list of per-layer residual-stream outputs [T,k]) as float64 NumPy.
    mask_bool [T,T]: True = may attend (None = causal)."""
    outs = []
    hooks = [lyr.register_forward_hook(lambda mod, a, o: outs.append((o[0] if isinstance(o, tuple) else o)[0].numpy().copy()))
             for lyr in model.model.layers]
    kw = {}
    T = len(ids)
    if mask_bool is not None:
        add = torch.zeros(1, 1, T, T, dtype=torch.float64)
        add[0, 0][~torch.from_numpy(np.asarray(mask_bool))] = float("-inf")
        kw["attention_mask"] = add
    if position_ids is not None:
        kw["position_ids"] = torch.as_tensor(np.asarray(position_ids), dtype=torch.long)[None]
    with torch.no_grad():
        logits = model(input_ids=torch.as_tensor(np.asarray(ids), dtype=torch.long)[None], **kw).logits[0].numpy()
    for h in hooks:
        h.remove()
    return logits, outs
