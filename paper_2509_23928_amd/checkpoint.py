"""Weights from safetensors files -> the weight dictionary that `Hivis(cfg, weights)` takes.

Target: the tensor naming of the Hugging Face LLaMA family, which the language models of the paper's targets use
(section 4, "Models and Tasks": LLaVA-1.5 / LLaVA-NeXT; Qwen2.5-VL's language model has the same names plus q/k/v
biases, which are loaded as bq / bk / bv when any of them is non-zero; an o_proj bias is refused).  The prefix in front
of `embed_tokens` / `layers.N` / `norm` is detected (`model.`, `language_model.model.`, `model.language_model.` ...).
Linear weights are stored [out][in] there and [in][out] here, so they are transposed.

Drafter: the paper publishes trained drafters but not their tensor names, so this is a format of this library:
  fc.weight                          [d][2d]   fusion FC on the concatenation [f_fused ; Embed(x)]  (section 3.2)
  layers.0.<LLaMA layer names>                 the drafter's single decoder layer
  residual.rho [n_resid][d]   or   residual.r [n_resid][m] and residual.w [m][d]   (rho_i = r^i w, Algorithm 1 steps 2-3)

Only marshalling happens here (renaming, transposing, folding r w); every step of the method runs in the HIP library.
bf16 tensors are handed over as their 16-bit patterns (numpy uint16), float32 as float32.
"""
import json
import re

import numpy as np

_LAYER = {"wq": "self_attn.q_proj.weight", "wk": "self_attn.k_proj.weight", "wv": "self_attn.v_proj.weight",
          "wo": "self_attn.o_proj.weight", "wg": "mlp.gate_proj.weight", "wu": "mlp.up_proj.weight",
          "wd": "mlp.down_proj.weight", "norm1": "input_layernorm.weight", "norm2": "post_attention_layernorm.weight"}


def _load_all(paths):
    """All tensors of the files as torch CPU tensors (safetensors never executes anything from the file)."""
    from safetensors.torch import load_file
    if isinstance(paths, (str, bytes)):
        paths = [paths]
    out = {}
    for p in paths:
        out.update(load_file(p, device="cpu"))
    return out


def _to_numpy(t, transpose=False):
    """float32 -> float32 array; bfloat16 -> uint16 bit patterns; anything else is converted to float32."""
    import torch
    if transpose:
        t = t.t()
    t = t.contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.to(torch.float32).numpy()


def _layer(tensors, prefix):
    lw = {}
    for ours, theirs in _LAYER.items():
        key = prefix + theirs
        if key not in tensors:
            raise KeyError(f"missing tensor {key}")
        lw[ours] = _to_numpy(tensors[key], transpose=not ours.startswith("norm"))
    biases = {ours: tensors.get(prefix + f"self_attn.{proj}.bias") for ours, proj in (("bq", "q_proj"), ("bk", "k_proj"), ("bv", "v_proj"))}
    if any(b is not None and bool((b != 0).any()) for b in biases.values()):
        # q/k/v projection biases (Qwen2.5 language model): all three are handed over, a missing one as zeros
        import torch
        for ours, b in biases.items():
            n = lw["wq" if ours == "bq" else "wk"].shape[1]
            lw[ours] = _to_numpy(b if b is not None else torch.zeros(n, dtype=tensors[prefix + _LAYER["wq"]].dtype))
    b = tensors.get(prefix + "self_attn.o_proj.bias")
    if b is not None and bool((b != 0).any()):
        raise ValueError(f"{prefix}self_attn.o_proj.bias is non-zero: an output-projection bias is not implemented")
    return lw


def load_target(paths):
    """Returns (weights, n_layers): embed, lm_head, final_norm and layers[...] of the target's language model."""
    tensors = _load_all(paths)
    emb = [k for k in tensors if k.endswith("embed_tokens.weight")]
    if len(emb) != 1:
        raise KeyError(f"expected exactly one *embed_tokens.weight tensor, found {emb}")
    prefix = emb[0][: -len("embed_tokens.weight")]
    pat = re.compile(re.escape(prefix) + r"layers\.(\d+)\.")
    idx = sorted({int(m.group(1)) for k in tensors for m in [pat.match(k)] if m})
    if not idx or idx != list(range(len(idx))):
        raise KeyError(f"layer indices under {prefix}layers are not 0..n-1: {idx[:8]}")
    w = {"embed": _to_numpy(tensors[emb[0]]), "final_norm": _to_numpy(tensors[prefix + "norm.weight"]),
         "layers": [_layer(tensors, f"{prefix}layers.{i}.") for i in idx]}
    heads = [k for k in tensors if k.endswith("lm_head.weight")]
    if len(heads) > 1:
        raise KeyError(f"more than one lm_head.weight: {heads}")
    w["lm_head"] = _to_numpy(tensors[heads[0]]) if heads else w["embed"]      # tied embeddings: no separate LM head
    return w, len(idx)


def load_drafter(path, dtype_like=None):
    """Returns draft_layer, fuse_w, resid_rho (see the module docstring for the format).  dtype_like: an array of the target
    (e.g. its embed) whose storage type the folded residuals take."""
    import torch
    tensors = _load_all(path)
    w = {"draft_layer": _layer(tensors, "layers.0."), "fuse_w": _to_numpy(tensors["fc.weight"], transpose=True)}
    if "residual.rho" in tensors:
        rho = tensors["residual.rho"].to(torch.float32)
    else:
        rho = tensors["residual.r"].to(torch.float32) @ tensors["residual.w"].to(torch.float32)
    as_bf16 = dtype_like is not None and np.asarray(dtype_like).dtype == np.uint16
    w["resid_rho"] = _to_numpy(rho.to(torch.bfloat16) if as_bf16 else rho)
    return w


def load_weights(target_paths, drafter_path):
    """The complete dictionary for Hivis(cfg, weights), and the number of target layers found."""
    w, n_layers = load_target(target_paths)
    w.update(load_drafter(drafter_path, dtype_like=w["embed"]))
    return w, n_layers


def config_fields(config_json_path):
    """Shape fields of a Hugging Face config.json (the `text_config` of a vision-language model if present), named as
    synth.HivisConfig names them."""
    with open(config_json_path) as fh:
        c = json.load(fh)
    c = c.get("text_config", c)
    n_q = c["num_attention_heads"]
    return {"n_layers": c["num_hidden_layers"], "d": c["hidden_size"], "n_q_heads": n_q,
            "n_kv_heads": c.get("num_key_value_heads", n_q), "head_dim": c.get("head_dim") or c["hidden_size"] // n_q,
            "ffn": c["intermediate_size"], "vocab": c["vocab_size"], "rope_theta": float(c.get("rope_theta", 10000.0)),
            "rms_eps": float(c.get("rms_norm_eps", 1e-5))}
