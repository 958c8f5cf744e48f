"""The safetensors loader (paper_2509_23928_amd/checkpoint.py): round trips through files written in the Hugging Face
LLaMA naming by the `transformers` model itself, prefix / tied-embedding / bias handling, and, on the GPU, the HIP
library prefilled from such a checkpoint against the logits of the `transformers` model that wrote it (a reference
that shares nothing with this repository's oracle)."""
import json
import os

import numpy as np
import pytest
import torch

import synth
from paper_2509_23928_amd import checkpoint
from small_models import tiny_cfg
from test_oracle_pins import hf_llama_from


def write_target(tmp_path, cfg, w, prefix="", dtype=torch.float32, drop_lm_head=False, bias=None):
    from safetensors.torch import save_file
    m = hf_llama_from(cfg, w)
    sd = {}
    for k, v in m.state_dict().items():
        if "rotary" in k or (drop_lm_head and k == "lm_head.weight"):
            continue
        sd[prefix + k] = v.to(dtype).contiguous()
    if bias is not None:
        sd[prefix + "model.layers.0.self_attn.q_proj.bias"] = torch.full((cfg.q_dim,), bias, dtype=dtype)
    # two shards, as large checkpoints are stored
    keys = sorted(sd)
    paths = [str(tmp_path / "model-00001-of-00002.safetensors"), str(tmp_path / "model-00002-of-00002.safetensors")]
    save_file({k: sd[k] for k in keys[: len(keys) // 2]}, paths[0])
    save_file({k: sd[k] for k in keys[len(keys) // 2:]}, paths[1])
    return m, paths


def write_drafter(tmp_path, cfg, w, folded=True, dtype=torch.float32):
    from safetensors.torch import save_file
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj", "wo": "self_attn.o_proj",
             "wg": "mlp.gate_proj", "wu": "mlp.up_proj", "wd": "mlp.down_proj"}
    lw = w["draft_layer"]
    sd = {f"layers.0.{hf}.weight": torch.tensor(np.ascontiguousarray(lw[k].T)) for k, hf in names.items()}
    sd["layers.0.input_layernorm.weight"] = torch.tensor(lw["norm1"])
    sd["layers.0.post_attention_layernorm.weight"] = torch.tensor(lw["norm2"])
    sd["fc.weight"] = torch.tensor(np.ascontiguousarray(w["fuse_w"].T))
    if folded:
        sd["residual.rho"] = torch.tensor(w["resid_rho"])
    else:
        # rho = r w with r = identity rows padded: r [n_resid][n_resid], w = rho itself
        sd["residual.r"] = torch.eye(cfg.n_resid)
        sd["residual.w"] = torch.tensor(w["resid_rho"])
    path = str(tmp_path / "drafter.safetensors")
    save_file({k: v.to(dtype).contiguous() for k, v in sd.items()}, path)
    return path


def assert_same_weights(a, b):
    for k in ("embed", "lm_head", "final_norm", "fuse_w", "resid_rho"):
        if k in a and k in b:
            np.testing.assert_array_equal(np.asarray(a[k]), np.asarray(b[k]), err_msg=k)
    for la, lb in zip(a["layers"] + [a.get("draft_layer", {})], b["layers"] + [b.get("draft_layer", {})]):
        for k in la:
            np.testing.assert_array_equal(np.asarray(la[k]), np.asarray(lb[k]), err_msg=k)


@pytest.mark.parametrize("prefix", ["", "language_model."])
def test_round_trip_float32(tmp_path, prefix):
    cfg = tiny_cfg(n_q_heads=6, n_kv_heads=2)
    w = synth.make_weights(cfg, seed=5)
    _, paths = write_target(tmp_path, cfg, w, prefix=prefix)
    dpath = write_drafter(tmp_path, cfg, w, folded=(prefix == ""))
    got, n_layers = checkpoint.load_weights(paths, dpath)
    assert n_layers == cfg.n_layers
    assert_same_weights(w, got)
    assert got["layers"][0]["wq"].shape == (cfg.d, cfg.q_dim) and got["fuse_w"].shape == (2 * cfg.d, cfg.d)


def test_round_trip_bf16_bits(tmp_path):
    cfg = tiny_cfg(dtype="bf16")
    w = synth.make_weights(cfg, seed=6)                       # float32 values that are bf16-representable
    bits = synth.make_weights(cfg, seed=6, bits=True)        # the same values as 16-bit patterns
    _, paths = write_target(tmp_path, cfg, w, dtype=torch.bfloat16)
    dpath = write_drafter(tmp_path, cfg, w, dtype=torch.bfloat16)
    got, _ = checkpoint.load_weights(paths, dpath)
    assert got["embed"].dtype == np.uint16 and got["resid_rho"].dtype == np.uint16
    assert_same_weights(bits, got)


def test_tied_embeddings_and_bias_handling(tmp_path):
    cfg = tiny_cfg()
    w = synth.make_weights(cfg, seed=7)
    d1 = tmp_path / "tied"; d1.mkdir()
    _, paths = write_target(d1, cfg, w, drop_lm_head=True)
    got, _ = checkpoint.load_target(paths)
    np.testing.assert_array_equal(got["lm_head"], got["embed"])
    d2 = tmp_path / "zero_bias"; d2.mkdir()
    _, paths = write_target(d2, cfg, w, bias=0.0)
    checkpoint.load_target(paths)                             # all-zero biases are accepted
    d3 = tmp_path / "bias"; d3.mkdir()
    _, paths = write_target(d3, cfg, w, bias=0.5)
    got, _ = checkpoint.load_target(paths)                    # a non-zero q bias: all three come back, k and v as zeros
    np.testing.assert_array_equal(got["layers"][0]["bq"], np.full(cfg.q_dim, 0.5, np.float32))
    assert not got["layers"][0]["bk"].any() and got["layers"][0]["bv"].shape == (cfg.kv_dim,)
    assert "bq" not in got["layers"][1]
    d4 = tmp_path / "obias"; d4.mkdir()
    from safetensors.torch import save_file
    _, paths = write_target(d4, cfg, w)
    extra = str(d4 / "extra.safetensors")
    save_file({"model.layers.0.self_attn.o_proj.bias": torch.full((cfg.d,), 0.25)}, extra)
    with pytest.raises(ValueError):
        checkpoint.load_target(paths + [extra])


def test_residual_fold_matches_oracle_fuse():
    """The loader folds rho_i = r^i w on the host (the one product of the method outside the library).  Pin: the oracle's
    fusion f w1 + e w2 + rho with the folded vector equals the unfolded form written out, (f w1 + e w2) + r^i w, in float64."""
    from oracle import fuse
    rng = np.random.default_rng(5)
    d, m, n_resid = 24, 7, 4
    r = rng.standard_normal((n_resid, m)).astype(np.float32)
    wmat = rng.standard_normal((m, d)).astype(np.float32)
    f = rng.standard_normal((3, d)); e = rng.standard_normal((3, d)); fw = rng.standard_normal((2 * d, d))
    import tempfile
    from safetensors.torch import save_file
    cfg = tiny_cfg(d=d, n_q_heads=3, n_kv_heads=3, head_dim=8)
    w = synth.make_weights(cfg, seed=1)
    with tempfile.TemporaryDirectory() as td:
        import pathlib
        path = write_drafter(pathlib.Path(td), cfg, w)
        from safetensors.torch import load_file
        sd = load_file(path)
        del sd["residual.rho"]
        sd["residual.r"] = torch.tensor(r); sd["residual.w"] = torch.tensor(wmat)
        save_file(sd, path)
        got = checkpoint.load_drafter(path)
    rho = got["resid_rho"]
    assert rho.shape == (n_resid, d)
    for i in range(n_resid):
        unfolded = (f @ fw[:d] + e @ fw[d:]) + r[i].astype(np.float64) @ wmat.astype(np.float64)
        np.testing.assert_allclose(fuse(f, e, fw, rho[i]), unfolded, rtol=0, atol=2e-5)       # the fold itself is a float32 product


def test_config_fields(tmp_path):
    cfg = tiny_cfg(n_q_heads=6, n_kv_heads=2)
    m = hf_llama_from(cfg, synth.make_weights(cfg, seed=8))
    p = tmp_path / "config.json"
    p.write_text(json.dumps({"model_type": "llava", "text_config": m.config.to_dict()}))
    f = checkpoint.config_fields(str(p))
    for k in ("n_layers", "d", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab"):
        assert f[k] == getattr(cfg, k), k
    assert f["rope_theta"] == cfg.rope_theta and abs(f["rms_eps"] - cfg.rms_eps) < 1e-12


@pytest.mark.gpu
def test_library_from_checkpoint_matches_transformers(tmp_path):
    """HIP library prefilled from a checkpoint written by the transformers LLaMA model, against that model's own logits."""
    from paper_2509_23928_amd import Hivis
    cfg = synth.get_config("C1").scaled(n_q_heads=4, n_kv_heads=2, n_vis=20, n_text=15)
    w = synth.make_weights(cfg, seed=9)
    vis, ids = synth.make_prompt(cfg, seed=9)
    m, paths = write_target(tmp_path, cfg, w, prefix="language_model.")
    dpath = write_drafter(tmp_path, cfg, w)
    got, n_layers = checkpoint.load_weights(paths, dpath)
    hv = Hivis(cfg.scaled(n_layers=n_layers), got)
    first = hv.prefill(vis, ids)
    logits = hv.get_logits(2)[0]
    x = torch.cat([torch.tensor(vis[0], dtype=torch.float64), m.get_input_embeddings()(torch.tensor(ids[0].astype(np.int64)))], dim=0)
    with torch.no_grad():
        ref = m(inputs_embeds=x[None]).logits[0, -1].numpy()
    assert float(np.max(np.abs(logits - ref))) <= 1e-4
    assert int(first[0]) == int(np.argmax(ref))
    # chain and tree cycles on the loaded drafter: the emitted text must be the transformers model's own greedy decoding
    out = [int(first[0])]
    for cyc in range(4):
        if cyc % 2 == 0:
            hv.draft(cfg.K); hv.verify(); n, toks = hv.accept()
            out += [int(t) for t in toks[0][: int(n[0]) + 1]]
        else:
            hv.tree_draft(4, 3, 12); hv.tree_verify(); n, toks = hv.tree_accept()
            out += [int(t) for t in toks[: n + 1]]
    seq = [int(t) for t in ids[0]]
    gaps = []
    with torch.no_grad():
        for tok in out:
            xs = torch.cat([torch.tensor(vis[0], dtype=torch.float64), m.get_input_embeddings()(torch.tensor(seq, dtype=torch.int64))], dim=0)
            lg = m(inputs_embeds=xs[None]).logits[0, -1].numpy()
            top = np.sort(lg)
            if int(np.argmax(lg)) != tok:
                assert top[-1] - lg[tok] <= 2e-4, f"token {tok} is not the transformers model's greedy token (gap {top[-1] - lg[tok]})"
                break                                 # a near-tie: the two texts may legitimately part here
            seq.append(tok)


@pytest.mark.gpu
def test_library_from_qwen2_checkpoint_with_qkv_biases(tmp_path):
    """A checkpoint written by the transformers Qwen2 model (q/k/v biases of order 1, GQA) loaded and prefilled by the HIP
    library, against that model's own logits; then chain cycles must emit its greedy text."""
    from safetensors.torch import save_file
    from transformers import Qwen2Config, Qwen2ForCausalLM
    from paper_2509_23928_amd import Hivis
    cfg = synth.get_config("C1").scaled(n_q_heads=4, n_kv_heads=2, n_vis=20, n_text=15, rope_theta=1.0e6, rms_eps=1e-6, qkv_bias=True)
    w = synth.make_weights(cfg, seed=10)
    vis, ids = synth.make_prompt(cfg, seed=10)
    hc = Qwen2Config(vocab_size=cfg.vocab, hidden_size=cfg.d, intermediate_size=cfg.ffn, num_hidden_layers=cfg.n_layers,
                     num_attention_heads=cfg.n_q_heads, num_key_value_heads=cfg.n_kv_heads, rms_norm_eps=cfg.rms_eps,
                     rope_theta=cfg.rope_theta, tie_word_embeddings=False, max_position_embeddings=512, use_sliding_window=False,
                     attn_implementation="eager")
    m = Qwen2ForCausalLM(hc).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "lm_head.weight": w["lm_head"], "model.norm.weight": w["final_norm"]}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj", "wo": "self_attn.o_proj",
             "wg": "mlp.gate_proj", "wu": "mlp.up_proj", "wd": "mlp.down_proj"}
    for i, lw in enumerate(w["layers"]):
        for k, hfk in names.items():
            sd[f"model.layers.{i}.{hfk}.weight"] = lw[k].T
        for k, hfk in (("bq", "q_proj"), ("bk", "k_proj"), ("bv", "v_proj")):
            sd[f"model.layers.{i}.self_attn.{hfk}.bias"] = lw[k]
        sd[f"model.layers.{i}.input_layernorm.weight"] = lw["norm1"]
        sd[f"model.layers.{i}.post_attention_layernorm.weight"] = lw["norm2"]
    m.load_state_dict({k: torch.tensor(np.ascontiguousarray(v), dtype=torch.float64) for k, v in sd.items()}, strict=False)
    tpath = str(tmp_path / "qwen.safetensors")
    save_file({k: v.to(torch.float32).contiguous() for k, v in m.state_dict().items() if "rotary" not in k}, tpath)
    # drafter file: its layer carries biases too
    dpath = write_drafter(tmp_path, cfg, w)
    from safetensors.torch import load_file
    dsd = load_file(dpath)
    for k, hfk in (("bq", "q_proj"), ("bk", "k_proj"), ("bv", "v_proj")):
        dsd[f"layers.0.self_attn.{hfk}.bias"] = torch.tensor(w["draft_layer"][k])
    save_file(dsd, dpath)
    got, n_layers = checkpoint.load_weights([tpath], dpath)
    np.testing.assert_array_equal(got["layers"][1]["bk"], w["layers"][1]["bk"])
    np.testing.assert_array_equal(got["draft_layer"]["bv"], w["draft_layer"]["bv"])
    hv = Hivis(cfg.scaled(n_layers=n_layers), got)
    first = hv.prefill(vis, ids)
    logits = hv.get_logits(2)[0]
    x = torch.cat([torch.tensor(vis[0], dtype=torch.float64), m.get_input_embeddings()(torch.tensor(ids[0].astype(np.int64)))], dim=0)
    with torch.no_grad():
        ref = m(inputs_embeds=x[None]).logits[0, -1].numpy()
    assert float(np.max(np.abs(logits - ref))) <= 1e-4
    assert int(first[0]) == int(np.argmax(ref))
    out = [int(first[0])]
    for cyc in range(3):
        hv.draft(cfg.K); hv.verify(); n, toks = hv.accept()
        out += [int(t) for t in toks[0][: int(n[0]) + 1]]
    seq = [int(t) for t in ids[0]]
    with torch.no_grad():
        for tok in out:
            xs = torch.cat([torch.tensor(vis[0], dtype=torch.float64), m.get_input_embeddings()(torch.tensor(seq, dtype=torch.int64))], dim=0)
            lg = m(inputs_embeds=xs[None]).logits[0, -1].numpy()
            if int(np.argmax(lg)) != tok:
                assert np.max(lg) - lg[tok] <= 2e-4, f"token {tok} is not the transformers model's greedy token"
                break
            seq.append(tok)
    hv.close()
