"""Pins of the CPU oracle against things that are not the oracle: closed forms, library
routines (torch functional ops, the transformers LLaMA model), brute-force loops, and
the invariants the method itself states (verification in one pass equals sequential
decoding; greedy speculative decoding is lossless; the drafter never sees visual rows).
All CPU, float64."""
import itertools
import math

import numpy as np
import pytest
import torch

import synth
from oracle import (rmsnorm, rope, attention, silu, softmax_rows, Target, Drafter, HivisOracle,
                    greedy_reference, fuse, accept_length, decoder_layer, KVCache, top2_gap)
from small_models import tiny_cfg

RNG = np.random.default_rng(1234)


# ---------------------------------------------------------------- elementwise / reductions
def test_rmsnorm_matches_torch_and_unit_rms():
    x = RNG.standard_normal((5, 48))
    g = 1.0 + 0.1 * RNG.standard_normal(48)
    ref = torch.nn.functional.rms_norm(torch.tensor(x), (48,), torch.tensor(g), eps=1e-5).numpy()
    np.testing.assert_allclose(rmsnorm(x, g, 1e-5), ref, rtol=1e-12, atol=1e-12)
    y = rmsnorm(x, np.ones(48), 0.0)
    np.testing.assert_allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0, rtol=1e-12)


def test_silu_matches_torch():
    x = np.linspace(-8, 8, 101)
    np.testing.assert_allclose(silu(x), torch.nn.functional.silu(torch.tensor(x)).numpy(), rtol=1e-12, atol=1e-14)


def test_rope_closed_form_two_dims():
    # hd = 2: a single pair rotated by the angle pos * theta^0 = pos (counter-clockwise)
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[2.0, -3.0]]])
    pos = np.array([1, 2, 5])
    y = rope(x, pos, 10000.0)
    exp = [[math.cos(1), math.sin(1)], [-math.sin(2), math.cos(2)],
           [2 * math.cos(5) + 3 * math.sin(5), -3 * math.cos(5) + 2 * math.sin(5)]]
    np.testing.assert_allclose(y[:, 0, :], exp, rtol=1e-13, atol=1e-13)


def test_rope_pairing_and_frequencies():
    # hd = 8: element i pairs with i+4; pair i rotates by pos * theta^(-2i/8)
    hd, theta, p = 8, 100.0, 3
    for i in range(4):
        x = np.zeros((1, 1, hd)); x[0, 0, i] = 1.0
        y = rope(x, [p], theta)[0, 0]
        ang = p * theta ** (-2.0 * i / hd)
        exp = np.zeros(hd); exp[i] = math.cos(ang); exp[i + 4] = math.sin(ang)
        np.testing.assert_allclose(y, exp, atol=1e-13)


def test_rope_norm_and_relative_position():
    q = RNG.standard_normal((1, 1, 16)); k = RNG.standard_normal((1, 1, 16))
    for (p, s) in [(7, 3), (104, 100), (4, 0)]:
        a = rope(q, [p], 10000.0); b = rope(k, [s], 10000.0)
        np.testing.assert_allclose(np.linalg.norm(a), np.linalg.norm(q), rtol=1e-12)
        dots = float(np.sum(a * b))
        if p - s == 4:
            if "ref" in locals():
                np.testing.assert_allclose(dots, ref, rtol=1e-10)
            ref = dots


def test_rope_position_zero_is_identity():
    x = RNG.standard_normal((3, 2, 8))
    np.testing.assert_allclose(rope(x, [0, 0, 0], 10000.0), x, atol=0)


# ---------------------------------------------------------------- attention
def brute_attention(q, k, v, q_pos, k_pos):
    m, Hq, hd = q.shape
    n, Hkv, _ = k.shape
    out = np.zeros((m, Hq, hd))
    for i in range(m):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            ws, tot = [], 0.0
            for j in range(n):
                if k_pos[j] <= q_pos[i]:
                    e = math.exp(sum(q[i, h, c] * k[j, g, c] for c in range(hd)) / math.sqrt(hd))
                else:
                    e = 0.0
                ws.append(e); tot += e
            for j in range(n):
                for c in range(hd):
                    out[i, h, c] += ws[j] / tot * v[j, g, c]
    return out


@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (4, 2), (7, 1), (6, 6)])
def test_attention_brute_force(Hq, Hkv):
    hd, n, m = 4, 9, 3
    q = RNG.standard_normal((m, Hq, hd)); k = RNG.standard_normal((n, Hkv, hd)); v = RNG.standard_normal((n, Hkv, hd))
    k_pos = np.arange(n); q_pos = np.arange(n - m, n)      # the last m rows are the queries' own keys
    np.testing.assert_allclose(attention(q, k, v, q_pos, k_pos), brute_attention(q, k, v, q_pos, k_pos),
                               rtol=1e-11, atol=1e-12)


def test_attention_matches_torch_sdpa_causal_gqa():
    Hq, Hkv, hd, n = 6, 2, 8, 11
    q = RNG.standard_normal((n, Hq, hd)); k = RNG.standard_normal((n, Hkv, hd)); v = RNG.standard_normal((n, Hkv, hd))
    ours = attention(q, k, v, np.arange(n), np.arange(n))
    tq = torch.tensor(q).permute(1, 0, 2)[None]
    tk = torch.tensor(k).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.tensor(v).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(ours, ref, rtol=1e-11, atol=1e-12)


def test_softmax_rows_sum_to_one_and_shift_invariant():
    s = RNG.standard_normal((4, 13)) * 30
    p = softmax_rows(s)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(softmax_rows(s + 1000.0), p, rtol=1e-9)


def test_single_key_attention_returns_value():
    q = RNG.standard_normal((1, 2, 4)); k = RNG.standard_normal((1, 2, 4)); v = RNG.standard_normal((1, 2, 4))
    np.testing.assert_allclose(attention(q, k, v, [0], [0]), v, rtol=1e-13)


# ---------------------------------------------------------------- whole target vs an independent library model
def hf_llama_from(cfg, w):
    from transformers import LlamaConfig, LlamaForCausalLM
    hc = LlamaConfig(vocab_size=cfg.vocab, hidden_size=cfg.d, intermediate_size=cfg.ffn,
                     num_hidden_layers=cfg.n_layers, num_attention_heads=cfg.n_q_heads,
                     num_key_value_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, rms_norm_eps=cfg.rms_eps,
                     rope_theta=cfg.rope_theta, attention_bias=False, mlp_bias=False, tie_word_embeddings=False,
                     max_position_embeddings=512, attn_implementation="eager")
    m = LlamaForCausalLM(hc).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "lm_head.weight": w["lm_head"], "model.norm.weight": w["final_norm"]}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj", "wo": "self_attn.o_proj",
             "wg": "mlp.gate_proj", "wu": "mlp.up_proj", "wd": "mlp.down_proj"}
    for i, lw in enumerate(w["layers"]):
        for k, hfk in names.items():
            sd[f"model.layers.{i}.{hfk}.weight"] = lw[k].T        # library stores [out][in]
        sd[f"model.layers.{i}.input_layernorm.weight"] = lw["norm1"]
        sd[f"model.layers.{i}.post_attention_layernorm.weight"] = lw["norm2"]
    missing = m.load_state_dict({k: torch.tensor(np.ascontiguousarray(v), dtype=torch.float64) for k, v in sd.items()},
                                strict=False)
    assert not [k for k in missing.missing_keys if "rotary" not in k]
    return m


@pytest.mark.parametrize("heads", [(6, 2), (4, 4)])
def test_target_forward_matches_transformers_llama(heads):
    cfg = tiny_cfg(n_q_heads=heads[0], n_kv_heads=heads[1], d=heads[0] * 8, rope_theta=500.0)
    w = synth.make_weights(cfg, seed=3)
    # larger weights than the recipe, so that attention is far from uniform
    for lw in w["layers"]:
        for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
            lw[k] = lw[k] * 8.0
    vis, ids = synth.make_prompt(cfg, seed=3)
    tgt = Target(cfg, w)
    x = np.concatenate([vis[0].astype(np.float64), tgt.embed(ids[0])], axis=0)
    f = tgt.forward(x, 0)
    logits = tgt.logits(f)
    m = hf_llama_from(cfg, w)
    with torch.no_grad():
        ref = m(inputs_embeds=torch.tensor(x)[None]).logits[0].numpy()
    # the library builds its rotary cos/sin tables in float32 even for a float64 model, hence ~1e-7
    np.testing.assert_allclose(logits, ref, rtol=1e-5, atol=2e-6)
    assert np.abs(ref).max() > 0.3


def test_target_forward_with_qkv_bias_matches_transformers_qwen2():
    """The q/k/v bias term (Qwen2.5 language model) against the transformers Qwen2 model: GQA 6/2, biases of order 1."""
    from transformers import Qwen2Config, Qwen2ForCausalLM
    cfg = tiny_cfg(n_q_heads=6, n_kv_heads=2, d=48, rope_theta=1.0e6, rms_eps=1e-6, qkv_bias=True)
    w = synth.make_weights(cfg, seed=4)
    for lw in w["layers"]:
        assert lw["bq"].shape == (cfg.q_dim,) and lw["bk"].shape == (cfg.kv_dim,) and np.abs(lw["bv"]).max() > 0.3
        for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
            lw[k] = lw[k] * 8.0
    vis, ids = synth.make_prompt(cfg, seed=4)
    tgt = Target(cfg, w)
    x = np.concatenate([vis[0].astype(np.float64), tgt.embed(ids[0])], axis=0)
    logits = tgt.logits(tgt.forward(x, 0))
    hc = Qwen2Config(vocab_size=cfg.vocab, hidden_size=cfg.d, intermediate_size=cfg.ffn, num_hidden_layers=cfg.n_layers,
                     num_attention_heads=cfg.n_q_heads, num_key_value_heads=cfg.n_kv_heads, rms_norm_eps=cfg.rms_eps,
                     rope_theta=cfg.rope_theta, tie_word_embeddings=False, max_position_embeddings=512, use_sliding_window=False,
                     attn_implementation="eager")
    assert hc.hidden_size // hc.num_attention_heads == cfg.head_dim
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
    missing = m.load_state_dict({k: torch.tensor(np.ascontiguousarray(v), dtype=torch.float64) for k, v in sd.items()}, strict=False)
    assert not [k for k in missing.missing_keys if "rotary" not in k] and not missing.unexpected_keys
    with torch.no_grad():
        ref = m(inputs_embeds=torch.tensor(x)[None]).logits[0].numpy()
    np.testing.assert_allclose(logits, ref, rtol=1e-5, atol=2e-6)
    # and the term matters: the same weights without the biases give different logits
    w0 = {k: v for k, v in w.items()}
    w0["layers"] = [{k: v for k, v in lw.items() if k not in ("bq", "bk", "bv")} for lw in w["layers"]]
    t0 = Target(cfg, w0)
    assert np.abs(t0.logits(t0.forward(x, 0)) - logits).max() > 1e-2


# ---------------------------------------------------------------- method invariants
@pytest.fixture(scope="module")
def tiny():
    cfg = tiny_cfg()
    w = synth.make_weights(cfg, seed=11)
    for lw in w["layers"] + [w["draft_layer"]]:
        for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
            lw[k] = lw[k] * 6.0
    vis, ids = synth.make_prompt(cfg, seed=11)
    return cfg, w, vis[0], ids[0]


def test_verify_equals_sequential_decodes(tiny):
    cfg, w, vis, ids = tiny
    o = HivisOracle(cfg, w); o.prefill(vis, ids)
    drafts = [5, 17, 33]
    g, logits, t = o.verify(drafts)
    # the same rows one at a time through a fresh target
    tgt = Target(cfg, w)
    tgt.forward(np.concatenate([vis.astype(np.float64), tgt.embed(ids)], 0), 0)
    rows = [o.text[-1]] + drafts
    for i, tok in enumerate(rows):
        gi = tgt.forward(tgt.embed([tok]), cfg.n_vis + cfg.n_text + i)[0]
        np.testing.assert_allclose(g[i], gi, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(logits[i], tgt.logits(gi), rtol=1e-10, atol=1e-12)


def test_prefill_prefix_consistency(tiny):
    cfg, w, vis, ids = tiny
    a = Target(cfg, w)
    fa = a.forward(np.concatenate([vis.astype(np.float64), a.embed(ids)], 0), 0)
    b = Target(cfg, w)
    b.forward(np.concatenate([vis.astype(np.float64), b.embed(ids[:-1])], 0), 0)
    fb = b.forward(b.embed(ids[-1:]), cfg.n_vis + cfg.n_text - 1)
    np.testing.assert_allclose(fa[-1], fb[0], rtol=1e-10, atol=1e-12)


def run_cycles(cfg, w, vis, ids, n_cycles, plant_lengths=None):
    """plant_lengths: per cycle, how many leading drafts are the target's true continuation."""
    ref, _ = greedy_reference(cfg, w, vis, ids, 1 + n_cycles * (cfg.K + 1))
    o = HivisOracle(cfg, w)
    x, _ = o.prefill(vis, ids)
    out, ns = [x], []
    for c in range(n_cycles):
        planted = None
        if plant_lengths is not None:
            m = plant_lengths[c]
            good = ref[len(out): len(out) + m]
            bad = [(ref[len(out) + j] + 1 + j) % cfg.vocab for j in range(m, cfg.K)]
            planted = good + bad
        r = o.cycle(cfg.K, planted=planted)
        out += r["emitted"]; ns.append(r["n"])
        assert o.drafter.kv_len == o.l == len(o.text) - 1
        assert o.target.kv_len == cfg.n_vis + o.l
    return out, ns, ref


def test_lossless_own_drafts(tiny):
    cfg, w, vis, ids = tiny
    out, ns, ref = run_cycles(cfg, w, vis, ids, 5)
    assert out == ref[: len(out)]


def test_lossless_and_lengths_with_planted_drafts(tiny):
    cfg, w, vis, ids = tiny
    plan = [0, 1, 2, 3, 3, 1, 0, 2]
    out, ns, ref = run_cycles(cfg, w, vis, ids, len(plan), plan)
    assert ns == plan                                  # accepted length == planted matching prefix
    assert out == ref[: len(out)]                      # and the stream is the plain greedy decode
    assert len(out) == 1 + sum(n + 1 for n in ns)


def test_acceptance_rule_exhaustive():
    K = 5
    t = [10, 11, 12, 13, 14, 15]
    for pattern in itertools.product([0, 1], repeat=K):
        drafts = [t[i] if pattern[i] else t[i] + 100 for i in range(K)]
        n = accept_length(drafts, t[:K])
        exp = next((i for i, p in enumerate(pattern) if not p), K)
        assert n == exp
    assert accept_length([], []) == 0


def test_drafter_is_blind_to_visual_rows(tiny):
    cfg, w, vis, ids = tiny
    o1 = HivisOracle(cfg, w); o1.prefill(vis, ids)
    o2 = HivisOracle(cfg, w); o2.prefill(vis * -3.0 + 1.0, ids)         # very different image
    assert o1.drafter.kv_len == o2.drafter.kv_len == cfg.n_text           # text-only cache
    assert not np.allclose(o1.f_next, o2.f_next)                          # (the features do differ)
    # hand both drafters the SAME true features: outputs must be bit-identical
    feats = RNG.standard_normal((cfg.n_text, cfg.d))
    toks = list(range(1, cfg.n_text + 1))
    d1 = Drafter(cfg, w); d2 = Drafter(cfg, w)
    u = fuse(feats, o1.target.embed(toks), w["fuse_w"], o1.rho(0))
    assert np.array_equal(d1.forward(u, 0), d2.forward(u, 0))
    assert not hasattr(o1.drafter, "target") and not hasattr(o1.drafter, "caches")


def test_fusion_identities():
    d = 6
    f = RNG.standard_normal((3, d)); e = RNG.standard_normal((3, d)); rho = RNG.standard_normal(d)
    w1 = RNG.standard_normal((d, d)); w2 = RNG.standard_normal((d, d))
    W = np.concatenate([w1, w2], 0)
    np.testing.assert_allclose(fuse(f, e, W, rho), np.concatenate([f, e], 1) @ W + rho, rtol=1e-12)
    np.testing.assert_allclose(fuse(f, e, W, 0 * rho), f @ w1 + e @ w2, rtol=1e-12)
    W0 = np.concatenate([np.zeros((d, d)), np.eye(d)], 0)
    np.testing.assert_allclose(fuse(f, e, W0, 0 * rho), e, atol=0)
    W1 = np.concatenate([np.eye(d), np.zeros((d, d))], 0)
    np.testing.assert_allclose(fuse(f, e, W1, 0 * rho), f, atol=0)


def test_residual_schedule():
    """With the fusion FC zeroed and a drafter layer that adds nothing, the drafter's hidden
    state IS the residual vector of the row; with one-hot residuals and an identity-like LM
    head the draft tokens spell the schedule: r^0 (true-feature row), r^1, r^2, r^3, r^3, ..."""
    cfg = tiny_cfg(K=6, vocab=97)
    w = synth.make_weights(cfg, seed=5)
    w["fuse_w"] = np.zeros_like(w["fuse_w"])
    w["draft_layer"]["wo"] = np.zeros_like(w["draft_layer"]["wo"])
    w["draft_layer"]["wd"] = np.zeros_like(w["draft_layer"]["wd"])
    rho = np.zeros((cfg.n_resid, cfg.d), np.float32)
    for i in range(cfg.n_resid):
        rho[i, 10 + i] = 1.0
    w["resid_rho"] = rho
    lm = np.zeros((cfg.vocab, cfg.d), np.float32); lm[np.arange(cfg.d), np.arange(cfg.d)] = 1.0
    w["lm_head"] = lm
    vis, ids = synth.make_prompt(cfg, seed=5)
    o = HivisOracle(cfg, w); o.prefill(vis[0], ids[0])
    for _ in range(3):
        r = o.cycle(cfg.K)
        assert r["drafts"] == [10, 11, 12, 13, 13, 13]


def test_k_zero_accept_reduces_to_plain_decode(tiny):
    # drafts that never match: every cycle emits exactly the target's next token
    cfg, w, vis, ids = tiny
    out, ns, ref = run_cycles(cfg, w, vis, ids, 6, [0] * 6)
    assert ns == [0] * 6 and out == ref[:7]


def test_follow_mode_tracks_foreign_trajectory(tiny):
    cfg, w, vis, ids = tiny
    o = HivisOracle(cfg, w); o.prefill(vis, ids)
    own = HivisOracle(cfg, w); own.prefill(vis, ids)
    r_own = own.cycle(cfg.K)
    r = o.cycle(cfg.K, follow_drafts=r_own["drafts"], force=(r_own["n"], r_own["emitted"]))
    assert r["emitted"] == r_own["emitted"] and np.array_equal(o.f_next, own.f_next)


def test_top2_gap():
    np.testing.assert_allclose(top2_gap(np.array([[1.0, 5.0, 4.5], [2.0, 2.0, 0.0]])), [0.5, 0.0])


def test_roll_forward_equals_fresh_prefill(tiny):
    """Eq. (1): a drafting round starts from the target's true features of ALL earlier text
    positions.  So the state after some cycles must equal the state of a fresh prefill whose
    prompt is the text so far (pins KV truncation, re-feed rows, positions and residual r^0)."""
    cfg, w, vis, ids = tiny
    plan = [1, 0, 3, 2]
    ref, _ = greedy_reference(cfg, w, vis, ids, 32)
    o = HivisOracle(cfg, w); x, _ = o.prefill(vis, ids)
    out = [x]
    for m in plan:
        planted = ref[len(out): len(out) + m] + [(ref[len(out) + j] + 7) % cfg.vocab for j in range(m, cfg.K)]
        out += o.cycle(cfg.K, planted=planted)["emitted"]
    fresh = HivisOracle(cfg, w)
    x2, _ = fresh.prefill(vis, o.text[:-1])
    assert x2 == o.text[-1]
    np.testing.assert_allclose(fresh.f_next, o.f_next, rtol=1e-9, atol=1e-11)
    assert fresh.drafter.kv_len == o.drafter.kv_len and fresh.target.kv_len == o.target.kv_len
    d1, l1 = fresh.draft(cfg.K); d2, l2 = o.draft(cfg.K)
    assert d1 == d2
    np.testing.assert_allclose(l1, l2, rtol=1e-8, atol=1e-10)
