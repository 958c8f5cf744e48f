"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs (tokens bit-exact up to near-ties, logits within the stated tolerance)."""
import numpy as np
import pytest

import synth
from oracle import greedy_reference
from parity_utils import SideBySide

pytestmark = pytest.mark.gpu


def make(cfg, seed):
    from paper_2509_23928_amd import Hivis
    w = synth.make_weights(cfg, seed=seed)
    vis, ids = synth.make_prompt(cfg, seed=seed)
    hv = Hivis(cfg, w)
    return w, vis, ids, hv


def small_bf16(**kw):
    base = dict(name="small-bf16", n_layers=2, d=512, n_q_heads=4, n_kv_heads=4, head_dim=128, ffn=1376, vocab=2048,
                dtype="bf16", n_vis=150, n_text=37, K=5, batch=1, gen_tokens=0, gen_cycles=6)
    base.update(kw)
    return synth.HivisConfig(**base)


def test_c1_end_to_end_own_drafts():
    cfg = synth.get_config("C1")
    w, vis, ids, hv = make(cfg, 0)
    sbs = SideBySide(cfg, w, hv, vis, ids)
    for c in range(cfg.gen_cycles):
        sbs.cycle(cfg.K)
    print("C1:", sbs.summary())
    # lossless: the emitted stream is the plain greedy decode of the target
    ref, _ = greedy_reference(cfg, w, vis[0], ids[0], len(sbs.emitted[0]))
    if sbs.near_ties == 0:
        assert sbs.emitted[0] == ref


def test_c1_planted_drafts_accept_lengths():
    cfg = synth.get_config("C1")
    w, vis, ids, hv = make(cfg, 1)
    ref, _ = greedy_reference(cfg, w, vis[0], ids[0], 1 + 10 * (cfg.K + 1))
    sbs = SideBySide(cfg, w, hv, vis, ids)
    plan = [0, 1, 2, 3, 4, 4, 2, 0, 3, 1]
    for m in plan:
        done = len(sbs.emitted[0])
        good = ref[done: done + m]
        bad = [(ref[done + j] + 1 + j) % cfg.vocab for j in range(m, cfg.K)]
        r = sbs.cycle(cfg.K, planted=np.array([good + bad], np.int32))
        if sbs.near_ties == 0:
            assert r[0]["n"] == m
    if sbs.near_ties == 0:
        assert sbs.emitted[0] == ref[: len(sbs.emitted[0])]
    print("C1 planted max error / tolerance:", sbs.max_err)


@pytest.mark.parametrize("variant", ["mha", "gqa", "hd64"])
def test_small_bf16_end_to_end(variant):
    if variant == "mha":
        cfg = small_bf16()
    elif variant == "gqa":
        cfg = small_bf16(n_q_heads=7, n_kv_heads=1, d=896, ffn=2368, K=6, n_vis=200, n_text=70, rope_theta=1e6, rms_eps=1e-6)
    else:
        cfg = small_bf16(n_q_heads=8, n_kv_heads=4, head_dim=64, K=3)
    w, vis, ids, hv = make(cfg, 5)
    sbs = SideBySide(cfg, w, hv, vis, ids)
    ref, _ = greedy_reference(cfg, w, vis[0], ids[0], 1 + 6 * (cfg.K + 1))
    for c in range(3):
        sbs.cycle(cfg.K)
    for m in [cfg.K, 1, 2]:
        done = len(sbs.emitted[0])
        if sbs.emitted[0] != ref[:done]:
            break                                 # a near-tie moved the trajectory: planted prefixes no longer apply
        planted = ref[done: done + m] + [(ref[done + j] + 3) % cfg.vocab for j in range(m, cfg.K)]
        sbs.cycle(cfg.K, planted=np.array([planted], np.int32))
    print(variant, ":", sbs.summary())


def test_batch_per_sequence_acceptance():
    cfg = small_bf16(batch=4, K=7, n_vis=90, n_text=45, n_q_heads=4, n_kv_heads=4)
    w, vis, ids, hv = make(cfg, 9)
    sbs = SideBySide(cfg, w, hv, vis, ids)
    refs = [greedy_reference(cfg, w, vis[b], ids[b], 40)[0] for b in range(cfg.batch)]
    sbs.cycle(cfg.K)
    plans = [[0, 3, 7, 2], [7, 7, 0, 1], [1, 0, 5, 4]]
    for plan in plans:
        planted = []
        for b in range(cfg.batch):
            done = len(sbs.emitted[b])
            ok = sbs.emitted[b] == refs[b][:done]
            m = plan[b] if ok else 0
            planted.append(refs[b][done: done + m] + [(refs[b][done + j] + 5) % cfg.vocab for j in range(m, cfg.K)])
        r = sbs.cycle(cfg.K, planted=np.array(planted, np.int32))
        if sbs.near_ties == 0:
            assert [x["n"] for x in r] == plan
    print("batch:", sbs.summary())


def test_error_codes():
    from paper_2509_23928_amd import Hivis, HivisError, HIVIS_ESTATE, HIVIS_EINVAL, HIVIS_ECAP
    cfg = synth.get_config("C1")
    w, vis, ids, hv = make(cfg, 0)
    with pytest.raises(HivisError) as e:
        hv.draft(2)
    assert e.value.code == HIVIS_ESTATE
    with pytest.raises(HivisError) as e:
        hv.verify()
    assert e.value.code == HIVIS_ESTATE
    bad = ids.copy(); bad[0, 3] = cfg.vocab
    with pytest.raises(HivisError) as e:
        hv.prefill(vis, bad)
    assert e.value.code == HIVIS_EINVAL
    hv.prefill(vis, ids)
    with pytest.raises(HivisError) as e:
        hv.draft(cfg.K + 1)
    assert e.value.code == HIVIS_EINVAL
    with pytest.raises(HivisError) as e:
        hv.accept()
    assert e.value.code == HIVIS_ESTATE
    hv.draft(cfg.K)
    with pytest.raises(HivisError) as e:
        hv.draft(cfg.K)
    assert e.value.code == HIVIS_ESTATE
    hv.verify(); hv.accept()
    small = Hivis(cfg, w, max_text=cfg.n_text + cfg.K + 2 + 3)
    small.prefill(vis, ids)
    with pytest.raises(HivisError) as e:
        for _ in range(10):
            small.draft(cfg.K); small.verify(); small.accept()
    assert e.value.code == HIVIS_ECAP
    with pytest.raises(HivisError) as e:
        small.prefill(np.concatenate([vis, vis], 1), ids)
    assert e.value.code == HIVIS_ECAP


def run_generic(cfg, seed, cycles, plant=(), k_list=None):
    """own drafts for `cycles` cycles (optionally a different K each), then planted prefixes of the given lengths"""
    w, vis, ids, hv = make(cfg, seed)
    sbs = SideBySide(cfg, w, hv, vis, ids)
    for c in range(cycles):
        sbs.cycle(k_list[c] if k_list else cfg.K)
    if plant:
        ref, _ = greedy_reference(cfg, w, vis[0], ids[0], len(sbs.emitted[0]) + len(plant) * (cfg.K + 1) + 1)
        for m in plant:
            done = len(sbs.emitted[0])
            if sbs.emitted[0] != ref[:done]:
                break
            planted = ref[done: done + m] + [(ref[done + j] + 3) % cfg.vocab for j in range(m, cfg.K)]
            r = sbs.cycle(cfg.K, planted=np.array([planted], np.int32))
            if sbs.near_ties == 0:
                assert r[0]["n"] == m
    hv.close()
    return sbs


def test_long_cache_uses_key_splits():
    # 1500 visual rows: the verify attention splits the key range over several workgroups and runs the merge launch
    cfg = small_bf16(n_vis=1500, n_text=40, d=256, n_q_heads=2, n_kv_heads=2, ffn=512, vocab=1024, K=5)
    sbs = run_generic(cfg, 21, 2, plant=(5, 2))
    print("long cache:", sbs.summary())


def test_forced_small_key_splits_hd64_and_hd128():
    # 48 keys per workgroup: many key splits (ragged last split, splits of a single 16-key tile) for both head sizes
    import os
    os.environ["HIVIS_KEYS_PER_SPLIT"] = "48"
    try:
        sbs = run_generic(small_bf16(), 27, 2, plant=(4,))
        print("forced key splits hd128:", sbs.summary())
        sbs = run_generic(small_bf16(head_dim=64, n_q_heads=8, n_kv_heads=2), 28, 2, plant=(2,))
        print("forced key splits hd64 gqa:", sbs.summary())
        # batch 4, K = 7: 32-row passes, whose attention is launched outside a phase program (same split + elected merge)
        cfg = small_bf16(batch=4, K=7, n_vis=90, n_text=45, n_q_heads=4, n_kv_heads=4)
        w, vis, ids, hv = make(cfg, 29)
        sbs = SideBySide(cfg, w, hv, vis, ids)
        for _ in range(3):
            sbs.cycle(cfg.K)
        hv.close()
        print("forced key splits batch 4 (32-row passes):", sbs.summary())
    finally:
        del os.environ["HIVIS_KEYS_PER_SPLIT"]


def test_prefill_large_tile_gemm_on_small_shapes():
    # the 128-row x 256-column prefill GEMM tile is normally chosen only where it fills the CUs (7B-13B widths, covered at
    # depth elsewhere); forced here on small ragged shapes: 187 and 420 prompt rows (1.46 and 3.3 row blocks), column counts
    # that are not multiples of 256, K blocks from 8 to 74
    import os
    os.environ["HIVIS_TALL_BIG_FILL"] = "0"
    try:
        sbs = run_generic(small_bf16(), 51, 1, plant=(3,))
        print("large-tile prefill GEMM, default small model:", sbs.summary())
        cfg = small_bf16(n_q_heads=7, n_kv_heads=1, d=896, ffn=2368, K=4, n_vis=380, n_text=40, rope_theta=1e6, rms_eps=1e-6)
        sbs = run_generic(cfg, 52, 1, plant=(2,))
        print("large-tile prefill GEMM, gqa7 d896 F2368, 420 rows:", sbs.summary())
    finally:
        del os.environ["HIVIS_TALL_BIG_FILL"]


def test_gqa_group7_k6_qwen_like_shape():
    # 28 query / 4 kv heads (group 7), K = 6 -> 7 rows per sequence, as in the Qwen2.5-VL-shaped workload, at reduced width
    cfg = small_bf16(n_q_heads=28, n_kv_heads=4, head_dim=64, d=1792, ffn=2368, vocab=4096, K=6, n_vis=130, n_text=50,
                     rope_theta=1e6, rms_eps=1e-6, n_layers=2)
    sbs = run_generic(cfg, 22, 2, plant=(6, 3))
    print("gqa 28/4:", sbs.summary())


def test_edge_shapes_no_visual_single_text_and_varying_k():
    # no visual rows at all, a one-token prompt, and a different K every cycle (1 .. k_max)
    cfg = small_bf16(n_vis=0, n_text=1, K=5, d=256, n_q_heads=2, n_kv_heads=2, ffn=512, vocab=1024)
    sbs = run_generic(cfg, 23, 5, k_list=[1, 5, 2, 3, 4])
    print("edge shapes:", sbs.summary())
    cfg = small_bf16(n_vis=1, n_text=2, K=2, d=256, n_q_heads=2, n_kv_heads=2, ffn=512, vocab=1024)
    run_generic(cfg, 24, 2)


def test_fp32_sixteen_rows_and_gqa():
    # fp32 path with 14 verify rows (one fp32 MFMA tile holds 16) and grouped heads
    cfg = synth.get_config("C1").scaled(name="f32-gqa", n_q_heads=4, n_kv_heads=2, K=6, batch=2, gen_cycles=3, n_vis=70, n_text=33)
    w, vis, ids, hv = make(cfg, 25)
    sbs = SideBySide(cfg, w, hv, vis, ids)
    for _ in range(3):
        sbs.cycle(cfg.K)
    print("fp32 gqa batch-2:", sbs.summary())
    assert max(sbs.max_err.values()) < 0.1


def test_rerun_is_bit_identical():
    cfg = small_bf16()
    w, vis, ids, hv = make(cfg, 5)
    outs = []
    for _ in range(2):
        hv.prefill(vis, ids)
        seq = [hv.get_logits(2).copy()]
        for _c in range(3):
            hv.draft(cfg.K); hv.verify()
            seq.append(hv.get_logits(0).copy()); seq.append(hv.get_logits(1).copy())
            n, t = hv.accept()
            seq.append(t.copy())
        outs.append(seq)
    for a, b in zip(*outs):
        assert np.array_equal(a, b), "two runs of the same prompt differ bitwise"


@pytest.mark.parametrize("seed", list(range(100, 112)))
def test_random_shape_sweep(seed):
    """Seeded random small shapes inside the documented limits: odd tile counts (grids smaller than the chip, ragged K
    passes, partial tile groups), both head sizes, grouped heads, batches, K from 1 to 7, caches from a few keys to several
    key tiles, and row counts on both sides of one MFMA tile."""
    rng = np.random.default_rng(seed)
    hd = int(rng.choice([64, 128]))
    n_kv = int(rng.choice([1, 2, 4]))
    group = int(rng.choice([1, 2, 3]))
    n_q = n_kv * group
    d = 32 * int(rng.integers(4, 20))
    ffn = 32 * int(rng.integers(5, 60))
    vocab = 32 * int(rng.integers(8, 200))
    K = int(rng.integers(1, 8))
    batch = int(rng.choice([1, 1, 2, 3, 4]))
    while batch * (K + 1) > 32:
        batch -= 1
    cfg = small_bf16(name=f"sweep-{seed}", d=d, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=hd, ffn=ffn, vocab=vocab, K=K, batch=batch,
                     n_vis=int(rng.integers(0, 300)), n_text=int(rng.integers(1, 60)), n_layers=int(rng.integers(1, 4)))
    w, vis, ids, hv = make(cfg, seed)
    try:
        sbs = SideBySide(cfg, w, hv, vis, ids)
    except AssertionError as e:
        if "near-tie at the first token" in str(e):
            pytest.skip("near-tie at the first token for this seed")
        raise
    sbs.cycle(K)
    sbs.cycle(max(1, K - 1))
    hv.close()
    print(f"sweep {seed}: d={d} Hq/Hkv={n_q}/{n_kv} hd={hd} F={ffn} V={vocab} K={K} B={batch} v={cfg.n_vis} l={cfg.n_text} N={cfg.n_layers}",
          ":", sbs.summary())


def test_standalone_kernel_path_matches_oracle():
    # HIVIS_FUSED=0: every operation as its own launch (the kernels the 32-row passes and the fp32 prefill also use)
    import os
    os.environ["HIVIS_FUSED"] = "0"
    try:
        sbs = run_generic(small_bf16(K=4), 29, 2, plant=(3,))
        print("stand-alone kernels bf16:", sbs.summary())
        run_generic(synth.get_config("C1"), 3, 2, plant=(2,))
    finally:
        del os.environ["HIVIS_FUSED"]


def test_persistent_mode_matches_oracle():
    # the opt-in single-launch (cooperative, grid-barrier) execution of the same phase programs
    import os
    os.environ["HIVIS_PERSISTENT"] = "1"
    try:
        cfg = small_bf16(K=4)
        sbs = run_generic(cfg, 26, 2, plant=(3,))
        cfg1 = synth.get_config("C1")
        run_generic(cfg1, 2, 2)
    finally:
        del os.environ["HIVIS_PERSISTENT"]
    print("persistent mode max error / tolerance:", sbs.max_err)


def test_qwen_vocab_lm_head_many_tile_groups():
    # V = 152064 (the Qwen2.5-VL-shaped workload): 9504 LM-head tiles, 37-38 per workgroup = 5 tile groups with the greedy
    # candidate carried across groups; narrow d keeps the oracle quick
    cfg = small_bf16(vocab=152064, d=512, n_q_heads=4, n_kv_heads=2, ffn=1376, K=6, n_vis=60, n_text=24, rope_theta=1e6, rms_eps=1e-6)
    sbs = run_generic(cfg, 31, 2, plant=(4,))
    print("V=152064:", sbs.summary())


def test_qwen_width_ffn_two_layer_slice():
    # Qwen2.5-VL-7B widths without the vocabulary: d 3584, 28/4 heads of 128, F 18944 (gate|up 2368 tiles = two tile groups per
    # workgroup; down projection K = 18944 = 9 full passes + a ragged one), K = 6 -> 7 rows
    cfg = synth.get_config("C4").scaled(n_layers=2, vocab=4096, n_vis=130, n_text=50, gen_tokens=0, gen_cycles=2)
    sbs = run_generic(cfg, 32, 1, plant=(3,))
    print("Qwen-width 2-layer:", sbs.summary())


def test_13b_width_batch4_k7_thirty_two_rows():
    # LLaVA-1.5-13B widths (d 5120, 40 heads, F 13824), batch 4, K = 7: 32 verify rows, the path for more rows than one MFMA tile
    cfg = synth.get_config("C5").scaled(n_layers=2, vocab=4096, n_vis=96, n_text=40, gen_tokens=0, gen_cycles=2)
    w, vis, ids, hv = make(cfg, 33)
    sbs = SideBySide(cfg, w, hv, vis, ids)
    sbs.cycle(cfg.K)
    sbs.cycle(cfg.K)
    hv.close()
    print("13B-width batch-4:", sbs.summary())


def test_full_width_7b_layers_two_layer_slice():
    """LLaVA-1.5-7B widths (d 4096, 32 heads, F 11008, V 32000, 576 + 64 rows, K 5) with 2 of the 32 layers: the launch
    configuration bench.py times (same tile groups, K passes, LM-head tiling), against the oracle on every logit."""
    cfg = synth.get_config("C2").scaled(n_layers=2, gen_tokens=0, gen_cycles=2)
    w, vis, ids, hv = make(cfg, 0)
    sbs = SideBySide(cfg, w, hv, vis, ids)
    sbs.cycle(cfg.K)
    ref, _ = greedy_reference(cfg, w, vis[0], ids[0], len(sbs.emitted[0]) + cfg.K + 2)
    done = len(sbs.emitted[0])
    if sbs.emitted[0] == ref[:done]:
        planted = ref[done: done + 3] + [(ref[done + j] + 3) % cfg.vocab for j in range(3, cfg.K)]
        r = sbs.cycle(cfg.K, planted=np.array([planted], np.int32))
        if sbs.near_ties == 0:
            assert r[0]["n"] == 3
    hv.close()
    print("7B-width 2-layer:", sbs.summary())


def test_two_live_contexts_with_different_head_sizes():
    """Two contexts alive at once (head_dim 128 created first, then 64) used alternately: per-kernel launch attributes set
    for one must not break the other."""
    cfg_a = small_bf16(name="live-a", n_q_heads=4, n_kv_heads=4, head_dim=128)
    cfg_b = small_bf16(name="live-b", n_q_heads=8, n_kv_heads=2, head_dim=64)
    wa, va, ia, ha = make(cfg_a, 31)
    wb, vb, ib, hb = make(cfg_b, 32)
    sa = SideBySide(cfg_a, wa, ha, va, ia)
    sb = SideBySide(cfg_b, wb, hb, vb, ib)
    for _ in range(2):
        sa.cycle(cfg_a.K)
        sb.cycle(cfg_b.K)
    ha.tree_draft(4, 3, 20); ha.tree_verify(); ha.tree_accept()
    hb.tree_draft(4, 3, 20); hb.tree_verify(); hb.tree_accept()
    print("two live contexts max error / tolerance:", sa.max_err, sb.max_err)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_qkv_biases_gqa7(dtype):
    """q/k/v projection biases (Qwen2.5 language model): 7 query heads per kv head, biases of order 0.5 in every target
    layer and in the drafter's layer; prefill, own-draft cycles, a planted cycle, and a draft-tree cycle (the bias is
    added in four different kernels: the fused QKV epilogue, the prefill's and the stand-alone RoPE kernels, and the
    wide-pass RoPE kernel)."""
    if dtype == "bf16":
        cfg = small_bf16(name="bias-bf16", n_q_heads=7, n_kv_heads=1, d=896, ffn=2368, K=4, n_vis=120, n_text=40, rope_theta=1e6, rms_eps=1e-6,
                         qkv_bias=True, gen_cycles=10)
    else:
        cfg = synth.get_config("C1").scaled(name="bias-f32", n_q_heads=4, n_kv_heads=2, qkv_bias=True)
    w, vis, ids, hv = make(cfg, 21)
    sbs = SideBySide(cfg, w, hv, vis, ids)
    ref, _ = greedy_reference(cfg, w, vis[0], ids[0], 1 + 4 * (cfg.K + 1))
    sbs.cycle(cfg.K)
    sbs.cycle(2)
    done = len(sbs.emitted[0])
    if sbs.emitted[0] == ref[:done]:
        planted = ref[done: done + 2] + [(ref[done + j] + 3) % cfg.vocab for j in range(2, cfg.K)]
        r = sbs.cycle(cfg.K, planted=np.array([planted], np.int32))
        if sbs.near_ties == 0:
            assert r[0]["n"] == 2
    print("q/k/v biases", dtype, ":", sbs.summary())
    # a draft-tree cycle on the same state (12-row passes through the wide-pass kernels for bf16): lossless means its
    # tokens continue the oracle's greedy text
    done = len(sbs.emitted[0])
    if sbs.near_ties == 0 and sbs.emitted[0] == ref[:done]:
        hv.tree_draft(4, 3, 11)
        hv.tree_verify()
        n, toks = hv.tree_accept()
        got = [int(t) for t in toks[: n + 1]]
        ref2, lg2 = greedy_reference(cfg, w, vis[0], ids[0], done + len(got))
        from oracle import top2_gap
        from parity_utils import logit_tol
        if float(np.min(top2_gap(lg2[done:]))) > 2 * logit_tol(cfg, lg2):
            assert got == ref2[done: done + len(got)], (got, ref2[done:])
    # the oracle without the biases must NOT match (the term is visible at this tolerance)
    w0 = dict(w); w0["layers"] = [{k: v for k, v in lw.items() if k not in ("bq", "bk", "bv")} for lw in w["layers"]]
    from oracle import HivisOracle
    _, l0 = HivisOracle(cfg, w0).prefill(vis[0], ids[0])
    _, l1 = HivisOracle(cfg, w).prefill(vis[0], ids[0])
    from parity_utils import logit_tol
    assert float(np.max(np.abs(l0 - l1))) > 3 * logit_tol(cfg, l1)
    hv.close()
