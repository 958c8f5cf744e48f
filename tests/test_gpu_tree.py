"""GPU parity of the draft-tree calls (hivis_tree_draft / hivis_tree_verify / hivis_tree_accept) against the oracle.

Floating point is compared with the tolerances of the chain tests (oracle in follow mode: it is handed the
library's tree and recomputes every row on its own state).  Every index the tree method decides from floating
point (top-k tokens of a row, the rows expanded at a level, the candidates, the followed path) is re-decided by
the oracle's routines from the library's OWN float32 numbers, where it must agree exactly; that the numbers
themselves are right is the tolerance check."""
import numpy as np
import pytest

import synth
from oracle import greedy_reference, sampling_reference, softmax_temperature
from oracle import rng as orng
from oracle.tree import HivisTreeOracle, accept_path, log_softmax, pool_size, sample_tree_tokens, top_k_lowest
from parity_utils import check_token, logit_tol
from test_gpu_parity import small_bf16

pytestmark = pytest.mark.gpu


def c1(**kw):
    return synth.get_config("C1").scaled(**kw)


def make_tree(cfg, seed, room):
    from paper_2509_23928_amd import Hivis
    w = synth.make_weights(cfg, seed=seed)
    vis, ids = synth.make_prompt(cfg, seed=seed)
    hv = Hivis(cfg, w, max_text=cfg.n_text + room, k_max=max(cfg.K, 1))
    return w, vis, ids, hv


class TreeSideBySide:
    def __init__(self, cfg, seed, room=400):
        self.cfg = cfg
        self.w, self.vis, self.ids, self.hv = make_tree(cfg, seed, room)
        self.o = HivisTreeOracle(cfg, self.w)
        first = self.hv.prefill(self.vis, self.ids)
        x, logits = self.o.prefill(self.vis[0], self.ids[0])
        assert x == int(first[0]), "near-tie at the first token: pick another seed"
        self.emitted = [x]
        self.near_ties = 0
        self.n_hist = []
        self.max_err = {"draft": 0.0, "score": 0.0, "verify": 0.0, "g": 0.0, "fnext": 0.0}
        self.draws = self.edge = 0
        self.used_u = []                    # uniforms in the order in which emitted tokens consumed them (sampling cycles)
        self._check_fnext()

    def _check_fnext(self):
        f = self.hv.get_hidden(1)[0]
        scale = float(np.sqrt(np.mean(self.o.f_next ** 2)))
        rel = float(np.max(np.abs(f - self.o.f_next))) / scale
        lim = 2e-4 if self.cfg.dtype == "f32" else 6e-2
        self.max_err["fnext"] = max(self.max_err["fnext"], rel / lim)
        assert rel <= lim, f"drafter pending hidden state off by {rel}"

    def _verify_accept(self, tokens, parents, depth, sample=None):
        """Shared tail of a cycle: the oracle's tree (self.o.tree) already equals the library's.
        sample = (T, u): acceptance at temperature T; u = [depth+1] uniforms handed to the library, or a callable that
        returns the uniforms the library must have drawn itself (then it is given none)."""
        cfg, hv, o = self.cfg, self.hv, self.o
        hv.tree_verify()
        N = len(tokens)
        tr = hv.tree_get(verified=True)
        assert list(tr["row_tokens"][1:]) == list(tokens) and list(tr["row_parents"][1:]) == list(parents)
        assert int(tr["row_parents"][0]) == -1 and int(tr["row_tokens"][0]) == o.text[-1] and int(tr["row_depths"][0]) == 0
        vlog = hv.get_logits(0)[0]
        g = hv.get_hidden(0)[0]
        og, ologits, ot = o.tree_verify()
        tol = logit_tol(cfg, ologits)
        err = float(np.max(np.abs(vlog - ologits)))
        self.max_err["verify"] = max(self.max_err["verify"], err / tol)
        assert err <= tol, f"tree verify logits off by {err} > {tol}"
        gerr = float(np.max(np.abs(g - og))) / float(np.sqrt(np.mean(og ** 2)))
        glim = 1e-4 if cfg.dtype == "f32" else 6e-2
        self.max_err["g"] = max(self.max_err["g"], gerr / glim)
        assert gerr <= glim, f"tree verify features off by {gerr}"
        ttok = tr["target_tokens"]
        for i in range(N + 1):
            self.near_ties += check_token(ttok[i], ologits[i], tol)
        if sample is None:
            n, toks = hv.tree_accept()
        else:
            # every row's token is DRAWN: re-drawn here in float64 from the library's own float32 logits with the same
            # uniform (row of depth j: u[j]); a difference only within 1e-5 of a boundary of the running sum
            T, u = sample
            if callable(u):
                n, toks = hv.tree_accept_sample(T, None)
                u = u()
            else:
                n, toks = hv.tree_accept_sample(T, u)
            ttok = hv.tree_get(verified=True)["target_tokens"]
            dep = [0] + [int(x) for x in tr["row_depths"][1:]]
            mine = sample_tree_tokens(vlog.astype(np.float64), dep, T, u)
            for i in range(N + 1):
                self.draws += 1
                if mine[i] != int(ttok[i]):
                    pr = softmax_temperature(vlog[i].astype(np.float64), T)
                    c = np.cumsum(pr)
                    lo, hi = min(mine[i], int(ttok[i])), max(mine[i], int(ttok[i]))
                    assert np.min(np.abs(c[lo:hi] - float(u[dep[i]]) * c[-1])) <= 1e-5 * c[-1], (i, mine[i], int(ttok[i]))
                    self.edge += 1
            self.used_u += [float(x) for x in u[: n + 1]]
            ot = [int(x) for x in ttok]
        # acceptance: bit-exact given the library's own target tokens
        path = accept_path([-1] + list(parents), [o.text[-1]] + list(tokens), ttok)
        exp = [int(tokens[r - 1]) for r in path] + [int(ttok[path[-1] if path else 0])]
        assert n == len(path) and [int(t) for t in toks[:n + 1]] == exp and all(int(t) == -1 for t in toks[n + 1:])
        o.tree_accept(og, ot, force=(path, exp))
        tl, dl = hv.kv_lengths()
        assert int(tl[0]) == o.target.kv_len and int(dl[0]) == o.drafter.kv_len == o.l
        self.emitted += exp
        self.n_hist.append(n)
        self._check_fnext()
        return n, path

    def cycle(self, k, depth, N, sample=None):
        cfg, hv, o = self.cfg, self.hv, self.o
        hv.tree_draft(k, depth, N)
        tr = hv.tree_get()
        dlog = hv.tree_get_logits().astype(np.float64)              # [1 + (depth-1) k][V]
        P = pool_size(k, depth)
        ptok, ppar, psc = tr["pool_tokens"], tr["pool_parents"], tr["pool_scores"].astype(np.float64)
        # --- decisions re-taken from the library's own numbers: exact
        lp_own = log_softmax(dlog)
        lo, n = 0, k
        for j in range(depth):
            rows = [0] if j == 0 else [1 + (j - 1) * k + r for r in range(k)]
            first = 0 if j == 0 else lo + n
            for r, row in enumerate(rows):
                kids = list(range(first + r * k, first + (r + 1) * k))
                assert [int(ptok[i]) for i in kids] == top_k_lowest(dlog[row], k), (j, r)
                parent = -1 if j == 0 else int(tr["expand"][j - 1][r])
                assert all(int(ppar[i]) == parent for i in kids)
                base = 0.0 if parent < 0 else psc[parent]
                for i in kids:                                        # fp32 sum of fp32 log-probabilities
                    assert abs(psc[i] - (base + lp_own[row][ptok[i]])) <= 2e-5 * (1 + abs(psc[i]))
            if j > 0:
                lo, n = first, k * k
            if j < depth - 1:
                l0, ln = (0, k) if j == 0 else (first, k * k)
                assert [int(e) for e in tr["expand"][j]] == [l0 + i for i in top_k_lowest(psc[l0:l0 + ln], k)], j
        assert [int(s) for s in tr["selected"]] == sorted(top_k_lowest(psc, N))
        # --- the numbers themselves: the oracle follows the library's tree
        ot = o.tree_draft(k, depth, N, follow={"pool_tokens": ptok, "expand": tr["expand"], "selected": tr["selected"]})
        tol = logit_tol(cfg, dlog)
        err = float(np.max(np.abs(lp_own - ot["logp"])))
        self.max_err["draft"] = max(self.max_err["draft"], err / (2 * tol))
        assert err <= 2 * tol, f"tree draft log-probabilities off by {err} > {2 * tol}"
        serr = float(np.max(np.abs(psc - ot["pool_scores"])))
        self.max_err["score"] = max(self.max_err["score"], serr / (2 * tol * depth))
        assert serr <= 2 * tol * depth
        assert list(tr["row_tokens"][1:]) == ot["tokens"] and list(tr["row_parents"][1:]) == ot["parents"] and list(tr["row_depths"][1:]) == ot["depths"]
        return self._verify_accept(ot["tokens"], ot["parents"], depth, sample)

    def planted_cycle(self, tokens, parents, sample=None):
        o = self.o
        self.hv.tree_set(tokens, parents)
        depths = {0: 0}
        for i, p in enumerate(parents, start=1):
            depths[i] = depths[int(p)] + 1
        o.tree = {"tokens": [int(t) for t in tokens], "parents": [int(p) for p in parents], "depths": [depths[i] for i in range(1, len(tokens) + 1)]}
        return self._verify_accept(o.tree["tokens"], o.tree["parents"], max(depths.values()), sample)


def branching_plant(ref, done, vocab, good, shape):
    """A tree whose followed path is ref[done:done+good] placed on NON-first siblings: at every level `shape` siblings
    hang under the previous level's path node, the path token sits at the last of them, the others carry wrong tokens;
    below the path's end one more level of wrong tokens."""
    tokens, parents = [], []
    parent = 0
    for lvl in range(good + 1):
        want = ref[done + lvl]
        first = len(tokens) + 1
        for s in range(shape):
            on_path = (s == shape - 1) and lvl < good
            tokens.append(want if on_path else (want + 1 + s) % vocab)
            parents.append(parent)
        parent = first + shape - 1
    return tokens, parents


def test_tree_own_drafts_tiny_fp32():
    cfg = c1(n_vis=40, n_text=19, n_q_heads=4, n_kv_heads=2)
    t = TreeSideBySide(cfg, 5)
    for (k, depth, N) in [(3, 3, 9), (4, 2, 12), (2, 4, 7), (1, 3, 3), (5, 3, 31), (3, 1, 3)]:
        t.cycle(k, depth, N)
    print("tiny tree max error / tolerance:", t.max_err, "accepted:", t.n_hist, "near ties:", t.near_ties)
    if t.near_ties == 0:
        ref, _ = greedy_reference(cfg, t.w, t.vis[0], t.ids[0], len(t.emitted))
        assert t.emitted == ref


def test_tree_planted_paths_and_compaction_fp32():
    """Planted trees whose followed path sits on scattered rows: accepted lengths 0..4, cache compaction, and the
    following cycles (chain and tree) still exact."""
    cfg = c1(n_vis=33, n_text=9, K=3)
    t = TreeSideBySide(cfg, 6)
    ref, _ = greedy_reference(cfg, t.w, t.vis[0], t.ids[0], 60)
    for good, shape in [(3, 3), (0, 2), (4, 4), (1, 1), (2, 5)]:
        tokens, parents = branching_plant(ref, len(t.emitted), cfg.vocab, good, shape)
        n, path = t.planted_cycle(tokens, parents)
        if t.near_ties == 0:
            assert n == good
            assert path == [shape * (lvl + 1) for lvl in range(good)]       # the last sibling of every level
        t.cycle(3, 2, 6)                                                      # an own-draft tree cycle on the compacted state
    # a chain cycle on the same context afterwards
    hv = t.hv
    hv.draft(cfg.K); hv.verify(); n, toks = hv.accept()
    if t.near_ties == 0:
        done = len(t.emitted)
        assert [int(x) for x in toks[0][: n[0] + 1]] == ref[done: done + n[0] + 1]
        assert t.emitted == ref[: len(t.emitted)]
    print("planted tree max error / tolerance:", t.max_err, "accepted:", t.n_hist)


@pytest.mark.parametrize("variant", ["mha128", "gqa64"])
def test_tree_small_bf16(variant):
    kw = dict(n_q_heads=4, n_kv_heads=4, head_dim=128) if variant == "mha128" else dict(n_q_heads=8, n_kv_heads=2, head_dim=64)
    cfg = small_bf16(**kw)
    t = TreeSideBySide(cfg, 7)
    ref, _ = greedy_reference(cfg, t.w, t.vis[0], t.ids[0], 40)
    t.cycle(4, 3, 15)
    tokens, parents = branching_plant(ref, len(t.emitted), cfg.vocab, 3, 3)
    t.planted_cycle(tokens, parents)
    t.cycle(10, 6, 60)                    # the paper's setting: 61 verify rows (two GEMM row blocks), 50 drafter tree rows
    t.cycle(8, 4, 30)                     # the supplementary setting
    print(variant, "tree max error / tolerance:", t.max_err, "accepted:", t.n_hist, "near ties:", t.near_ties)
    if t.near_ties == 0:
        assert t.emitted == ref[: len(t.emitted)]


def test_tree_verify_two_skinny_passes(monkeypatch):
    """HIVIS_WIDE_GEMM=0: the 61-row GEMMs as two passes of the 32-row kernel instead of the split-K kernel."""
    monkeypatch.setenv("HIVIS_WIDE_GEMM", "0")
    cfg = small_bf16()
    t = TreeSideBySide(cfg, 12)
    t.cycle(10, 6, 60)
    t.cycle(6, 3, 40)
    print("two-pass tree max error / tolerance:", t.max_err)


def test_tree_without_phase_programs(monkeypatch):
    """HIVIS_FUSED=0: every pass on the stand-alone kernels, the half-precision cache read by the vector-ALU attention
    (its ancestor-mask branch) instead of the MFMA routine."""
    monkeypatch.setenv("HIVIS_FUSED", "0")
    cfg = small_bf16(n_q_heads=8, n_kv_heads=2, head_dim=64)
    t = TreeSideBySide(cfg, 14)
    t.cycle(5, 4, 25)
    ref, _ = greedy_reference(cfg, t.w, t.vis[0], t.ids[0], 12)
    tokens, parents = branching_plant(ref, len(t.emitted), cfg.vocab, 2, 4)
    t.planted_cycle(tokens, parents)
    t.cycle(10, 6, 60)
    print("stand-alone tree max error / tolerance:", t.max_err, "accepted:", t.n_hist)


def test_tree_error_codes():
    from paper_2509_23928_amd import Hivis, HivisError, HIVIS_EINVAL, HIVIS_ESTATE, HIVIS_ECAP
    cfg = c1(n_vis=8, n_text=9)
    w, vis, ids, hv = make_tree(cfg, 8, 40)
    with pytest.raises(HivisError) as e:
        hv.tree_draft(3, 3, 9)                              # nothing prefilled
    assert e.value.code == HIVIS_ESTATE
    hv.prefill(vis, ids)
    for bad in [(0, 3, 3), (17, 2, 3), (3, 0, 3), (3, 17, 3), (3, 3, 0), (3, 3, 22), (16, 6, 60), (10, 6, 64)]:
        with pytest.raises(HivisError) as e:
            hv.tree_draft(*bad)
        assert e.value.code == HIVIS_EINVAL, bad
    with pytest.raises(HivisError) as e:
        hv.tree_verify()
    assert e.value.code == HIVIS_ESTATE
    with pytest.raises(HivisError) as e:
        hv.tree_set([1, 2], [0, 2])                         # parent does not precede its child
    assert e.value.code == HIVIS_EINVAL
    with pytest.raises(HivisError) as e:
        hv.tree_draft(10, 6, 60)                            # 50 drafter tree rows do not fit max_text = n_text + 40
    assert e.value.code == HIVIS_ECAP
    hv.tree_draft(3, 2, 5)
    with pytest.raises(HivisError) as e:
        hv.verify()                                         # chain verify on a tree round
    assert e.value.code == HIVIS_ESTATE
    with pytest.raises(HivisError) as e:
        hv.tree_accept()
    assert e.value.code == HIVIS_ESTATE
    hv.tree_verify()
    n, toks = hv.tree_accept()
    assert 0 <= n <= 2 and toks[n] >= 0
    cfg2 = c1(n_vis=8, n_text=9, batch=2)
    w2 = synth.make_weights(cfg2, seed=8)
    vis2, ids2 = synth.make_prompt(cfg2, seed=8)
    hv2 = Hivis(cfg2, w2)
    hv2.prefill(vis2, ids2)
    with pytest.raises(HivisError) as e:
        hv2.tree_draft(2, 2, 3)                             # batch 2
    assert e.value.code == HIVIS_EINVAL


def test_tree_full_width_7b_two_layer_slice():
    """The paper's tree setting (top-10, depth 6, 60 candidates) at LLaVA-1.5-7B layer width and vocabulary, two target
    layers (what the oracle finishes in seconds): 61 verify rows against 576 visual + 64 text cached rows."""
    cfg = synth.get_config("C2").scaled(name="C2-2layer", n_layers=2, gen_tokens=0, gen_cycles=2)
    t = TreeSideBySide(cfg, 9, room=160)
    t.cycle(10, 6, 60)
    t.cycle(8, 4, 30)
    print("7B-width tree max error / tolerance:", t.max_err, "accepted:", t.n_hist, "near ties:", t.near_ties)


def test_tree_full_size_c2_emits_the_chain_text():
    """BASELINE's C2 at full size (32 layers), where the oracle cannot run: tree cycles (the paper's 10/6/60 setting, the
    61-row verify pass of bench.py --tree) and chain cycles on the same prompt must emit the same text, both being the
    target's greedy decoding; at a disagreement the library's own verify logits must show a near-tie there."""
    from paper_2509_23928_amd import Hivis
    cfg = synth.get_config("C2")
    w = synth.make_weights(cfg, seed=3, bits=True, threads=8)
    vis, ids = synth.make_prompt(cfg, seed=3)
    hv = Hivis(cfg, w, max_text=cfg.n_text + 200)
    del w
    want = 24

    def run(tree):
        first = hv.prefill(vis, ids)
        out, gaps = [int(first[0])], [np.inf]
        while len(out) < want:
            if tree:
                hv.tree_draft(10, 6, 60); hv.tree_verify()
                vlog = hv.get_logits(0)[0]
                rows = hv.tree_get(verified=True)
                n, toks = hv.tree_accept()
                path = accept_path(list(rows["row_parents"]), list(rows["row_tokens"]), rows["target_tokens"])
                assert n == len(path)
                used = [0] + path
            else:
                hv.draft(cfg.K); hv.verify()
                vlog = hv.get_logits(0)[0]
                nn, tt = hv.accept()
                n, toks = int(nn[0]), tt[0]
                used = list(range(n + 1))
            for i, r in enumerate(used):
                srt = np.sort(vlog[r])
                out.append(int(toks[i])); gaps.append(float(srt[-1] - srt[-2]))
                assert int(toks[i]) == int(np.argmax(vlog[r]))
        return out[:want], gaps[:want], float(np.sqrt(np.mean(vlog.astype(np.float64) ** 2)))

    chain, gaps_c, rms = run(False)
    tree, gaps_t, _ = run(True)
    for i in range(want):
        if chain[i] != tree[i]:
            assert min(gaps_c[i], gaps_t[i]) <= 6e-2 * rms, f"token {i}: chain {chain[i]} vs tree {tree[i]} with top-2 gaps {gaps_c[i]}, {gaps_t[i]}"
            break       # after a near-tie the two texts legitimately differ
    print("full-size C2: tree and chain agree on", i + 1 if chain[i] == tree[i] else i, "tokens")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tree_maximum_sizes(dtype):
    """The library's limits at once: top_k 16, 64 drafter tree rows (mask bit 63), 63 candidates = 64 verify rows."""
    cfg = c1(n_vis=40, n_text=11) if dtype == "f32" else small_bf16(n_vis=90, n_text=21)
    t = TreeSideBySide(cfg, 13)
    t.cycle(16, 5, 63)
    ref, _ = greedy_reference(cfg, t.w, t.vis[0], t.ids[0], 12)
    tokens, parents = branching_plant(ref, len(t.emitted), cfg.vocab, 8, 7)      # 63 planted rows, depth 9, path on rows 7, 14, .. 56
    n, path = t.planted_cycle(tokens, parents)
    if t.near_ties == 0:
        assert n == 8 and path[-1] == 56
    t.cycle(16, 5, 63)
    print(dtype, "maximum-size tree max error / tolerance:", t.max_err, "accepted:", t.n_hist)


@pytest.mark.parametrize("seed", list(range(40, 50)))
def test_tree_random_shape_sweep(seed):
    """Seeded random model shapes and tree shapes inside the documented limits: both head sizes, grouped heads, odd tile
    counts, vocabularies on both sides of one top-k segment (4096), caches from a few keys to several key tiles, trees
    from a single chain to 64 verify rows, fp32 and bf16."""
    rng = np.random.default_rng(seed)
    hd = int(rng.choice([64, 128]))
    n_kv = int(rng.choice([1, 2, 4]))
    n_q = n_kv * int(rng.choice([1, 2, 3]))
    k = int(rng.integers(1, 17))
    depth = int(rng.integers(1, min(8, 64 // k + 1) + 1))
    P = pool_size(k, depth)
    n_nodes = int(rng.integers(1, min(P, 63) + 1))
    common = dict(name=f"tree-sweep-{seed}", d=32 * int(rng.integers(4, 20)), n_q_heads=n_q, n_kv_heads=n_kv, head_dim=hd, ffn=32 * int(rng.integers(5, 60)),
                  vocab=32 * int(rng.integers(8, 300)), n_vis=int(rng.integers(0, 200)), n_text=int(rng.integers(1, 50)), n_layers=int(rng.integers(1, 4)))
    cfg = small_bf16(**common) if seed % 3 else c1(**common)
    try:
        t = TreeSideBySide(cfg, seed)
    except AssertionError as e:
        if "near-tie at the first token" in str(e):
            pytest.skip("near-tie at the first token for this seed")
        raise
    t.cycle(k, depth, n_nodes)
    ref, _ = greedy_reference(cfg, t.w, t.vis[0], t.ids[0], len(t.emitted) + 6)
    good, shape = int(rng.integers(0, 5)), int(rng.integers(1, 6))
    tokens, parents = branching_plant(ref, len(t.emitted), cfg.vocab, good, shape)
    t.planted_cycle(tokens, parents)
    t.cycle(k, depth, n_nodes)
    t.hv.close()
    print(f"tree sweep {seed}: {cfg.dtype} d={cfg.d} Hq/Hkv={n_q}/{n_kv} hd={hd} F={cfg.ffn} V={cfg.vocab} v={cfg.n_vis} l={cfg.n_text} N={cfg.n_layers} "
          f"tree {k}/{depth}/{n_nodes}", "max error / tolerance:", t.max_err, "accepted:", t.n_hist, "near ties:", t.near_ties)


def test_tree_qwen_vocabulary():
    """V = 152064 (38 top-k segments per row; LM head of the 41-row verify pass with 9504 column tiles)."""
    cfg = small_bf16(name="tree-bigvocab", d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512, vocab=152064, n_vis=60, n_text=12, n_layers=1)
    t = TreeSideBySide(cfg, 15)
    t.cycle(10, 3, 40)
    t.cycle(16, 2, 63)
    print("V=152064 tree max error / tolerance:", t.max_err, "accepted:", t.n_hist, "near ties:", t.near_ties)


def run_tree_sampling(cfg, seed, T, shapes, plant, device_seed=None):
    """Tree cycles accepted at temperature T.  shapes: one (k, depth, N) per cycle; plant: {cycle: m}: that cycle runs a
    planted branching tree whose followed path carries the next m tokens that token-by-token sampling with the cycle's
    uniforms emits.  device_seed: the library draws the uniforms itself (call c of the context)."""
    t = TreeSideBySide(cfg, seed)
    g = np.random.default_rng(500 + seed)
    if device_seed is not None:
        assert t.hv.rng_seed(device_seed) == 0
    for c, (k, depth, N) in enumerate(shapes):
        if c in plant:
            m = plant[c]
            depth = m + 1                                  # branching_plant: m path levels and one level of wrong tokens
        u = orng.uniforms(device_seed, c, orng.TREE, depth + 1) if device_seed is not None else g.random(depth + 1).astype(np.float32)
        give = (lambda uu=u: uu) if device_seed is not None else u
        if c in plant:
            done = len(t.emitted)
            ref = sampling_reference(cfg, t.w, t.vis[0], t.ids[0], done + m + 1, T, [0.0] + t.used_u + [float(x) for x in u])
            assert ref[:done] == t.emitted, "the text so far is not what token-by-token sampling emits"
            toks, pars = branching_plant(ref, done, cfg.vocab, m, 3)
            n, _ = t.planted_cycle(toks, pars, sample=(T, give))
            if t.edge == 0:
                assert n == m
        else:
            t.cycle(k, depth, N, sample=(T, give))
    if t.edge == 0 and t.near_ties == 0:
        ref = sampling_reference(cfg, t.w, t.vis[0], t.ids[0], len(t.emitted), T, [0.0] + t.used_u)
        assert t.emitted == ref, "tree cycles at T > 0 must emit what drawing one token at a time emits with the same uniforms"
    if device_seed is not None:
        assert t.hv.rng_seed(0) == len(shapes)
    return t


def test_tree_sampling_tiny_fp32_host_uniforms():
    cfg = c1(n_vis=40, n_text=19, n_q_heads=4, n_kv_heads=2)
    t = run_tree_sampling(cfg, 61, 1.0, [(3, 3, 9), (4, 2, 12), (2, 4, 7), (3, 3, 9), (5, 3, 31), (3, 2, 6)], {1: 2, 3: 4, 5: 1})
    print("tree sampling fp32:", t.max_err, "accepted:", t.n_hist, "draws:", t.draws, "edge:", t.edge)
    assert t.n_hist[1] >= 2 and t.n_hist[3] >= 4


def test_tree_sampling_bf16_device_uniforms():
    cfg = small_bf16(K=4)
    t = run_tree_sampling(cfg, 62, 0.8, [(3, 3, 9), (4, 3, 20), (2, 2, 4), (10, 3, 40)], {1: 3, 2: 1}, device_seed=0xC0FFEE1234)
    print("tree sampling bf16, device-drawn uniforms:", t.max_err, "accepted:", t.n_hist, "draws:", t.draws, "edge:", t.edge)


def test_tree_accept_sample_error_codes():
    from paper_2509_23928_amd import HivisError, HIVIS_EINVAL, HIVIS_ESTATE
    cfg = c1(n_vis=10, n_text=9, n_q_heads=4, n_kv_heads=2)
    w, vis, ids, hv = make_tree(cfg, 63, 100)
    hv.prefill(vis, ids)
    hv.tree_draft(3, 2, 6)
    with pytest.raises(HivisError) as e:
        hv.tree_accept_sample(1.0, [0.5, 0.5, 0.5])                  # not verified yet
    assert e.value.code == HIVIS_ESTATE
    hv.tree_verify()
    with pytest.raises(HivisError) as e:
        hv.tree_accept_sample(0.0, [0.5, 0.5, 0.5])
    assert e.value.code == HIVIS_EINVAL
    with pytest.raises(HivisError) as e:
        hv.tree_accept_sample(1.0, [0.5, 1.0, 0.5])
    assert e.value.code == HIVIS_EINVAL
    with pytest.raises(HivisError) as e:
        hv.tree_accept_sample(1.0, None)                             # no seed given yet
    assert e.value.code == HIVIS_ESTATE
    n, toks = hv.tree_accept_sample(1.0, [0.5, 0.5, 0.5])
    assert 0 <= n <= 2 and all(int(x) >= 0 for x in toks[: n + 1])
    hv.close()
