"""Pins of the oracle's draft-tree part (CPU only).  The tree cycle is pinned to things other than itself:
the chain cycle (a tree with k = 1), plain greedy decoding of the target (lossless output), plain causal
passes along every root-to-node path (tree mask and positions), scipy's log-softmax (scores), a sort-based
brute force and a hand-made example (selection), and an enumeration of all paths (acceptance)."""
import copy

import numpy as np
import scipy.special

import synth
from oracle import HivisOracle, greedy_reference
from oracle.tree import (HivisTreeOracle, accept_path, ancestors_visible, log_softmax, pool_size, top_k_lowest)
from small_models import tiny_cfg


def make(seed, **kw):
    cfg = tiny_cfg(**kw)
    w = synth.make_weights(cfg, seed=seed)
    vis, ids = synth.make_prompt(cfg, seed=seed)
    return cfg, w, vis[0], ids[0]


def path_to(parents, tokens, row):
    """Tokens and rows from the root's first child down to `row` (tree rows, 0 = root)."""
    rows = []
    while row > 0:
        rows.append(row)
        row = parents[row - 1]
    rows.reverse()
    return rows, [tokens[r - 1] for r in rows]


def test_top_k_lowest_against_sort_and_ties():
    rng = np.random.default_rng(0)
    for _ in range(300):
        n = int(rng.integers(1, 60))
        v = np.round(rng.normal(size=n), 1)                 # rounding makes ties frequent
        k = int(rng.integers(1, n + 1))
        brute = [i for _, i in sorted((-float(x), i) for i, x in enumerate(v))][:k]
        assert top_k_lowest(v, k) == brute
    assert top_k_lowest([1.0, 3.0, 3.0, 2.0, 3.0], 3) == [1, 2, 4]
    assert top_k_lowest([-np.inf, 0.0, -np.inf], 2) == [1, 0]


def test_log_softmax_against_scipy():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(6, 41)) * 4
    np.testing.assert_allclose(log_softmax(x), scipy.special.log_softmax(x, axis=-1), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(np.exp(log_softmax(x)).sum(-1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(log_softmax(x + 1000.0), log_softmax(x), rtol=0, atol=1e-11)


def test_ancestor_mask_hand_example():
    #      0
    #    1   2
    #   3 4    5
    #   6
    parents = [-1, 0, 0, 1, 1, 2, 3]
    vis = ancestors_visible(parents)
    expect = {0: [0], 1: [0, 1], 2: [0, 2], 3: [0, 1, 3], 4: [0, 1, 4], 5: [0, 2, 5], 6: [0, 1, 3, 6]}
    for i in range(7):
        assert [j for j in range(7) if vis[i, j]] == expect[i]


def test_accept_path_hand_examples_and_brute_force():
    parents = [-1, 0, 0, 1, 1, 2, 3]
    tokens = [9, 5, 7, 2, 4, 2, 8]
    # target continues 5, 2, 8 after the root: path 1 -> 3 -> 6
    assert accept_path(parents, tokens, [5, 2, 2, 8, 0, 0, 1]) == [1, 3, 6]
    # the target's first token is in no child of the root
    assert accept_path(parents, tokens, [6, 2, 2, 8, 0, 0, 1]) == []
    # the second branch: 7 then 2 (row 5), whose own continuation is not in the tree
    assert accept_path(parents, tokens, [7, 0, 2, 0, 0, 3, 0]) == [2, 5]
    # brute force: for every root-to-node path, the number of leading tokens that agree with the target's token at the
    # previous node; the accepted path is the longest fully agreeing one
    rng = np.random.default_rng(2)
    for _ in range(200):
        m = int(rng.integers(2, 14))
        par = [-1] + [int(rng.integers(0, i)) for i in range(1, m)]
        tok = [0] * m
        for p in range(m):                                    # siblings get distinct tokens (top-k of one distribution)
            kids = [c for c in range(1, m) if par[c] == p]
            for c, t in zip(kids, rng.permutation(6)[:len(kids)] if len(kids) <= 6 else range(len(kids))):
                tok[c] = int(t)
        tt = [int(t) for t in rng.integers(0, 6, m)]
        best = []
        for node in range(1, m):
            rows = []
            r = node
            while r > 0:
                rows.append(r); r = par[r]
            rows.reverse()
            ok = all(tok[c] == tt[par[c]] for c in rows)
            if ok and len(rows) > len(best):
                best = rows
        assert accept_path(par, tok, tt) == best


def test_tree_with_k1_is_the_chain():
    """top-1 expansion: the pool is the chain of Algorithm 1, every step (drafts, verify features, accepted
    length, emitted tokens, state afterwards) equals the chain cycle."""
    cfg, w, vis, ids = make(11)
    a, b = HivisOracle(cfg, w), HivisTreeOracle(cfg, w)
    a.prefill(vis, ids); b.prefill(vis, ids)
    for cyc in range(4):
        K = 1 + cyc % 3
        ra = a.cycle(K)
        rb = b.tree_cycle(1, K, K)
        assert rb["tree"]["tokens"] == ra["drafts"]
        assert rb["tree"]["parents"] == list(range(K)) and rb["tree"]["depths"] == list(range(1, K + 1))
        np.testing.assert_allclose(rb["g"], ra["g"], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(rb["tree"]["logp"], scipy.special.log_softmax(ra["draft_logits"], axis=-1), rtol=1e-9, atol=1e-11)
        assert rb["n"] == ra["n"] and rb["emitted"] == ra["emitted"]
        np.testing.assert_allclose(b.f_next, a.f_next, rtol=1e-10, atol=1e-12)
        assert b.l == a.l and b.target.kv_len == a.target.kv_len and b.drafter.kv_len == a.drafter.kv_len
        np.testing.assert_allclose(b.target.caches[-1].k, a.target.caches[-1].k, rtol=1e-10, atol=1e-12)


def test_tree_cycles_reproduce_greedy_decoding():
    """Lossless at T = 0: whatever the tree holds, the emitted text is the target's own greedy text."""
    for seed, (k, depth, n_nodes) in [(21, (3, 3, 7)), (22, (2, 4, 9)), (23, (4, 2, 20)), (24, (3, 4, 30))]:
        cfg, w, vis, ids = make(seed)
        o = HivisTreeOracle(cfg, w)
        x, _ = o.prefill(vis, ids)
        out = [x]
        for _ in range(5):
            out += o.tree_cycle(k, depth, n_nodes)["emitted"]
        ref, _ = greedy_reference(cfg, w, vis, ids, len(out))
        assert out == ref


def planted_follow(o, k, depth, n_nodes, continuation):
    """Choices of a tree that contains `continuation` as its first-ranked path: the oracle's own tree is built
    first, then the rank-0 child at every level of the rank-0 row is replaced by the continuation's token."""
    probe = copy.deepcopy(o)
    own = probe.tree_draft(k, depth, n_nodes)
    toks = np.array(own["pool_tokens"]).copy()
    first = 0
    for j in range(depth):
        if j < len(continuation):
            t = int(continuation[j])
            group = list(range(first, first + k))
            # keep siblings distinct: if the token is already another sibling, swap
            for i in group:
                if toks[i] == t:
                    toks[i] = toks[first]
            toks[first] = t
        first = k if j == 0 else first + k * k     # rank-0 child group of the rank-0 row of the next level
    expand = []
    lf, ln = 0, k
    for j in range(1, depth):
        expand.append([lf + i for i in range(k)])          # the first k nodes of each level (contains the planted path)
        lf, ln = lf + ln, k * k
    sel = sorted(set(list(range(k)) + [e for E in expand for e in E] + [lf + i for i in range(k)]))[:n_nodes]
    return {"pool_tokens": toks, "expand": expand, "selected": sel}


def test_planted_path_is_accepted_whole():
    """A tree that contains the target's own continuation accepts all of it (depth tokens) and emits depth + 1."""
    cfg, w, vis, ids = make(31)
    k, depth = 3, 3
    n_nodes = 9
    ref, _ = greedy_reference(cfg, w, vis, ids, 12)
    o = HivisTreeOracle(cfg, w)
    x, _ = o.prefill(vis, ids)
    assert x == ref[0]
    out = [x]
    for _ in range(2):
        cont = ref[len(out): len(out) + depth]
        f = planted_follow(o, k, depth, n_nodes, cont)
        o.tree_draft(k, depth, n_nodes, follow=f)
        g, logits, t = o.tree_verify()
        n, emitted, path = o.tree_accept(g, t)
        assert n == depth and emitted == ref[len(out): len(out) + depth + 1]
        out += emitted
    # state after compaction: the next plain chain cycle still reproduces greedy decoding
    out += o.cycle(2)["emitted"]
    assert out == ref[:len(out)]


def test_every_tree_row_equals_a_plain_causal_pass_along_its_path():
    """Tree mask + positions: the verify features of node i equal those of an ordinary causal pass over
    [root, path to i]; the drafter's distribution behind node i equals the chain drafter fed that path."""
    cfg, w, vis, ids = make(41)
    k, depth, n_nodes = 3, 3, 18
    o = HivisTreeOracle(cfg, w)
    o.prefill(vis, ids)
    o.tree_cycle(k, depth, n_nodes)                                         # move off the prompt state first
    before = copy.deepcopy(o)
    tree = o.tree_draft(k, depth, n_nodes)
    g, logits, t = o.tree_verify()
    assert len(set(tree["depths"])) == depth                                # the tree reaches every depth
    for row in range(1, n_nodes + 1):
        rows, toks = path_to(tree["parents"], tree["tokens"], row)
        assert tree["depths"][row - 1] == len(rows)
        chain = HivisOracle(cfg, w)
        chain.__dict__.update(copy.deepcopy(before.__dict__))
        gc, lc, _ = chain.verify(toks)
        np.testing.assert_allclose(g[row], gc[-1], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(g[0], gc[0], rtol=1e-9, atol=1e-11)
    # drafter side: every pool node's score is the sum of chain log-probabilities along its path
    pt, pp, ps = tree["pool_tokens"], tree["pool_parents"], tree["pool_scores"]
    for node in range(pool_size(k, depth)):
        toks, a = [], node
        while a >= 0:
            toks.append(int(pt[a])); a = int(pp[a])
        toks.reverse()
        chain = HivisOracle(cfg, w)
        chain.__dict__.update(copy.deepcopy(before.__dict__))
        _, dl = chain.draft(len(toks), follow=toks)
        lp = scipy.special.log_softmax(dl, axis=-1)
        assert abs(sum(lp[i][toks[i]] for i in range(len(toks))) - ps[node]) < 1e-9
        # siblings are the k most probable continuations, best first
        if node % k == 0:
            sib = [int(pt[node + r]) for r in range(k)]
            assert sib == [int(i) for i in np.argsort(-lp[-1], kind="stable")[:k]]


def test_pool_layout_selection_and_closure():
    cfg, w, vis, ids = make(51)
    k, depth, n_nodes = 3, 4, 14
    o = HivisTreeOracle(cfg, w)
    o.prefill(vis, ids)
    tree = o.tree_draft(k, depth, n_nodes)
    P = pool_size(k, depth)
    pp, ps, pd = tree["pool_parents"], tree["pool_scores"], tree["pool_depths"]
    assert len(pp) == P == 3 + 3 * 9
    # level layout: k nodes of depth 1, then k*k per further level; parents precede children and never score lower
    assert list(pd[:k]) == [1] * k and all(pp[:k] == -1)
    for j in range(1, depth):
        lo = k + (j - 1) * k * k
        assert list(pd[lo:lo + k * k]) == [j + 1] * (k * k)
        assert [int(pp[lo + r * k + c]) for r in range(k) for c in range(k)] == [e for e in tree["expand"][j - 1] for _ in range(k)]
        # the expanded rows are the k best-scored nodes of the level before
        prev_lo, prev_n = (0, k) if j == 1 else (k + (j - 2) * k * k, k * k)
        brute = [i for _, i in sorted((-float(ps[i]), i) for i in range(prev_lo, prev_lo + prev_n))][:k]
        assert tree["expand"][j - 1] == brute
    assert all(pp[i] < i and ps[i] <= ps[pp[i]] for i in range(k, P))
    # candidates: the n_nodes best of the whole pool, in pool order, closed under ancestors
    brute = sorted([i for _, i in sorted((-float(ps[i]), i) for i in range(P))][:n_nodes])
    assert tree["selected"] == brute
    assert all(int(pp[s]) == -1 or int(pp[s]) in tree["selected"] for s in tree["selected"])
    assert all(p < r for r, p in enumerate(tree["parents"], start=1))
    # candidate sets are nested in n_nodes, so the accepted length cannot shrink when more candidates are verified
    n_prev = -1
    for nn in (3, 8, 14, 25):
        oo = HivisTreeOracle(cfg, w); oo.prefill(vis, ids)
        r = oo.tree_cycle(k, depth, nn)
        assert set(r["tree"]["selected"]) >= set(brute[:0]) and r["n"] >= n_prev
        n_prev = r["n"]


def test_follow_mode_reproduces_own_choices():
    """Feeding the oracle its own choices back changes nothing (the follow plumbing is neutral)."""
    cfg, w, vis, ids = make(61)
    a, b = HivisTreeOracle(cfg, w), HivisTreeOracle(cfg, w)
    a.prefill(vis, ids); b.prefill(vis, ids)
    ta = a.tree_draft(3, 3, 10)
    tb = b.tree_draft(3, 3, 10, follow={"pool_tokens": ta["pool_tokens"], "expand": ta["expand"], "selected": ta["selected"]})
    np.testing.assert_array_equal(ta["pool_tokens"], tb["pool_tokens"])
    np.testing.assert_allclose(ta["pool_scores"], tb["pool_scores"], rtol=0, atol=0)
    assert ta["parents"] == tb["parents"] and ta["tokens"] == tb["tokens"]


# ---- acceptance at T > 0 (sample_tree_tokens: a reading, see its docstring) -------------------------------------

def run_tree_sampling(cfg, w, vis, ids, shape, T, cycles, seed, plant=None):
    """Tree cycles with drawn target tokens.  Returns (text after the first token, the uniforms in the order in which
    emitted tokens consumed them, accepted lengths)."""
    from oracle import sampling_reference
    k, depth, n_nodes = shape
    g = np.random.default_rng(seed)
    o = HivisTreeOracle(cfg, w)
    first, _ = o.prefill(vis, ids)
    text, used, ns = [], [], []
    for c in range(cycles):
        u = g.random(depth + 1)
        follow = None
        if plant is not None and c in plant:
            # a tree holding what token-by-token sampling with THESE uniforms is about to emit
            ref = sampling_reference(cfg, w, vis, ids, 1 + len(text) + depth, T, [0.0] + used + list(u))
            follow = planted_follow(o, k, depth, n_nodes, ref[1 + len(text): 1 + len(text) + plant[c]])
        o.tree_draft(k, depth, n_nodes, follow=follow)
        gfeat, logits, _ = o.tree_verify()
        n, emitted, path, _ = o.tree_accept_sample(gfeat, logits, T, u)
        assert len(emitted) == n + 1 and len(path) == n
        text += emitted
        used += list(u[: n + 1])
        ns.append(n)
    return first, text, used, ns


def test_tree_sampling_emits_exactly_the_token_by_token_samples():
    """With the same uniform numbers, tree cycles at T > 0 emit the very text that drawing one token at a time from
    the target emits (the plain definition): own trees (mostly rejected at once), and planted trees whose first path
    carries 1..depth of the coming samples (accepted exactly that far)."""
    from oracle import sampling_reference
    for seed, shape, T, plant in [(31, (3, 3, 7), 1.0, None), (32, (2, 4, 8), 0.7, {1: 2, 3: 4}), (33, (3, 3, 9), 1.3, {0: 3, 2: 1})]:
        cfg, w, vis, ids = make(seed)
        first, text, used, ns = run_tree_sampling(cfg, w, vis, ids, shape, T, 5, 100 + seed, plant)
        ref = sampling_reference(cfg, w, vis, ids, 1 + len(text), T, [0.0] + used)
        assert [first] + text == ref
        if plant:
            for c, m in plant.items():
                assert ns[c] >= m                      # the planted prefix is followed (further only by coincidence)
        # the state afterwards is a valid one: greedy chain cycles continue the text like a fresh prefill would
        assert sum(ns) >= (sum(plant.values()) if plant else 0)


def test_tree_sampling_first_token_distribution_is_the_targets():
    """Over a fine grid of u_0 the first emitted token is distributed as softmax(logits / T) of the root row, whether or
    not the tree holds it (the fraction of the grid that emits token x is p(x) within the grid's resolution)."""
    from oracle import softmax_temperature
    from oracle.tree import sample_tree_tokens
    cfg, w, vis, ids = make(34)
    o = HivisTreeOracle(cfg, w)
    o.prefill(vis, ids)
    o.tree_draft(3, 2, 6)
    gfeat, logits, _ = o.tree_verify()
    T = 0.9
    p = softmax_temperature(logits[0], T)
    n = 4000
    counts = np.zeros(cfg.vocab)
    accepted_mass = 0
    kids = {o.tree["tokens"][i] for i in range(len(o.tree["tokens"])) if o.tree["parents"][i] == 0}
    for i in range(n):
        u = [(i + 0.5) / n, 0.5, 0.5]
        t = sample_tree_tokens(logits, [0] + o.tree["depths"], T, u)
        counts[t[0]] += 1
        path = accept_path([-1] + o.tree["parents"], [o.text[-1]] + o.tree["tokens"], t)
        accepted_mass += 1 if path else 0
    assert np.max(np.abs(counts / n - p)) <= 1.0 / n + 1e-12
    assert abs(accepted_mass / n - sum(p[x] for x in kids)) <= len(kids) / n + 1e-12      # followed iff the draw is a child's token


def test_tree_sampling_cold_temperature_is_the_greedy_walk():
    """T -> 0: the drawn tokens are the greedy ones (for any u away from 0 and 1), so the walk is tree_accept's."""
    from oracle.tree import sample_tree_tokens
    cfg, w, vis, ids = make(35)
    o = HivisTreeOracle(cfg, w)
    o.prefill(vis, ids)
    o.tree_draft(3, 3, 9)
    gfeat, logits, t_greedy = o.tree_verify()
    t = sample_tree_tokens(logits, [0] + o.tree["depths"], 1e-4, [0.37, 0.81, 0.05, 0.5])
    assert t == t_greedy
