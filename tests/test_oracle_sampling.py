"""Pins of the oracle's temperature-sampling part (CPU only): inversion sampling against a plain loop and
exact dyadic cases, the temperature softmax against scipy, the acceptance rule's special cases, the
distribution-preservation property of speculative sampling (section 2.1 and the works it cites) by
Monte Carlo, and the T -> 0 limit against the greedy cycle."""
import numpy as np
import scipy.special

import synth
from oracle import (HivisOracle, HivisSamplingOracle, greedy_reference, sample_inverse_cdf, sampling_reference,
                    softmax_temperature, speculative_accept)
from small_models import tiny_cfg


def loop_inverse_cdf(w, u):
    total = 0.0
    for x in w:
        total += float(x)
    run, target = 0.0, u * total
    for j, x in enumerate(w):
        run += float(x)
        if run > target:
            return j
    return max(j for j, x in enumerate(w) if x > 0)


def test_inverse_cdf_matches_plain_loop():
    rng = np.random.default_rng(0)
    for _ in range(2000):
        n = int(rng.integers(1, 40))
        w = rng.random(n) ** 3
        w[rng.random(n) < 0.3] = 0.0
        if not np.any(w > 0):
            w[int(rng.integers(0, n))] = 1.0
        u = float(rng.random())
        assert sample_inverse_cdf(w, u) == loop_inverse_cdf(w, u)


def test_inverse_cdf_exact_dyadic_boundaries():
    w = [1.0, 1.0, 2.0]                       # running sums 1, 2, 4 of a total of 4: boundaries at u = 1/4 and 1/2
    assert sample_inverse_cdf(w, 0.0) == 0
    assert sample_inverse_cdf(w, 0.2499) == 0
    assert sample_inverse_cdf(w, 0.25) == 1   # the boundary belongs to the next index (running sum must EXCEED u * total)
    assert sample_inverse_cdf(w, 0.4999) == 1
    assert sample_inverse_cdf(w, 0.5) == 2
    assert sample_inverse_cdf(w, 0.999999) == 2
    assert sample_inverse_cdf([0.0, 0.0, 3.0, 0.0], 0.0) == 2      # leading zero weights are never drawn
    assert sample_inverse_cdf([2.0, 0.0, 0.0], 0.999) == 0         # trailing zero weights neither


def test_softmax_temperature_against_scipy_and_limits():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(5, 33)) * 3
    assert np.allclose(softmax_temperature(x, 1.0), scipy.special.softmax(x, axis=-1), rtol=1e-13, atol=0)
    assert np.allclose(softmax_temperature(x, 0.7), scipy.special.softmax(x / 0.7, axis=-1), rtol=1e-13, atol=0)
    assert np.allclose(softmax_temperature(x, 2.0).sum(-1), 1.0)
    assert np.allclose(softmax_temperature(x + 100.0, 1.3), softmax_temperature(x, 1.3))        # shift invariance
    cold = softmax_temperature(x, 1e-3)
    assert np.array_equal(cold.argmax(-1), x.argmax(-1)) and np.all(cold.max(-1) > 1 - 1e-9)     # T -> 0: one-hot on the argmax


def test_acceptance_rule_special_cases():
    rng = np.random.default_rng(2)
    V, K = 9, 4
    p = softmax_temperature(rng.normal(size=(K + 1, V)), 1.0)
    drafts = [int(t) for t in rng.integers(0, V, K)]
    # drafter == target: every draft accepted for any u < 1, the extra token is a sample of p[K]
    for _ in range(50):
        ua, ur = rng.random(K), float(rng.random())
        n, tok = speculative_accept(p, p[:K], drafts, ua, ur)
        assert n == K and tok == sample_inverse_cdf(p[K], ur)
    # the drafter proposes (with certainty) a token the target gives zero mass: rejected at once, replacement ~ p[0]
    p0 = p.copy(); p0[0, drafts[0]] = 0.0; p0[0] /= p0[0].sum()
    q = np.zeros((K, V)); q[np.arange(K), drafts] = 1.0
    for _ in range(50):
        ua, ur = rng.random(K), float(rng.random())
        n, tok = speculative_accept(p0, q, drafts, ua, ur)
        assert n == 0 and tok == sample_inverse_cdf(p0[0], ur)
    # acceptance probability is exactly p/q when p < q: p = 1/4, q = 1/2 -> accept iff u < 1/2
    pp = np.array([[0.25, 0.75], [0.5, 0.5]]); qq = np.array([[0.5, 0.5]])
    assert speculative_accept(pp, qq, [0], [0.4999], 0.3)[0] == 1
    assert speculative_accept(pp, qq, [0], [0.5], 0.3)[0] == 0
    # on that rejection the replacement comes from max(p - q, 0) = (0, 0.25): always token 1
    assert speculative_accept(pp, qq, [0], [0.9], 0.0) == (0, 1)
    # p >= q at the drafted token: always accepted
    assert speculative_accept(pp, qq, [1], [0.999999], 0.3)[0] == 1


def test_speculative_sampling_preserves_the_target_distribution():
    """Every emitted position is distributed as the target's own distribution for that position, whatever
    the drafter proposes (position-wise fixed p_i, q_i; 60000 seeded trials; 5 sigma)."""
    rng = np.random.default_rng(3)
    V, K, N = 7, 3, 60000
    p = softmax_temperature(rng.normal(size=(K + 1, V)) * 1.5, 1.0)
    q = softmax_temperature(rng.normal(size=(K, V)) * 1.5, 1.0)
    counts = np.zeros((K + 1, V)); trials = np.zeros(K + 1)
    n_hist = np.zeros(K + 1)
    for _ in range(N):
        drafts = [sample_inverse_cdf(q[i], float(rng.random())) for i in range(K)]
        n, tok = speculative_accept(p, q, drafts, rng.random(K), float(rng.random()))
        emitted = drafts[:n] + [tok]
        n_hist[n] += 1
        for i, t in enumerate(emitted):
            counts[i, t] += 1; trials[i] += 1
    for i in range(K + 1):
        freq = counts[i] / trials[i]
        sigma = np.sqrt(p[i] * (1 - p[i]) / trials[i])
        assert np.all(np.abs(freq - p[i]) < 5 * sigma + 1e-9), (i, freq, p[i])
    # expected acceptance probability of the first draft is sum_x min(p, q)
    assert abs((1 - n_hist[0] / N) - np.minimum(p[0], q[0]).sum()) < 5 * 0.5 / np.sqrt(N)


def test_cold_sampling_cycle_equals_greedy_cycle():
    cfg = tiny_cfg()
    w = synth.make_weights(cfg, seed=4)
    vis, ids = synth.make_prompt(cfg, seed=4)
    a, b = HivisOracle(cfg, w), HivisSamplingOracle(cfg, w)
    xa, _ = a.prefill(vis[0], ids[0]); xb, _ = b.prefill(vis[0], ids[0])
    assert xa == xb
    rng = np.random.default_rng(5)
    ea, eb = [xa], [xb]
    for _ in range(4):
        ra = a.cycle(cfg.K)
        rb = b.cycle_sample(cfg.K, 1e-4, rng.random(cfg.K), rng.random(cfg.K), float(rng.random()))
        ea += ra["emitted"]; eb += rb["emitted"]
        assert ra["n"] == rb["n"]
    assert ea == eb
    ref, _ = greedy_reference(cfg, w, vis[0], ids[0], len(ea))
    assert ea == ref
    assert sampling_reference(cfg, w, vis[0], ids[0], len(ea), 1e-4, rng.random(len(ea))) == ref


def test_sampling_cycle_state_equals_fresh_prefill():
    """After sampled cycles the oracle's caches equal those of a fresh prefill on the text so far (roll-forward intact).
    The fresh prefill picks its own (greedy) last token, so the drafter's last row, which carries that token's
    embedding, is left out of the comparison."""
    cfg = tiny_cfg()
    w = synth.make_weights(cfg, seed=6)
    vis, ids = synth.make_prompt(cfg, seed=6)
    o = HivisSamplingOracle(cfg, w)
    o.prefill(vis[0], ids[0])
    rng = np.random.default_rng(7)
    for _ in range(3):
        o.cycle_sample(cfg.K, 1.0, rng.random(cfg.K), rng.random(cfg.K), float(rng.random()))
    fresh = HivisSamplingOracle(cfg, w)
    fresh.prefill(vis[0], o.text[:-1])
    assert fresh.l == o.l and fresh.drafter.kv_len == o.drafter.kv_len and fresh.target.kv_len == o.target.kv_len
    n = o.drafter.kv_len - 1
    np.testing.assert_allclose(fresh.drafter.cache.k[:n], o.drafter.cache.k[:n], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(fresh.drafter.cache.v[:n], o.drafter.cache.v[:n], rtol=1e-9, atol=1e-11)
    # target side: the same next rows through both give the same features
    fresh.text[-1] = o.text[-1]
    drafts = [3, 1, 4]
    g1, l1, _ = fresh.verify(drafts); g2, l2, _ = o.verify(drafts)
    np.testing.assert_allclose(g1, g2, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(l1, l2, rtol=1e-8, atol=1e-10)


def test_prefill_sample_first_token():
    """The first token drawn at temperature T: equals the inversion draw from the prefill logits; a cold
    temperature gives the greedy token; a followed token is fed forward while the own draw is reported."""
    cfg = tiny_cfg()
    w = synth.make_weights(cfg, seed=8)
    vis, ids = synth.make_prompt(cfg, seed=8)
    g = HivisOracle(cfg, w); xg, lg = g.prefill(vis[0], ids[0])
    o = HivisSamplingOracle(cfg, w); x, logits = o.prefill_sample(vis[0], ids[0], 1.0, 0.37)
    np.testing.assert_allclose(logits, lg, rtol=1e-12, atol=1e-14)
    assert x == sample_inverse_cdf(softmax_temperature(lg, 1.0), 0.37) and o.text[-1] == x
    c = HivisSamplingOracle(cfg, w); xc, _ = c.prefill_sample(vis[0], ids[0], 1e-4, 0.9)
    assert xc == xg and np.array_equal(c.f_next, g.f_next)
    f = HivisSamplingOracle(cfg, w); xf, _ = f.prefill_sample(vis[0], ids[0], 1.0, 0.37, follow=(x + 1) % cfg.vocab)
    assert xf == x and f.text[-1] == (x + 1) % cfg.vocab
    ref = sampling_reference(cfg, w, vis[0], ids[0], 1, 1.0, [0.37], sample_first=True)
    assert ref == [x]
