"""GPU parity of the temperature-sampling calls (hivis_draft_sample / hivis_accept_sample) against the oracle.

Logits are compared as in the greedy tests (oracle in follow mode).  Every sampling DECISION (drawn draft, accepted
length, replacement / extra token) is an integer decided by floating point, so both sides take it from the same
numbers: the oracle re-takes each decision in float64 from the library's own float32 logits and the same uniforms;
a difference is tolerated only where the uniform lies within 1e-5 of the decision boundary (counted).

With `device_seed` the library draws its uniforms itself (hivis_rng_seed, NULL arrays); the test derives the numbers it
must have used from the oracle's own generator (oracle/rng.py: seed, call count, purpose, index) and checks every
decision exactly as above, so a wrong counter layout, key or bit-to-float mapping in the kernel shows as wrong draws."""
import numpy as np
import pytest

import synth
from oracle import HivisSamplingOracle, sample_inverse_cdf, softmax_temperature, speculative_accept
from oracle import rng as orng
from parity_utils import logit_tol
from test_gpu_parity import make, small_bf16

pytestmark = pytest.mark.gpu
EDGE = 1e-5


def near_cdf_boundary(weights, u, a, b):
    """u * total within EDGE * total of a running-sum boundary between indices a and b"""
    c = np.cumsum(np.asarray(weights, np.float64))
    lo, hi = min(a, b), max(a, b)
    return bool(np.min(np.abs(c[lo:hi] - u * c[-1])) <= EDGE * c[-1])


def run_sampling(cfg, seed, cycles, T, sample_first=False, device_seed=None):
    from paper_2509_23928_amd import HivisError, HIVIS_ESTATE, HIVIS_EINVAL
    w, vis, ids, hv = make(cfg, seed)
    B, K = cfg.batch, cfg.K
    rng = np.random.default_rng(1000 + seed)
    dev = device_seed is not None
    call = 0                                        # the library's count of drawing calls since the seeding
    if dev:
        with pytest.raises(HivisError) as e:        # NULL uniforms before any seeding
            hv.prefill_sample(vis, ids, T, None)
        assert e.value.code == HIVIS_ESTATE
        assert hv.rng_seed(device_seed) == 0
    stats = {"draws": 0, "edge": 0, "n_hist": np.zeros(K + 1, int), "max_err": 0.0}
    oracles = [HivisSamplingOracle(cfg, w) for _ in range(B)]
    if sample_first:
        if dev:
            u_f = orng.uniforms(device_seed, call, orng.FIRST_TOKEN, B); call += 1
            first = hv.prefill_sample(vis, ids, T, None)
        else:
            u_f = rng.random(B).astype(np.float32)
            first = hv.prefill_sample(vis, ids, T, u_f)
        plog = hv.get_logits(2).astype(np.float64)
        for b, o in enumerate(oracles):
            _, ologits = o.prefill_sample(vis[b], ids[b], T, float(u_f[b]), follow=int(first[b]))
            tol = logit_tol(cfg, ologits)
            assert float(np.max(np.abs(plog[b] - ologits))) <= tol
            pr = softmax_temperature(plog[b], T)
            mine = sample_inverse_cdf(pr, float(u_f[b]))
            stats["draws"] += 1
            if mine != int(first[b]):
                assert near_cdf_boundary(pr, float(u_f[b]), mine, int(first[b]))
                stats["edge"] += 1
    else:
        first = hv.prefill(vis, ids)
        for b, o in enumerate(oracles):
            x, _ = o.prefill(vis[b], ids[b])
            assert x == int(first[b]), "near-tie at the first token: pick another seed"
    # error paths: bad temperature / uniforms, and acceptance by sampling after greedy drafts
    with pytest.raises(HivisError) as e:
        hv.draft_sample(K, 0.0, rng.random((B, K)))
    assert e.value.code == HIVIS_EINVAL
    with pytest.raises(HivisError) as e:
        hv.draft_sample(K, 1.0, np.full((B, K), 1.0))
    assert e.value.code == HIVIS_EINVAL
    for cyc in range(cycles):
        if dev:
            u_d = orng.uniforms(device_seed, call, orng.DRAFT, B * K).reshape(B, K)
            u_a = orng.uniforms(device_seed, call + 1, orng.ACCEPT, B * K).reshape(B, K)
            u_r = orng.uniforms(device_seed, call + 1, orng.RESAMPLE, B)
            call += 2
            hv.draft_sample(K, T, None)
        else:
            u_d = rng.random((B, K)).astype(np.float32)
            u_a = rng.random((B, K)).astype(np.float32)
            u_r = rng.random(B).astype(np.float32)
            hv.draft_sample(K, T, u_d)
        hv.verify()
        drafts, _ = hv.get_tokens()
        dlog = hv.get_logits(1).astype(np.float64)      # [K][B][V]
        vlog = hv.get_logits(0).astype(np.float64)      # [B][K+1][V]
        if dev and cyc == 0:
            with pytest.raises(HivisError) as e:    # one array given, the other not
                hv.accept_sample(T, u_a, None)
            assert e.value.code == HIVIS_EINVAL
        n, toks = hv.accept_sample(T, None, None) if dev else hv.accept_sample(T, u_a, u_r)
        for b, o in enumerate(oracles):
            _, ologits = o.draft_sample(K, T, u_d[b], follow=drafts[b])
            tol = logit_tol(cfg, ologits)
            err = float(np.max(np.abs(dlog[:, b, :] - ologits)))
            stats["max_err"] = max(stats["max_err"], err / tol)
            assert err <= tol, f"draft logits off by {err} > {tol}"
            q = softmax_temperature(dlog[:, b, :], T)
            for i in range(K):
                mine = sample_inverse_cdf(q[i], float(u_d[b, i]))
                stats["draws"] += 1
                if mine != int(drafts[b, i]):
                    assert near_cdf_boundary(q[i], float(u_d[b, i]), mine, int(drafts[b, i])), (cyc, b, i, mine, drafts[b, i])
                    stats["edge"] += 1
            g, ovlog, _ = o.verify(drafts[b])
            tol = logit_tol(cfg, ovlog)
            err = float(np.max(np.abs(vlog[b] - ovlog)))
            stats["max_err"] = max(stats["max_err"], err / tol)
            assert err <= tol, f"verify logits off by {err} > {tol}"
            p = softmax_temperature(vlog[b], T)
            n_or, tok_or = speculative_accept(p, q, drafts[b], u_a[b], float(u_r[b]))
            n_lib, tok_lib = int(n[b]), int(toks[b, n[b]])
            stats["draws"] += 1
            if n_or != n_lib:
                i = min(n_or, n_lib)                         # the draft the two sides disagree about
                x = int(drafts[b, i])
                assert abs(float(u_a[b, i]) * q[i][x] - p[i][x]) <= EDGE * p[i][x], (cyc, b, "accept edge", n_or, n_lib)
                stats["edge"] += 1
            elif tok_or != tok_lib:
                wts = p[n_lib] if n_lib == K else np.maximum(p[n_lib] - q[n_lib], 0.0)
                assert near_cdf_boundary(wts, float(u_r[b]), tok_or, tok_lib), (cyc, b, "token edge", tok_or, tok_lib)
                stats["edge"] += 1
            assert list(toks[b, :n_lib]) == [int(t) for t in drafts[b, :n_lib]] and np.all(toks[b, n_lib + 1:] == -1)
            stats["n_hist"][n_lib] += 1
            o.accept_sample(drafts[b], dlog[:, b, :], g, ovlog, T, u_a[b], float(u_r[b]), force=(n_lib, list(toks[b, :n_lib + 1])))
        tl, dl = hv.kv_lengths()
        for b, o in enumerate(oracles):
            assert tl[b] == o.v + o.l and dl[b] == o.l
    # after a greedy draft the drafter's distributions are not the ones the drafts came from: refused
    hv.draft(K); hv.verify()
    with pytest.raises(HivisError) as e:
        hv.accept_sample(T, rng.random((B, K)), rng.random(B))
    assert e.value.code == HIVIS_ESTATE
    hv.accept()
    if dev:
        assert hv.rng_seed(device_seed + 1) == call         # every drawing call was counted once
    hv.close()
    assert stats["edge"] <= max(3, stats["draws"] // 5), stats
    return stats


def test_sampling_c1_fp32_temperature_one():
    st = run_sampling(synth.get_config("C1"), 0, 8, 1.0, sample_first=True)
    print("C1 T=1 sampling:", st)
    assert st["n_hist"].sum() == 8


def test_sampling_small_bf16_two_temperatures_batch2():
    cfg = small_bf16(batch=2, K=4)
    st = run_sampling(cfg, 41, 6, 1.0, sample_first=True)
    print("bf16 T=1 sampling:", st)
    st2 = run_sampling(cfg, 42, 6, 0.05)
    print("bf16 T=0.05 sampling:", st2)
    # a cold temperature makes the two models disagree visibly: rejections must occur
    assert st2["n_hist"][: cfg.K].sum() > 0


def test_sampling_full_vocab_width():
    # 7B-width LM head and vocabulary (V = 32000) on a 2-layer slice: the sampling kernels at the benchmark's row length
    cfg = synth.get_config("C2").scaled(n_layers=2, gen_tokens=0, gen_cycles=2, n_vis=64, n_text=24)
    st = run_sampling(cfg, 43, 2, 1.0)
    print("V=32000 T=1 sampling:", st)


def test_sampling_standalone_kernel_path():
    # HIVIS_FUSED=0: the draft loop draws its tokens with the stand-alone row-sampling kernel
    import os
    os.environ["HIVIS_FUSED"] = "0"
    try:
        st = run_sampling(small_bf16(K=3), 44, 4, 0.7)
        print("stand-alone path T=0.7 sampling:", st)
    finally:
        del os.environ["HIVIS_FUSED"]


def test_sampling_device_rng_fp32_and_bf16_batch2():
    # uniforms drawn on the device (Philox4x32-10); a 64-bit seed with both halves in use
    st = run_sampling(synth.get_config("C1"), 0, 6, 1.0, sample_first=True, device_seed=0x9E3779B97F4A7C15)
    print("C1 T=1 device-drawn uniforms:", st)
    assert st["n_hist"].sum() == 6
    st = run_sampling(small_bf16(batch=2, K=4), 45, 5, 0.8, sample_first=True, device_seed=7)
    print("bf16 batch 2 T=0.8 device-drawn uniforms:", st)
    assert st["n_hist"].sum() == 10
