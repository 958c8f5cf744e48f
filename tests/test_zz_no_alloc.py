"""hivis_draft_noalloc (the draft round with its intermediate buffers in the library's static scratch array, for callers
that cannot allocate device memory) against hivis_draft on the same seeded inputs, through the C ABI.

Two contexts with the same weights: A drafts with hivis_draft, B with hivis_draft_noalloc.  Two rounds in a row on each,
the second on a smaller input (shorter prompt, fewer visual rows, smaller K), so that B's second round runs over the
scratch contents the first one left behind.  The kernels and their order are the same on both sides, so the drafted
tokens must be identical and the logits equal within the float tolerance of the parity tests (in practice bit-equal);
the pending state afterwards (cache lengths, verify logits of the drafted rows, next hidden state) must agree too.
The first of B's two draft rounds is also checked against the CPU oracle."""
import numpy as np
import pytest

import synth
from parity_utils import logit_tol, check_token
from oracle import HivisOracle

pytestmark = pytest.mark.gpu


def small_bf16(**kw):
    base = dict(name="small-bf16", n_layers=2, d=512, n_q_heads=4, n_kv_heads=4, head_dim=128, ffn=1376, vocab=2048,
                dtype="bf16", n_vis=150, n_text=37, K=5, batch=1, gen_tokens=0, gen_cycles=6)
    base.update(kw)
    return synth.HivisConfig(**base)


def one_round(hv, K, noalloc):
    if noalloc:
        hv.draft_noalloc(K)
    else:
        hv.draft(K)
    dlog = hv.get_logits(1)
    hv.verify()
    drafts, ttok = hv.get_tokens()
    vlog = hv.get_logits(0)
    n, toks = hv.accept()
    return {"drafts": drafts, "dlog": dlog, "ttok": ttok, "vlog": vlog, "n": n, "toks": toks,
            "lens": hv.kv_lengths(), "fnext": hv.get_hidden(1)}


def compare(a, b, cfg):
    assert np.array_equal(a["drafts"], b["drafts"]), (a["drafts"], b["drafts"])
    tol = logit_tol(cfg, a["dlog"])
    err = float(np.max(np.abs(a["dlog"] - b["dlog"])))
    assert err <= tol, f"draft logits differ by {err} > {tol}"
    assert np.array_equal(a["ttok"], b["ttok"]) and np.array_equal(a["n"], b["n"]) and np.array_equal(a["toks"], b["toks"])
    assert float(np.max(np.abs(a["vlog"] - b["vlog"]))) <= logit_tol(cfg, a["vlog"])
    assert np.array_equal(a["lens"][0], b["lens"][0]) and np.array_equal(a["lens"][1], b["lens"][1])
    scale = float(np.sqrt(np.mean(a["fnext"].astype(np.float64) ** 2)))
    assert float(np.max(np.abs(a["fnext"] - b["fnext"]))) <= (2e-4 if cfg.dtype == "f32" else 6e-2) * scale
    return err


@pytest.mark.parametrize("which", ["c1_f32", "small_bf16", "bf16_batch4"])
def test_draft_noalloc_matches_draft_two_calls_in_a_row(which):
    from paper_2509_23928_amd import Hivis
    if which == "c1_f32":
        cfg = synth.get_config("C1")
    elif which == "small_bf16":
        cfg = small_bf16()
    else:
        cfg = small_bf16(batch=4, K=7, n_vis=90, n_text=45)
    w = synth.make_weights(cfg, seed=3)
    vis, ids = synth.make_prompt(cfg, seed=3)
    A, B = Hivis(cfg, w), Hivis(cfg, w)
    # ---- call 1: the full prompt, K drafts
    fa, fb = A.prefill(vis, ids), B.prefill(vis, ids)
    assert np.array_equal(fa, fb)
    ra, rb = one_round(A, cfg.K, False), one_round(B, cfg.K, True)
    e1 = compare(ra, rb, cfg)
    # the same round against the oracle (follow mode): logits within tolerance, tokens up to near-ties
    for b in range(cfg.batch):
        o = HivisOracle(cfg, w)
        x, _ = o.prefill(vis[b], ids[b])
        if x != int(fb[b]):
            continue                                   # near-tie at the first token: nothing to follow
        _, ologits = o.draft(cfg.K, follow=rb["drafts"][b])
        tol = logit_tol(cfg, ologits)
        assert float(np.max(np.abs(rb["dlog"][:, b, :] - ologits))) <= tol
        for i in range(cfg.K):
            check_token(rb["drafts"][b, i], ologits[i], tol)
    # ---- call 2, straight after: a smaller input (shorter prompt, fewer visual rows, fewer drafts)
    v2, l2, K2 = cfg.n_vis // 2, cfg.n_text // 2 + 1, max(1, cfg.K // 2)
    vis2 = np.ascontiguousarray(vis[:, :v2]); ids2 = np.ascontiguousarray(ids[:, :l2])
    fa, fb = A.prefill(vis2, ids2), B.prefill(vis2, ids2)
    assert np.array_equal(fa, fb)
    ra, rb = one_round(A, K2, False), one_round(B, K2, True)
    e2 = compare(ra, rb, cfg)
    # and one more cycle on the rolled-forward state, back at the full K
    ra, rb = one_round(A, cfg.K, False), one_round(B, cfg.K, True)
    e3 = compare(ra, rb, cfg)
    print(which, "max |draft logits (noalloc) - draft logits|:", e1, e2, e3)
    A.close(); B.close()


def test_draft_noalloc_rejects_what_it_cannot_hold():
    from paper_2509_23928_amd import Hivis, HivisError, HIVIS_ESTATE, HIVIS_EINVAL, HIVIS_ECAP
    cfg = synth.get_config("C1")
    w = synth.make_weights(cfg, seed=0)
    vis, ids = synth.make_prompt(cfg, seed=0)
    hv = Hivis(cfg, w)
    with pytest.raises(HivisError) as e:
        hv.draft_noalloc(2)                            # before prefill
    assert e.value.code == HIVIS_ESTATE
    hv.prefill(vis, ids)
    with pytest.raises(HivisError) as e:
        hv.draft_noalloc(cfg.K + 1)
    assert e.value.code == HIVIS_EINVAL
    hv.draft_noalloc(cfg.K)                            # still usable afterwards
    hv.verify(); hv.accept()
    hv.close()
    # a round whose buffers exceed the static array (31 draft steps x ~1 MB of attention key-split partials each, with 32
    # kv heads): refused, nothing runs
    big = small_bf16(K=31, gen_cycles=2, n_q_heads=32, n_kv_heads=32)
    w = synth.make_weights(big, seed=0)
    vis, ids = synth.make_prompt(big, seed=0)
    hv = Hivis(big, w)
    hv.prefill(vis, ids)
    with pytest.raises(HivisError) as e:
        hv.draft_noalloc(31)
    assert e.value.code == HIVIS_ECAP and "scratch" in str(e.value)
    hv.draft_noalloc(4)                                # a round that fits still runs on the same context
    hv.verify(); hv.accept()
    hv.close()
