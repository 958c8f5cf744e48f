"""The oracle still reproduces the trace that tests/golden/make_golden.py wrote from it
(a regression pin: any later change to the oracle's arithmetic shows up here)."""
import json
import os

import numpy as np

import synth
from oracle import HivisOracle
from oracle.tree import HivisTreeOracle

HERE = os.path.dirname(os.path.abspath(__file__))


def test_c1_trace_reproduces():
    with open(os.path.join(HERE, "golden", "c1_seed0_trace.json")) as fh:
        gold = json.load(fh)
    cfg = synth.get_config("C1")
    w = synth.make_weights(cfg, seed=0)
    vis, ids = synth.make_prompt(cfg, seed=0)
    o = HivisOracle(cfg, w)
    x, logits = o.prefill(vis[0], ids[0])
    assert x == gold["first_token"]
    np.testing.assert_allclose(logits[:4], gold["first_logits_0_4"], rtol=1e-9)
    for c in gold["cycles"]:
        r = o.cycle(cfg.K)
        assert r["drafts"] == c["drafts"] and r["target_tokens"] == c["target_tokens"] and r["n"] == c["n"]
        np.testing.assert_allclose(r["verify_logits"][0, :4], c["verify_logit_row0_0_4"], rtol=1e-9)
        np.testing.assert_allclose(r["draft_logits"][0, :4], c["draft_logit_step1_0_4"], rtol=1e-9)


def test_c1_tree_trace_reproduces():
    with open(os.path.join(HERE, "golden", "c1_seed0_tree_trace.json")) as fh:
        gold = json.load(fh)
    cfg = synth.get_config("C1")
    w = synth.make_weights(cfg, seed=0)
    vis, ids = synth.make_prompt(cfg, seed=0)
    o = HivisTreeOracle(cfg, w)
    x, _ = o.prefill(vis[0], ids[0])
    assert x == gold["first_token"]
    for c in gold["cycles"]:
        r = o.tree_cycle(gold["top_k"], gold["depth"], gold["n_nodes"])
        tr = r["tree"]
        assert [int(v) for v in tr["pool_tokens"]] == c["pool_tokens"] and tr["expand"] == c["expand"] and tr["selected"] == c["selected"]
        assert tr["parents"] == c["parents"] and r["target_tokens"] == c["target_tokens"] and r["n"] == c["n"] and r["emitted"] == c["emitted"]
        np.testing.assert_allclose(tr["pool_scores"][:4], c["pool_scores_0_4"], rtol=1e-9)
