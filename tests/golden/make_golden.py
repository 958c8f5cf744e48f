"""Writes tests/golden/c1_seed0_trace.json and tests/golden/c1_seed0_tree_trace.json from the CPU oracle alone (no GPU code is
imported or called).  The paper prints no value a synthetic run can reproduce, so this
file is a regression pin of the oracle on the tiny fp32 workload, not a value of the
paper: per cycle the drafts, the target's greedy tokens, the accepted length, and a few
logit samples.  Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth  # noqa: E402
from oracle import HivisOracle  # noqa: E402
from oracle.tree import HivisTreeOracle  # noqa: E402


def main():
    cfg = synth.get_config("C1")
    w = synth.make_weights(cfg, seed=0)
    vis, ids = synth.make_prompt(cfg, seed=0)
    o = HivisOracle(cfg, w)
    x, logits = o.prefill(vis[0], ids[0])
    trace = {"config": "C1", "seed": 0, "first_token": x, "first_logits_0_4": [float(t) for t in logits[:4]],
             "cycles": []}
    for c in range(cfg.gen_cycles):
        r = o.cycle(cfg.K)
        trace["cycles"].append({"drafts": r["drafts"], "target_tokens": r["target_tokens"], "n": r["n"],
                                "emitted": r["emitted"],
                                "verify_logit_row0_0_4": [float(t) for t in r["verify_logits"][0, :4]],
                                "draft_logit_step1_0_4": [float(t) for t in r["draft_logits"][0, :4]]})
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_seed0_trace.json")
    with open(path, "w") as fh:
        json.dump(trace, fh, indent=1)
    print("wrote", path)
    # draft-tree cycles on the same workload (top-3 tree, depth 3, 8 candidates)
    t = HivisTreeOracle(cfg, w)
    x, _ = t.prefill(vis[0], ids[0])
    tree_trace = {"config": "C1", "seed": 0, "top_k": 3, "depth": 3, "n_nodes": 8, "first_token": x, "cycles": []}
    for c in range(4):
        r = t.tree_cycle(3, 3, 8)
        tr = r["tree"]
        tree_trace["cycles"].append({"pool_tokens": [int(v) for v in tr["pool_tokens"]], "expand": tr["expand"], "selected": tr["selected"],
                                     "parents": tr["parents"], "target_tokens": r["target_tokens"], "n": r["n"], "emitted": r["emitted"],
                                     "pool_scores_0_4": [float(v) for v in tr["pool_scores"][:4]]})
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_seed0_tree_trace.json")
    with open(path, "w") as fh:
        json.dump(tree_trace, fh, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
