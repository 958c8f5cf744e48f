"""GPU parity AT DEPTH: the benchmarked LLaVA-1.5-7B-shaped model as configured (32 layers, 576 + 64 prompt rows,
K = 5), the Qwen2.5-VL-7B- and LLaVA-1.5-13B-shaped widths at 8 layers, and the LLaVA-NeXT prompt (2880 visual + 128
text rows) at 4 layers, against the CPU oracle.

What depth adds over the 2-layer slices of test_gpu_parity.py is rounding that accumulates layer after layer: the
quantity the tolerance (3e-2 x logit RMS for bf16 models) exists to bound.  Every logit of the prefill row, of the
draft rows and of the verify rows is compared; tokens follow the near-tie rule; the worst error / tolerance is printed.

The oracle computes in float64 and cannot hold a 7B model widened (53 GB): it reads the SAME bf16 bit patterns the
library is given through synth.LazyWeights, which widens one tensor at a time on access (exact values, no arithmetic of
the method).  One full-depth oracle prefill takes ~20-40 s on 16 host cores and one cycle ~10-20 s.
"""
import time

import numpy as np
import pytest

import synth
from synth.lazy import LazyWeights
from parity_utils import SideBySide

pytestmark = pytest.mark.gpu


def build(cfg, seed):
    from paper_2509_23928_amd import Hivis
    t0 = time.time()
    bits = synth.make_weights(cfg, seed=seed, bits=True, threads=16)
    vis, ids = synth.make_prompt(cfg, seed=seed)
    hv = Hivis(cfg, bits)
    print(f"[{cfg.name}] weights generated + uploaded in {time.time() - t0:.1f}s", flush=True)
    return bits, vis, ids, hv


def library_continuation(hv, cfg, vis, ids, n_cycles):
    """The library's own greedy text after the prompt (first token + what n_cycles chain cycles emit), per sequence:
    used to plant drafts the target will accept.  The side-by-side run afterwards checks each of these tokens against
    the oracle's logits (near-tie rule), so nothing is taken on trust."""
    first = hv.prefill(vis, ids)
    text = [[int(first[b])] for b in range(hv.B)]
    for _ in range(n_cycles):
        hv.draft(cfg.K)
        hv.verify()
        n, toks = hv.accept()
        for b in range(hv.B):
            text[b] += [int(t) for t in toks[b, : int(n[b]) + 1]]
    return text


def run_depth_case(cfg, seed, plant):
    """plant: per sequence, how many leading drafts of the second cycle are the target's own continuation."""
    assert len(plant) == cfg.batch
    bits, vis, ids, hv = build(cfg, seed)
    cont = library_continuation(hv, cfg, vis, ids, max(plant) + 2)
    t0 = time.time()
    sbs = SideBySide(cfg, LazyWeights(bits), hv, vis, ids)       # prefills the library again (state reset) and the oracle
    print(f"[{cfg.name}] oracle prefill + comparison {time.time() - t0:.1f}s: {sbs.summary()}", flush=True)
    # cycle 1: the library's own drafts (a random-init drafter is almost never accepted)
    t0 = time.time()
    r1 = sbs.cycle(cfg.K)
    print(f"[{cfg.name}] own-draft cycle {time.time() - t0:.1f}s: accepted {[x['n'] for x in r1]}", flush=True)
    # cycle 2: planted drafts whose first `plant` tokens are the target's own continuation, the rest wrong
    planted = []
    for b in range(cfg.batch):
        done = len(sbs.emitted[b])
        assert sbs.emitted[b] == cont[b][:done], "the library's text is not reproducible run to run"
        good = cont[b][done: done + plant[b]]
        assert len(good) == plant[b]
        bad = [(cont[b][min(done + j, len(cont[b]) - 1)] + 1 + j) % cfg.vocab for j in range(plant[b], cfg.K)]
        planted.append(good + bad)
    t0 = time.time()
    r2 = sbs.cycle(cfg.K, planted=np.array(planted, np.int32))
    print(f"[{cfg.name}] planted cycle {time.time() - t0:.1f}s: accepted {[x['n'] for x in r2]}", flush=True)
    assert all(x["n"] >= m for x, m in zip(r2, plant))        # SideBySide has checked every accepted token against the oracle
    if sbs.near_ties == 0:
        assert [x["n"] for x in r2] == list(plant)
    print(f"[{cfg.name}] N={cfg.n_layers}: {sbs.summary()}", flush=True)
    hv.close()
    return sbs


@pytest.mark.timeout(600)
def test_c2_full_depth_32_layers():
    """BASELINE's headline workload as benchmarked: 32 layers, d 4096, 32 heads, F 11008, V 32000, 576 visual + 64 text
    rows, K = 5, batch 1."""
    cfg = synth.get_config("C2")
    sbs = run_depth_case(cfg, seed=0, plant=[3])
    assert max(sbs.max_err.values()) <= 1.0


@pytest.mark.timeout(600)
def test_c4_widths_8_layers():
    """Qwen2.5-VL-7B widths (d 3584, 28 query / 4 kv heads, F 18944, V 152064, theta 1e6, 1024 visual + 96 text rows,
    K = 6) at 8 layers."""
    cfg = synth.get_config("C4").scaled(n_layers=8, name="C4-widths-8-layers", gen_tokens=0, gen_cycles=8)
    sbs = run_depth_case(cfg, seed=0, plant=[2])
    assert max(sbs.max_err.values()) <= 1.0


@pytest.mark.timeout(600)
def test_c5_widths_8_layers_batch4():
    """LLaVA-1.5-13B widths (d 5120, 40 heads, F 13824, 576 visual + 256 text rows, K = 7, batch 4: 32-row passes) at
    8 layers, per-sequence acceptance with a different planted length per sequence."""
    cfg = synth.get_config("C5").scaled(n_layers=8, name="C5-widths-8-layers", gen_tokens=0, gen_cycles=8)
    sbs = run_depth_case(cfg, seed=0, plant=[2, 0, 3, 1])
    assert max(sbs.max_err.values()) <= 1.0


@pytest.mark.timeout(600)
def test_c3_prompt_3008_rows_4_layers():
    """LLaVA-NeXT-7B prompt shape (2880 visual + 128 text rows: 24 row blocks of the prefill GEMM's large tile, 24 row
    blocks x 32 heads of the shared-tile prefill attention, 16 key splits per head in the verify attention) at 4 layers."""
    cfg = synth.get_config("C3").scaled(n_layers=4, name="C3-rows-4-layers", gen_tokens=0, gen_cycles=8)
    sbs = run_depth_case(cfg, seed=0, plant=[4])
    assert max(sbs.max_err.values()) <= 1.0
