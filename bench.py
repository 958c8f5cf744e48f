#!/usr/bin/env python3
"""Benchmark of the HiViS draft-verify path on one MI355X.

One "step" = the whole hot path on one batch of synthetic input: target prefill over
[visual ; text], drafter prefill over the text rows, then draft(K) -> verify -> accept cycles
until the workload's number of tokens has been generated.  Default workload: the
LLaVA-1.5-7B-shaped bf16 model (32 layers, d 4096, 576 visual + 64 text rows, K = 5 chain,
128 generated tokens, batch 1) with seeded random weights.

Prints ONE JSON line: whole-job tokens/s, per-phase latencies from HIP events recorded on the
library's stream inside the timed region, the HBM roofline of the verify pass (algorithmic
bytes / event-timed duration vs 8 TB/s), and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth  # noqa: E402

HBM_PEAK_GBS = 8000.0
GEMM_GATEUP = 4      # kind id of the fused gate|up GEMM (+RMSNorm prologue, SiLU*up epilogue): the kernel with the most bytes
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/): filled in from the
# committed counter runs; None where no counter run exists for the workload.
TRAFFIC_BYTES_PER_LAUNCH = {"C2": 181.7e6}     # profiles/gateup_gemm_C2_hbm_counters.txt: (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000) per launch
PAPER_TAU = {"C2": 5.37, "C3": 5.06, "C4": 4.39, "C5": 5.15}    # Table 2, T=0 averages (tree drafting, A800): context only


def run_step(hv, cfg, vis, ids, K, temperature=0.0, rng=None, tree=None):
    """prefill + cycles until cfg.gen_tokens tokens (or cfg.gen_cycles cycles).  Returns (tokens, cycles, accepted).
    temperature > 0: the sampling calls, with uniforms drawn on the device (hivis_rng_seed; not the headline configuration).
    tree = (top_k, depth, n_nodes): draft-tree cycles instead of chain cycles (not the headline configuration)."""
    first = hv.prefill(vis, ids)
    produced = np.ones(hv.B, np.int64)
    cycles = 0
    accepted = 0
    target = cfg.gen_tokens
    while True:
        if tree:
            hv.tree_draft(*tree)
            hv.tree_verify()
            n1, _ = hv.tree_accept_sample(temperature) if temperature > 0.0 else hv.tree_accept()
            n = np.array([n1], np.int64)
        elif temperature > 0.0:
            hv.draft_sample(K, temperature)
            hv.verify()
            n, _ = hv.accept_sample(temperature)
        else:
            hv.draft(K)
            hv.verify()
            n, _ = hv.accept()
        produced += n + 1
        accepted += int(n.sum())
        cycles += 1
        if cfg.gen_cycles and cycles >= cfg.gen_cycles:
            break
        if target and int(produced.min()) >= target:
            break
    tokens = int(np.minimum(produced, target).sum()) if target else int(produced.sum())
    return tokens, cycles, accepted, first


def cpu_baseline(cfg, K, weights, vis, ids, gpu_tokens_per_cycle):
    """The CPU oracle, as it stands, timed on the SAME model at its full depth (the weights handed to the library; bf16
    models are read through synth.LazyWeights, which widens one tensor at a time) on a bounded sample of the workload:
    sequence 0's prompt, one prefill and one draft-verify-accept cycle.  `value` is that cycle's tokens per second (the
    steady-state rate of the job: 127 of its 128 tokens come from cycles); the prefill time is reported beside it, and
    the whole-job rate that the two timed pieces imply."""
    from oracle import HivisOracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    if cfg.dtype == "bf16":
        from synth.lazy import LazyWeights
        weights = LazyWeights(weights)
    o = HivisOracle(cfg, weights)
    t0 = time.time()
    o.prefill(vis[0], ids[0])
    t_prefill = time.time() - t0
    t0 = time.time()
    drafts, _ = o.draft(K)
    t_draft = time.time() - t0
    t0 = time.time()
    g, logits, t = o.verify(drafts)
    t_verify = time.time() - t0
    t0 = time.time()
    n, emitted = o.accept(drafts, g, t)
    t_accept = time.time() - t0
    cycle = t_draft + t_verify + t_accept
    gen = cfg.gen_tokens or cfg.gen_cycles * (K + 1)
    cycles_needed = max(1.0, (gen - 1) / max(gpu_tokens_per_cycle, 1e-9))
    return {"value": (n + 1) / cycle, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": (f"full depth (N={cfg.n_layers}), sequence 0 of the batch: one prefill over {cfg.n_vis}+{cfg.n_text} rows ({t_prefill:.1f}s, timed, "
                       f"not in value) and ONE timed draft-verify-accept cycle: {K} draft steps {t_draft:.2f}s + verify {t_verify:.2f}s + accept/roll "
                       f"{t_accept:.2f}s, {n + 1} token(s) emitted; float64 numpy, weights widened from bf16 bits on access"),
            "prefill_s": t_prefill, "draft_step_us": t_draft / K * 1e6, "verify_us": t_verify * 1e6, "cycle_s": cycle,
            "whole_job_tokens_per_s_implied": gen / (t_prefill + cycles_needed * cycle)}


def stream_ceiling(stream=None):
    """hivis_calib_stream over buffer sizes like the verify pass's weight matrices (O projection 33.5 MB, down 90 MB,
    gate|up 180 MB, LM head 262 MB at C2) and one large buffer, each in rotation over >= 1.4 GB so that nothing comes from a
    cache; one launch per buffer, back to back, each timed by start / stop events attached to its dispatch (the kernel's own
    duration, as `roofline` times the GEMM).  256 workgroups = one per compute unit, as the GEMM phases run; 1024 = four
    per compute unit."""
    from paper_2509_23928_amd import calib_stream
    out = {"unit": "GB/s", "peak": HBM_PEAK_GBS, "kernel": "calib_stream_kernel: read-only, 1 KiB per wavefront and instruction, 8 independent 16-byte loads per lane",
           "cases": []}
    best = 0.0
    for mb, nbuf in ((33.5, 48), (90.2, 16), (180.4, 8), (262.1, 6), (1024.0, 2)):
        for wgs in (256, 1024):
            gbs, us = calib_stream(int(mb * 1e6), nbuf, 3, wgs, stream)
            out["cases"].append({"buffer_mb": mb, "buffers": nbuf, "workgroups": wgs, "gbs": round(gbs, 1), "us_per_launch": round(us, 2),
                                 "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)})
            best = max(best, gbs)
    out["best_gbs"] = round(best, 1)
    out["best_frac_of_peak"] = round(best / HBM_PEAK_GBS, 4)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C2")
    ap.add_argument("--layers", type=int, default=0, help="override the number of target layers (debug only; invalid as a result)")
    ap.add_argument("--batch", type=int, default=0, help="override the batch size (experiments only; not the named workload)")
    ap.add_argument("--K", type=int, default=0, help="override the chain draft length (experiments only; not the named workload)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--temperature", type=float, default=0.0, help="> 0: time the temperature-sampling calls instead of the greedy ones (extra measurement, not the headline metric)")
    ap.add_argument("--tree", default="", help="top_k,depth,n_nodes: time draft-tree cycles instead of chain cycles (extra measurement, not the headline metric; batch 1)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", action="store_true", help="also run a plain 1 GiB device copy first (reference for rocprofv3 byte counters)")
    ap.add_argument("--calib-stream", action="store_true", help="only run the read-only streaming calibration (hivis_calib_stream) and print its JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_23928_amd import Hivis
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.calib_stream:
        print(json.dumps({"stream_ceiling": stream_ceiling()}))
        return

    cfg = synth.get_config(args.config)
    if args.layers:
        cfg = cfg.scaled(n_layers=args.layers)
    if args.batch:
        cfg = cfg.scaled(batch=args.batch)
    if args.K:
        cfg = cfg.scaled(K=args.K)
    K = cfg.K
    t0 = time.time()
    nthreads = min(16, os.cpu_count() or 1)
    w = synth.make_weights(cfg, seed=args.seed, bits=(cfg.dtype == "bf16"), threads=nthreads)
    vis, ids = synth.make_prompt(cfg, seed=args.seed)
    t_gen = time.time() - t0
    t0 = time.time()
    stream = torch.cuda.Stream()
    tree = tuple(int(x) for x in args.tree.split(",")) if args.tree else None
    # batch 1: room for the draft tree's rows too (the tree cycle is timed after the headline region, see "tree_cycle" below)
    side_tree = tree or ((10, 6, 60) if cfg.batch == 1 else None)
    if side_tree:
        gen = cfg.gen_tokens or cfg.gen_cycles * (max(side_tree[1], K) + 1)
        hv = Hivis(cfg, w, stream=stream.cuda_stream, max_text=cfg.n_text + gen + max((side_tree[1] - 1) * side_tree[0], side_tree[2]) + side_tree[1] + 2 * (K + 2))
    else:
        hv = Hivis(cfg, w, stream=stream.cuda_stream)
    if args.no_cpu_baseline:
        del w                                   # otherwise kept (13 GB of bf16 bits at C2) for the oracle's timed sample below
    t_load = time.time() - t0
    # inputs resident in HBM before the timed region
    if cfg.dtype == "bf16":
        vis_dev = torch.from_numpy(synth.to_bf16_bits(vis).reshape(vis.shape).view(np.int16)).cuda()
    else:
        vis_dev = torch.from_numpy(vis).cuda()
    ids_dev = torch.from_numpy(ids).cuda()
    torch.cuda.synchronize()
    print(f"[bench] {cfg.name}: weights generated in {t_gen:.1f}s, uploaded+packed in {t_load:.1f}s", file=sys.stderr, flush=True)

    if args.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB read + 1 GiB written by one elementwise kernel
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    rng = None
    if args.temperature > 0.0:
        hv.rng_seed(args.seed + 12345)
    for _ in range(args.warmup):
        run_step(hv, cfg, vis_dev, ids_dev, K, args.temperature, rng, tree)
    hv.timing(True)
    hv.kernel_timing(GEMM_GATEUP)
    for ph in range(4):
        hv.phase_ms(ph)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tokens = cycles = accepted = 0
    for _ in range(args.steps):
        tk, cy, ac, _ = run_step(hv, cfg, vis_dev, ids_dev, K, args.temperature, rng, tree)
        tokens += tk; cycles += cy; accepted += ac
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    phases = [hv.phase_ms(ph) for ph in range(4)]
    k_ms, k_launches, k_bytes = hv.kernel_ms()
    hv.kernel_timing(-1)
    verify_bytes_end, draft_bytes_end = hv.algorithmic_bytes()
    # extra measurement outside the headline region: the same workload decoded with draft-tree cycles (the tree setting of the
    # paper's experiments, section 4: top-10 expansion, depth 6, 60 candidates)
    tree_cycle = None
    if side_tree and not tree and args.temperature <= 0.0:
        run_step(hv, cfg, vis_dev, ids_dev, K, 0.0, rng, side_tree)
        for ph in range(4):
            hv.phase_ms(ph)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        tk_t, cy_t, ac_t, _ = run_step(hv, cfg, vis_dev, ids_dev, K, 0.0, rng, side_tree)
        torch.cuda.synchronize()
        dt_t = time.perf_counter() - t1
        ph_t = [hv.phase_ms(ph) for ph in range(4)]
        per = [ph_t[i][0] / max(ph_t[i][1], 1) * 1e3 for i in (1, 2, 3)]
        tree_cycle = {"setting": f"top_k={side_tree[0]} depth={side_tree[1]} candidates={side_tree[2]} ({side_tree[2] + 1} verify rows)",
                      "tree_draft_us": per[0], "verify_us": per[1], "accept_refeed_us": per[2], "cycle_us": sum(per),
                      "tokens_per_s": tk_t / dt_t, "cycles": cy_t, "mean_accepted_drafts": ac_t / max(cy_t, 1),
                      "note": "one step, timed after the headline region; random-init drafts are almost never accepted"}
    hv.timing(False)

    prefill_ms = phases[0][0] / max(phases[0][1], 1)
    Kd = 1 if tree else K                      # tree: phase 1 is the whole tree draft (depth LM-head passes, depth-1 drafter passes)
    draft_us = phases[1][0] / max(phases[1][1], 1) / Kd * 1e3
    verify_us = phases[2][0] / max(phases[2][1], 1) * 1e3
    accept_us = phases[3][0] / max(phases[3][1], 1) * 1e3
    # algorithmic bytes of an average verify / draft step: weights once + KV at the mean length of the run
    esize = 2 if cfg.dtype == "bf16" else 4
    kd = cfg.kv_dim
    gen_per_seq = tokens / args.steps / cfg.batch
    mean_text = cfg.n_text + gen_per_seq / 2.0
    w_layer = (2 * cfg.d * cfg.q_dim + 2 * cfg.d * kd + 3 * cfg.d * cfg.ffn) * esize
    verify_bytes = cfg.n_layers * w_layer + cfg.vocab * cfg.d * esize + cfg.batch * cfg.n_layers * 2 * (cfg.n_vis + mean_text) * kd * esize
    draft_bytes = w_layer + 2 * cfg.d * cfg.d * esize + cfg.vocab * cfg.d * esize + cfg.batch * 2 * mean_text * kd * esize
    verify_gbs = verify_bytes / (verify_us * 1e-6) / 1e9
    draft_gbs = draft_bytes / (draft_us * 1e-6) / 1e9

    out = {
        "metric": "tokens/s at fixed K (draft+verify cycles incl. prefill), with draft/verify step latency and HBM GB/s",
        "value": tokens / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.config}: {cfg.name} N={cfg.n_layers} d={cfg.d} Hq/Hkv={cfg.n_q_heads}/{cfg.n_kv_heads} F={cfg.ffn} V={cfg.vocab}, "
                               f"{cfg.n_vis} visual + {cfg.n_text} text rows, K={K} chain, {cfg.gen_tokens or cfg.gen_cycles * (K + 1)} generated tokens, batch {cfg.batch}, "
                               "random-init weights (seeded)" + (f", temperature {args.temperature} sampling" if args.temperature > 0 else "")
                               + (f"; DRAFT TREE top_k={tree[0]} depth={tree[1]} candidates={tree[2]} instead of the chain (draft_step_us = one whole tree draft; "
                                  f"verify = {tree[2] + 1} rows; the *_hbm_gbs / frac figures below price ONE weight pass and do not apply)" if tree else ""), "K": K, "batch": cfg.batch},
        "prefill_ms": prefill_ms, "draft_step_us": draft_us, "verify_us": verify_us, "accept_roll_us": accept_us,
        "cycle_us": Kd * draft_us + verify_us + accept_us,
        "draft_step_hbm_gbs": draft_gbs, "draft_step_frac_of_peak": draft_gbs / HBM_PEAK_GBS,
        "cycles": cycles, "mean_accepted_drafts": accepted / max(cycles * cfg.batch, 1),
        "verify_pass_hbm_gbs": verify_gbs, "verify_pass_frac_of_peak": verify_gbs / HBM_PEAK_GBS, "verify_pass_algorithmic_bytes": verify_bytes,
    }
    k_us = k_ms / max(k_launches, 1) * 1e3
    k_gbs = k_bytes / (k_us * 1e-6) / 1e9 if k_launches else 0.0
    out["roofline"] = {"bound": "hbm",
                       "kernel": "phase_kernel<bf16, GEMM, gate|up>: fused RMSNorm + [d x 2F] weight stream + SiLU*up of the verify pass "
                                 "(largest share of bytes and of time); HIP start/stop events attached to every 8th launch on the library's stream (hipExtLaunchKernel: the kernel's own begin/end timestamps, no marker packets in the queue)",
                       "achieved": k_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": k_gbs / HBM_PEAK_GBS,
                       "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(args.config), "algorithmic_bytes_per_launch": k_bytes,
                       "avg_launch_us": k_us, "launches_timed": k_launches}
    tau = PAPER_TAU.get(args.config)
    if tau:
        out["projected_tokens_per_s_at_paper_tau"] = cfg.batch * tau / ((Kd * draft_us + verify_us + accept_us) * 1e-6)
        out["projection_note"] = f"PROJECTION: (paper tau {tau} tokens/cycle, Table 2 T=0 avg, tree drafting on A800) / measured cycle time; random-init drafts are almost never accepted"
    if tree_cycle:
        out["tree_cycle"] = tree_cycle
    # what a plain read-only streaming kernel reaches on this machine, measured in this run (outside the timed region)
    out["stream_ceiling"] = stream_ceiling(stream.cuda_stream)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, K, w, vis, ids, (tokens / args.steps - cfg.batch) / max(cycles / args.steps, 1) / cfg.batch)
    hv.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
