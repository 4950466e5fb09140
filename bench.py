#!/usr/bin/env python3
"""Throughput of the speculative-decoding hot path on one MI355X.

A step is one speculative round over the whole batch: hh_draft(k) + hh_verify + hh_commit
through the C ABI, on a seeded random-init model with the prompts already prefilled and
everything resident in HBM.  The default workload is the largest configuration that fits one
GPU: the Falcon-H1-3B-shaped model, 64 sequences with 32768-token prompts, k = 8, acceptance
from the seeded fixed pattern with per-token probability 0.68 (`--workload c1|c2|c2f|c3` select
the others).  Prints ONE JSON line: committed tokens/s (value), draft tokens/s, verify passes/s,
per-segment and per-kernel HBM roofline fractions, and the CPU oracle timed on the host cores on
a bounded sample.

    python bench.py --gpus 1 --steps 20 --warmup 5 [--workload c4] [--cpu-seconds 20]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak


def measured_traffic(workload):
    """HBM bytes per launch of this workload's kernels, from rocprofv3 --pmc runs of
    `bench.py --counters` (FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter reads for
    a device-to-device copy of known size in the same run).  The summary with the commands is
    profiles/<workload>_hbm_traffic.md; its last json block holds {"traffic_bytes_per_launch": {...}}.
    Returns ({kernel: bytes}, file name) or ({}, None) when no summary is committed."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.md")
    if not os.path.exists(path):
        return {}, None
    blocks = re.findall(r"```json\s*(\{.*?\})\s*```", open(path).read(), re.S)
    if not blocks:
        return {}, None
    return json.loads(blocks[-1]).get("traffic_bytes_per_launch", {}), os.path.relpath(path, ROOT)


KIND_NAMES = {0: "in_proj", 1: "ssm_scan", 2: "rope_append", 3: "attention", 4: "out_proj", 5: "o_proj",
              6: "mlp_gate_up", 7: "mlp_down", 8: "lm_head"}
PHASE_NAMES = {0: "prefill", 1: "draft", 2: "verify", 3: "commit"}


def algorithmic_bytes(cfg, B, k, kv_len):
    """HBM bytes the method must move: weights once per pass, recurrent state, KV cache.
    Activations, logits and page tables are excluded (well under 1 %)."""
    esz = 2 if cfg.w_dtype == "bf16" else 4
    D, F, V, L = cfg.d_model, cfg.d_ff, cfg.vocab, cfg.n_layers
    state = cfg.m_heads * cfg.m_head_dim * cfg.d_state * 4
    conv = (cfg.conv_dim + cfg.m_heads) * 4                       # one ring row
    kv_tok = 2 * cfg.n_kv_heads * cfg.head_dim * esz               # per layer
    T = k + 1
    per_kind = {
        (1, 0): cfg.d_in_proj * D * esz,
        (1, 1): B * (2 * state + 4 * conv),
        (1, 4): D * cfg.d_inner * esz,
        (1, 6): 2 * F * D * esz,
        (1, 7): D * F * esz,
        (1, 8): V * D * esz,
        (2, 0): (cfg.d_in_proj + cfg.d_q + 2 * cfg.d_kv) * D * esz,
        (2, 1): B * (state + (3 + 2 * T) * conv),
        (2, 3): B * (kv_len + 2 * T) * kv_tok,
        (2, 4): D * cfg.d_inner * esz,
        (2, 5): D * cfg.d_q * esz,
        (2, 6): 2 * F * D * esz,
        (2, 7): D * F * esz,
        (2, 8): V * D * esz,
        (3, 1): L * B * (2 * state + (3 + T) * conv),
    }
    draft_step = sum(per_kind[(1, i)] for i in (0, 1, 4, 6, 7)) * L + per_kind[(1, 8)]
    verify = sum(per_kind[(2, i)] for i in (0, 1, 3, 4, 5, 6, 7)) * L + per_kind[(2, 8)]
    commit = per_kind[(3, 1)]
    return per_kind, draft_step, verify, commit


def cpu_baseline(wl, weights, prompts, seconds, sample_prompt):
    """The oracle, as it stands, on the host cores: prefill of `sample_prompt` tokens of sequence 0
    (multi-position pass, not counted), then speculative rounds for about `seconds`; returns committed
    tokens/s over the rounds.  Workloads with a forced acceptance pattern use the same pattern."""
    from oracle.hybrid_lm import HybridLM
    from oracle.protocol import SpecDecoder
    from paper_2605_01106_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    lm = HybridLM(wl.cfg, weights.values)
    dec = SpecDecoder(lm, sample_prompt + wl.gen_len + 2 * wl.k + 4, engine="pass", chunk=64)
    t0 = time.perf_counter()
    dec.prefill([prompts[0][:sample_prompt]], wl.gen_len)
    t_prefill = time.perf_counter() - t0
    forced = None if wl.forced_p is None else W.make_forced_pattern(4096, 1, wl.k, wl.forced_p, wl.seed)
    rounds, t_draft, t_verify = 0, 0.0, 0.0
    before = sum(len(o) for o in dec.out)
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds and not dec.all_finished():
        a = time.perf_counter()
        dec.draft(wl.k)
        b = time.perf_counter()
        dec.verify()
        c = time.perf_counter()
        dec.commit(None if forced is None else forced[rounds])
        t_draft += b - a
        t_verify += c - b
        rounds += 1
    dt = time.perf_counter() - t0
    toks = sum(len(o) for o in dec.out) - before
    mode = "greedy acceptance" if forced is None else f"forced acceptance p={wl.forced_p}"
    return {"value": toks / dt, "unit": "committed tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"sequence 0 of {wl.batch} alone (per-sequence rate, not scaled to the batch): prefill of the first "
                      f"{sample_prompt} of its {wl.prompt_len} prompt tokens ({t_prefill:.1f} s, not counted), then "
                      f"{rounds} rounds of k={wl.k}, {mode} ({dt:.1f} s)",
            "draft_tokens_per_s": rounds * wl.k / max(t_draft, 1e-9),
            "verify_passes_per_s": rounds / max(t_verify, 1e-9)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--forced-p", type=float, default=None,
                    help="per-token accept probability of the forced-pattern leg (default: the workload's, else 0.68)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="0 disables the oracle baseline")
    ap.add_argument("--cpu-prompt", type=int, default=256,
                    help="prompt tokens of sequence 0 the oracle baseline prefills (at most the workload's prompt)")
    ap.add_argument("--graphs", type=int, default=1)
    ap.add_argument("--keep-logits", type=int, default=0,
                    help="1: the library materialises the logits rows (parity runs); 0: argmax only at temperature 0")
    ap.add_argument("--temperature", type=float, default=0.6,
                    help="temperature of the stochastic-acceptance leg (the paper's second setting); 0 skips the leg")
    ap.add_argument("--counters", action="store_true",
                    help="short eager run for rocprofv3 --pmc: prefill, a few rounds, four 256 MiB copies for calibration")
    ap.add_argument("--prefill-chunk", type=int, default=0,
                    help="prompt positions per sequence per prefill pass (0: the library's default)")
    ap.add_argument("--prompt-len", type=int, default=None,
                    help="override the workload's prompt length (a shorter stand-in; named in config.workload)")
    ap.add_argument("--kernel-flags", type=int, default=0, help="hh_cfg.kernel_flags (HH_KF_* bits: kernel selection)")
    ap.add_argument("--adaptive-rounds", type=int, default=0,
                    help="extra leg of this many rounds in which k is re-chosen every 4 rounds from the library's acceptance "
                         "statistics and the measured cost ratio (Eq. 1); forced acceptance pattern cut off at k")
    ap.add_argument("--prefill-profile", action="store_true",
                    help="after the timed prefill, run it once more with per-launch events (serial, no branch overlap) and "
                         "report the time per kind of kernel under prefill_kernels")
    ap.add_argument("--attn-target-blocks", type=int, default=0, help="hh_cfg.attn_target_blocks (0: the library's 512)")
    ap.add_argument("--attn-max-splits", type=int, default=0, help="hh_cfg.attn_max_splits (0: the library's 16)")
    ap.add_argument("--overlap-mode", type=int, default=0, help="hh_cfg.overlap_mode (0 automatic, 1 never, 2 prefill only, 3 always)")
    ap.add_argument("--k", type=int, default=None, help="draft length (default: the workload's)")
    ap.add_argument("--draft-state", choices=("shared", "strict"), default="shared",
                    help="strict: the draft model keeps its own recurrent state over the whole prefix")
    ap.add_argument("--draft-mask", default=None,
                    help="draft model by layers, comma-separated ssm|full|skip, each optionally *count (e.g. ssm*30,full*2)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards by sequence with no exchange step); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_01106_amd import binding as B
    from paper_2605_01106_amd import workloads as W

    wl = W.WORKLOADS[args.workload]
    if args.prompt_len is not None:
        import dataclasses
        wl = dataclasses.replace(wl, prompt_len=args.prompt_len)
    cfg, k, Bn = wl.cfg, (wl.k if args.k is None else args.k), wl.batch
    if k < 1 or k > 64:
        print("bench.py: the draft length must be in 1..64", file=sys.stderr)
        sys.exit(2)
    draft_mask = None
    if args.draft_mask:
        draft_mask = []
        for item in args.draft_mask.split(","):
            mode, _, count = item.partition("*")
            draft_mask += [mode.strip()] * (int(count) if count else 1)
        if len(draft_mask) != cfg.n_layers or any(m not in B.DRAFT_MODES for m in draft_mask):
            print(f"bench.py: --draft-mask needs {cfg.n_layers} entries of ssm|full|skip", file=sys.stderr)
            sys.exit(2)
    K, Wm = args.steps, args.warmup
    prof_rounds, greedy_rounds = 3, min(K, 32)
    forced_p = args.forced_p if args.forced_p is not None else (wl.forced_p or 0.68)
    primary_forced = wl.forced_p is not None          # the workload's own acceptance mode is the headline leg
    total_rounds = Wm + K + K + K + prof_rounds + greedy_rounds + 6 + args.adaptive_rounds
    G = max(wl.gen_len, total_rounds * (k + 1) + 2)
    max_seq = wl.prompt_len + G + 2 * k + 4

    def say(msg):   # progress on stderr: the JSON line on stdout stays the only stdout output
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    say(f"workload {args.workload}: generating weights")
    t0 = time.perf_counter()
    weights = W.make_weights(cfg, args.seed)
    prompts = W.make_prompts(cfg.vocab, Bn, wl.prompt_len, args.seed)
    t_gen = time.perf_counter() - t0
    stream = torch.cuda.Stream()          # HIP graphs cannot be captured on the default stream
    torch.cuda.set_stream(stream)
    say(f"weights in {t_gen:.1f} s; creating the context")
    n_pass_hint = 16 if wl.prompt_len * Bn > (1 << 18) else 0
    ctx = B.Context(weights, Bn, max_seq, k, G, use_graphs=0 if args.counters else args.graphs,
                    prefill_chunk=args.prefill_chunk, keep_logits=args.keep_logits, prefill_progress=n_pass_hint,
                    draft_state_mode=1 if args.draft_state == "strict" else 0, kernel_flags=args.kernel_flags, overlap_mode=args.overlap_mode,
                    attn_target_blocks=args.attn_target_blocks, attn_max_splits=args.attn_max_splits)
    ctx.hh_set_draft_mask(draft_mask)
    torch.cuda.synchronize()
    say("prefill")
    t0 = time.perf_counter()
    ctx.hh_prefill(prompts, [wl.prompt_len] * Bn, G)
    torch.cuda.synchronize()
    t_prefill = time.perf_counter() - t0

    prefill_kernels = None
    if args.prefill_profile:
        ctx.hh_profile(True)
        ctx.hh_prefill(prompts, [wl.prompt_len] * Bn, G)
        prof = ctx.hh_profile_read()
        ctx.hh_profile(False)
        tot = sum(ms for (ph, _), (_, ms) in prof.items() if ph == 0)
        prefill_kernels = {KIND_NAMES[kd]: {"launches": c, "total_ms": round(ms, 2), "avg_us": round(ms / c * 1e3, 1),
                                            "share": round(ms / tot, 3)}
                           for (ph, kd), (c, ms) in sorted(prof.items()) if ph == 0}

    def run_rounds(n, kk, forced=None, timed=False):
        evs = []
        for r in range(n):
            if timed:
                e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
                e[0].record()
            ctx.hh_draft(kk)
            if timed:
                e[1].record()
            ctx.hh_verify()
            if timed:
                e[2].record()
            ctx.hh_commit(None if forced is None else forced[r])
            if timed:
                e[3].record()
                evs.append(e)
        return evs

    def timed_leg(n, kk, forced=None):
        torch.cuda.synchronize()
        _, c0, _ = ctx.hh_get_lengths()
        t0 = time.perf_counter()
        evs = run_rounds(n, kk, forced, timed=True)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        _, c1, _ = ctx.hh_get_lengths()
        seg = [sum(e[i].elapsed_time(e[i + 1]) for e in evs) * 1e-3 for i in range(3)]
        return dt, sum(c1) - sum(c0), seg

    pattern = W.make_forced_pattern(Wm + K, Bn, k, forced_p, args.seed)
    forced_dev = [torch.from_numpy(pattern[r]).to(ctx.device) for r in range(Wm + K)]
    if args.counters:
        run_rounds(max(K, 1), k, forced_dev[:max(K, 1)] if primary_forced and K <= Wm + K else None)
        torch.cuda.synchronize()
        src = torch.empty(256 << 20, dtype=torch.uint8, device=ctx.device).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"counters_run": True, "rounds": max(K, 1), "copy_bytes": 256 << 20, "copies": 4}))
        return
    say(f"prefill in {t_prefill:.2f} s; {Wm} warm-up and {K} timed rounds")
    # headline leg: the workload's own acceptance mode (the seeded fixed pattern where the workload names one)
    run_rounds(Wm, k, forced_dev[:Wm] if primary_forced else None)
    dt, toks, (t_draft, t_verify, t_commit) = timed_leg(K, k, forced_dev[Wm:] if primary_forced else None)
    say(f"timed rounds: {toks / dt:.1f} tokens/s; other acceptance mode and plain-greedy legs")
    kv_len, _, _ = ctx.hh_get_lengths()
    kv_mid = int(np.mean(kv_len)) - K * (k + 1) // 4
    # the other acceptance mode: greedy acceptance of the random-init model's own drafts, or the pattern
    dt_o, toks_o, _ = timed_leg(K, k, None if primary_forced else forced_dev[Wm:])
    # plain greedy decoding of the full model (k = 0) for the speedup the paper's Table 7 reports
    dt_g, toks_g, _ = timed_leg(greedy_rounds, 0)

    # per-kernel timing leg, on the launch stream: every kind of kernel is launched alone, in its
    # place in the pass (consecutive launches stream different layers' weights), between one HIP
    # event pair, so the average is launch duration + launch gap without per-launch event overhead
    say("per-kernel timing")
    per_kind, draft_bytes, verify_bytes, commit_bytes = algorithmic_bytes(cfg, Bn, k, kv_mid)
    kernels = {}
    per_round = {1: k, 2: 1}
    dqkv = (cfg.n_q_heads + 2 * cfg.n_kv_heads) * cfg.head_dim
    gemm_shapes = {0: (cfg.d_in_proj + dqkv, cfg.d_model), 4: (cfg.d_model, cfg.d_inner), 5: (cfg.d_model, cfg.n_q_heads * cfg.head_dim),
                   6: (2 * cfg.d_ff, cfg.d_model), 7: (cfg.d_model, cfg.d_ff), 8: (cfg.vocab, cfg.d_model)}
    # the attention branch of verification (attention, o_proj) runs on a side stream beside scan + out_proj
    # only when asked (overlap_mode 3)
    side_branch = args.overlap_mode == 3
    for ph in (1, 2):
        for kind in sorted(KIND_NAMES):
            if kind == 2 or (ph == 1 and kind in (3, 5)):   # RoPE/append is fused into attention
                continue
            # best of three repeats of 4 passes each: the boxes show run-to-run clock noise
            avg_us, n = min(ctx.hh_time_kind(ph, kind, k, 4) for _ in range(3))
            by = per_kind.get((ph, kind))
            launches = (1 if kind == 8 else cfg.n_layers) * per_round[ph]
            entry = {
                "launches_per_round": launches, "avg_us": round(avg_us, 3), "us_per_round": round(avg_us * launches, 1),
                "bytes": by, "gbs": None if by is None else round(by / (avg_us * 1e-6) / 1e9, 1),
                "stream": "side" if side_branch and ph == 2 and kind in (3, 5) else "launch"}
            # the dense products also against the matrix-core peak: bf16 weights x float32 activations split
            # exactly into three bf16 terms, i.e. three bf16 MFMA products per multiply-add of the method
            shape = gemm_shapes.get(kind)
            if shape is not None and cfg.w_dtype == "bf16":
                rows = Bn * (k + 1 if ph == 2 else 1)
                n_out, k_in = shape if not (kind == 0 and ph == 1) else (cfg.d_in_proj, cfg.d_model)
                tf = 2.0 * rows * n_out * k_in * 3 / (avg_us * 1e-6) / 1e12
                entry["mfma_tflops_3_terms"] = round(tf, 1)
                entry["mfma_frac"] = round(tf / MFMA_BF16_PEAK_TFLOPS, 4)
            kernels[f"{PHASE_NAMES[ph]}.{KIND_NAMES[kind]}"] = entry
    # commit rebuild: timed with the per-launch events (one launch per round)
    ctx.hh_profile(True)
    run_rounds(prof_rounds, k)
    prof = ctx.hh_profile_read()
    ctx.hh_profile(False)
    if (3, 1) in prof:
        cnt, ms = prof[(3, 1)]
        by = per_kind[(3, 1)]
        kernels["commit.ssm_scan"] = {"launches_per_round": 1, "avg_us": round(ms / cnt * 1e3, 3),
                                      "us_per_round": round(ms / cnt * 1e3, 1), "bytes": by,
                                      "gbs": round(by / (ms / cnt * 1e-3) / 1e9, 1), "stream": "launch"}
    # dominant kernel: the kind of kernel (draft and verification launches together) with the largest
    # share of a round on the launch stream (the in-order critical path; the side-stream kernels
    # overlap it), reported for the phase in which it takes longer
    share = {}
    for n, v in kernels.items():
        if v["bytes"] and v["stream"] == "launch":
            share[n.split(".")[1]] = share.get(n.split(".")[1], 0.0) + v["us_per_round"]
    dom_kind = max(share, key=share.get)
    dom_name, dom = max(((n, v) for n, v in kernels.items()
                         if v["bytes"] and v["stream"] == "launch" and n.split(".")[1] == dom_kind),
                        key=lambda nv: nv[1]["us_per_round"])
    traffic, traffic_file = measured_traffic(args.workload) if args.prompt_len is None else ({}, None)
    roofline = {"bound": "hbm", "kernel": dom_name, "achieved": dom["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(dom["gbs"] / HBM_PEAK_GBS, 4),
                "traffic": traffic.get(dom_name), "traffic_source": traffic_file if dom_name in traffic else None,
                "bytes_per_launch": dom["bytes"], "avg_us": dom["avg_us"],
                "share_of_round": round(share[dom_kind] / sum(share.values()), 3)}

    # stochastic-acceptance leg (Eq. 6) at the paper's temperature: same kernels plus the draws (last, so that
    # the per-kernel timings above see the same cache lengths whether or not this leg runs)
    stochastic = None
    if args.temperature > 0:
        ctx.hh_set_sampling(args.temperature, args.seed)
        run_rounds(2, k)       # first use of the temperature's launch sequences (eager, then captured)
        dt_s, toks_s, _ = timed_leg(K, k)
        ctx.hh_set_sampling(0.0, 0)
        stochastic = {"temperature": args.temperature, "committed_tokens_per_s": round(toks_s / dt_s, 2),
                      "mean_accepted_per_round": round(toks_s / (K * Bn) - 1, 3)}

    # adaptive draft length (Section 7): k re-chosen every 4 rounds as the maximiser of Eq. 1 for the acceptance rate
    # the library has counted in this leg and the cost ratio measured above
    adaptive = None
    if args.adaptive_rounds > 0:
        ratio = (t_draft / (K * k)) / (t_verify / K)
        pat = W.make_forced_pattern(args.adaptive_rounds, Bn, k, forced_p, args.seed + 1)
        a0, t0_ = ctx.hh_get_acceptance()
        _, c0, _ = ctx.hh_get_lengths()
        torch.cuda.synchronize()
        ts = time.perf_counter()
        kk, ks_used = k, []
        for r in range(args.adaptive_rounds):
            if r and r % 4 == 0:
                a1, t1_ = ctx.hh_get_acceptance()
                if t1_ > t0_:
                    kk = B.hh_optimal_draft_length((a1 - a0) / (t1_ - t0_), ratio, list(range(1, k + 1)))
            ks_used.append(kk)
            ctx.hh_draft(kk)
            ctx.hh_verify()
            ctx.hh_commit(torch.from_numpy(np.minimum(pat[r], kk).astype(np.int32)).to(ctx.device))
        torch.cuda.synchronize()
        dt_a = time.perf_counter() - ts
        _, c1, _ = ctx.hh_get_lengths()
        a1, t1_ = ctx.hh_get_acceptance()
        adaptive = {"rounds": args.adaptive_rounds, "cost_ratio": round(ratio, 4), "alpha_measured": round((a1 - a0) / max(t1_ - t0_, 1), 4),
                    "k_last": kk, "k_mean": round(float(np.mean(ks_used)), 2),
                    "committed_tokens_per_s": round((sum(c1) - sum(c0)) / dt_a, 2),
                    "note": "includes the eager first use and graph capture of every new k"}

    mode = f"forced acceptance p={forced_p}" if primary_forced else "greedy acceptance"
    other = {"mode": "greedy acceptance" if primary_forced else f"forced acceptance p={forced_p}",
             "committed_tokens_per_s": round(toks_o / dt_o, 2),
             "mean_accepted_per_round": round(toks_o / (K * Bn) - 1, 3)}
    prompt_note = "" if args.prompt_len is None else " (shortened stand-in)"
    cost_ratio = (t_draft / (K * max(k, 1))) / (t_verify / K) if k > 0 else 0.0
    out = {
        "metric": "committed tokens/s (speculative rounds); draft tok/s and verify passes/s alongside",
        "value": round(toks / dt, 2), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(dt / K * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {cfg.name}, bf16 weights and KV cache, batch {Bn}, prompt {wl.prompt_len}"
                               f"{prompt_note}, k={k}, {mode}, seed {args.seed}"
                               if cfg.w_dtype == "bf16" else
                               f"{args.workload}: {cfg.name}, f32 weights, batch {Bn}, prompt {wl.prompt_len}, k={k}, {mode}",
                   "rounds_timed": K, "graphs": args.graphs, "keep_logits": args.keep_logits,
                   "draft_state": args.draft_state, "draft_mask": args.draft_mask, "overlap_mode": args.overlap_mode},
        "draft_tokens_per_s": round(Bn * k * K / t_draft, 1),
        "verify_passes_per_s": round(K / t_verify, 1),
        "commit_us": round(t_commit / K * 1e6, 2),
        "mean_accepted_per_round": round(toks / (K * Bn) - 1, 3),
        "segments": {
            "draft_step": {"bytes": draft_bytes, "us": round(t_draft / (K * k) * 1e6, 2),
                           "hbm_frac": round(draft_bytes / (t_draft / (K * k)) / 1e9 / HBM_PEAK_GBS, 4)},
            "verify_pass": {"bytes": verify_bytes, "us": round(t_verify / K * 1e6, 2),
                            "hbm_frac": round(verify_bytes / (t_verify / K) / 1e9 / HBM_PEAK_GBS, 4)},
            "commit": {"bytes": commit_bytes, "us": round(t_commit / K * 1e6, 2),
                       "hbm_frac": round(commit_bytes / (t_commit / K) / 1e9 / HBM_PEAK_GBS, 4)}},
        # Eq. 1 with the measured costs of this run: c = one draft step / one verification pass
        "draft_length_model": {
            "alpha": forced_p, "cost_ratio": round(cost_ratio, 4),
            "k_star": B.hh_optimal_draft_length(forced_p, cost_ratio, list(range(1, max(k, 8) + 1))),
            "k_star_of_2_4_8": B.hh_optimal_draft_length(forced_p, cost_ratio, [2, 4, 8])},
        "other_acceptance": other,
        "stochastic": stochastic,
        "adaptive_k": adaptive,
        "plain_greedy_tokens_per_s": round(toks_g / dt_g, 2),
        "speedup_vs_plain_greedy": round((toks / dt) / (toks_g / dt_g), 4),
        "prefill_s": round(t_prefill, 3), "prefill_tokens_per_s": round(Bn * wl.prompt_len / t_prefill, 1),
        "weight_gen_s": round(t_gen, 1),
        "prefill_kernels": prefill_kernels,
        "roofline": roofline,
        "kernels": kernels,
    }
    if args.cpu_seconds > 0:
        say("oracle baseline on the host cores")
        out["cpu_baseline"] = cpu_baseline(wl, weights, prompts, args.cpu_seconds, min(args.cpu_prompt, wl.prompt_len))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
