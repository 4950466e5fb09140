"""Parity at the full sizes of the paper-shaped workloads, in the launch configuration the
benchmark times (HIP graphs on, default page and chunk sizes).  The oracle runs the sequences it
can afford (float64 numpy); rows of a batch are independent, so for the batched workload it
follows the first and the last sequence while the library runs all of them."""
import time

import numpy as np
import pytest

from paper_2605_01106_amd import workloads as W

pytestmark = pytest.mark.gpu

from parity_util import run_lockstep  # noqa: E402


def _run(name, seed, G, rounds, batch=None, lens=None, rows=None, layers=None, forced_p=None, min_gap=0.0,
         invariance_rows=None, draft_state="shared", draft_mask=None):
    import torch
    from paper_2605_01106_amd import binding as B
    wl = W.WORKLOADS[name]
    Bn = wl.batch if batch is None else batch
    lens = [wl.prompt_len] * Bn if lens is None else lens
    t0 = time.time()
    wts = W.make_weights(wl.cfg, seed)
    prompts = W.make_prompts(wl.cfg.vocab, Bn, lens, seed)
    forced = None if forced_p is None else W.make_forced_pattern(rounds + 2, Bn, wl.k, forced_p, seed)
    print(f"[{name}] inputs {time.time() - t0:.1f}s", flush=True)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = B.Context(wts, Bn, max(lens) + G + 2 * wl.k + 4, wl.k, G, use_graphs=1, kernel_flags=B.HH_KF_CANARIES,
                        draft_state_mode=1 if draft_state == "strict" else 0)
        w = run_lockstep(ctx, wts, prompts, lens, G, wl.k, forced=forced, engine="pass", chunk=64,
                         max_rounds=rounds, check_state_every=max(rounds // 2, 1), oracle_rows=rows, layers=layers,
                         min_gap=min_gap, draft_state=draft_state, draft_mask=draft_mask)
        # guard bytes behind every workspace region: no kernel wrote past its buffer at these sizes
        assert ctx.hh_check_canaries() == 0, B.hh_last_error(ctx.ctx)
        if invariance_rows is not None:
            w["invariance"] = _batch_invariance(B, torch, ctx, wts, prompts, lens, G, wl.k, forced, rounds, invariance_rows)
            assert ctx.hh_check_canaries() == 0, B.hh_last_error(ctx.ctx)
    stream.synchronize()
    print(f"[{name}] {time.time() - t0:.1f}s rounds={w['rounds']} mean_n={w['mean_n']:.2f} min_gap={w['min_gap']:.2e} "
          f"err: logits={w['logits']:.2e} ssm={w['ssm']:.2e} conv={w['conv']:.2e} kv={w['kv']:.2e}", flush=True)
    return w


def _batch_invariance(B, torch, big, wts, prompts, lens, G, k, forced, rounds, rows):
    """The sequences `rows` of the batch again, as a batch of their own on a second context (other
    kernels: fewer activation rows pick the weight-streaming and skinny products instead of the
    many-row ones): same committed tokens, verification logits of the last round within the logit
    tolerance of each other.  This is what lets the oracle follow a few rows of a large batch."""
    from parity_util import assert_close, tolerances
    atol, rtol = tolerances(wts.cfg.w_dtype)
    sub_lens = [lens[b] for b in rows]
    sub_prompts = np.stack([prompts[b] for b in rows])
    small = B.Context(wts, len(rows), max(lens) + G + 2 * k + 4, k, G, use_graphs=1)
    out = {}
    for name, ctx, pr, ln, sel in (("big", big, prompts, lens, rows), ("small", small, sub_prompts, sub_lens, list(range(len(rows))))):
        ctx.hh_prefill(pr, ln, G)
        for r in range(rounds):
            ctx.hh_draft(k)
            ctx.hh_verify()
            f = None
            if forced is not None:
                fr = forced[r] if name == "big" else forced[r][rows]
                f = torch.from_numpy(np.ascontiguousarray(fr, np.int32)).to(ctx.device)
            ctx.hh_commit(f)
        out[name] = ([ctx.hh_get_tokens(b) for b in sel], ctx.hh_get_logits(1)[sel], [ctx.hh_get_state(0)[0][b] for b in sel])
    assert out["big"][0] == out["small"][0], "committed tokens depend on the batch a sequence is in"
    e1 = assert_close("batch invariance: verification logits", out["small"][1], out["big"][1], 2 * atol, 2 * rtol)
    e2 = assert_close("batch invariance: SSM state", np.array(out["small"][2]), np.array(out["big"][2]), 2 * atol, 2 * rtol, scale_to_ref=True)
    print(f"[batch invariance] rows {rows}: tokens equal, logits differ by at most {e1:.2e}, state by {e2:.2e} (relative)", flush=True)
    return e1


def test_c1_falcon_h1_0p5b_shape():
    """36 layers, d_model 1024, vocab 32768, bf16, batch 1, prompt 512, k = 2."""
    w = _run("c1", seed=0, G=40, rounds=12, layers=[0, 17, 35], min_gap=4e-4)      # seed audited: smallest gap 1.9e-3
    assert w["rounds"] == 12


def test_c1_shape_strict_state_and_layer_mask():
    """The 0.5B shape with the draft model's own recurrent state (a second prefill pass with attention
    suppressed, k + 1 draft steps, two rebuilds per commit), and with a draft mask in which the first and the
    last third of the layers keep their attention branch and the middle third is skipped (the draft steps then
    run one-row attention over the 256-token cache)."""
    w = _run("c1", seed=0, G=16, rounds=5, lens=[256], layers=[0, 35], draft_state="strict")
    assert w["rounds"] == 5 and w["ms_ssm"] > 0
    mask = ["full"] * 12 + ["skip"] * 12 + ["ssm"] * 12
    w2 = _run("c1", seed=0, G=16, rounds=5, lens=[256], layers=[0, 35], draft_mask=mask)
    n = min(len(w["tokens"][0]), len(w2["tokens"][0]))       # five rounds commit different counts; the streams agree
    assert n >= 5 and w2["tokens"][0][:n] == w["tokens"][0][:n]


def test_c2_batch16_ragged_forced():
    """Same shape, batch 16, k = 4, ragged prompts around 600 tokens, forced acceptance pattern
    p = 0.37; oracle on rows 0 and 15 (a ragged batch: slices and passes end at different places
    per sequence)."""
    lens = [600 - 13 * i for i in range(16)]
    w = _run("c2f", seed=0, G=24, rounds=6, lens=lens, rows=[0, 15], layers=[0, 35], forced_p=0.37,
             min_gap=1e-4)                                                           # seed audited: smallest gap 5.6e-4
    assert w["rounds"] == 6


def test_c2_batch16_full_prompts():
    """The second workload at its real size: 16 independent prompts of 2048 tokens, k = 4, HIP graphs,
    default pages and chunks (8 prefill passes of 256 positions per sequence over a growing cache,
    16 key slices per KV head merged by the merge kernel in verification).  The float64 oracle's
    prefill of 2048 tokens at this shape takes minutes per sequence on the host cores, so it follows
    sequence 0 only; the other rows run the same kernels on the same shapes."""
    w = _run("c2", seed=0, G=16, rounds=3, rows=[0], layers=[0, 35], min_gap=5e-3)   # seed audited: smallest gap 2.4e-2
    assert w["rounds"] == 3


def test_c3_falcon_h1_3b_shape():
    """32 layers, d_model 2560, vocab 65536, head_dim 128, d_state 256, bf16, batch 1, k = 4.
    Prompt 1024 here (the oracle's float64 prefill of 4096 tokens takes minutes)."""
    w = _run("c3", seed=0, G=16, rounds=4, lens=[1024], layers=[0, 31], min_gap=2e-3)   # seed audited: smallest gap 7.4e-3
    assert w["rounds"] == 4


def test_c4_batch64_k8_forced():
    """3B shape, batch 64, k = 8, forced acceptance p = 0.68 (the paper's per-token rate): the
    9-position verification runs 576 rows per pass.  Ragged prompts of 71..260 tokens stand in
    for the 32768-token prompts, which neither the float64 oracle nor a test-sized prefill can
    afford; the oracle follows the longest and the shortest sequence, and three sequences are run
    again as a batch of their own (batch invariance: what the other 61 rows rest on)."""
    lens = [260 - 3 * i for i in range(64)]
    w = _run("c4", seed=0, G=30, rounds=3, lens=lens, rows=[0, 63], layers=[0, 31], forced_p=0.68,
             min_gap=2e-3, invariance_rows=[0, 31, 63])                              # seed audited: smallest gap 7.6e-3
    assert w["rounds"] == 3
