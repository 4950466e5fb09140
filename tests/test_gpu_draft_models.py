"""Draft models other than the default (HIP library vs CPU oracle through the C ABI, needs an MI355X):
the strict draft state (M_S as a model of its own over the whole prefix, Eq. 4 / Section 3.3 draft
phase) and per-layer draft masks (full / SSM-only / skipped blocks, Section 4.2 and Eq. 5)."""
import numpy as np
import pytest

from paper_2605_01106_amd import workloads as W

pytestmark = pytest.mark.gpu

from parity_util import run_lockstep  # noqa: E402


@pytest.fixture(scope="module")
def B():
    from paper_2605_01106_amd import binding
    return binding


def _say(tag):
    def f(w):
        print(f"[{tag}] rounds={w['rounds']} mean_n={w['mean_n']:.2f} min_gap={w['min_gap']:.2e} "
              f"err: logits={w['logits']:.2e} ssm={w['ssm']:.2e} conv={w['conv']:.2e} kv={w['kv']:.2e} "
              f"M_S ssm={w['ms_ssm']:.2e} conv={w['ms_conv']:.2e}", flush=True)
    return f


def _lively(dtype, n_layers=3):
    cfg = W.scaled_config("lively", n_layers=n_layers, d_model=72, vocab=200, m_heads=3, m_head_dim=40, d_state=16,
                          n_q_heads=6, n_kv_heads=2, head_dim=24, d_ff=104, w_dtype=dtype)
    return cfg, W.make_lively_weights(cfg, 7)


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_strict_draft_state_lockstep(B, dtype):
    """draft_state_mode = 1 against the oracle's strict mode, call by call: drafts, draft logits,
    targets, accepted counts, both committed states (M_H's and M_S's own) after prefill (ragged
    prompts over several passes) and after every commit.  The committed stream equals the shared
    mode's.  (These weights accept few drafts; commits that keep several drafts are in the forced-count
    test below.)"""
    cfg, wts = _lively(dtype)
    lens = [37, 5, 70, 18]
    prompts = W.make_prompts(cfg.vocab, 4, lens, 3)
    ctx = B.Context(wts, 4, 160, 4, 24, kv_page_tokens=16, prefill_chunk=16, draft_state_mode=1)
    w = run_lockstep(ctx, wts, prompts, lens, 24, 3, engine="pass", draft_state="strict", report=_say(f"strict-{dtype}"))
    shared = B.Context(wts, 4, 160, 4, 24, kv_page_tokens=16, prefill_chunk=16)
    w2 = run_lockstep(shared, wts, prompts, lens, 24, 3, engine="pass", report=_say(f"shared-{dtype}"))
    assert w["tokens"] == w2["tokens"]
    with pytest.raises(B.HHError):
        shared.hh_get_draft_state(0)
    with pytest.raises(B.HHError):
        ctx.hh_set_draft_mask(["full", "ssm", "ssm"])      # the strict state is the SSM-only draft's


def test_strict_state_with_draft_schedule_forced_counts_and_replaced_drafts(B):
    """The strict state through the other ways a round can go: a different k every round (k = 0
    included: M_S still consumes the pending token), forced accepted counts, caller-supplied
    drafts (M_S re-reads the replaced tokens), HIP graphs, and a second prefill on the same context."""
    import torch
    cfg, wts = _lively(W.BF16)
    lens = [12, 30, 7]
    prompts = W.make_prompts(cfg.vocab, 3, lens, 9)
    k, G = 4, 20
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = B.Context(wts, 3, 128, k, G, kv_page_tokens=32, prefill_chunk=32, draft_state_mode=1, use_graphs=1)
        a = run_lockstep(ctx, wts, prompts, lens, G, [3, 0, 1, 4, 2], draft_state="strict", report=_say("strict k-schedule"))
        forced = W.make_forced_pattern(64, 3, k, 0.6, 1)
        run_lockstep(ctx, wts, prompts, lens, G, k, forced=forced, draft_state="strict", report=_say("strict forced"))
        override = W.make_random_drafts(cfg.vocab, 64, 3, k, 2)
        b = run_lockstep(ctx, wts, prompts, lens, G, k, override=override, draft_state="strict", report=_say("strict random drafts"))
    stream.synchronize()
    assert a["tokens"] == b["tokens"]


def test_strict_state_stochastic(B):
    """Temperature > 0 with the strict state: the draft distribution is M_S's over the whole prefix."""
    cfg, wts = _lively(W.F32)
    lens = [37, 5, 70, 18]
    prompts = W.make_prompts(cfg.vocab, 4, lens, 3)
    ctx = B.Context(wts, 4, 160, 4, 24, kv_page_tokens=16, prefill_chunk=16, draft_state_mode=1)
    run_lockstep(ctx, wts, prompts, lens, 24, 3, engine="pass", draft_state="strict", temperature=0.6, sample_seed=59,
                 report=_say("strict T=0.6"))


MASKS = [("full", "full", "full"), ("skip", "skip", "skip"), ("full", "ssm", "skip"), ("skip", "full", "ssm"),
         ("ssm", "skip", "full")]


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_draft_masks_lockstep(B, dtype):
    """Every mask against the oracle's masked draft, on one context (the mask changes between
    prefills).  The all-full mask drafts with M_H itself: every draft is accepted.  The committed
    stream is the same under every mask; the default mask restores the Eq. 4 draft."""
    cfg, wts = _lively(dtype)
    lens = [37, 5, 70, 18]
    prompts = W.make_prompts(cfg.vocab, 4, lens, 3)
    ctx = B.Context(wts, 4, 160, 4, 24, kv_page_tokens=16, prefill_chunk=16)
    base = run_lockstep(ctx, wts, prompts, lens, 24, 3, engine="pass", report=_say(f"mask default {dtype}"))
    for mask in MASKS:
        w = run_lockstep(ctx, wts, prompts, lens, 24, 3, engine="pass", draft_mask=mask,
                         report=_say(f"mask {'/'.join(mask)} {dtype}"))
        assert w["tokens"] == base["tokens"]
        if mask == ("full", "full", "full"):
            assert w["mean_n"] == 3.0
    again = run_lockstep(ctx, wts, prompts, lens, 24, 3, engine="pass", draft_mask=None)
    assert again["mean_n"] == base["mean_n"] and again["tokens"] == base["tokens"]
    with pytest.raises(B.HHError):
        ctx.hh_set_draft_mask([0, 1, 7])


def test_draft_mask_long_cache_and_graphs(B):
    """A full-attention draft layer over caches long enough for several key slices (the draft step
    is a one-row attention pass, a shape the verification pass never has), replayed as HIP graphs;
    the mask is changed on the live context, which drops the captured draft sequences."""
    import torch
    cfg = W.scaled_config("thin", n_layers=2, d_model=64, vocab=128, m_heads=2, m_head_dim=32, d_state=16,
                          n_q_heads=4, n_kv_heads=2, head_dim=64, d_ff=64, w_dtype=W.BF16)
    wts = W.make_lively_weights(cfg, 47)
    lens = [1500, 700]
    prompts = W.make_prompts(cfg.vocab, 2, lens, 5)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = B.Context(wts, 2, 1600, 3, 12, prefill_chunk=256, use_graphs=1, attn_single_slice_steps=-1)
        a = run_lockstep(ctx, wts, prompts, lens, 12, 3, engine="pass", draft_mask=("full", "ssm"), check_kv=False,
                         report=_say("mask full/ssm long"))
        b = run_lockstep(ctx, wts, prompts, lens, 12, 3, engine="pass", draft_mask=("ssm", "full"), check_kv=False,
                         report=_say("mask ssm/full long"))
    stream.synchronize()
    assert a["tokens"] == b["tokens"]
