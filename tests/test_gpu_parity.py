"""HIP library vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import json
import os

import numpy as np
import pytest

from paper_2605_01106_amd import workloads as W

pytestmark = pytest.mark.gpu

from parity_util import run_lockstep  # noqa: E402


@pytest.fixture(scope="module")
def B():
    from paper_2605_01106_amd import binding
    return binding


def _ctx(B, weights, batch, max_seq, kmax, G, **kw):
    return B.Context(weights, batch, max_seq, kmax, G, **kw)


def _say(tag):
    def f(w):
        print(f"[{tag}] rounds={w['rounds']} mean_n={w['mean_n']:.2f} min_gap={w['min_gap']:.2e} "
              f"err: logits={w['logits']:.2e} ssm={w['ssm']:.2e} conv={w['conv']:.2e} kv={w['kv']:.2e}", flush=True)
    return f


def test_c0_full_run(B):
    """Config 0 end to end: tiny fp32 hybrid, prompt 32, 64 new tokens, k = 2."""
    wl = W.WORKLOADS["c0"]
    seed = 1
    wts = W.make_weights(wl.cfg, seed)
    prompts = W.make_prompts(wl.cfg.vocab, 1, wl.prompt_len, seed)
    ctx = _ctx(B, wts, 1, 128, wl.k, wl.gen_len)
    w = run_lockstep(ctx, wts, prompts, [wl.prompt_len], wl.gen_len, wl.k, engine="step", min_gap=2e-5,
                     report=_say("c0"))
    assert w["rounds"] >= 20


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_lively_ragged_batch(B, dtype):
    """Odd sizes, O(1) recurrence and attention (so state, window and cache errors move the
    logits), ragged prompts that span several prefill passes, several KV pages and tiles."""
    cfg = W.scaled_config("lively", n_layers=3, d_model=72, vocab=200, m_heads=3, m_head_dim=40, d_state=16,
                          n_q_heads=6, n_kv_heads=2, head_dim=24, d_ff=104, w_dtype=dtype)
    wts = W.make_lively_weights(cfg, 7)
    lens = [37, 5, 70, 18]
    prompts = W.make_prompts(cfg.vocab, 4, lens, 3)
    ctx = _ctx(B, wts, 4, 160, 4, 24, kv_page_tokens=16, prefill_chunk=16)
    run_lockstep(ctx, wts, prompts, lens, 24, 3, engine="pass", report=_say(f"lively-{dtype}"))


@pytest.mark.parametrize("k", [0, 1, 5])
def test_draft_lengths_and_plain_greedy(B, k):
    cfg = W.scaled_config("klen", n_layers=2, d_model=64, vocab=128, m_heads=2, m_head_dim=32, d_state=32,
                          n_q_heads=4, n_kv_heads=4, head_dim=16, d_ff=64, w_dtype=W.F32)
    wts = W.make_lively_weights(cfg, 11)
    lens = [9, 20]
    prompts = W.make_prompts(cfg.vocab, 2, lens, 5)
    ctx = _ctx(B, wts, 2, 96, 5, 16, prefill_chunk=8)
    run_lockstep(ctx, wts, prompts, lens, 16, k, engine="step", report=_say(f"k={k}"))


@pytest.mark.parametrize("k,d_state,dtype", [(2, 32, W.BF16), (4, 64, W.BF16), (8, 64, W.F32), (0, 128, W.BF16)])
def test_aligned_shapes_fast_paths(B, k, d_state, dtype):
    """Shapes whose rows are 16-byte aligned (heads and head dimension multiples of 4, state a
    multiple of 32) take the few-positions SSM kernel (8 or 16 lanes per state row, a partly
    filled last workgroup) and, with a bf16 cache and 32-token pages, the matrix-core attention
    with one to three 16-row tiles (k + 1 positions x 4 query heads per KV head); prompts straddle
    pages and key steps, one sequence finishes early."""
    cfg = W.scaled_config("aligned", n_layers=2, d_model=64, vocab=160, m_heads=4, m_head_dim=12, d_state=d_state,
                          n_q_heads=8, n_kv_heads=2, head_dim=32, d_ff=96, w_dtype=dtype)
    wts = W.make_lively_weights(cfg, 17)
    lens = [33, 6, 95]
    prompts = W.make_prompts(cfg.vocab, 3, lens, 21)
    ctx = _ctx(B, wts, 3, 160, 8, 30, kv_page_tokens=32, prefill_chunk=32)
    run_lockstep(ctx, wts, prompts, lens, 30, k, engine="pass", report=_say(f"aligned-k{k}-N{d_state}-{dtype}"))


# ---------------------------------------------------------------------------------------------
# Long caches on thin models: the key-slice paths of the matrix-core attention that the
# paper-shaped workloads take at their real prompt lengths (Section 3.3, verification phase: M_H
# attends over the whole prefix), at a cost the float64 oracle can afford.

def _thin(name, head_dim, n_q, n_kv, **kw):
    base = dict(n_layers=2, d_model=64, vocab=192, m_heads=4, m_head_dim=16, d_state=32, n_q_heads=n_q,
                n_kv_heads=n_kv, head_dim=head_dim, d_ff=96, w_dtype=W.BF16)
    base.update(kw)
    return W.scaled_config(name, **base)


def test_long_cache_ticket_merge(B):
    """Head dimension 64, one sequence, 1100 cached keys, 32-token pages: 35 key steps, so the
    verification attention runs 9 key slices per KV head whose partial results are merged inside the
    kernel by the workgroup that draws the last ticket (18 workgroups, 37 KB of partials per row
    chunk: under both limits of that path).  Prefill chunks of 256 positions run the multi-tile
    kernel over a growing cache."""
    cfg = _thin("thin-ticket", 64, 4, 2)
    wts = W.make_lively_weights(cfg, 47)          # seeds audited: top-1/top-2 gap 5.4e-3
    lens = [1100]
    prompts = W.make_prompts(cfg.vocab, 1, lens, 12)
    ctx = _ctx(B, wts, 1, 1100 + 40, 2, 12, kv_page_tokens=32, prefill_chunk=256)
    w = run_lockstep(ctx, wts, prompts, lens, 12, 2, engine="pass", chunk=64, min_gap=1e-3, report=_say("ticket-merge"))
    assert w["rounds"] >= 4


def test_long_cache_merge_kernel_batch16(B):
    """Head dimension 64 (two 32-wide key blocks), 16 sequences with 1900..2110 cached keys, k = 4:
    16 key slices x 32 (sequence, KV head) pairs = 512 workgroups, so the slices are merged by the
    separate merge kernel; the batch is ragged, so slices end at different steps per sequence.
    The oracle follows the longest and the shortest sequence."""
    cfg = _thin("thin-merge", 64, 8, 2)
    wts = W.make_lively_weights(cfg, 47)          # seeds audited: top-1/top-2 gap 3.4e-3
    lens = [2110 - 14 * i for i in range(16)]
    prompts = W.make_prompts(cfg.vocab, 16, lens, 13)
    ctx = _ctx(B, wts, 16, 2110 + 48, 4, 10, kv_page_tokens=64, prefill_chunk=128)
    w = run_lockstep(ctx, wts, prompts, lens, 10, 4, engine="pass", chunk=64, oracle_rows=[0, 15],
                     min_gap=1e-3, report=_say("merge-kernel-b16"))
    assert w["rounds"] >= 2


@pytest.mark.parametrize("overlap_mode", [1, 3])
def test_long_cache_head128_three_row_tiles(B, overlap_mode):
    """Head dimension 128, 5 query heads per KV head, k = 8: 45 query rows = three 16-row tiles per
    workgroup, the new keys appended and scored inside the kernel, 3 sequences of about 1150 cached
    keys (10 slices per KV head, 245 KB of partials per row chunk: the separate merge kernel, as at
    the 3B shape).  Forced accepted counts exercise the rollback to every position.  Run once with the
    attention branch in line (overlap_mode 1) and once forked to the side stream beside the SSM
    branch in every pass (overlap_mode 3): the schedule must not change a result."""
    cfg = _thin("thin-h128", 128, 10, 2)
    wts = W.make_lively_weights(cfg, 41)          # seeds audited: top-1/top-2 gap 8.2e-4
    lens = [1150, 1101, 1127]
    prompts = W.make_prompts(cfg.vocab, 3, lens, 14)
    forced = W.make_forced_pattern(32, 3, 8, 0.68, 3)
    ctx = _ctx(B, wts, 3, 1150 + 80, 8, 27, kv_page_tokens=64, prefill_chunk=192, overlap_mode=overlap_mode)
    w = run_lockstep(ctx, wts, prompts, lens, 27, 8, forced=forced, engine="pass", chunk=64,
                     min_gap=4e-4, report=_say(f"h128-rt3-overlap{overlap_mode}"))
    assert w["rounds"] >= 3


@pytest.mark.parametrize("max_splits,single", [(1, 0), (3, -1), (32, -1)])
def test_key_slices_do_not_change_results(B, max_splits, single):
    """The number of key slices is a tunable: one slice, three, and as many as the cache allows
    (split from the first step on), on caches of 70..200 keys with 32-token pages."""
    cfg = _thin("thin-slices", 32, 8, 2, d_state=64)
    wts = W.make_lively_weights(cfg, 42)          # seeds audited: top-1/top-2 gap 2.6e-3
    lens = [200, 70, 131]
    prompts = W.make_prompts(cfg.vocab, 3, lens, 15)
    ctx = _ctx(B, wts, 3, 256, 4, 12, kv_page_tokens=32, prefill_chunk=64, attn_max_splits=max_splits,
               attn_single_slice_steps=single)
    run_lockstep(ctx, wts, prompts, lens, 12, 3, engine="pass", min_gap=1e-3, report=_say(f"slices-{max_splits}"))


@pytest.mark.parametrize("flag", ["HH_KF_ATTN_SCALAR", "HH_KF_SSM_GENERAL", "HH_KF_MID_OFF", "HH_KF_SKINNY_OFF",
                                  "HH_KF_SSM_SCALAR_CONV", "HH_KF_MID_OFF|HH_KF_ROWS_LDS", "HH_KF_NO_HANDOVER"])
def test_kernel_selection_flags_do_not_change_results(B, flag):
    """Every kernel-selection switch routes a family of launches to the slower kernel that computes
    the same thing; each variant is checked against the oracle on a workload that reaches the family:
    6 sequences with k = 3 give 6 draft rows (skinny), 24 verification rows (mid) and 6 x 32 = 192
    prefill rows (many-row GEMM), a bf16 cache with 32-token pages and aligned SSM shapes."""
    cfg = _thin("thin-flags", 32, 4, 2, d_model=96, d_ff=160, d_state=32)
    wts = W.make_lively_weights(cfg, 46)          # seeds audited: top-1/top-2 gap 8.9e-4
    lens = [61, 33, 90, 47, 75, 52]
    prompts = W.make_prompts(cfg.vocab, 6, lens, 16)
    bits = 0
    for name in flag.split("|"):
        bits |= getattr(B, name)
    ctx = _ctx(B, wts, 6, 128, 3, 10, kv_page_tokens=32, prefill_chunk=32, kernel_flags=bits)
    run_lockstep(ctx, wts, prompts, lens, 10, 3, engine="pass", min_gap=4e-4, report=_say(flag))


def test_mid_rows_long_k_and_wide_head(B):
    """17..96 activation rows through the K-loop kernel with several K windows per workgroup:
    d_model 320 (2.5 windows of 128 columns, so the last window is partly outside K) and a
    24000-row LM head (enough weight tiles that a workgroup walks two windows: the loop, its
    tail and the K-chunk reduction); 5 sequences, k = 4: 25 rows in verification, 80 in the
    prefill passes, 5 in the draft steps."""
    cfg = W.scaled_config("midk", n_layers=2, d_model=320, vocab=24000, m_heads=4, m_head_dim=40, d_state=16,
                          n_q_heads=4, n_kv_heads=2, head_dim=32, d_ff=520, w_dtype=W.BF16)
    wts = W.make_lively_weights(cfg, 37)          # seeds audited: top-1/top-2 gap 2.5e-4
    lens = [40, 9, 70, 23, 33]
    prompts = W.make_prompts(cfg.vocab, 5, lens, 7)
    ctx = _ctx(B, wts, 5, 128, 4, 16, kv_page_tokens=32, prefill_chunk=16)
    run_lockstep(ctx, wts, prompts, lens, 16, 4, engine="pass", report=_say("midk"))


@pytest.mark.parametrize("keep_logits", [1, 0])
def test_row_block_kernel_chunks_planes_and_argmax(B, keep_logits):
    """17..96 activation rows with a long, thin model (d_inner = d_ff = 2048 against d_model 64):
    the out and down projections have few weight tiles and a long K (many K chunks per product, norm
    scale from the chunks' sums of squares), 25 verification rows and 80-row prefill passes (two and
    five row tiles).  The LM head's argmax is raised with atomic maxima in the chunk reduction; with
    keep_logits = 0 no logits are written at all: tokens, counts, state and cache must still match."""
    cfg = W.scaled_config("rowblock", n_layers=2, d_model=64, vocab=200, m_heads=32, m_head_dim=64, d_state=16,
                          n_q_heads=4, n_kv_heads=2, head_dim=32, d_ff=2048, w_dtype=W.BF16)
    wts = W.make_lively_weights(cfg, 50)          # seeds audited: top-1/top-2 gap 7.3e-4
    lens = [40, 9, 70, 23, 33]
    prompts = W.make_prompts(cfg.vocab, 5, lens, 7)
    ctx = _ctx(B, wts, 5, 128, 4, 12, kv_page_tokens=32, prefill_chunk=16, keep_logits=keep_logits)
    run_lockstep(ctx, wts, prompts, lens, 12, 4, engine="pass", min_gap=4e-4, compare_logits=bool(keep_logits),
                 report=_say(f"rowblock-keep{keep_logits}"))
    if not keep_logits:
        with pytest.raises(B.HHError) as ei:
            ctx.hh_get_logits(1)
        assert ei.value.status == B.HH_ESTATE


def test_many_rows_lively(B):
    """More than 96 activation rows (10 sequences x 16-position prefill chunks = 160 rows: the
    tiled matrix-core GEMM over pre-split activations) on the initialisation with order-one
    activations, which amplifies any loss of precision in the projections: a two-term bf16 split
    of the activations there (16 mantissa bits) puts hundreds of logits outside the tolerance."""
    cfg = W.scaled_config("lively", n_layers=3, d_model=72, vocab=200, m_heads=3, m_head_dim=40, d_state=16,
                          n_q_heads=6, n_kv_heads=2, head_dim=24, d_ff=104, w_dtype=W.BF16)
    wts = W.make_lively_weights(cfg, 8)           # seeds audited: top-1/top-2 gap 1.1e-4
    lens = [37, 5, 70, 18, 44, 63, 29, 51, 12, 66]
    prompts = W.make_prompts(cfg.vocab, 10, lens, 4)
    ctx = _ctx(B, wts, 10, 160, 4, 24, kv_page_tokens=32, prefill_chunk=16)
    run_lockstep(ctx, wts, prompts, lens, 24, 3, engine="pass", report=_say("many-rows-lively"))


def _say_t(tag):
    def f(w):
        print(f"[{tag}] rounds={w['rounds']} mean_n={w['mean_n']:.2f} min_margin={w['min_margin']:.2e} "
              f"err: logits={w['logits']:.2e} ssm={w['ssm']:.2e} conv={w['conv']:.2e} kv={w['kv']:.2e}", flush=True)
    return f


@pytest.mark.parametrize("dtype,runs", [(W.F32, [(0.6, 59), (0.3, 10)]), (W.BF16, [(0.6, 21), (0.3, 32)])])
def test_stochastic_acceptance_lockstep(B, dtype, runs):
    """Temperature > 0 (Eq. 6): first token, draft draws, rejection tests, correction and bonus
    tokens equal the oracle's, decision by decision, with the same counter-based uniforms; the
    targets row has the oracle's form, and state, window and cache follow the committed stream.
    Odd vocabulary (203: ragged tail of the drawing kernel's 4-element groups).  Seeds audited:
    no decision within 1e-4 of flipping (a logit error e moves a CDF edge by at most e / T times the
    mass it touches; the measured logit errors are 1e-6 for float32 and, on single entries, up to
    1e-3 for bf16 storage).  One context runs temperature 0.6, then greedy, then temperature 0.3
    with another seed: the captured launch sequences must pick up the new parameters."""
    cfg = W.scaled_config("lively", n_layers=3, d_model=72, vocab=203, m_heads=3, m_head_dim=40, d_state=16,
                          n_q_heads=6, n_kv_heads=2, head_dim=24, d_ff=104, w_dtype=dtype)
    wts = W.make_lively_weights(cfg, 7)
    lens = [37, 5, 70, 18]
    prompts = W.make_prompts(cfg.vocab, 4, lens, 3)
    ctx = _ctx(B, wts, 4, 160, 4, 12, kv_page_tokens=16, prefill_chunk=16)
    streams = []
    for i, (T, seed) in enumerate(runs):
        w = run_lockstep(ctx, wts, prompts, lens, 12, 3, engine="pass", temperature=T, sample_seed=seed,
                         min_margin=1e-4, report=_say_t(f"stochastic-{dtype}-T{T}"))
        assert 0.0 < w["mean_n"] < 3.0            # both kept and rejected drafts occurred
        streams.append(w["tokens"])
        if i == 0:   # back to temperature 0 on the same context: the greedy stream again
            run_lockstep(ctx, wts, prompts, lens, 12, 3, engine="pass", report=_say("greedy-after-stochastic"))
    assert streams[0] != streams[1]


def test_stochastic_wide_vocabulary_and_plain_sampling(B):
    """A 24001-entry vocabulary (every wavefront of the drawing workgroup walks its segment in
    several 256-entry groups, ragged end) with float32 weights, few decisions: the CDF edges are
    4e-5 apart, the audited seed keeps 8e-6 from the nearest one, the float32 logit error of 2e-6
    moves an edge by at most 4e-6 at T = 0.5.  Then k = 0: plain sampling from M_H."""
    cfg = W.scaled_config("widev", n_layers=1, d_model=64, vocab=24001, m_heads=2, m_head_dim=32, d_state=16,
                          n_q_heads=2, n_kv_heads=1, head_dim=32, d_ff=64, w_dtype=W.F32)
    wts = W.make_lively_weights(cfg, 3)
    lens = [11, 6]
    prompts = W.make_prompts(cfg.vocab, 2, lens, 2)
    ctx = _ctx(B, wts, 2, 64, 2, 4, prefill_chunk=8)
    run_lockstep(ctx, wts, prompts, lens, 4, 2, engine="pass", temperature=0.5, sample_seed=327, min_margin=8e-6,
                 report=_say_t("stochastic-wide"))
    cfg = W.scaled_config("klen", n_layers=2, d_model=64, vocab=128, m_heads=2, m_head_dim=32, d_state=32,
                          n_q_heads=4, n_kv_heads=4, head_dim=16, d_ff=64, w_dtype=W.F32)
    wts = W.make_lively_weights(cfg, 5)
    lens = [9, 21]
    prompts = W.make_prompts(cfg.vocab, 2, lens, 2)
    ctx = _ctx(B, wts, 2, 96, 5, 12, prefill_chunk=8)
    run_lockstep(ctx, wts, prompts, lens, 12, 0, engine="step", temperature=0.8, sample_seed=27, min_margin=4e-4,
                 report=_say_t("plain-sampling"))


def test_stochastic_call_rules(B):
    """At temperature > 0 replaced drafts and forced counts are refused (neither has a draft
    distribution or a correction token); a bad temperature is refused; sampling cannot change
    inside a round."""
    import torch
    cfg = W.scaled_config("rules", n_layers=1, d_model=64, vocab=96, m_heads=2, m_head_dim=32, d_state=16,
                          n_q_heads=2, n_kv_heads=1, head_dim=32, d_ff=64, w_dtype=W.F32)
    wts = W.make_lively_weights(cfg, 1)
    lens = [8, 5]
    prompts = W.make_prompts(cfg.vocab, 2, lens, 1)
    ctx = _ctx(B, wts, 2, 64, 2, 8, prefill_chunk=8)
    with pytest.raises(B.HHError):
        ctx.hh_set_sampling(-1.0, 0)
    with pytest.raises(B.HHError):
        ctx.hh_set_sampling(float("nan"), 0)
    ctx.hh_set_sampling(0.7, 3)
    ctx.hh_prefill(prompts, lens, 8)
    ctx.hh_draft(2)
    with pytest.raises(B.HHError):
        ctx.hh_set_sampling(0.5, 3)
    with pytest.raises(B.HHError):
        ctx.hh_set_drafts(np.zeros((2, 2), np.int32))
    ctx.hh_verify()
    with pytest.raises(B.HHError):
        ctx.hh_commit(torch.zeros(2, dtype=torch.int32, device=ctx.device))
    ctx.hh_commit()
    d, g = ctx.hh_get_round()
    _, _, last_n = ctx.hh_get_lengths()
    for b in range(2):
        n = last_n[b]
        assert list(g[b][:n]) == list(d[b][:n]) and 0 <= g[b][n] < cfg.vocab and all(v == -1 for v in g[b][n + 1:])
        if n < 2:
            assert g[b][n] != d[b][n]


def test_draft_length_changes_every_round(B):
    """A different k every round on one context (the choice of k per round is the caller's: the
    adaptive draft length the paper names as future work needs nothing else from the library).
    Every round matches the oracle, and the committed stream equals that of a fixed k."""
    cfg = W.scaled_config("lively", n_layers=3, d_model=72, vocab=200, m_heads=3, m_head_dim=40, d_state=16,
                          n_q_heads=6, n_kv_heads=2, head_dim=24, d_ff=104, w_dtype=W.BF16)
    wts = W.make_lively_weights(cfg, 7)
    lens = [37, 5, 70, 18]
    prompts = W.make_prompts(cfg.vocab, 4, lens, 3)
    ctx = _ctx(B, wts, 4, 160, 4, 24, kv_page_tokens=16, prefill_chunk=16)
    w = run_lockstep(ctx, wts, prompts, lens, 24, [3, 0, 1, 4, 2], engine="pass", report=_say("k-schedule"))
    w2 = run_lockstep(ctx, wts, prompts, lens, 24, 3, engine="pass", report=_say("k-fixed"))
    assert w["tokens"] == w2["tokens"]


def test_forced_acceptance_and_arbitrary_drafts(B):
    """Forced accepted counts (drafts committed as drafted) and caller-supplied draft tokens."""
    cfg = W.scaled_config("forced", n_layers=2, d_model=64, vocab=96, m_heads=4, m_head_dim=16, d_state=8,
                          n_q_heads=2, n_kv_heads=1, head_dim=32, d_ff=128, w_dtype=W.BF16)
    wts = W.make_lively_weights(cfg, 13)
    lens = [12, 30, 7]
    prompts = W.make_prompts(cfg.vocab, 3, lens, 9)
    k, G = 4, 20
    forced = W.make_forced_pattern(64, 3, k, 0.6, 1)
    ctx = _ctx(B, wts, 3, 128, k, G, kv_page_tokens=32, prefill_chunk=32)
    run_lockstep(ctx, wts, prompts, lens, G, k, forced=forced, report=_say("forced"))
    override = W.make_random_drafts(cfg.vocab, 64, 3, k, 2)
    w = run_lockstep(ctx, wts, prompts, lens, G, k, override=override, report=_say("random-drafts"))
    # the committed stream does not depend on the draft source
    w2 = run_lockstep(ctx, wts, prompts, lens, G, k, report=_say("ssm-drafts"))
    assert w["tokens"] == w2["tokens"]


def test_graph_replay_matches_oracle(B):
    """With use_graphs the draft and verify launch sequences are captured on their second use and
    replayed afterwards; every replay (one per round, with read-backs and eager commits between
    them) is compared with the oracle, and the token stream with the eager run."""
    import torch
    wl = W.WORKLOADS["c0"]
    seed = 1
    wts = W.make_weights(wl.cfg, seed)
    prompts = W.make_prompts(wl.cfg.vocab, 1, wl.prompt_len, seed)
    eager = run_lockstep(_ctx(B, wts, 1, 128, wl.k, 40), wts, prompts, [wl.prompt_len], 40, wl.k, engine="step")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = _ctx(B, wts, 1, 128, wl.k, 40, use_graphs=1)
        w = run_lockstep(ctx, wts, prompts, [wl.prompt_len], 40, wl.k, engine="step", report=_say("graphs"))
        # a second batch on the same context reuses the instantiated graphs
        w2 = run_lockstep(ctx, wts, prompts, [wl.prompt_len], 40, wl.k, engine="step", check_state_every=4)
    stream.synchronize()
    assert w["tokens"] == eager["tokens"] == w2["tokens"] and w["rounds"] >= 10


@pytest.mark.parametrize("dtype,d_state,chunk", [(W.F32, 64, 64), (W.F32, 128, 256), (W.BF16, 64, 128), (W.BF16, 256, 40)])
def test_prefill_scan_matmul_form(B, dtype, d_state, chunk):
    """Prefill passes of 16 and more positions take the matmul (state-space dual) form of the scan on
    the matrix cores: head dimension 64, state sizes 64 / 128 / 256, passes of 40 to 256 positions
    (several 32-position chunks per pass, a ragged last chunk and a ragged last pass per sequence, a
    sequence shorter than one chunk), weights with order-one recurrence so that a wrong decay factor,
    a dropped intra-chunk term or a wrong carried state moves the logits.  The state after prefill,
    the conv window, the logits and every later round are compared with the sequential float64 oracle;
    the same run with the position-by-position kernel (HH_KF_SSM_SEQUENTIAL) gives the same tokens."""
    cfg = W.scaled_config("ssd", n_layers=2, d_model=64, vocab=160, m_heads=2, m_head_dim=64, d_state=d_state,
                          n_q_heads=2, n_kv_heads=1, head_dim=32, d_ff=96, w_dtype=dtype)
    wts = W.make_lively_weights(cfg, 61)
    lens = [333, 17, 290, 97]
    prompts = W.make_prompts(cfg.vocab, 4, lens, 23)
    # (the library takes the matmul form by itself from 128 workgroups on; HH_KF_SSM_MATMUL forces it for these 4 x 1)
    ctx = _ctx(B, wts, 4, 400, 3, 10, kv_page_tokens=32, prefill_chunk=chunk, kernel_flags=B.HH_KF_SSM_MATMUL)
    w = run_lockstep(ctx, wts, prompts, lens, 10, 3, engine="pass", chunk=64, report=_say(f"ssd-{dtype}-N{d_state}-T{chunk}"))
    seq = _ctx(B, wts, 4, 400, 3, 10, kv_page_tokens=32, prefill_chunk=chunk, kernel_flags=B.HH_KF_SSM_SEQUENTIAL)
    w2 = run_lockstep(seq, wts, prompts, lens, 10, 3, engine="pass", chunk=64)
    assert w["tokens"] == w2["tokens"]
