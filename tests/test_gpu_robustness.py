"""Robustness of the library on a live context (needs an MI355X): calls out of order or beyond
capacity are refused on the host and leave every piece of device state bit-identical; identical
inputs give bit-identical results, with the launch sequences enqueued directly and replayed as
HIP graphs; nothing is written outside the workspace the caller handed over."""
import numpy as np
import pytest

from paper_2605_01106_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2605_01106_amd import binding
    return binding


def _model(dtype=W.BF16):
    cfg = W.scaled_config("robust", n_layers=2, d_model=64, vocab=160, m_heads=4, m_head_dim=16, d_state=32,
                          n_q_heads=4, n_kv_heads=2, head_dim=32, d_ff=96, w_dtype=dtype)
    return cfg, W.make_lively_weights(cfg, 5)


def _snapshot(ctx, layers):
    """Everything a caller can read back, as bytes."""
    kv_len, committed, last_n = ctx.hh_get_lengths()
    out = [np.array(kv_len), np.array(committed), np.array(last_n)]
    for b in range(ctx.B):
        out.append(np.array(ctx.hh_get_tokens(b), np.int32))
    for l in range(layers):
        ssm, conv = ctx.hh_get_state(l)
        out += [ssm, conv]
        for b in range(ctx.B):
            out += list(ctx.hh_get_kv(l, b, kv_len[b]))
    return [a.tobytes() for a in out]


def test_refused_calls_leave_state_untouched(B):
    import torch
    cfg, wts = _model()
    lens = [40, 17, 63]
    prompts = W.make_prompts(cfg.vocab, 3, lens, 2)
    ctx = B.Context(wts, 3, 128, 4, 20, kv_page_tokens=32, prefill_chunk=32)

    def refused(status, call, *a):
        before = _snapshot(ctx, cfg.n_layers) if ctx.B else None
        with pytest.raises(B.HHError) as ei:
            call(*a)
        assert ei.value.status == status, ei.value
        assert str(ei.value).split(": ", 1)[1]            # a message, not just a code
        if before is not None:
            assert _snapshot(ctx, cfg.n_layers) == before

    # before any prefill
    refused(B.HH_ESTATE, ctx.hh_draft, 2)
    refused(B.HH_ESTATE, ctx.hh_verify)
    refused(B.HH_ESTATE, ctx.hh_commit)
    # capacity: batch, generation budget, sequence length
    refused(B.HH_ECAPACITY, ctx.hh_prefill, W.make_prompts(cfg.vocab, 4, 8, 1), [8] * 4, 8)
    refused(B.HH_ECAPACITY, ctx.hh_prefill, prompts, lens, 21)
    refused(B.HH_ECAPACITY, ctx.hh_prefill, W.make_prompts(cfg.vocab, 1, 110, 1), [110], 20)
    refused(B.HH_EINVAL, ctx.hh_prefill, prompts, [40, 0, 63], 20)
    ctx.hh_prefill(prompts, lens, 20)
    # ready: verify and commit need a draft; k beyond max_draft
    refused(B.HH_ESTATE, ctx.hh_verify)
    refused(B.HH_ESTATE, ctx.hh_commit)
    refused(B.HH_ECAPACITY, ctx.hh_draft, 5)
    refused(B.HH_ECAPACITY, ctx.hh_draft, -1)
    refused(B.HH_ESTATE, ctx.hh_set_drafts, np.zeros((3, 2), np.int32))
    ctx.hh_draft(3)
    # drafted: no second draft, no commit yet
    refused(B.HH_ESTATE, ctx.hh_draft, 3)
    refused(B.HH_ESTATE, ctx.hh_commit)
    ctx.hh_verify()
    # verified: no draft, no second verify, no replaced drafts
    refused(B.HH_ESTATE, ctx.hh_draft, 3)
    refused(B.HH_ESTATE, ctx.hh_verify)
    refused(B.HH_ESTATE, ctx.hh_set_drafts, np.zeros((3, 3), np.int32))
    ctx.hh_commit()
    refused(B.HH_ESTATE, ctx.hh_commit)                  # commit twice
    refused(B.HH_ESTATE, ctx.hh_commit, torch.zeros(3, dtype=torch.int32, device=ctx.device))
    # and the context still works
    ctx.hh_draft(2)
    ctx.hh_verify()
    ctx.hh_commit()
    _, committed, _ = ctx.hh_get_lengths()
    assert all(3 <= c <= 8 for c in committed)


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_bitwise_determinism_eager_and_graphs(B, dtype):
    """Two contexts fed the same inputs, and one context run twice, give identical bits: logits of
    every pass, tokens, lengths, recurrent state and cache.  With HIP graphs on, the replayed
    launch sequences give the same bits as the directly enqueued ones."""
    import torch
    cfg, wts = _model(dtype)
    lens = [70, 9, 33, 51]
    prompts = W.make_prompts(cfg.vocab, 4, lens, 3)
    forced = W.make_forced_pattern(8, 4, 3, 0.6, 4)

    def run(ctx, rounds=6):
        trace = []
        ctx.hh_prefill(prompts, lens, 24)
        trace.append(ctx.hh_get_logits(2).tobytes())
        for r in range(rounds):
            ctx.hh_draft(3)
            trace.append(ctx.hh_get_logits(0).tobytes())
            ctx.hh_verify()
            trace.append(ctx.hh_get_logits(1).tobytes())
            d, g = ctx.hh_get_round()
            trace += [d.tobytes(), g.tobytes()]
            ctx.hh_commit(torch.from_numpy(forced[r]).to(ctx.device) if r % 2 else None)
        return trace + _snapshot(ctx, cfg.n_layers)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        a = B.Context(wts, 4, 160, 3, 24, kv_page_tokens=32, prefill_chunk=32)
        ta = run(a)
        assert run(a) == ta                                # the same context again
        b = B.Context(wts, 4, 160, 3, 24, kv_page_tokens=32, prefill_chunk=32, use_graphs=1)
        assert run(b) == ta                                # first uses are enqueued directly, later ones replayed
        assert run(b) == ta                                # every launch sequence replayed
    stream.synchronize()


@pytest.mark.parametrize("strict", [0, 1])
def test_nothing_is_written_outside_the_workspace(B, strict):
    """The workspace sits between two guard regions filled with a known byte, and (HH_KF_CANARIES)
    every region the library carves from it is followed by 256 guard bytes of its own; after prefill
    (several passes, ragged batch), speculative rounds with every k, replaced drafts, a stochastic
    round, a masked draft and every read-back call all of them still hold that byte - no kernel writes
    past the end of its buffer, into a neighbouring region or outside the workspace.  Also with the
    second recurrent state of the strict draft model."""
    cfg, wts = _model()
    lens = [100, 3, 64, 31, 77]
    prompts = W.make_prompts(cfg.vocab, 5, lens, 6)
    ctx = B.Context(wts, 5, 160, 4, 30, kv_page_tokens=32, prefill_chunk=32, guard_bytes=1 << 20,
                    kernel_flags=B.HH_KF_CANARIES, draft_state_mode=strict)

    def intact():
        return ctx.guards_intact() and ctx.hh_check_canaries() == 0

    assert intact()
    ctx.hh_prefill(prompts, lens, 30)
    assert intact(), B.hh_last_error(ctx.ctx)
    for k in (4, 0, 1, 3, 2):
        ctx.hh_draft(k)
        if k == 3:
            ctx.hh_set_drafts(W.make_random_drafts(cfg.vocab, 1, 5, 3, 2)[0])
        ctx.hh_verify()
        ctx.hh_commit()
        assert intact(), B.hh_last_error(ctx.ctx)
    ctx.hh_set_sampling(0.7, 9)
    ctx.hh_draft(4)
    ctx.hh_verify()
    ctx.hh_commit()
    ctx.hh_set_sampling(0.0, 0)
    if not strict:
        ctx.hh_set_draft_mask(["full", "skip"] + ["ssm"] * (cfg.n_layers - 2))
        ctx.hh_draft(4)
        ctx.hh_verify()
        ctx.hh_commit()
    _snapshot(ctx, cfg.n_layers)
    ctx.hh_get_logits(0), ctx.hh_get_logits(1), ctx.hh_get_logits(2)
    assert intact(), B.hh_last_error(ctx.ctx)
    plain = B.Context(wts, 5, 160, 4, 30)
    with pytest.raises(B.HHError):
        plain.hh_check_canaries()
