"""Lock-step comparison of the HIP library with the CPU oracle on the same seeded inputs."""
from __future__ import annotations

from typing import Optional

import numpy as np

from oracle.hybrid_lm import HybridLM
from oracle.protocol import SpecDecoder, accepted_prefix
from paper_2605_01106_amd import workloads as W


def tolerances(dtype: str):
    """Logit / state tolerances: float32 path 1e-4; bf16-storage path 2e-2 abs + 1e-2 rel."""
    return (1e-4, 1e-4) if dtype == W.F32 else (2e-2, 1e-2)


def assert_close(name, got, ref, atol, rtol, scale_to_ref=False):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    if scale_to_ref:   # states are tiny under the 0.02 init: compare relative to their own size
        s = max(np.abs(ref).max(), 1e-30)
        got, ref = got / s, ref / s
    err = np.abs(got - ref)
    bound = atol + rtol * np.abs(ref)
    bad = err > bound
    if bad.any():
        at = np.unravel_index((err - bound).argmax(), err.shape)
        raise AssertionError(f"{name}: {bad.sum()} of {bad.size} out of tolerance; worst at {at}: got {got[at]!r} "
                             f"ref {ref[at]!r} err {err[at]:.3e} bound {bound[at]:.3e}")
    return float(err.max())


def run_lockstep(ctx, weights: W.Weights, prompts, lens, G: int, k: int, forced: Optional[np.ndarray] = None,
                 override: Optional[np.ndarray] = None, engine: str = "pass", max_rounds: int = 10 ** 9,
                 check_state_every: int = 1, check_kv: bool = True, min_gap: float = 0.0, report=None,
                 layers=None, oracle_rows=None, chunk: int = 5, temperature: float = 0.0, sample_seed: int = 0,
                 min_margin: float = 0.0, compare_logits: bool = True, draft_state: str = "shared", draft_mask=None):
    """Runs prefill and rounds on both sides, comparing after every call:
    tokens, accepted counts, cache lengths and committed counts bit-exactly;
    logits, SSM state, conv window and KV entries within tolerance.
    `layers`: layers whose state and cache are read back (default all).  `oracle_rows`: batch
    rows the oracle runs (default all); the library always runs the whole batch, rows are
    independent, so the remaining rows are covered by the batch-invariance of the kernels.
    `k`: the draft length, or a sequence of draft lengths used round after round (cyclically).
    `temperature` > 0: both sides draw tokens and apply the rejection test with the uniforms of
    `sample_seed`; `min_margin` is the seed audit of those decisions (the analogue of `min_gap`).
    `compare_logits` False: the context keeps no logits (keep_logits = 0); tokens, counts, lengths,
    state and cache are still compared.
    `draft_state` "strict": the context was created with draft_state_mode = 1; the oracle keeps M_S's
    own state, which is compared as well.  `draft_mask`: per-layer "full" | "ssm" | "skip" of the draft
    model, set on both sides.
    Returns a dict of the worst errors seen."""
    import torch
    cfg = weights.cfg
    atol, rtol = tolerances(cfg.w_dtype)
    rows = list(range(len(lens))) if oracle_rows is None else list(oracle_rows)
    B = len(rows)
    layer_list = list(range(cfg.n_layers)) if layers is None else list(layers)
    lm = HybridLM(cfg, weights.values)
    ks = [int(k)] if np.isscalar(k) else [int(v) for v in k]
    cap = int(max(lens)) + G + 2 * max(ks) + 4
    dec = SpecDecoder(lm, cap, engine=engine, chunk=chunk, temperature=temperature, seed=sample_seed,
                      draft_state=draft_state, draft_mask=draft_mask)
    ctx.hh_set_draft_mask(draft_mask)
    plist = [np.asarray(prompts[b][:lens[b]]) for b in rows]
    dec.prefill(plist, G)
    if temperature > 0:
        assert oracle_rows is None, "the uniforms are keyed by the batch row"
    ctx.hh_set_sampling(temperature, sample_seed)
    ctx.hh_prefill(prompts, lens, G)
    worst = {"logits": 0.0, "ssm": 0.0, "conv": 0.0, "kv": 0.0, "ms_ssm": 0.0, "ms_conv": 0.0}
    if compare_logits:
        worst["logits"] = max(worst["logits"], assert_close(
            "prefill logits", ctx.hh_get_logits(2)[rows], np.array(dec.prefill_logits), atol, rtol))

    def check_state(tag):
        kv_len, committed, last_n = ctx.hh_get_lengths()
        kv_len, committed = [kv_len[b] for b in rows], [committed[b] for b in rows]
        assert kv_len == [s.kv_len for s in dec.st], (tag, kv_len, [s.kv_len for s in dec.st])
        assert committed == [len(o) for o in dec.out], (tag, committed)
        for b in range(B):
            assert ctx.hh_get_tokens(rows[b]) == dec.out[b], (tag, b)
        for l in layer_list:
            ssm, conv = ctx.hh_get_state(l)
            ssm, conv = ssm[rows], conv[rows]
            worst["ssm"] = max(worst["ssm"], assert_close(
                f"{tag} ssm L{l}", ssm, np.array([s.S[l] for s in dec.st]), atol, rtol, scale_to_ref=True))
            worst["conv"] = max(worst["conv"], assert_close(
                f"{tag} conv L{l}", conv, np.array([s.conv[l] for s in dec.st]), atol, rtol, scale_to_ref=True))
            if draft_state == "strict":
                ssm, conv = ctx.hh_get_draft_state(l)
                worst["ms_ssm"] = max(worst["ms_ssm"], assert_close(
                    f"{tag} M_S ssm L{l}", ssm[rows], np.array([s.S[l] for s in dec.ms]), atol, rtol, scale_to_ref=True))
                worst["ms_conv"] = max(worst["ms_conv"], assert_close(
                    f"{tag} M_S conv L{l}", conv[rows], np.array([s.conv[l] for s in dec.ms]), atol, rtol, scale_to_ref=True))
            if check_kv:
                for b in range(B):
                    n = dec.st[b].kv_len
                    kk, vv = ctx.hh_get_kv(l, rows[b], n)
                    # float32 evaluation error of the projection, plus one storage ulp for bf16:
                    # rounding a float32 vs a float64 input may pick neighbouring bf16 values
                    # (and such a flip in an earlier layer moves later layers' inputs by ~1e-3 of their scale)
                    bf = cfg.w_dtype == W.BF16
                    ulp = 2.0 ** -7 if bf else 1e-5
                    for nm, got_, ref_ in (("K", kk, dec.st[b].K[l][:n]), ("V", vv, dec.st[b].V[l][:n])):
                        a_ = 2e-3 * max(np.abs(ref_).max(), 1e-30) if bf else 1e-5
                        worst["kv"] = max(worst["kv"], assert_close(f"{tag} {nm} L{l} b{b}", got_, ref_, a_, ulp))

    check_state("prefill")
    r = 0
    n_hist = []
    while not dec.all_finished() and r < max_rounds:
        active = [not dec.finished(b) for b in range(B)]
        ov = None if override is None else override[r]
        k = ks[r % len(ks)]
        dec.draft(k, None if ov is None else ov[rows])
        ctx.hh_draft(k)
        if k > 0:
            gl = ctx.hh_get_logits(0)[rows] if compare_logits else None
            for b in range(B):
                if active[b] and compare_logits:
                    worst["logits"] = max(worst["logits"], assert_close(
                        f"round {r} draft logits b{b}", gl[b], dec.draft_logits[b], atol, rtol))
            if ov is not None:
                ctx.hh_set_drafts(np.ascontiguousarray(ov[:, :k], np.int32))
            d_gpu, _ = ctx.hh_get_round()
            d_gpu = d_gpu[rows]
            for b in range(B):
                if active[b]:
                    assert list(d_gpu[b]) == list(dec.drafts[b]), (r, b, list(d_gpu[b]), dec.drafts[b])
        dec.verify()
        ctx.hh_verify()
        vl = ctx.hh_get_logits(1)[rows] if compare_logits else None
        _, g_gpu = ctx.hh_get_round()
        g_gpu = g_gpu[rows]
        for b in range(B):
            if active[b]:
                if compare_logits:
                    worst["logits"] = max(worst["logits"], assert_close(
                        f"round {r} verify logits b{b}", vl[b], dec.verify_logits[b], atol, rtol))
                # targets up to the first mismatch decide tokens and must agree exactly (their top-2 gaps
                # are audited by min_gap); behind it they are never used: there a near-tie of M_H's logits on
                # junk input may fall either way, and the library's choice only has to be a maximum within
                # the logit tolerance
                if temperature > 0:
                    n_dec = len(dec.targets[b])
                elif forced is not None:
                    n_dec = int(forced[r][rows[b]]) + 1
                else:
                    n_dec = accepted_prefix(dec.drafts[b], dec.targets[b]) + 1
                assert list(g_gpu[b][:n_dec]) == list(dec.targets[b][:n_dec]), (r, b, list(g_gpu[b]), dec.targets[b])
                for j in range(n_dec, len(dec.targets[b])):
                    if int(g_gpu[b][j]) != int(dec.targets[b][j]):
                        row = dec.verify_logits[b][j]
                        top = float(np.max(row))
                        assert 0 <= g_gpu[b][j] < len(row) and row[g_gpu[b][j]] >= top - 2 * (atol + rtol * abs(top)), \
                            (r, b, j, list(g_gpu[b]), dec.targets[b], float(row[g_gpu[b][j]]), top)
        if forced is None:
            dec.commit()
            ctx.hh_commit()
        else:
            dec.commit(forced[r][rows])
            ctx.hh_commit(torch.from_numpy(np.ascontiguousarray(forced[r], np.int32)).to(ctx.device))
        _, _, last_n = ctx.hh_get_lengths()
        last_n = [last_n[b] for b in rows]
        for b in range(B):
            if active[b]:
                assert last_n[b] == dec.last_n[b], (r, b, last_n[b], dec.last_n[b])
        n_hist.append([dec.last_n[b] if active[b] else -1 for b in range(B)])
        if check_state_every and (r % check_state_every == 0 or dec.all_finished()):
            check_state(f"round {r}")
        r += 1
    check_state("end")
    if oracle_rows is None:   # the library counts over the whole batch
        assert ctx.hh_get_acceptance() == (dec.accepted, dec.tested), (ctx.hh_get_acceptance(), dec.accepted, dec.tested)
    if min_gap > 0:
        assert min(dec.gaps) > min_gap, f"seed audit: smallest top-1/top-2 gap {min(dec.gaps):.3e} <= {min_gap}"
    worst["rounds"] = r
    if min_margin > 0:
        assert min(dec.margins) > min_margin, f"seed audit: a random decision was within {min(dec.margins):.3e} of flipping"
    worst["min_gap"] = float(min(dec.gaps)) if dec.gaps else float("inf")
    worst["min_margin"] = float(min(dec.margins)) if dec.margins else float("inf")
    worst["mean_n"] = float(np.mean([n for row in n_hist for n in row if n >= 0])) if n_hist else 0.0
    worst["tokens"] = dec.out
    if report is not None:
        report(worst)
    return worst
