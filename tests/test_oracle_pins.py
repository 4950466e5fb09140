"""Pins of the CPU oracle against things other than itself.

Each test states which mistake it would catch.  All CPU, all tiny.
"""
import json
import os

import numpy as np
import pytest

from oracle import hybrid_lm as H
from oracle import ssd
from oracle.hybrid_lm import HybridLM
from oracle.passes import full_pass
from oracle.protocol import (SpecDecoder, accepted_prefix, expected_tokens_per_round,
                             greedy_generate, speedup_model)
from paper_2605_01106_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_cfg(**kw):
    return W.scaled_config("pin", **kw)


def lively(cfg, seed=1):
    return HybridLM(cfg, W.make_lively_weights(cfg, seed).values)


# ------------------------------------------------------------------ brute force (cache-free)

def brute_force_logits(cfg, vals, tokens, attention=True):
    """Whole-sequence evaluation with no cache and no recurrence: the conv is a
    zero-padded correlation, the SSM output is the fully unrolled sum over
    earlier positions, RoPE is a complex rotation and attention is an explicit
    T x T masked softmax.  Returns logits for every position."""
    g = lambda n: np.asarray(vals[n], np.float64)
    T = len(tokens)
    Hm, P, N = cfg.m_heads, cfg.m_head_dim, cfg.d_state
    di, cd = cfg.d_inner, cfg.conv_dim
    Hq, Hkv, Dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    eps = cfg.rms_eps

    def norm(v, w):
        return v / np.sqrt((v ** 2).mean(-1, keepdims=True) + eps) * w

    def sig(v):
        return 1.0 / (1.0 + np.exp(-v))

    h = g("embed")[np.asarray(tokens)]
    for l in range(cfg.n_layers):
        p = lambda n: g(f"L{l}.{n}")
        u = norm(h, p("norm1"))
        zx = u @ p("w_in").T
        z, raw, dtr = zx[:, :di], zx[:, di:di + cd], zx[:, di + cd:]
        padded = np.vstack([np.zeros((cfg.d_conv - 1, cd)), raw])
        conv = np.stack([(padded[t:t + cfg.d_conv].T * p("conv_w")).sum(1) for t in range(T)]) + p("conv_b")
        xbc = conv * sig(conv)
        x = xbc[:, :di].reshape(T, Hm, P)
        Bm, Cm = xbc[:, di:di + N], xbc[:, di + N:]
        dt = np.log1p(np.exp(dtr + p("dt_bias")))
        loga = -np.exp(p("a_log")) * dt                                # [T][Hm]
        y = np.zeros((T, Hm, P))
        for t in range(T):
            for i in range(t + 1):
                decay = np.exp(loga[i + 1:t + 1].sum(0))               # prod_{i<l<=t} a_l
                y[t] += (decay * dt[i] * (Cm[t] @ Bm[i]))[:, None] * x[i]
            y[t] += p("d_skip")[:, None] * x[t]
        m = norm(y.reshape(T, di) * (z * sig(z)), p("gnorm")) @ p("w_out").T
        att = 0.0
        if attention:
            q = (u @ p("w_q").T).reshape(T, Hq, Dh)
            k = (u @ p("w_k").T).reshape(T, Hkv, Dh)
            v = (u @ p("w_v").T).reshape(T, Hkv, Dh)
            half = Dh // 2
            theta = cfg.rope_base ** (-np.arange(half) * 2.0 / Dh)
            rot = np.exp(1j * np.arange(T)[:, None] * theta[None, :])   # [T][half]

            def rotate(a):
                cplx = (a[..., :half] + 1j * a[..., half:]) * rot[:, None, :]
                return np.concatenate([cplx.real, cplx.imag], -1)
            q, k = rotate(q), rotate(k)
            if cfg.w_dtype == "bf16":
                k = W.bf16_bits_to_f32(W.to_bf16_bits(k.astype(np.float32))).astype(np.float64)
                v = W.bf16_bits_to_f32(W.to_bf16_bits(v.astype(np.float32))).astype(np.float64)
            else:
                k, v = k.astype(np.float32).astype(np.float64), v.astype(np.float32).astype(np.float64)
            o = np.zeros((T, Hq, Dh))
            mask = np.tril(np.ones((T, T), bool))
            for i in range(Hq):
                kv = i * Hkv // Hq
                s = q[:, i] @ k[:, kv].T / np.sqrt(Dh)
                e = np.where(mask, np.exp(s - s.max()), 0.0)
                o[:, i] = (e / e.sum(1, keepdims=True)) @ v[:, kv]
            att = o.reshape(T, Hq * Dh) @ p("w_o").T
        h = h + m + att
        r = norm(h, p("norm2"))
        gate = r @ p("w_gate").T
        h = h + ((gate * sig(gate)) * (r @ p("w_up").T)) @ p("w_down").T
    return norm(h, g("final_norm")) @ g("lm_head").T


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_step_matches_cache_free_brute_force(dtype):
    """Catches any error in the cached single-token path: window order, decay
    indexing, RoPE position or pairing, GQA head mapping, KV slot, residuals."""
    cfg = tiny_cfg(n_layers=2, d_model=24, vocab=40, m_heads=3, m_head_dim=4, d_state=6,
                   n_q_heads=4, n_kv_heads=2, head_dim=6, d_ff=20, w_dtype=dtype)
    wts = W.make_lively_weights(cfg, 3)
    lm = HybridLM(cfg, wts.values)
    toks = W.make_prompts(cfg.vocab, 1, 9, 5)[0]
    ref = brute_force_logits(cfg, wts.values, toks)
    st = lm.new_state(16)
    got = np.array([lm.step(st, int(t), "full") for t in toks])
    assert np.abs(ref).max() > 0.1
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-11)
    assert st.kv_len == len(toks)


def test_draft_is_full_model_with_attention_zeroed():
    """Eq. 4: the draft equals M_H with every attention output set to zero; a
    draft that skipped a norm/MLP or touched the KV cache fails here."""
    cfg = tiny_cfg(n_layers=3)
    wts = W.make_lively_weights(cfg, 4)
    lm = HybridLM(cfg, wts.values)
    zeroed = dict(wts.values)
    for i in range(cfg.n_layers):
        zeroed[f"L{i}.w_o"] = np.zeros_like(wts.values[f"L{i}.w_o"])
    lm0 = HybridLM(cfg, zeroed)
    toks = W.make_prompts(cfg.vocab, 1, 7, 2)[0]
    a, b = lm.new_state(8), lm0.new_state(8)
    for t in toks:
        la = lm.step(a, int(t), "draft")
        lb = lm0.step(b, int(t), "full")
        np.testing.assert_allclose(la, lb, rtol=1e-12, atol=1e-13)
    assert a.kv_len == 0 and all(np.all(k == 0) for k in a.K)
    # ... and also equals the cache-free evaluation without the attention term
    ref = brute_force_logits(cfg, wts.values, toks, attention=False)
    np.testing.assert_allclose(la, ref[-1], rtol=1e-9, atol=1e-11)
    # attention does matter for this model (the test would be vacuous otherwise)
    full = brute_force_logits(cfg, wts.values, toks, attention=True)
    assert np.abs(full[-1] - ref[-1]).max() > 1e-3


# ------------------------------------------------------------------ scan forms

def _scan_inputs(T, Hh=3, P=4, N=5, seed=0):
    r = np.random.default_rng(seed)
    dt = r.uniform(0.05, 1.0, (T, Hh))
    a = np.exp(-r.uniform(0.2, 3.0, Hh)[None, :] * dt)
    x = r.standard_normal((T, Hh, P))
    B = r.standard_normal((T, N))
    C = r.standard_normal((T, N))
    D = r.standard_normal(Hh)
    S0 = r.standard_normal((Hh, P, N))
    return S0, dt, a, x, B, C, D


def test_sequential_scan_matches_unrolled_closed_form():
    """S_t = (prod a) S_0 + sum_i (prod_{l>i} a_l) dt_i x_i B_i^T written out with
    explicit loops; catches an off-by-one in which decays multiply which input."""
    S0, dt, a, x, B, C, D = _scan_inputs(6)
    y, states = ssd.scan_sequential(S0, dt, a, x, B, C, D)
    for t in range(6):
        S = S0 * np.prod(a[:t + 1], axis=0)[:, None, None]
        for i in range(t + 1):
            S = S + (np.prod(a[i + 1:t + 1], axis=0) * dt[i])[:, None, None] * np.einsum("hp,n->hpn", x[i], B[i])
        np.testing.assert_allclose(states[t], S, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(y[t], np.einsum("hpn,n->hp", S, C[t]) + D[:, None] * x[t], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("T,chunk", [(1, 1), (5, 1), (9, 4), (16, 4), (23, 8), (7, 64)])
def test_chunked_scan_equals_sequential(T, chunk):
    """Any chunk size, ragged last chunk included, same y and same final state."""
    S0, dt, a, x, B, C, D = _scan_inputs(T, seed=T)
    y_seq, states = ssd.scan_sequential(S0, dt, a, x, B, C, D)
    y_ch, S_end = ssd.scan_chunked(S0, dt, a, x, B, C, D, chunk)
    np.testing.assert_allclose(y_ch, y_seq, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(S_end, states[-1], rtol=1e-11, atol=1e-12)
    for j, Sj in enumerate(ssd.prefix_states(S0, dt, a, x, B)):
        np.testing.assert_allclose(Sj, states[j], rtol=1e-11, atol=1e-12)


def test_scan_reduces_to_prefix_sum():
    """a = 1, dt = 1: the state is the running sum of x (outer) B."""
    S0, dt, a, x, B, C, D = _scan_inputs(8)
    one = np.ones_like(dt)
    _, states = ssd.scan_sequential(np.zeros_like(S0), one, one, x, B, C, D)
    run = np.cumsum(np.einsum("thp,tn->thpn", x, B), axis=0)
    for t in range(8):
        np.testing.assert_allclose(states[t], run[t], rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ model-level special cases

def test_step_reduces_to_prefix_sum_and_identity_conv():
    """A_log -> -inf (no decay), dt = 1, conv taps (0,0,0,1), bias 0: then
    xBC = silu(raw input) and S after t tokens is the plain sum of x B^T."""
    cfg = tiny_cfg(n_layers=1)
    wts = W.make_lively_weights(cfg, 8)
    v = dict(wts.values)
    v["L0.a_log"] = np.full(cfg.m_heads, -800.0)
    w_in = v["L0.w_in"].copy()
    w_in[cfg.d_inner + cfg.conv_dim:] = 0.0                # dt_raw = 0
    v["L0.w_in"] = w_in
    v["L0.dt_bias"] = np.full(cfg.m_heads, np.log(np.e - 1.0))   # softplus = 1
    taps = np.zeros((cfg.conv_dim, cfg.d_conv)); taps[:, -1] = 1.0
    v["L0.conv_w"] = taps
    v["L0.conv_b"] = np.zeros(cfg.conv_dim)
    lm = HybridLM(cfg, v)
    st = lm.new_state(8)
    toks = [3, 17, 5, 90]
    acc = np.zeros((cfg.m_heads, cfg.m_head_dim, cfg.d_state))
    # one layer: the stream entering it is always the token embedding
    for t in toks:
        u = H.rmsnorm(np.asarray(v["embed"], np.float64)[t], np.asarray(v["L0.norm1"], np.float64), cfg.rms_eps)
        raw = (np.asarray(v["L0.w_in"], np.float64) @ u)[cfg.d_inner:cfg.d_inner + cfg.conv_dim]
        act = raw / (1 + np.exp(-raw))
        acc += np.einsum("hp,n->hpn", act[:cfg.d_inner].reshape(cfg.m_heads, cfg.m_head_dim),
                         act[cfg.d_inner:cfg.d_inner + cfg.d_state])
        lm.step(st, t, "draft")
        np.testing.assert_allclose(st.S[0], acc, rtol=1e-10, atol=1e-12)
    assert np.abs(acc).max() > 1e-2


def test_single_key_attention_returns_value():
    """At position 0 there is one key, so softmax = 1 and the attention branch is
    W_o applied to the stored V, repeated over the query heads of each group.
    One layer, MLP switched off, so the pre-head stream is h + m + att."""
    cfg = tiny_cfg(n_layers=1, n_q_heads=4, n_kv_heads=2)
    v = dict(W.make_lively_weights(cfg, 9).values)
    v["L0.w_down"] = np.zeros_like(v["L0.w_down"])
    lm = HybridLM(cfg, v)
    tok = 11
    f64 = lambda n: np.asarray(v[n], np.float64)
    u = H.rmsnorm(f64("embed")[tok], f64("L0.norm1"), cfg.rms_eps)
    vv = (f64("L0.w_v") @ u).astype(np.float32).astype(np.float64).reshape(cfg.n_kv_heads, cfg.head_dim)
    o = np.repeat(vv, cfg.n_q_heads // cfg.n_kv_heads, axis=0).reshape(-1)
    att = f64("L0.w_o") @ o
    st = lm.new_state(4)
    lf = lm.step(st, tok, "full")
    np.testing.assert_array_equal(st.V[0][0], vv)
    hd = _pre_head_stream(lm, tok)
    expect = f64("lm_head") @ H.rmsnorm(hd + att, f64("final_norm"), cfg.rms_eps)
    np.testing.assert_allclose(lf, expect, rtol=1e-10, atol=1e-12)
    assert np.abs(att).max() > 1e-2


def _pre_head_stream(lm, tok):
    """h + m before the final norm for the first token of a one-layer, MLP-off
    model, written by hand (empty conv history, S_0 = 0 so S = dt x B^T)."""
    c = lm.cfg
    w = lm.layers[0]
    h = lm.embed[tok].copy()
    u = H.rmsnorm(h, w["norm1"], c.rms_eps)
    zx = w["w_in"] @ u
    di, cd = c.m_heads * c.m_head_dim, c.m_heads * c.m_head_dim + 2 * c.d_state
    z, raw, dtr = zx[:di], zx[di:di + cd], zx[di + cd:]
    conv = w["conv_b"] + w["conv_w"][:, -1] * raw                     # empty history
    xbc = conv / (1 + np.exp(-conv))
    x = xbc[:di].reshape(c.m_heads, c.m_head_dim)
    Bv, Cv = xbc[di:di + c.d_state], xbc[di + c.d_state:]
    dt = np.log1p(np.exp(dtr + w["dt_bias"]))
    y = (dt[:, None] * x) * (Bv @ Cv) + w["d_skip"][:, None] * x      # S_0 = 0 => S = dt x B^T
    gated = y.reshape(-1) * (z / (1 + np.exp(-z)))
    return h + w["w_out"] @ H.rmsnorm(gated, w["gnorm"], c.rms_eps)


def test_rope_invariances():
    """Position 0 is the identity; rotation preserves norms; <rope(q,m), rope(k,n)>
    depends on m - n only; pairs are (i, i + Dh/2)."""
    r = np.random.default_rng(0)
    q, k = r.standard_normal(16), r.standard_normal(16)
    np.testing.assert_allclose(H.rope(q, 0, 1e4), q, atol=0)
    np.testing.assert_allclose(np.linalg.norm(H.rope(q, 1234, 1e4)), np.linalg.norm(q), rtol=1e-12)
    d1 = H.rope(q, 40, 1e4) @ H.rope(k, 33, 1e4)
    d2 = H.rope(q, 1007, 1e4) @ H.rope(k, 1000, 1e4)
    np.testing.assert_allclose(d1, d2, rtol=1e-9)
    e = np.zeros(16); e[3] = 1.0
    out = H.rope(e, 5, 1e4)
    ang = 5 * 1e4 ** (-2 * 3 / 16)
    assert np.flatnonzero(np.abs(out) > 1e-15).tolist() == [3, 11]
    np.testing.assert_allclose(out[[3, 11]], [np.cos(ang), np.sin(ang)], rtol=1e-12)


def test_elementary_maps():
    x = np.linspace(-30, 30, 13)
    np.testing.assert_allclose(H.softplus(x), np.logaddexp(0, x), rtol=1e-12)
    np.testing.assert_allclose(H.silu(x), x * 0.5 * (1 + np.tanh(x / 2)), rtol=1e-12, atol=1e-15)
    v = np.random.default_rng(1).standard_normal((3, 50))
    out = H.rmsnorm(v, np.ones(50), 0.0)
    np.testing.assert_allclose(np.sqrt((out ** 2).mean(-1)), 1.0, rtol=1e-12)
    assert H.argmax_lowest(np.array([1.0, 3.0, 3.0, 2.0])) == 1
    with pytest.raises(FloatingPointError):
        H.argmax_lowest(np.array([1.0, np.nan]))
    # bf16 storage rounding: nearest, ties to even, decided from the float32 value
    vals = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -3.14159])
    got = H.round_storage(vals, "bf16")
    np.testing.assert_array_equal(got[:4], [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7])
    assert abs(got[4] + 3.14159) < 2 ** -7 and got[4] == np.float64(np.float32(got[4]))


# ------------------------------------------------------------------ passes and protocol

@pytest.mark.parametrize("dtype,chunk", [("f32", 3), ("bf16", 64)])
def test_multi_position_pass_equals_single_steps(dtype, chunk):
    """Section 3.3 verification: one pass over T positions gives the same
    distributions, KV entries and per-position recurrent snapshots as T steps."""
    cfg = tiny_cfg(n_layers=2, n_q_heads=4, n_kv_heads=2, w_dtype=dtype)
    lm = lively(cfg, 5)
    toks = W.make_prompts(cfg.vocab, 1, 13, 7)[0]
    a, b = lm.new_state(20), lm.new_state(20)
    for t in toks[:4]:
        lm.step(a, int(t), "full")
    full_pass(lm, b, toks[:4], chunk)
    ref, snaps = [], []
    for t in toks[4:]:
        ref.append(lm.step(a, int(t), "full"))
        snaps.append(a.recurrent_copy())
    got, ck = full_pass(lm, b, toks[4:], chunk, checkpoints=True)
    np.testing.assert_allclose(got, np.array(ref), rtol=1e-9, atol=1e-11)
    for l in range(cfg.n_layers):
        np.testing.assert_allclose(b.K[l], a.K[l], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(b.V[l], a.V[l], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(b.S[l], a.S[l], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(b.conv[l], a.conv[l], rtol=1e-9, atol=1e-12)
        for j in range(len(ref)):
            np.testing.assert_allclose(ck[j][0][l], snaps[j][0][l], rtol=1e-9, atol=1e-12)
            np.testing.assert_allclose(ck[j][1][l], snaps[j][1][l], rtol=1e-9, atol=1e-12)
    assert a.kv_len == b.kv_len == 13


def test_accepted_prefix_rule():
    assert accepted_prefix([5, 6, 7], [5, 6, 7, 9]) == 3
    assert accepted_prefix([5, 6, 7], [5, 9, 7, 1]) == 1      # a later match after a mismatch does not count
    assert accepted_prefix([5], [4, 5]) == 0
    assert accepted_prefix([], [4]) == 0


@pytest.mark.parametrize("source", ["ssm", "random", "right", "wrong"])
@pytest.mark.parametrize("k", [1, 3])
@pytest.mark.parametrize("engine", ["step", "pass"])
def test_speculative_stream_equals_plain_greedy(source, k, engine):
    """Losslessness (Section 3.3): for any draft source the committed tokens are
    plain greedy decoding of M_H.  Also checks, after every commit, that the
    recurrent state, conv window, KV prefix and cache length equal those of a
    model that simply consumed the committed tokens."""
    cfg = tiny_cfg(n_layers=2)
    lm = lively(cfg, 6)
    G = 14
    prompt = W.make_prompts(cfg.vocab, 1, 6, 11)[0]
    ref = greedy_generate(lm, prompt, G)
    rounds = G + 2
    override = None
    if source == "random":
        override = W.make_random_drafts(cfg.vocab, rounds, 1, k, 3)
    dec = SpecDecoder(lm, capacity=64, engine=engine, chunk=2)
    dec.prefill([prompt], G)
    shadow = lm.new_state(64)
    for t in prompt:
        lm.step(shadow, int(t), "full")
    consumed = 0
    r = 0
    while not dec.all_finished():
        ov = None
        have = len(dec.out[0])
        if source == "right":     # the true continuation
            nxt = greedy_generate(lm, list(prompt) + dec.out[0], k) if True else None
            ov = np.array([nxt])
        elif source == "wrong":
            nxt = greedy_generate(lm, list(prompt) + dec.out[0], 1)
            ov = np.array([[(nxt[0] + 1) % cfg.vocab] * k])
        elif source == "random":
            ov = override[r]
        dec.draft(k, ov)
        dec.verify()
        dec.commit()
        n = dec.last_n[0]
        if source == "right":
            assert n == k
        if source == "wrong":
            assert n == 0
        stream = list(prompt) + dec.out[0]
        # state must equal that of plain consumption of everything but the pending token
        upto = len(prompt) + have + n
        full_stream = list(prompt) + (ref + greedy_generate(lm, prompt, G + k + 2)[G:])
        while consumed < have + n:
            lm.step(shadow, int(full_stream[len(prompt) + consumed]), "full")
            consumed += 1
        assert dec.st[0].kv_len == shadow.kv_len == upto
        for l in range(cfg.n_layers):
            np.testing.assert_allclose(dec.st[0].S[l], shadow.S[l], rtol=1e-9, atol=1e-12)
            np.testing.assert_allclose(dec.st[0].conv[l], shadow.conv[l], rtol=1e-9, atol=1e-12)
            np.testing.assert_allclose(dec.st[0].K[l][:upto], shadow.K[l][:upto], rtol=1e-9, atol=1e-12)
        r += 1
    assert dec.out[0] == ref
    assert min(dec.gaps) > 1e-7       # decisions were not coin flips


def test_engines_agree_and_batch_rows_are_independent():
    cfg = tiny_cfg(n_layers=2)
    lm = lively(cfg, 12)
    prompts = W.make_prompts(cfg.vocab, 3, [5, 9, 2], 4)
    plist = [prompts[0][:5], prompts[1][:9], prompts[2][:2]]
    a = SpecDecoder(lm, 64, "step")
    b = SpecDecoder(lm, 64, "pass", chunk=4)
    out_a = a.run(plist, 10, 2)
    out_b = b.run(plist, 10, 2)
    assert out_a == out_b and a.n_hist == b.n_hist
    solo = SpecDecoder(lm, 64, "step").run([plist[1]], 10, 2)
    assert solo[0] == out_a[1]
    for p, o in zip(plist, out_a):
        assert o == greedy_generate(lm, p, 10)


def test_forced_acceptance_commits_drafts_as_given():
    """Forced counts: d_1..d_n are committed as drafted, then M_H's token g_n;
    state and cache stay consistent because verification consumed exactly those
    tokens: the next round's pending token continues from them."""
    cfg = tiny_cfg(n_layers=2)
    lm = lively(cfg, 13)
    prompt = W.make_prompts(cfg.vocab, 1, 5, 1)[0]
    k, G = 3, 16
    forced = W.make_forced_pattern(40, 1, k, 0.6, 2)
    dec = SpecDecoder(lm, 128, "step")
    out = dec.run([prompt], G, k, forced=forced)[0]
    assert len(out) == G
    # replay: every committed token after a forced run must be either the draft of its
    # round or M_H's greedy token given everything before it
    st = lm.new_state(128)
    for t in prompt:
        logits = lm.step(st, int(t), "full")
    pos, r = 0, 0
    assert out[0] == int(np.argmax(logits))
    pos = 1
    while pos < G:
        n = int(forced[r][0])
        # the n drafted tokens are taken as given; consume pending + n drafts
        for i in range(n + 1):
            if pos - 1 + i >= G:
                break
            logits = lm.step(st, int(out[pos - 1 + i]), "full")
        if pos + n < G:
            assert out[pos + n] == int(np.argmax(logits))
        pos += n + 1
        r += 1
    assert dec.n_hist[:r] == [[int(x)] for x in forced[:r, 0]]


# ------------------------------------------------------------------ Eq. 1 and bookkeeping

def test_eq1_and_paper_worked_example():
    with open(os.path.join(GOLDEN, "paper_values.json")) as f:
        gold = json.load(f)
    ex = gold["section_5_5_worked_example"]
    alpha, c, k = ex["alpha_k2"], ex["cost_ratio"], ex["k"]
    # closed form == explicit geometric sum
    for a in (0.0, 0.186, 0.37, 0.68, 0.999):
        for kk in (1, 2, 4, 8):
            assert abs(expected_tokens_per_round(a, kk) - sum(a ** i for i in range(kk + 1))) < 1e-12
    assert expected_tokens_per_round(1.0, 4) == 5.0
    # Eq. 1 evaluated literally with the printed inputs
    assert abs(speedup_model(alpha, k, c) - 0.8343) < 5e-4
    # the value the paper prints is reproduced by (1 + k*alpha(k)) / (1 + k*c): the
    # all-token rate plugged into a linear numerator (documented as a garbled passage)
    assert abs((1 + k * alpha) / (1 + k * c) - ex["printed_speedup"]) < 5e-3
    assert abs(ex["printed_speedup"] / ex["wallclock_speedup"] - ex["printed_gap"]) < 0.05


@pytest.mark.parametrize("p,k", [(0.37, 4), (0.68, 8), (0.68, 2)])
def test_forced_pattern_matches_eq1_numerator(p, k):
    n = W.make_forced_pattern(20000, 4, k, p, 0)
    assert n.min() >= 0 and n.max() <= k
    mean = (n + 1).mean()
    assert abs(mean - expected_tokens_per_round(p, k)) < 0.03
    for j in range(k):
        assert abs((n == j).mean() - p ** j * (1 - p)) < 0.01


def test_parameter_count_ratio():
    """Section 3.4 estimates the draft cost by parameter counting (78.4 % for the
    real 0.5B model).  The tiny workload's shapes give 0.7886 by the same count."""
    c0 = W.WORKLOADS["c0"].cfg
    ratio = c0.step_params(draft=True) / c0.step_params(draft=False)
    assert c0.total_params() == 2122352
    assert abs(ratio - 0.7886) < 2e-3
    assert c0.params_per_layer(True) == 602296 and c0.params_per_layer(False) == 798904
    c1 = W.WORKLOADS["c1"].cfg
    assert c1.params_per_layer(True) == 17600840 and c1.params_per_layer(False) == 18911560
    c3 = W.WORKLOADS["c3"].cfg
    assert c3.params_per_layer(True) == 74181240 and c3.params_per_layer(False) == 82045560


# ------------------------------------------------------------------ masked drafts, strict draft state, draft length

def test_layer_modes_reduce_to_the_full_model_the_ssm_draft_and_a_layerless_model():
    """Per-layer draft modes (Eq. 4 / Eq. 5 generalised): all "full" is the full step bit for bit
    (logits, state, K/V), all "ssm" the Eq. 4 draft step, all "skip" leaves nothing but the
    embedding, the final norm and the LM head (written out by hand here), and a single skipped
    layer is the model whose output, attention-output and down projections of that layer are zero
    (the block then adds nothing to the stream)."""
    cfg = tiny_cfg(n_layers=3)
    wts = W.make_lively_weights(cfg, 4)
    lm = HybridLM(cfg, wts.values)
    toks = [3, 9, 1, 4, 7]
    a, b = lm.new_state(16), lm.new_state(16)
    for t in toks:
        la = lm.step(a, t, "full")
        lb = lm.step(b, t, ["full"] * 3)
        assert np.array_equal(la, lb)
    assert a.kv_len == b.kv_len == 5
    for l in range(3):
        assert np.array_equal(a.S[l], b.S[l]) and np.array_equal(a.K[l], b.K[l]) and np.array_equal(a.V[l], b.V[l])
    c, d = lm.new_state(16), lm.new_state(16)
    for t in toks:
        assert np.array_equal(lm.step(c, t, "draft"), lm.step(d, t, ["ssm"] * 3))
    assert c.kv_len == 0 and d.kv_len == 5 and not d.K[0].any()          # the SSM-only layers write no K/V
    e = lm.new_state(16)
    got = lm.step(e, 6, ["skip"] * 3)
    x = np.asarray(wts.values["embed"], np.float64)[6]
    want = np.asarray(wts.values["lm_head"], np.float64) @ (x / np.sqrt((x * x).mean() + cfg.rms_eps) * wts.values["final_norm"])
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-15)
    assert not any(s.any() for s in e.S)                                  # skipped layers keep their state
    # one skipped layer == that layer's three output projections zeroed
    vals = dict(wts.values)
    for n in ("w_out", "w_o", "w_down"):
        vals[f"L1.{n}"] = np.zeros_like(vals[f"L1.{n}"])
    lm0 = HybridLM(cfg, vals)
    f, g = lm.new_state(16), lm0.new_state(16)
    for t in toks:
        np.testing.assert_allclose(lm.step(f, t, ["full", "skip", "ssm"]), lm0.step(g, t, ["full", "full", "ssm"]),
                                   rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("mask", [("full", "full"), ("ssm", "skip"), ("skip", "full"), ("full", "ssm")])
@pytest.mark.parametrize("k", [1, 3])
def test_masked_drafts_are_lossless_and_the_full_mask_is_always_accepted(mask, k):
    """Losslessness does not depend on the draft (Section 3.3), so it holds for every layer
    mask; the all-"full" mask drafts with M_H itself and has all k drafts accepted every round.
    After every commit the committed state equals plain consumption (a masked draft writes K/V
    only into dead slots)."""
    cfg = tiny_cfg(n_layers=2)
    lm = lively(cfg, 6)
    G = 12
    prompt = W.make_prompts(cfg.vocab, 1, 6, 11)[0]
    ref = greedy_generate(lm, prompt, G + k + 2)
    dec = SpecDecoder(lm, capacity=64, engine="step", draft_mask=mask)
    dec.prefill([prompt], G)
    while not dec.all_finished():
        have = len(dec.out[0])
        dec.draft(k)
        dec.verify()
        dec.commit()
        if mask == ("full", "full"):
            assert dec.last_n[0] == k
        shadow = lm.new_state(64)
        for t in list(prompt) + ref[:have + dec.last_n[0]]:
            lm.step(shadow, int(t), "full")
        assert dec.st[0].kv_len == shadow.kv_len
        for l in range(cfg.n_layers):
            np.testing.assert_allclose(dec.st[0].S[l], shadow.S[l], rtol=1e-9, atol=1e-12)
            np.testing.assert_allclose(dec.st[0].K[l][:shadow.kv_len], shadow.K[l][:shadow.kv_len], rtol=1e-9, atol=1e-12)
    assert dec.out[0] == ref[:G]


def test_strict_draft_state_is_m_s_over_the_whole_prefix():
    """Strict reading of Eq. 4 / Section 3.3 "Draft phase": the draft model's own recurrent state
    equals M_S run from scratch over the prompt and every token the caches have consumed; the
    committed stream is still plain greedy decoding; and when the attention output projection is
    zero (M_H == M_S) the strict and the shared state coincide, every draft is accepted, in both."""
    cfg = tiny_cfg(n_layers=2)
    lm = lively(cfg, 6)
    G, k = 12, 3
    prompt = W.make_prompts(cfg.vocab, 1, 7, 5)[0]
    ref = greedy_generate(lm, prompt, G)
    dec = SpecDecoder(lm, 64, engine="step", draft_state="strict")
    dec.prefill([prompt], G)
    shared = SpecDecoder(lm, 64, engine="step")
    shared.prefill([prompt], G)
    n_strict, n_shared = [], []
    while not dec.all_finished():
        consumed_before = list(prompt) + dec.out[0][:-1]
        dec.draft(k); dec.verify(); dec.commit()
        n_strict.append(dec.last_n[0])
        brute = lm.new_state(1)
        for t in list(prompt) + dec.out[0][:-1]:                         # everything but the pending token
            lm.step(brute, int(t), "draft")
        assert len(dec.out[0]) - 1 - (len(consumed_before) - len(prompt)) == dec.last_n[0] + 1 or dec.finished(0)
        if not dec.finished(0) or len(dec.out[0]) == G:
            for l in range(cfg.n_layers):
                np.testing.assert_allclose(dec.ms[0].S[l], brute.S[l], rtol=1e-10, atol=1e-13)
                np.testing.assert_allclose(dec.ms[0].conv[l], brute.conv[l], rtol=1e-10, atol=1e-13)
    while not shared.all_finished():
        shared.draft(k); shared.verify(); shared.commit()
        n_shared.append(shared.last_n[0])
    assert dec.out[0] == ref == shared.out[0]
    assert n_strict != n_shared                                            # the two readings differ in what they accept
    # M_H == M_S: zero attention output projection
    vals = dict(W.make_lively_weights(cfg, 6).values)
    for l in range(cfg.n_layers):
        vals[f"L{l}.w_o"] = np.zeros_like(vals[f"L{l}.w_o"])
    lm0 = HybridLM(cfg, vals)
    for mode in ("strict", "shared"):
        d0 = SpecDecoder(lm0, 64, engine="step", draft_state=mode)
        d0.prefill([prompt], G)
        while not d0.all_finished():
            d0.draft(k); d0.verify(); d0.commit()
            assert d0.last_n[0] == k
        assert d0.out[0] == greedy_generate(lm0, prompt, G)


def test_optimal_draft_length_follows_eq1():
    """The draft length that maximises Eq. 1: brute force over the candidates; the paper's own
    conclusion (Section 7: k* = 2 among the evaluated lengths at the high cost ratios, for both
    readings of the printed acceptance rate); and its remark that a lower effective cost ratio
    makes larger k optimal (k* never shrinks as the ratio falls)."""
    from oracle.protocol import optimal_draft_length, speedup_model
    golden = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))
    c = golden["section_3_4_cost_ratio_falcon_h1_0p5b"]
    for alpha_k2 in (golden["table_3_alpha_greedy"]["falcon_h1_0p5b"]["k2"], golden["table_3_alpha_greedy"]["falcon_h1_3b"]["k2"]):
        for alpha in (alpha_k2, alpha_k2 ** 0.5):                        # per-token reading, and the all-token rate's root
            assert optimal_draft_length(alpha, c, [2, 4, 8]) == 2
    for alpha in (0.3, 0.68, 0.9, 0.97):
        prev = 0
        for ratio in (1.0, 0.784, 0.5, 0.2, 0.05, 0.01):
            ks = list(range(1, 17))
            best = optimal_draft_length(alpha, ratio, ks)
            assert all(speedup_model(alpha, best, ratio) >= speedup_model(alpha, k, ratio) - 1e-12 for k in ks)
            assert best >= prev
            prev = best
    assert optimal_draft_length(0.9, 0.05, range(1, 17)) > 2
    assert optimal_draft_length(0.0, 0.5, [1, 2, 3]) == 1                # nothing is ever accepted: shortest draft


def test_acceptance_counts_estimate_alpha():
    """The acceptance statistics behind the choice of k (Eq. 1's alpha, Section 7): by hand on a few
    rounds; with k = 1 it is the plain success rate; and on simulated rounds in which every test passes
    independently with probability alpha (the model of Eq. 1) accepted / tested recovers alpha although
    the rounds are cut off at k - unlike the naive mean(n) / k."""
    from oracle.protocol import acceptance_counts
    assert acceptance_counts([0, 2, 3, 1], 3) == (6, 1 + 3 + 3 + 2)
    assert acceptance_counts([1, 0, 1, 1], 1) == (3, 4)
    assert acceptance_counts([0, 0], 0) == (0, 0)
    rng = np.random.default_rng(5)
    for alpha in (0.37, 0.68, 0.9):
        for k in (2, 8):
            ns = []
            for _ in range(20000):
                n = 0
                while n < k and rng.random() < alpha:
                    n += 1
                ns.append(n)
            acc, tested = acceptance_counts(ns, k)
            assert abs(acc / tested - alpha) < 0.01, (alpha, k, acc / tested)
            # mean tokens per round matches Eq. 1's numerator
            assert abs(np.mean(ns) + 1 - expected_tokens_per_round(alpha, k)) < 0.05
    assert abs(np.mean(ns) / 8 - 0.9) > 0.15            # the naive estimate is biased by the cut-off
