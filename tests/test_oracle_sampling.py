"""Pins of the oracle's stochastic acceptance (Section 3.3, Eq. 6) against things other than itself.

Each test states which mistake it would catch.  All CPU, all tiny.
"""
import itertools

import numpy as np
import pytest

from oracle import sampling as S
from oracle.hybrid_lm import HybridLM
from oracle.protocol import SpecDecoder, greedy_generate
from paper_2605_01106_amd import workloads as W


def test_splitmix64_published_sequence():
    """The first outputs of SplitMix64 for seed 1234567 as printed with the published
    reference implementation (wrong constants, shifts or increment order fail)."""
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423, 4593380528125082431,
            16408922859458223821]
    assert [S.splitmix64_at(1234567, i) for i in range(5)] == want


def test_uniform_is_24_bit_and_keyed():
    us = [S.uniform(3, b, i, p) for b in range(3) for i in range(50) for p in range(3)]
    assert all(0.0 <= u < 1.0 and (u * 2 ** 24) == int(u * 2 ** 24) for u in us)
    assert len(set(us)) == len(us)                       # sequence, position and purpose all enter the key
    assert abs(np.mean(us) - 0.5) < 0.05
    assert S.uniform(3, 1, 2, 0) != S.uniform(4, 1, 2, 0)


def test_draw_is_the_inverse_cdf():
    """On a regular grid of uniforms the counts reproduce p to one grid cell (an
    off-by-one in the edge search or a reversed comparison fails); zero-mass
    entries are never drawn; u = 0 returns the first entry with mass."""
    p = np.array([0.0, 0.125, 0.25, 0.0, 0.5, 0.125])
    n = 4096
    counts = np.zeros(len(p), int)
    for j in range(n):
        counts[S.draw(p, j / n)[0]] += 1
    assert list(counts) == [0, 512, 1024, 0, 2048, 512]
    assert S.draw(p, 0.0)[0] == 1
    assert S.draw(3.0 * p, 0.124)[0] == 1 and S.draw(3.0 * p, 0.126)[0] == 2     # scale-free
    i, m = S.draw(p, 0.130)
    assert i == 2 and abs(m - 0.005) < 1e-12


def test_softmax_temperature():
    l = np.array([0.3, -1.2, 2.0, 0.0])
    p = S.softmax_t(l, 0.6)
    np.testing.assert_allclose(p.sum(), 1.0, rtol=1e-14)
    np.testing.assert_allclose(np.log(p[2] / p[1]), (2.0 + 1.2) / 0.6, rtol=1e-12)
    np.testing.assert_allclose(S.softmax_t(l + 7.0, 0.6), p, rtol=1e-12)            # shift invariance
    assert S.softmax_t(l, 1e-3)[2] > 1 - 1e-12                                      # T -> 0 is the argmax


def _exact_output_distribution(p_s, p_h):
    """Eq. 6 integrated by hand for one position: draft d with probability p_s[d], kept with
    probability min(1, p_h/p_s), else replaced by a draw from norm(max(0, p_h - p_s))."""
    keep = np.minimum(p_s, p_h)
    res = np.maximum(0.0, p_h - p_s)
    rej = 1.0 - keep.sum()
    return keep + (rej * res / res.sum() if rej > 0 else 0.0)


def test_one_position_rule_returns_p_h_in_closed_form():
    """The algebra the paper relies on (min + residual = P_H), so that the Monte Carlo
    test below checks the code and not the rule."""
    rng = np.random.default_rng(0)
    for _ in range(20):
        p_s, p_h = rng.dirichlet(np.ones(7)), rng.dirichlet(np.ones(7))
        np.testing.assert_allclose(_exact_output_distribution(p_s, p_h), p_h, atol=1e-14)


@pytest.mark.parametrize("case", [0, 1, 2])
def test_committed_token_follows_p_h(case):
    """Losslessness of Eq. 6 on the oracle's own functions, by integrating over a
    regular grid of the three uniforms (draft, test, correction): the first emitted
    token has distribution P_H and the keep probability is sum(min(P_S, P_H)).  A
    swapped ratio, a residual with the wrong sign, or a missing renormalisation fail."""
    rng = np.random.default_rng(10 + case)
    V = 5
    p_s, p_h = rng.dirichlet(np.ones(V) * 0.7), rng.dirichlet(np.ones(V) * 0.7)
    if case == 2:
        p_s[1] = 0.0                                  # a token the draft never proposes
        p_s /= p_s.sum()
    n = 48
    grid = (np.arange(n) + 0.5) / n
    counts = np.zeros(V)
    kept = 0
    for u_d in grid:
        d, _ = S.draw(p_s, u_d)
        for u_a, u_c in itertools.product(grid, grid):
            k_, tok, _ = S.stochastic_round([p_s], [p_h, p_h], [d], [u_a], lambda n_: u_c)
            first = d if k_ == 1 else tok
            counts[first] += 1
            kept += k_
    total = n ** 3
    np.testing.assert_allclose(counts / total, p_h, atol=2.5 / n)
    np.testing.assert_allclose(kept / total, np.minimum(p_s, p_h).sum(), atol=2.5 / n)


def test_identical_distributions_keep_everything_and_disjoint_keep_nothing():
    rng = np.random.default_rng(3)
    p = [rng.dirichlet(np.ones(6)) for _ in range(4)]
    for trial in range(50):
        us = [S.uniform(trial, 0, i, 1) for i in range(3)]
        d = [S.draw(p[i], S.uniform(trial, 0, i, 0))[0] for i in range(3)]
        n, tok, _ = S.stochastic_round(p[:3], p, d, us, lambda n_: 0.5)
        assert n == 3 and tok == S.draw(p[3], 0.5)[0]              # bonus token from P_H at position k+1
    p_s = np.array([0.5, 0.5, 0.0, 0.0])
    p_h = np.array([0.0, 0.0, 0.25, 0.75])
    n, tok, _ = S.stochastic_round([p_s], [p_h, p_h], [1], [0.0], lambda n_: 0.3)
    assert n == 0 and tok == 3
    assert S.stochastic_targets([4, 9, 2], 1, 7) == [4, 7, -1, -1]


def _tiny():
    cfg = W.scaled_config("pin", n_layers=2)
    return cfg, HybridLM(cfg, W.make_lively_weights(cfg, 6).values)


def test_low_temperature_stream_is_greedy():
    """T -> 0 reduces Eq. 6 to the greedy rule of Section 3.3: the committed stream equals
    plain greedy decoding."""
    cfg, lm = _tiny()
    prompt = W.make_prompts(cfg.vocab, 1, 6, 11)[0]
    ref = greedy_generate(lm, prompt, 12)
    dec = SpecDecoder(lm, capacity=64, engine="step", temperature=1e-4, seed=5)
    assert dec.run([prompt], 12, 3)[0] == ref


def test_plain_sampling_is_the_k0_case_and_state_follows_the_committed_stream():
    """With k = 0 every token is the purpose-2 draw at its stream position from the full model's
    distribution (recomputed here with single steps).  With k = 3 some drafts are kept and some
    rejected, and after the commits the caches equal plain consumption of the committed stream."""
    cfg, lm = _tiny()
    prompt = W.make_prompts(cfg.vocab, 1, 6, 11)[0]
    T, seed, G = 0.8, 11, 10
    plain = SpecDecoder(lm, capacity=64, engine="step", temperature=T, seed=seed)
    out0 = plain.run([prompt], G, 0)[0]
    st = lm.new_state(64)
    for t in prompt:
        logits = lm.step(st, int(t), "full")
    want = []
    for i in range(G):
        tok = S.draw(S.softmax_t(logits, T), S.uniform(seed, 0, i, S.PURPOSE_CORRECT))[0]
        want.append(tok)
        logits = lm.step(st, tok, "full")
    assert out0 == want
    spec = SpecDecoder(lm, capacity=64, engine="pass", chunk=2, temperature=T, seed=seed)
    out3 = spec.run([prompt], 40, 3, max_rounds=4)[0]          # 40: no round is cut short by the token budget
    assert out3[0] == out0[0]
    assert any(0 < n for row in spec.n_hist for n in row)        # some drafts were kept
    assert any(n < 3 for row in spec.n_hist for n in row)        # and some rejected
    # every state after a commit equals plain consumption of the committed stream
    shadow = lm.new_state(64)
    for t in list(prompt) + out3[:-1]:
        lm.step(shadow, int(t), "full")
    assert spec.st[0].kv_len == shadow.kv_len
    for l in range(cfg.n_layers):
        np.testing.assert_allclose(spec.st[0].S[l], shadow.S[l], rtol=1e-9, atol=1e-12)


def test_first_token_statistics_over_seeds():
    """Monte Carlo over seeds on the tiny model: the first token after a k = 2 round (kept draft
    or correction) has the full model's distribution at that position."""
    cfg, lm = _tiny()
    prompt = W.make_prompts(cfg.vocab, 1, 6, 11)[0]
    T = 1.0
    st = lm.new_state(64)
    for t in prompt:
        logits = lm.step(st, int(t), "full")
    trials = 400
    counts = np.zeros(cfg.vocab)
    second_logits = {}
    for seed in range(trials):
        dec = SpecDecoder(lm, capacity=64, engine="step", temperature=T, seed=seed)
        dec.prefill([prompt], 4)
        first = dec.out[0][0]
        dec.draft(2)
        dec.verify()
        dec.commit()
        counts[dec.out[0][1]] += 1
        second_logits.setdefault(first, dec.verify_logits[0][0])
    # expected distribution of the second token: mixture over the first
    p_first = S.softmax_t(logits, T)
    expect = np.zeros(cfg.vocab)
    for first, l2 in second_logits.items():
        expect += p_first[first] * S.softmax_t(l2, T)
    seen = sum(p_first[f] for f in second_logits)
    assert seen > 0.9
    # total variation distance, against the sampling noise of 400 draws over a small vocabulary
    tv = 0.5 * np.abs(counts / trials - expect / seen).sum()
    assert tv < 0.5 * np.sqrt(cfg.vocab / trials) + 0.1 * (1 - seen) + 0.05, tv


def test_residual_without_mass_and_ids_that_are_no_token():
    """The case Eq. 6 leaves open.  With P_S == P_H the ratio is 1, so every real uniform keeps the
    draft; a test value of 1.0 (outside the generator's range) forces the rejection and with it a
    residual without mass: the token then is the inverse-CDF draw from P_H (hand-computed grid
    below), or its successor when that draw is the rejected draft, so the targets row encodes n.
    A draft id that is no token is rejected where it stands and never used as an index."""
    p = np.array([0.125, 0.5, 0.25, 0.125])
    for u_c, d, want in [(0.0, 2, 0), (0.2, 0, 1), (0.2, 1, 2), (0.7, 1, 2), (0.7, 2, 3), (0.95, 3, 0), (0.95, 0, 3)]:
        n, tok, _ = S.stochastic_round([p], [p, p], [d], [1.0], lambda n_: u_c)
        assert (n, tok) == (0, want), (u_c, d, tok)
        assert S.stochastic_targets([d], n, tok)[0] != d
    # real uniforms: identical distributions keep the draft
    assert S.stochastic_round([p], [p, p], [1], [0.99999994], lambda n_: 0.3)[0] == 1
    # ids outside the vocabulary: position 1 is rejected, position 0 (ratio 1) kept; the residual of
    # identical rows has no mass, so the token comes from P_H: u = 0.7 -> index 2
    for bad in (-1, 4, 99):
        n, tok, _ = S.stochastic_round([p, p], [p, p, p], [3, bad], [0.5, 0.5], lambda n_: 0.7)
        assert (n, tok) == (1, 2)
        assert S.stochastic_targets([3, bad], n, tok) == [3, 2, -1]
