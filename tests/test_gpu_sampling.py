"""The token-choice kernels of temperature > 0 alone (Eq. 6), through the C ABI, on seeded synthetic
logits at the benchmark's vocabulary sizes and batch shapes (needs an MI355X).

The oracle evaluates the same float32 logits in float64.  A decision whose uniform lies further than
DELTA (relative to the total mass) from every CDF edge, or from the acceptance ratio, has one right
answer and must match it; a closer one may fall on either side, and then the answer must still be
valid: an entry with mass whose CDF interval lies within DELTA of the uniform."""
import numpy as np
import pytest

from oracle import sampling as S
from paper_2605_01106_amd import workloads as W

pytestmark = pytest.mark.gpu

DELTA = 2e-5      # float32 exp and sums over up to 131072 entries against float64: about 1e-6; 20x that


@pytest.fixture(scope="module")
def B():
    from paper_2605_01106_amd import binding
    return binding


def _check_draw(tag, p, u, tok, stats):
    c = np.cumsum(p)
    total = c[-1]
    want, margin = S.draw(p, u)
    if margin > DELTA:
        assert tok == want, (tag, tok, want, margin)
        stats["exact"] += 1
    else:
        assert 0 <= tok < len(p) and p[tok] > 0, (tag, tok)
        assert c[tok] - p[tok] - DELTA * total <= u * total <= c[tok] + DELTA * total, (tag, tok, want, margin)
        stats["close"] += 1


@pytest.mark.parametrize("batch,k,vocab,T", [(64, 8, 131072, 0.6), (1, 2, 32784, 0.6), (3, 3, 203, 1.0), (5, 0, 1000, 0.3)])
def test_draws_and_acceptance_on_synthetic_logits(B, batch, k, vocab, T):
    import torch
    seed = 11
    dev = torch.device("cuda:0")
    draft, verify = W.make_logit_rows(batch, k, vocab, seed)
    positions = np.arange(batch, dtype=np.int32) * 3 + 1
    d_dev, v_dev = torch.from_numpy(draft).to(dev), torch.from_numpy(verify).to(dev)
    pos_dev = torch.from_numpy(positions).to(dev)
    stats = {"exact": 0, "close": 0}
    p_s = [[S.softmax_t(draft[b, i], T) for i in range(k)] for b in range(batch)]
    p_h = [[S.softmax_t(verify[b, i], T) for i in range(k + 1)] for b in range(batch)]
    # draft draws, one launch per step as in the draft loop (row stride k * vocab)
    drafts = np.zeros((batch, max(k, 1)), np.int32)
    for i in range(k):
        got = B.hh_draw_tokens(d_dev[:, i, :], T, seed, positions=pos_dev, position_offset=i,
                               purpose=S.PURPOSE_DRAFT).cpu().numpy()
        for b in range(batch):
            u = S.uniform(seed, b, int(positions[b]) + i, S.PURPOSE_DRAFT)
            _check_draw(f"draft b{b} i{i}", p_s[b][i], u, int(got[b]), stats)
            drafts[b, i] = S.draw(p_s[b][i], u)[0]          # the round goes on with the oracle's drafts
    # first-token form: no positions, purpose 2
    got = B.hh_draw_tokens(v_dev[:, 0, :], T, seed).cpu().numpy()
    for b in range(batch):
        _check_draw(f"first b{b}", p_h[b][0], S.uniform(seed, b, 0, S.PURPOSE_CORRECT), int(got[b]), stats)
    # the round's acceptance
    dr_dev = torch.from_numpy(np.ascontiguousarray(drafts[:, :k])).to(dev) if k else None
    targets = B.hh_accept_tokens(d_dev if k else None, v_dev, dr_dev, pos_dev, T, seed).cpu().numpy()
    same = 0
    n_hist = []
    for b in range(batch):
        g = targets[b]
        n = int(np.max(np.nonzero(g >= 0)[0]))
        assert all(g[i] == drafts[b, i] for i in range(n)) and all(v == -1 for v in g[n + 1:]), (b, g)
        base = int(positions[b])
        u_acc = [S.uniform(seed, b, base + i, S.PURPOSE_ACCEPT) for i in range(k)]
        ratios = [p_h[b][i][drafts[b, i]] / p_s[b][i][drafts[b, i]] for i in range(k)]
        for i in range(n):
            assert u_acc[i] < ratios[i] + DELTA, (b, i, "kept a draft that fails the test")
        u_c = S.uniform(seed, b, base + n, S.PURPOSE_CORRECT)
        if n < k:
            assert u_acc[n] >= ratios[n] - DELTA, (b, n, "rejected a draft that passes the test")
            assert g[n] != drafts[b, n]
            _check_draw(f"correction b{b} n{n}", S.residual(p_h[b][n], p_s[b][n]), u_c, int(g[n]), stats)
        else:
            _check_draw(f"bonus b{b}", p_h[b][k], u_c, int(g[n]), stats)
        n_o, tok_o, _ = S.stochastic_round(p_s[b], p_h[b], list(drafts[b, :k]), u_acc,
                                           lambda n_: S.uniform(seed, b, base + n_, S.PURPOSE_CORRECT))
        same += int(n_o == n and tok_o == g[n])
        n_hist.append(n)
    print(f"[sampling {batch}x{k}x{vocab} T={T}] decisions exact {stats['exact']} close {stats['close']}; "
          f"rounds identical to the oracle's {same}/{batch}; kept {sorted(set(n_hist))}", flush=True)
    if batch >= 16:                           # enough decisions for a rate
        assert stats["exact"] > 0.9 * (stats["exact"] + stats["close"])
        assert same >= 0.9 * batch
    if k >= 3 and batch >= 3:
        assert len(set(n_hist)) > 1           # both kept and rejected drafts occurred


def test_stand_alone_argument_checks(B):
    import torch
    dev = torch.device("cuda:0")
    logits = torch.zeros((2, 16), dtype=torch.float32, device=dev)
    with pytest.raises(B.HHError):
        B.hh_draw_tokens(logits, 0.0, 1)
    with pytest.raises(B.HHError):
        B.hh_draw_tokens(logits, float("inf"), 1)
    with pytest.raises(B.HHError):
        B.hh_draw_tokens(logits, 0.5, 1, purpose=7)
    # a draft id that is no token is rejected where it stands, and the emitted token is a valid one
    v = torch.zeros((1, 3, 16), dtype=torch.float32, device=dev)
    dl = torch.zeros((1, 2, 16), dtype=torch.float32, device=dev)
    bad = torch.tensor([[3, 99]], dtype=torch.int32, device=dev)
    g = B.hh_accept_tokens(dl, v, bad, torch.zeros(1, dtype=torch.int32, device=dev), 1.0, 2).cpu().numpy()[0]
    assert g[0] == 3 and 0 <= g[1] < 16 and g[2] == -1          # equal distributions keep draft 0 (ratio 1)
    # all-equal logits: the draw is floor(u * vocab)
    got = B.hh_draw_tokens(logits, 0.5, 5).cpu().numpy()
    assert [int(v) for v in got] == [int(S.uniform(5, b, 0, 2) * 16) for b in range(2)]


def test_residual_without_mass_draws_from_p_h(B):
    """Identical draft and verification rows and a draft id that is no token: the id is rejected
    where it stands, the residual max(0, P_H - P_S) is exactly zero on both sides, and the emitted
    token is the inverse-CDF draw from P_H with the correction uniform - the oracle's rule for the
    case Eq. 6 leaves open.  Seeds whose uniform lies within DELTA of a CDF edge are skipped."""
    import torch
    dev = torch.device("cuda:0")
    batch, k, vocab, T = 6, 3, 777, 0.8
    _, verify = W.make_logit_rows(batch, k, vocab, 31)
    draft = np.ascontiguousarray(verify[:, :k])
    positions = np.arange(batch, dtype=np.int32) * 2
    checked = 0
    for seed in range(40, 48):
        drafts = np.zeros((batch, k), np.int32)
        bad_at = [b % k for b in range(batch)]
        for b in range(batch):
            for i in range(k):
                drafts[b, i] = (7 * b + i) % vocab
            drafts[b, bad_at[b]] = vocab + b if b % 2 else -1 - b
        g = B.hh_accept_tokens(torch.from_numpy(draft).to(dev), torch.from_numpy(verify).to(dev),
                               torch.from_numpy(drafts).to(dev), torch.from_numpy(positions).to(dev), T, seed).cpu().numpy()
        for b in range(batch):
            p_h = [S.softmax_t(verify[b, i], T) for i in range(k + 1)]
            u_acc = [S.uniform(seed, b, int(positions[b]) + i, S.PURPOSE_ACCEPT) for i in range(k)]
            n, tok, margin = S.stochastic_round(p_h[:k], p_h, list(drafts[b]), u_acc,
                                                lambda n_: S.uniform(seed, b, int(positions[b]) + n_, S.PURPOSE_CORRECT))
            assert n == bad_at[b]                       # ratio 1 keeps every real token before it
            assert list(g[b][:n]) == list(drafts[b][:n]) and all(v == -1 for v in g[b][n + 1:])
            if margin > DELTA:
                assert g[b][n] == tok, (seed, b, g[b], tok)
                checked += 1
    assert checked > 30
