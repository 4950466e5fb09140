"""Speculative round protocol and plain greedy decoding (test oracle).

Section 3.3 of the paper: a round drafts k tokens with the SSM-only subgraph
M_S, verifies them with one pass of the full hybrid M_H, and under greedy
decoding accepts draft token i iff it equals M_H's argmax at that position;
every token up to the first mismatch is kept and M_H's own token is emitted at
the mismatch (or after the last draft when all match).  The committed stream
is therefore exactly plain greedy decoding of M_H, whatever the draft was.

Reading used for the caches (the paper's prototype shares none): the last
committed token is "pending" (emitted but not yet consumed by the caches).
The draft starts from the committed recurrent state and works on a scratch
copy; verification consumes pending, d_1 .. d_k at positions len .. len+k and
snapshots the recurrent state after each; committing n accepted drafts
restores snapshot n and sets the cache length to len + n + 1 (later KV slots
are dead).  Sequences in a batch are independent.

`expected_tokens_per_round` and `speedup_model` are Eq. 1.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from .hybrid_lm import HybridLM, SeqState, argmax_lowest, top2_gap
from .passes import full_pass
from . import sampling


def expected_tokens_per_round(alpha: float, k: int) -> float:
    """Numerator of Eq. 1: (1 - alpha^(k+1)) / (1 - alpha) for per-token
    acceptance probability alpha."""
    if alpha == 1.0:
        return float(k + 1)
    return (1.0 - alpha ** (k + 1)) / (1.0 - alpha)


def speedup_model(alpha: float, k: int, cost_ratio: float) -> float:
    """Eq. 1: expected tokens per round over the round's cost in units of one
    verification, 1 + k * c_draft / c_verify."""
    return expected_tokens_per_round(alpha, k) / (1.0 + k * cost_ratio)


def optimal_draft_length(alpha: float, cost_ratio: float, candidates: Sequence[int]) -> int:
    """The draft length among `candidates` that maximises Eq. 1 for per-token
    acceptance probability alpha and cost ratio c_draft / c_verify (the choice the
    paper's Section 7 "Optimal draft length" describes); the smallest on ties."""
    best, best_s = None, -1.0
    for k in sorted(int(v) for v in candidates):
        s = speedup_model(alpha, k, cost_ratio)
        if s > best_s + 1e-15:
            best, best_s = k, s
    return best


def acceptance_counts(n_accepted: Sequence[int], k: int):
    """(accepted, tested) drafts of rounds with k drafts each: a round that accepts n drafts tested
    min(n + 1, k) of them (drafts 1..n passed, draft n+1 - if it exists - failed).  Under the model
    behind Eq. 1 (each test passes independently with probability alpha) accepted / tested is the
    maximum-likelihood estimate of alpha."""
    acc = sum(int(n) for n in n_accepted)
    tested = sum(min(int(n) + 1, k) for n in n_accepted) if k > 0 else 0
    return acc, tested


def accepted_prefix(drafts: Sequence[int], targets: Sequence[int]) -> int:
    """Greedy acceptance (Section 3.3): the number n of leading draft tokens with
    drafts[i] == targets[i], where targets[i] is M_H's argmax given the prefix
    that ends just before draft i."""
    n = 0
    for d, g in zip(drafts, targets):
        if int(d) != int(g):
            break
        n += 1
    return n


def greedy_generate(lm: HybridLM, prompt, n_new: int, gaps: Optional[list] = None) -> List[int]:
    """Plain autoregressive greedy decoding of the full model: n_new tokens."""
    st = lm.new_state(len(prompt) + n_new + 1)
    logits = None
    for t in prompt:
        logits = lm.step(st, int(t), "full")
    out = []
    for _ in range(n_new):
        tok = argmax_lowest(logits)
        if gaps is not None:
            gaps.append(top2_gap(logits))
        out.append(tok)
        if len(out) < n_new:
            logits = lm.step(st, tok, "full")
    return out


class SpecDecoder:
    """prefill -> (draft -> verify -> commit)* over a batch of independent
    sequences.  engine="step" uses only single-token steps (the definition);
    engine="pass" uses the multi-position pass for prefill and verification."""

    def __init__(self, lm: HybridLM, capacity: int, engine: str = "step", chunk: int = 64,
                 temperature: float = 0.0, seed: int = 0, draft_state: str = "shared",
                 draft_mask: Optional[Sequence[str]] = None):
        """temperature 0: greedy acceptance.  temperature > 0: tokens are drawn from
        softmax(logits / T) and drafts pass the rejection test of Eq. 6, with the
        counter-based uniforms of `sampling.uniform(seed, ...)`.

        draft_state "shared" (default): every round the draft starts from the committed
        recurrent state of the full model.  "strict": the draft model M_S is its own
        model over the whole prefix (Eq. 4 applied at every position, Section 3.3
        "Draft phase": P_S(. | x_{1:t+i-1})): it keeps a recurrent state of its own,
        advanced with attention suppressed over the prompt and over every committed
        token.  Either way the committed stream is the full model's; only the accepted
        counts differ.

        draft_mask: one entry per layer, "full" | "ssm" | "skip": the draft steps run
        the masked model of `HybridLM.step` (all "ssm" is Eq. 4, the default)."""
        assert engine in ("step", "pass")
        assert draft_state in ("shared", "strict")
        assert draft_mask is None or draft_state == "shared", "the strict state is defined for the SSM-only draft"
        self.draft_state = draft_state
        self.draft_mask = None if draft_mask is None else list(draft_mask)
        self.lm, self.capacity, self.engine, self.chunk = lm, capacity, engine, chunk
        self.T, self.seed = float(temperature), int(seed)
        self.gaps: List[float] = []          # top-1/top-2 gap of every greedy decision taken
        self.margins: List[float] = []       # distance of every random decision from flipping (T > 0)

    def _pick(self, logits, b: int, idx: int, purpose: int) -> int:
        """Next token from one row of logits: argmax (T = 0) or a draw from softmax(logits / T)."""
        if self.T == 0.0:
            self.gaps.append(top2_gap(logits))
            return argmax_lowest(logits)
        tok, m = sampling.draw(sampling.softmax_t(logits, self.T), sampling.uniform(self.seed, b, idx, purpose))
        self.margins.append(m)
        return tok

    # ---------------------------------------------------------------- prefill
    def prefill(self, prompts: Sequence[Sequence[int]], max_new_tokens: int) -> None:
        self.B = len(prompts)
        self.G = int(max_new_tokens)
        self.st: List[SeqState] = []
        self.out: List[List[int]] = []
        self.pending: List[int] = []
        self.last_n = [0] * self.B
        self.accepted = 0            # running acceptance statistics (see acceptance_counts)
        self.tested = 0
        self.prefill_logits = []
        self.ms: List[SeqState] = []             # strict mode: M_S's own recurrent state per sequence
        for b, p in enumerate(prompts):
            if self.draft_state == "strict":
                ms = self.lm.new_state(1)
                for t in p:
                    self.lm.step(ms, int(t), "draft")
                self.ms.append(ms)
            st = self.lm.new_state(self.capacity)
            if self.engine == "pass":
                logits = full_pass(self.lm, st, p, self.chunk, last_only=True)[0][0]
            else:
                for t in p:
                    logits = self.lm.step(st, int(t), "full")
            tok = self._pick(logits, b, 0, sampling.PURPOSE_CORRECT)
            self.st.append(st)
            self.out.append([tok][:self.G])
            self.pending.append(tok)
            self.prefill_logits.append(logits)
        self.drafts: List[List[int]] = [[] for _ in range(self.B)]
        self.targets: List[List[int]] = [[] for _ in range(self.B)]
        self._ckpt = [None] * self.B

    def finished(self, b: int) -> bool:
        return len(self.out[b]) >= self.G

    def all_finished(self) -> bool:
        return all(self.finished(b) for b in range(self.B))

    # ---------------------------------------------------------------- draft
    def draft(self, k: int, override: Optional[np.ndarray] = None) -> None:
        """k SSM-only steps per active sequence from a scratch copy of the committed
        recurrent state.  `override[b][i]` replaces the draft tokens (any draft
        source must leave the committed stream unchanged)."""
        self.k = k
        self.draft_logits = [None] * self.B
        for b in range(self.B):
            if self.finished(b):
                continue
            st = self.st[b]
            S, conv = (self.ms[b] if self.draft_state == "strict" else st).recurrent_copy()
            # (a masked draft with "full" layers writes K/V at the positions it drafts: slots at and
            # behind kv_len are dead until verification rewrites them)
            scratch = SeqState(S=S, conv=conv, K=st.K, V=st.V, kv_len=st.kv_len)
            t = self.pending[b]
            ds, ls = [], []
            for i in range(k):
                logits = self.lm.step(scratch, t, "draft" if self.draft_mask is None else self.draft_mask)
                t = self._pick(logits, b, len(self.out[b]) + i, sampling.PURPOSE_DRAFT)
                ds.append(t)
                ls.append(logits)
            if override is not None:
                assert self.T == 0.0, "replaced drafts have no draft distribution to test against"
                ds = [int(v) for v in override[b][:k]]
            self.drafts[b] = ds
            self.draft_logits[b] = np.array(ls).reshape(k, -1) if k else None

    # ---------------------------------------------------------------- verify
    def verify(self) -> None:
        """Full-model pass over pending, d_1..d_k; keeps M_H's argmax g_j and a
        snapshot of the recurrent state after every position."""
        self.verify_logits = [None] * self.B
        for b in range(self.B):
            if self.finished(b):
                continue
            st = self.st[b]
            xs = [self.pending[b]] + list(self.drafts[b])
            if self.engine == "pass":
                logits, ck = full_pass(self.lm, st, xs, self.chunk, checkpoints=True)
            else:
                logits, ck = [], []
                for t in xs:
                    logits.append(self.lm.step(st, int(t), "full"))
                    ck.append(st.recurrent_copy())
                logits = np.array(logits)
            self.verify_logits[b] = logits
            if self.T == 0.0:
                self.targets[b] = [argmax_lowest(r) for r in logits]
                self._gaps_v = [top2_gap(r) for r in logits]
            else:
                self.targets[b] = self._stochastic_targets(b, logits)
                self._gaps_v = []
            self._ckpt[b] = (ck, st.kv_len - len(xs), self._gaps_v)

    def _stochastic_targets(self, b: int, logits_h) -> List[int]:
        """Eq. 6 over the round's k drafts; the outcome in the targets form of
        `sampling.stochastic_targets`."""
        d = self.drafts[b]
        k = len(d)
        base = len(self.out[b])
        p_s = [sampling.softmax_t(self.draft_logits[b][i], self.T) for i in range(k)]
        p_h = [sampling.softmax_t(logits_h[i], self.T) for i in range(k + 1)]
        u_acc = [sampling.uniform(self.seed, b, base + i, sampling.PURPOSE_ACCEPT) for i in range(k)]
        n, tok, m = sampling.stochastic_round(
            p_s, p_h, d, u_acc, lambda n_: sampling.uniform(self.seed, b, base + n_, sampling.PURPOSE_CORRECT))
        self.margins.append(m)
        return sampling.stochastic_targets(d, n, tok)

    # ---------------------------------------------------------------- commit
    def commit(self, forced_n: Optional[Sequence[int]] = None) -> None:
        """Accept n drafts (longest matching prefix, or forced_n[b] taken as
        given), emit d_1..d_n and g_n, roll the recurrent state back to the
        snapshot after position n and truncate the cache length to len+n+1."""
        for b in range(self.B):
            if self.finished(b):
                continue
            ck, len0, gaps_v = self._ckpt[b]
            d, g = self.drafts[b], self.targets[b]
            assert forced_n is None or self.T == 0.0, "a forced count has no correction token at T > 0"
            n = accepted_prefix(d, g) if forced_n is None else int(forced_n[b])
            assert 0 <= n <= len(d)
            a_, t_ = acceptance_counts([n], len(d))
            self.accepted += a_
            self.tested += t_
            self.gaps.extend(gaps_v[:n + 1])     # only positions that decided a token
            if self.draft_state == "strict":     # M_S consumes what the caches consumed: pending, d_1 .. d_n
                for t in [self.pending[b]] + list(d[:n]):
                    self.lm.step(self.ms[b], int(t), "draft")
            emit = list(d[:n]) + [g[n]]
            room = self.G - len(self.out[b])
            self.out[b].extend(emit[:room])
            self.pending[b] = g[n]
            st = self.st[b]
            st.S = [s.copy() for s in ck[n][0]]
            st.conv = [c.copy() for c in ck[n][1]]
            st.kv_len = len0 + n + 1
            self.last_n[b] = n

    # ---------------------------------------------------------------- whole runs
    def run(self, prompts, max_new_tokens: int, k: int, forced: Optional[np.ndarray] = None,
            override: Optional[np.ndarray] = None, max_rounds: int = 1 << 30) -> List[List[int]]:
        """Rounds until every sequence has max_new_tokens tokens.  forced[r][b]:
        accepted counts taken as given; override[r][b][i]: draft tokens replaced."""
        self.prefill(prompts, max_new_tokens)
        self.n_hist: List[List[int]] = []
        r = 0
        while not self.all_finished() and r < max_rounds:
            active = [not self.finished(b) for b in range(self.B)]
            self.draft(k, None if override is None else override[r])
            self.verify()
            self.commit(None if forced is None else forced[r])
            self.n_hist.append([self.last_n[b] if active[b] else -1 for b in range(self.B)])
            r += 1
        return self.out
