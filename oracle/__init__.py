"""CPU oracle for the component-aware self-speculative decoding hot path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, float64 numpy
statement of what the hot path computes, written from the paper's Section 3
(Eq. 2 parallel hybrid block, Eq. 4 SSM-only draft, Section 3.3 draft /
verification / greedy acceptance) and from the published Mamba-2 scalar-decay
recurrence the paper builds on.  It shares no code with the HIP library and
imports nothing from it.  Only the tests, the smoke check and the
``cpu_baseline`` leg of the benchmark may import it; the product path never does.

Pins (see tests/test_oracle_*.py): closed-form unrolled recurrence, chunked
scan == sequential recurrence, one multi-position pass == single-token steps,
draft == full model with attention zeroed, speculative stream == plain greedy
stream for any draft, cache-free brute force on tiny shapes, textbook special
cases (prefix sums, identity conv, one-key attention, RoPE invariances), and
the expected-tokens-per-round closed form of Eq. 1.  Stochastic acceptance
(Eq. 6, ``sampling.py``; tests/test_oracle_sampling.py): the published
SplitMix64 sequence, inverse-CDF counts on regular grids, exact integration of
the rule over its three uniforms (committed token ~ P_H, keep probability
sum(min(P_S, P_H))), the T -> 0 limit and the k = 0 case.

Parity unpinned: absolute logit values of the large random-init shapes (the
paper prints none) and the paper's acceptance rates (trained weights needed).
"""
