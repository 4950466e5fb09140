"""Scalar-decay selective state-space scan: sequential and chunked forms
(test oracle, float64).

Recurrence, per head h with state S[P][N] (the O(1)-memory SSM pathway the
paper's draft relies on, Section 1 and Section 3.4):

    S_t = a_t * S_{t-1} + dt_t * x_t (outer) B_t
    y_t = S_t C_t + D * x_t

`scan_sequential` is that definition.  `scan_chunked` is the state-space-dual
(chunked) evaluation used for multi-position passes: inside a chunk the output
is an attention-like masked product, between chunks only the state is carried.
Both must agree (pinned in the tests, together with a third, fully unrolled
closed form written in the test itself).

Shapes: dt, a: [T][H]; x: [T][H][P]; B, C: [T][N]; D: [H]; S: [H][P][N].
"""
from __future__ import annotations

import numpy as np


def scan_sequential(S0, dt, a, x, B, C, D):
    """Returns y[T][H][P], the list of states after each position, and nothing else."""
    T = dt.shape[0]
    S = S0.copy()
    ys, states = [], []
    for t in range(T):
        S = a[t][:, None, None] * S + dt[t][:, None, None] * x[t][:, :, None] * B[t][None, None, :]
        ys.append(S @ C[t] + D[:, None] * x[t])
        states.append(S.copy())
    return np.array(ys).reshape(T, *S0.shape[:2]), states


def chunk_state(S_in, dt, a, x, B):
    """State after a whole chunk, in closed form:
    S_out = (prod_t a_t) S_in + sum_i (prod_{t>i} a_t) dt_i x_i (outer) B_i."""
    Q = dt.shape[0]
    cum = np.cumsum(np.log(a), axis=0)                      # [Q][H], log of prod_{t<=i} a_t
    w = np.exp(cum[-1][None, :] - cum) * dt                  # [Q][H]
    return (np.exp(cum[-1])[:, None, None] * S_in
            + np.einsum("qh,qhp,qn->hpn", w, x, B))


def chunk_output(S_in, dt, a, x, B, C, D):
    """Outputs of one chunk given the state entering it."""
    Q = dt.shape[0]
    cum = np.cumsum(np.log(a), axis=0)                      # [Q][H]
    # inter-chunk term: decayed incoming state read out by C_t
    y_inter = np.exp(cum)[:, :, None] * np.einsum("hpn,qn->qhp", S_in, C)
    # intra-chunk term: causal mask of decay products times (C_t . B_i)
    G = C @ B.T                                              # [Q][Q]
    causal = np.tril(np.ones((Q, Q), bool))
    decay = np.where(causal[:, :, None], np.exp(cum[:, None, :] - cum[None, :, :]), 0.0)  # [t][i][H]
    M = G[:, :, None] * decay                                # [t][i][H]
    y_intra = np.einsum("tih,ih,ihp->thp", M, dt, x)
    return y_inter + y_intra + D[None, :, None] * x


def scan_chunked(S0, dt, a, x, B, C, D, chunk: int):
    """y[T][H][P] and the final state, evaluating `chunk` positions at a time
    (the last chunk may be shorter)."""
    T = dt.shape[0]
    S = S0.copy()
    ys = []
    for s in range(0, T, chunk):
        e = min(T, s + chunk)
        ys.append(chunk_output(S, dt[s:e], a[s:e], x[s:e], B[s:e], C[s:e], D))
        S = chunk_state(S, dt[s:e], a[s:e], x[s:e], B[s:e])
    y = np.concatenate(ys, axis=0) if ys else np.zeros((0,) + S0.shape[:2])
    return y, S


def prefix_states(S0, dt, a, x, B):
    """Per-position checkpoints S_j (state after positions 0..j), each from the
    closed form over its own prefix -- what a rollback to position j restores."""
    return [chunk_state(S0, dt[:j + 1], a[:j + 1], x[:j + 1], B[:j + 1]) for j in range(dt.shape[0])]
