"""Multi-position full-model pass (test oracle, float64).

The verification phase of Section 3.3 runs the hybrid model M_H once over
several positions and obtains P_H(. | prefix) for all of them simultaneously.
With caches that is: T new tokens at positions len .. len+T-1, projections as
matrix products over the T rows, the SSM branch as a chunked scan started from
the cached state, attention as an explicit causally masked score matrix over
cached plus new keys.  The same pass, without checkpoints, serves as prefill.

Written separately from `HybridLM.step`; the tests pin the two against each
other (one T-position pass == T single-token steps).
"""
from __future__ import annotations

from typing import List, Optional, Tuple

import numpy as np

from .hybrid_lm import F64, HybridLM, SeqState, rmsnorm, rope, round_storage, silu, softplus
from .ssd import prefix_states, scan_chunked


def full_pass(lm: HybridLM, st: SeqState, tokens, chunk: int = 64, checkpoints: bool = False,
              last_only: bool = False):
    """Consume `tokens` (length T) at positions st.kv_len ... ; advances st to
    after the last of them.  Returns (logits, ckpts): logits[T][V] (or [1][V] for
    the last position when last_only), ckpts[j] = (S per layer, conv window per
    layer) after position j when `checkpoints`."""
    c = lm.cfg
    tokens = np.asarray(tokens, np.int64)
    T = tokens.shape[0]
    Hm, P, N = c.m_heads, c.m_head_dim, c.d_state
    d_inner = Hm * P
    conv_dim = d_inner + 2 * N
    Hq, Hkv, Dh = c.n_q_heads, c.n_kv_heads, c.head_dim
    Kc = c.d_conv
    pos0 = st.kv_len
    ck_S: List[List[np.ndarray]] = [[] for _ in range(T)]
    ck_c: List[List[np.ndarray]] = [[] for _ in range(T)]

    h = lm.embed[tokens].copy()                                          # [T][D]
    for l, w in enumerate(lm.layers):
        u = rmsnorm(h, w["norm1"], c.rms_eps)
        zxbcdt = u @ w["w_in"].T
        z = zxbcdt[:, :d_inner]
        xbc_raw = zxbcdt[:, d_inner:d_inner + conv_dim]
        dt_raw = zxbcdt[:, d_inner + conv_dim:]
        # conv: history (d_conv-1 raw inputs, oldest first) followed by the T new ones
        hist = np.concatenate([st.conv[l].T, xbc_raw], axis=0)           # [Kc-1+T][conv_dim]
        acc = np.zeros((T, conv_dim), F64)
        for j in range(Kc):
            acc += hist[j:j + T] * w["conv_w"][:, j][None, :]
        xbc = silu(acc + w["conv_b"][None, :])
        x = xbc[:, :d_inner].reshape(T, Hm, P)
        Bm = xbc[:, d_inner:d_inner + N]
        Cm = xbc[:, d_inner + N:]
        dt = softplus(dt_raw + w["dt_bias"][None, :])
        a = np.exp(-np.exp(w["a_log"])[None, :] * dt)
        if checkpoints:
            for j, Sj in enumerate(prefix_states(st.S[l], dt, a, x, Bm)):
                ck_S[j].append(Sj)
                ck_c[j].append(hist[j + 1:j + Kc].T.copy())              # window ending at position j
        y, S_end = scan_chunked(st.S[l], dt, a, x, Bm, Cm, w["d_skip"], chunk)
        st.S[l] = S_end
        st.conv[l] = hist[T:T + Kc - 1].T.copy()
        m = rmsnorm(y.reshape(T, d_inner) * silu(z), w["gnorm"], c.rms_eps) @ w["w_out"].T
        # attention over cache + new positions, explicit masked matrix
        q = (u @ w["w_q"].T).reshape(T, Hq, Dh)
        kk = (u @ w["w_k"].T).reshape(T, Hkv, Dh)
        vv = (u @ w["w_v"].T).reshape(T, Hkv, Dh)
        for j in range(T):
            q[j] = rope(q[j], pos0 + j, c.rope_base)
            st.K[l][pos0 + j] = round_storage(rope(kk[j], pos0 + j, c.rope_base), c.w_dtype)
            st.V[l][pos0 + j] = round_storage(vv[j], c.w_dtype)
        n_keys = pos0 + T
        visible = np.arange(n_keys)[None, :] <= (pos0 + np.arange(T))[:, None]   # [T][n_keys]
        o = np.zeros((T, Hq, Dh), F64)
        for i in range(Hq):
            g = i // (Hq // Hkv)
            s = q[:, i, :] @ st.K[l][:n_keys, g, :].T / np.sqrt(F64(Dh))
            s = np.where(visible, s, -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p = p / p.sum(axis=1, keepdims=True)
            o[:, i, :] = p @ st.V[l][:n_keys, g, :]
        att = o.reshape(T, Hq * Dh) @ w["w_o"].T
        h = h + m + att
        r = rmsnorm(h, w["norm2"], c.rms_eps)
        h = h + (silu(r @ w["w_gate"].T) * (r @ w["w_up"].T)) @ w["w_down"].T
    st.kv_len = pos0 + T
    hh = h[-1:] if last_only else h
    logits = rmsnorm(hh, lm.final_norm, c.rms_eps) @ lm.lm_head.T
    ckpts = [(ck_S[j], ck_c[j]) for j in range(T)] if checkpoints else None
    return logits, ckpts
