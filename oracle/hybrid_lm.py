"""Single-token definition of the parallel-hybrid decoder (test oracle, float64).

One call to :meth:`HybridLM.step` consumes one token for one sequence and
returns the next-token logits.  ``mode="full"`` is the hybrid model M_H of
Eq. 2 (SSM branch + attention branch, summed); ``mode="draft"`` is the
SSM-only subgraph M_S of Eq. 4: the attention output is zero at every layer
and everything else (norms, MLP, LM head) is unchanged (Section 3.2).

The paper does not print the layer equations.  The Mamba-2 branch follows the
published scalar-decay selective state-space recurrence it cites; the block
layout (pre-norm residual stream, one shared input norm, SwiGLU MLP) follows
the workload description.  No blocking, fusion or reordering: each line below
is one equation.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------- elementary maps

def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * w over the last axis."""
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * w


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def softplus(x: np.ndarray) -> np.ndarray:
    """log(1 + exp(x)); equal to x (to double precision) above 20."""
    x = np.asarray(x, F64)
    return np.where(x > 20.0, x, np.log1p(np.exp(np.minimum(x, 20.0))))


def rope(v: np.ndarray, pos: int, base: float) -> np.ndarray:
    """Rotary embedding of v[..., Dh] at integer position pos: element i is paired
    with element i + Dh/2 and the pair is rotated by pos * base^(-2i/Dh)."""
    dh = v.shape[-1]
    half = dh // 2
    i = np.arange(half, dtype=F64)
    ang = F64(pos) * np.power(F64(base), -2.0 * i / dh)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = v[..., :half], v[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def round_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Value of x after being written to the KV cache.  bf16: the float32 value
    of x rounded to bfloat16, nearest-even (the product computes K/V in float32
    and rounds once on the cache write, so the decision is taken from float32).
    f32: rounded to float32."""
    x32 = np.asarray(x, np.float32)
    if dtype == "f32":
        return x32.astype(F64)
    u = x32.view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(F64)


def argmax_lowest(v: np.ndarray) -> int:
    """Index of the maximum; the lowest index among equal maxima.  NaN is an error."""
    if np.isnan(v).any():
        raise FloatingPointError("NaN in logits")
    return int(np.argmax(v))


def top2_gap(v: np.ndarray) -> float:
    """Difference between the largest and second-largest entry (audit of how
    close a greedy decision was to flipping, cf. the paper's Table 9 remark)."""
    p = np.partition(v, -2)
    return float(p[-1] - p[-2])


# ----------------------------------------------------------------- per-sequence state

@dataclass
class SeqState:
    """Everything one sequence carries between tokens: per layer the SSM state
    S[Hm][P][N], the last d_conv-1 raw conv inputs (oldest first), and the KV
    cache with its length."""

    S: List[np.ndarray]
    conv: List[np.ndarray]
    K: List[np.ndarray]
    V: List[np.ndarray]
    kv_len: int

    def recurrent_copy(self):
        """Copy of the recurrent part (S, conv) only -- what a checkpoint holds."""
        return [s.copy() for s in self.S], [c.copy() for c in self.conv]


class HybridLM:
    def __init__(self, cfg, values: Dict[str, np.ndarray]):
        """cfg: any object with the shape attributes (n_layers, d_model, vocab,
        m_heads, m_head_dim, d_state, d_conv, n_q_heads, n_kv_heads, head_dim,
        d_ff, rope_base, rms_eps, w_dtype).  values: name -> array of the stored
        weight values (already rounded to the storage type)."""
        if getattr(cfg, "n_groups", 1) != 1:
            raise ValueError("only n_groups = 1")
        self.cfg = cfg
        self.embed = np.asarray(values["embed"], F64)
        self.lm_head = np.asarray(values["lm_head"], F64)
        self.final_norm = np.asarray(values["final_norm"], F64)
        names = ("norm1", "w_in", "conv_w", "conv_b", "a_log", "d_skip", "dt_bias", "gnorm", "w_out",
                 "w_q", "w_k", "w_v", "w_o", "norm2", "w_gate", "w_up", "w_down")
        self.layers = [{n: np.asarray(values[f"L{i}.{n}"], F64) for n in names}
                       for i in range(cfg.n_layers)]

    # -- state
    def new_state(self, capacity: int) -> SeqState:
        c = self.cfg
        d_inner = c.m_heads * c.m_head_dim
        conv_dim = d_inner + 2 * c.d_state
        L = c.n_layers
        return SeqState(
            S=[np.zeros((c.m_heads, c.m_head_dim, c.d_state), F64) for _ in range(L)],
            conv=[np.zeros((conv_dim, c.d_conv - 1), F64) for _ in range(L)],
            K=[np.zeros((capacity, c.n_kv_heads, c.head_dim), F64) for _ in range(L)],
            V=[np.zeros((capacity, c.n_kv_heads, c.head_dim), F64) for _ in range(L)],
            kv_len=0)

    # -- one token
    def step(self, st: SeqState, tok: int, mode="full") -> np.ndarray:
        """Consume token `tok` at position st.kv_len (full) or on the recurrent
        state only (draft); returns logits[V].  Full mode appends to the KV cache
        and advances kv_len; draft mode never touches the cache.

        `mode` may also be a sequence of one entry per layer, "full" | "ssm" | "skip"
        (a masked draft): a "full" layer computes both branches of Eq. 2 at position
        st.kv_len and writes its K/V there, an "ssm" layer suppresses its attention
        output (Eq. 4), a "skip" layer passes the stream through unchanged and leaves
        its state alone (the identity pass-through of Eq. 5 applied to a whole block,
        and the layer skipping of the generic drafts of Section 4.2).  A masked step
        advances st.kv_len, so it is run on a scratch state."""
        c = self.cfg
        if isinstance(mode, str):
            assert mode in ("full", "draft")
            layer_modes = ["full" if mode == "full" else "ssm"] * c.n_layers
            advance = mode == "full"
        else:
            layer_modes = list(mode)
            assert len(layer_modes) == c.n_layers and all(m in ("full", "ssm", "skip") for m in layer_modes)
            advance = True
        Hm, P, N = c.m_heads, c.m_head_dim, c.d_state
        d_inner = Hm * P
        conv_dim = d_inner + 2 * N
        Hq, Hkv, Dh = c.n_q_heads, c.n_kv_heads, c.head_dim
        pos = st.kv_len

        h = self.embed[tok].copy()
        for l, w in enumerate(self.layers):
            if layer_modes[l] == "skip":
                continue
            # shared input norm and the Mamba-2 input projection
            u = rmsnorm(h, w["norm1"], c.rms_eps)
            zxbcdt = w["w_in"] @ u
            z = zxbcdt[:d_inner]
            xbc_raw = zxbcdt[d_inner:d_inner + conv_dim]
            dt_raw = zxbcdt[d_inner + conv_dim:]
            # causal depthwise conv over the last d_conv raw inputs, then SiLU
            win = np.concatenate([st.conv[l], xbc_raw[:, None]], axis=1)   # oldest first
            xbc = silu(w["conv_b"] + np.sum(w["conv_w"] * win, axis=1))
            st.conv[l] = win[:, 1:]
            x = xbc[:d_inner].reshape(Hm, P)
            Bv = xbc[d_inner:d_inner + N]
            Cv = xbc[d_inner + N:]
            # selective state update with one scalar decay per head
            dt = softplus(dt_raw + w["dt_bias"])
            a = np.exp(-np.exp(w["a_log"]) * dt)
            st.S[l] = (a[:, None, None] * st.S[l]
                       + dt[:, None, None] * x[:, :, None] * Bv[None, None, :])
            y = st.S[l] @ Cv + w["d_skip"][:, None] * x
            # gate, normalise over all of d_inner, project out
            m = w["w_out"] @ rmsnorm(y.reshape(-1) * silu(z), w["gnorm"], c.rms_eps)
            # attention branch (Eq. 2); suppressed in the draft (Eq. 4)
            if layer_modes[l] == "full":
                q = rope((w["w_q"] @ u).reshape(Hq, Dh), pos, c.rope_base)
                kk = rope((w["w_k"] @ u).reshape(Hkv, Dh), pos, c.rope_base)
                vv = (w["w_v"] @ u).reshape(Hkv, Dh)
                st.K[l][pos] = round_storage(kk, c.w_dtype)
                st.V[l][pos] = round_storage(vv, c.w_dtype)
                o = np.zeros((Hq, Dh), F64)
                for i in range(Hq):
                    g = i // (Hq // Hkv)
                    s = st.K[l][:pos + 1, g, :] @ q[i] / np.sqrt(F64(Dh))
                    p = np.exp(s - s.max())
                    p = p / p.sum()
                    o[i] = p @ st.V[l][:pos + 1, g, :]
                att = w["w_o"] @ o.reshape(-1)
            else:
                att = 0.0
            h = h + m + att
            # SwiGLU MLP
            r = rmsnorm(h, w["norm2"], c.rms_eps)
            h = h + w["w_down"] @ (silu(w["w_gate"] @ r) * (w["w_up"] @ r))
        if advance:
            st.kv_len = pos + 1
        return self.lm_head @ rmsnorm(h, self.final_norm, c.rms_eps)
