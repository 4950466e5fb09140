"""Seeded synthetic inputs for the parallel-hybrid speculative-decoding hot path.

This module only *describes and draws inputs*: model shapes, random-init weights,
random prompts and forced-acceptance tables.  It contains none of the method's
arithmetic (no norm, no SSM, no attention, no acceptance rule), so that the CPU
oracle and the HIP path can both be fed from it without sharing any computation.

The paper evaluates trained Falcon-H1 checkpoints on WikiText-2 prompts
(Section 4, "Models" and "Evaluation Protocol").  Neither is available offline;
the shapes below mirror the paper's Table 1 parallel hybrids (36-layer 0.5B and
32-layer 3B, one Mamba-2 branch plus one attention branch per block) and the
prompt lengths, with random-init weights and uniform-random token ids.

Every tensor is drawn from its own counter-based stream keyed by (seed, name),
so the order in which tensors are generated never matters.
"""
from __future__ import annotations

import dataclasses
import zlib
from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

F32 = "f32"
BF16 = "bf16"


@dataclass(frozen=True)
class HybridConfig:
    """Shape of a parallel-hybrid decoder (Section 3.1, Eq. 2: every block adds an
    SSM branch and an attention branch computed from the same input)."""

    name: str
    n_layers: int
    d_model: int
    vocab: int
    m_heads: int        # Mamba-2 heads (Hm)
    m_head_dim: int     # Mamba-2 head dim (P)
    d_state: int        # N
    n_q_heads: int
    n_kv_heads: int
    head_dim: int       # attention head dim (Dh)
    d_ff: int           # SwiGLU width (F)
    w_dtype: str = BF16  # storage type of the matrices and of the KV cache
    n_groups: int = 1
    d_conv: int = 4
    rope_base: float = 1e4
    rms_eps: float = 1e-5

    @property
    def d_inner(self) -> int:
        return self.m_heads * self.m_head_dim

    @property
    def conv_dim(self) -> int:
        return self.d_inner + 2 * self.n_groups * self.d_state

    @property
    def d_in_proj(self) -> int:
        return 2 * self.d_inner + 2 * self.n_groups * self.d_state + self.m_heads

    @property
    def d_q(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.head_dim

    def params_per_layer(self, draft: bool) -> int:
        """Parameters touched by one block in draft (attention suppressed) or
        full mode -- the counting behind the paper's 78.4 % cost ratio
        (Section 3.4)."""
        D = self.d_model
        n = D                                   # norm1
        n += self.d_in_proj * D                 # w_in
        n += self.conv_dim * self.d_conv + self.conv_dim
        n += 3 * self.m_heads                   # a_log, d_skip, dt_bias
        n += self.d_inner                       # gated norm weight
        n += D * self.d_inner                   # w_out
        if not draft:
            n += (self.d_q + 2 * self.d_kv) * D + D * self.d_q
        n += D                                  # norm2
        n += 3 * D * self.d_ff
        return n

    def step_params(self, draft: bool) -> int:
        """Parameters multiplied per token (the embedding lookup costs none)."""
        return (self.n_layers * self.params_per_layer(draft)
                + self.vocab * self.d_model + self.d_model)

    def total_params(self) -> int:
        return self.step_params(False) + self.vocab * self.d_model


@dataclass(frozen=True)
class Workload:
    """One run: a model shape plus batch, prompt length, generation budget and
    draft length k (Section 3.3)."""

    cfg: HybridConfig
    batch: int
    prompt_len: int
    gen_len: int
    k: int
    forced_p: Optional[float] = None  # per-token accept probability of the forced pattern
    seed: int = 0


_TINY = HybridConfig("tiny-fp32", n_layers=2, d_model=256, vocab=1024, m_heads=8, m_head_dim=32,
                     d_state=16, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ff=512, w_dtype=F32)
_H05B = HybridConfig("falcon-h1-0.5b-shaped", n_layers=36, d_model=1024, vocab=32768, m_heads=24,
                     m_head_dim=64, d_state=128, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ff=4096)
_H3B = HybridConfig("falcon-h1-3b-shaped", n_layers=32, d_model=2560, vocab=65536, m_heads=40,
                    m_head_dim=64, d_state=256, n_q_heads=10, n_kv_heads=2, head_dim=128, d_ff=6912)

WORKLOADS: Dict[str, Workload] = {
    "c0": Workload(_TINY, batch=1, prompt_len=32, gen_len=64, k=2),
    "c1": Workload(_H05B, batch=1, prompt_len=512, gen_len=256, k=2),
    "c2": Workload(_H05B, batch=16, prompt_len=2048, gen_len=256, k=4),
    "c2f": Workload(_H05B, batch=16, prompt_len=2048, gen_len=256, k=4, forced_p=0.37),
    "c3": Workload(_H3B, batch=1, prompt_len=4096, gen_len=256, k=4),
    "c4": Workload(_H3B, batch=64, prompt_len=32768, gen_len=128, k=8, forced_p=0.68),
}


def scaled_config(name: str, **kw) -> HybridConfig:
    """A small model for tests: same structure, caller-chosen (possibly odd) sizes."""
    base = dict(n_layers=2, d_model=64, vocab=128, m_heads=2, m_head_dim=8, d_state=8,
                n_q_heads=2, n_kv_heads=1, head_dim=8, d_ff=96, w_dtype=F32)
    base.update(kw)
    return HybridConfig(name, **base)


# --------------------------------------------------------------------------- streams

def _rng(seed: int, name: str) -> np.random.Generator:
    key = zlib.crc32(name.encode("utf-8"))
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), int(key)])))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bfloat16 (nearest, ties to even); returns the uint16
    bit patterns.  Storage preparation only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


MATRIX_NAMES = ("w_in", "w_out", "w_q", "w_k", "w_v", "w_o", "w_gate", "w_up", "w_down")
VECTOR_NAMES = ("norm1", "conv_w", "conv_b", "a_log", "d_skip", "dt_bias", "gnorm", "norm2")
LAYER_NAMES = ("norm1", "w_in", "conv_w", "conv_b", "a_log", "d_skip", "dt_bias", "gnorm", "w_out",
               "w_q", "w_k", "w_v", "w_o", "norm2", "w_gate", "w_up", "w_down")
GLOBAL_MATRICES = ("embed", "lm_head")


def layer_shapes(cfg: HybridConfig) -> Dict[str, tuple]:
    D = cfg.d_model
    return {
        "norm1": (D,), "w_in": (cfg.d_in_proj, D),
        "conv_w": (cfg.conv_dim, cfg.d_conv), "conv_b": (cfg.conv_dim,),
        "a_log": (cfg.m_heads,), "d_skip": (cfg.m_heads,), "dt_bias": (cfg.m_heads,),
        "gnorm": (cfg.d_inner,), "w_out": (D, cfg.d_inner),
        "w_q": (cfg.d_q, D), "w_k": (cfg.d_kv, D), "w_v": (cfg.d_kv, D), "w_o": (D, cfg.d_q),
        "norm2": (D,), "w_gate": (cfg.d_ff, D), "w_up": (cfg.d_ff, D), "w_down": (D, cfg.d_ff),
    }


class Weights:
    """Host copy of a model's weights.

    ``values[name]`` holds fp32 arrays whose entries are exactly representable
    in the storage type (matrices are rounded to bf16 when ``cfg.w_dtype`` is
    bf16; vectors stay fp32).  ``bits[name]`` holds the uint16 bf16 patterns of
    the matrices when the storage type is bf16.  Names: global ``embed``,
    ``final_norm``, ``lm_head``; per layer ``L{i}.{name}``.
    """

    def __init__(self, cfg: HybridConfig):
        self.cfg = cfg
        self.values: Dict[str, np.ndarray] = {}
        self.bits: Dict[str, np.ndarray] = {}

    def put_matrix(self, name: str, x32: np.ndarray) -> None:
        if self.cfg.w_dtype == BF16:
            b = to_bf16_bits(x32)
            self.bits[name] = b
            self.values[name] = bf16_bits_to_f32(b)
        else:
            self.values[name] = np.ascontiguousarray(x32, dtype=np.float32)

    def put_vector(self, name: str, x32: np.ndarray) -> None:
        self.values[name] = np.ascontiguousarray(x32, dtype=np.float32)

    def layer(self, i: int) -> Dict[str, np.ndarray]:
        return {n: self.values[f"L{i}.{n}"] for n in LAYER_NAMES}


def make_weights(cfg: HybridConfig, seed: int, std: float = 0.02,
                 overrides: Optional[Dict[str, np.ndarray]] = None) -> Weights:
    """Random-init weights: every matrix (conv taps and embedding included)
    ~ N(0, std^2); conv bias 0; A_log = ln U[1,16]; dt_bias = inverse-softplus
    of a log-uniform step in [1e-3, 1e-1]; D skip 1; norm weights 1."""
    w = Weights(cfg)

    def normal(name, shape):
        return (_rng(seed, name).standard_normal(shape, dtype=np.float32) * np.float32(std))

    w.put_matrix("embed", normal("embed", (cfg.vocab, cfg.d_model)))
    w.put_matrix("lm_head", normal("lm_head", (cfg.vocab, cfg.d_model)))
    w.put_vector("final_norm", np.ones(cfg.d_model, np.float32))
    shapes = layer_shapes(cfg)
    for i in range(cfg.n_layers):
        for n in LAYER_NAMES:
            full = f"L{i}.{n}"
            shp = shapes[n]
            if n in MATRIX_NAMES:
                w.put_matrix(full, normal(full, shp))
            elif n == "conv_w":
                w.put_vector(full, normal(full, shp))
            elif n == "conv_b":
                w.put_vector(full, np.zeros(shp, np.float32))
            elif n == "a_log":
                w.put_vector(full, np.log(_rng(seed, full).uniform(1.0, 16.0, shp)))
            elif n == "dt_bias":
                dt = np.exp(_rng(seed, full).uniform(np.log(1e-3), np.log(1e-1), shp))
                w.put_vector(full, dt + np.log(-np.expm1(-dt)))
            else:  # norms and D skip
                w.put_vector(full, np.ones(shp, np.float32))
    if overrides:
        for name, arr in overrides.items():
            if name.split(".")[-1] in MATRIX_NAMES or name in GLOBAL_MATRICES:
                w.put_matrix(name, arr)
            else:
                w.put_vector(name, arr)
    return w


def make_lively_weights(cfg: HybridConfig, seed: int) -> Weights:
    """Test-only variant whose SSM recurrence, conv taps and norm weights are
    O(1), so that a wrong state, window or rollback visibly moves the logits
    (under the N(0,0.02) init the recurrent term is ~1e-4 of the skip term)."""
    w = make_weights(cfg, seed)
    shapes = layer_shapes(cfg)
    for i in range(cfg.n_layers):
        r = _rng(seed, f"L{i}.lively")
        w.put_vector(f"L{i}.conv_w", r.standard_normal(shapes["conv_w"]).astype(np.float32) * 0.5)
        w.put_vector(f"L{i}.conv_b", r.standard_normal(shapes["conv_b"]).astype(np.float32) * 0.1)
        w.put_vector(f"L{i}.d_skip", r.uniform(0.5, 1.5, shapes["d_skip"]).astype(np.float32))
        dt = np.exp(r.uniform(np.log(5e-2), np.log(5e-1), shapes["dt_bias"]))
        w.put_vector(f"L{i}.dt_bias", (dt + np.log(-np.expm1(-dt))).astype(np.float32))
        w.put_vector(f"L{i}.a_log", np.log(r.uniform(0.5, 4.0, shapes["a_log"])).astype(np.float32))
        for n in ("norm1", "gnorm", "norm2"):
            w.put_vector(f"L{i}.{n}", r.uniform(0.5, 1.5, shapes[n]).astype(np.float32))
        w.put_matrix(f"L{i}.w_in", r.standard_normal(shapes["w_in"]).astype(np.float32)
                     * np.float32(2.0 / np.sqrt(cfg.d_model)))
        for n in ("w_q", "w_k", "w_v"):
            w.put_matrix(f"L{i}.{n}", r.standard_normal(shapes[n]).astype(np.float32)
                         * np.float32(1.5 / np.sqrt(cfg.d_model)))
        w.put_matrix(f"L{i}.w_o", r.standard_normal(shapes["w_o"]).astype(np.float32)
                     * np.float32(1.0 / np.sqrt(cfg.d_q)))
    w.put_vector("final_norm", _rng(seed, "final_norm.lively").uniform(0.5, 1.5, cfg.d_model)
                 .astype(np.float32))
    return w


def make_prompts(vocab: int, batch: int, lens, seed: int) -> np.ndarray:
    """Uniform iid token ids, one row per sequence, padded with 0 to max(lens)."""
    lens = [int(lens)] * batch if np.isscalar(lens) else [int(x) for x in lens]
    out = np.zeros((batch, max(lens) if lens else 0), np.int32)
    for b, n in enumerate(lens):
        out[b, :n] = _rng(seed, f"prompt{b}").integers(0, vocab, n, dtype=np.int32)
    return out


def make_forced_pattern(rounds: int, batch: int, k: int, p: float, seed: int) -> np.ndarray:
    """Accepted-draft counts n[round][seq] in 0..k with P(n=j)=p^j(1-p) for j<k and
    P(n=k)=p^k: each draft token is accepted independently with probability p
    until the first rejection (the per-token model behind Eq. 1)."""
    u = _rng(seed, f"forced{k}:{p}").random((rounds, batch, k))
    ok = u < p
    n = np.where(ok.all(axis=2), k, np.argmin(ok, axis=2))
    return n.astype(np.int32)


def make_logit_rows(batch: int, k: int, vocab: int, seed: int, spread: float = 3.0, draft_noise: float = 0.7):
    """Synthetic logits of one round for the token-choice kernels alone: verification rows
    [batch][k+1][vocab] ~ N(0, spread^2) (a few tokens carry most of the mass after the softmax,
    a long tail carries the rest, as for a language model's head) and draft rows [batch][k][vocab]
    = the matching verification rows + N(0, draft_noise^2) (a draft that mostly agrees).  float32."""
    g = _rng(seed, "logit-rows")
    verify = (g.standard_normal((batch, k + 1, vocab), dtype=np.float32) * np.float32(spread))
    draft = verify[:, :k] + g.standard_normal((batch, k, vocab), dtype=np.float32) * np.float32(draft_noise)
    return np.ascontiguousarray(draft, np.float32), np.ascontiguousarray(verify, np.float32)


def make_random_drafts(vocab: int, rounds: int, batch: int, k: int, seed: int) -> np.ndarray:
    """Arbitrary draft tokens, for tests that the committed stream does not depend
    on the draft source."""
    return _rng(seed, "rand-drafts").integers(0, vocab, (rounds, batch, k), dtype=np.int32)
