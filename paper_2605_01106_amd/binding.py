"""Thin ctypes binding of libhh.so: the same entry points as include/hh.h.

Argument marshalling only -- every step of the hot path runs inside the
library's HIP kernels.  PyTorch appears here solely as the owner of device
memory (weights, workspace, token buffers) and of the HIP stream.

Importing this module fails loudly if the library has not been built
(``python -m paper_2605_01106_amd.build``); there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch  # first: libhh must bind to the HIP runtime PyTorch has already loaded, not to a second copy

from . import workloads as W

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhh.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2605_01106_amd.build`")
lib = C.CDLL(_LIB_PATH)

HH_OK, HH_EINVAL, HH_ESTATE, HH_ECAPACITY, HH_EWORKSPACE, HH_EDEVICE = 0, -1, -2, -3, -4, -5
HH_F32, HH_BF16 = 0, 1
HH_KF_ATTN_SCALAR, HH_KF_SSM_GENERAL, HH_KF_MID_OFF, HH_KF_SKINNY_OFF, HH_KF_SSM_SCALAR_CONV, HH_KF_ROWS_LDS, HH_KF_SSM_SEQUENTIAL, HH_KF_NO_HANDOVER, HH_KF_CANARIES, HH_KF_SSM_MATMUL, HH_KF_MID_WIDE = 1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024
HH_DRAFT_SSM, HH_DRAFT_FULL, HH_DRAFT_SKIP = 0, 1, 2
DRAFT_MODES = {"ssm": HH_DRAFT_SSM, "full": HH_DRAFT_FULL, "skip": HH_DRAFT_SKIP}
STATUS_NAMES = {0: "HH_OK", -1: "HH_EINVAL", -2: "HH_ESTATE", -3: "HH_ECAPACITY", -4: "HH_EWORKSPACE",
                -5: "HH_EDEVICE"}


class hh_cfg(C.Structure):
    _fields_ = [("struct_size", C.c_uint32),
                ("n_layers", C.c_int32), ("d_model", C.c_int32), ("vocab", C.c_int32),
                ("m_heads", C.c_int32), ("m_head_dim", C.c_int32), ("d_state", C.c_int32),
                ("n_groups", C.c_int32), ("d_conv", C.c_int32),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("rope_base", C.c_float), ("d_ff", C.c_int32), ("rms_eps", C.c_float),
                ("w_dtype", C.c_int32), ("max_batch", C.c_int32), ("max_seq_len", C.c_int32),
                ("max_draft", C.c_int32), ("max_new_tokens", C.c_int32), ("kv_page_tokens", C.c_int32),
                ("prefill_chunk", C.c_int32), ("keep_logits", C.c_int32), ("use_graphs", C.c_int32),
                ("overlap_mode", C.c_int32), ("attn_max_splits", C.c_int32), ("attn_target_blocks", C.c_int32), ("attn_single_slice_steps", C.c_int32),
                ("kernel_flags", C.c_int32), ("prefill_progress", C.c_int32), ("draft_state_mode", C.c_int32),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


_LAYER_FIELDS = ("norm1", "w_in", "conv_w", "conv_b", "a_log", "d_skip", "dt_bias", "gnorm", "w_out",
                 "w_q", "w_k", "w_v", "w_o", "norm2", "w_gate", "w_up", "w_down")


class hh_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_FIELDS]


class hh_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(hh_layer_weights))]


_ctx_p = C.c_void_p
_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)

EXPORTS = {
    "hh_workspace_bytes": (C.c_size_t, [C.POINTER(hh_cfg)]),
    "hh_create": (C.c_int, [C.POINTER(hh_weights), C.POINTER(hh_cfg), C.POINTER(_ctx_p)]),
    "hh_destroy": (C.c_int, [_ctx_p]),
    "hh_prefill": (C.c_int, [_ctx_p, C.c_void_p, C.c_int32, _i32p, C.c_int32, C.c_int32, C.c_void_p]),
    "hh_set_sampling": (C.c_int, [_ctx_p, C.c_float, C.c_uint64, C.c_void_p]),
    "hh_draw_tokens": (C.c_int, [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_float, C.c_uint64, C.c_void_p,
                                 C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "hh_accept_tokens": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                   C.c_float, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hh_accept_tokens_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                          C.c_float, C.c_uint64, C.c_void_p, C.c_void_p]),
    "hh_draft": (C.c_int, [_ctx_p, C.c_int32, C.c_void_p]),
    "hh_set_drafts": (C.c_int, [_ctx_p, C.c_void_p, C.c_void_p]),
    "hh_set_draft_mask": (C.c_int, [_ctx_p, _i32p]),
    "hh_optimal_draft_length": (C.c_int32, [C.c_double, C.c_double, _i32p, C.c_int32]),
    "hh_verify": (C.c_int, [_ctx_p, C.c_void_p]),
    "hh_commit": (C.c_int, [_ctx_p, C.c_void_p, C.c_void_p]),
    "hh_get_tokens": (C.c_int, [_ctx_p, C.c_int32, _i32p, C.c_int32, _i32p, C.c_void_p]),
    "hh_get_lengths": (C.c_int, [_ctx_p, _i32p, _i32p, _i32p, C.c_void_p]),
    "hh_check_canaries": (C.c_int, [_ctx_p, _i32p, C.c_void_p]),
    "hh_get_acceptance": (C.c_int, [_ctx_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.c_void_p]),
    "hh_get_round": (C.c_int, [_ctx_p, _i32p, _i32p, C.c_void_p]),
    "hh_get_logits": (C.c_int, [_ctx_p, C.c_int32, _f32p, C.c_void_p]),
    "hh_get_state": (C.c_int, [_ctx_p, C.c_int32, _f32p, _f32p, C.c_void_p]),
    "hh_get_draft_state": (C.c_int, [_ctx_p, C.c_int32, _f32p, _f32p, C.c_void_p]),
    "hh_get_kv": (C.c_int, [_ctx_p, C.c_int32, C.c_int32, C.c_int32, _f32p, _f32p, C.c_void_p]),
    "hh_profile": (C.c_int, [_ctx_p, C.c_int32]),
    "hh_profile_read": (C.c_int, [_ctx_p, C.c_int32, _i32p, _f32p, C.c_void_p]),
    "hh_time_kind": (C.c_int, [_ctx_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _f32p, _i32p, C.c_void_p]),
    "hh_last_error": (C.c_char_p, [_ctx_p]),
}
for _name, (_res, _args) in EXPORTS.items():
    _fn = getattr(lib, _name)
    _fn.restype, _fn.argtypes = _res, _args


class HHError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


def make_cfg(cfg: W.HybridConfig, max_batch: int, max_seq_len: int, max_draft: int, max_new_tokens: int,
             kv_page_tokens: int = 0, prefill_chunk: int = 0, keep_logits: int = 1, use_graphs: int = 0,
             overlap_mode: int = 0, attn_max_splits: int = 0, attn_single_slice_steps: int = 0, kernel_flags: int = 0,
             prefill_progress: int = 0, draft_state_mode: int = 0, attn_target_blocks: int = 0) -> hh_cfg:
    c = hh_cfg()
    c.struct_size = C.sizeof(hh_cfg)
    c.n_layers, c.d_model, c.vocab = cfg.n_layers, cfg.d_model, cfg.vocab
    c.m_heads, c.m_head_dim, c.d_state = cfg.m_heads, cfg.m_head_dim, cfg.d_state
    c.n_groups, c.d_conv = cfg.n_groups, cfg.d_conv
    c.n_q_heads, c.n_kv_heads, c.head_dim = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    c.rope_base, c.d_ff, c.rms_eps = cfg.rope_base, cfg.d_ff, cfg.rms_eps
    c.w_dtype = HH_BF16 if cfg.w_dtype == W.BF16 else HH_F32
    c.max_batch, c.max_seq_len, c.max_draft, c.max_new_tokens = max_batch, max_seq_len, max_draft, max_new_tokens
    c.kv_page_tokens, c.prefill_chunk, c.keep_logits, c.use_graphs = kv_page_tokens, prefill_chunk, keep_logits, use_graphs
    c.overlap_mode, c.attn_max_splits, c.attn_single_slice_steps = overlap_mode, attn_max_splits, attn_single_slice_steps
    c.kernel_flags, c.prefill_progress, c.draft_state_mode = kernel_flags, prefill_progress, draft_state_mode
    c.attn_target_blocks = attn_target_blocks
    c.workspace, c.workspace_bytes = None, 0
    return c


def hh_workspace_bytes(cfg: hh_cfg) -> int:
    return int(lib.hh_workspace_bytes(C.byref(cfg)))


def hh_last_error(ctx=None) -> str:
    return (lib.hh_last_error(ctx) or b"").decode()


def _check(st: int, ctx=None) -> None:
    if st != HH_OK:
        raise HHError(st, hh_last_error(ctx))


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


def hh_optimal_draft_length(alpha: float, cost_ratio: float, candidates: Sequence[int]) -> int:
    """The candidate draft length that maximises Eq. 1 (-1 for bad arguments)."""
    ks = (C.c_int32 * len(candidates))(*[int(k) for k in candidates])
    return int(lib.hh_optimal_draft_length(float(alpha), float(cost_ratio), ks, len(candidates)))


def hh_draw_tokens(logits, temperature: float, seed: int, positions=None, position_offset: int = 0, purpose: int = 2,
                   stream=None):
    """logits: float32 device tensor [rows][vocab] (last dimension contiguous).  Returns int32 [rows]."""
    assert logits.dtype == torch.float32 and logits.dim() == 2 and logits.stride(1) == 1
    rows, vocab = logits.shape
    out = torch.empty(rows, dtype=torch.int32, device=logits.device)
    pos = None if positions is None else C.c_void_p(positions.data_ptr())
    _check(lib.hh_draw_tokens(C.c_void_p(logits.data_ptr()), logits.stride(0), vocab, rows, C.c_float(temperature),
                              C.c_uint64(seed), pos, position_offset, purpose, C.c_void_p(out.data_ptr()),
                              _stream_ptr(stream)))
    return out


def hh_accept_tokens(draft_logits, verify_logits, drafts, positions, temperature: float, seed: int, stream=None):
    """draft_logits [batch][k][vocab], verify_logits [batch][k+1][vocab] float32, drafts int32 [batch][k],
    positions int32 [batch], all contiguous device tensors.  Returns the targets rows, int32 [batch][k+1]."""
    batch, k1, vocab = verify_logits.shape
    k = k1 - 1
    assert verify_logits.is_contiguous() and verify_logits.dtype == torch.float32 and positions.dtype == torch.int32
    if k > 0:
        assert draft_logits.shape == (batch, k, vocab) and draft_logits.is_contiguous() and drafts.is_contiguous()
        assert draft_logits.dtype == torch.float32 and drafts.dtype == torch.int32 and drafts.shape == (batch, k)
    scratch = torch.empty(batch * (2 * k + 1) * 2, dtype=torch.float32, device=verify_logits.device)
    targets = torch.empty((batch, k + 1), dtype=torch.int32, device=verify_logits.device)
    dl = None if k == 0 else C.c_void_p(draft_logits.data_ptr())
    dr = None if k == 0 else C.c_void_p(drafts.data_ptr())
    _check(lib.hh_accept_tokens(dl, C.c_void_p(verify_logits.data_ptr()), vocab, batch, k, dr,
                                C.c_void_p(positions.data_ptr()), C.c_float(temperature), C.c_uint64(seed),
                                C.c_void_p(scratch.data_ptr()), C.c_void_p(targets.data_ptr()), _stream_ptr(stream)))
    return targets


def hh_accept_tokens_static(draft_logits, verify_logits, drafts, positions, targets, temperature: float, seed: int,
                            stream=None):
    """hh_accept_tokens without a scratch argument; `targets` (int32 [batch][k+1], device) is written in place:
    the call itself allocates nothing."""
    batch, k1, vocab = verify_logits.shape
    k = k1 - 1
    dl = None if k == 0 else C.c_void_p(draft_logits.data_ptr())
    dr = None if k == 0 else C.c_void_p(drafts.data_ptr())
    _check(lib.hh_accept_tokens_static(dl, C.c_void_p(verify_logits.data_ptr()), vocab, batch, k, dr,
                                       C.c_void_p(positions.data_ptr()), C.c_float(temperature), C.c_uint64(seed),
                                       C.c_void_p(targets.data_ptr()), _stream_ptr(stream)))
    return targets


def upload_weights(weights: W.Weights, device="cuda:0"):
    """Copies a host `Weights` to device tensors; returns (hh_weights, keepalive)."""
    cfg = weights.cfg
    keep: Dict[str, "torch.Tensor"] = {}

    def dev(name: str) -> int:
        if name in weights.bits:
            t = torch.from_numpy(weights.bits[name].view(np.int16)).to(device)
        else:
            t = torch.from_numpy(weights.values[name]).to(device)
        keep[name] = t
        return t.data_ptr()

    layers = (hh_layer_weights * cfg.n_layers)()
    for i in range(cfg.n_layers):
        for n in _LAYER_FIELDS:
            setattr(layers[i], n, dev(f"L{i}.{n}"))
    hw = hh_weights()
    hw.embed, hw.final_norm, hw.lm_head = dev("embed"), dev("final_norm"), dev("lm_head")
    hw.layers = layers
    keep["__layers__"] = layers
    return hw, keep


class Context:
    """Owns one hh_ctx plus the device memory it borrows (weights, workspace)."""

    def __init__(self, weights: W.Weights, max_batch: int, max_seq_len: int, max_draft: int,
                 max_new_tokens: int, device="cuda:0", guard_bytes: int = 0, **cfg_kw):
        """guard_bytes (a multiple of 256): the workspace is handed over from inside a larger buffer
        whose first and last guard_bytes hold the byte 0xA5, so that a caller can check
        (`guards_intact`) that the library never writes outside what it was given."""
        self.torch = torch
        self.device = device
        self.model_cfg = weights.cfg
        self.cfg = make_cfg(weights.cfg, max_batch, max_seq_len, max_draft, max_new_tokens, **cfg_kw)
        need = hh_workspace_bytes(self.cfg)
        if need == 0:
            raise HHError(HH_EINVAL, hh_last_error(None))
        assert guard_bytes % 256 == 0
        self.guard_bytes = guard_bytes
        self.workspace = torch.empty(need + 2 * guard_bytes, dtype=torch.uint8, device=device)
        if guard_bytes:
            self.workspace[:guard_bytes].fill_(0xA5)
            self.workspace[guard_bytes + need:].fill_(0xA5)
        self.cfg.workspace = self.workspace.data_ptr() + guard_bytes
        self.cfg.workspace_bytes = need
        self.hw, self._keep = upload_weights(weights, device)
        self.ctx = _ctx_p()
        _check(lib.hh_create(C.byref(self.hw), C.byref(self.cfg), C.byref(self.ctx)))
        self.B = 0
        self.k = 0

    def guards_intact(self) -> bool:
        g = self.guard_bytes
        self.torch.cuda.synchronize()
        return bool((self.workspace[:g] == 0xA5).all().item()) and bool((self.workspace[-g:] == 0xA5).all().item())

    def close(self):
        if self.ctx:
            lib.hh_destroy(self.ctx)
            self.ctx = _ctx_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- work calls (asynchronous on the current torch stream unless given)
    def hh_prefill(self, tokens: np.ndarray, lens: Sequence[int], max_new: int, stream=None):
        torch = self.torch
        t = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).to(self.device)
        self._prompt = t
        lens_arr = (C.c_int32 * len(lens))(*[int(x) for x in lens])
        _check(lib.hh_prefill(self.ctx, C.c_void_p(t.data_ptr()), t.shape[1], lens_arr, len(lens), max_new,
                              _stream_ptr(stream)), self.ctx)
        self.B = len(lens)

    def hh_draft(self, k: int, stream=None):
        _check(lib.hh_draft(self.ctx, k, _stream_ptr(stream)), self.ctx)
        self.k = k

    def hh_set_sampling(self, temperature: float, seed: int = 0, stream=None):
        _check(lib.hh_set_sampling(self.ctx, C.c_float(temperature), C.c_uint64(seed), _stream_ptr(stream)), self.ctx)

    def hh_set_drafts(self, drafts, stream=None):
        torch = self.torch
        t = drafts if isinstance(drafts, torch.Tensor) else torch.from_numpy(
            np.ascontiguousarray(drafts, dtype=np.int32)).to(self.device)
        self._drafts_keep = t
        _check(lib.hh_set_drafts(self.ctx, C.c_void_p(t.data_ptr()), _stream_ptr(stream)), self.ctx)

    def hh_set_draft_mask(self, modes):
        """modes: None (every layer SSM-only) or one of "ssm" | "full" | "skip" (or HH_DRAFT_*) per layer."""
        if modes is None:
            _check(lib.hh_set_draft_mask(self.ctx, None), self.ctx)
            return
        assert len(modes) == self.model_cfg.n_layers
        arr = (C.c_int32 * len(modes))(*[DRAFT_MODES.get(m, m) for m in modes])
        _check(lib.hh_set_draft_mask(self.ctx, arr), self.ctx)

    def hh_verify(self, stream=None):
        _check(lib.hh_verify(self.ctx, _stream_ptr(stream)), self.ctx)

    def hh_commit(self, n_accepted=None, stream=None):
        """n_accepted: None (greedy rule) or a device int32 tensor [B]."""
        ptr = None if n_accepted is None else C.c_void_p(n_accepted.data_ptr())
        _check(lib.hh_commit(self.ctx, ptr, _stream_ptr(stream)), self.ctx)

    # ---- read-back
    def hh_get_tokens(self, seq: int, stream=None) -> List[int]:
        cap = self.cfg.max_new_tokens
        out = (C.c_int32 * cap)()
        n = C.c_int32(0)
        _check(lib.hh_get_tokens(self.ctx, seq, out, cap, C.byref(n), _stream_ptr(stream)), self.ctx)
        return list(out[:n.value])

    def hh_get_lengths(self, stream=None):
        B = self.B
        a, b, c = (C.c_int32 * B)(), (C.c_int32 * B)(), (C.c_int32 * B)()
        _check(lib.hh_get_lengths(self.ctx, a, b, c, _stream_ptr(stream)), self.ctx)
        return list(a), list(b), list(c)

    def hh_check_canaries(self, stream=None) -> int:
        """Number of damaged guards behind the workspace regions (context created with HH_KF_CANARIES)."""
        n = C.c_int32(0)
        _check(lib.hh_check_canaries(self.ctx, C.byref(n), _stream_ptr(stream)), self.ctx)
        return int(n.value)

    def hh_get_acceptance(self, stream=None):
        """(accepted, tested) draft counts since the last prefill; accepted / tested estimates alpha of Eq. 1."""
        a, t = C.c_uint64(0), C.c_uint64(0)
        _check(lib.hh_get_acceptance(self.ctx, C.byref(a), C.byref(t), _stream_ptr(stream)), self.ctx)
        return int(a.value), int(t.value)

    def hh_get_round(self, stream=None):
        B, k = self.B, self.k
        d = np.zeros((B, max(k, 1)), np.int32)
        g = np.zeros((B, k + 1), np.int32)
        _check(lib.hh_get_round(self.ctx, d.ctypes.data_as(_i32p), g.ctypes.data_as(_i32p), _stream_ptr(stream)),
               self.ctx)
        return d[:, :k], g

    def hh_get_logits(self, which: int, stream=None) -> np.ndarray:
        B, k, V = self.B, self.k, self.model_cfg.vocab
        shape = {0: (B, k, V), 1: (B, k + 1, V), 2: (B, V)}[which]
        out = np.zeros(shape, np.float32)
        if out.size:
            _check(lib.hh_get_logits(self.ctx, which, out.ctypes.data_as(_f32p), _stream_ptr(stream)), self.ctx)
        return out

    def hh_get_state(self, layer: int, stream=None):
        c = self.model_cfg
        ssm = np.zeros((self.B, c.m_heads, c.m_head_dim, c.d_state), np.float32)
        conv = np.zeros((self.B, c.conv_dim, c.d_conv - 1), np.float32)
        _check(lib.hh_get_state(self.ctx, layer, ssm.ctypes.data_as(_f32p), conv.ctypes.data_as(_f32p),
                                _stream_ptr(stream)), self.ctx)
        return ssm, conv

    def hh_get_draft_state(self, layer: int, stream=None):
        c = self.model_cfg
        ssm = np.zeros((self.B, c.m_heads, c.m_head_dim, c.d_state), np.float32)
        conv = np.zeros((self.B, c.conv_dim, c.d_conv - 1), np.float32)
        _check(lib.hh_get_draft_state(self.ctx, layer, ssm.ctypes.data_as(_f32p), conv.ctypes.data_as(_f32p),
                                      _stream_ptr(stream)), self.ctx)
        return ssm, conv

    def hh_profile(self, enable: bool):
        _check(lib.hh_profile(self.ctx, 1 if enable else 0), self.ctx)

    def hh_profile_read(self, stream=None):
        """{(phase, kind): (launches, total_ms)} of the launches timed since hh_profile(True)."""
        n = 64
        cnt, ms = (C.c_int32 * n)(), (C.c_float * n)()
        _check(lib.hh_profile_read(self.ctx, n, cnt, ms, _stream_ptr(stream)), self.ctx)
        return {(t // 16, t % 16): (cnt[t], ms[t]) for t in range(n) if cnt[t]}

    def hh_time_kind(self, phase: int, kind: int, k: int, reps: int, stream=None):
        """(average microseconds per launch, launches) of one kind of kernel, launched alone."""
        ms, n = C.c_float(0), C.c_int32(0)
        _check(lib.hh_time_kind(self.ctx, phase, kind, k, reps, C.byref(ms), C.byref(n), _stream_ptr(stream)), self.ctx)
        return ms.value * 1e3 / max(n.value, 1), n.value

    def hh_get_kv(self, layer: int, seq: int, n_tokens: int, stream=None):
        c = self.model_cfg
        k = np.zeros((n_tokens, c.n_kv_heads, c.head_dim), np.float32)
        v = np.zeros_like(k)
        _check(lib.hh_get_kv(self.ctx, layer, seq, n_tokens, k.ctypes.data_as(_f32p), v.ctypes.data_as(_f32p),
                             _stream_ptr(stream)), self.ctx)
        return k, v
