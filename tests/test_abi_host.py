"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes workspaces, and rejects bad configurations and out-of-order calls
before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2605_01106_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2605_01106_amd import binding
    return binding


def test_exports_match_header(B):
    text = open(os.path.join(ROOT, "include", "hh.h")).read()
    declared = set(re.findall(r"HH_API [\w\s\*]+?\b(hh_\w+)\(", text))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name)
    assert C.sizeof(B.hh_cfg) == 144 and C.sizeof(B.hh_layer_weights) == 17 * 8


def test_workspace_sizes(B):
    c1 = W.WORKLOADS["c1"]
    cfg = B.make_cfg(c1.cfg, 1, 1024, 2, 256)
    n = B.hh_workspace_bytes(cfg)
    # at least the KV pool, both SSM states and the library's copies of the bf16 matrices (tile
    # layout of the matrix-core kernels, plus the stacked input projections)
    kv = 36 * 1024 * 2 * 2 * 64 * 2
    ssm = 2 * 36 * 24 * 64 * 128 * 4
    mats = 2 * c1.cfg.step_params(False)
    assert n > kv + ssm + mats and n < 4 * (kv + ssm) + (1 << 28) + 1.4 * mats
    c4 = W.WORKLOADS["c4"]
    big = B.hh_workspace_bytes(B.make_cfg(c4.cfg, 64, 32768 + 128 + 18, 8, 128, prefill_chunk=16))
    assert 69e9 < big < 130e9


@pytest.mark.parametrize("field,value", [("n_groups", 2), ("d_conv", 3), ("n_kv_heads", 3), ("head_dim", 12),
                                         ("d_state", 24), ("kv_page_tokens", 48), ("w_dtype", 7),
                                         ("d_model", 60), ("max_batch", 0), ("struct_size", 8),
                                         ("overlap_mode", 4), ("attn_max_splits", 33), ("attn_target_blocks", 32), ("attn_single_slice_steps", -2),
                                         ("kernel_flags", 1 << 13), ("prefill_progress", -1), ("keep_logits", 2),
                                         ("use_graphs", -1)])
def test_bad_configs_are_rejected(B, field, value):
    cfg = B.make_cfg(W.WORKLOADS["c0"].cfg, 1, 128, 2, 64)
    setattr(cfg, field, value)
    assert B.hh_workspace_bytes(cfg) == 0
    hw = B.hh_weights()
    ctx = C.c_void_p()
    st = B.lib.hh_create(C.byref(hw), C.byref(cfg), C.byref(ctx))
    assert st == B.HH_EINVAL and not ctx.value
    assert B.hh_last_error(None)


def test_create_needs_workspace_and_weights(B):
    cfg = B.make_cfg(W.WORKLOADS["c0"].cfg, 1, 128, 2, 64)
    ctx = C.c_void_p()
    hw = B.hh_weights()
    assert B.lib.hh_create(C.byref(hw), C.byref(cfg), C.byref(ctx)) == B.HH_EINVAL      # NULL weights
    layers = (B.hh_layer_weights * 2)()
    for l in layers:
        for n, _ in B.hh_layer_weights._fields_:
            setattr(l, n, 256)
    hw.embed = hw.final_norm = hw.lm_head = 256
    hw.layers = layers
    assert B.lib.hh_create(C.byref(hw), C.byref(cfg), C.byref(ctx)) == B.HH_EWORKSPACE  # no workspace
    cfg.workspace, cfg.workspace_bytes = 4096 + 8, 1 << 40                               # misaligned
    assert B.lib.hh_create(C.byref(hw), C.byref(cfg), C.byref(ctx)) == B.HH_EWORKSPACE
    cfg.workspace, cfg.workspace_bytes = 4096, 1024                                       # too small
    assert B.lib.hh_create(C.byref(hw), C.byref(cfg), C.byref(ctx)) == B.HH_EWORKSPACE
    assert "workspace" in B.hh_last_error(None)
    assert B.lib.hh_destroy(None) == B.HH_EINVAL
    assert B.lib.hh_draft(None, 1, None) == B.HH_EINVAL


def test_stand_alone_token_choice_rejects_bad_arguments(B):
    """hh_draw_tokens / hh_accept_tokens validate on the host before any launch: NULL pointers, a
    row stride below the vocabulary, an unknown purpose, and temperatures that are not finite
    and > 0 (temperature 0 is the greedy path of the context calls, not a draw)."""
    fake = C.c_void_p(256)          # never dereferenced: every call below fails validation first
    def draw(logits=fake, stride=16, vocab=16, rows=1, t=0.5, purpose=2, out=fake):
        return B.lib.hh_draw_tokens(logits, stride, vocab, rows, C.c_float(t), C.c_uint64(1), None, 0, purpose, out, None)
    assert draw(logits=None) == B.HH_EINVAL
    assert draw(out=None) == B.HH_EINVAL
    assert draw(stride=8) == B.HH_EINVAL
    assert draw(vocab=0) == B.HH_EINVAL
    assert draw(purpose=9) == B.HH_EINVAL
    for t in (0.0, -1.0, float("inf"), float("nan")):
        assert draw(t=t) == B.HH_EINVAL
    def accept(dl=fake, vl=fake, k=2, drafts=fake, pos=fake, t=0.5, scratch=fake, targets=fake):
        return B.lib.hh_accept_tokens(dl, vl, 16, 1, k, drafts, pos, C.c_float(t), C.c_uint64(1), scratch, targets, None)
    assert accept(vl=None) == B.HH_EINVAL
    assert accept(dl=None) == B.HH_EINVAL            # k > 0 needs the draft rows and the drafts
    assert accept(drafts=None) == B.HH_EINVAL
    assert accept(pos=None) == B.HH_EINVAL
    assert accept(scratch=None) == B.HH_EINVAL
    assert accept(targets=None) == B.HH_EINVAL
    assert accept(k=-1) == B.HH_EINVAL
    assert accept(t=0.0) == B.HH_EINVAL
    def accept_static(dl=fake, vl=fake, k=2, drafts=fake, pos=fake, t=0.5, targets=fake):
        return B.lib.hh_accept_tokens_static(dl, vl, 16, 1, k, drafts, pos, C.c_float(t), C.c_uint64(1), targets, None)
    assert accept_static(vl=None) == B.HH_EINVAL
    assert accept_static(dl=None) == B.HH_EINVAL
    assert accept_static(targets=None) == B.HH_EINVAL
    assert accept_static(k=-1) == B.HH_EINVAL
    assert accept_static(t=float("nan")) == B.HH_EINVAL
    assert "hh_accept_tokens_static" in B.hh_last_error(None)


def test_optimal_draft_length_matches_the_oracle(B):
    """hh_optimal_draft_length against the oracle's maximiser of Eq. 1 on a grid; bad arguments give -1."""
    from oracle.protocol import optimal_draft_length
    for alpha in (0.0, 0.3, 0.68, 0.9, 0.97, 1.0):
        for c in (0.0, 0.05, 0.2, 0.5, 0.784, 1.0):
            for cand in ([2, 4, 8], list(range(0, 17)), [8, 1, 3]):
                assert B.hh_optimal_draft_length(alpha, c, cand) == optimal_draft_length(alpha, c, cand), (alpha, c, cand)
    assert B.hh_optimal_draft_length(1.5, 0.5, [1, 2]) == -1
    assert B.hh_optimal_draft_length(0.5, -1.0, [1, 2]) == -1
    assert B.hh_optimal_draft_length(0.5, 0.5, [1, -2]) == -1


def test_context_calls_reject_a_null_context(B):
    """Every entry point that takes a context returns HH_EINVAL for NULL before touching anything."""
    import ctypes as C
    i32 = (C.c_int32 * 4)()
    f32 = (C.c_float * 4)()
    u64a, u64b = C.c_uint64(0), C.c_uint64(0)
    n = C.c_int32(0)
    L = B.lib
    assert L.hh_prefill(None, None, 1, i32, 1, 1, None) == B.HH_EINVAL
    assert L.hh_set_sampling(None, C.c_float(0.5), C.c_uint64(1), None) == B.HH_EINVAL
    assert L.hh_draft(None, 1, None) == B.HH_EINVAL
    assert L.hh_set_drafts(None, None, None) == B.HH_EINVAL
    assert L.hh_set_draft_mask(None, i32) == B.HH_EINVAL
    assert L.hh_verify(None, None) == B.HH_EINVAL
    assert L.hh_commit(None, None, None) == B.HH_EINVAL
    assert L.hh_get_tokens(None, 0, i32, 4, C.byref(n), None) == B.HH_EINVAL
    assert L.hh_get_lengths(None, i32, i32, i32, None) == B.HH_EINVAL
    assert L.hh_get_round(None, i32, i32, None) == B.HH_EINVAL
    assert L.hh_get_acceptance(None, C.byref(u64a), C.byref(u64b), None) == B.HH_EINVAL
    assert L.hh_check_canaries(None, C.byref(n), None) == B.HH_EINVAL
    assert L.hh_get_logits(None, 0, f32, None) == B.HH_EINVAL
    assert L.hh_get_state(None, 0, f32, f32, None) == B.HH_EINVAL
    assert L.hh_get_draft_state(None, 0, f32, f32, None) == B.HH_EINVAL
    assert L.hh_get_kv(None, 0, 0, 1, f32, f32, None) == B.HH_EINVAL
    assert L.hh_profile(None, 1) == B.HH_EINVAL
    assert L.hh_profile_read(None, 4, i32, f32, None) == B.HH_EINVAL
    assert L.hh_time_kind(None, 1, 0, 1, 1, f32, i32, None) == B.HH_EINVAL
    assert L.hh_destroy(None) == B.HH_EINVAL
    assert B.hh_last_error(None) is not None


def test_workspace_grows_with_the_strict_state_and_the_guards(B):
    """draft_state_mode = 1 adds a second recurrent state and ring per layer; HH_KF_CANARIES adds 256 bytes
    (plus alignment) behind every region."""
    c2 = W.WORKLOADS["c2"]
    base = B.hh_workspace_bytes(B.make_cfg(c2.cfg, 16, 2048 + 300, 4, 256))
    strict = B.hh_workspace_bytes(B.make_cfg(c2.cfg, 16, 2048 + 300, 4, 256, draft_state_mode=1))
    guarded = B.hh_workspace_bytes(B.make_cfg(c2.cfg, 16, 2048 + 300, 4, 256, kernel_flags=B.HH_KF_CANARIES))
    state = 36 * 16 * 24 * 64 * 128 * 4
    ring = 36 * 16 * 512 * (1536 + 2 * 128 + 24) * 4      # 512 slots: the next power of two above the 256-position prefill pass + 3
    assert state + ring <= strict - base < state + ring + (1 << 20)
    assert 0 < guarded - base < 1 << 20
