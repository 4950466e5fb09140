"""The acceptance entry point that allocates nothing (hh_accept_tokens_static: per-row statistics in
an array built into the library) against hh_accept_tokens (statistics in a caller-provided buffer),
through the C ABI: same kernels, so the targets rows must be identical.  Two calls in a row on one
GPU, the second with a smaller input, so that whatever the first call left in the shared array lies
beside and behind what the second one uses."""
import numpy as np
import pytest

from paper_2605_01106_amd import workloads as W

pytestmark = pytest.mark.gpu


def _round(B, batch, k, vocab, T, seed, dev):
    import torch
    draft, verify = W.make_logit_rows(batch, k, vocab, seed)
    rng = np.random.default_rng(seed)
    drafts = rng.integers(0, vocab, (batch, max(k, 1)), dtype=np.int32)
    # half of the drafts are the verification row's most likely token (mostly kept), the rest random (mostly rejected)
    for b in range(0, batch, 2):
        for i in range(k):
            drafts[b, i] = int(np.argmax(verify[b, i]))
    positions = (np.arange(batch, dtype=np.int32) * 5 + 2)
    d_dev = torch.from_numpy(draft).to(dev) if k else None
    v_dev = torch.from_numpy(verify).to(dev)
    dr_dev = torch.from_numpy(np.ascontiguousarray(drafts[:, :k])).to(dev) if k else None
    pos_dev = torch.from_numpy(positions).to(dev)
    want = B.hh_accept_tokens(d_dev, v_dev, dr_dev, pos_dev, T, seed)
    got = torch.full((batch, k + 1), -7, dtype=torch.int32, device=dev)      # allocated by the caller, before the call
    torch.cuda.synchronize()
    B.hh_accept_tokens_static(d_dev, v_dev, dr_dev, pos_dev, got, T, seed)
    torch.cuda.synchronize()
    return want.cpu().numpy(), got.cpu().numpy()


def test_static_scratch_matches_workspace_variant_twice():
    import torch
    from paper_2605_01106_amd import binding as B
    dev = torch.device("cuda:0")
    kept = set()
    for batch, k, vocab, T, seed in [(48, 8, 4099, 0.6, 5), (7, 3, 1000, 0.9, 6)]:   # the second call is smaller
        want, got = _round(B, batch, k, vocab, T, seed, dev)
        assert np.array_equal(want, got), (batch, k, np.argwhere(want != got)[:4])
        for row in got:
            n = int(np.max(np.nonzero(row >= 0)[0]))
            assert 0 <= row[n] < vocab and all(v == -1 for v in row[n + 1:])
            kept.add(n)
    assert len(kept) > 2          # kept and rejected drafts both occurred


def test_static_scratch_capacity_and_arguments():
    import torch
    from paper_2605_01106_amd import binding as B
    dev = torch.device("cuda:0")
    # batch * (2k + 1) * 2 floats of statistics beyond the built-in 65536: refused before any launch
    batch, k, vocab = 4000, 4, 8
    v = torch.zeros((batch, k + 1, vocab), dtype=torch.float32, device=dev)
    d = torch.zeros((batch, k, vocab), dtype=torch.float32, device=dev)
    dr = torch.zeros((batch, k), dtype=torch.int32, device=dev)
    pos = torch.zeros(batch, dtype=torch.int32, device=dev)
    out = torch.full((batch, k + 1), -7, dtype=torch.int32, device=dev)
    with pytest.raises(B.HHError) as ei:
        B.hh_accept_tokens_static(d, v, dr, pos, out, 0.7, 1)
    assert ei.value.status == B.HH_ECAPACITY and "65536" in str(ei.value)
    torch.cuda.synchronize()
    assert int((out != -7).sum()) == 0
    with pytest.raises(B.HHError) as ei:
        B.hh_accept_tokens_static(d, v, dr, pos, out, 0.0, 1)
    assert ei.value.status == B.HH_EINVAL
