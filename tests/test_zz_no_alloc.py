"""topk_select_static -- the entry point for callers that cannot allocate -- against topk_select, through the C ABI:
indices, values and counts bit for bit, on two calls in a row (the second on a smaller input, so that whatever the
first left in the library's fixed workspace is still there), in every selection mode; sizes beyond the fixed
workspace are refused."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2411_18873_amd import eck, synth

pytestmark = pytest.mark.gpu


def _outputs(S, k):
    return (torch.full((S, k), -7, dtype=torch.int32, device="cuda"), torch.full((S, k), -7.0, dtype=torch.float32, device="cuda"),
            torch.full((S,), -7, dtype=torch.int32, device="cuda"))


def _both(e, lat, legal, S, k, **kw):
    want = _outputs(S, k)
    m = kw.get("m_latency", 0) if kw.get("mode", eck.SELECT_THRESHOLD) == eck.SELECT_RANK else 0
    ws = torch.empty(eck.topk_select_workspace_bytes(e.numel(), S, k, m_latency=m), dtype=torch.uint8, device="cuda")
    eck.topk_select(e, lat, legal, S, k, *want, ws, **kw)
    got = _outputs(S, k)
    eck.topk_select_static(e, lat, legal, S, k, *got, **kw)
    torch.cuda.synchronize()
    for g, w in zip(got, want):
        assert np.array_equal(g.cpu().numpy().view(np.uint32), w.cpu().numpy().view(np.uint32))
    return int(got[2].sum().item())


def test_static_workspace_entry_point_matches_topk_select_on_consecutive_calls():
    dev = "cuda"
    n1, S1, k1 = 1 << 20, 16, 32
    e = torch.from_numpy(synth.gaussian_scores(n1, 41, ties=0.3, quantum=0.01)).to(dev)
    lat = torch.from_numpy(synth.gaussian_scores(n1, 42) * 0.3 + 2.0).to(dev)
    legal = torch.from_numpy(synth.legal_mask(n1, 43, 0.5)).to(dev)
    # first call: several levels, every mode
    assert _both(e, lat, legal, S1, k1, alpha=float("inf")) == S1 * k1
    _both(e, lat, legal, S1, k1, alpha=1.1)
    _both(e, None, legal, S1, k1)
    _both(e, lat, legal, S1, k1, mode=eck.SELECT_RANK, m_latency=500)
    # second call in a row on a smaller input (one level, fewer segments, other k): stale lists of the first
    # call are still in the workspace and must not matter
    n2, S2, k2 = 6400, 2, 100
    _both(e[:n2].contiguous(), lat[:n2].contiguous(), legal[:n2].contiguous(), S2, k2, alpha=1.5)
    _both(e[:n2].contiguous(), lat[:n2].contiguous(), None, S2, k2, mode=eck.SELECT_RANK, m_latency=300)
    # and a larger one again
    assert _both(e, lat, None, 1, 1024, alpha=float("inf")) == 1024


def test_static_workspace_entry_point_refuses_what_does_not_fit():
    L = eck.lib()
    n = 1 << 24
    assert eck.topk_select_workspace_bytes(n, 1, 4096) > eck.TOPK_STATIC_BYTES
    e = torch.zeros(n, dtype=torch.float32, device="cuda")
    idx, eo, cnt = _outputs(1, 4096)
    p = lambda t: C.c_void_p(t.data_ptr())
    rc = L.topk_select_static(p(e), None, None, n, 1, 4096, eck.SELECT_THRESHOLD, 1.1, 0, p(idx), p(eo), p(cnt), None)
    assert rc == eck.EWORKSPACE
    # the ordinary argument checks come first
    assert L.topk_select_static(p(e), None, None, n, 1, 0, eck.SELECT_THRESHOLD, 1.1, 0, p(idx), p(eo), p(cnt), None) == eck.EINVAL
    assert L.topk_select_static(p(e), None, None, n, 3, 16, eck.SELECT_THRESHOLD, 1.1, 0, p(idx), p(eo), p(cnt), None) == eck.ESHAPE
    torch.cuda.synchronize()
    assert int(cnt.item()) == -7          # a refused call touches nothing
    # the benchmark's selection fits
    assert eck.topk_select_workspace_bytes(1 << 24, 64, 32) <= eck.TOPK_STATIC_BYTES
