"""GPU: costmodel_score_min (scores plus the least legal score of every segment, Alg. 1 LatencyEvaAndPick / the latency
gate of Sec. 4.3) and topk_select_known_min, the selection that takes those minima instead of reading the latencies twice.

The scores must be the bits costmodel_score writes; the minima are integer work on those bits and are compared exactly
with numpy's minimum over the legal, non-NaN scores of each segment; the selection must equal the oracle's."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_18873_amd import eck, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _key(x):
    """order-preserving uint32 key of a float32, as the header defines it"""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return np.where(b >> 31 != 0, ~b, b | np.uint32(0x80000000)).astype(np.uint32)


def _want_keys(scores, legal, S):
    n = scores.size
    keys = _key(scores)
    dead = np.isnan(scores)
    if legal is not None:
        dead |= legal[:n] == 0
    keys = np.where(dead, np.uint32(0xFFFFFFFF), keys)
    return keys.reshape(S, n // S).min(axis=1)


def _score_min(G, model, feat_dev, n, legal, S):
    out = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    lg = None if legal is None else G.to_dev(np.ascontiguousarray(legal, dtype=np.uint8))
    keys = torch.full((S,), 12345, dtype=torch.int32, device="cuda")
    eck.costmodel_score_min(model, feat_dev, n, out, lg, S, keys)
    torch.cuda.synchronize()
    return out.cpu().numpy(), keys.cpu().numpy().view(np.uint32)


def _features(n, n_feat, seed=3):
    pb = synth.CONFIGS["c2"]["problem"]
    ref = oracle.Space(pb, oracle.SPACE_SPLIT)
    genes = oracle.enumerate_candidates(ref, oracle.MODE_SAMPLE, n, seed=seed)
    _, f32, b16, _ = oracle.features(ref, genes, n_feat)
    return f32, b16


# segments of 3000/24 = 125 and 9984/96 = 104 candidates start inside wavefronts' groups of 64 or 128 candidates;
# segments of 2048 and 1024 candidates are whole tiles (the kernel's 32-bit bookkeeping), and with 2^18 candidates a
# block's consecutive tiles lie 64 segments apart
@pytest.mark.parametrize("widths", [[64, 512, 512, 1], [64, 256, 256, 1], [64, 128, 128, 1], [32, 64, 64, 1]])
@pytest.mark.parametrize("n,ld,S", [(3000, 3000, 1), (3000, 3000, 24), (2998, 2998, 2), (9984, 10000, 96), (1001, 1002, 7),
                                    (64, 64, 64), (5, 6, 1), (8192, 8192, 4), (1 << 18, 1 << 18, 256)])
def test_bf16_models(G, widths, n, ld, S):
    f32, b16 = _features(ld, widths[0])
    theta = synth.mlp_theta(widths, 8, bf16=True, bias_scale=0.5)
    model = G.make_model(widths, eck.BF16, theta)
    legal = synth.legal_mask(ld, 5, 0.4)
    legal[: n // S] = 0 if S > 2 else legal[: n // S]        # with several segments the first has no legal candidate
    for dev in (G.bf16_dev(b16), G.to_dev(f32)):
        plain = G.score_gpu(model, dev, n)
        for lg in (legal, None):
            got, keys = _score_min(G, model, dev, n, lg, S)
            assert np.array_equal(got.view(np.uint32), plain.view(np.uint32))
            assert np.array_equal(keys, _want_keys(plain, lg, S))
        if S > 2:
            assert _want_keys(plain, legal, S)[0] == 0xFFFFFFFF


def test_fp32_model(G):
    widths = synth.CONFIGS["c1"]["widths"]
    pb = synth.CONFIGS["c1"]["problem"]
    ref = oracle.Space(pb, oracle.SPACE_KNOB)
    genes = oracle.enumerate_candidates(ref, oracle.MODE_EXHAUSTIVE, 6400)
    _, f32, _, _ = oracle.features(ref, genes, 32)
    theta = synth.mlp_theta(widths, 2, bias_scale=0.3)
    model = G.make_model(widths, eck.F32, theta)
    dev = G.to_dev(f32)
    plain = G.score_gpu(model, dev, 6400)
    legal = synth.legal_mask(6400, 9, 0.3)
    for S in (1, 5, 100):
        for lg in (legal, None):
            got, keys = _score_min(G, model, dev, 6400, lg, S)
            assert np.array_equal(got.view(np.uint32), plain.view(np.uint32))
            assert np.array_equal(keys, _want_keys(plain, lg, S))


@pytest.mark.parametrize("dtype,widths", [(eck.BF16, [64, 256, 256, 1]), (eck.F32, [32, 64, 64, 1])])
def test_scores_that_are_not_numbers_never_become_the_minimum(G, dtype, widths):
    f32, b16 = _features(2048, widths[0])
    theta = synth.mlp_theta(widths, 4, bf16=dtype == eck.BF16)
    theta[-1] = np.nan                                                  # the output bias: every score is NaN
    model = G.make_model(widths, dtype, theta)
    got, keys = _score_min(G, model, G.bf16_dev(b16) if dtype == eck.BF16 else G.to_dev(f32), 2048, None, 4)
    assert np.isnan(got).all() and np.all(keys == 0xFFFFFFFF)


def test_argument_checks(G):
    import ctypes as C
    widths = [64, 256, 256, 1]
    _, b16 = _features(1024, 64)
    model = G.make_model(widths, eck.BF16, synth.mlp_theta(widths, 4, bf16=True))
    dev = G.bf16_dev(b16)
    out = torch.zeros(1024, dtype=torch.float32, device="cuda")
    keys = torch.zeros(8, dtype=torch.int32, device="cuda")
    legal = torch.ones(1026, dtype=torch.uint8, device="cuda")
    L = eck.lib()
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t, off=0: C.c_void_p(t.data_ptr() + off)
    call = lambda n, lg, S, k: L.costmodel_score_min(model.h, p(dev), eck.BF16, 1024, n, p(out), lg, S, k, st)
    assert call(1024, p(legal), 8, None) == eck.EINVAL
    assert call(1024, p(legal), 0, p(keys)) == eck.EINVAL
    assert call(1000, p(legal), 7, p(keys)) == eck.ESHAPE
    assert call(1024, p(legal, 1), 8, p(keys)) == eck.EALIGN
    assert call(1024, p(legal, 2), 8, p(keys)) == eck.OK                 # flags aligned to 2: two candidates per load
    torch.cuda.synchronize()


@pytest.mark.parametrize("n,S,k", [(1 << 16, 1, 64), (3000 * 16, 16, 32), (1 << 18, 4, 1024)])
def test_selection_with_known_minima(G, n, S, k):
    """latencies from a model, minima from the same launch, selection without a second pass over the latencies:
    the oracle's selection on the same scores, and topk_select's, bit for bit"""
    widths = [64, 256, 256, 1]
    _, b16 = _features(n, 64, seed=11)
    lat_model = G.make_model(widths, eck.BF16, synth.mlp_theta(widths, 21, bf16=True, bias_scale=0.5))
    legal = synth.legal_mask(n, 3, 0.4)
    lg = G.to_dev(legal)
    lat = torch.empty(n, dtype=torch.float32, device="cuda")
    keys = torch.empty(S, dtype=torch.int32, device="cuda")
    eck.costmodel_score_min(lat_model, G.bf16_dev(b16), n, lat, lg, S, keys)
    e = synth.gaussian_scores(n, 1, ties=0.3, quantum=0.01)
    e_dev = G.to_dev(e)
    lat_np = lat.cpu().numpy()
    for alpha in (1.1, 1.0, 3.0, float("inf")):
        idx = torch.zeros((S, k), dtype=torch.int32, device="cuda")
        eo = torch.zeros((S, k), dtype=torch.float32, device="cuda")
        cnt = torch.zeros((S,), dtype=torch.int32, device="cuda")
        ws = torch.empty(eck.topk_select_workspace_bytes(n, S, k), dtype=torch.uint8, device="cuda")
        eck.topk_select_known_min(e_dev, lat, lg, S, k, keys, idx, eo, cnt, ws, alpha=alpha)
        torch.cuda.synchronize()
        got = (idx.cpu().numpy().view(np.uint32), eo.cpu().numpy(), cnt.cpu().numpy().view(np.uint32))
        want = oracle.topk(e, lat_np, legal, S, k, alpha=alpha)
        two_pass = G.topk_dev(e_dev, lat, lg, S, k, alpha=alpha)
        for other in (want, two_pass):
            assert np.array_equal(got[2], other[2])
            assert np.array_equal(got[0], other[0])
            assert np.array_equal(got[1].view(np.uint32), other[1].view(np.uint32))
