"""GPU parity: topk_select against the oracle -- indices, values and counts bit for bit."""
import numpy as np
import pytest

import oracle
from paper_2411_18873_amd import eck, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _same(got, want):
    gi, ge, gc = got
    wi, we, wc = want
    assert np.array_equal(gc, wc)
    assert np.array_equal(gi, wi)
    assert np.array_equal(ge.view(np.uint32), we.view(np.uint32))


@pytest.mark.parametrize("n,S,k,ties", [(6400, 1, 16, 0.0), (1 << 16, 1, 64, 0.3), ((1 << 16) + 8 * 13, 8, 32, 0.5),
                                        (50000, 1, 1024, 0.9), (4096, 64, 32, 0.2), (100, 1, 100, 0.0), (7, 7, 1, 0.0)])
def test_threshold_mode(G, n, S, k, ties):
    e = synth.gaussian_scores(n, 1, ties=ties, quantum=0.01 if ties else None)
    lat = synth.gaussian_scores(n, 2, ties=ties / 2) * 0.3 + 2.0
    legal = synth.legal_mask(n, 3, 0.4)
    for alpha in (1.1, 1.0, 2.5, float("inf")):
        _same(G.topk_gpu(e, lat, legal, S, k, alpha=alpha), oracle.topk(e, lat, legal, S, k, alpha=alpha))
    _same(G.topk_gpu(e, lat, None, S, k), oracle.topk(e, lat, None, S, k))
    _same(G.topk_gpu(e, None, legal, S, k), oracle.topk(e, None, legal, S, k))
    _same(G.topk_gpu(e, None, None, S, k), oracle.topk(e, None, None, S, k))


def test_negative_latencies_and_mixed_signs(G):
    n = 30000
    e = synth.gaussian_scores(n, 5)
    for shift in (-3.0, 0.0):
        lat = synth.gaussian_scores(n, 6) * 0.2 + shift
        legal = synth.legal_mask(n, 7, 0.5)
        _same(G.topk_gpu(e, lat, legal, 1, 64, alpha=1.1), oracle.topk(e, lat, legal, 1, 64, alpha=1.1))


def test_degenerate_inputs(G):
    n = 20000
    const = np.full(n, 2.5, dtype=np.float32)
    _same(G.topk_gpu(const, None, None, 1, 100), oracle.topk(const, None, None, 1, 100))           # all equal
    _same(G.topk_gpu(const, const, None, 4, 50), oracle.topk(const, const, None, 4, 50))
    e = synth.gaussian_scores(n, 8)
    none_legal = np.zeros(n, dtype=np.uint8)
    _same(G.topk_gpu(e, e, none_legal, 2, 10), oracle.topk(e, e, none_legal, 2, 10))                 # nothing feasible
    few = none_legal.copy()
    few[[5, 77, 19999]] = 1
    _same(G.topk_gpu(e, None, few, 1, 10), oracle.topk(e, None, few, 1, 10))                         # fewer than k
    # NaN, infinities, signed zeros, denormals
    sp = e.copy()
    sp[::7] = np.nan
    sp[1::11] = -0.0
    sp[2::11] = 0.0
    sp[3::13] = -np.inf
    sp[4::13] = np.inf
    sp[5::17] = 1e-42
    lat = np.abs(synth.gaussian_scores(n, 9)) + 0.5
    lat[::5] = np.nan
    _same(G.topk_gpu(sp, lat, None, 1, 4000, alpha=3.0), oracle.topk(sp, lat, None, 1, 4000, alpha=3.0))
    _same(G.topk_gpu(sp, None, None, 1, 4096), oracle.topk(sp, None, None, 1, 4096))
    # two distinct values only: the k-th falls inside a huge tie
    two = (np.arange(n) % 3 == 0).astype(np.float32)
    _same(G.topk_gpu(two, None, None, 1, 4096), oracle.topk(two, None, None, 1, 4096))


@pytest.mark.parametrize("n,S,k,m", [(20000, 1, 50, 500), (1 << 15, 4, 64, 128), (3000, 1, 16, 5000), (5000, 1, 100, 100)])
def test_rank_mode(G, n, S, k, m):
    e = synth.gaussian_scores(n, 11, ties=0.3, quantum=0.05)
    lat = synth.gaussian_scores(n, 12, ties=0.3, quantum=0.05)
    legal = synth.legal_mask(n, 13, 0.6)
    _same(G.topk_gpu(e, lat, legal, S, k, mode=eck.SELECT_RANK, m_latency=m),
          oracle.topk(e, lat, legal, S, k, mode=oracle.SEL_RANK, m_latency=m))
    _same(G.topk_gpu(e, lat, None, S, k, mode=eck.SELECT_RANK, m_latency=m),
          oracle.topk(e, lat, None, S, k, mode=oracle.SEL_RANK, m_latency=m))


def test_children_of_few_parents_tie_heavily(G):
    # like an evolutionary round: 2^18 children of 1024 parents, most of them exact copies
    rng = np.random.default_rng(0)
    parents_e = synth.gaussian_scores(1024, 14)
    parents_l = np.abs(synth.gaussian_scores(1024, 15)) + 1
    n = 1 << 18
    who = np.arange(n) % 1024
    mutated = rng.random(n) < 0.47
    e = np.where(mutated, synth.gaussian_scores(n, 16), parents_e[who]).astype(np.float32)
    lat = np.where(mutated, np.abs(synth.gaussian_scores(n, 17)) + 1, parents_l[who]).astype(np.float32)
    legal = synth.legal_mask(n, 18, 0.8)
    _same(G.topk_gpu(e, lat, legal, 1, 1024, alpha=1.1), oracle.topk(e, lat, legal, 1, 1024, alpha=1.1))


def test_repeatable(G):
    n = 1 << 18
    e = synth.gaussian_scores(n, 21, ties=0.5, quantum=0.001)
    lat = np.abs(synth.gaussian_scores(n, 22)) + 1
    a = G.topk_gpu(e, lat, None, 4, 512)
    b = G.topk_gpu(e, lat, None, 4, 512)
    _same(a, b)


def test_scalar_and_vector_streaming_paths_agree_with_the_oracle(G):
    """The streaming kernels read four candidates per load when segment length and pointers allow it and one
    per load otherwise: odd segment lengths, and score / flag arrays that start one element into an allocation,
    take the scalar path at a size that spans many blocks; the result is the oracle's either way."""
    import torch
    S, seg = 3, 123457                                   # odd segment length
    n = S * seg
    e = synth.gaussian_scores(n, 11, ties=0.2, quantum=0.01)
    lat = synth.gaussian_scores(n, 12) * 0.3 + 2.0
    legal = synth.legal_mask(n, 13, 0.5)
    want = oracle.topk(e, lat, legal, S, 200, alpha=1.1)
    _same(G.topk_gpu(e, lat, legal, S, 200, alpha=1.1), want)
    # aligned length, misaligned pointers: views that start at element 1
    n2 = 1 << 18
    e2, l2, g2 = e[:n2], lat[:n2], legal[:n2]
    want2 = oracle.topk(e2, l2, g2, 4, 77, alpha=1.1)
    pad_f = lambda a: torch.cat([torch.zeros(1, dtype=torch.float32), torch.from_numpy(a.copy())]).cuda()[1:]
    pad_b = torch.cat([torch.zeros(1, dtype=torch.uint8), torch.from_numpy(g2.copy())]).cuda()[1:]
    assert pad_f(e2).data_ptr() % 16 != 0
    _same(G.topk_dev(pad_f(e2), pad_f(l2), pad_b, 4, 77, alpha=1.1), want2)
    # and the aligned (vector) path on the same data
    _same(G.topk_gpu(e2, l2, g2, 4, 77, alpha=1.1), want2)


@pytest.mark.parametrize("n,S,k", [(1 << 22, 1, 4096), (1 << 22, 1, 300), (1 << 22, 1, 1), (3 * ((1 << 20) + 4), 3, 257),
                                   (1 << 21, 512, 16), (40000, 1, 4096)])
def test_selections_that_take_several_levels(G, n, S, k):
    """A block selects among 4096 (k <= 256 on a full chip) or 16384 candidates; longer segments go through
    further levels over the lists of the level before.  Sizes here take one to four levels, with k from 1 to the
    largest the library accepts, ties included so that index digits decide."""
    e = synth.gaussian_scores(n, 31, ties=0.4, quantum=0.02)
    lat = synth.gaussian_scores(n, 32) * 0.3 + 2.0
    legal = synth.legal_mask(n, 33, 0.7)
    _same(G.topk_gpu(e, None, legal, S, k), oracle.topk(e, None, legal, S, k))
    _same(G.topk_gpu(e, lat, legal, S, k, alpha=1.3), oracle.topk(e, lat, legal, S, k, alpha=1.3))
    m = min(4096, max(k, 1000))
    _same(G.topk_gpu(e, lat, legal, S, k, mode=eck.SELECT_RANK, m_latency=m),
          oracle.topk(e, lat, legal, S, k, mode=oracle.SEL_RANK, m_latency=m))


def test_rank_gate_limits_and_workspace(G):
    import ctypes as C
    import torch
    L = eck.lib()
    n = 1 << 16
    # a gate wider than the library's largest selection is refused unless it admits the whole segment anyway
    assert L.topk_select_rank_workspace_bytes(n, 1, 16, 5000) == 0
    assert L.topk_select_rank_workspace_bytes(n, 1, 16, n) > 0
    assert L.topk_select_rank_workspace_bytes(n, 1, 16, 0) == 0
    need = eck.topk_select_workspace_bytes(n, 1, 16, m_latency=4096)
    assert need >= eck.topk_select_workspace_bytes(n, 1, 16)
    e = torch.zeros(n, dtype=torch.float32, device="cuda")
    idx = torch.zeros(16, dtype=torch.int32, device="cuda")
    eo = torch.zeros(16, dtype=torch.float32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    p = lambda t: C.c_void_p(t.data_ptr())
    call = lambda m, ws_bytes: L.topk_select(p(e), p(e), None, n, 1, 16, eck.SELECT_RANK, 1.1, m, p(idx), p(eo), p(cnt),
                                             p(ws), ws_bytes, None)
    assert call(5000, need) == eck.EUNSUPPORTED
    assert call(4096, eck.topk_select_workspace_bytes(n, 1, 16) - 8) == eck.EWORKSPACE
    assert call(4096, need) == eck.OK and call(n, need) == eck.OK
    torch.cuda.synchronize()
    assert cnt.item() == 16 and idx.cpu().numpy().tolist() == list(range(16))
