"""Pins for the oracle's selection step: brute force on small inputs, edge cases.  CPU only."""
import numpy as np
import pytest

import oracle
from paper_2411_18873_amd import synth


def _brute(energy, latency, legal, k, alpha=None, m_latency=None):
    """Independent reference with python sorting on (value, index) tuples."""
    n = len(energy)
    ok = [bool(legal[i]) if legal is not None else True for i in range(n)]
    if latency is not None:
        cand = [i for i in range(n) if ok[i] and not np.isnan(latency[i])]
        if m_latency is None:
            if cand:
                lmin = np.float32(min(latency[i] for i in cand))
                if np.isinf(alpha):
                    tau = np.float32(np.inf)
                else:
                    slack = np.float32(np.float32(alpha) - np.float32(1.0)) * np.abs(lmin)
                    tau = np.float32(lmin + np.float32(slack))
                keep = {i for i in cand if latency[i] <= tau}
            else:
                keep = set()
        else:
            order = sorted(cand, key=lambda i: (latency[i], i))
            keep = set(order[:m_latency])
        ok = [ok[i] and i in keep for i in range(n)]
    feas = [i for i in range(n) if ok[i] and not np.isnan(energy[i])]
    feas.sort(key=lambda i: (energy[i], i))
    return feas[:k]


@pytest.mark.parametrize("seed", range(6))
def test_threshold_mode_bruteforce(seed):
    n, k = 500, 16
    e = synth.gaussian_scores(n, seed, ties=0.2, quantum=0.05)
    lat = synth.gaussian_scores(n, seed + 100) * 0.2 + (3.0 if seed % 2 == 0 else -3.0)  # positive and negative latencies
    legal = synth.legal_mask(n, seed + 200, 0.6)
    idx, eo, cnt = oracle.topk(e, lat, legal, 1, k, oracle.SEL_THRESHOLD, alpha=1.1)
    want = _brute(e, lat, legal, k, alpha=1.1)
    assert cnt[0] == len(want)
    assert list(idx[0, :cnt[0]]) == want
    assert np.array_equal(eo[0, :cnt[0]], e[want])
    assert np.all(idx[0, cnt[0]:] == 0xFFFFFFFF) and np.all(np.isinf(eo[0, cnt[0]:]))


def test_plain_topk_equals_sort_and_alpha_inf():
    n, k = 4096, 64
    e = synth.gaussian_scores(n, 11, ties=0.3)
    idx, eo, cnt = oracle.topk(e, None, None, 1, k)
    order = np.lexsort((np.arange(n), e))[:k]
    assert np.array_equal(idx[0], order.astype(np.uint32)) and cnt[0] == k
    lat = synth.gaussian_scores(n, 12)
    idx2, _, _ = oracle.topk(e, lat, None, 1, k, oracle.SEL_THRESHOLD, alpha=float("inf"))
    assert np.array_equal(idx2, idx)


def test_segments_are_independent_and_indices_are_local():
    S, L, k = 8, 256, 8
    e = synth.gaussian_scores(S * L, 21)
    lat = np.abs(synth.gaussian_scores(S * L, 22)) + 1
    legal = synth.legal_mask(S * L, 23, 0.5)
    idx, eo, cnt = oracle.topk(e, lat, legal, S, k, alpha=1.5)
    for s in range(S):
        sl = slice(s * L, (s + 1) * L)
        i1, e1, c1 = oracle.topk(e[sl], lat[sl], legal[sl], 1, k, alpha=1.5)
        assert np.array_equal(idx[s], i1[0]) and c1[0] == cnt[s]
        assert list(idx[s, :cnt[s]]) == _brute(e[sl], lat[sl], legal[sl], k, alpha=1.5)


def test_all_equal_scores_give_lowest_indices():
    e = np.full(100, 2.5, dtype=np.float32)
    idx, _, cnt = oracle.topk(e, None, None, 1, 10)
    assert list(idx[0]) == list(range(10)) and cnt[0] == 10


def test_fewer_feasible_than_k_pads():
    e = np.arange(20, dtype=np.float32)[::-1].copy()
    legal = np.zeros(20, dtype=np.uint8)
    legal[[3, 7, 11]] = 1
    idx, eo, cnt = oracle.topk(e, None, legal, 1, 5)
    assert cnt[0] == 3 and list(idx[0, :3]) == [11, 7, 3]
    assert list(idx[0, 3:]) == [0xFFFFFFFF] * 2 and np.all(np.isinf(eo[0, 3:]))
    idx, eo, cnt = oracle.topk(e, None, np.zeros(20, dtype=np.uint8), 1, 5)
    assert cnt[0] == 0 and np.all(idx == 0xFFFFFFFF)


def test_nan_and_signed_zero():
    e = np.array([0.0, -0.0, np.nan, -1.0, 1.0], dtype=np.float32)
    idx, _, cnt = oracle.topk(e, None, None, 1, 5)
    assert cnt[0] == 4 and list(idx[0, :4]) == [3, 1, 0, 4]  # -1 < -0 < +0 < 1; NaN never selected
    lat = np.array([1.0, np.nan, 1.0, 1.0, 1.05], dtype=np.float32)
    idx, _, cnt = oracle.topk(e, lat, None, 1, 5, alpha=1.1)
    assert list(idx[0, :cnt[0]]) == [3, 0, 4]  # NaN latency infeasible


def test_threshold_worked_example():
    # latencies 10, 10.9, 11.0, 11.1, 12; alpha 1.1 -> tau = 10 + fl(0.1f*10) keeps everything <= tau
    lat = np.array([10, 10.9, 11.0, 11.1, 12], dtype=np.float32)
    e = np.array([5, 4, 3, 2, 1], dtype=np.float32)
    tau = np.float32(10) + np.float32(np.float32(1.1) - np.float32(1)) * np.float32(10)
    idx, _, cnt = oracle.topk(e, lat, None, 1, 2, alpha=1.1)
    want = [i for i in (4, 3, 2, 1, 0) if lat[i] <= tau][:2]
    assert list(idx[0, :cnt[0]]) == want and 2 in want and 4 not in want
    # the illegal fastest candidate does not set the threshold
    legal = np.array([0, 1, 1, 1, 1], dtype=np.uint8)
    idx, _, cnt = oracle.topk(e, lat, legal, 1, 5, alpha=1.1)
    assert list(idx[0, :cnt[0]]) == [3, 2, 1]  # tau = 1.1*10.9 = 11.99 excludes 12


@pytest.mark.parametrize("seed", range(4))
def test_rank_mode_bruteforce(seed):
    n, k, m = 300, 10, 40
    e = synth.gaussian_scores(n, seed, ties=0.2, quantum=0.1)
    lat = synth.gaussian_scores(n, seed + 50, quantum=0.1)
    legal = synth.legal_mask(n, seed + 60, 0.7)
    idx, eo, cnt = oracle.topk(e, lat, legal, 1, k, oracle.SEL_RANK, m_latency=m)
    want = _brute(e, lat, legal, k, m_latency=m)
    assert list(idx[0, :cnt[0]]) == want and cnt[0] == len(want)
    # "parents = lower-energy half of the fastest M": k = M/2
    idx, _, cnt = oracle.topk(e, lat, legal, 1, m // 2, oracle.SEL_RANK, m_latency=m)
    assert list(idx[0, :cnt[0]]) == _brute(e, lat, legal, m // 2, m_latency=m)


def test_selected_set_is_permutation_invariant():
    n, k = 1000, 32
    e = synth.gaussian_scores(n, 31)  # distinct with probability ~1
    assert len(np.unique(e)) == n
    lat = np.abs(synth.gaussian_scores(n, 32)) + 1
    perm = np.random.default_rng(33).permutation(n)
    idx, _, c1 = oracle.topk(e, lat, None, 1, k, alpha=1.3)
    idxp, _, c2 = oracle.topk(e[perm], lat[perm], None, 1, k, alpha=1.3)
    assert c1[0] == c2[0]
    assert list(perm[idxp[0, :c2[0]]]) == list(idx[0, :c1[0]])
