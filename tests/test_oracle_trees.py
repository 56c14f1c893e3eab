"""Pins of the tree-ensemble oracle (prediction and boosting with the loss of Eq. (1)) against things other
than itself: a hand-walked ensemble, the closed-form result of a one-split fit, a brute-force search of the best
split, a library regression tree fitted to the same weighted problem, and the loss going down round by round."""
import numpy as np
import pytest

import oracle


def _empty(depth, n_trees):
    return (np.zeros((n_trees, (1 << depth) - 1), dtype=np.uint8),
            np.zeros((n_trees, (1 << depth) - 1), dtype=np.float32),
            np.zeros((n_trees, 1 << depth), dtype=np.float32))


def test_hand_walked_ensemble(golden):
    rows = golden("hand_trees.txt")
    base = float(rows[0][0])
    trees = [[float(t) for t in r] for r in rows[1:3]]
    nf = np.array([t[0:3] for t in trees], dtype=np.uint8)
    nt = np.array([t[3:6] for t in trees], dtype=np.float32)
    lf = np.array([t[6:10] for t in trees], dtype=np.float32)
    cases = np.array([[float(t) for t in r] for r in rows[3:]], dtype=np.float64)
    feat = np.ascontiguousarray(cases[:, :3].T, dtype=np.float32)
    got = oracle.trees_predict(3, 2, nf, nt, lf, base, feat)
    assert np.allclose(got, cases[:, 3], rtol=0, atol=1e-6)
    got32 = oracle.trees_predict(3, 2, nf, nt, lf, base, feat, fp32_sequential=True)
    assert np.allclose(got32, cases[:, 3], rtol=0, atol=1e-6)


def test_one_split_fit_gives_the_harmonic_means():
    """One feature with two well separated groups, depth 1, eta = 1, lambda = 0: the Newton step of a quadratic
    loss lands on the minimiser, which for sum (p - y)^2 / y over a group is n / sum(1/y): the harmonic mean."""
    rng = np.random.default_rng(5)
    e = rng.uniform(0.5, 4.0, size=60).astype(np.float32)
    x = np.where(np.arange(60) % 3 == 0, 0.1, 10.1).astype(np.float32)[None, :]
    nf, nt, lf = _empty(1, 1)
    snr, loss = oracle.trees_boost(1, 1, nf, nt, lf, 0, 1, 0.5, x, e, eta=1.0, lam=0.0)
    y = (e / e.max()).astype(np.float64)
    left = x[0] < 5
    hm_left, hm_right = left.sum() / (1 / y[left]).sum(), (~left).sum() / (1 / y[~left]).sum()
    assert nf[0, 0] == 0 and 0.1 < nt[0, 0] <= 10.0
    assert abs(0.5 + lf[0, 0] - hm_left) < 1e-5 and abs(0.5 + lf[0, 1] - hm_right) < 1e-5
    pred = oracle.trees_predict(1, 1, nf, nt, lf, 0.5, x)
    want_loss = np.mean((pred - y) ** 2 / y)
    assert abs(loss - want_loss) < 1e-7
    assert abs(snr - (y ** 2).sum() / ((0.5 - y) ** 2).sum()) < 1e-6 * snr


def _gains_brute_force(x, g, h, lam):
    """all (feature, bin) gains from the definition, float64, no prefix sums"""
    F, P = x.shape
    bins = np.clip(np.floor(x.astype(np.float64) * 4), 0, 255).astype(int)
    out = np.full((F, 255), -np.inf)
    G, H = g.sum(), h.sum()
    for f in range(F):
        for b in range(255):
            left = bins[f] <= b
            if left.sum() == 0 or left.sum() == P:
                continue
            GL, HL = g[left].sum(), h[left].sum()
            out[f, b] = GL ** 2 / (HL + lam) + (G - GL) ** 2 / (H - HL + lam) - G ** 2 / (H + lam)
    return out


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_root_split_is_the_brute_force_argmax(seed):
    rng = np.random.default_rng(seed)
    F, P = 5, 150
    x = rng.uniform(0, 40, size=(F, P)).astype(np.float32)
    e = np.exp(0.05 * x[1] + 0.02 * x[3] + 0.1 * rng.standard_normal(P)).astype(np.float32)
    y = (e / e.max()).astype(np.float64)
    base, lam = 0.4, 1.0
    g, h = 2 * (base - y) / y, 2 / y
    gains = _gains_brute_force(x, g, h, lam)
    # bins without samples repeat the gain of the bin below them: the winner is the first (feature, bin) in
    # feature-major order that reaches the maximum, and every other maximiser is the same partition
    top = gains.max()
    winners = np.argwhere(gains >= top * (1 - 1e-12))
    f_best, b_best = winners[0]
    assert np.all(winners[:, 0] == f_best) and np.all(np.diff(winners[:, 1]) == 1)
    others = gains.copy()
    others[f_best, winners[:, 1]] = -np.inf
    assert top - others.max() > 1e-6 * top  # the data leave no near-tie between different partitions
    nf, nt, lf = _empty(2, 1)
    oracle.trees_boost(F, 2, nf, nt, lf, 0, 1, base, x, e, eta=0.3, lam=lam)
    assert nf[0, 0] == f_best and nt[0, 0] == np.float32((b_best + 1) * 0.25)
    # and the leaves are -eta G / (H + lambda) of the samples that reach them
    at = np.zeros(P, dtype=int)
    for _ in range(2):
        at = 2 * at + np.where(x[nf[0, at], np.arange(P)] < nt[0, at], 1, 2)
    for leaf in range(4):
        m = at == 3 + leaf
        want = -0.3 * g[m].sum() / (h[m].sum() + lam) if m.any() else 0.0
        assert abs(lf[0, leaf] - want) < 2e-6 * max(1.0, abs(want))


def test_first_tree_matches_a_library_regression_tree():
    """With eta = 1 and lambda = 0 one boosting round is a weighted least-squares regression tree on the
    residuals y - p with weights 1/y (Eq. (1) is quadratic in the prediction).  scikit-learn's tree, fitted to
    the bin indices with those weights, must predict the same values."""
    sk = pytest.importorskip("sklearn.tree")
    rng = np.random.default_rng(11)
    F, P, depth = 6, 400, 3
    x = rng.uniform(0, 60, size=(F, P)).astype(np.float32)
    e = (1.0 + 0.03 * x[0] + 0.5 * (x[2] > 30) + 0.2 * rng.random(P)).astype(np.float32)
    y = (e / e.max()).astype(np.float64)
    base = 0.5
    nf, nt, lf = _empty(depth, 1)
    oracle.trees_boost(F, depth, nf, nt, lf, 0, 1, base, x, e, eta=1.0, lam=0.0)
    mine = oracle.trees_predict(F, depth, nf, nt, lf, base, x)
    bins = np.clip(np.floor(x.astype(np.float64) * 4), 0, 255).T
    ref = sk.DecisionTreeRegressor(max_depth=depth, criterion="squared_error", random_state=0)
    ref.fit(bins, y - base, sample_weight=1.0 / y)
    theirs = base + ref.predict(bins)
    assert np.allclose(mine, theirs, rtol=0, atol=2e-6)


def test_training_loss_falls_and_rounds_compose():
    rng = np.random.default_rng(3)
    F, P, depth, R = 8, 512, 4, 12
    x = rng.uniform(0, 50, size=(F, P)).astype(np.float32)
    e = np.exp(0.04 * x[0] - 0.03 * x[5] + 0.3 * np.sin(x[2]) + 0.05 * rng.standard_normal(P)).astype(np.float32)
    nf, nt, lf = _empty(depth, R)
    losses, snrs = [], []
    for r in range(R):
        snr, loss = oracle.trees_boost(F, depth, nf, nt, lf, r, 1, 0.5, x, e, eta=0.5, lam=1.0)
        losses.append(loss)
        snrs.append(snr)
    assert all(b < a for a, b in zip(losses, losses[1:]))
    assert all(b > a for a, b in zip(snrs, snrs[1:]))      # entry SNR of round r+1 = quality after round r
    nf2, nt2, lf2 = _empty(depth, R)
    _, loss_all = oracle.trees_boost(F, depth, nf2, nt2, lf2, 0, R, 0.5, x, e, eta=0.5, lam=1.0)
    assert np.array_equal(nf, nf2) and np.array_equal(nt, nt2) and np.array_equal(lf, lf2)
    assert loss_all == losses[-1]
    # fp32 sequential prediction is what the iteration used: both modes agree to fp32 rounding
    a = oracle.trees_predict(F, depth, nf, nt, lf, 0.5, x)
    b = oracle.trees_predict(F, depth, nf, nt, lf, 0.5, x, fp32_sequential=True)
    assert np.max(np.abs(a - b)) < 1e-5


def test_bad_labels_and_degenerate_nodes():
    x = np.full((2, 8), 3.0, dtype=np.float32)           # every sample in the same bin: nothing can split
    e = np.linspace(1, 2, 8).astype(np.float32)
    nf, nt, lf = _empty(2, 1)
    snr, loss = oracle.trees_boost(2, 2, nf, nt, lf, 0, 1, 0.5, x, e, eta=1.0, lam=0.0)
    assert np.all(np.isinf(nt[0])) and np.all(nf[0] == 0)
    assert lf[0, 1] == 0 and lf[0, 2] == 0 and lf[0, 3] == 0 and lf[0, 0] != 0
    e[3] = 0.0
    nf, nt, lf = _empty(2, 3)
    nf[:], nt[:], lf[:] = 1, 7.0, 9.0
    snr, loss = oracle.trees_boost(2, 2, nf, nt, lf, 1, 2, 0.5, x, e)
    assert np.isnan(snr) and np.isnan(loss)
    # a rejected call appends its trees empty: no split anywhere, every leaf 0; earlier trees are not touched
    assert np.all(nf[0] == 1) and np.all(nt[0] == 7.0) and np.all(lf[0] == 9.0)
    assert np.all(nf[1:] == 0) and np.all(np.isinf(nt[1:])) and np.all(lf[1:] == 0)
    grown = oracle.trees_predict(2, 2, nf, nt, lf, 0.5, x)
    assert np.array_equal(grown, oracle.trees_predict(2, 2, nf[:1], nt[:1], lf[:1], 0.5, x))
