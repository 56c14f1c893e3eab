"""Pins for the oracle's loss, gradient, Adam refit, SNR and k controller.  CPU only."""
import math

import numpy as np
import pytest

import oracle
from paper_2411_18873_amd import synth


def test_eq1_values():
    assert oracle.loss(3.0, 2.0) == 0.5          # (3-2)^2 / 2
    assert oracle.loss(1.0, 4.0) == 2.25         # 9/4
    assert oracle.loss_grad(3.0, 2.0) == 1.0     # 2(3-2)/2
    assert oracle.loss_grad(1.0, 4.0) == -1.5
    # the weight 1/E_m: the same absolute error costs more on a low-energy kernel
    assert oracle.loss(1.5, 1.0) > oracle.loss(10.5, 10.0)


def _mean_loss(widths, theta64, feat, y, rows):
    pred = oracle.score(widths, theta64.astype(np.float32), feat, n=rows)
    return float(np.mean((pred - y[:rows]) ** 2 / y[:rows]))


def test_gradient_by_finite_differences():
    widths = [8, 6, 5, 1]
    rng = np.random.default_rng(0)
    P = synth.param_count(widths)
    # values exactly representable in fp32 so that score() sees the same numbers
    theta = (rng.integers(-64, 64, P) / 64.0).astype(np.float64)
    feat = (rng.integers(0, 64, (8, 16)) / 16.0).astype(np.float32)
    y = (rng.integers(1, 32, 16) / 8.0).astype(np.float64)
    val, grad = oracle.batch_gradient(widths, theta, feat, y, 0, 16)
    assert abs(val - _mean_loss(widths, theta, feat, y, 16)) < 1e-12
    h = 2.0 ** -10  # keeps theta +- h exact in fp32
    worst = 0.0
    for i in range(P):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h
        tm[i] -= h
        fd = (_mean_loss(widths, tp, feat, y, 16) - _mean_loss(widths, tm, feat, y, 16)) / (2 * h)
        worst = max(worst, abs(fd - grad[i]))
    assert worst < 1e-4 * max(1.0, np.abs(grad).max()), worst
    assert np.abs(grad).max() > 1e-2
    # a sub-range of rows
    val2, grad2 = oracle.batch_gradient(widths, theta, feat, y, 8, 8)
    pred = oracle.score(widths, theta.astype(np.float32), feat)[8:]
    assert abs(val2 - np.mean((pred - y[8:]) ** 2 / y[8:])) < 1e-12


def test_adam_first_steps_on_a_one_parameter_model():
    # model p = w*x + b with x = 1, one pair, E_m = 2 -> y = 1 (normalised by the max)
    widths = [1, 1]
    state = np.array([3.0, 0.0, 0, 0, 0, 0, 0], dtype=np.float64)  # w=3, b=0
    feat = np.ones((1, 1), dtype=np.float32)
    e = np.array([2.0], dtype=np.float32)
    lr, b1, b2, eps = 0.1, 0.9, 0.999, 1e-8
    snr, loss = oracle.update(widths, state, feat, e, 1, 1, lr=lr, beta1=b1, beta2=b2, eps=eps)
    # pred = 3, y = 1: SNR = 1/(3-1)^2, loss = 4, g = 2(3-1)/1 = 4 for both w and b
    assert snr == 0.25 and loss == 4.0
    # first Adam step: m_hat = g, v_hat = g^2 -> theta -= lr * g/(|g|+eps)
    step = lr * 4 / (4 + eps)
    assert abs(state[0] - (3 - step)) < 1e-15 and abs(state[1] - (0 - step)) < 1e-15
    assert state[6] == 1.0
    # second step by the textbook recurrences
    w, b = state[0], state[1]
    g = 2 * (w + b - 1)
    m = b1 * (1 - b1) * 4 + (1 - b1) * g
    v = b2 * (1 - b2) * 16 + (1 - b2) * g * g
    want = w - lr * (m / (1 - b1 ** 2)) / (math.sqrt(v / (1 - b2 ** 2)) + eps)
    snr2, loss2 = oracle.update(widths, state, feat, e, 1, 1, lr=lr, beta1=b1, beta2=b2, eps=eps)
    assert abs(state[0] - want) < 1e-14
    assert abs(loss2 - (w + b - 1) ** 2) < 1e-14
    assert abs(snr2 - 1 / (w + b - 1) ** 2) < 1e-12  # SNR uses the model as it was on entry
    assert state[6] == 2.0


def test_snr_definition_and_label_normalisation():
    widths = [2, 1]
    state = np.zeros(3 * 3 + 1)
    state[2] = 0.5  # bias only: every prediction is 0.5
    feat = np.random.default_rng(0).random((2, 8)).astype(np.float32)
    e = np.array([1, 2, 3, 4, 5, 6, 7, 8], dtype=np.float32)
    snr, _ = oracle.update(widths, state, feat, e, 0, 8)
    y = e.astype(np.float64) / 8.0
    assert abs(snr - (y ** 2).sum() / ((0.5 - y) ** 2).sum()) < 1e-14
    assert state[2] == 0.5 and state[-1] == 0  # zero steps: untouched
    # scaling all energies leaves everything unchanged (ranking-invariant normaliser)
    snr2, _ = oracle.update(widths, state, feat, e * 1024, 0, 8)
    assert snr2 == snr


def test_minibatches_walk_the_buffer_in_order():
    widths = [4, 3, 1]
    rng = np.random.default_rng(1)
    P = synth.param_count(widths)
    theta0 = rng.standard_normal(P) * 0.5
    feat = rng.random((4, 12)).astype(np.float32)
    e = (rng.random(12) + 0.5).astype(np.float32)
    y = e.astype(np.float64) / float(e.max())
    state = np.concatenate([theta0, np.zeros(2 * P + 1)])
    oracle.update(widths, state, feat, e, 1, 4, lr=0.01)
    _, g0 = oracle.batch_gradient(widths, theta0, feat, y, 0, 4)
    moved = np.abs(state[:P] - theta0) > 0
    assert np.array_equal(moved, g0 != 0)  # first step moves exactly the coordinates minibatch 0 touches
    assert np.allclose((theta0 - state[:P])[moved], 0.01 * np.sign(g0[moved]), rtol=1e-4)
    theta1 = state[:P].copy()
    m1 = state[P:2 * P].copy()
    oracle.update(widths, state, feat, e, 1, 4, lr=0.01)  # step counter carries on, but rows restart at 0
    _, g1 = oracle.batch_gradient(widths, theta1, feat, y, 0, 4)
    assert np.allclose(state[P:2 * P], 0.9 * m1 + 0.1 * g1, rtol=1e-12, atol=1e-15)
    # within one call, step 1 uses rows 4..7
    state2 = np.concatenate([theta0, np.zeros(2 * P + 1)])
    oracle.update(widths, state2, feat, e, 2, 4, lr=0.01)
    _, g1b = oracle.batch_gradient(widths, theta1, feat, y, 4, 4)
    assert np.allclose(state2[P:2 * P], 0.9 * m1 + 0.1 * g1b, rtol=1e-12, atol=1e-15)


def test_refit_learns_a_positive_linear_energy():
    cfg = synth.CONFIGS["c4"]
    widths = cfg["widths"]
    sp = oracle.Space(cfg["problem"], oracle.SPACE_SPLIT)
    n = 1024
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, n, seed=cfg["pair_seed"])
    _, f32, _, _ = oracle.features(sp, genes, 64)
    e = synth.measured_energy(f32, cfg["label_seed"])
    assert e.min() > 0
    P = synth.param_count(widths)
    theta0 = synth.mlp_theta(widths, 3)
    state = np.concatenate([theta0.astype(np.float64), np.zeros(2 * P + 1)])
    y = e.astype(np.float64) / float(e.max())
    snr0, loss_first = oracle.update(widths, state, f32, e, 1, 256, lr=cfg["lr"])
    snr1, loss_last = oracle.update(widths, state, f32, e, 39, 256, lr=cfg["lr"])
    snr2, _ = oracle.update(widths, state, f32, e, 0, 256)
    assert loss_last < 0.2 * loss_first
    assert snr2 > snr1 > snr0
    # (the labels' lognormal noise is ~3x the spread of the linear form, so rank correlation with the
    # labels is capped near 0.3 and is not a usable signal at this length of training)
    pred = oracle.score(widths, state[:P].astype(np.float32), f32)
    assert abs(snr2 - (y ** 2).sum() / ((pred - y) ** 2).sum()) < 1e-5 * snr2  # theta went through fp32
    assert state[-1] == 40


def _bf16_rne(x):
    """round-to-nearest-even to bfloat16, written on the bit pattern with numpy (independent of the oracle's C)"""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return r.astype(np.uint32).view(np.float32).astype(np.float64)


def test_bf16_weight_mode_is_the_plain_step_on_rounded_weights():
    """The bf16 mode of the refit: forward and backward see the master weights rounded to bf16, the step is applied
    to the unrounded master.  So from any state, one step in that mode must move the master by exactly what one
    plain step moves a model whose weights ARE the rounded ones, and leave the same moments -- checked with the
    rounding redone in numpy, from a fresh state and from one with moments.  And weights that are bf16 values
    already make the two modes the same function."""
    widths = [8, 16, 8, 1]
    P = synth.param_count(widths)
    rng = np.random.default_rng(4)
    feat = rng.uniform(0, 4, (8, 64)).astype(np.float32)
    y = rng.uniform(0.5, 3.0, 64)
    theta = rng.normal(0, 0.3, P)
    st = np.concatenate([theta, np.zeros(2 * P + 1)])
    for _ in range(3):
        before = st.copy()
        a = before.copy()
        oracle.update(widths, a, feat, y, 1, 16, bf16_weights=True)
        rounded = before.copy()
        rounded[:P] = _bf16_rne(before[:P])
        assert np.any(rounded[:P] != before[:P])
        b = rounded.copy()
        oracle.update(widths, b, feat, y, 1, 16, bf16_weights=False)
        assert np.allclose(a[:P] - before[:P], b[:P] - rounded[:P], rtol=0, atol=1e-15)
        assert np.array_equal(a[P:], b[P:])
        # and the plain mode from the unrounded weights is a different step
        c = before.copy()
        oracle.update(widths, c, feat, y, 1, 16, bf16_weights=False)
        assert not np.array_equal(c[P:2 * P], a[P:2 * P])
        st = a
    exact = np.concatenate([_bf16_rne(theta), np.zeros(2 * P + 1)])
    p_, q_ = exact.copy(), exact.copy()
    oracle.update(widths, p_, feat, y, 1, 16, bf16_weights=True)
    oracle.update(widths, q_, feat, y, 1, 16, bf16_weights=False)
    assert np.array_equal(p_, q_)


def test_nonpositive_energy_is_a_data_error():
    widths = [2, 1]
    state = np.arange(10, dtype=np.float64)
    before = state.copy()
    feat = np.ones((2, 4), dtype=np.float32)
    snr, loss = oracle.update(widths, state, feat, np.array([1, 0, 2, 3], dtype=np.float32), 3, 4)
    assert math.isnan(snr) and math.isnan(loss) and np.array_equal(state, before)


def test_k_controller_traces():
    mu, M = 10.0, 100
    # accurate model (SNR above mu): k walks down 1.0 -> 0 in fifths and then stays (no measurements, no signal)
    k, seen = 1.0, []
    for _ in range(7):
        k = oracle.k_step(k, 50.0, mu, M)
        seen.append(round(k, 9))
    assert seen == [0.8, 0.6, 0.4, 0.2, 0.0, 0.0, 0.0]
    # poor model: k climbs back and saturates at 1
    k, seen = 0.4, []
    for _ in range(5):
        k = oracle.k_step(k, 1.0, mu, M)
        seen.append(round(k, 9))
    assert seen == [0.6, 0.8, 1.0, 1.0, 1.0]
    # mixed script
    k = 1.0
    for snr, want in [(5, 1.0), (20, 0.8), (20, 0.6), (5, 0.8), (20, 0.6), (20, 0.4)]:
        k = oracle.k_step(k, snr, mu, M)
        assert abs(k - want) < 1e-12
    # k = 0.5 halves the measurements of a round
    assert round(0.5 * M) == M // 2
    # a ratio that does not exist (rejected energies) is no evidence of a good model
    assert abs(oracle.k_step(0.4, float("nan"), mu, M) - 0.6) < 1e-12
