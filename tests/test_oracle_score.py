"""Pins for the oracle's model forward pass.  CPU only."""
import numpy as np

import oracle
from paper_2411_18873_amd import synth


def test_single_layer_is_a_dot_product():
    rng = np.random.default_rng(0)
    F, n = 32, 50
    theta = rng.standard_normal(F + 1).astype(np.float32)
    feat = rng.standard_normal((F, n)).astype(np.float32)
    got = oracle.score([F, 1], theta, feat)
    want = feat.astype(np.float64).T @ theta[:F].astype(np.float64) + float(theta[F])
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)


def test_hand_worked_two_layer_network():
    # x = (1, 2); W1 = [[1, -1], [0.5, 1]], b1 = (0, -2); W2 = (2, 3), b2 = 1
    # pre1 = (1*1 + 2*0.5, 1*-1 + 2*1 - 2) = (2, -1) -> relu (2, 0) -> 2*2 + 0*3 + 1 = 5
    theta = np.array([1, -1, 0.5, 1, 0, -2, 2, 3, 1], dtype=np.float32)
    feat = np.array([[1.0, 0.0], [2.0, 0.0]], dtype=np.float32)  # second candidate: x = 0
    got = oracle.score([2, 2, 1], theta, feat)
    assert got[0] == 5.0
    assert got[1] == 1.0  # relu(b1) = (0,0) -> b2


def test_three_layers_against_matmul():
    widths = [64, 256, 256, 1]
    theta = synth.mlp_theta(widths, seed=3, bias_scale=0.5)
    rng = np.random.default_rng(1)
    feat = (rng.random((64, 300)) * 40).astype(np.float32)
    got = oracle.score(widths, theta, feat)
    t = theta.astype(np.float64)
    o = 0
    h = feat.astype(np.float64).T
    for li, (fi, fo) in enumerate(zip(widths[:-1], widths[1:])):
        W = t[o:o + fi * fo].reshape(fi, fo)
        b = t[o + fi * fo:o + fi * fo + fo]
        o += fi * fo + fo
        h = h @ W + b
        if li < 2:
            h = np.maximum(h, 0)
    assert np.allclose(got, h[:, 0], rtol=1e-12, atol=1e-12)
    # leading dimension larger than n
    got2 = oracle.score(widths, theta, feat, n=123)
    assert np.array_equal(got2, got[:123])


def test_transposed_weights_or_dropped_bias_would_show():
    widths = [32, 64, 64, 1]
    theta = synth.mlp_theta(widths, seed=1, bias_scale=0.5)
    rng = np.random.default_rng(2)
    feat = (rng.random((32, 64)) * 30).astype(np.float32)
    base = oracle.score(widths, theta, feat)
    # second layer is square: transposing it must change the answer
    t2 = theta.copy()
    o = 32 * 64 + 64
    t2[o:o + 64 * 64] = theta[o:o + 64 * 64].reshape(64, 64).T.ravel()
    assert not np.allclose(oracle.score(widths, t2, feat), base, rtol=1e-3)
    t3 = theta.copy()
    t3[o + 64 * 64:o + 64 * 64 + 64] = 0
    assert not np.allclose(oracle.score(widths, t3, feat), base, rtol=1e-3)


def test_bf16_emulation_rounds_only_the_first_hidden_layer():
    widths = [64, 256, 256, 1]
    theta = synth.mlp_theta(widths, seed=4, bf16=True)
    rng = np.random.default_rng(5)
    feat = synth.round_to_bf16((rng.random((64, 200)) * 40).astype(np.float32))
    exact = oracle.score(widths, theta, feat)
    emu = oracle.score(widths, theta, feat, emulate_bf16=True)
    rms = np.sqrt((exact ** 2).mean())
    err = np.abs(emu - exact).max() / rms
    assert 0 < err < 1e-2
    # independent emulation in numpy
    t = theta.astype(np.float64)
    W1, b1 = t[:64 * 256].reshape(64, 256), t[64 * 256:64 * 256 + 256]
    o = 64 * 256 + 256
    W2, b2 = t[o:o + 256 * 256].reshape(256, 256), t[o + 256 * 256:o + 256 * 256 + 256]
    o += 256 * 256 + 256
    w3, b3 = t[o:o + 256], t[o + 256]
    h1 = np.maximum(feat.astype(np.float64).T @ W1 + b1, 0)
    h1 = synth.round_to_bf16(h1.astype(np.float32)).astype(np.float64)
    h2 = np.maximum(h1 @ W2 + b2, 0)
    assert np.allclose(emu, h2 @ w3 + b3, rtol=1e-12, atol=1e-12)


def test_output_magnitude_yardstick():
    # hand-worked 2-2-1 network of test_hand_worked_two_layer_network with a negative output weight:
    # x = (1, 2): h = (2, 0) -> o = 2*2 - 3*0 - 1 = 3, magnitude |2|*2 + |-3|*0 + |-1| = 5
    theta = np.array([1, -1, 0.5, 1, 0, -2, 2, -3, -1], dtype=np.float32)
    feat = np.array([[1.0, 4.0], [2.0, 0.0]], dtype=np.float32)
    assert list(oracle.score([2, 2, 1], theta, feat)) == [3.0, 7.0]
    assert list(oracle.score_magnitude([2, 2, 1], theta, feat)) == [5.0, 9.0]
    # with non-negative output weights and bias the magnitude is the score itself
    widths = [32, 64, 64, 1]
    t = synth.mlp_theta(widths, 2, bias_scale=0.3)
    t[-65:] = np.abs(t[-65:])
    x = (np.random.default_rng(0).random((32, 50)) * 30).astype(np.float32)
    assert np.allclose(oracle.score(widths, t, x), oracle.score_magnitude(widths, t, x), rtol=1e-14)


def test_why_the_tolerance_refers_to_the_magnitude_of_the_sum():
    """The outputs of these random networks are small differences of large terms: relative to |o| or
    rms(o) the unavoidable bf16-activation rounding looks like anything from 0.1 % to 6 % depending on the
    weight seed, relative to the magnitude M of the sum it is a stable ~1e-3."""
    import oracle as orc
    widths = [64, 256, 256, 1]
    sp = orc.Space(synth.CONFIGS["c2"]["problem"], orc.SPACE_SPLIT)
    genes = orc.enumerate_candidates(sp, orc.MODE_SAMPLE, 1 << 13, seed=2024)
    _, _, b16, _ = orc.features(sp, genes, 64)
    x = orc.bf16_bits_to_f32(b16)
    vs_rms, vs_mag = [], []
    for seed in (3, 4):
        theta = synth.mlp_theta(widths, seed, bf16=True)
        exact = orc.score(widths, theta, x)
        emu = orc.score(widths, theta, x, emulate_bf16=True)
        mag = orc.score_magnitude(widths, theta, x)
        rms = np.sqrt((exact ** 2).mean())
        vs_rms.append((np.abs(emu - exact) / np.maximum(np.abs(exact), rms)).max())
        vs_mag.append((np.abs(emu - exact) / mag).max())
        assert mag.min() > 3 * np.abs(exact).max() or seed == 3
    assert vs_rms[1] > 10 * vs_rms[0]          # same arithmetic, wildly different "relative" error
    assert max(vs_mag) < 2e-3 and max(vs_mag) < 2 * min(vs_mag)
