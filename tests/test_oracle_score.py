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


def test_why_a_few_candidates_may_differ_from_the_bf16_activation_oracle():
    """The bf16-activation mode rounds an fp64 sum to bf16; a kernel that accumulates in fp32 rounds an fp32 sum.
    The two sums differ by ~2^-24 of their terms, so once in a few 10^5 activations they fall on different sides
    of a bf16 rounding boundary; that one activation then differs by a whole bf16 step (2^-8 of its value) and
    moves the output by a few 1e-4 of the sum's magnitude M.  Measured here with numpy's fp32 matrix product
    standing in for any fp32 accumulation order: the rate per activation and the largest effect, which size the
    allowance of the GPU parity gate (at most 1 + 5e-4 n candidates beyond 1e-4 M, none beyond 1e-3 M)."""
    widths = [64, 256, 256, 1]
    cfg = synth.CONFIGS["c2"]
    sp = oracle.Space(cfg["problem"], oracle.SPACE_SPLIT)
    n = 1 << 15
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, n, seed=cfg["sample_seed"])
    _, _, b16, _ = oracle.features(sp, genes, 64)
    x = oracle.bf16_bits_to_f32(b16)
    theta = synth.mlp_theta(widths, cfg["weight_seeds"][0], bf16=True)
    W1, b1 = theta[:64 * 256].reshape(64, 256), theta[64 * 256:64 * 256 + 256]
    pre32 = np.maximum(x.T @ W1 + b1, 0).astype(np.float32)                               # fp32 accumulation
    pre64 = np.maximum(x.T.astype(np.float64) @ W1.astype(np.float64) + b1, 0).astype(np.float32)
    def rne(v):    # round-to-nearest-even to bf16 on the bits (finite inputs); checked against the oracle's below
        u = np.ascontiguousarray(v, dtype=np.float32).view(np.uint32).astype(np.uint64)
        return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    some = pre32.reshape(-1)[::9973]
    assert [int(b) for b in rne(some)] == [oracle.bf16_rne(float(v)) for v in some]
    flips = rne(pre32) != rne(pre64)
    rate = flips.mean()
    assert 0 < flips.sum() and rate < 5e-5                 # rare, but it happens
    # the effect of those flips on the output: replace the oracle's rounded activations by the fp32-rounded ones
    h32 = oracle.bf16_bits_to_f32(rne(pre32)).astype(np.float64)
    h64 = oracle.bf16_bits_to_f32(rne(pre64)).astype(np.float64)
    o = 64 * 256 + 256
    W2, b2 = theta[o:o + 256 * 256].reshape(256, 256).astype(np.float64), theta[o + 256 * 256:o + 256 * 256 + 256]
    w3, b3 = theta[-257:-1].astype(np.float64), float(theta[-1])
    out = lambda h: np.maximum(h @ W2 + b2, 0) @ w3 + b3
    mag = oracle.score_magnitude(widths, theta, x)
    emu = oracle.score(widths, theta, x, emulate_bf16=True)
    assert np.max(np.abs(out(h64) - emu) / mag) < 1e-12    # the reconstruction above is the oracle's mode
    moved = np.abs(out(h32) - out(h64)) / mag
    assert moved.max() < 1e-3
    assert (moved > 1e-4).sum() <= 1 + int(5e-4 * n)
    assert np.all(moved[~flips.any(axis=1)] == 0)          # nothing else differs
