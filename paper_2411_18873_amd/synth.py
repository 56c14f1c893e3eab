"""Seeded synthetic inputs: operator problems, schedule-space configs, model
weights, measured-energy labels, score arrays.

This module serves the tests, the benchmark and the smoke check, for both the
HIP library and the CPU checker.  It holds none of the method's arithmetic (no
feature formula, no hash, no model evaluation, no selection) and imports
neither side.  Everything is numpy on the host; callers upload what they need.

The operator shapes stand in for the paper's MM / Conv workloads (Sec. 7.1);
the schedule populations the paper obtained from its auto-scheduler are
replaced by seeded samples of the spaces described below.
"""
import numpy as np

OP_GEMM, OP_BGEMM, OP_CONV2D = 0, 1, 2
SPACE_KNOB, SPACE_SPLIT, SPACE_SPLIT_XRED = 0, 1, 2

# (num_cu, wave, lds_bytes, max_threads_cu, max_blocks_cu)
HW_MI355X = (256, 64, 160 * 1024, 2048, 32)
# the case-study machine of Table 5: 108 multiprocessors, 32-wide warps
HW_CASE_STUDY = (108, 32, 164 * 1024, 2048, 32)

P_MUT_Q32 = 429496729  # floor(0.1 * 2**32)


def problem(op, dims, elem_bytes, hw=HW_MI355X):
    """15 int32 fields: op, dim[8], elem_bytes, 5 hardware parameters."""
    d = list(dims) + [0] * (8 - len(dims))
    return np.array([op] + d + [elem_bytes] + list(hw), dtype=np.int32)


def gemm(M, N, K, elem_bytes=2, hw=HW_MI355X):
    return problem(OP_GEMM, [1, M, N, K], elem_bytes, hw)


def bgemm(B, M, N, K, elem_bytes=2, hw=HW_MI355X):
    return problem(OP_BGEMM, [B, M, N, K], elem_bytes, hw)


def conv2d(N, C, K, H, W, R, S, stride=1, pad=0, elem_bytes=2, hw=HW_MI355X):
    return problem(OP_CONV2D, [N, C, K, H, W, R, S, stride | (pad << 16)], elem_bytes, hw)


def sweep_shapes():
    """The 64 GEMM shapes of the whole-network sweep, shape-major (M slowest)."""
    vals = [1024, 2048, 4096, 8192]
    return [(m, n, k) for m in vals for n in vals for k in vals]


CONFIGS = {
    # exhaustive knob space of one small GEMM, fp32 model
    "c1": dict(problem=gemm(512, 512, 512), kind=SPACE_KNOB, n=6400, n_feat=32, widths=[32, 64, 64, 1],
               bf16=False, k=16, alpha=1.1, weight_seeds=(1, 2)),
    # sampled split space of one convolution
    "c2": dict(problem=conv2d(1, 256, 256, 14, 14, 3, 3, 1, 1), kind=SPACE_SPLIT, n=1 << 20, n_feat=64,
               widths=[64, 256, 256, 1], bf16=True, k=64, alpha=1.1, sample_seed=2024, weight_seeds=(3, 4)),
    # evolutionary rounds on a batched GEMM
    "c3": dict(problem=bgemm(32, 2048, 2048, 128), kind=SPACE_SPLIT, n=1 << 20, n_feat=64,
               widths=[64, 256, 256, 1], bf16=True, k=1024, alpha=float("inf"), rounds=8, survivors=1024, seed=7,
               weight_seeds=(5, 6)),
    # dynamic update on measured pairs, then rescoring
    "c4": dict(problem=conv2d(1, 256, 256, 14, 14, 3, 3, 1, 1), kind=SPACE_SPLIT, n_pairs=4096, n_feat=64,
               widths=[64, 256, 256, 1], bf16=True, n_steps=100, minibatch=512, lr=1e-3, pair_seed=11,
               label_seed=13, rescore_n=1 << 22, weight_seeds=(3, 4)),
    # whole-network sweep: 64 shapes x 2^18 candidates
    "c5": dict(shapes=sweep_shapes(), kind=SPACE_SPLIT, n_per_shape=1 << 18, n_feat=64,
               widths=[64, 512, 512, 1], bf16=True, k=32, alpha=1.1, seed_base=100, weight_seeds=(8, 9)),
}


def paper_operators(hw=HW_MI355X):
    """The operator shapes of the paper's evaluation (Sec. 7.2), as problems of this library.  MM / MV are
    (batch, M, N, K): batch 1 is a GEMM, batch 8 a batched GEMM, MV has M = 1.  CONV is (batch, height, width,
    in channels, out channels, kernel, stride, padding).  MV1's N is taken as printed (49512)."""
    ops = {
        "MM1": gemm(512, 512, 512, hw=hw), "MM2": gemm(1024, 1024, 1024, hw=hw),
        "MM3": bgemm(8, 512, 512, 512, hw=hw), "MM4": bgemm(8, 1024, 1024, 1024, hw=hw),
        "MV1": gemm(1, 49512, 12288, hw=hw), "MV2": gemm(1, 32768, 16384, hw=hw),
        "MV3": bgemm(8, 1, 4096, 1024, hw=hw), "MV4": bgemm(8, 1, 8192, 2048, hw=hw),
        "CONV1": conv2d(8, 512, 512, 7, 7, 3, 3, 1, 1, hw=hw),
        "CONV2": conv2d(16, 64, 64, 56, 56, 1, 1, 1, 0, hw=hw),
        "CONV3": conv2d(64, 64, 64, 56, 56, 1, 1, 1, 0, hw=hw),
    }
    return ops


def round_to_bf16(x):
    """fp32 array -> nearest-even bf16 value, returned as fp32 (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def mlp_theta(widths, seed, bf16=False, bias_scale=0.0):
    """Parameter vector: per layer W[fan_in][fan_out] ~ N(0, 1/fan_in) (variance), then b.

    Biases are zero unless bias_scale > 0 (tests use non-zero biases so that a
    dropped bias cannot hide)."""
    rng = np.random.default_rng(seed)
    parts = []
    for fi, fo in zip(widths[:-1], widths[1:]):
        W = rng.standard_normal((fi, fo)).astype(np.float32) / np.float32(np.sqrt(fi))
        b = (rng.standard_normal(fo) * bias_scale).astype(np.float32)
        parts += [W.ravel(), b]
    theta = np.concatenate(parts).astype(np.float32)
    return round_to_bf16(theta) if bf16 else theta


def param_count(widths):
    return sum(fi * fo + fo for fi, fo in zip(widths[:-1], widths[1:]))


def measured_energy(feat, seed):
    """Synthetic measured energies for feature columns feat[F][n]:
    a positive-weight linear form times lognormal(0, 0.1) noise."""
    rng = np.random.default_rng(seed)
    F, n = feat.shape
    u = rng.random(F)
    w = u / u.sum()
    z = rng.standard_normal(n)
    e = (w[:, None] * feat.astype(np.float64)).sum(axis=0) * np.exp(0.1 * z)
    return e.astype(np.float32)


def gaussian_scores(n, seed, ties=0.0, quantum=None):
    """Near-Gaussian scores like those of a random MLP; `ties` = fraction of
    entries overwritten with copies of other entries; `quantum` rounds to a grid."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(n).astype(np.float32)
    if quantum:
        x = (np.round(x / quantum) * quantum).astype(np.float32)
    if ties > 0:
        m = int(n * ties)
        dst = rng.integers(0, n, m)
        src = rng.integers(0, n, m)
        x[dst] = x[src]
    return x


def legal_mask(n, seed, frac=0.3):
    rng = np.random.default_rng(seed)
    return (rng.random(n) < frac).astype(np.uint8)


def simulated_kernel_metrics(feat, seed, batch):
    """Stand-in for running kernels under a power meter and a timer: (energy, latency) of the feature
    columns feat[F][m].  Two fixed log-linear forms of the features (the "hardware", drawn from `seed`;
    exp(0.5 (w . x - 8)) with positive weights summing to one, so schedules differ by factors, not percent)
    times lognormal(0, 0.03) measurement noise drawn from (seed, batch) in column order."""
    F, m = feat.shape
    hw = np.random.default_rng(seed)
    we, wl = hw.random(F), hw.random(F)
    we, wl = we / we.sum(), wl / wl.sum()
    noise = np.random.default_rng([seed, batch])
    x = np.asarray(feat, dtype=np.float64)
    energy = np.exp(0.5 * ((we[:, None] * x).sum(axis=0) - 8.0) + 0.03 * noise.standard_normal(m))
    latency = np.exp(0.5 * ((wl[:, None] * x).sum(axis=0) - 8.0) + 0.03 * noise.standard_normal(m))
    return energy.astype(np.float32), latency.astype(np.float32)
