"""Pin for the oracle's features of staged schedules (space kind SPLIT): a walker that executes the loop nest of tiny
schedules literally -- every block, every stage, every thread, every reduction step, every output of the thread --
and counts what it does: the multiply-adds, the operand elements a block stages per stage, the operand elements a
thread reads from the staged tile per reduction step.  The counts must equal the oracle's features, among them
feature 20 (shared-memory loads), which no figure of the paper pins.  CPU only."""
import itertools
import math

import numpy as np

import oracle
from paper_2411_18873_amd import synth


def _walk(op, f, R, S, stride):
    sp_axes = range(4)
    blocks = list(itertools.product(*[range(f[a][0]) for a in sp_axes]))
    threads = list(itertools.product(*[range(f[a][1]) for a in sp_axes]))
    serial = list(itertools.product(*[range(f[a][2] * f[a][3]) for a in sp_axes]))
    stages, tile_red = f[4][0], f[4][1] * f[4][2] * f[4][3]
    seen = {}
    block_sizes, step_sizes, aligned_sizes = set(), set(), set()
    staged = shared_loads = 0
    steps_per_thread = set()
    for blk in blocks:
        thread_steps = {thr: 0 for thr in threads}
        for k0 in range(stages):
            blk_a, blk_b, aligned = set(), set(), set()
            for thr in threads:
                for kk in range(tile_red):
                    k = k0 * tile_red + kk
                    for r in range(R):
                        for s in range(S):
                            a_set, b_set = set(), set()
                            for ser in serial:
                                out = tuple((blk[a] * f[a][1] + thr[a]) * f[a][2] * f[a][3] + ser[a] for a in sp_axes)
                                seen[(out, k, r, s)] = seen.get((out, k, r, s), 0) + 1
                                if op == "conv":   # out = (n, k_out, h, w)
                                    a_set.add((out[0], k, out[2] * stride + r, out[3] * stride + s))
                                    b_set.add((out[1], k, r, s))
                                    aligned.add((out[0], k, out[2], out[3]))
                                else:              # out = (b, m, n, -)
                                    a_set.add((out[0], out[1], k))
                                    b_set.add((out[0], k, out[2]))
                            step_sizes.add((len(a_set), len(b_set)))
                            shared_loads += len(a_set) + len(b_set)
                            thread_steps[thr] += 1
                            blk_a |= a_set
                            blk_b |= b_set
            block_sizes.add((len(blk_a), len(blk_b)))
            aligned_sizes.add(len(aligned))
            staged += len(blk_a) + len(blk_b)
        steps_per_thread |= set(thread_steps.values())
    assert set(seen.values()) == {1}                      # every (output, reduction) pair exactly once
    assert len(block_sizes) == 1 and len(step_sizes) == 1 and len(steps_per_thread) == 1
    (fp_a, fp_b), (pa, pb) = next(iter(block_sizes)), next(iter(step_sizes))
    return dict(macs=len(seen), G=len(blocks), T=len(threads), Pt=len(serial), stages=stages, fp_a=fp_a, fp_b=fp_b,
                pa=pa, pb=pb, staged=staged, shared_loads=shared_loads, steps=next(iter(steps_per_thread)),
                aligned=next(iter(aligned_sizes)) if op == "conv" else fp_a)


def _check(pb, op, ext, R, S, stride, n_samples, seed):
    sp = oracle.Space(pb, oracle.SPACE_SPLIT)
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, n_samples, seed=seed)
    raw, _, _, _ = oracle.features(sp, genes, 64)
    raw = raw.astype(object)
    b, n_cu, wave = pb[9], pb[10], pb[11]
    outputs = math.prod(ext[:4])
    shapes = set()
    for c in range(n_samples):
        x = [int(v) for v in raw[:, c]]
        f = [[x[32 + 4 * a + l] for l in range(4)] for a in range(5)]
        U, V = x[27], x[30]
        w = _walk(op, f, R, S, stride)
        shapes.add((w["G"], w["T"], w["Pt"], w["stages"]))
        assert w["macs"] == outputs * ext[4] * R * S
        assert x[0] == 2 * w["macs"] and x[1] == 2 * w["macs"]
        assert x[2] == w["Pt"] * w["steps"] and x[2] * w["G"] * w["T"] == w["macs"]
        assert x[4] == w["Pt"] and x[5] == w["Pt"] + w["pa"] + w["pb"]
        assert x[6] == w["G"] and x[7] == w["T"] and x[8] == -(-w["T"] // wave)
        assert x[10] == min(w["G"], n_cu) and x[11] == n_cu - x[10]
        loads_thread_stage = -(-(w["fp_a"] + w["fp_b"]) // (w["T"] * V))     # cooperative vector loads
        assert x[14] == w["G"] * w["T"] * w["stages"] * loads_thread_stage
        assert x[15] == -(-w["staged"] * b // 32)
        assert x[16] == -(-outputs * b // 32)
        assert x[17] == w["G"] * w["T"] * -(-w["Pt"] // V)
        assert x[18] == (w["fp_a"] + w["fp_b"]) * b
        assert x[19] == -(-w["staged"] * b // 128)
        assert x[20] == w["shared_loads"]                                       # the feature no figure of the paper pins
        assert x[21] == (x[1] * 8) // (x[15] + x[16])
        assert x[24] == w["stages"] and x[24] * x[25] == w["steps"]
        assert x[57] == w["fp_a"] and x[58] == w["fp_b"]
        assert x[59] == (w["fp_a"] * 256) // w["aligned"]
        assert x[62] == outputs and x[63] * x[62] == w["macs"]
        # integer work: per stage 4 per load and 2 of loop control, 2 per unrolled trip of the reduction
        assert x[3] == w["G"] * w["T"] * (w["stages"] * (4 * loads_thread_stage + 2) + 2 * -(-w["steps"] // U))
    assert len(shapes) > n_samples // 3                                         # the samples really differ


def test_walked_schedules_of_a_batched_product():
    pb = synth.bgemm(2, 4, 6, 12, elem_bytes=2, hw=(4, 64, 4096, 256, 8))
    _check(pb, "gemm", [2, 4, 6, 1, 12], 1, 1, 1, 60, seed=3)


def test_walked_schedules_of_a_product_with_four_byte_elements():
    pb = synth.gemm(8, 6, 16, elem_bytes=4, hw=(4, 64, 4096, 256, 8))
    _check(pb, "gemm", [1, 8, 6, 1, 16], 1, 1, 1, 60, seed=4)


def test_walked_schedules_of_a_convolution():
    # 4x4 image, pad 1, 3x3 filter, stride 1 -> 4x4 outputs; input coordinates are counted unclipped
    pb = synth.conv2d(1, 4, 2, 4, 4, 3, 3, 1, 1, elem_bytes=2, hw=(4, 64, 4096, 256, 8))
    _check(pb, "conv", [1, 2, 4, 4, 4], 3, 3, 1, 40, seed=5)
    # stride 2: 7x7 image, pad 1, 3x3 -> 4x4 outputs
    pb = synth.conv2d(1, 2, 2, 7, 7, 3, 3, 2, 1, elem_bytes=4, hw=(4, 64, 4096, 256, 8))
    _check(pb, "conv", [1, 2, 4, 4, 2], 3, 3, 2, 30, seed=6)


def test_a_planted_mistake_in_the_shared_load_count_would_show():
    """the walker's count is not the formula retyped: counting the operand elements of a thread's whole tile
    instead of those of one reduction step, or forgetting one operand, gives other numbers on these schedules"""
    pb = synth.bgemm(2, 4, 6, 12, elem_bytes=2, hw=(4, 64, 4096, 256, 8))
    sp = oracle.Space(pb, oracle.SPACE_SPLIT)
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, 60, seed=3)
    raw, _, _, _ = oracle.features(sp, genes, 64)
    raw = raw.astype(object)
    differ_a = differ_b = 0
    for c in range(60):
        x = [int(v) for v in raw[:, c]]
        f = [[x[32 + 4 * a + l] for l in range(4)] for a in range(5)]
        w = _walk("gemm", f, 1, 1, 1)
        differ_a += w["G"] * w["T"] * w["steps"] * w["pa"] != x[20]             # one operand forgotten
        differ_b += w["G"] * w["T"] * w["stages"] * (w["fp_a"] + w["fp_b"]) != x[20]   # the staged tile per thread
    assert differ_a == 60 and differ_b > 30
