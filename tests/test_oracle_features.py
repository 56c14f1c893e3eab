"""Pins for the oracle's analytic features: the counters the paper prints for
its case study, two schedules worked by hand, closed-form invariants, and the
fixed-point log transform.  CPU only."""
import itertools
import math

import numpy as np
import pytest

import oracle
from paper_2411_18873_amd import synth

TILE_MN = [16, 32, 64, 128, 256]
TILE_K = [8, 16, 32, 64]
THREADS = [64, 128, 256, 512]
POW2 = [1, 2, 4, 8, 16]


def _one(space, gene_list, n_feat=64):
    genes = np.array(gene_list, dtype=np.uint16).reshape(-1, 1)
    raw, f32, b16, legal = oracle.features(space, genes, n_feat)
    return [int(v) for v in raw[:, 0]], int(legal[0]), f32[:, 0], b16[:, 0]


def test_table5_counters(golden):
    pb = synth.gemm(512, 512, 512, elem_bytes=4, hw=synth.HW_CASE_STUDY)
    sp = oracle.Space(pb, oracle.SPACE_KNOB)
    for row in golden("table5_case_study.txt"):
        name = row[0]
        tm, tn, thr, grid, block, glb_ld, glb_st, shared_ld, shared_st = (int(t) for t in row[1:])
        for tk_i, u_i in itertools.product(range(4), range(4)):  # printed values do not depend on tile_k / unroll
            x, legal, _, _ = _one(sp, [TILE_MN.index(tm), TILE_MN.index(tn), tk_i, THREADS.index(thr), u_i, 0])
            assert x[6] == grid and x[7] == block
            assert x[15] == glb_ld
            assert x[19] == shared_st
            if name == "K2":
                assert x[16] == glb_st  # K1's store count depends on an unprinted thread layout
            assert x[10] == min(grid, 108) and x[11] == 108 - min(grid, 108)
            assert legal == 1
    # K1 leaves 44 of 108 units idle, K2 none (the paper's static-energy argument)
    k1, _, _, _ = _one(sp, [2, 2, 0, 2, 0, 0])
    k2, _, _, _ = _one(sp, [0, 2, 0, 1, 0, 0])
    assert k1[11] == 44 and k2[11] == 0
    # more reuse inside a block => fewer shared loads, as the paper reports (direction only)
    assert k1[20] < k2[20]
    # a 32x32 tile would not reproduce K2's printed global loads
    alt, _, _, _ = _one(sp, [1, 1, 0, 1, 0, 0])
    assert alt[15] == 1048576 != 1310720


def _gene_of(extent, tup):
    divs = [d for d in range(1, extent + 1) if extent % d == 0]
    table = sorted(t for t in itertools.product(divs, repeat=4) if math.prod(t) == extent)
    return table.index(tuple(tup))


def test_hand_computed_bgemm(golden):
    rows = golden("hand_bgemm.txt")
    want, want_legal = [int(t) for t in rows[0]], int(rows[1][0])
    assert len(want) == 64
    pb = synth.bgemm(2, 8, 12, 6, elem_bytes=2, hw=(4, 64, 1024, 256, 8))
    sp = oracle.Space(pb, oracle.SPACE_SPLIT)
    genes = [_gene_of(2, (1, 1, 2, 1)), _gene_of(8, (2, 2, 1, 2)), _gene_of(12, (1, 3, 2, 2)),
             _gene_of(6, (3, 1, 2, 1)), POW2.index(2), POW2.index(2)]
    x, legal, _, _ = _one(sp, genes)
    assert x == want
    assert legal == want_legal
    x32, _, _, _ = _one(sp, genes, n_feat=32)
    assert x32 == want[:32]


def test_hand_computed_conv(golden):
    rows = golden("hand_conv.txt")
    want, want_legal = [int(t) for t in rows[0]], int(rows[1][0])
    pb = synth.conv2d(2, 4, 8, 6, 6, 3, 3, 1, 1, elem_bytes=4, hw=(8, 64, 65536, 1024, 16))
    sp = oracle.Space(pb, oracle.SPACE_SPLIT)
    assert sp.radix[:5] == [len(oracle.split_table(e)) for e in (2, 8, 6, 6, 4)]
    genes = [_gene_of(2, (1, 2, 1, 1)), _gene_of(8, (1, 4, 2, 1)), _gene_of(6, (3, 2, 1, 1)),
             _gene_of(6, (1, 3, 1, 2)), _gene_of(4, (2, 1, 1, 2)), POW2.index(4), POW2.index(2)]
    x, legal, _, _ = _one(sp, genes)
    assert x == want
    assert legal == want_legal


def test_hand_computed_knob_schedules_whose_tiles_do_not_divide_the_problem(golden):
    """The record a KNOB candidate derives (threads along N and M, outputs per thread along both) feeds the
    per-thread features 2-5, 14, 17, 20, 28; here all 64 values of two such schedules, worked by hand."""
    rows = golden("hand_knob.txt")
    pb = synth.bgemm(3, 40, 100, 20, elem_bytes=2, hw=(6, 64, 16384, 512, 4))
    sp = oracle.Space(pb, oracle.SPACE_KNOB)
    tiles, tile_k, threads = [16, 32, 64, 128, 256], [8, 16, 32, 64], [64, 128, 256, 512]
    for row, (tm, tn, tk, T, U, V) in ((0, (32, 64, 8, 128, 4, 1)), (2, (16, 256, 16, 64, 8, 2))):
        want, want_legal = [int(t) for t in rows[row]], int(rows[row + 1][0])
        assert len(want) == 64
        genes = [tiles.index(tm), tiles.index(tn), tile_k.index(tk), threads.index(T), POW2.index(U), POW2.index(V)]
        x, legal, _, _ = _one(sp, genes)
        assert x == want, [(i, a, b) for i, (a, b) in enumerate(zip(x, want)) if a != b]
        assert legal == want_legal
        x32, _, _, _ = _one(sp, genes, n_feat=32)
        assert x32 == want[:32]
        assert x[1] > x[0]          # padded tiles execute more than the useful flop


def test_split_candidates_execute_exactly_the_useful_flops():
    for name in ("c2", "c3"):
        cfg = synth.CONFIGS[name]
        sp = oracle.Space(cfg["problem"], oracle.SPACE_SPLIT)
        genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, 4096, seed=5)
        raw, _, _, legal = oracle.features(sp, genes, 64)
        assert np.array_equal(raw[0], raw[1])
        assert legal.sum() > 0
        # outputs are covered exactly once: grid * block * per-thread == true outputs
        assert np.array_equal(raw[6] * raw[7] * raw[4], raw[62])
        # every axis's four levels multiply back to the extent
        d = cfg["problem"][1:9]
        ext = [d[0], d[2], 14, 14, d[1]] if name == "c2" else [d[0], d[1], d[2], 1, d[3]]
        for a in range(5):
            assert np.all(raw[32 + 4 * a:36 + 4 * a].prod(axis=0) == ext[a])
    # closed forms
    c2 = oracle.Space(synth.CONFIGS["c2"]["problem"], oracle.SPACE_SPLIT)
    raw, _, _, _ = oracle.features(c2, oracle.enumerate_candidates(c2, oracle.MODE_SAMPLE, 8, seed=1), 64)
    assert np.all(raw[0] == 2 * 1 * 256 * 14 * 14 * 256 * 3 * 3)
    assert np.all(raw[22] == (256 * 14 * 14 + 256 * 256 * 9 + 256 * 14 * 14) * 2)
    c3 = oracle.Space(synth.CONFIGS["c3"]["problem"], oracle.SPACE_SPLIT)
    raw, _, _, _ = oracle.features(c3, oracle.enumerate_candidates(c3, oracle.MODE_SAMPLE, 8, seed=1), 64)
    assert np.all(raw[0] == 2 * 32 * 2048 * 2048 * 128)
    assert np.all(raw[22] == 32 * (2048 * 128 + 128 * 2048 + 2048 * 2048) * 2)
    assert np.all(raw[59] == 256)


def test_knob_padding_and_legality():
    pb = synth.gemm(100, 100, 100, elem_bytes=2)
    sp = oracle.Space(pb, oracle.SPACE_KNOB)
    x, legal, _, _ = _one(sp, [4, 4, 3, 2, 0, 0])  # 256x256 tile on a 100^3 problem
    assert x[0] == 2 * 100 ** 3
    assert x[1] == 2 * 256 * 256 * 128  # padded to whole tiles / whole k-steps
    assert x[6] == 1
    # 512 threads on a 16x16 tile: 32 thread rows do not fit 16 tile rows
    _, legal, _, _ = _one(sp, [0, 0, 0, 3, 0, 0])
    assert legal == 0
    # vector width must divide the contiguous per-thread extent along N
    x, legal, _, _ = _one(sp, [2, 4, 0, 0, 0, 2])  # tn=256, T=64 -> 4 per thread along N, vec 4
    assert legal == 1 and x[31] == 4
    _, legal, _, _ = _one(sp, [2, 4, 0, 0, 0, 3])  # vec 8 does not divide 4
    assert legal == 0
    # shared memory over the limit
    small_lds = synth.gemm(512, 512, 512, elem_bytes=4, hw=(256, 64, 16384, 2048, 32))
    sp2 = oracle.Space(small_lds, oracle.SPACE_KNOB)
    x, legal, _, _ = _one(sp2, [4, 4, 3, 2, 0, 0])
    assert x[18] == (256 * 64 + 256 * 64) * 4 and legal == 0 and x[9] == 0
    # 16-byte vector limit: 8 x 4-byte elements is too wide
    _, legal, _, _ = _one(sp2, [0, 4, 0, 0, 0, 3])
    assert legal == 0


def test_c1_space_has_a_usable_legal_fraction():
    cfg = synth.CONFIGS["c1"]
    sp = oracle.Space(cfg["problem"], oracle.SPACE_KNOB)
    genes = oracle.enumerate_candidates(sp, oracle.MODE_EXHAUSTIVE, 6400)
    raw, f32, b16, legal = oracle.features(sp, genes, 32)
    assert 0.1 < legal.mean() < 0.9
    assert np.all(raw[0] == 2 * 512 ** 3)
    assert np.all(raw[1] >= raw[0])


def test_transform_special_values_and_bounds():
    for k in range(0, 64):
        assert oracle.transform((1 << k) - 1) == float(k)
    assert oracle.transform((1 << 64) - 1) == oracle.transform((1 << 64) - 2)  # saturating +1
    assert oracle.transform(2) == 1.5          # v=3: e=1, mantissa 1/2
    assert oracle.transform(5) == 2.5          # v=6 = 4*(1+1/2)
    assert oracle.transform(6) == 2.75         # v=7
    assert oracle.transform(1024 + 2048 - 1) == 11.5  # v = 3072 = 2^11 * 1.5
    rng = np.random.default_rng(0)
    prev_v, prev_x = 0, -1.0
    vals = sorted(set(int(v) for v in np.concatenate([
        rng.integers(0, 1 << 20, 3000), rng.integers(0, 1 << 62, 3000, dtype=np.uint64), np.arange(0, 5000)])))
    for raw in vals:
        x = oracle.transform(raw)
        assert x >= prev_x  # monotone
        prev_x = x
        true = math.log2(raw + 1)
        # piecewise-linear log2 lies under log2 by at most 0.0861 (max of log2(1+t)-t) plus 2^-10 truncation
        assert -1e-9 <= true - x <= 0.0861 + 2 ** -10 + 1e-9, raw
        assert x * 1024 == int(x * 1024)


def test_bf16_rounding_is_nearest_even():
    assert oracle.bf16_rne(1.0) == 0x3F80
    assert oracle.bf16_rne(1.0 + 2 ** -8) == 0x3F80       # tie -> even (down)
    assert oracle.bf16_rne(1.0 + 3 * 2 ** -8) == 0x3F82   # tie -> even (up)
    assert oracle.bf16_rne(1.0 + 2 ** -8 + 2 ** -20) == 0x3F81
    assert oracle.bf16_rne(-2.5) == 0xC020
    x = np.array([11.5, 40.0, 17.3330078125, 63.9990234375], dtype=np.float32)
    got = oracle.bf16_bits_to_f32([oracle.bf16_rne(v) for v in x])
    assert np.all(np.abs(got - x) <= np.abs(x) * 2 ** -8)
    assert np.array_equal(got, synth.round_to_bf16(x))


def test_feature_matrix_outputs_are_consistent():
    sp = oracle.Space(synth.CONFIGS["c2"]["problem"], oracle.SPACE_SPLIT)
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, 513, seed=3)
    raw, f32, b16, legal = oracle.features(sp, genes, 64)
    for f, i in [(0, 0), (15, 17), (23, 512), (59, 100)]:
        assert f32[f, i] == oracle.transform(int(raw[f, i]))
        assert b16[f, i] == oracle.bf16_rne(f32[f, i])
    assert f32.min() >= 0 and f32.max() < 64
    with pytest.raises(ValueError):
        bad = genes.copy()
        bad[1, 0] = 165
        oracle.features(sp, bad, 64)


def test_paper_operator_shapes_have_the_closed_form_work():
    """The eleven operators of the paper's evaluation (Sec. 7.2): useful flop 2BMNK (MM, MV) and
    2 N K Ho Wo C R S (CONV), whatever the schedule."""
    want = {"MM1": 2 * 512 ** 3, "MM2": 2 * 1024 ** 3, "MM3": 2 * 8 * 512 ** 3, "MM4": 2 * 8 * 1024 ** 3,
            "MV1": 2 * 49512 * 12288, "MV2": 2 * 32768 * 16384, "MV3": 2 * 8 * 4096 * 1024, "MV4": 2 * 8 * 8192 * 2048,
            "CONV1": 2 * 8 * 512 * 7 * 7 * 512 * 9, "CONV2": 2 * 16 * 64 * 56 * 56 * 64, "CONV3": 2 * 64 * 64 * 56 * 56 * 64}
    ops = synth.paper_operators()
    assert set(ops) == set(want)
    for name, pb in ops.items():
        sp = oracle.Space(pb, oracle.SPACE_SPLIT)
        genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, 64, seed=3)
        raw, _, _, _ = oracle.features(sp, genes, 64)
        assert np.all(raw[0] == want[name]), name
        assert np.all(raw[1] == raw[0]), name          # exact factorisations: executed = useful
