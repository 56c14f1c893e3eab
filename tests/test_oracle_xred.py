"""Pins for the oracle's features of reduction-parallel schedules (space kind SPLIT_XRED): a schedule worked by
hand, a walker that executes the loop nest of tiny schedules thread by thread and counts what it does, closed
forms, and what the kind is for -- matrix-vector products get launchable schedules.  CPU only."""
import itertools
import math

import numpy as np

import oracle
from paper_2411_18873_amd import synth

POW2 = [1, 2, 4, 8, 16]


def _gene_of(extent, tup):
    divs = [d for d in range(1, extent + 1) if extent % d == 0]
    table = sorted(t for t in itertools.product(divs, repeat=4) if math.prod(t) == extent)
    return table.index(tuple(tup))


def _raw(space, genes):
    raw, _, _, legal = oracle.features(space, np.asarray(genes, dtype=np.uint16), 64)
    return raw.astype(object), legal


def test_hand_computed_matrix_vector(golden):
    rows = golden("hand_mv_xred.txt")
    want, want_legal = [int(t) for t in rows[0]], int(rows[1][0])
    assert len(want) == 64
    pb = synth.gemm(1, 8, 32, elem_bytes=2, hw=(4, 64, 1024, 256, 8))
    sp = oracle.Space(pb, oracle.SPACE_SPLIT_XRED)
    genes = [_gene_of(1, (1, 1, 1, 1)), _gene_of(8, (2, 2, 1, 2)), _gene_of(32, (2, 4, 2, 2)), POW2.index(2),
             POW2.index(2)]
    raw, legal = _raw(sp, np.array(genes).reshape(-1, 1))
    assert [int(v) for v in raw[:, 0]] == want
    assert int(legal[0]) == want_legal


def _walk(op, ext, levels, R, S, stride):
    """Executes one reduction-parallel schedule literally: every block, every thread, every stage, every serial
    step; records each multiply-add's output and reduction coordinate and the operand elements it reads, then
    folds the partial sums of each output with a halving tree.  Returns plain counts."""
    sp_axes = range(4)
    f = levels
    blocks = list(itertools.product(*[range(f[a][0]) for a in sp_axes]))
    threads = list(itertools.product(*[range(f[a][1]) for a in sp_axes], range(f[4][1])))
    serial = list(itertools.product(*[range(f[a][2] * f[a][3]) for a in sp_axes]))
    seen = {}
    thr_loads = set()   # (elements of A, elements of B) one thread reads in one stage
    blk_loads = set()
    macs_per_thread = set()
    loaded_elems = 0
    for blk in blocks:
        for k0 in range(f[4][0]):
            blk_a, blk_b = set(), set()
            for thr in threads:
                a_set, b_set = set(), set()
                for ser in serial:
                    out = tuple((blk[a] * f[a][1] + thr[a]) * f[a][2] * f[a][3] + ser[a] for a in sp_axes)
                    for k23 in range(f[4][2] * f[4][3]):
                        k = ((k0 * f[4][1] + thr[4]) * f[4][2] * f[4][3]) + k23
                        for r in range(R):
                            for s in range(S):
                                seen[(out, k, r, s)] = seen.get((out, k, r, s), 0) + 1
                                if op == "conv":  # out = (n, k_out, h, w); input (n, c, h*st + r, w*st + s), filter (k_out, c, r, s)
                                    a_set.add((out[0], k, out[2] * stride + r, out[3] * stride + s))
                                    b_set.add((out[1], k, r, s))
                                else:             # out = (b, m, n, -); A (b, m, k), B (b, k, n)
                                    a_set.add((out[0], out[1], k))
                                    b_set.add((out[0], k, out[2]))
                thr_loads.add((len(a_set), len(b_set)))
                loaded_elems += len(a_set) + len(b_set)
                blk_a |= a_set
                blk_b |= b_set
            blk_loads.add((len(blk_a), len(blk_b)))
    # every (output, reduction) pair of the operator exactly once
    assert set(seen.values()) == {1}
    assert len(seen) == math.prod(ext[:4]) * ext[4] * R * S
    # the tree over the partial sums of one output
    kt = f[4][1]
    adds = loads = stores = steps = 0
    if kt > 1:
        stores += kt
        half = 1
        while half * 2 < kt:
            half *= 2
        live = kt
        while half >= 1:
            steps += 1
            for t in range(half):
                if t + half < live:
                    adds += 1
                    loads += 2
                    stores += 1
            live = min(live, half)
            half //= 2
    n_out = len(blocks) * (len(threads) // kt) * len(serial)
    assert len(thr_loads) == 1 and len(blk_loads) == 1
    return dict(macs=len(seen), blocks=len(blocks), threads=len(threads), outs_thread=len(serial), n_out=n_out,
                thr_a=next(iter(thr_loads))[0], thr_b=next(iter(thr_loads))[1], blk_a=next(iter(blk_loads))[0],
                blk_b=next(iter(blk_loads))[1], loaded=loaded_elems, tree_adds=adds, tree_loads=loads,
                tree_stores=stores, tree_steps=steps)


def _check_against_walk(pb, op, ext, R, S, stride, n_samples, seed):
    sp = oracle.Space(pb, oracle.SPACE_SPLIT_XRED)
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, n_samples, seed=seed)
    raw, _ = _raw(sp, genes)
    b = pb[9]
    wave, n_cu = pb[11], pb[10]
    some_tree = False
    for c in range(n_samples):
        x = [int(v) for v in raw[:, c]]
        levels = [[x[32 + 4 * a + l] for l in range(4)] for a in range(5)]
        U, V = x[27], x[30]
        w = _walk(op, ext, levels, R, S, stride)
        kt, stages = levels[4][1], levels[4][0]
        some_tree |= kt > 1
        assert x[0] == 2 * w["macs"]
        assert x[1] == 2 * w["macs"] + w["n_out"] * w["tree_adds"]
        assert x[2] * w["blocks"] * w["threads"] == w["macs"]
        assert x[4] == w["outs_thread"] and x[6] == w["blocks"] and x[7] == w["threads"]
        assert x[8] == -(-w["threads"] // wave)
        assert x[10] == min(w["blocks"], n_cu) and x[11] == n_cu - x[10]
        loads_thread_stage = -(-(w["thr_a"] + w["thr_b"]) // V)
        assert x[14] == w["blocks"] * w["threads"] * stages * loads_thread_stage
        assert x[15] == -(-w["loaded"] * b // 32)
        assert x[16] == -(-w["n_out"] * b // 32)
        assert x[18] == (w["threads"] * w["outs_thread"] * 4 if kt > 1 else 0)
        assert x[19] == -(-w["n_out"] * w["tree_stores"] * 4 // 128)
        assert x[20] == w["n_out"] * w["tree_loads"]
        assert x[21] == (x[1] * 8) // (x[15] + x[16])
        assert x[57] == w["blk_a"] and x[58] == w["blk_b"]
        assert x[62] == w["n_out"] and x[63] * x[62] == w["macs"]
        # integer work: per stage 4 per load and 2 of loop control, 2 per unrolled trip, 2 per tree step
        trips = -(-(x[2] // w["outs_thread"]) // U)
        assert x[3] == w["blocks"] * w["threads"] * (stages * (4 * loads_thread_stage + 2) + 2 * trips
                                                     + 2 * w["tree_steps"])
    assert some_tree


def test_walked_schedules_of_a_batched_product():
    pb = synth.bgemm(2, 4, 6, 12, elem_bytes=2, hw=(4, 64, 4096, 256, 8))
    _check_against_walk(pb, "gemm", [2, 4, 6, 1, 12], 1, 1, 1, 60, seed=3)


def test_walked_schedules_of_a_matrix_vector_product():
    pb = synth.gemm(1, 12, 48, elem_bytes=4, hw=(4, 64, 4096, 256, 8))
    _check_against_walk(pb, "gemm", [1, 1, 12, 1, 48], 1, 1, 1, 80, seed=4)


def test_walked_schedules_of_a_convolution():
    # 4x4 image, pad 1, 3x3 filter, stride 1 -> 4x4 outputs; input coordinates are counted unclipped
    pb = synth.conv2d(1, 4, 2, 4, 4, 3, 3, 1, 1, elem_bytes=2, hw=(4, 64, 4096, 256, 8))
    _check_against_walk(pb, "conv", [1, 2, 4, 4, 4], 3, 3, 1, 40, seed=5)
    # stride 2: 7x7 image, pad 1, 3x3 -> 4x4 outputs
    pb = synth.conv2d(1, 2, 2, 7, 7, 3, 3, 2, 1, elem_bytes=4, hw=(4, 64, 4096, 256, 8))
    _check_against_walk(pb, "conv", [1, 2, 4, 4, 2], 3, 3, 2, 30, seed=6)


def test_one_reduction_thread_needs_no_shared_memory_and_no_tree():
    pb = synth.gemm(1, 4096, 1024)
    sp = oracle.Space(pb, oracle.SPACE_SPLIT_XRED)
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, 4096, seed=9)
    raw, _ = _raw(sp, genes)
    alone = raw[49] == 1
    assert alone.any() and (~alone).any()
    assert np.all(raw[18][alone] == 0) and np.all(raw[19][alone] == 0) and np.all(raw[20][alone] == 0)
    assert np.all(raw[1][alone] == raw[0][alone])
    # with a tree: one addition less than partial sums, per output
    assert np.all(raw[1] - raw[0] == raw[62] * (raw[49] - 1))
    assert np.all(raw[7] == raw[33] * raw[37] * raw[41] * raw[45] * raw[49])
    # spaces of the two kinds hold the same gene tuples
    other = oracle.Space(pb, oracle.SPACE_SPLIT)
    assert other.radix == sp.radix
    assert np.array_equal(oracle.enumerate_candidates(other, oracle.MODE_SAMPLE, 4096, seed=9), genes)


def test_matrix_vector_products_get_launchable_schedules():
    """What the kind is for: in the staged reading nearly no schedule of the paper's matrix-vector operators
    (Sec. 7.2) can launch, in the reduction-parallel reading a usable share can."""
    ops = synth.paper_operators()
    for name in ("MV1", "MV2", "MV3", "MV4"):
        staged = oracle.Space(ops[name], oracle.SPACE_SPLIT)
        across = oracle.Space(ops[name], oracle.SPACE_SPLIT_XRED)
        genes = oracle.enumerate_candidates(staged, oracle.MODE_SAMPLE, 1 << 14, seed=11)
        _, _, _, legal_staged = oracle.features(staged, genes, 32)
        _, _, _, legal_across = oracle.features(across, genes, 32)
        assert legal_staged.mean() < 0.04
        assert legal_across.mean() > 3 * max(legal_staged.mean(), 0.01), (name, legal_across.mean())
