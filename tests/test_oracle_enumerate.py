"""Pins for the oracle's candidate generation (exhaustive decode, sampling,
mutation) and its schedule-space tables.  CPU only."""
import itertools
import math

import numpy as np
import pytest

import oracle
from paper_2411_18873_amd import synth

M64 = (1 << 64) - 1
GOLDEN_GAMMA = 0x9E3779B97F4A7C15


def _mix(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def _splitmix_output(state0, nth):
    """nth (1-based) output of SplitMix64 started at state0."""
    return _mix((state0 + GOLDEN_GAMMA * nth) & M64)


def test_local_splitmix_matches_published_vectors(golden):
    for row in golden("splitmix64_kat.txt"):
        seed, outs = int(row[0]), [int(t) for t in row[1:]]
        assert [_splitmix_output(seed, i + 1) for i in range(len(outs))] == outs


@pytest.mark.parametrize("seed,rnd,idx,gene", [(0, 0, 0, 0), (2024, 0, 12345, 3), (7, 5, (1 << 40) + 17, 6),
                                               (M64, 4000000000, (1 << 63) + 5, 15)])
def test_hash_is_splitmix_stream(seed, rnd, idx, gene):
    # stream state = first-stage SplitMix finaliser of seed + gamma*(round+1); word = output 16*idx+gene+1
    key = _mix((seed + GOLDEN_GAMMA * (rnd + 1)) & M64)
    assert oracle.hash64(seed, rnd, idx, gene) == _splitmix_output(key, (idx * 16 + gene + 1) & M64)


def _brute_table(extent):
    divs = [d for d in range(1, extent + 1) if extent % d == 0]
    tuples = [t for t in itertools.product(divs, repeat=4) if t[0] * t[1] * t[2] * t[3] == extent]
    return sorted(tuples)


@pytest.mark.parametrize("extent", [1, 2, 6, 12, 14, 32, 36])
def test_split_table_bruteforce(extent):
    tab = oracle.split_table(extent)
    assert [tuple(int(v) for v in r) for r in tab] == _brute_table(extent)


def _count_formula(extent):
    # ordered factorisations into 4 parts: product over primes of C(a+3, 3)
    n, cnt, p = extent, 1, 2
    while n > 1:
        a = 0
        while n % p == 0:
            n //= p
            a += 1
        if a:
            cnt *= math.comb(a + 3, 3)
        p += 1
    return cnt


@pytest.mark.parametrize("extent,count", [(1, 1), (14, 16), (32, 56), (128, 120), (256, 165), (1024, 286),
                                          (2048, 364), (4096, 455), (8192, 560)])
def test_split_table_sizes(extent, count):
    assert _count_formula(extent) == count
    tab = oracle.split_table(extent)
    assert tab.shape == (count, 4)
    assert np.all(tab.astype(np.uint64).prod(axis=1) == extent)
    as_tuples = [tuple(r) for r in tab.tolist()]
    assert as_tuples == sorted(set(as_tuples))  # strictly increasing lexicographic


def test_space_shapes_of_the_configs():
    c1 = oracle.Space(synth.CONFIGS["c1"]["problem"], oracle.SPACE_KNOB)
    assert c1.radix == [5, 5, 4, 4, 4, 4] and c1.size == 6400
    c2 = oracle.Space(synth.CONFIGS["c2"]["problem"], oracle.SPACE_SPLIT)
    assert c2.radix == [1, 165, 16, 16, 165, 5, 4] and c2.size == 139392000
    c3 = oracle.Space(synth.CONFIGS["c3"]["problem"], oracle.SPACE_SPLIT)
    assert c3.radix == [56, 364, 364, 120, 5, 4]
    g = oracle.Space(synth.gemm(8192, 1024, 4096), oracle.SPACE_SPLIT)
    assert g.radix == [560, 286, 455, 5, 4]


def test_exhaustive_is_a_bijection_first_gene_most_significant():
    sp = oracle.Space(synth.CONFIGS["c1"]["problem"], oracle.SPACE_KNOB)
    genes = oracle.enumerate_candidates(sp, oracle.MODE_EXHAUSTIVE, 6400)
    cols = {tuple(genes[:, i]) for i in range(6400)}
    assert len(cols) == 6400
    for j, r in enumerate(sp.radix):
        assert genes[j].max() == r - 1
    # index 1 moves the last gene; index 4*4*4*4*5 moves the first
    assert tuple(genes[:, 1]) == (0, 0, 0, 0, 0, 1)
    assert tuple(genes[:, 1280]) == (1, 0, 0, 0, 0, 0)
    # numpy's unravel is the same mixed-radix convention
    want = np.array(np.unravel_index(np.arange(6400), sp.radix)).astype(np.uint16)
    assert np.array_equal(genes, want)
    # a window equals the same slice
    win = oracle.enumerate_candidates(sp, oracle.MODE_EXHAUSTIVE, 100, first_index=1234)
    assert np.array_equal(win, genes[:, 1234:1334])
    with pytest.raises(ValueError):
        oracle.enumerate_candidates(sp, oracle.MODE_EXHAUSTIVE, 10, first_index=6395)


def test_sample_follows_multiply_high_of_the_hash():
    sp = oracle.Space(synth.CONFIGS["c2"]["problem"], oracle.SPACE_SPLIT)
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, 257, seed=2024, rnd=3, first_index=1000)
    for i in (0, 1, 100, 256):
        for j, r in enumerate(sp.radix):
            u = oracle.hash64(2024, 3, 1000 + i, j)
            assert genes[j, i] == ((u & 0xFFFFFFFF) * r) >> 32


def test_sample_is_uniform_per_gene():
    sp = oracle.Space(synth.CONFIGS["c2"]["problem"], oracle.SPACE_SPLIT)
    n = 1 << 18
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, n, seed=99)
    for j, r in enumerate(sp.radix):
        assert genes[j].max() < r
        if r == 1:
            continue
        counts = np.bincount(genes[j], minlength=r).astype(np.float64)
        expect = n / r
        chi2 = ((counts - expect) ** 2 / expect).sum()
        dof = r - 1
        # chi-square mean dof, sd sqrt(2 dof): six sigma
        assert abs(chi2 - dof) < 6 * math.sqrt(2 * dof), (j, chi2, dof)
    # different genes of one candidate are not copies of each other
    assert np.corrcoef(genes[1].astype(float), genes[4].astype(float))[0, 1] < 0.02


def test_mutation_rate_and_inheritance():
    sp = oracle.Space(synth.CONFIGS["c3"]["problem"], oracle.SPACE_SPLIT)
    P, n = 1024, 1 << 18
    parents = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, P, seed=7)
    kids = oracle.enumerate_candidates(sp, oracle.MODE_MUTATE, n, seed=7, rnd=1, parents=parents,
                                       p_mut_q32=synth.P_MUT_Q32)
    inherited = parents[:, np.arange(n) % P]
    changed = kids != inherited
    G = sp.n_genes
    for j, r in enumerate(sp.radix):
        # a mutated gene is redrawn over all r values, so it shows as changed w.p. 0.1*(1-1/r)
        p = 0.1 * (1 - 1 / r)
        sd = math.sqrt(p * (1 - p) / n)
        assert abs(changed[j].mean() - p) < 5 * sd, (j, changed[j].mean(), p)
        assert kids[j].max() < r
    p_same = np.prod([1 - 0.1 * (1 - 1 / r) for r in sp.radix])
    same = (~changed).all(axis=0).mean()
    assert abs(same - p_same) < 5 * math.sqrt(p_same * (1 - p_same) / n)
    # coin and value come from the high and low word of the same hash
    for c in (0, 5, 4097, n - 1):
        for j, r in enumerate(sp.radix):
            u = oracle.hash64(7, 1, c, j)
            want = ((u & 0xFFFFFFFF) * r) >> 32 if (u >> 32) < synth.P_MUT_Q32 else parents[j, c % P]
            assert kids[j, c] == want
    # p = 0 copies, p = 2^32-1 (almost) always redraws
    copies = oracle.enumerate_candidates(sp, oracle.MODE_MUTATE, 4096, seed=7, rnd=2, parents=parents, p_mut_q32=0)
    assert np.array_equal(copies, parents[:, np.arange(4096) % P])
    assert G == 6


def test_crossover_follows_its_definition_from_the_hash():
    """Every gene of a child is re-derived here from the independent SplitMix model: second parent from word 14,
    source mask from word 15, mutation coin and value from the gene's own word."""
    sp = oracle.Space(synth.CONFIGS["c3"]["problem"], oracle.SPACE_SPLIT)
    P, n, seed, rnd, first, p_mut = 37, 3000, 7, 4, 1234567, synth.P_MUT_Q32
    parents = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, P, seed=3)
    kids = oracle.enumerate_candidates(sp, oracle.MODE_CROSSOVER, n, seed=seed, rnd=rnd, first_index=first,
                                       parents=parents, p_mut_q32=p_mut)
    key = _mix((seed + GOLDEN_GAMMA * (rnd + 1)) & M64)
    word = lambda c, g: _splitmix_output(key, 16 * c + g + 1)
    for i in range(0, n, 7):
        c = first + i
        pa, pb = c % P, ((word(c, 14) & 0xFFFFFFFF) * P) >> 32
        mask = word(c, 15)
        for g in range(sp.n_genes):
            u = word(c, g)
            want = parents[g, pb if (mask >> g) & 1 else pa]
            if (u >> 32) < p_mut:
                want = ((u & 0xFFFFFFFF) * sp.radix[g]) >> 32
            assert kids[g, i] == want


def test_crossover_statistics_and_degenerate_cases():
    sp = oracle.Space(synth.CONFIGS["c3"]["problem"], oracle.SPACE_SPLIT)
    P, n = 64, 1 << 15
    parents = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, P, seed=11)
    assert len({tuple(parents[:, j]) for j in range(P)}) == P
    kids = oracle.enumerate_candidates(sp, oracle.MODE_CROSSOVER, n, seed=5, rnd=1, parents=parents, p_mut_q32=0)
    # without mutation every gene is one of the two parents' genes, about half of them the second parent's
    pa = np.arange(n) % P
    from_a = kids == parents[:, pa]
    others = ~from_a
    assert 0.40 < others.mean() < 0.52        # a little under 1/2: the two parents sometimes agree on a gene
    for g in range(sp.n_genes):
        assert set(np.unique(kids[g])) <= set(np.unique(parents[g]))
    # one parent only: crossover has nothing to mix, children are copies
    one = parents[:, :1].copy()
    kids1 = oracle.enumerate_candidates(sp, oracle.MODE_CROSSOVER, 100, seed=5, rnd=1, parents=one, p_mut_q32=0)
    assert np.all(kids1 == one)
    # with mutation, the mutated fraction per gene is p (1 - P(redraw equals the inherited value))
    kids_m = oracle.enumerate_candidates(sp, oracle.MODE_CROSSOVER, n, seed=5, rnd=1, parents=parents,
                                         p_mut_q32=synth.P_MUT_Q32)
    changed = (kids_m != kids).mean(axis=1)
    assert np.all(changed < 0.1 + 0.01) and np.all(changed > 0.1 * (1 - 1 / 4) - 0.02)


def test_dedup_keeps_first_occurrences_like_numpy_unique():
    rng = np.random.default_rng(2)
    genes = rng.integers(0, 3, size=(4, 2000)).astype(np.uint16)      # 81 distinct tuples, many repeats
    keep = oracle.dedup(genes)
    _, first = np.unique(genes.T, axis=0, return_index=True)
    want = np.zeros(2000, dtype=np.uint8)
    want[first] = 1
    assert np.array_equal(keep, want) and keep.sum() == 81
    assert np.all(oracle.dedup(np.arange(50, dtype=np.uint16)[None, :]) == 1)
    same = np.zeros((3, 10), dtype=np.uint16)
    assert list(oracle.dedup(same)) == [1] + [0] * 9
    # n < ld: columns past n are ignored
    assert list(oracle.dedup(same, n=4)) == [1, 0, 0, 0]
