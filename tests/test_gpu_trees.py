"""GPU parity of the boosted-tree cost model (treemodel_score, treemodel_update) against the oracle.

Scores: the kernel adds leaf values in fp32 in tree order, which is the oracle's fp32-sequential mode, so the
comparison is bit for bit; against the oracle's fp64 sum the gap is bounded by the rounding of T additions.
Boosting: gradient statistics are exact integers on both sides and the gains are the same fp64 expressions, so
the appended trees (features, thresholds, leaf values) are compared bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_18873_amd import eck, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _pairs(n, seed=11):
    cfg = synth.CONFIGS["c4"]
    ref = oracle.Space(cfg["problem"], oracle.SPACE_SPLIT)
    genes = oracle.enumerate_candidates(ref, oracle.MODE_SAMPLE, n + (n & 1), seed=seed)
    _, f32, b16, _ = oracle.features(ref, genes, 64)
    e = synth.measured_energy(f32[:, :n], cfg["label_seed"])
    return f32, b16, e


def _random_ensemble(n_feat, depth, T, seed):
    rng = np.random.default_rng(seed)
    nodes, leaves = (1 << depth) - 1, 1 << depth
    nf = rng.integers(0, n_feat, size=(T, nodes)).astype(np.uint8)
    nt = (rng.integers(0, 200, size=(T, nodes)) * 0.25).astype(np.float32)
    odd = rng.random((T, nodes)) < 0.3
    nt[odd] = rng.uniform(0, 50, size=odd.sum()).astype(np.float32)   # thresholds off the bin grid too
    nt[rng.random((T, nodes)) < 0.05] = np.inf
    lf = (rng.standard_normal((T, leaves)) * 0.1).astype(np.float32)
    return nf, nt, lf


def _load(trees, G, nf, nt, lf):
    trees.set(torch.from_numpy(nf).cuda(), torch.from_numpy(nt).cuda(), torch.from_numpy(lf).cuda())


def _score(trees, feat_dev, n):
    out = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    eck.treemodel_score(trees, feat_dev, n, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("depth,T", [(6, 70), (6, 3), (1, 5), (8, 21), (4, 256)])
def test_score_matches_the_oracle_bit_for_bit(G, depth, T):
    n = 5000 + 37
    f32, b16, _ = _pairs(n)
    nf, nt, lf = _random_ensemble(64, depth, T, seed=depth * 1000 + T)
    base = float(np.float32(0.37))
    trees = eck.Trees(64, depth, T, base)
    _load(trees, G, nf, nt, lf)
    for feat_dev, feat_ref in ((G.to_dev(f32), f32), (G.bf16_dev(b16), oracle.bf16_bits_to_f32(b16))):
        got = _score(trees, feat_dev, n)
        want32 = oracle.trees_predict(64, depth, nf, nt, lf, base, feat_ref, n=n, fp32_sequential=True)
        assert np.array_equal(got, want32.astype(np.float32))
        want64 = oracle.trees_predict(64, depth, nf, nt, lf, base, feat_ref, n=n)
        bound = (T + 1) * 2.0 ** -23 * (abs(base) + np.abs(lf).max(axis=1).sum())
        assert np.max(np.abs(got - want64)) <= bound


def test_score_edge_cases(G, golden):
    # the hand-walked ensemble of the oracle's pin, through the GPU
    rows = golden("hand_trees.txt")
    base = float(rows[0][0])
    tr = [[float(t) for t in r] for r in rows[1:3]]
    nf = np.array([t[0:3] for t in tr], dtype=np.uint8)
    nt = np.array([t[3:6] for t in tr], dtype=np.float32)
    lf = np.array([t[6:10] for t in tr], dtype=np.float32)
    cases = np.array([[float(t) for t in r] for r in rows[3:]], dtype=np.float64)
    x = np.zeros((3, 6), dtype=np.float32)
    x[:, :5] = cases[:, :3].T
    trees = eck.Trees(3, 2, 4, base)
    assert trees.n_trees == 0
    assert np.all(_score(trees, G.to_dev(x), 5) == np.float32(base))       # no trees: the base score
    _load(trees, G, nf, nt, lf)
    assert trees.n_trees == 2
    assert np.allclose(_score(trees, G.to_dev(x), 5), cases[:, 3], rtol=0, atol=1e-6)
    a, b, c = trees.get()
    assert np.array_equal(a.cpu().numpy(), nf) and np.array_equal(b.cpu().numpy(), nt) and np.array_equal(c.cpu().numpy(), lf)
    # a feature index beyond n_feat reads the last feature
    nf_bad = nf.copy()
    nf_bad[0, 0] = 200
    nf_clamped = nf.copy()
    nf_clamped[0, 0] = 2
    _load(trees, G, nf_bad, nt, lf)
    want = oracle.trees_predict(3, 2, nf_clamped, nt, lf, base, x, n=5, fp32_sequential=True)
    assert np.array_equal(_score(trees, G.to_dev(x), 5), want.astype(np.float32))
    # nothing is written past n
    out = torch.full((6,), 7.0, dtype=torch.float32, device="cuda")
    eck.treemodel_score(trees, G.to_dev(x), 5, out)
    torch.cuda.synchronize()
    assert out.cpu().numpy()[5] == 7.0


@pytest.mark.parametrize("n_feat,depth,T,bf16", [(5, 3, 9, True), (5, 3, 9, False), (200, 6, 20, True), (100, 5, 17, False),
                                                  (1, 2, 3, True), (33, 8, 10, True)])
def test_score_feature_counts_off_the_beaten_path(G, n_feat, depth, T, bf16):
    """Feature counts that are no multiple of the staging width, and ones large enough that only the smaller
    block of candidates fits a compute unit."""
    rng = np.random.default_rng(n_feat * 7 + depth)
    n = 3000 + 11
    x = rng.uniform(0, 50, size=(n_feat, n + 1)).astype(np.float32)
    if bf16:
        bits = (x.view(np.uint32) >> 16).astype(np.uint16)
        feat_dev, feat_ref = G.bf16_dev(bits), oracle.bf16_bits_to_f32(bits)
    else:
        feat_dev, feat_ref = G.to_dev(x), x
    nf, nt, lf = _random_ensemble(n_feat, depth, T, seed=n_feat + T)
    trees = eck.Trees(n_feat, depth, T, 0.1)
    _load(trees, G, nf, nt, lf)
    got = _score(trees, feat_dev, n)
    want = oracle.trees_predict(n_feat, depth, nf, nt, lf, 0.1, feat_ref, n=n, fp32_sequential=True)
    assert np.array_equal(got, want.astype(np.float32))


def test_score_special_values_and_thresholds_between_bfloat16_values(G):
    """bfloat16 features are compared as integer keys against thresholds rounded up to bfloat16.  Every decision
    must stay that of the float comparison x < t: negative values, both zeros, infinities, NaN (never below
    anything), subnormals, and thresholds on, just above and just below a bfloat16 value."""
    rng = np.random.default_rng(5)
    n, n_feat, depth, T = 4096, 16, 4, 24
    special = np.array([0x0000, 0x8000, 0x7F80, 0xFF80, 0x7FC0, 0xFFC0, 0x0001, 0x8001, 0x0080, 0x8080, 0x3F80, 0xBF80,
                        0x7F7F, 0xFF7F, 0x4000, 0xC000], dtype=np.uint16)
    b16 = rng.integers(0, 1 << 16, size=(n_feat, n), dtype=np.uint16)
    b16[:, :512] = special[rng.integers(0, special.size, size=(n_feat, 512))]
    x = oracle.bf16_bits_to_f32(b16)
    nodes, leaves = (1 << depth) - 1, 1 << depth
    nf = rng.integers(0, n_feat, size=(T, nodes)).astype(np.uint8)
    # thresholds: values the features take, and their float neighbours on either side; zeros, infinities, NaN
    picks = x[rng.integers(0, n_feat, size=(T, nodes)), rng.integers(0, n, size=(T, nodes))].astype(np.float32)
    picks[~np.isfinite(picks)] = 1.5
    side = rng.integers(0, 3, size=(T, nodes))
    nt = np.where(side == 0, picks, np.where(side == 1, np.nextafter(picks, np.float32(np.inf)),
                                             np.nextafter(picks, np.float32(-np.inf)))).astype(np.float32)
    extra = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-40, -1e-40, 3.0e38, -3.0e38], dtype=np.float32)
    where = rng.random((T, nodes)) < 0.2
    nt[where] = extra[rng.integers(0, extra.size, size=where.sum())]
    lf = (rng.standard_normal((T, leaves)) * 0.1).astype(np.float32)
    trees = eck.Trees(n_feat, depth, T, 0.25)
    _load(trees, G, nf, nt, lf)
    with np.errstate(invalid="ignore"):
        want = oracle.trees_predict(n_feat, depth, nf, nt, lf, 0.25, x, n=n, fp32_sequential=True).astype(np.float32)
    got_bf16 = _score(trees, G.bf16_dev(b16), n)
    assert np.array_equal(got_bf16, want)
    got_f32 = _score(trees, G.to_dev(x), n)       # the float path on the same values
    assert np.array_equal(got_f32, want)


def _boost_gpu(trees, feat_dev, e, rounds, eta, lam):
    snr = torch.zeros(1, dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(eck.treemodel_update_workspace_bytes(trees, e.size), dtype=torch.uint8, device="cuda")
    eck.treemodel_update(trees, feat_dev, torch.from_numpy(e).cuda(), rounds, snr, loss, ws, eta=eta, lam=lam)
    torch.cuda.synchronize()
    return float(snr.item()), float(loss.item())


def _empty(depth, T):
    return (np.zeros((T, (1 << depth) - 1), dtype=np.uint8), np.zeros((T, (1 << depth) - 1), dtype=np.float32),
            np.zeros((T, 1 << depth), dtype=np.float32))


@pytest.mark.parametrize("n_pairs,depth,rounds,bf16", [(4096, 6, 20, True), (1000, 4, 8, False), (77, 3, 5, True),
                                                       (2048, 8, 3, True)])
def test_boosting_appends_the_oracles_trees(G, n_pairs, depth, rounds, bf16):
    f32, b16, e = _pairs(n_pairs)
    eta, lam, base = float(np.float32(0.3)), float(np.float32(1.0)), float(np.float32(0.5))
    feat_ref = oracle.bf16_bits_to_f32(b16) if bf16 else f32
    feat_dev = G.bf16_dev(b16) if bf16 else G.to_dev(f32)
    nf, nt, lf = _empty(depth, rounds)
    snr_o, loss_o = oracle.trees_boost(64, depth, nf, nt, lf, 0, rounds, base, feat_ref[:, :n_pairs], e, eta=eta, lam=lam)
    trees = eck.Trees(64, depth, rounds, base)
    # the pairs are the first n_pairs columns of a wider matrix (ld > n_pairs when n_pairs is odd)
    snr_g, loss_g = _boost_gpu(trees, feat_dev, e, rounds, eta, lam)
    assert trees.n_trees == rounds
    a, b, c = (t.cpu().numpy() for t in trees.get())
    assert np.array_equal(a, nf), "split features differ"
    assert np.array_equal(b, nt), "thresholds differ"
    assert np.array_equal(c.view(np.uint32), lf.view(np.uint32)), "leaf values differ"
    assert abs(snr_g - snr_o) <= 1e-6 * snr_o and abs(loss_g - loss_o) <= 1e-6 * loss_o
    assert np.isfinite(loss_g) and loss_g > 0


def test_boosting_in_two_calls_equals_one_call_and_improves_the_fit(G):
    f32, b16, e = _pairs(4096)
    eta, lam, base = float(np.float32(0.3)), float(np.float32(1.0)), float(np.float32(0.5))
    feat_dev = G.bf16_dev(b16)
    one = eck.Trees(64, 5, 16, base)
    _boost_gpu(one, feat_dev, e, 16, eta, lam)
    two = eck.Trees(64, 5, 16, base)
    snr1, loss1 = _boost_gpu(two, feat_dev, e, 6, eta, lam)
    snr2, loss2 = _boost_gpu(two, feat_dev, e, 10, eta, lam)
    for x, y in zip(one.get(), two.get()):
        assert torch.equal(x, y)
    assert snr2 > snr1 and loss2 < loss1                      # entry SNR of the second call = after six trees
    # zero rounds: reports the quality of the ensemble as it stands, appends nothing
    snr3, loss3 = _boost_gpu(two, feat_dev, e, 0, eta, lam)
    assert two.n_trees == 16 and snr3 > snr2 and abs(loss3 - loss2) <= 1e-6 * loss2
    # rescoring a larger population with the fitted ensemble: same numbers as the oracle
    n = 20000
    f32b, b16b, _ = _pairs(n, seed=5)
    a, b, c = (t.cpu().numpy() for t in two.get())
    got = _score(two, G.bf16_dev(b16b), n)
    want = oracle.trees_predict(64, 5, a, b, c, base, oracle.bf16_bits_to_f32(b16b), n=n, fp32_sequential=True)
    assert np.array_equal(got, want.astype(np.float32))


def test_boosting_rejects_bad_energies_without_changing_predictions(G):
    f32, b16, e = _pairs(512)
    base = float(np.float32(0.5))
    feat_dev = G.bf16_dev(b16)
    trees = eck.Trees(64, 4, 8, base)
    _boost_gpu(trees, feat_dev, e, 4, 0.3, 1.0)
    before = _score(trees, feat_dev, 512)
    bad = e.copy()
    bad[100] = -1.0
    snr, loss = _boost_gpu(trees, feat_dev, bad, 2, 0.3, 1.0)
    assert np.isnan(snr) and np.isnan(loss)
    assert np.array_equal(_score(trees, feat_dev, 512), before)
    a, b, c = (t.cpu().numpy() for t in trees.get())
    assert np.all(np.isinf(b[4:])) and np.all(c[4:] == 0)
    # the same two calls on the oracle leave the same ensemble, tree for tree: six trees, the last two empty
    nodes, leaves = 15, 16
    nf, nt, lf = np.zeros((8, nodes), np.uint8), np.zeros((8, nodes), np.float32), np.zeros((8, leaves), np.float32)
    x = oracle.bf16_bits_to_f32(b16)
    oracle.trees_boost(64, 4, nf, nt, lf, 0, 4, base, x, e, eta=float(np.float32(0.3)), lam=1.0)
    s_o, l_o = oracle.trees_boost(64, 4, nf, nt, lf, 4, 2, base, x, bad, eta=float(np.float32(0.3)), lam=1.0)
    assert np.isnan(s_o) and np.isnan(l_o) and trees.n_trees == 6
    assert np.array_equal(a, nf[:6]) and np.array_equal(b, nt[:6]) and np.array_equal(c.view(np.uint32), lf[:6].view(np.uint32))


def test_tree_scores_at_the_benchmark_size(G):
    """The c5 population (2^24 candidates of 64 GEMM shapes, bf16 features) scored by an ensemble boosted on
    2048 measured pairs, in the launch configuration bench.py --only treescore times; every 4099th candidate
    and the ends of the range are checked against the oracle, bit for bit."""
    cfg = synth.CONFIGS["c5"]
    shapes, per = cfg["shapes"], cfg["n_per_shape"]
    S, N = len(shapes), len(shapes) * cfg["n_per_shape"]
    spaces = [eck.Space(synth.gemm(*s), eck.SPACE_SPLIT) for s in shapes]
    seeds = [cfg["seed_base"] + s for s in range(S)]
    genes = torch.zeros((5, N), dtype=torch.int16, device="cuda")
    feat = torch.zeros((64, N), dtype=torch.bfloat16, device="cuda")
    eck.candidate_enumerate_batch(spaces, eck.MODE_SAMPLE, per, genes, seeds)
    eck.features_compute_batch(spaces, genes, per, 64, eck.BF16, feat_out=feat)
    # measured pairs: 32 candidates of every shape, as in the benchmark
    pg = torch.zeros((5, 2048), dtype=torch.int16, device="cuda")
    pf = torch.zeros((64, 2048), dtype=torch.bfloat16, device="cuda")
    eck.candidate_enumerate_batch(spaces, eck.MODE_SAMPLE, 32, pg, [5000 + s for s in range(S)])
    eck.features_compute_batch(spaces, pg, 32, 64, eck.BF16, feat_out=pf)
    torch.cuda.synchronize()
    e = synth.measured_energy(pf.float().cpu().numpy(), 13)
    base = float(np.float32(0.5))
    trees = eck.Trees(64, 6, 100, base)
    snr, loss = _boost_gpu(trees, pf, e, 100, float(np.float32(0.3)), float(np.float32(1.0)))
    assert np.isfinite(snr) and loss < 1e-3
    out = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
    eck.treemodel_score(trees, feat, N, out)
    torch.cuda.synchronize()
    cols = np.unique(np.concatenate([np.arange(0, N, 4099), np.arange(N - 300, N), np.arange(0, 300)]))
    sub = feat[:, torch.from_numpy(cols).cuda()].view(torch.int16).cpu().numpy().view(np.uint16)
    a, b, c = (t.cpu().numpy() for t in trees.get())
    want = oracle.trees_predict(64, 6, a, b, c, base, oracle.bf16_bits_to_f32(sub), fp32_sequential=True)
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    assert np.array_equal(got[cols], want.astype(np.float32))


def test_the_two_model_forms_on_the_same_measurements(G):
    """The model form the workloads prescribe (MLP, refitted by Adam on Eq. (1)) beside the paper's own (boosted
    trees, Sec. 5.4) on one set of simulated measurements: 3072 kernels of config 2's space to fit, 1024 held out.
    Both must rank the held-out kernels nearly as the meter does; the figures are printed for the record."""
    n, n_train = 4096, 3072
    f32, b16, _ = _pairs(n)
    energy, _ = synth.simulated_kernel_metrics(f32[:, :n], 21, 0)
    feat = G.bf16_dev(b16)
    train = torch.from_numpy(energy[:n_train].copy()).cuda()
    snr = torch.zeros(1, dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    y = energy / energy[:n_train].max()
    held = slice(n_train, n)

    trees = eck.Trees(64, 6, 100, 0.5)
    ws = torch.empty(eck.treemodel_update_workspace_bytes(trees, n_train), dtype=torch.uint8, device="cuda")
    eck.treemodel_update(trees, feat, train, 100, snr, loss, ws, eta=0.3, lam=1.0)
    p_trees = _score(trees, feat, n)

    widths = [64, 256, 256, 1]
    model = eck.Model(widths, eck.BF16)
    model.set_state(torch.from_numpy(synth.mlp_theta(widths, 3, bf16=False)).cuda())
    ws = torch.empty(eck.costmodel_update_workspace_bytes(model, n_train, 512), dtype=torch.uint8, device="cuda")
    for _ in range(50):                                           # 3000 Adam steps = 500 passes over the pairs
        eck.costmodel_update(model, feat, train, 60, 512, snr, loss, ws, lr=1e-3)
    p_mlp = torch.zeros(n, dtype=torch.float32, device="cuda")
    eck.costmodel_score(model, feat, n, p_mlp)
    torch.cuda.synchronize()
    p_mlp = p_mlp.cpu().numpy()

    def rank_corr(a, b):
        return np.corrcoef(np.argsort(np.argsort(a)), np.argsort(np.argsort(b)))[0, 1]
    for name, p in (("trees", p_trees), ("mlp", p_mlp)):
        eq1 = float(np.mean((p[held] - y[held]) ** 2 / y[held]))
        print("%s: held-out r = %.4f, rank correlation = %.4f, Eq. (1) loss = %.3e"
              % (name, np.corrcoef(p[held], y[held])[0, 1], rank_corr(p[held], y[held]), eq1))
    assert rank_corr(p_trees[held], y[held]) > 0.9
    assert rank_corr(p_mlp[held], y[held]) > 0.9
