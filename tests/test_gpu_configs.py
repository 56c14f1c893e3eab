"""GPU parity, end to end, on the five workload configurations -- at their full sizes and in the
launch configuration bench.py times.  Integer stages are compared bit for bit (all candidates where
the oracle finishes in seconds, a regular sample otherwise); scores on a regular sample plus every
selected candidate (config 5: 2^18 strided candidates, every selected one and every one whose energy lies
within 1 % of its segment's k-th selected energy), each against both oracle modes; selection against the
oracle run on the GPU's own scores ("given identical scores")."""
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


def _bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def _select_and_check(G, energy, latency, legal, S, k, alpha):
    idx, eo, cnt = G.topk_dev(energy, latency, legal, S, k, alpha=alpha)
    io, eo_o, co = oracle.topk(energy.cpu().numpy(), latency.cpu().numpy(), legal.cpu().numpy(), S, k, alpha=alpha)
    assert np.array_equal(cnt, co) and np.array_equal(idx, io)
    assert np.array_equal(eo.view(np.uint32), eo_o.view(np.uint32))
    return idx, cnt


def test_config1_exhaustive_gemm_fp32(G):
    cfg = synth.CONFIGS["c1"]
    n, k, widths = cfg["n"], cfg["k"], cfg["widths"]
    mine, ref = eck.Space(cfg["problem"], eck.SPACE_KNOB), oracle.Space(cfg["problem"], oracle.SPACE_KNOB)
    genes = torch.zeros((6, n), dtype=torch.int16, device="cuda")
    eck.candidate_enumerate(mine, eck.MODE_EXHAUSTIVE, n, genes)
    feat = torch.zeros((32, n), dtype=torch.float32, device="cuda")
    legal = torch.zeros(n, dtype=torch.uint8, device="cuda")
    eck.features_compute(mine, genes, n, 32, eck.F32, feat_out=feat, legal_out=legal)
    genes_o = oracle.enumerate_candidates(ref, oracle.MODE_EXHAUSTIVE, n)
    _, f32_o, _, legal_o = oracle.features(ref, genes_o, 32)
    assert np.array_equal(_bits(genes), genes_o)
    assert np.array_equal(feat.cpu().numpy().view(np.uint32), f32_o.view(np.uint32))
    assert np.array_equal(legal.cpu().numpy(), legal_o)
    scores = []
    for seed in cfg["weight_seeds"]:
        theta = synth.mlp_theta(widths, seed)
        out = torch.zeros(n, dtype=torch.float32, device="cuda")
        eck.costmodel_score(G.make_model(widths, eck.F32, theta), feat, n, out)
        assert G.within(out.cpu().numpy(), oracle.score(widths, theta, f32_o),
                        oracle.score_magnitude(widths, theta, f32_o), 1e-5) <= 1.0
        scores.append(out)
    idx, cnt = _select_and_check(G, scores[0], scores[1], legal, 1, k, cfg["alpha"])
    assert cnt[0] == k
    # the oracle's own end-to-end pick agrees on the selected set up to near-ties of the fp32 scores
    e_o = oracle.score(widths, synth.mlp_theta(widths, cfg["weight_seeds"][0]), f32_o).astype(np.float32)
    l_o = oracle.score(widths, synth.mlp_theta(widths, cfg["weight_seeds"][1]), f32_o).astype(np.float32)
    io, _, _ = oracle.topk(e_o, l_o, legal_o, 1, k, alpha=cfg["alpha"])
    assert len(set(idx[0].tolist()) & set(io[0].tolist())) >= k - 2


def _bf16_pipeline(G, mine, n, seed, rnd, mode, widths, thetas, parents=None, p_mut=0):
    genes = torch.zeros((mine.n_genes, n), dtype=torch.int16, device="cuda")
    eck.candidate_enumerate(mine, mode, n, genes, seed=seed, round=rnd, parents=parents, p_mut_q32=p_mut)
    feat = torch.zeros((64, n), dtype=torch.bfloat16, device="cuda")
    legal = torch.zeros(n, dtype=torch.uint8, device="cuda")
    eck.features_compute(mine, genes, n, 64, eck.BF16, feat_out=feat, legal_out=legal)
    outs = []
    for theta in thetas:
        out = torch.zeros(n, dtype=torch.float32, device="cuda")
        eck.costmodel_score(G.make_model(widths, eck.BF16, theta), feat, n, out)
        outs.append(out)
    return genes, feat, legal, outs


def _check_scores_sample(G, widths, theta, b16_o, got, cols, label=""):
    G.check_bf16_scores(widths, theta, np.ascontiguousarray(b16_o[:, cols]), got.cpu().numpy()[cols], label)


def test_config2_sampled_conv_full_size(G):
    cfg = synth.CONFIGS["c2"]
    n, k, widths = cfg["n"], cfg["k"], cfg["widths"]
    mine, ref = eck.Space(cfg["problem"], eck.SPACE_SPLIT), oracle.Space(cfg["problem"], oracle.SPACE_SPLIT)
    thetas = [synth.mlp_theta(widths, s, bf16=True) for s in cfg["weight_seeds"]]
    genes, feat, legal, (energy, latency) = _bf16_pipeline(G, mine, n, cfg["sample_seed"], 0, eck.MODE_SAMPLE, widths,
                                                           thetas)
    genes_o = oracle.enumerate_candidates(ref, oracle.MODE_SAMPLE, n, seed=cfg["sample_seed"])
    assert np.array_equal(_bits(genes), genes_o)
    _, _, b16_o, legal_o = oracle.features(ref, genes_o, 64)
    assert np.array_equal(_bits(feat), b16_o) and np.array_equal(legal.cpu().numpy(), legal_o)
    idx, cnt = _select_and_check(G, energy, latency, legal, 1, k, cfg["alpha"])
    assert 1 <= cnt[0] <= k  # an untrained latency model leaves few candidates within 1.1x of its minimum
    cols = np.unique(np.concatenate([np.arange(0, n, 97), idx[0][:cnt[0]].astype(np.int64)]))
    _check_scores_sample(G, widths, thetas[0], b16_o, energy, cols, "c2 energy")
    _check_scores_sample(G, widths, thetas[1], b16_o, latency, cols, "c2 latency")
    # "top-k" without the latency gate, too
    i2, e2, c2 = G.topk_dev(energy, None, legal, 1, k)
    io, eo, co = oracle.topk(energy.cpu().numpy(), None, legal_o, 1, k)
    assert np.array_equal(i2, io) and np.array_equal(c2, co)


def test_config3_evolutionary_rounds_full_size(G):
    cfg = synth.CONFIGS["c3"]
    n, k, widths, P = cfg["n"], cfg["k"], cfg["widths"], cfg["survivors"]
    mine, ref = eck.Space(cfg["problem"], eck.SPACE_SPLIT), oracle.Space(cfg["problem"], oracle.SPACE_SPLIT)
    thetas = [synth.mlp_theta(widths, s, bf16=True) for s in cfg["weight_seeds"]]
    parents = torch.zeros((mine.n_genes, P), dtype=torch.int16, device="cuda")
    eck.candidate_enumerate(mine, eck.MODE_SAMPLE, P, parents, seed=cfg["seed"])
    parents_o = oracle.enumerate_candidates(ref, oracle.MODE_SAMPLE, P, seed=cfg["seed"])
    best = []
    for rnd in range(cfg["rounds"]):
        assert np.array_equal(_bits(parents), parents_o)
        genes, feat, legal, (energy, latency) = _bf16_pipeline(G, mine, n, cfg["seed"], rnd + 1, eck.MODE_MUTATE, widths,
                                                               thetas, parents=parents, p_mut=synth.P_MUT_Q32)
        genes_o = oracle.enumerate_candidates(ref, oracle.MODE_MUTATE, n, seed=cfg["seed"], rnd=rnd + 1,
                                              parents=parents_o, p_mut_q32=synth.P_MUT_Q32)
        assert np.array_equal(_bits(genes), genes_o)
        if rnd in (0, cfg["rounds"] - 1):  # the feature check of a whole generation costs a few seconds
            _, _, b16_o, legal_o = oracle.features(ref, genes_o, 64)
            assert np.array_equal(_bits(feat), b16_o) and np.array_equal(legal.cpu().numpy(), legal_o)
            _check_scores_sample(G, widths, thetas[0], b16_o, energy, np.arange(0, n, 257), "c3 round %d" % rnd)
        idx_dev = torch.zeros((1, k), dtype=torch.int32, device="cuda")
        if rnd == 0:
            _select_and_check(G, energy, latency, legal, 1, k, 1.1)
        idx, cnt = _select_and_check(G, energy, latency, legal, 1, k, cfg["alpha"])
        assert cnt[0] == k
        idx_dev.copy_(torch.from_numpy(idx.view(np.int32)))
        eck.candidates_gather(genes, n, idx_dev, k, parents)
        parents_o = genes_o[:, idx[0]]
        best.append(float(energy.cpu().numpy()[idx[0][0]]))
    assert best[-1] <= best[0]  # survivors only improve under a fixed model


def test_config4_rescoring_after_the_update(G):
    cfg = synth.CONFIGS["c4"]
    widths, n = cfg["widths"], cfg["rescore_n"]
    ref, mine = oracle.Space(cfg["problem"], oracle.SPACE_SPLIT), eck.Space(cfg["problem"], eck.SPACE_SPLIT)
    genes_p = oracle.enumerate_candidates(ref, oracle.MODE_SAMPLE, cfg["n_pairs"], seed=cfg["pair_seed"])
    _, f32_p, b16_p, _ = oracle.features(ref, genes_p, 64)
    e_meas = synth.measured_energy(f32_p, cfg["label_seed"])
    model = G.make_model(widths, eck.BF16, synth.mlp_theta(widths, cfg["weight_seeds"][0], bf16=True))
    snr, loss = G.update_gpu(model, G.bf16_dev(b16_p), e_meas, cfg["n_steps"], cfg["minibatch"], lr=cfg["lr"])
    assert np.isfinite(snr) and np.isfinite(loss)
    genes = torch.zeros((mine.n_genes, n), dtype=torch.int16, device="cuda")
    eck.candidate_enumerate(mine, eck.MODE_SAMPLE, n, genes, seed=cfg["sample_seed"] if "sample_seed" in cfg else 2024)
    feat = torch.zeros((64, n), dtype=torch.bfloat16, device="cuda")
    eck.features_compute(mine, genes, n, 64, eck.BF16, feat_out=feat)
    out = torch.zeros(n, dtype=torch.float32, device="cuda")
    eck.costmodel_score(model, feat, n, out)
    # the oracle scores the same candidates with the weights the GPU refit produced (rounded to bf16 as the
    # scorer uses them): isolates the rescoring from the training trajectory
    P = synth.param_count(widths)
    theta = synth.round_to_bf16(model.get_state().cpu().numpy()[:P])
    cols = np.arange(0, n, 509)
    genes_o = oracle.enumerate_candidates(ref, oracle.MODE_SAMPLE, n, seed=2024)
    assert np.array_equal(_bits(genes)[:, cols], genes_o[:, cols])
    _, _, b16_o, _ = oracle.features(ref, np.ascontiguousarray(genes_o[:, cols]), 64)
    assert np.array_equal(_bits(feat)[:, cols], b16_o)
    G.check_bf16_scores(widths, theta, b16_o, out.cpu().numpy()[cols], "c4 rescoring")


@pytest.fixture(scope="module")
def c5(G):
    """The benchmark's step on the benchmark's buffers and through the benchmark's calls: two batched launches, the two
    score launches (the second with the per-shape least latency), the selection on known minima."""
    cfg = synth.CONFIGS["c5"]
    shapes, per, widths, K = cfg["shapes"], cfg["n_per_shape"], cfg["widths"], cfg["k"]
    S, N = len(shapes), len(shapes) * cfg["n_per_shape"]
    spaces = [eck.Space(synth.gemm(*s), eck.SPACE_SPLIT) for s in shapes]
    genes = torch.zeros((5, N), dtype=torch.int16, device="cuda")
    feat = torch.zeros((64, N), dtype=torch.bfloat16, device="cuda")
    legal = torch.zeros(N, dtype=torch.uint8, device="cuda")
    eck.candidate_enumerate_batch(spaces, eck.MODE_SAMPLE, per, genes, [cfg["seed_base"] + s for s in range(S)])
    eck.features_compute_batch(spaces, genes, per, 64, eck.BF16, feat_out=feat, legal_out=legal)
    thetas = [synth.mlp_theta(widths, s, bf16=True) for s in cfg["weight_seeds"]]
    energy = torch.zeros(N, dtype=torch.float32, device="cuda")
    latency = torch.zeros(N, dtype=torch.float32, device="cuda")
    eck.costmodel_score(G.make_model(widths, eck.BF16, thetas[0]), feat, N, energy)
    # as the benchmark runs it: the latency launch also reduces its scores to the least legal latency of every shape,
    # and the selection takes those minima instead of a pass of its own over the latencies
    m_latency = G.make_model(widths, eck.BF16, thetas[1])
    lat_min = torch.zeros(S, dtype=torch.int32, device="cuda")
    eck.costmodel_score_min(m_latency, feat, N, latency, legal, S, lat_min)
    idx_b = torch.zeros((S, K), dtype=torch.int32, device="cuda")
    e_b = torch.zeros((S, K), dtype=torch.float32, device="cuda")
    cnt_b = torch.zeros(S, dtype=torch.int32, device="cuda")
    ws = torch.empty(eck.topk_select_workspace_bytes(N, S, K), dtype=torch.uint8, device="cuda")
    eck.topk_select_known_min(energy, latency, legal, S, K, lat_min, idx_b, e_b, cnt_b, ws, alpha=cfg["alpha"])
    # the same latencies, bit for bit, as the plain scoring call; the minima as numpy finds them; the same selection
    # as the oracle's (and as topk_select's own two passes)
    plain = torch.zeros(N, dtype=torch.float32, device="cuda")
    eck.costmodel_score(m_latency, feat, N, plain)
    assert torch.equal(plain.view(torch.int32), latency.view(torch.int32))
    del plain
    bits = latency.cpu().numpy().view(np.uint32)
    keys = np.where(bits >> 31 != 0, ~bits, bits | np.uint32(0x80000000)).astype(np.uint32)
    keys[(legal.cpu().numpy() == 0) | np.isnan(latency.cpu().numpy())] = 0xFFFFFFFF
    assert np.array_equal(lat_min.cpu().numpy().view(np.uint32), keys.reshape(S, per).min(axis=1))
    idx, cnt = _select_and_check(G, energy, latency, legal, S, K, cfg["alpha"])
    assert np.array_equal(idx_b.cpu().numpy().view(np.uint32), idx) and np.array_equal(cnt_b.cpu().numpy().view(np.uint32), cnt)
    assert cnt.min() > 0
    # the columns whose scores are checked: 2^18 strided candidates, every selected candidate, and every feasible
    # candidate whose energy lies within 1 % of its segment's k-th selected energy (the ones a scoring error
    # could move across the selection boundary)
    e_h, l_h, legal_h = energy.cpu().numpy(), latency.cpu().numpy(), legal.cpu().numpy()
    picked, near = [], []
    for s in range(S):
        seg = slice(s * per, (s + 1) * per)
        sel = idx[s][:cnt[s]].astype(np.int64)
        picked.append(s * per + sel)
        kth = e_h[seg][sel[-1]]
        l_ok = legal_h[seg] != 0
        l_min = l_h[seg][l_ok].min()
        tau = np.float32(l_min) + np.float32(np.float32(cfg["alpha"]) - np.float32(1.0)) * np.abs(np.float32(l_min))
        feasible = l_ok & (l_h[seg] <= tau)
        close = feasible & (np.abs(e_h[seg] - kth) <= 0.01 * abs(kth))
        near.append(s * per + np.flatnonzero(close))
    picked, near = np.concatenate(picked), np.concatenate(near)
    strided = np.arange(0, N, N >> 18)
    cols = np.unique(np.concatenate([strided, picked, near]))
    print("c5 score columns: %d strided, %d selected, %d within 1 %% of a k-th energy" % (len(strided), len(picked),
                                                                                         len(near)), flush=True)
    return dict(cfg=cfg, genes=genes, feat=feat, legal=legal, energy=e_h, latency=l_h, thetas=thetas, idx=idx, cnt=cnt,
                cols=cols, picked=picked)


def test_config5_sweep_full_size_as_benchmarked(G, c5):
    cfg = c5["cfg"]
    shapes, per = cfg["shapes"], cfg["n_per_shape"]
    idx, cnt = c5["idx"], c5["cnt"]
    # integer stages: every 61st candidate of every shape, plus everything selected
    stride = np.arange(0, per, 61)
    genes_h, legal_h = _bits(c5["genes"]), c5["legal"].cpu().numpy()
    for s, shape in enumerate(shapes):
        ref = oracle.Space(synth.gemm(*shape), oracle.SPACE_SPLIT)
        local = np.unique(np.concatenate([stride, idx[s][:cnt[s]].astype(np.int64)]))
        if len(local) & 1:
            local = local[:-1]
        want_genes = np.stack([oracle.enumerate_candidates(ref, oracle.MODE_SAMPLE, 1, seed=cfg["seed_base"] + s,
                                                           first_index=int(c))[:, 0] for c in local[:64]], axis=1)
        cols = s * per + local
        assert np.array_equal(genes_h[:, cols[:64]], want_genes)
        g_sub = np.ascontiguousarray(genes_h[:, cols])
        _, _, b16_o, legal_o = oracle.features(ref, g_sub, 64)
        got = _bits(c5["feat"].index_select(1, torch.from_numpy(cols).cuda()))
        assert np.array_equal(got, b16_o) and np.array_equal(legal_h[cols], legal_o)
    # whole-shape gene check for two shapes
    for s in (0, 37):
        ref = oracle.Space(synth.gemm(*shapes[s]), oracle.SPACE_SPLIT)
        want = oracle.enumerate_candidates(ref, oracle.MODE_SAMPLE, per, seed=cfg["seed_base"] + s)
        assert np.array_equal(genes_h[:, s * per:(s + 1) * per], want)


@pytest.mark.parametrize("which", ["energy", "latency"])
def test_config5_scores_of_the_strided_sample_and_around_every_selection_boundary(G, c5, which):
    """Scores of the 2^24-candidate launch against the oracle, which recomputes genes -> features -> score for
    each checked column itself: 2^18 strided columns, every selected candidate, every candidate within 1 % of a
    segment's k-th energy; both gates (1e-2 M exact, 1e-4 M with bf16 activations)."""
    cfg = c5["cfg"]
    shapes, per, widths = cfg["shapes"], cfg["n_per_shape"], cfg["widths"]
    cols = c5["cols"]
    b16 = np.zeros((64, len(cols)), dtype=np.uint16)
    for s, shape in enumerate(shapes):
        lo, hi = np.searchsorted(cols, [s * per, (s + 1) * per])
        if hi == lo:
            continue
        ref = oracle.Space(synth.gemm(*shape), oracle.SPACE_SPLIT)
        # the oracle's own genes for the whole shape, then its features of the checked columns
        genes_o = oracle.enumerate_candidates(ref, oracle.MODE_SAMPLE, per, seed=cfg["seed_base"] + s)
        sub = np.zeros((genes_o.shape[0], hi - lo + ((hi - lo) & 1)), dtype=np.uint16)
        sub[:, :hi - lo] = genes_o[:, cols[lo:hi] - s * per]
        _, _, b, _ = oracle.features(ref, sub, 64)
        b16[:, lo:hi] = b[:, :hi - lo]
    got_feat = _bits(c5["feat"].index_select(1, torch.from_numpy(cols).cuda()))
    assert np.array_equal(got_feat, b16)
    theta = c5["thetas"][0 if which == "energy" else 1]
    G.check_bf16_scores(widths, theta, b16, c5[which][cols], "c5 " + which)
