#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

Workload ("c5", the whole-network sweep): 64 GEMM shapes x 2^18 seeded schedule
samples = 2^24 candidates, 64 bf16 features, energy and latency models
64-512-512-1 (bf16 on the matrix cores), per-shape top-32 under the
latency-then-energy objective.  One step =

    candidate_enumerate (64 spaces) -> features_compute (64 spaces)
    -> costmodel_score (energy) -> costmodel_score_min (latency, and the least legal latency of every shape)
    -> topk_select_known_min (64 segments, k = 32, alpha = 1.1)
    -> costmodel_update (energy model, 2048 measured pairs resident in HBM, one epoch = 4 Adam steps)

Everything is resident in HBM before the timed region.  Prints ONE JSON line: the contract's keys for
the c5 step (ms_per_step = the median of the timed steps), `roofline` for the score kernel,
`hbm` for the calls that only move data (features; top-k for alpha = 1.1, for alpha = inf and, for
comparison, for alpha = 1.1 when the selection has to find the least latencies itself),
`other_configs` (configs 1-4, each timed after the c5 region) and `cpu_baseline` (the oracle on 2^20 candidates).
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_FLOPS = 2.5e15  # MI355X dense bf16 matrix peak
PEAK_HBM = 8e12

# HBM bytes of one score launch on c5 as the counters saw them (FETCH_SIZE x calibration + WRITE_SIZE, rocprofv3 --pmc):
# a constant of the profile named here, not a measurement of this run
TRAFFIC = {"file": "profiles/c5_hbm_traffic_pmc.txt", "score_bf16_kernel<64,512,512>": 2.167e9 + 0.0671e9}


def cpu_baseline(cfg, sample_log2=20):
    """The oracle, as it stands, on a bounded sample of the same workload: one shape, 2^sample_log2
    candidates through enumerate -> features -> two scores -> top-k, plus the same 4-step update."""
    import numpy as np

    import oracle
    from paper_2411_18873_amd import synth

    n = 1 << sample_log2
    widths = cfg["widths"]
    m, nn, k = cfg["shapes"][21]
    sp = oracle.Space(synth.gemm(m, nn, k), oracle.SPACE_SPLIT)
    th_e = synth.mlp_theta(widths, cfg["weight_seeds"][0], bf16=True)
    th_l = synth.mlp_theta(widths, cfg["weight_seeds"][1], bf16=True)
    P = synth.param_count(widths)
    t0 = time.perf_counter()
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, n, seed=cfg["seed_base"] + 21)
    _, _, b16, legal = oracle.features(sp, genes, cfg["n_feat"])
    x = oracle.bf16_bits_to_f32(b16)
    e = oracle.score(widths, th_e, x).astype(np.float32)
    lat = oracle.score(widths, th_l, x).astype(np.float32)
    oracle.topk(e, lat, legal, 1, cfg["k"], alpha=cfg["alpha"])
    t1 = time.perf_counter()
    # update share: the step refits on 2048 pairs per 2^24 candidates; charge the sample its proportional part
    upd_rows = 2048
    state = np.concatenate([th_e.astype(np.float64), np.zeros(2 * P + 1)])
    meas = synth.measured_energy(x[:, :upd_rows], 13)
    t2 = time.perf_counter()
    oracle.update(widths, state, x[:, :upd_rows], meas, 4, 512, bf16_weights=True)
    t3 = time.perf_counter()
    total = (t1 - t0) + (t3 - t2) * (n / float(cfg["n_per_shape"] * len(cfg["shapes"])))
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": n / total, "unit": "candidates/s", "cores": threads, "kind": "oracle",
            "sample": "shape (%d,%d,%d), 2^%d candidates: enumerate+features+2 scores+top-%d in %.2f s; "
                      "4-step update on 2048 pairs %.2f s charged pro rata" % (m, nn, k, sample_log2, cfg["k"],
                                                                            t1 - t0, t3 - t2)}


class Timer:
    """Milliseconds between HIP events on the stream the library launches on (torch's current stream)."""

    def __init__(self, torch):
        self.torch, self.spans = torch, {}

    def call(self, name, fn):
        a, b = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        self.spans.setdefault(name, []).append((a, b))

    def median(self, name):
        return statistics.median(a.elapsed_time(b) for a, b in self.spans[name])

    def repeat(self, name, fn, reps, warm=3):
        for _ in range(warm):
            fn()
        for _ in range(reps):
            self.call(name, fn)
        self.torch.cuda.synchronize()
        return self.median(name)


def flop_per_candidate(widths):
    return 2 * sum(fi * fo for fi, fo in zip(widths[:-1], widths[1:]))


def other_configs(torch, np, eck, synth, reps):
    """Configs 1-4, each as the chain of library calls its description names, timed between HIP events on
    resident buffers: median of `reps` passes."""
    dev = torch.device("cuda:0")
    T = Timer(torch)
    out = {}

    def upload(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    def models(cfg, dtype):
        ms = []
        for seed in cfg["weight_seeds"]:
            m = eck.Model(cfg["widths"], dtype)
            m.set_state(upload(synth.mlp_theta(cfg["widths"], seed, bf16=dtype == eck.BF16)))
            ms.append(m)
        return ms

    def select_buffers(n, S, k, m_latency=0):
        return (torch.zeros((S, k), dtype=torch.int32, device=dev), torch.zeros((S, k), dtype=torch.float32, device=dev),
                torch.zeros(S, dtype=torch.int32, device=dev),
                torch.empty(eck.topk_select_workspace_bytes(n, S, k, m_latency=m_latency), dtype=torch.uint8, device=dev))

    # ---- config 1: 6400 exhaustive schedules of one GEMM, fp32 model, top-16 under alpha = 1.1
    cfg = synth.CONFIGS["c1"]
    n, k = cfg["n"], cfg["k"]
    sp = eck.Space(cfg["problem"], eck.SPACE_KNOB)
    genes = torch.zeros((sp.n_genes, n), dtype=torch.int16, device=dev)
    feat = torch.zeros((32, n), dtype=torch.float32, device=dev)
    legal = torch.zeros(n, dtype=torch.uint8, device=dev)
    e, l = torch.zeros(n, dtype=torch.float32, device=dev), torch.zeros(n, dtype=torch.float32, device=dev)
    me, ml = models(cfg, eck.F32)
    idx, eo, cnt, ws = select_buffers(n, 1, k)

    def c1():
        eck.candidate_enumerate(sp, eck.MODE_EXHAUSTIVE, n, genes)
        eck.features_compute(sp, genes, n, 32, eck.F32, feat_out=feat, legal_out=legal)
        eck.costmodel_score(me, feat, n, e)
        eck.costmodel_score(ml, feat, n, l)
        eck.topk_select(e, l, legal, 1, k, idx, eo, cnt, ws, alpha=cfg["alpha"])

    ms = T.repeat("c1", c1, reps)
    assert int(cnt.item()) == k
    out["c1"] = {"workload": "6400 exhaustive GEMM schedules, 32 fp32 features, 2 x MLP 32-64-64-1 fp32, top-16",
                 "ms": ms, "candidates_per_s": n / (ms * 1e-3), "launches": 6,
                 "bound": "launch latency (6 dependent launches, 77 KB of genes, 0.8 MB of features)"}

    # ---- config 2: 2^20 sampled schedules of one convolution, bf16 models 64-256-256-1, top-64
    cfg = synth.CONFIGS["c2"]
    n, k = cfg["n"], cfg["k"]
    sp2 = eck.Space(cfg["problem"], eck.SPACE_SPLIT)
    genes = torch.zeros((sp2.n_genes, n), dtype=torch.int16, device=dev)
    feat = torch.zeros((64, n), dtype=torch.bfloat16, device=dev)
    legal = torch.zeros(n, dtype=torch.uint8, device=dev)
    e, l = torch.zeros(n, dtype=torch.float32, device=dev), torch.zeros(n, dtype=torch.float32, device=dev)
    me2, ml2 = models(cfg, eck.BF16)
    idx, eo, cnt, ws = select_buffers(n, 1, k)

    def c2():
        eck.candidate_enumerate(sp2, eck.MODE_SAMPLE, n, genes, seed=cfg["sample_seed"])
        eck.features_compute(sp2, genes, n, 64, eck.BF16, feat_out=feat, legal_out=legal)
        T.call("c2.score", lambda: eck.costmodel_score(me2, feat, n, e))
        eck.costmodel_score(ml2, feat, n, l)
        eck.topk_select(e, l, legal, 1, k, idx, eo, cnt, ws, alpha=cfg["alpha"])

    ms = T.repeat("c2", c2, reps)
    score_ms = T.median("c2.score")
    flop = flop_per_candidate(cfg["widths"])
    out["c2"] = {"workload": "2^20 sampled conv schedules, 64 bf16 features, 2 x MLP 64-256-256-1 bf16, top-64 (alpha 1.1)",
                 "ms": ms, "candidates_per_s": n / (ms * 1e-3), "score_ms": score_ms,
                 "score_frac_of_bf16_peak": n * flop / (score_ms * 1e-3) / PEAK_BF16_FLOPS}

    # ---- config 3: 8 evolutionary rounds, each 1024 survivors -> 2^20 children -> top-1024
    cfg = synth.CONFIGS["c3"]
    n, k, P = cfg["n"], cfg["k"], cfg["survivors"]
    sp3 = eck.Space(cfg["problem"], eck.SPACE_SPLIT)
    genes = torch.zeros((sp3.n_genes, n), dtype=torch.int16, device=dev)
    parents = torch.zeros((sp3.n_genes, P), dtype=torch.int16, device=dev)
    me3, ml3 = models(cfg, eck.BF16)
    idx, eo, cnt, ws = select_buffers(n, 1, k)

    def c3_round(r):
        eck.candidate_enumerate(sp3, eck.MODE_MUTATE, n, genes, seed=cfg["seed"], round=r + 1, parents=parents,
                                p_mut_q32=synth.P_MUT_Q32)
        eck.features_compute(sp3, genes, n, 64, eck.BF16, feat_out=feat, legal_out=legal)
        T.call("c3.score", lambda: eck.costmodel_score(me3, feat, n, e))
        eck.costmodel_score(ml3, feat, n, l)
        eck.topk_select(e, l, legal, 1, k, idx, eo, cnt, ws, alpha=cfg["alpha"])
        eck.candidates_gather(genes, n, idx.view(-1), k, parents)

    def c3():
        eck.candidate_enumerate(sp3, eck.MODE_SAMPLE, P, parents, seed=cfg["seed"])
        for r in range(cfg["rounds"]):
            T.call("c3.round", lambda: c3_round(r))

    ms = T.repeat("c3", c3, max(3, reps // 4), warm=1)
    assert int(cnt.item()) == k
    score_ms = T.median("c3.score")
    out["c3"] = {"workload": "8 rounds x (mutate 1024 -> 2^20 children of a batched GEMM, features, 2 x MLP 64-256-256-1 "
                             "bf16, top-1024, gather)",
                 "ms": ms, "ms_per_round": T.median("c3.round"), "candidates_per_s": cfg["rounds"] * n / (ms * 1e-3),
                 "score_ms": score_ms,
                 "score_frac_of_bf16_peak": n * flop / (score_ms * 1e-3) / PEAK_BF16_FLOPS}

    # ---- config 4: 100 Adam steps on 4096 measured pairs (minibatch 512), then 2^22 conv schedules rescored
    cfg = synth.CONFIGS["c4"]
    n_pairs, n = cfg["n_pairs"], cfg["rescore_n"]
    pg = torch.zeros((sp2.n_genes, n_pairs), dtype=torch.int16, device=dev)
    pf = torch.zeros((64, n_pairs), dtype=torch.bfloat16, device=dev)
    eck.candidate_enumerate(sp2, eck.MODE_SAMPLE, n_pairs, pg, seed=cfg["pair_seed"])
    eck.features_compute(sp2, pg, n_pairs, 64, eck.BF16, feat_out=pf)
    torch.cuda.synchronize()
    pe = upload(synth.measured_energy(pf.float().cpu().numpy(), cfg["label_seed"]))
    model = eck.Model(cfg["widths"], eck.BF16)
    theta0 = upload(synth.mlp_theta(cfg["widths"], cfg["weight_seeds"][0], bf16=True))
    ws_u = torch.empty(eck.costmodel_update_workspace_bytes(model, n_pairs, cfg["minibatch"]), dtype=torch.uint8, device=dev)
    snr, loss = torch.zeros(1, dtype=torch.float32, device=dev), torch.zeros(1, dtype=torch.float32, device=dev)
    genes = torch.zeros((sp2.n_genes, n), dtype=torch.int16, device=dev)
    feat4 = torch.zeros((64, n), dtype=torch.bfloat16, device=dev)
    e4 = torch.zeros(n, dtype=torch.float32, device=dev)
    eck.candidate_enumerate(sp2, eck.MODE_SAMPLE, n, genes, seed=2024)
    eck.features_compute(sp2, genes, n, 64, eck.BF16, feat_out=feat4)

    def c4_update():
        model.set_state(theta0)
        T.call("c4.update", lambda: eck.costmodel_update(model, pf, pe, cfg["n_steps"], cfg["minibatch"], snr, loss, ws_u,
                                                         lr=cfg["lr"]))

    T.repeat("c4", c4_update, max(3, reps // 4), warm=1)
    upd_ms = T.median("c4.update")
    assert bool(torch.isfinite(loss).all())
    rescore_ms = T.repeat("c4.rescore", lambda: eck.costmodel_score(model, feat4, n, e4), reps)
    # what a dependent launch costs on this stream: the median of back-to-back one-element fills
    one = torch.zeros(1, dtype=torch.float32, device=dev)

    def fills():
        for _ in range(100):
            one.zero_()

    floor_us = 10.0 * T.repeat("floor", fills, 10)
    out["c4"] = {"workload": "100 Adam steps (lr 1e-3, minibatch 512) on 4096 measured pairs, MLP 64-256-256-1 bf16 / fp32 "
                             "master; then 2^22 conv schedules rescored",
                 "update_ms": upd_ms, "update_ms_per_step": upd_ms / cfg["n_steps"], "empty_launch_floor_us": floor_us,
                 "rescore_ms": rescore_ms, "rescore_candidates_per_s": n / (rescore_ms * 1e-3),
                 "rescore_frac_of_bf16_peak": n * flop / (rescore_ms * 1e-3) / PEAK_BF16_FLOPS,
                 "final_loss": float(loss.item())}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--cpu-sample-log2", type=int, default=20)
    ap.add_argument("--only", choices=["enumerate", "features", "score", "score_min", "topk", "topk_two_pass", "topk_inf", "update", "treescore",
                                       "treeupdate", "search", "others"],
                    default=None,
                    help="profiling aid: after set-up run only this call of the step (prints a short JSON)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (candidates are independent and would shard by shape, with only "
              "the per-segment selection exchanging a few KB). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2411_18873_amd import eck, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    eck.lib()  # fails loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.only == "others":
        print(json.dumps({"only": "others", "other_configs": other_configs(torch, np, eck, synth, args.steps)}))
        return

    if args.only == "search":
        # Alg. 1 closed into a loop (config 3's operator, 2^20 children per round, M = 128, boosted-tree models,
        # simulated meter): rounds per second and candidates per second through the whole round
        from paper_2411_18873_amd.search import EnergySearch
        pop, rounds = 1 << 20, args.steps
        s = EnergySearch(synth.CONFIGS["c3"]["problem"], eck.SPACE_SPLIT,
                         lambda f, b: synth.simulated_kernel_metrics(f, 77, b), population=pop, M=128,
                         depth=6, init_rounds=40, update_rounds=8, mu=1000.0, max_rounds=rounds + args.warmup,
                         meter_seconds=1.0)
        s.initialise()
        for _ in range(args.warmup):
            s.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(rounds):
            s.step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        print(json.dumps({"only": "search", "ms_per_round": 1e3 * dt / rounds, "candidates_per_s": pop * rounds / dt,
                          "population": pop, "rounds": rounds, "measured": sum(h["measured"] for h in s.history),
                          "k": [round(h["k"], 2) for h in s.history],
                          # at one second per energy measurement: the meter's share with the k controller, and
                          # what measuring all M kernels of every round would have cost
                          "meter_s_at_1s_per_kernel": s.account()["meter_seconds"],
                          "meter_s_if_all_measured": s.account()["full_measurement_seconds"]}))
        return

    cfg = synth.CONFIGS["c5"]
    shapes, per = cfg["shapes"], cfg["n_per_shape"]
    S, F, K = len(shapes), cfg["n_feat"], cfg["k"]
    N = S * per
    widths = cfg["widths"]
    spaces = [eck.Space(synth.gemm(m, n, k), eck.SPACE_SPLIT) for (m, n, k) in shapes]
    G = spaces[0].n_genes

    genes = torch.zeros((G, N), dtype=torch.int16, device=dev)
    feat = torch.zeros((F, N), dtype=torch.bfloat16, device=dev)
    legal = torch.zeros(N, dtype=torch.uint8, device=dev)
    energy = torch.zeros(N, dtype=torch.float32, device=dev)
    latency = torch.zeros(N, dtype=torch.float32, device=dev)
    idx = torch.zeros((S, K), dtype=torch.int32, device=dev)
    e_out = torch.zeros((S, K), dtype=torch.float32, device=dev)
    count = torch.zeros(S, dtype=torch.int32, device=dev)
    ws_topk = torch.empty(eck.topk_select_workspace_bytes(N, S, K), dtype=torch.uint8, device=dev)

    def upload(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    m_energy, m_latency = eck.Model(widths, eck.BF16), eck.Model(widths, eck.BF16)
    m_energy.set_state(upload(synth.mlp_theta(widths, cfg["weight_seeds"][0], bf16=True)))
    m_latency.set_state(upload(synth.mlp_theta(widths, cfg["weight_seeds"][1], bf16=True)))

    # measured buffer of the dynamic update: 32 candidates of every shape, synthetic energies (resident in HBM)
    upd_rows, upd_mb, upd_steps = 2048, 512, 4
    upd_genes = torch.zeros((G, upd_rows), dtype=torch.int16, device=dev)
    upd_feat = torch.zeros((F, upd_rows), dtype=torch.bfloat16, device=dev)
    eck.candidate_enumerate_batch(spaces, eck.MODE_SAMPLE, 32, upd_genes, [5000 + s for s in range(S)])
    eck.features_compute_batch(spaces, upd_genes, 32, F, eck.BF16, feat_out=upd_feat)
    torch.cuda.synchronize()
    upd_energy = upload(synth.measured_energy(upd_feat.float().cpu().numpy(), 13))
    ws_upd = torch.empty(eck.costmodel_update_workspace_bytes(m_energy, upd_rows, upd_mb), dtype=torch.uint8, device=dev)
    snr = torch.zeros(1, dtype=torch.float32, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)

    seeds = [cfg["seed_base"] + s for s in range(S)]
    T = Timer(torch)

    lat_min = torch.zeros(S, dtype=torch.int32, device=dev)  # least legal latency of every shape, as order keys

    def select(alpha):
        eck.topk_select(energy, latency, legal, S, K, idx, e_out, count, ws_topk, alpha=alpha)

    def select_known_min(alpha):
        eck.topk_select_known_min(energy, latency, legal, S, K, lat_min, idx, e_out, count, ws_topk, alpha=alpha)

    def step(i, timed):
        call = T.call if timed else (lambda name, fn: fn())
        call("enumerate", lambda: eck.candidate_enumerate_batch(spaces, eck.MODE_SAMPLE, per, genes, seeds, round=i))
        call("features", lambda: eck.features_compute_batch(spaces, genes, per, F, eck.BF16, feat_out=feat,
                                                            legal_out=legal))
        call("score", lambda: eck.costmodel_score(m_energy, feat, N, energy))
        # the latency pass also reduces what it writes to the least legal latency of every shape, so the selection
        # reads energy, latency and flag of a candidate exactly once
        call("score_min", lambda: eck.costmodel_score_min(m_latency, feat, N, latency, legal, S, lat_min))
        call("topk", lambda: select_known_min(cfg["alpha"]))
        call("update", lambda: eck.costmodel_update(m_energy, upd_feat, upd_energy, upd_steps, upd_mb, snr, loss, ws_upd,
                                                    lr=1e-3))

    if args.only:
        trees = None
        if args.only in ("treescore", "treeupdate"):
            # the paper's own model form on the same workload: 100 trees of depth 6, each refit call adds 4
            trees = eck.Trees(F, 6, 100 + 4 * (args.steps + args.warmup + 1), 0.5)
            ws_trees = torch.empty(eck.treemodel_update_workspace_bytes(trees, upd_rows), dtype=torch.uint8, device=dev)
            eck.treemodel_update(trees, upd_feat, upd_energy, 100, snr, loss, ws_trees)
        step(0, False)  # fills every buffer once
        torch.cuda.synchronize()

        def one(i):
            if args.only == "enumerate":
                eck.candidate_enumerate_batch(spaces, eck.MODE_SAMPLE, per, genes, seeds, round=i)
            elif args.only == "features":
                eck.features_compute_batch(spaces, genes, per, F, eck.BF16, feat_out=feat, legal_out=legal)
            elif args.only == "score":
                eck.costmodel_score(m_energy, feat, N, energy)
            elif args.only == "treescore":
                eck.treemodel_score(trees, feat, N, energy)
            elif args.only == "treeupdate":
                eck.treemodel_update(trees, upd_feat, upd_energy, 4, snr, loss, ws_trees)
            elif args.only == "score_min":
                eck.costmodel_score_min(m_latency, feat, N, latency, legal, S, lat_min)
            elif args.only == "topk":
                select_known_min(cfg["alpha"])
            elif args.only == "topk_two_pass":
                select(cfg["alpha"])
            elif args.only == "topk_inf":
                select(float("inf"))
            else:
                eck.costmodel_update(m_energy, upd_feat, upd_energy, upd_steps, upd_mb, snr, loss, ws_upd, lr=1e-3)

        for i in range(args.warmup):
            one(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            one(args.warmup + i)
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / args.steps
        print(json.dumps({"only": args.only, "ms_per_call": ms, "candidates": N, "steps": args.steps}))
        return

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record()
        step(args.warmup + i, True)
    marks[args.steps].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]
    ms_per_step = statistics.median(step_ms)
    feasible_alpha = int(count.sum().item())
    assert int(count.min().item()) > 0 and torch.isfinite(snr).all()

    score_ms = T.median("score")
    flop_per_cand = flop_per_candidate(widths)
    achieved = N * flop_per_cand / (score_ms * 1e-3)

    # the same selection without the latency gate's bite (alpha = inf: every legal candidate is feasible, every
    # segment has k of them, nothing ends early)
    topk_inf_ms = T.repeat("topk_inf", lambda: select(float("inf")), max(20, args.steps))
    assert int(count.min().item()) == K
    # and the selection that finds the least latencies itself (a pass over the latencies before the selection)
    topk_two_pass_ms = T.repeat("topk_two_pass", lambda: select(cfg["alpha"]), max(20, args.steps))
    assert int(count.sum().item()) == feasible_alpha

    result = {
        "metric": "candidate schedules scored+ranked/sec at 1 GPU; % MFMA / HBM peak",
        "value": N / (ms_per_step * 1e-3),
        "unit": "candidates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_mean_wall": 1e3 * elapsed / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "c5: 64 GEMM shapes x 2^18 sampled schedules = 2^24 candidates, 64 features, "
                               "2 x MLP 64-512-512-1 bf16, per-shape top-32 (alpha 1.1), 4-step refit on 2048 pairs",
                   "candidates": N, "segments": S, "k": K},
        "roofline": {"bound": "mfma", "kernel": "score_bf16_kernel<64,512,512>", "achieved": achieved / 1e12,
                     "peak": PEAK_BF16_FLOPS / 1e12, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_FLOPS,
                     "ms_per_launch": score_ms,
                     "traffic": TRAFFIC["score_bf16_kernel<64,512,512>"] if (F, N) == (64, 1 << 24) else None,
                     "traffic_unit": "bytes/launch", "traffic_source": TRAFFIC["file"]},
    }
    # the other calls of the step, each between HIP events: median milliseconds per call, and for the two calls that
    # only move data the algorithmic bytes per second against the 8 TB/s of HBM (features: genes in, 64 bf16 features
    # and a flag out; top-k: energy, latency and flag of every candidate once)
    calls_ms = {name: T.median(name) for name in ("enumerate", "features", "score", "score_min", "topk", "update")}
    calls_ms["topk_alpha_inf"] = topk_inf_ms
    calls_ms["topk_two_pass"] = topk_two_pass_ms
    result["calls_ms"] = calls_ms

    def hbm(nbytes, ms):
        return {"algorithmic_bytes": nbytes, "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                "frac": nbytes / (ms * 1e-3) / PEAK_HBM, "ms": ms}

    result["hbm"] = {"features": hbm(N * (2 * G + 2 * F + 1), calls_ms["features"]),
                     "topk": dict(hbm(N * 9, calls_ms["topk"]), input="alpha = 1.1, least latencies from the scoring "
                                  "launch: %d of %d slots filled" % (feasible_alpha, S * K)),
                     "topk_two_pass": dict(hbm(N * 13, topk_two_pass_ms), input="alpha = 1.1, least latencies found by "
                                           "the selection (latencies read twice)"),
                     "topk_alpha_inf": dict(hbm(N * 9, topk_inf_ms), input="alpha = inf: every segment selects k")}
    if not args.no_other_configs:
        result["other_configs"] = other_configs(torch, np, eck, synth, max(8, args.steps))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, args.cpu_sample_log2)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
