#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

Workload ("c5", the whole-network sweep): 64 GEMM shapes x 2^18 seeded schedule
samples = 2^24 candidates, 64 bf16 features, energy and latency models
64-512-512-1 (bf16 on the matrix cores), per-shape top-32 under the
latency-then-energy objective.  One step =

    candidate_enumerate (64 spaces) -> features_compute (64 spaces)
    -> costmodel_score (energy) -> costmodel_score (latency)
    -> topk_select (64 segments, k = 32, alpha = 1.1)
    -> costmodel_update (energy model, 2048 measured pairs resident in HBM, one epoch = 4 Adam steps)

Everything is resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_FLOPS = 2.5e15  # MI355X dense bf16 matrix peak


def cpu_baseline(cfg, sample_log2=18):
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-log2", type=int, default=18)
    ap.add_argument("--only", choices=["enumerate", "features", "score", "topk", "update", "copy", "treescore", "treeupdate", "search"],
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

    if args.only == "search":
        # Alg. 1 closed into a loop (config 3's operator, 2^20 children per round, M = 128, boosted-tree models,
        # simulated meter): rounds per second and candidates per second through the whole round
        from paper_2411_18873_amd.search import EnergySearch
        pop, rounds = 1 << 20, args.steps
        s = EnergySearch(synth.CONFIGS["c3"]["problem"], eck.SPACE_SPLIT,
                         lambda f, b: synth.simulated_kernel_metrics(f, 77, b), population=pop, M=128, n_parents=128,
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

    score_events = []

    seeds = [cfg["seed_base"] + s for s in range(S)]

    call_events = {name: [] for name in ("enumerate", "features", "topk", "update")}

    def timed_call(events, timed, fn):
        """fn() between two events on the stream the library launches on (torch's current stream)"""
        if not timed:
            return fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        events.append((a, b))

    def step(i, timed):
        timed_call(call_events["enumerate"], timed,
                   lambda: eck.candidate_enumerate_batch(spaces, eck.MODE_SAMPLE, per, genes, seeds, round=i))
        timed_call(call_events["features"], timed,
                   lambda: eck.features_compute_batch(spaces, genes, per, F, eck.BF16, feat_out=feat, legal_out=legal))
        for model, out in ((m_energy, energy), (m_latency, latency)):
            timed_call(score_events, timed, lambda: eck.costmodel_score(model, feat, N, out))
        timed_call(call_events["topk"], timed,
                   lambda: eck.topk_select(energy, latency, legal, S, K, idx, e_out, count, ws_topk, alpha=cfg["alpha"]))
        timed_call(call_events["update"], timed,
                   lambda: eck.costmodel_update(m_energy, upd_feat, upd_energy, upd_steps, upd_mb, snr, loss, ws_upd,
                                                lr=1e-3))

    if args.only:
        feat_copy = torch.empty_like(feat) if args.only == "copy" else None
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
            elif args.only == "copy":
                # plain device copy of known size (2^24 x 64 bf16 = 2 GiB read + 2 GiB written): calibrates
                # the FETCH_SIZE / WRITE_SIZE counters
                feat_copy.copy_(feat)
            elif args.only == "treescore":
                eck.treemodel_score(trees, feat, N, energy)
            elif args.only == "treeupdate":
                eck.treemodel_update(trees, upd_feat, upd_energy, 4, snr, loss, ws_trees)
            elif args.only == "topk":
                eck.topk_select(energy, latency, legal, S, K, idx, e_out, count, ws_topk, alpha=cfg["alpha"])
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
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps

    score_ms = sum(a.elapsed_time(b) for a, b in score_events) / len(score_events)
    flop_per_cand = 2 * sum(fi * fo for fi, fo in zip(widths[:-1], widths[1:]))
    achieved = N * flop_per_cand / (score_ms * 1e-3)
    assert int(count.min().item()) > 0 and torch.isfinite(snr).all()

    result = {
        "metric": "candidate schedules scored+ranked/sec at 1 GPU; % MFMA / HBM peak",
        "value": N / (ms_per_step * 1e-3),
        "unit": "candidates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
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
                     # HBM bytes per launch from FETCH_SIZE x 2.0 + WRITE_SIZE (rocprofv3 --pmc, calibrated with a
                     # plain copy; profiles/c5_hbm_traffic_pmc.txt); algorithmic: 2^24 x (128 B in + 4 B out)
                     "traffic": 2.155e9 + 0.0692e9 if (F, N) == (64, 1 << 24) else None,
                     "traffic_unit": "bytes/launch"},
    }
    # the other calls of the step, each between HIP events: milliseconds per call, and for the two calls that only
    # move data the algorithmic bytes per second against the 8 TB/s of HBM (features: genes in, 64 bf16 features and
    # a flag out; top-k: energy, latency and flag of every candidate once)
    calls_ms = {name: sum(a.elapsed_time(b) for a, b in ev) / len(ev) for name, ev in call_events.items()}
    calls_ms["score"] = score_ms
    hbm_bytes = {"features": N * (2 * G + 2 * F + 1), "topk": N * 9}
    result["calls_ms"] = calls_ms
    result["hbm"] = {name: {"algorithmic_bytes": b, "achieved": b / (calls_ms[name] * 1e-3) / 1e9, "peak": 8000.0,
                            "unit": "GB/s", "frac": b / (calls_ms[name] * 1e-3) / 8e12}
                     for name, b in hbm_bytes.items()}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, args.cpu_sample_log2)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
