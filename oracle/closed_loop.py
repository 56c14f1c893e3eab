"""Alg. 1 as a closed loop, on the CPU with the oracle's primitives -- TEST INFRASTRUCTURE ONLY.

Sec. 6.4 and Alg. 1, statement by statement.  First training set: random kernels, M of them measured, both
models fitted.  Then per round:

    Kernel_generation <- GeneticReproduction(Kernel_parents)            mutation (optionally crossover first)
    Kernel_M          <- LatencyEvaAndPick(Kernel_generation, M)        the M launchable kernels the latency
                                                                        model rates fastest
    Kernel_kM, EnergyPredicted_kM <- EnergyModelEvaAndPick(Kernel_M, EnergyModel, k*M)
                                                                        the round(k M) of them of least
                                                                        predicted energy
    EnergyMeasured_kM <- measurement                                    the callback
    EnergyModel       <- ModelUpdate(EnergyModel, EnergyMeasured_kM)
    PredictionError   <- SNR(EnergyPredicted_kM, EnergyMeasured_kM)     of the predictions made BEFORE the update
    k                 <- Min(1, k + 0.2) if PredictionError < mu else Max(0, k - 0.2)
    Kernel_parents    <- EnergyModelEvaAndPick(Kernel_M, EnergyModel, 0.5*M)
                                                                        Kernel_M re-rated by the UPDATED model,
                                                                        its better half reproduces

Where Alg. 1 leaves a choice open (all listed with the other readings in the design notes):
  * round(k M) = 0 measures nothing: no ratio exists, the model is not updated and k stays where it is;
  * ModelUpdate boosts `update_rounds` further trees on everything measured so far;
  * the ratio is that of the new batch alone, led by the kernel of largest energy measured so far so that its
    labels share the normaliser of the whole record;
  * the latency model is fitted once, on the first training set (the paper takes it from its host framework);
  * the first parents are the better half, by the freshly fitted energy model, of the first training set;
  * a short pick (fewer launchable kernels than asked for) is filled up with its first kernel.
Two departures from the printed algorithm exist as named options and are off by default:
  * parents="measured": the n_parents measured kernels of least MEASURED energy over the whole record reproduce;
  * k_min > 0: k never falls below k_min, so the model never stops being checked against the meter.
"""
import numpy as np

import oracle


def run(problem, kind, measure, rounds, population=1 << 14, M=64, n_parents=None, depth=6, init_rounds=40,
        update_rounds=8, mu=20.0, k_min=0.0, eta=0.3, lam=1.0, p_mut_q32=429496729, seed=1, crossover=False,
        dedup=False, parents="model", trace=False):
    assert parents in ("model", "measured")
    sp = oracle.Space(problem, kind)
    N = population
    P = M // 2 if parents == "model" else int(n_parents)       # 0.5 * M (Alg. 1, last statement)
    nodes, leaves = (1 << depth) - 1, 1 << depth
    cap = init_rounds + update_rounds * (rounds + 1)
    e_nf, e_nt, e_lf = (np.zeros((cap, nodes), np.uint8), np.zeros((cap, nodes), np.float32),
                        np.zeros((cap, leaves), np.float32))
    l_nf, l_nt, l_lf = (np.zeros((init_rounds, nodes), np.uint8), np.zeros((init_rounds, nodes), np.float32),
                        np.zeros((init_rounds, leaves), np.float32))
    history = []

    def energy_predictions(x, n_trees):
        return oracle.trees_predict(64, depth, e_nf[:n_trees], e_nt[:n_trees], e_lf[:n_trees], 0.5, x,
                                    fp32_sequential=True).astype(np.float32)

    def filled(cols):
        """a pick of fewer than P kernels is filled up with its first kernel"""
        cols = np.asarray(cols, dtype=np.int64)
        return np.concatenate([cols, np.full(P - len(cols), cols[0], dtype=np.int64)])

    def measured_parents():
        order = np.argsort(m_energy, kind="stable")[:P]
        return np.ascontiguousarray(m_genes[:, order[np.arange(P) % len(order)]])

    # ---- the first training set (Sec. 6.4)
    genes = oracle.enumerate_candidates(sp, oracle.MODE_SAMPLE, N, seed=seed, rnd=0)
    _, f32, b16, legal = oracle.features(sp, genes, 64)
    first = np.flatnonzero(legal)[:M]
    m_genes = genes[:, first]
    energy, latency = measure(f32[:, first], 0)
    m_feat = oracle.bf16_bits_to_f32(b16[:, first])     # the models see bf16 features
    m_energy = energy.astype(np.float32)
    oracle.trees_boost(64, depth, l_nf, l_nt, l_lf, 0, init_rounds, 0.5, m_feat, latency, eta=eta, lam=lam)
    oracle.trees_boost(64, depth, e_nf, e_nt, e_lf, 0, init_rounds, 0.5, m_feat, m_energy, eta=eta, lam=lam)
    n_e = init_rounds
    if parents == "model":
        pidx, _, pcnt = oracle.topk(energy_predictions(m_feat, n_e), None, None, 1, min(P, len(first)))
        par = np.ascontiguousarray(m_genes[:, filled(pidx[0, :pcnt[0]])])
    else:
        par = measured_parents()
    k = 1.0
    history.append(dict(round=0, measured=len(first), k=k, snr=float("nan"), best=float(m_energy.min())))

    for r in range(1, rounds + 1):
        genes = oracle.enumerate_candidates(sp, oracle.MODE_CROSSOVER if crossover else oracle.MODE_MUTATE, N,
                                            seed=seed, rnd=r, parents=par, p_mut_q32=p_mut_q32)
        _, f32, b16, legal = oracle.features(sp, genes, 64)
        if dedup:
            legal = legal & oracle.dedup(genes)
        x = oracle.bf16_bits_to_f32(b16)
        l_pred = oracle.trees_predict(64, depth, l_nf, l_nt, l_lf, 0.5, x, fp32_sequential=True).astype(np.float32)
        e_pred = energy_predictions(x, n_e)
        want = int(np.floor(k * M + 0.5))
        snr = float("nan")
        picked = np.zeros(0, dtype=np.uint32)
        if want >= 1:
            # Kernel_M by latency, then the `want` of least predicted energy inside it
            idx, _, cnt = oracle.topk(e_pred, l_pred, legal, 1, want, mode=oracle.SEL_RANK, m_latency=M)
            picked = idx[0, :cnt[0]].copy()
            energy, _ = measure(f32[:, picked], r)
            ref = int(np.argmax(m_energy))
            batch_x = np.concatenate([m_feat[:, ref:ref + 1], x[:, picked]], axis=1)
            batch_e = np.concatenate([m_energy[ref:ref + 1], energy.astype(np.float32)])
            # zero boosting rounds: only the ratio of the model as it stands
            snr, _ = oracle.trees_boost(64, depth, e_nf, e_nt, e_lf, n_e, 0, 0.5, batch_x, batch_e, eta=eta, lam=lam)
            m_genes = np.concatenate([m_genes, genes[:, picked]], axis=1)
            m_feat = np.concatenate([m_feat, x[:, picked]], axis=1)
            m_energy = np.concatenate([m_energy, energy.astype(np.float32)])
            oracle.trees_boost(64, depth, e_nf, e_nt, e_lf, n_e, update_rounds, 0.5, m_feat, m_energy, eta=eta,
                               lam=lam)
            n_e += update_rounds
            k = max(k_min, oracle.k_step(k, float(np.float32(snr)), mu, M))
        entry = dict(round=r, measured=len(picked), k=k, snr=snr, best=float(m_energy.min()), picked=picked)
        if parents == "model":
            e_new = energy_predictions(x, n_e)
            pidx, _, pcnt = oracle.topk(e_new, l_pred, legal, 1, P, mode=oracle.SEL_RANK, m_latency=M)
            cols = filled(pidx[0, :pcnt[0]])
            par = np.ascontiguousarray(genes[:, cols])
            entry["parents"] = cols.astype(np.uint32)
            if trace:
                entry.update(latency_predicted=l_pred, energy_updated=e_new, legal=legal.copy())
        else:
            par = measured_parents()
        history.append(entry)
    return history, (e_nf[:n_e], e_nt[:n_e], e_lf[:n_e]), m_energy
