"""Alg. 1 as a closed loop, on the CPU with the oracle's primitives -- TEST INFRASTRUCTURE ONLY.

Sec. 6.4: a first training set from the initial random sample; then per round GeneticReproduction (mutation),
LatencyEvaAndPick (the M kernels the latency model rates fastest), EnergyModelEvaAndPick (the round(k M) of
them of lowest predicted energy), measurement, the signal-to-noise ratio of prediction against measurement,
ModelUpdate, the k rule, and the measured kernels of lowest energy as the next parents.  Both models are
boosted trees (Sec. 5.4); readings as in the library's closed loop: the energy model is refitted on everything
measured so far, the batch that yields the ratio is led by the kernel of largest energy so far (one normaliser),
the latency model is fitted once on the initial sample, k never drops below k_min.
"""
import numpy as np

import oracle


def run(problem, kind, measure, rounds, population=1 << 14, M=64, n_parents=64, depth=6, init_rounds=40,
        update_rounds=8, mu=20.0, k_min=0.2, eta=0.3, lam=1.0, p_mut_q32=429496729, seed=1, crossover=False,
        dedup=False):
    sp = oracle.Space(problem, kind)
    N, P = population, n_parents
    nodes, leaves = (1 << depth) - 1, 1 << depth
    cap = init_rounds + update_rounds * (rounds + 1)
    e_nf, e_nt, e_lf = (np.zeros((cap, nodes), np.uint8), np.zeros((cap, nodes), np.float32),
                        np.zeros((cap, leaves), np.float32))
    l_nf, l_nt, l_lf = (np.zeros((init_rounds, nodes), np.uint8), np.zeros((init_rounds, nodes), np.float32),
                        np.zeros((init_rounds, leaves), np.float32))
    n_e = 0
    history = []

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

    def parents_of():
        order = np.argsort(m_energy, kind="stable")[:P]
        return np.ascontiguousarray(m_genes[:, order[np.arange(P) % len(order)]])

    parents = parents_of()
    k = 1.0
    history.append(dict(round=0, measured=len(first), k=k, snr=float("nan"), best=float(m_energy.min())))
    for r in range(1, rounds + 1):
        genes = oracle.enumerate_candidates(sp, oracle.MODE_CROSSOVER if crossover else oracle.MODE_MUTATE, N,
                                            seed=seed, rnd=r, parents=parents, p_mut_q32=p_mut_q32)
        _, f32, b16, legal = oracle.features(sp, genes, 64)
        if dedup:
            legal = legal & oracle.dedup(genes)
        x = oracle.bf16_bits_to_f32(b16)
        l_pred = oracle.trees_predict(64, depth, l_nf, l_nt, l_lf, 0.5, x, fp32_sequential=True).astype(np.float32)
        e_pred = oracle.trees_predict(64, depth, e_nf[:n_e], e_nt[:n_e], e_lf[:n_e], 0.5, x,
                                      fp32_sequential=True).astype(np.float32)
        want = max(1, int(np.floor(k * M + 0.5)))
        idx, _, cnt = oracle.topk(e_pred, l_pred, legal, 1, want, mode=oracle.SEL_RANK, m_latency=M)
        picked = idx[0, :cnt[0]]
        energy, _ = measure(f32[:, picked], r)
        ref = int(np.argmax(m_energy))
        batch_x = np.concatenate([m_feat[:, ref:ref + 1], x[:, picked]], axis=1)
        batch_e = np.concatenate([m_energy[ref:ref + 1], energy.astype(np.float32)])
        snr, _ = oracle.trees_boost(64, depth, e_nf, e_nt, e_lf, n_e, 0, 0.5, batch_x, batch_e, eta=eta, lam=lam)
        m_genes = np.concatenate([m_genes, genes[:, picked]], axis=1)
        m_feat = np.concatenate([m_feat, x[:, picked]], axis=1)
        m_energy = np.concatenate([m_energy, energy.astype(np.float32)])
        oracle.trees_boost(64, depth, e_nf, e_nt, e_lf, n_e, update_rounds, 0.5, m_feat, m_energy, eta=eta, lam=lam)
        n_e += update_rounds
        k = max(k_min, oracle.k_step(k, float(np.float32(snr)), mu, M))
        parents = parents_of()
        history.append(dict(round=r, measured=int(cnt[0]), k=k, snr=snr, best=float(m_energy.min()),
                            picked=picked.copy()))
    return history, (e_nf[:n_e], e_nt[:n_e], e_lf[:n_e]), m_energy
