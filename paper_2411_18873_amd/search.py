"""The search round of Alg. 1, closed into a loop on one GPU (Sec. 6.4): reproduce a generation from the
parents, keep the M kernels the latency model rates fastest, measure the round(k * M) of them the energy
model rates lowest, compare prediction with measurement (a signal-to-noise ratio), update the energy model,
move k by 0.2 up or down, and let the better half of the M fastest kernels -- rated by the updated energy
model -- be the next parents (Alg. 1, last statement).

Every per-candidate step and every decision runs in the library through the C ABI (candidate_enumerate,
features_compute, treemodel_score, topk_select in RANK mode, eck_candidates_gather, treemodel_update,
eck_k_count, eck_k_step).  What stays on the host is what the paper does on the host too: the measurement itself
(a callback; the power meter is outside this repository) and the record of a few hundred measured kernels.

Both cost models are boosted trees, the paper's model form (Sec. 5.4).  The energy model is refitted every round
on all kernels measured so far, labels normalised by the largest energy measured so far; the latency model
is fitted once on the initial sample (the paper takes it from its host framework) and then left alone.  A round
whose round(k * M) is 0 measures nothing, leaves the model and k alone and still picks parents.

Options that depart from the printed algorithm (off by default): parents="measured" lets the n_parents measured
kernels of least measured energy over the whole record reproduce; k_min > 0 keeps k from falling below it."""
import numpy as np
import torch

from . import eck


class EnergySearch:
    def __init__(self, problem, kind, measure, population=1 << 14, M=64, n_parents=None, depth=6, init_rounds=40,
                 update_rounds=8, mu=20.0, k_min=0.0, eta=0.3, lam=1.0, p_mut_q32=429496729, seed=1,
                 max_rounds=64, crossover=False, dedup=False, meter_seconds=0.0, parents="model"):
        assert parents in ("model", "measured")
        self.space = eck.Space(problem, kind)
        self.measure, self.N, self.M = measure, int(population), int(M)
        self.parent_rule = parents
        self.P = eck.k_count(0.5, self.M) if parents == "model" else int(n_parents)   # Alg. 1: 0.5 * M
        self.init_rounds, self.update_rounds = int(init_rounds), int(update_rounds)
        self.mu, self.k_min, self.eta, self.lam = float(mu), float(k_min), float(eta), float(lam)
        self.p_mut, self.seed = int(p_mut_q32), int(seed)
        self.crossover, self.dedup = bool(crossover), bool(dedup)
        # what one measurement costs on the real meter (Sec. 6.4: energy measurement is what dominates the search
        # time); only book-kept here, so that a run can say how long its measurements would have taken
        self.meter_seconds = float(meter_seconds)
        G, N, dev = self.space.n_genes, self.N, "cuda"
        cap_trees = init_rounds + update_rounds * (max_rounds + 1)
        self.energy_model = eck.Trees(64, depth, cap_trees, 0.5)
        self.latency_model = eck.Trees(64, depth, init_rounds, 0.5)
        self.genes = torch.zeros((G, N), dtype=torch.int16, device=dev)
        self.feat = torch.zeros((64, N), dtype=torch.bfloat16, device=dev)
        self.legal = torch.zeros(N, dtype=torch.uint8, device=dev)
        self.e_pred = torch.zeros(N, dtype=torch.float32, device=dev)
        self.l_pred = torch.zeros(N, dtype=torch.float32, device=dev)
        self.idx = torch.zeros((1, self.M), dtype=torch.int32, device=dev)
        self.e_sel = torch.zeros((1, self.M), dtype=torch.float32, device=dev)
        self.count = torch.zeros(1, dtype=torch.int32, device=dev)
        self.ws_topk = torch.empty(eck.topk_select_workspace_bytes(N, 1, self.M, m_latency=self.M), dtype=torch.uint8,
                                   device=dev)
        self.ws_dedup = torch.empty(eck.candidates_dedup_workspace_bytes(N), dtype=torch.uint8, device=dev) if dedup else None
        # everything measured so far: genes and features side by side, energies, in order of measurement
        self.cap = self.M * (max_rounds + 2)
        self.buf_genes = torch.zeros((G, self.cap), dtype=torch.int16, device=dev)
        self.buf_feat = torch.zeros((64, self.cap), dtype=torch.bfloat16, device=dev)
        self.buf_energy = torch.zeros(self.cap, dtype=torch.float32, device=dev)
        self.n_buf = 0
        pad = self.M + 2 + (self.M & 1)  # one more than a batch, even (the feature kernels want an even row stride)
        self.new_genes = torch.zeros((G, pad), dtype=torch.int16, device=dev)
        self.new_feat = torch.zeros((64, pad), dtype=torch.bfloat16, device=dev)
        self.new_feat32 = torch.zeros((64, pad), dtype=torch.float32, device=dev)
        self.snr = torch.zeros(1, dtype=torch.float32, device=dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.ws_upd = torch.empty(eck.treemodel_update_workspace_bytes(self.energy_model, self.cap), dtype=torch.uint8,
                                  device=dev)
        self.parents = torch.zeros((G, self.P), dtype=torch.int16, device=dev)
        self.par_idx = torch.zeros((1, self.P), dtype=torch.int32, device=dev)
        self.par_val = torch.zeros((1, self.P), dtype=torch.float32, device=dev)
        self.par_count = torch.zeros(1, dtype=torch.int32, device=dev)
        self.new_pred = torch.zeros(pad, dtype=torch.float32, device=dev)
        self.ws_par = torch.empty(max(eck.topk_select_workspace_bytes(N, 1, self.P, m_latency=self.M),
                                      eck.topk_select_workspace_bytes(self.M, 1, min(self.P, self.M))),
                                  dtype=torch.uint8, device=dev)
        # host-side record of the measured kernels (a few hundred rows)
        self.h_genes = np.zeros((G, 0), dtype=np.uint16)
        self.h_energy = np.zeros(0, dtype=np.float32)
        self.k, self.round, self.history = 1.0, 0, []

    # ---- helpers -------------------------------------------------------------------------------------------
    def _measure_columns(self, genes_dev, m, batch):
        """features of m gathered kernels (fp32 for the meter, bf16 for the models), then the callback"""
        eck.features_compute(self.space, genes_dev, m, 64, eck.F32, feat_out=self.new_feat32)
        eck.features_compute(self.space, genes_dev, m, 64, eck.BF16, feat_out=self.new_feat)
        torch.cuda.synchronize()
        energy, latency = self.measure(self.new_feat32[:, :m].cpu().numpy(), batch)
        return np.ascontiguousarray(energy, dtype=np.float32), np.ascontiguousarray(latency, dtype=np.float32)

    def _append(self, m, energy):
        a, b = self.n_buf, self.n_buf + m
        assert b <= self.cap, "measurement buffer full"
        self.buf_genes[:, a:b] = self.new_genes[:, :m]
        self.buf_feat[:, a:b] = self.new_feat[:, :m]
        self.buf_energy[a:b] = torch.from_numpy(energy).cuda()
        self.n_buf = b
        self.h_genes = np.concatenate([self.h_genes, self.new_genes[:, :m].cpu().numpy().view(np.uint16)], axis=1)
        self.h_energy = np.concatenate([self.h_energy, energy])

    def _parents_from_the_record(self):
        """option parents="measured": the P measured kernels of lowest energy (ties to the earlier measurement),
        repeated if fewer exist"""
        order = np.argsort(self.h_energy, kind="stable")[:self.P]
        cols = order[np.arange(self.P) % len(order)]
        self.parents.copy_(torch.from_numpy(np.ascontiguousarray(self.h_genes[:, cols]).view(np.int16)).cuda())

    def _parents_from_the_generation(self):
        """Alg. 1, last statement: the M fastest kernels of this generation, rated again by the energy model as
        it is now; the 0.5 * M of least predicted energy reproduce (a short pick is filled with its first kernel
        by the gather call)"""
        eck.treemodel_score(self.energy_model, self.feat, self.N, self.e_pred)
        eck.topk_select(self.e_pred, self.l_pred, self.legal, 1, self.P, self.par_idx, self.par_val, self.par_count,
                        self.ws_par, mode=eck.SELECT_RANK, m_latency=self.M)
        eck.candidates_gather(self.genes, self.N, self.par_idx.view(-1), self.P, self.parents)

    def _first_parents(self, m):
        """the better half, by the freshly fitted energy model, of the first training set"""
        eck.treemodel_score(self.energy_model, self.new_feat, m, self.new_pred)
        eck.topk_select(self.new_pred[:m], None, None, 1, min(self.P, m), self.par_idx, self.par_val, self.par_count,
                        self.ws_par)
        eck.candidates_gather(self.new_genes, m, self.par_idx.view(-1), self.P, self.parents)

    def _fit(self, model, feat, energy_dev, n, rounds):
        eck.treemodel_update(model, feat, energy_dev[:n], rounds, self.snr, self.loss, self.ws_upd, eta=self.eta,
                             lam=self.lam)

    # ---- Sec. 6.4, first paragraph: the first training set -----------------------------------------------
    def initialise(self):
        eck.candidate_enumerate(self.space, eck.MODE_SAMPLE, self.N, self.genes, seed=self.seed, round=0)
        eck.features_compute(self.space, self.genes, self.N, 64, eck.BF16, feat_out=self.feat, legal_out=self.legal)
        torch.cuda.synchronize()
        first = np.flatnonzero(self.legal.cpu().numpy())[:self.M]   # sampled kernels are in random order already
        m = len(first)
        assert m >= 2, "no launchable kernel in the initial sample"
        idx = torch.from_numpy(first.astype(np.int32)).cuda()
        eck.candidates_gather(self.genes, self.N, idx, m, self.new_genes)
        energy, latency = self._measure_columns(self.new_genes, m, 0)
        self._append(m, energy)
        lat_dev = torch.from_numpy(latency).cuda()
        self._fit(self.latency_model, self.buf_feat, lat_dev, m, self.init_rounds)
        self._fit(self.energy_model, self.buf_feat, self.buf_energy, m, self.init_rounds)
        if self.parent_rule == "model":
            self._first_parents(m)
        else:
            self._parents_from_the_record()
        self.history.append(dict(round=0, measured=m, k=self.k, snr=float("nan"), best=float(self.h_energy.min())))

    # ---- one round of Alg. 1 ---------------------------------------------------------------------------------
    def step(self):
        self.round += 1
        r = self.round
        eck.candidate_enumerate(self.space, eck.MODE_CROSSOVER if self.crossover else eck.MODE_MUTATE, self.N,
                                self.genes, seed=self.seed, round=r, parents=self.parents, p_mut_q32=self.p_mut)
        eck.features_compute(self.space, self.genes, self.N, 64, eck.BF16, feat_out=self.feat, legal_out=self.legal)
        if self.dedup:  # repeated children leave the selection (their first occurrence stays)
            eck.candidates_dedup(self.genes, self.N, self.legal, ws=self.ws_dedup)
        eck.treemodel_score(self.latency_model, self.feat, self.N, self.l_pred)
        eck.treemodel_score(self.energy_model, self.feat, self.N, self.e_pred)
        want = eck.k_count(self.k, self.M)
        m, snr, picked = 0, float("nan"), np.zeros(0, dtype=np.uint32)
        if want >= 1:
            eck.topk_select(self.e_pred, self.l_pred, self.legal, 1, want, self.idx, self.e_sel, self.count,
                            self.ws_topk, mode=eck.SELECT_RANK, m_latency=self.M)
            torch.cuda.synchronize()
            m = int(self.count.item())
            picked = self.idx.view(-1)[:m].cpu().numpy().astype(np.uint32)
            # the kernel of largest energy so far leads the new batch, so its labels share the buffer's normaliser
            ref = int(np.argmax(self.h_energy))
            eck.candidates_gather(self.genes, self.N, self.idx.view(-1), m, self.new_genes)
            energy, _ = self._measure_columns(self.new_genes, m, r)
            batch_f = torch.cat([self.buf_feat[:, ref:ref + 1], self.new_feat[:, :m]], dim=1).contiguous()
            batch_e = torch.cat([self.buf_energy[ref:ref + 1], torch.from_numpy(energy).cuda()]).contiguous()
            self._fit(self.energy_model, batch_f, batch_e, m + 1, 0)          # prediction against measurement
            torch.cuda.synchronize()
            snr = float(self.snr.item())
            self._append(m, energy)
            self._fit(self.energy_model, self.buf_feat, self.buf_energy, self.n_buf, self.update_rounds)
            self.k = max(self.k_min, eck.k_step(self.k, snr, self.mu, self.M))
        entry = dict(round=r, measured=m, k=self.k, snr=snr, best=float(self.h_energy.min()), picked=picked)
        if self.parent_rule == "model":
            self._parents_from_the_generation()
            torch.cuda.synchronize()
            n_par = int(self.par_count.item())
            cols = self.par_idx.view(-1)[:n_par].cpu().numpy().astype(np.uint32)
            entry["parents"] = np.concatenate([cols, np.full(self.P - n_par, cols[0], dtype=np.uint32)])
        else:
            self._parents_from_the_record()
        self.history.append(entry)
        return self.history[-1]

    def account(self):
        """Totals of the run so far: kernels measured, and the time the meter would have needed for them."""
        measured = sum(h["measured"] for h in self.history)
        return dict(rounds=self.round, measured=measured, meter_seconds=measured * self.meter_seconds,
                    full_measurement_seconds=(self.M * (self.round + 1)) * self.meter_seconds)
