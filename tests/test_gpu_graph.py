"""GPU: the calls of a search step recorded into a HIP graph and replayed.  Config 1 (6400 schedules, six dependent
launches) is bound by launch latency, which is what a graph is for; the library's calls allocate nothing, clear their
workspaces with kernels and take the stream they are given, so they can be captured.  Every replay must reproduce the
eager result bit for bit, with eager work and synchronisations between the replays and with new inputs in the captured
buffers."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_18873_amd import eck, synth

pytestmark = pytest.mark.gpu


def test_config1_chain_as_a_graph_reproduces_the_eager_results():
    import gpu_util as G
    cfg = synth.CONFIGS["c1"]
    n, k = cfg["n"], cfg["k"]
    sp = eck.Space(cfg["problem"], eck.SPACE_KNOB)
    genes = torch.zeros((sp.n_genes, n), dtype=torch.int16, device="cuda")
    feat = torch.zeros((32, n), dtype=torch.float32, device="cuda")
    legal = torch.zeros(n, dtype=torch.uint8, device="cuda")
    e = torch.zeros(n, dtype=torch.float32, device="cuda")
    l = torch.zeros(n, dtype=torch.float32, device="cuda")
    idx = torch.zeros((1, k), dtype=torch.int32, device="cuda")
    eo = torch.zeros((1, k), dtype=torch.float32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(eck.topk_select_workspace_bytes(n, 1, k), dtype=torch.uint8, device="cuda")
    thetas = [synth.mlp_theta(cfg["widths"], s) for s in cfg["weight_seeds"]]
    me, ml = (G.make_model(cfg["widths"], eck.F32, t) for t in thetas)

    def chain():
        eck.candidate_enumerate(sp, eck.MODE_EXHAUSTIVE, n, genes)
        eck.features_compute(sp, genes, n, 32, eck.F32, feat_out=feat, legal_out=legal)
        eck.costmodel_score(me, feat, n, e)
        eck.costmodel_score(ml, feat, n, l)
        eck.topk_select(e, l, legal, 1, k, idx, eo, cnt, ws, alpha=cfg["alpha"])

    def results():
        torch.cuda.synchronize()
        return idx.cpu().numpy().copy(), eo.cpu().numpy().copy(), cnt.cpu().numpy().copy()

    sp.upload()                                          # the one call of the chain's set-up that allocates and copies
    chain()                                              # eager: the reference
    want = results()
    io, eo_o, co = oracle.topk(e.cpu().numpy(), l.cpu().numpy(), legal.cpu().numpy(), 1, k, alpha=cfg["alpha"])
    assert np.array_equal(want[0].view(np.uint32), io) and np.array_equal(want[2].view(np.uint32), co)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    for replay in range(4):
        # eager work between the replays that overwrites every buffer the graph writes
        for t in (genes, feat, legal, e, l, idx, eo, cnt):
            t.fill_(1)
        torch.cuda.synchronize()
        graph.replay()
        got = results()
        for g, w in zip(got, want):
            assert np.array_equal(g.view(np.uint32) if g.dtype != np.int16 else g, w.view(np.uint32) if w.dtype != np.int16 else w), replay
    # a model refitted between replays: the graph holds the model's buffers, not their contents
    me.set_state(G.to_dev(np.ascontiguousarray(thetas[1], dtype=np.float32)))
    chain()
    changed = results()
    graph.replay()
    got = results()
    assert all(np.array_equal(a.view(np.uint32), b.view(np.uint32)) for a, b in zip(got, changed))
    assert not np.array_equal(changed[0], want[0])
