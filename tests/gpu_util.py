"""numpy-in / numpy-out wrappers over the HIP path for the GPU parity tests.
Every call goes through the C ABI via paper_2411_18873_amd.eck."""
import numpy as np
import torch

from paper_2411_18873_amd import eck


def to_dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).cuda()
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).cuda()
    return torch.from_numpy(a).cuda()


def bf16_dev(bits_u16):
    return to_dev(np.ascontiguousarray(bits_u16, dtype=np.uint16)).view(torch.bfloat16)


def enumerate_gpu(space, mode, n, seed=0, rnd=0, first_index=0, parents=None, p_mut_q32=0, ld=None):
    ld = n + (n & 1) if ld is None else ld
    genes = torch.full((space.n_genes, ld), -1, dtype=torch.int16, device="cuda")
    par = None if parents is None else to_dev(np.ascontiguousarray(parents, dtype=np.uint16))
    eck.candidate_enumerate(space, mode, n, genes, seed=seed, round=rnd, first_index=first_index, parents=par,
                            p_mut_q32=p_mut_q32)
    torch.cuda.synchronize()
    return genes.cpu().numpy().view(np.uint16)


def features_gpu(space, genes_u16, n, n_feat, out_dtype, want_raw=True):
    g = to_dev(np.ascontiguousarray(genes_u16, dtype=np.uint16))
    ld = g.shape[1]
    feat = torch.zeros((n_feat, ld), dtype=torch.float32 if out_dtype == eck.F32 else torch.bfloat16, device="cuda")
    raw = torch.zeros((n_feat, ld), dtype=torch.int64, device="cuda") if want_raw else None
    legal = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    eck.features_compute(space, g, n, n_feat, out_dtype, feat_out=feat, raw_out=raw, legal_out=legal)
    torch.cuda.synchronize()
    feat_np = feat.cpu().numpy() if out_dtype == eck.F32 else feat.view(torch.int16).cpu().numpy().view(np.uint16)
    return (raw.cpu().numpy().view(np.uint64) if want_raw else None), feat_np, legal.cpu().numpy()


def make_model(widths, dtype, theta):
    m = eck.Model(widths, dtype)
    m.set_state(to_dev(np.ascontiguousarray(theta, dtype=np.float32)))
    return m


def score_gpu(model, feat_dev, n):
    out = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    eck.costmodel_score(model, feat_dev, n, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def topk_gpu(energy, latency, legal, n_segments, k, mode=eck.SELECT_THRESHOLD, alpha=1.1, m_latency=0):
    e = to_dev(np.ascontiguousarray(energy, dtype=np.float32))
    lat = None if latency is None else to_dev(np.ascontiguousarray(latency, dtype=np.float32))
    lg = None if legal is None else to_dev(np.ascontiguousarray(legal, dtype=np.uint8))
    return topk_dev(e, lat, lg, n_segments, k, mode, alpha, m_latency)


def topk_dev(e, lat, lg, n_segments, k, mode=eck.SELECT_THRESHOLD, alpha=1.1, m_latency=0):
    idx = torch.zeros((n_segments, k), dtype=torch.int32, device="cuda")
    eo = torch.zeros((n_segments, k), dtype=torch.float32, device="cuda")
    cnt = torch.zeros((n_segments,), dtype=torch.int32, device="cuda")
    rank_gate = m_latency if (mode == eck.SELECT_RANK and lat is not None) else 0
    ws = torch.empty(eck.topk_select_workspace_bytes(e.numel(), n_segments, k, m_latency=rank_gate), dtype=torch.uint8,
                     device="cuda")
    eck.topk_select(e, lat, lg, n_segments, k, idx, eo, cnt, ws, mode=mode, alpha=alpha, m_latency=m_latency)
    torch.cuda.synchronize()
    return idx.cpu().numpy().view(np.uint32), eo.cpu().numpy(), cnt.cpu().numpy().view(np.uint32)


def update_gpu(model, feat_dev, energy, n_steps, minibatch, **kw):
    e = to_dev(np.ascontiguousarray(energy, dtype=np.float32))
    snr = torch.zeros(1, dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(eck.costmodel_update_workspace_bytes(model, e.numel(), minibatch), dtype=torch.uint8,
                     device="cuda")
    eck.costmodel_update(model, feat_dev, e, n_steps, minibatch, snr, loss, ws, **kw)
    torch.cuda.synchronize()
    return float(snr.item()), float(loss.item())


def within(got, want, magnitude, rtol):
    """Worst |g - o| / (rtol * M) over the candidates, M = the oracle's magnitude of the output sum
    (|b| + sum |w_j| h_j).  <= 1 means every candidate is inside the relative tolerance."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.max(np.abs(got - want) / (rtol * np.asarray(magnitude, dtype=np.float64))))


def check_bf16_scores(widths, theta, feat_bits_u16, got, label=""):
    """The gates of a bf16 model's scores against the fp64 oracle on the same bf16 feature bits
    (M = |b3| + sum |w3_j| h2_j, the magnitude of the output sum):
      1. |g - o| <= 1e-2 * M for every candidate, o = the exact forward pass;
      2. against o_b, the oracle mode that rounds the first hidden layer to bf16 where the kernel does:
         |g - o_b| <= 1e-4 * M for all but a few candidates and <= 1e-3 * M for every candidate.
    The few: the kernel rounds an fp32 sum to bf16, the oracle an fp64 sum; about 3 in 10^6 activations fall so
    close to a rounding boundary that the two round differently, and one such activation moves the output by up to
    ~3e-4 * M (tests/test_oracle_score.py measures both figures on the CPU).  At most 1 + 5e-4 * n candidates may
    exceed 1e-4 * M; everything else differs by fp32 summation order only (~1e-7 * M).
    Prints the margins and the worst error relative to max(|o|, rms(o))."""
    import oracle
    x = oracle.bf16_bits_to_f32(feat_bits_u16)
    want = oracle.score(widths, theta, x)
    emu = oracle.score(widths, theta, x, emulate_bf16=True)
    mag = oracle.score_magnitude(widths, theta, x)
    got = np.asarray(got, dtype=np.float64)
    assert np.isfinite(got).all()
    worst = within(got, want, mag, 1e-2)
    err_emu = np.abs(got - emu) / mag
    worst_emu = float(err_emu.max())
    flipped = int((err_emu > 1e-4).sum())
    typical = float(np.median(err_emu))
    rms = float(np.sqrt(np.mean(want * want)))
    rel = float(np.max(np.abs(got - want) / np.maximum(np.abs(want), rms)))
    print("bf16 scores %s n=%d: worst |g-o| = %.3f x 1e-2 M; vs bf16-activation oracle: median %.1e M, worst %.1e M, "
          "%d candidates beyond 1e-4 M (allowed %d); worst |g-o|/max(|o|, rms) = %.2e"
          % (label, got.size, worst, typical, worst_emu, flipped, 1 + int(5e-4 * got.size), rel), flush=True)
    assert worst <= 1.0, worst
    assert flipped <= 1 + int(5e-4 * got.size), flipped
    assert worst_emu <= 1e-3, worst_emu
    return worst, worst_emu, rel
