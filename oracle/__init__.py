"""CPU oracle for the cost-model evaluation path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy access to ``eck_oracle.c`` (plain C, fp64, no blocking or
fusion).  Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` may import this package; the product package never does.
It imports nothing from the HIP path.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "eck_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

OP_GEMM, OP_BGEMM, OP_CONV2D = 0, 1, 2
SPACE_KNOB, SPACE_SPLIT, SPACE_SPLIT_XRED = 0, 1, 2
MODE_EXHAUSTIVE, MODE_SAMPLE, MODE_MUTATE, MODE_CROSSOVER = 0, 1, 2, 3
SEL_THRESHOLD, SEL_RANK = 0, 1


def build(force=False):
    """Compile the oracle with gcc (contraction off so fp32 steps round as written)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        L.orc_space_create.restype = C.c_void_p
        L.orc_space_create.argtypes = [C.c_void_p, C.c_int32]
        L.orc_space_destroy.argtypes = [C.c_void_p]
        L.orc_space_destroy.restype = None
        L.orc_hash.restype = C.c_uint64
        L.orc_hash.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32]
        L.orc_split_table.restype = C.c_uint32
        L.orc_split_table.argtypes = [C.c_uint32, C.c_void_p, C.c_uint32]
        L.orc_transform.restype = C.c_float
        L.orc_transform.argtypes = [C.c_uint64]
        L.orc_bf16_rne.restype = C.c_uint16
        L.orc_bf16_rne.argtypes = [C.c_float]
        L.orc_param_count.restype = C.c_uint64
        L.orc_param_count.argtypes = [C.c_int32, C.c_void_p]
        L.orc_loss.restype = C.c_double
        L.orc_loss.argtypes = [C.c_double, C.c_double]
        L.orc_loss_grad.restype = C.c_double
        L.orc_loss_grad.argtypes = [C.c_double, C.c_double]
        L.orc_k_step.restype = C.c_double
        L.orc_k_step.argtypes = [C.c_double, C.c_double, C.c_double, C.c_int64]
        L.orc_batch_gradient.restype = C.c_double
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def pack_problem(op, dims, elem_bytes, hw):
    """hw = (num_cu, wave, lds_bytes, max_threads_cu, max_blocks_cu)."""
    d = list(dims) + [0] * (8 - len(dims))
    return np.array([op] + d + [elem_bytes] + list(hw), dtype=np.int32)


class Space:
    def __init__(self, problem_fields, kind):
        self._pb = np.ascontiguousarray(problem_fields, dtype=np.int32)
        assert self._pb.size == 15
        self.h = lib().orc_space_create(_p(self._pb), kind)
        if not self.h:
            raise ValueError("oracle: invalid problem/space")
        ng = C.c_int32()
        radix = (C.c_uint32 * 16)()
        size = C.c_uint64()
        lib().orc_space_info(C.c_void_p(self.h), C.byref(ng), radix, C.byref(size))
        self.n_genes = ng.value
        self.radix = [radix[i] for i in range(self.n_genes)]
        self.size = size.value

    def __del__(self):
        # at interpreter shutdown the module's globals may already be gone: then the process ends anyway
        if getattr(self, "h", None) and lib is not None and C is not None:
            lib().orc_space_destroy(C.c_void_p(self.h))
            self.h = None


def split_table(extent):
    n = lib().orc_split_table(extent, None, 0)
    out = np.zeros((n, 4), dtype=np.uint32)
    lib().orc_split_table(extent, _p(out), n)
    return out


def hash64(seed, rnd, idx, gene):
    return lib().orc_hash(seed, rnd, idx, gene)


def enumerate_candidates(space, mode, n, seed=0, rnd=0, first_index=0, parents=None, p_mut_q32=0, ld=None):
    ld = n if ld is None else ld
    genes = np.zeros((space.n_genes, ld), dtype=np.uint16)
    n_par = 0
    if parents is not None:
        parents = np.ascontiguousarray(parents, dtype=np.uint16)
        assert parents.shape[0] == space.n_genes
        n_par = parents.shape[1]
    rc = lib().orc_enumerate(
        C.c_void_p(space.h), C.c_int32(mode), C.c_uint64(seed), C.c_uint32(rnd), C.c_uint64(first_index),
        C.c_uint64(n), _p(parents), C.c_uint32(n_par), C.c_uint32(p_mut_q32), _p(genes), C.c_uint64(ld))
    if rc:
        raise ValueError("oracle enumerate: rc=%d" % rc)
    return genes


def features(space, genes, n_feat, n=None):
    """Returns (raw u64 [F][ld], feat f32 [F][ld], feat bf16 bits u16 [F][ld], legal u8 [n])."""
    genes = np.ascontiguousarray(genes, dtype=np.uint16)
    ld = genes.shape[1]
    n = ld if n is None else n
    raw = np.zeros((n_feat, ld), dtype=np.uint64)
    f32 = np.zeros((n_feat, ld), dtype=np.float32)
    b16 = np.zeros((n_feat, ld), dtype=np.uint16)
    legal = np.zeros(n, dtype=np.uint8)
    rc = lib().orc_features(C.c_void_p(space.h), _p(genes), C.c_uint64(ld), C.c_uint64(n), C.c_int32(n_feat),
                            _p(raw), _p(f32), _p(b16), _p(legal))
    if rc:
        raise ValueError("oracle features: rc=%d" % rc)
    return raw, f32, b16, legal


def transform(raw):
    return float(lib().orc_transform(C.c_uint64(int(raw))))


def bf16_rne(x):
    return int(lib().orc_bf16_rne(C.c_float(float(x))))


def bf16_bits_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def param_count(widths):
    w = np.asarray(widths, dtype=np.int32)
    return int(lib().orc_param_count(len(w) - 1, _p(w)))


def score(widths, theta, feat_f32, n=None, emulate_bf16=False):
    """theta: fp32 parameter vector (per layer W[in][out] then b[out]); feat [F][ld] fp32 -> fp64 scores."""
    w = np.asarray(widths, dtype=np.int32)
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    assert theta.size == param_count(widths)
    feat = np.ascontiguousarray(feat_f32, dtype=np.float32)
    assert feat.shape[0] == w[0]
    ld = feat.shape[1]
    n = ld if n is None else n
    out = np.zeros(n, dtype=np.float64)
    rc = lib().orc_score(C.c_int32(len(w) - 1), _p(w), _p(theta), _p(feat), C.c_uint64(ld), C.c_uint64(n),
                         C.c_int32(1 if emulate_bf16 else 0), _p(out))
    if rc:
        raise ValueError("oracle score: rc=%d" % rc)
    return out


def score_magnitude(widths, theta, feat_f32, n=None):
    """|b_last| + sum_j |w_last_j| h_j per candidate: the scale a relative error of the output sum refers to."""
    w = np.asarray(widths, dtype=np.int32)
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    feat = np.ascontiguousarray(feat_f32, dtype=np.float32)
    ld = feat.shape[1]
    n = ld if n is None else n
    out = np.zeros(n, dtype=np.float64)
    rc = lib().orc_score_magnitude(C.c_int32(len(w) - 1), _p(w), _p(theta), _p(feat), C.c_uint64(ld), C.c_uint64(n),
                                   _p(out))
    if rc:
        raise ValueError("oracle score_magnitude: rc=%d" % rc)
    return out


def topk(energy, latency, legal, n_segments, k, mode=SEL_THRESHOLD, alpha=1.1, m_latency=0):
    energy = np.ascontiguousarray(energy, dtype=np.float32)
    n = energy.size
    if latency is not None:
        latency = np.ascontiguousarray(latency, dtype=np.float32)
    if legal is not None:
        legal = np.ascontiguousarray(legal, dtype=np.uint8)
    idx = np.zeros((n_segments, k), dtype=np.uint32)
    eo = np.zeros((n_segments, k), dtype=np.float32)
    cnt = np.zeros(n_segments, dtype=np.uint32)
    rc = lib().orc_topk(_p(energy), _p(latency), _p(legal), C.c_uint64(n), C.c_uint32(n_segments), C.c_uint32(k),
                        C.c_int32(mode), C.c_float(alpha), C.c_uint32(m_latency), _p(idx), _p(eo), _p(cnt))
    if rc:
        raise ValueError("oracle topk: rc=%d" % rc)
    return idx, eo, cnt


def loss(pred, y):
    return lib().orc_loss(pred, y)


def loss_grad(pred, y):
    return lib().orc_loss_grad(pred, y)


def batch_gradient(widths, theta64, feat_f32, y64, row0, rows):
    w = np.asarray(widths, dtype=np.int32)
    theta64 = np.ascontiguousarray(theta64, dtype=np.float64)
    feat = np.ascontiguousarray(feat_f32, dtype=np.float32)
    y64 = np.ascontiguousarray(y64, dtype=np.float64)
    grad = np.zeros_like(theta64)
    val = lib().orc_batch_gradient(C.c_int32(len(w) - 1), _p(w), _p(theta64), _p(feat), C.c_uint64(feat.shape[1]),
                                   _p(y64), C.c_uint64(row0), C.c_uint64(rows), _p(grad))
    return val, grad


def update(widths, state64, feat_f32, e_meas, n_steps, minibatch, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
           bf16_weights=False):
    """state64 = [theta | m | v | t] fp64, updated in place.  Returns (snr, loss)."""
    w = np.asarray(widths, dtype=np.int32)
    P = param_count(widths)
    assert state64.dtype == np.float64 and state64.size == 3 * P + 1 and state64.flags.c_contiguous
    feat = np.ascontiguousarray(feat_f32, dtype=np.float32)
    e_meas = np.ascontiguousarray(e_meas, dtype=np.float32)
    snr = C.c_double()
    ls = C.c_double()
    rc = lib().orc_update(C.c_int32(len(w) - 1), _p(w), C.c_int32(1 if bf16_weights else 0), _p(state64), _p(feat),
                          C.c_uint64(feat.shape[1]), _p(e_meas), C.c_uint64(e_meas.size), C.c_int32(n_steps),
                          C.c_int32(minibatch), C.c_double(lr), C.c_double(beta1), C.c_double(beta2),
                          C.c_double(eps), C.byref(snr), C.byref(ls))
    if rc:
        raise ValueError("oracle update: rc=%d" % rc)
    return snr.value, ls.value


def k_step(k, snr, mu, M):
    return lib().orc_k_step(k, snr, mu, M)


def trees_predict(n_feat, depth, node_feat, node_thr, leaf, base, feat_f32, n=None, fp32_sequential=False):
    """node_feat uint8 [T][2^d-1], node_thr float32 [T][2^d-1], leaf float32 [T][2^d]; returns float64 [n]."""
    node_feat = np.ascontiguousarray(node_feat, dtype=np.uint8)
    node_thr = np.ascontiguousarray(node_thr, dtype=np.float32)
    leaf = np.ascontiguousarray(leaf, dtype=np.float32)
    T = leaf.shape[0] if leaf.ndim == 2 else leaf.size >> depth
    feat = np.ascontiguousarray(feat_f32, dtype=np.float32)
    n = feat.shape[1] if n is None else n
    out = np.zeros(n, dtype=np.float64)
    rc = lib().orc_trees_predict(C.c_int32(n_feat), C.c_int32(depth), C.c_int32(T), _p(node_feat), _p(node_thr),
                                 _p(leaf), C.c_double(base), _p(feat), C.c_uint64(feat.shape[1]), C.c_uint64(n),
                                 C.c_int32(1 if fp32_sequential else 0), _p(out))
    if rc:
        raise ValueError("oracle trees_predict: rc=%d" % rc)
    return out


def trees_boost(n_feat, depth, node_feat, node_thr, leaf, n_trees_in, n_rounds, base, feat_f32, e_meas, eta=0.3,
                lam=1.0):
    """Appends n_rounds trees in place (arrays hold at least n_trees_in + n_rounds trees).  Returns (snr, loss)."""
    for a, dt in ((node_feat, np.uint8), (node_thr, np.float32), (leaf, np.float32)):
        assert a.dtype == dt and a.flags.c_contiguous
    assert leaf.size >> depth >= n_trees_in + n_rounds
    feat = np.ascontiguousarray(feat_f32, dtype=np.float32)
    e_meas = np.ascontiguousarray(e_meas, dtype=np.float32)
    snr, ls = C.c_double(), C.c_double()
    rc = lib().orc_trees_boost(C.c_int32(n_feat), C.c_int32(depth), C.c_int32(n_trees_in), C.c_int32(n_rounds),
                               _p(node_feat), _p(node_thr), _p(leaf), C.c_double(base), _p(feat),
                               C.c_uint64(feat.shape[1]), _p(e_meas), C.c_uint64(e_meas.size), C.c_double(eta),
                               C.c_double(lam), C.byref(snr), C.byref(ls))
    if rc:
        raise ValueError("oracle trees_boost: rc=%d" % rc)
    return snr.value, ls.value


def dedup(genes, n=None):
    """keep[i] = 1 iff no earlier candidate has the same genes (uint16 [G][ld])"""
    genes = np.ascontiguousarray(genes, dtype=np.uint16)
    n = genes.shape[1] if n is None else n
    keep = np.zeros(n, dtype=np.uint8)
    rc = lib().orc_dedup(_p(genes), C.c_uint64(genes.shape[1]), C.c_uint64(n), C.c_int32(genes.shape[0]), _p(keep))
    if rc:
        raise ValueError("oracle dedup: rc=%d" % rc)
    return keep
