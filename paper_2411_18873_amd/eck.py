"""ctypes binding over libeck.so -- argument marshalling only.

Every function takes torch CUDA tensors (device memory and the current stream
come from PyTorch), passes raw pointers and sizes through the C ABI declared in
include/eck.h and raises EckError on a non-zero return code.  No arithmetic of
the method happens here, and there is no fallback: if the library is missing
the import of the library handle fails loudly.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libeck.so")

OK, EINVAL, ESHAPE, EUNSUPPORTED, EALIGN, EWORKSPACE, EDEVICE = 0, -1, -2, -3, -4, -5, -6
ERROR_NAMES = {EINVAL: "ECK_EINVAL", ESHAPE: "ECK_ESHAPE", EUNSUPPORTED: "ECK_EUNSUPPORTED", EALIGN: "ECK_EALIGN",
               EWORKSPACE: "ECK_EWORKSPACE", EDEVICE: "ECK_EDEVICE"}
OP_GEMM, OP_BGEMM, OP_CONV2D = 0, 1, 2
SPACE_KNOB, SPACE_SPLIT, SPACE_SPLIT_XRED = 0, 1, 2
MODE_EXHAUSTIVE, MODE_SAMPLE, MODE_MUTATE, MODE_CROSSOVER = 0, 1, 2, 3
F32, BF16 = 0, 1
SELECT_THRESHOLD, SELECT_RANK = 0, 1
MAX_K = 4096
MAX_BATCH = 128

EXPORTS = ["eck_version", "eck_space_create", "eck_space_upload", "eck_space_destroy", "eck_space_info", "eck_space_table",
           "candidate_enumerate", "candidate_enumerate_batch", "eck_candidates_gather", "features_compute",
           "features_compute_batch", "eck_model_create", "eck_model_destroy",
           "eck_model_param_count", "eck_model_set_state", "eck_model_get_state", "costmodel_score", "costmodel_score_min",
           "topk_select_known_min",
           "topk_select_workspace_bytes", "topk_select_rank_workspace_bytes", "topk_select", "topk_select_static", "costmodel_update_workspace_bytes", "costmodel_update",
           "eck_trees_create", "eck_trees_destroy", "eck_trees_count", "eck_trees_set", "eck_trees_get",
           "treemodel_score", "treemodel_update_workspace_bytes", "treemodel_update", "eck_k_step", "eck_k_count",
           "eck_candidates_dedup", "eck_candidates_dedup_workspace_bytes"]


class EckError(RuntimeError):
    def __init__(self, fn, code):
        super().__init__("%s failed: %s (%d)" % (fn, ERROR_NAMES.get(code, "?"), code))
        self.code = code


class Problem(C.Structure):
    _fields_ = [("op", C.c_int32), ("dim", C.c_int32 * 8), ("elem_bytes", C.c_int32), ("hw_num_cu", C.c_int32),
                ("hw_wave", C.c_int32), ("hw_lds_bytes", C.c_int32), ("hw_max_threads_cu", C.c_int32),
                ("hw_max_blocks_cu", C.c_int32)]

    @classmethod
    def from_fields(cls, fields):
        """fields: 15 int32 = op, dim[8], elem_bytes, 5 hardware parameters."""
        f = [int(v) for v in fields]
        assert len(f) == 15
        return cls(f[0], (C.c_int32 * 8)(*f[1:9]), *f[9:15])


_lib = None


def lib():
    """The loaded library; raises OSError when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("libeck.so is not built (run `python -m paper_2411_18873_amd.build`): " + LIB_PATH)
        L = C.CDLL(LIB_PATH)
        u64, u32, i32, vp, f32 = C.c_uint64, C.c_uint32, C.c_int32, C.c_void_p, C.c_float
        L.eck_version.restype = i32
        L.eck_space_create.argtypes = [C.POINTER(Problem), i32, C.POINTER(vp)]
        L.eck_space_upload.argtypes = [vp]
        L.eck_space_destroy.argtypes = [vp]
        L.eck_space_destroy.restype = None
        L.eck_space_info.argtypes = [vp, C.POINTER(i32), C.POINTER(u32), C.POINTER(u64)]
        L.eck_space_table.argtypes = [vp, i32, vp, u32]
        L.candidate_enumerate.argtypes = [vp, i32, u64, u32, u64, u64, vp, u32, u32, vp, u64, vp]
        L.candidate_enumerate_batch.argtypes = [vp, u32, i32, vp, u32, u64, u64, vp, u32, u32, vp, u64, vp]
        L.features_compute_batch.argtypes = [vp, u32, vp, u64, u64, i32, i32, vp, vp, vp, vp]
        L.eck_candidates_gather.argtypes = [vp, u64, u64, i32, vp, u32, vp, u64, vp]
        L.features_compute.argtypes = [vp, vp, u64, u64, i32, i32, vp, vp, vp, vp]
        L.eck_model_create.argtypes = [i32, C.POINTER(i32), i32, C.POINTER(vp)]
        L.eck_model_destroy.argtypes = [vp]
        L.eck_model_destroy.restype = None
        L.eck_model_param_count.argtypes = [i32, C.POINTER(i32), C.POINTER(u64)]
        L.eck_model_set_state.argtypes = [vp, vp, u64, vp]
        L.eck_model_get_state.argtypes = [vp, vp, u64, vp]
        L.costmodel_score.argtypes = [vp, vp, i32, u64, u64, vp, vp, u64, vp]
        L.costmodel_score_min.argtypes = [vp, vp, i32, u64, u64, vp, vp, u32, vp, vp]
        L.topk_select_known_min.argtypes = [vp, vp, vp, u64, u32, u32, f32, vp, vp, vp, vp, vp, u64, vp]
        L.eck_candidates_dedup_workspace_bytes.argtypes = [u64]
        L.eck_candidates_dedup_workspace_bytes.restype = u64
        L.eck_candidates_dedup.argtypes = [vp, u64, u64, i32, vp, i32, vp, u64, vp]
        L.eck_k_step.argtypes = [C.c_double, C.c_double, C.c_double, C.c_int64, C.POINTER(C.c_double)]
        L.eck_k_count.argtypes = [C.c_double, C.c_int64, C.POINTER(C.c_int64)]
        L.eck_trees_create.argtypes = [i32, i32, i32, f32, C.POINTER(vp)]
        L.eck_trees_destroy.argtypes = [vp]
        L.eck_trees_destroy.restype = None
        L.eck_trees_count.argtypes = [vp, C.POINTER(i32)]
        L.eck_trees_set.argtypes = [vp, i32, vp, vp, vp, vp]
        L.eck_trees_get.argtypes = [vp, vp, vp, vp, vp]
        L.treemodel_score.argtypes = [vp, vp, i32, u64, u64, vp, vp]
        L.treemodel_update_workspace_bytes.argtypes = [vp, u64]
        L.treemodel_update_workspace_bytes.restype = u64
        L.treemodel_update.argtypes = [vp, vp, i32, u64, vp, u64, i32, f32, f32, vp, vp, vp, u64, vp]
        L.topk_select_workspace_bytes.argtypes = [u64, u32, u32]
        L.topk_select_workspace_bytes.restype = u64
        L.topk_select_rank_workspace_bytes.argtypes = [u64, u32, u32, u32]
        L.topk_select_rank_workspace_bytes.restype = u64
        L.topk_select.argtypes = [vp, vp, vp, u64, u32, u32, i32, f32, u32, vp, vp, vp, vp, u64, vp]
        L.topk_select_static.argtypes = [vp, vp, vp, u64, u32, u32, i32, f32, u32, vp, vp, vp, vp]
        L.costmodel_update_workspace_bytes.argtypes = [vp, u64, i32]
        L.costmodel_update_workspace_bytes.restype = u64
        L.costmodel_update.argtypes = [vp, vp, i32, u64, vp, u64, i32, i32, f32, f32, f32, f32, vp, vp, vp, u64, vp]
        for name in EXPORTS:
            fn = getattr(L, name)
            if name not in ("eck_space_destroy", "eck_model_destroy", "topk_select_workspace_bytes",
                            "topk_select_rank_workspace_bytes", "eck_trees_destroy",
                            "eck_candidates_dedup_workspace_bytes", "treemodel_update_workspace_bytes",
                            "costmodel_update_workspace_bytes"):
                fn.restype = i32
        _lib = L
    return _lib


def _check(fn, rc):
    if rc != OK:
        raise EckError(fn, rc)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    if t is None:
        return
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (name, dtype))


class Space:
    """Schedule space of one operator (eck_space)."""

    def __init__(self, problem_fields, kind):
        self._pb = Problem.from_fields(problem_fields)
        h = C.c_void_p()
        _check("eck_space_create", lib().eck_space_create(C.byref(self._pb), kind, C.byref(h)))
        self.h = h
        ng, radix, size = C.c_int32(), (C.c_uint32 * 16)(), C.c_uint64()
        _check("eck_space_info", lib().eck_space_info(self.h, C.byref(ng), radix, C.byref(size)))
        self.n_genes = ng.value
        self.radix = [radix[i] for i in range(self.n_genes)]
        self.size = size.value
        self.kind = kind

    def table(self, gene):
        n = lib().eck_space_table(self.h, gene, None, 0)
        if n < 0:
            raise EckError("eck_space_table", n)
        buf = (C.c_uint32 * (4 * n))()
        lib().eck_space_table(self.h, gene, buf, n)
        return [tuple(buf[4 * i:4 * i + 4]) for i in range(n)]

    def upload(self):
        """make the device copy of the tables now (otherwise the first launch on the space does)"""
        _check("eck_space_upload", lib().eck_space_upload(self.h))
        return self

    def close(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.eck_space_destroy(self.h)
        self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Model:
    """Cost model (eck_model): fp32 master parameters, Adam moments, packed weights."""

    def __init__(self, widths, dtype):
        self.widths = [int(w) for w in widths]
        self.dtype = dtype
        w = (C.c_int32 * len(self.widths))(*self.widths)
        p = C.c_uint64()
        _check("eck_model_param_count", lib().eck_model_param_count(len(self.widths) - 1, w, C.byref(p)))
        self.n_params = p.value
        h = C.c_void_p()
        _check("eck_model_create", lib().eck_model_create(len(self.widths) - 1, w, dtype, C.byref(h)))
        self.h = h

    def set_state(self, blob):
        _dev(blob, torch.float32, "blob")
        _check("eck_model_set_state", lib().eck_model_set_state(self.h, _ptr(blob), blob.numel(), _stream()))

    def get_state(self):
        blob = torch.empty(3 * self.n_params + 1, dtype=torch.float32, device="cuda")
        _check("eck_model_get_state", lib().eck_model_get_state(self.h, _ptr(blob), blob.numel(), _stream()))
        return blob

    def close(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.eck_model_destroy(self.h)
        self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Trees:
    """Boosted regression-tree cost model (eck_trees): complete trees of one depth, level-order arrays."""

    def __init__(self, n_feat, depth, capacity, base_score=0.5):
        self.n_feat, self.depth, self.capacity, self.base_score = int(n_feat), int(depth), int(capacity), float(base_score)
        h = C.c_void_p()
        _check("eck_trees_create", lib().eck_trees_create(self.n_feat, self.depth, self.capacity, self.base_score,
                                                          C.byref(h)))
        self.h = h

    @property
    def n_trees(self):
        n = C.c_int32()
        _check("eck_trees_count", lib().eck_trees_count(self.h, C.byref(n)))
        return n.value

    def set(self, node_feat, node_thr, leaf):
        """uint8 [T][2^d-1], float32 [T][2^d-1], float32 [T][2^d] CUDA tensors"""
        n = int(leaf.shape[0])
        _dev(node_feat, torch.uint8, "node_feat")
        _dev(node_thr, torch.float32, "node_thr")
        _dev(leaf, torch.float32, "leaf")
        assert node_feat.shape == (n, (1 << self.depth) - 1) == node_thr.shape and leaf.shape[1] == 1 << self.depth
        _check("eck_trees_set", lib().eck_trees_set(self.h, n, _ptr(node_feat), _ptr(node_thr), _ptr(leaf), _stream()))

    def get(self):
        n = self.n_trees
        node_feat = torch.zeros((n, (1 << self.depth) - 1), dtype=torch.uint8, device="cuda")
        node_thr = torch.zeros((n, (1 << self.depth) - 1), dtype=torch.float32, device="cuda")
        leaf = torch.zeros((n, 1 << self.depth), dtype=torch.float32, device="cuda")
        _check("eck_trees_get", lib().eck_trees_get(self.h, _ptr(node_feat), _ptr(node_thr), _ptr(leaf), _stream()))
        return node_feat, node_thr, leaf

    def close(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.eck_trees_destroy(self.h)
        self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _at(t, col0):
    """pointer to column col0 of a row-major 2-D (or 1-D) tensor"""
    return None if t is None else C.c_void_p(t.data_ptr() + col0 * t.element_size())


def candidate_enumerate(space, mode, n, genes_out, seed=0, round=0, first_index=0, parents=None, p_mut_q32=0, col0=0):
    """genes_out: uint16 [n_genes][ld] CUDA tensor (torch.int16 storage is accepted as raw bits).
    col0: first column written (the n candidates land in columns col0 .. col0+n-1)."""
    _dev(genes_out, genes_out.dtype, "genes_out")
    assert genes_out.element_size() == 2 and genes_out.dim() == 2 and genes_out.shape[0] == space.n_genes
    n_par = 0
    if parents is not None:
        _dev(parents, parents.dtype, "parents")
        assert parents.element_size() == 2 and parents.shape[0] == space.n_genes
        n_par = parents.shape[1]
    _check("candidate_enumerate", lib().candidate_enumerate(
        space.h, mode, seed, round, first_index, n, _ptr(parents), n_par, p_mut_q32, _at(genes_out, col0),
        genes_out.shape[1], _stream()))


def _handles(spaces):
    return (C.c_void_p * len(spaces))(*[sp.h for sp in spaces])


def candidate_enumerate_batch(spaces, mode, n_per_space, genes_out, seeds, round=0, first_index=0, parents=None,
                              p_mut_q32=0):
    """One launch for all spaces: space s writes columns [s*n_per_space, (s+1)*n_per_space) of genes_out and, in
    MUTATE, inherits from columns [s*P, (s+1)*P) of parents (P = parents.shape[1] / len(spaces))."""
    _dev(genes_out, genes_out.dtype, "genes_out")
    assert genes_out.element_size() == 2 and genes_out.dim() == 2 and genes_out.shape[0] == spaces[0].n_genes
    assert len(seeds) == len(spaces)
    n_par = 0
    if parents is not None:
        _dev(parents, parents.dtype, "parents")
        assert parents.element_size() == 2 and parents.shape[0] == spaces[0].n_genes
        assert parents.shape[1] % len(spaces) == 0
        n_par = parents.shape[1] // len(spaces)
    seed_arr = (C.c_uint64 * len(seeds))(*[int(x) for x in seeds])
    _check("candidate_enumerate_batch", lib().candidate_enumerate_batch(
        _handles(spaces), len(spaces), mode, seed_arr, round, first_index, n_per_space, _ptr(parents), n_par,
        p_mut_q32, _ptr(genes_out), genes_out.shape[1], _stream()))


def features_compute_batch(spaces, genes, n_per_space, n_feat, out_dtype, feat_out=None, raw_out=None,
                           legal_out=None):
    """One launch for all spaces; columns [s*n_per_space, (s+1)*n_per_space) belong to spaces[s]."""
    assert genes.element_size() == 2 and genes.is_cuda and genes.is_contiguous()
    ld = genes.shape[1]
    total = n_per_space * len(spaces)
    assert total <= ld
    for t in (feat_out, raw_out):
        if t is not None:
            assert t.is_cuda and t.is_contiguous() and t.shape[0] == n_feat and t.shape[1] == ld
    if feat_out is not None:
        assert feat_out.dtype == (torch.float32 if out_dtype == F32 else torch.bfloat16)
    if raw_out is not None:
        assert raw_out.element_size() == 8
    if legal_out is not None:
        assert legal_out.is_cuda and legal_out.element_size() == 1 and legal_out.numel() >= total
    _check("features_compute_batch", lib().features_compute_batch(
        _handles(spaces), len(spaces), _ptr(genes), ld, n_per_space, n_feat, out_dtype, _ptr(feat_out),
        _ptr(raw_out), _ptr(legal_out), _stream()))


def candidates_gather(genes, n, idx, k, out, col0=0, idx_off=0):
    """out[g][j] = genes[g][col0 + idx[idx_off + j]] for j < k (survivors -> parents)."""
    assert genes.element_size() == 2 and out.element_size() == 2 and idx.element_size() == 4
    assert genes.is_cuda and out.is_cuda and idx.is_cuda and idx.numel() >= idx_off + k
    _check("eck_candidates_gather", lib().eck_candidates_gather(
        _at(genes, col0), genes.shape[1], n, genes.shape[0], _at(idx.view(-1), idx_off), k, _ptr(out), out.shape[1],
        _stream()))


def features_compute(space, genes, n, n_feat, out_dtype, feat_out=None, raw_out=None, legal_out=None, col0=0):
    """col0: first column read in genes and written in feat_out / raw_out / legal_out."""
    assert genes.element_size() == 2 and genes.is_cuda and genes.is_contiguous()
    ld = genes.shape[1]
    assert col0 + n <= ld
    for t in (feat_out, raw_out):
        if t is not None:
            assert t.is_cuda and t.is_contiguous() and t.shape[0] == n_feat and t.shape[1] == ld
    if feat_out is not None:
        assert feat_out.dtype == (torch.float32 if out_dtype == F32 else torch.bfloat16)
    if raw_out is not None:
        assert raw_out.element_size() == 8
    if legal_out is not None:
        assert legal_out.is_cuda and legal_out.element_size() == 1 and legal_out.numel() >= col0 + n
    _check("features_compute", lib().features_compute(space.h, _at(genes, col0), ld, n, n_feat, out_dtype,
                                                      _at(feat_out, col0), _at(raw_out, col0), _at(legal_out, col0),
                                                      _stream()))


def costmodel_score(model, feat, n, score_out):
    feat_dtype = {torch.float32: F32, torch.bfloat16: BF16}[feat.dtype]
    assert feat.is_cuda and feat.is_contiguous() and feat.shape[0] == model.widths[0]
    _dev(score_out, torch.float32, "score_out")
    assert score_out.numel() >= n
    _check("costmodel_score", lib().costmodel_score(model.h, _ptr(feat), feat_dtype, feat.shape[1], n,
                                                    _ptr(score_out), None, 0, _stream()))


def costmodel_score_min(model, feat, n, score_out, legal, n_segments, min_key_out):
    """costmodel_score plus the least score of the legal candidates of every segment (uint32 order keys)"""
    feat_dtype = {torch.float32: F32, torch.bfloat16: BF16}[feat.dtype]
    assert feat.is_cuda and feat.is_contiguous() and feat.shape[0] == model.widths[0]
    _dev(score_out, torch.float32, "score_out")
    assert score_out.numel() >= n
    if legal is not None:
        assert legal.is_cuda and legal.element_size() == 1 and legal.is_contiguous() and legal.numel() >= n
    assert min_key_out.is_cuda and min_key_out.element_size() == 4 and min_key_out.numel() >= n_segments
    _check("costmodel_score_min", lib().costmodel_score_min(model.h, _ptr(feat), feat_dtype, feat.shape[1], n,
                                                            _ptr(score_out), _ptr(legal), n_segments, _ptr(min_key_out),
                                                            _stream()))


def topk_select_known_min(energy, latency, legal, n_segments, k, latency_min_key, idx_out, energy_out, count_out, ws,
                          alpha=1.1):
    """topk_select in THRESHOLD mode with the per-segment least latency from costmodel_score_min"""
    _dev(energy, torch.float32, "energy")
    _dev(latency, torch.float32, "latency")
    if legal is not None:
        assert legal.is_cuda and legal.element_size() == 1 and legal.is_contiguous()
    assert latency_min_key.is_cuda and latency_min_key.element_size() == 4 and latency_min_key.numel() >= n_segments
    assert idx_out.is_cuda and idx_out.element_size() == 4 and idx_out.numel() >= n_segments * k
    _dev(energy_out, torch.float32, "energy_out")
    assert count_out.is_cuda and count_out.element_size() == 4 and count_out.numel() >= n_segments
    assert ws.is_cuda and ws.is_contiguous()
    _check("topk_select_known_min", lib().topk_select_known_min(
        _ptr(energy), _ptr(latency), _ptr(legal), energy.numel(), n_segments, k, alpha, _ptr(latency_min_key),
        _ptr(idx_out), _ptr(energy_out), _ptr(count_out), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def topk_select_workspace_bytes(n, n_segments, k, m_latency=0):
    """m_latency > 0: the workspace of a RANK-mode call with that latency gate"""
    if m_latency:
        return int(lib().topk_select_rank_workspace_bytes(n, n_segments, k, m_latency))
    return int(lib().topk_select_workspace_bytes(n, n_segments, k))


def topk_select(energy, latency, legal, n_segments, k, idx_out, energy_out, count_out, ws, mode=SELECT_THRESHOLD,
                alpha=1.1, m_latency=0):
    _dev(energy, torch.float32, "energy")
    _dev(latency, torch.float32, "latency")
    if legal is not None:
        assert legal.is_cuda and legal.element_size() == 1 and legal.is_contiguous()
    assert idx_out.is_cuda and idx_out.element_size() == 4 and idx_out.numel() >= n_segments * k
    _dev(energy_out, torch.float32, "energy_out")
    assert count_out.is_cuda and count_out.element_size() == 4 and count_out.numel() >= n_segments
    assert ws.is_cuda and ws.is_contiguous()
    _check("topk_select", lib().topk_select(
        _ptr(energy), _ptr(latency), _ptr(legal), energy.numel(), n_segments, k, mode, alpha, m_latency,
        _ptr(idx_out), _ptr(energy_out), _ptr(count_out), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


TOPK_STATIC_BYTES = 8 << 20


def topk_select_static(energy, latency, legal, n_segments, k, idx_out, energy_out, count_out, mode=SELECT_THRESHOLD,
                       alpha=1.1, m_latency=0):
    """topk_select on the library's own fixed workspace: allocates nothing; sizes needing more than
    TOPK_STATIC_BYTES are refused"""
    _dev(energy, torch.float32, "energy")
    _dev(latency, torch.float32, "latency")
    if legal is not None:
        assert legal.is_cuda and legal.element_size() == 1 and legal.is_contiguous()
    assert idx_out.is_cuda and idx_out.element_size() == 4 and idx_out.numel() >= n_segments * k
    _dev(energy_out, torch.float32, "energy_out")
    assert count_out.is_cuda and count_out.element_size() == 4 and count_out.numel() >= n_segments
    _check("topk_select_static", lib().topk_select_static(
        _ptr(energy), _ptr(latency), _ptr(legal), energy.numel(), n_segments, k, mode, alpha, m_latency,
        _ptr(idx_out), _ptr(energy_out), _ptr(count_out), _stream()))


def costmodel_update_workspace_bytes(model, n_pairs, minibatch):
    return int(lib().costmodel_update_workspace_bytes(model.h, n_pairs, minibatch))


def costmodel_update(model, feat, energy_measured, n_steps, minibatch, snr_out, loss_out, ws, lr=1e-3, beta1=0.9,
                     beta2=0.999, eps=1e-8):
    feat_dtype = {torch.float32: F32, torch.bfloat16: BF16}[feat.dtype]
    assert feat.is_cuda and feat.is_contiguous() and feat.shape[0] == model.widths[0]
    _dev(energy_measured, torch.float32, "energy_measured")
    _dev(snr_out, torch.float32, "snr_out")
    _dev(loss_out, torch.float32, "loss_out")
    assert ws.is_cuda and ws.is_contiguous()
    _check("costmodel_update", lib().costmodel_update(
        model.h, _ptr(feat), feat_dtype, feat.shape[1], _ptr(energy_measured), energy_measured.numel(), n_steps,
        minibatch, lr, beta1, beta2, eps, _ptr(snr_out), _ptr(loss_out), _ptr(ws), ws.numel() * ws.element_size(),
        _stream()))


def treemodel_score(trees, feat, n, score_out):
    feat_dtype = {torch.float32: F32, torch.bfloat16: BF16}[feat.dtype]
    assert feat.is_cuda and feat.is_contiguous() and feat.shape[0] == trees.n_feat
    _dev(score_out, torch.float32, "score_out")
    assert score_out.numel() >= n
    _check("treemodel_score", lib().treemodel_score(trees.h, _ptr(feat), feat_dtype, feat.shape[1], n, _ptr(score_out),
                                                    _stream()))


def treemodel_update_workspace_bytes(trees, n_pairs):
    return int(lib().treemodel_update_workspace_bytes(trees.h, n_pairs))


def treemodel_update(trees, feat, energy_measured, n_rounds, snr_out, loss_out, ws, eta=0.3, lam=1.0):
    feat_dtype = {torch.float32: F32, torch.bfloat16: BF16}[feat.dtype]
    assert feat.is_cuda and feat.is_contiguous() and feat.shape[0] == trees.n_feat
    _dev(energy_measured, torch.float32, "energy_measured")
    _dev(snr_out, torch.float32, "snr_out")
    _dev(loss_out, torch.float32, "loss_out")
    assert ws.is_cuda and ws.is_contiguous()
    _check("treemodel_update", lib().treemodel_update(
        trees.h, _ptr(feat), feat_dtype, feat.shape[1], _ptr(energy_measured), energy_measured.numel(), n_rounds, eta,
        lam, _ptr(snr_out), _ptr(loss_out), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def k_step(k, snr, mu, M):
    """next k of the measurement-budget controller (host only)"""
    out = C.c_double()
    _check("eck_k_step", lib().eck_k_step(k, snr, mu, M, C.byref(out)))
    return out.value


def k_count(k, M):
    """kernels to measure this round: round(k * M) (host only)"""
    out = C.c_int64()
    _check("eck_k_count", lib().eck_k_count(k, M, C.byref(out)))
    return out.value


def candidates_dedup_workspace_bytes(n):
    return int(lib().eck_candidates_dedup_workspace_bytes(n))


def candidates_dedup(genes, n, flags, overwrite=False, ws=None):
    """flags[i] (uint8) = first occurrence of its gene tuple (AND-ed into flags unless overwrite)"""
    assert genes.element_size() == 2 and genes.is_cuda and genes.is_contiguous()
    assert flags.is_cuda and flags.element_size() == 1 and flags.numel() >= n
    need = int(lib().eck_candidates_dedup_workspace_bytes(n))
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=genes.device)
    _check("eck_candidates_dedup", lib().eck_candidates_dedup(
        _ptr(genes), genes.shape[1], n, genes.shape[0], _ptr(flags), 1 if overwrite else 0, _ptr(ws),
        ws.numel() * ws.element_size(), _stream()))
