"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
what include/eck.h declares, builds the same schedule spaces as the oracle and
rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2411_18873_amd import eck, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "eck.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(?:int32_t|uint64_t|void)\s+(\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert {"candidate_enumerate", "features_compute", "costmodel_score", "costmodel_update", "topk_select"} <= set(names)
    L = eck.lib()
    for name in names:
        assert hasattr(L, name), name
    assert sorted(eck.EXPORTS) == names
    assert L.eck_version() >= 100


@pytest.mark.parametrize("cfg,kind", [("c1", 0), ("c2", 1), ("c3", 1), ("c2", 2), ("c3", 2)])
def test_spaces_match_the_oracle(cfg, kind):
    pb = synth.CONFIGS[cfg]["problem"]
    mine, ref = eck.Space(pb, kind), oracle.Space(pb, kind)
    assert mine.radix == ref.radix and mine.size == ref.size and mine.n_genes == ref.n_genes


def test_split_tables_match_the_oracle():
    pb = synth.conv2d(2, 12, 36, 9, 30, 3, 3, 1, 1)
    sp = eck.Space(pb, eck.SPACE_SPLIT)
    for gene, extent in enumerate([2, 36, 9, 30, 12]):
        assert sp.table(gene) == [tuple(int(v) for v in r) for r in oracle.split_table(extent)]
    big = eck.Space(synth.gemm(8192, 4096, 2048), eck.SPACE_SPLIT)
    assert big.table(0) == [tuple(int(v) for v in r) for r in oracle.split_table(8192)]
    huge = eck.Space(synth.bgemm(4, 60, 60, 60), eck.SPACE_SPLIT)
    assert huge.size == np.prod([len(oracle.split_table(e)) for e in (4, 60, 60, 60)]) * 20


def _rc_space(fields, kind):
    pb = eck.Problem.from_fields(fields)
    h = C.c_void_p()
    rc = eck.lib().eck_space_create(C.byref(pb), kind, C.byref(h))
    if rc == 0:
        eck.lib().eck_space_destroy(h)
    return rc


def test_space_create_rejects_bad_problems():
    good = synth.gemm(512, 512, 512)
    assert _rc_space(good, eck.SPACE_KNOB) == eck.OK
    assert _rc_space(good, 7) == eck.EINVAL
    bad = good.copy(); bad[9] = 3
    assert _rc_space(bad, eck.SPACE_KNOB) == eck.EINVAL            # elem_bytes
    bad = good.copy(); bad[0] = 9
    assert _rc_space(bad, eck.SPACE_KNOB) == eck.EINVAL            # op
    bad = good.copy(); bad[2] = 0
    assert _rc_space(bad, eck.SPACE_SPLIT) == eck.EINVAL           # zero extent
    bad = good.copy(); bad[1] = 2
    assert _rc_space(bad, eck.SPACE_SPLIT) == eck.EINVAL           # GEMM with a batch
    bad = good.copy(); bad[10] = 0
    assert _rc_space(bad, eck.SPACE_SPLIT) == eck.EINVAL           # hw_num_cu
    assert _rc_space(synth.conv2d(1, 8, 8, 8, 8, 3, 3), eck.SPACE_KNOB) == eck.EUNSUPPORTED
    assert _rc_space(good, eck.SPACE_SPLIT_XRED) == eck.OK and _rc_space(good, 3) == eck.EINVAL  # space kinds
    assert _rc_space(synth.gemm(65535, 65535, 65535), eck.SPACE_SPLIT) == eck.EUNSUPPORTED  # 2^48 multiply-adds
    assert _rc_space(synth.gemm(70000, 8, 8), eck.SPACE_SPLIT) == eck.EUNSUPPORTED
    assert _rc_space(synth.conv2d(1, 8, 8, 2, 2, 3, 3, 1, 0), eck.SPACE_SPLIT) == eck.EINVAL  # kernel larger than image
    assert eck.lib().eck_space_create(None, 0, None) == eck.EINVAL
    assert eck.lib().eck_space_upload(None) == eck.EINVAL


FAKE = C.c_void_p(0x1000)  # never dereferenced: every call below must fail validation first


def test_enumerate_and_features_validate_before_launch():
    L = eck.lib()
    sp = eck.Space(synth.CONFIGS["c1"]["problem"], eck.SPACE_KNOB)
    E = L.candidate_enumerate
    assert E(None, 0, 0, 0, 0, 16, None, 0, 0, FAKE, 16, None) == eck.EINVAL
    assert E(sp.h, 0, 0, 0, 0, 16, None, 0, 0, None, 16, None) == eck.EINVAL
    assert E(sp.h, 0, 0, 0, 0, 0, None, 0, 0, FAKE, 16, None) == eck.EINVAL
    assert E(sp.h, 5, 0, 0, 0, 16, None, 0, 0, FAKE, 16, None) == eck.EINVAL
    assert E(sp.h, 0, 0, 0, 0, 16, None, 0, 0, FAKE, 8, None) == eck.ESHAPE
    assert E(sp.h, 0, 0, 0, 0, 15, None, 0, 0, FAKE, 15, None) == eck.EALIGN
    assert E(sp.h, 0, 0, 0, 0, 16, None, 0, 0, C.c_void_p(0x1002), 16, None) == eck.EALIGN
    assert E(sp.h, 0, 0, 0, 6390, 16, None, 0, 0, FAKE, 16, None) == eck.EINVAL   # beyond the space
    assert E(sp.h, 2, 0, 0, 0, 16, None, 0, 0, FAKE, 16, None) == eck.EINVAL      # MUTATE without parents
    assert E(sp.h, 3, 0, 0, 0, 16, None, 0, 0, FAKE, 16, None) == eck.EINVAL      # CROSSOVER without parents
    assert E(sp.h, 4, 0, 0, 0, 16, FAKE, 4, 0, FAKE, 16, None) == eck.EINVAL      # no such mode
    F = L.features_compute
    assert F(sp.h, None, 16, 16, 32, 0, FAKE, None, None, None) == eck.EINVAL
    assert F(sp.h, FAKE, 16, 16, 32, 0, None, None, None, None) == eck.EINVAL
    assert F(sp.h, FAKE, 16, 16, 48, 0, FAKE, None, None, None) == eck.EUNSUPPORTED
    assert F(sp.h, FAKE, 8, 16, 32, 0, FAKE, None, None, None) == eck.ESHAPE
    assert F(sp.h, FAKE, 17, 16, 32, 0, FAKE, None, None, None) == eck.EALIGN
    assert F(sp.h, FAKE, 16, 16, 32, 5, FAKE, None, None, None) == eck.EINVAL


def test_batched_calls_validate_before_launch():
    L = eck.lib()
    knob = eck.Space(synth.CONFIGS["c1"]["problem"], eck.SPACE_KNOB)
    split = [eck.Space(synth.gemm(*s), eck.SPACE_SPLIT) for s in synth.CONFIGS["c5"]["shapes"][:3]]
    conv = eck.Space(synth.CONFIGS["c2"]["problem"], eck.SPACE_SPLIT)
    H = lambda *sp: (C.c_void_p * len(sp))(*[x.h if x is not None else None for x in sp])
    seeds = (C.c_uint64 * 200)(*range(200))
    E = L.candidate_enumerate_batch
    assert E(None, 3, 1, seeds, 0, 0, 16, None, 0, 0, FAKE, 64, None) == eck.EINVAL
    assert E(H(*split), 0, 1, seeds, 0, 0, 16, None, 0, 0, FAKE, 64, None) == eck.EINVAL
    assert E(H(*split), 3, 1, None, 0, 0, 16, None, 0, 0, FAKE, 64, None) == eck.EINVAL
    assert E(H(split[0], None, split[2]), 3, 1, seeds, 0, 0, 16, None, 0, 0, FAKE, 64, None) == eck.EINVAL
    assert E(H(*([split[0]] * 129)), 129, 1, seeds, 0, 0, 16, None, 0, 0, FAKE, 4096, None) == eck.EUNSUPPORTED
    assert E(H(split[0], knob), 2, 1, seeds, 0, 0, 16, None, 0, 0, FAKE, 64, None) == eck.ESHAPE   # kinds differ
    assert E(H(split[0], conv), 2, 1, seeds, 0, 0, 16, None, 0, 0, FAKE, 64, None) == eck.ESHAPE   # operators differ
    assert E(H(*split), 3, 1, seeds, 0, 0, 16, None, 0, 0, FAKE, 46, None) == eck.ESHAPE           # ld < 3*16
    assert E(H(*split), 3, 2, seeds, 0, 0, 16, None, 0, 0, FAKE, 64, None) == eck.EINVAL           # no parents
    F = L.features_compute_batch
    assert F(None, 3, FAKE, 64, 16, 64, 1, FAKE, None, None, None) == eck.EINVAL
    assert F(H(*split), 3, FAKE, 64, 16, 64, 1, None, None, None, None) == eck.EINVAL
    assert F(H(split[0], conv), 2, FAKE, 64, 16, 64, 1, FAKE, None, None, None) == eck.ESHAPE
    assert F(H(*split), 3, FAKE, 46, 16, 64, 1, FAKE, None, None, None) == eck.ESHAPE
    assert F(H(*split), 3, FAKE, 64, 16, 48, 1, FAKE, None, None, None) == eck.EUNSUPPORTED


def test_model_and_score_validation():
    L = eck.lib()
    W = lambda *w: (C.c_int32 * len(w))(*w)
    h = C.c_void_p()
    assert L.eck_model_create(3, W(64, 256, 256, 1), 9, C.byref(h)) == eck.EINVAL
    assert L.eck_model_create(2, W(64, 256, 1), eck.F32, C.byref(h)) == eck.EUNSUPPORTED
    assert L.eck_model_create(3, W(64, 256, 256, 2), eck.F32, C.byref(h)) == eck.ESHAPE
    assert L.eck_model_create(3, W(48, 256, 256, 1), eck.F32, C.byref(h)) == eck.EUNSUPPORTED
    assert L.eck_model_create(3, W(64, 250, 256, 1), eck.BF16, C.byref(h)) == eck.EUNSUPPORTED
    assert L.eck_model_create(3, W(64, 1024, 256, 1), eck.BF16, C.byref(h)) == eck.EUNSUPPORTED
    # bf16 models exist only in the shapes the matrix-core kernels are built for: refused before any allocation
    assert L.eck_model_create(3, W(64, 384, 384, 1), eck.BF16, C.byref(h)) == eck.EUNSUPPORTED
    assert L.eck_model_create(3, W(64, 512, 256, 1), eck.BF16, C.byref(h)) == eck.EUNSUPPORTED
    assert L.eck_model_create(3, W(32, 512, 512, 1), eck.BF16, C.byref(h)) == eck.EUNSUPPORTED
    assert L.eck_model_create(3, W(64, 0, 256, 1), eck.BF16, C.byref(h)) == eck.EINVAL
    p = C.c_uint64()
    assert L.eck_model_param_count(3, W(64, 256, 256, 1), C.byref(p)) == 0 and p.value == 82689
    assert L.eck_model_param_count(3, W(64, 512, 512, 1), C.byref(p)) == 0 and p.value == 296449
    assert p.value == synth.param_count([64, 512, 512, 1]) == oracle.param_count([64, 512, 512, 1])
    assert L.costmodel_score(None, FAKE, 0, 16, 16, FAKE, None, 0, None) == eck.EINVAL


def test_topk_validation_and_workspace():
    L = eck.lib()
    T = L.topk_select
    f = C.c_float
    args = lambda n, S, k, mode=0, alpha=1.1, m=0, ws=FAKE, wsb=1 << 30, lat=FAKE: (
        FAKE, lat, None, n, S, k, mode, f(alpha), m, FAKE, FAKE, FAKE, ws, wsb, None)
    assert T(*args(0, 1, 1)) == eck.EINVAL
    assert T(*args(1024, 1, 0)) == eck.EINVAL
    assert T(*args(1024, 1, 8, mode=3)) == eck.EINVAL
    assert T(*args(1024, 1, 8, alpha=0.9)) == eck.EINVAL
    assert T(*args(1024, 1, 8, alpha=float("nan"))) == eck.EINVAL
    assert T(*args(1024, 1, 8, mode=1, m=0)) == eck.EINVAL
    assert T(*args(1000, 3, 8)) == eck.ESHAPE
    assert T(*args(1024, 4, 257)) == eck.ESHAPE
    assert T(*args(1 << 20, 1, 5000)) == eck.EUNSUPPORTED
    assert T(*args(1024, 1, 8, ws=None)) == eck.EWORKSPACE
    assert T(*args(1024, 1, 8, wsb=16)) == eck.EWORKSPACE
    assert T(*args(1024, 1, 8, ws=C.c_void_p(0x1008))) == eck.EALIGN
    K = L.topk_select_known_min
    assert K(FAKE, None, None, 1024, 1, 8, f(1.1), FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == eck.EINVAL
    assert K(FAKE, FAKE, None, 1024, 1, 8, f(1.1), None, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == eck.EINVAL
    assert K(FAKE, FAKE, None, 1000, 3, 8, f(1.1), FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == eck.ESHAPE
    assert L.costmodel_score_min(None, FAKE, 0, 16, 16, FAKE, None, 1, FAKE, None) == eck.EINVAL
    need = L.topk_select_workspace_bytes(1 << 24, 64, 32)
    assert 0 < need < (8 << 20)
    assert L.topk_select_workspace_bytes(1000, 3, 8) == 0
    assert L.costmodel_update_workspace_bytes(None, 4096, 512) == 0


def test_binding_fails_loudly_without_the_library(monkeypatch):
    monkeypatch.setattr(eck, "_lib", None)
    monkeypatch.setattr(eck, "LIB_PATH", "/nonexistent/libeck.so")
    with pytest.raises(OSError):
        eck.lib()


def test_product_package_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2411_18873_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, name)).read()
                assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, name
    text = open(os.path.join(ROOT, "oracle", "__init__.py")).read() + open(os.path.join(ROOT, "oracle", "eck_oracle.c")).read()
    assert "paper_2411_18873_amd" not in text and "libeck" not in text and "eck.h" not in text


def test_tree_model_validation():
    L = eck.lib()
    h = C.c_void_p()
    T = L.eck_trees_create
    assert T(64, 6, 100, 0.5, None) == eck.EINVAL
    assert T(0, 6, 100, 0.5, C.byref(h)) == eck.EINVAL
    assert T(64, 0, 100, 0.5, C.byref(h)) == eck.EINVAL
    assert T(64, 6, 0, 0.5, C.byref(h)) == eck.EINVAL
    assert T(64, 6, 100, float("nan"), C.byref(h)) == eck.EINVAL
    assert T(257, 6, 100, 0.5, C.byref(h)) == eck.EUNSUPPORTED
    assert T(64, 9, 100, 0.5, C.byref(h)) == eck.EUNSUPPORTED
    assert T(64, 6, 70000, 0.5, C.byref(h)) == eck.EUNSUPPORTED
    assert h.value is None
    n = C.c_int32()
    assert L.eck_trees_count(None, C.byref(n)) == eck.EINVAL
    assert L.eck_trees_set(None, 0, None, None, None, None) == eck.EINVAL
    assert L.eck_trees_get(None, None, None, None, None) == eck.EINVAL
    assert L.treemodel_score(None, FAKE, 0, 16, 16, FAKE, None) == eck.EINVAL
    assert L.treemodel_update_workspace_bytes(None, 100) == 0
    assert L.treemodel_update(None, FAKE, 0, 16, FAKE, 16, 1, 0.3, 1.0, FAKE, FAKE, FAKE, 1 << 20, None) == eck.EINVAL
    L.eck_trees_destroy(None)


def test_k_controller_matches_the_oracle_and_validates():
    for k in (0.0, 0.1, 0.2, 0.5, 0.8, 1.0):
        for snr in (0.0, 1.0, 9.999, 10.0, 50.0, float("inf"), float("nan")):
            for M in (0, 1, 4, 100):
                assert eck.k_step(k, snr, 10.0, M) == oracle.k_step(k, snr, 10.0, M)
    L = eck.lib()
    out = C.c_double()
    assert L.eck_k_step(0.5, 1.0, 10.0, 64, None) == eck.EINVAL
    assert L.eck_k_step(1.5, 1.0, 10.0, 64, C.byref(out)) == eck.EINVAL
    assert L.eck_k_step(0.5, 1.0, 10.0, -1, C.byref(out)) == eck.EINVAL
    assert L.eck_k_step(0.5, 1.0, float("nan"), 64, C.byref(out)) == eck.EINVAL
    # how many kernels a round measures: round(k M), halves up; Alg. 1's k sequence on M = 64
    assert [eck.k_count(k, 64) for k in (1.0, 0.8, 0.6000000000000001, 0.4000000000000001, 0.2, 0.0)] == \
        [64, 51, 38, 26, 13, 0]
    assert eck.k_count(0.5, 5) == 3 and eck.k_count(0.5, 64) == 32 and eck.k_count(1e-9, 64) == 0
    cnt = C.c_int64()
    assert L.eck_k_count(0.5, 64, None) == eck.EINVAL
    assert L.eck_k_count(1.5, 64, C.byref(cnt)) == eck.EINVAL
    assert L.eck_k_count(float("nan"), 64, C.byref(cnt)) == eck.EINVAL
    assert L.eck_k_count(0.5, -1, C.byref(cnt)) == eck.EINVAL


def test_dedup_validation():
    L = eck.lib()
    D = L.eck_candidates_dedup
    assert L.eck_candidates_dedup_workspace_bytes(0) == 0
    assert L.eck_candidates_dedup_workspace_bytes(1000) == 2048 * 4
    assert L.eck_candidates_dedup_workspace_bytes((1 << 30) + 1) == 0
    assert D(None, 16, 16, 5, FAKE, 1, FAKE, 1 << 20, None) == eck.EINVAL
    assert D(FAKE, 16, 16, 5, None, 1, FAKE, 1 << 20, None) == eck.EINVAL
    assert D(FAKE, 16, 0, 5, FAKE, 1, FAKE, 1 << 20, None) == eck.EINVAL
    assert D(FAKE, 16, 16, 0, FAKE, 1, FAKE, 1 << 20, None) == eck.EINVAL
    assert D(FAKE, 8, 16, 5, FAKE, 1, FAKE, 1 << 20, None) == eck.ESHAPE
    assert D(FAKE, 16, 16, 5, FAKE, 1, FAKE, 16, None) == eck.EWORKSPACE
    assert D(FAKE, 16, 16, 5, FAKE, 1, C.c_void_p(0x1001), 1 << 20, None) == eck.EALIGN
