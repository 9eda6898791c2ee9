"""CPU-only checks of the C ABI: the library loads, exports every symbol the
header declares, validates arguments before touching the GPU, and its host-side
eta agrees with the oracle's."""
import ctypes as C
import os
import re

import pytest

import oracle
import paper_1908_10396_amd as avq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    with open(os.path.join(ROOT, "include", "avq.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    return sorted(set(re.findall(r"\b(avq_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = avq.lib()
    declared = _declared_symbols()
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(avq.SYMBOLS) == declared
    assert b"gfx950" in L.avq_version()


def test_eta_host_matches_oracle():
    for d, T, norm in [(100, 0.2, 1.0), (32, 0.2, 1.0), (256, 0.2, 0.8), (128, 0.5, 2.0), (16, 0.0, 1.0),
                       (10, 0.05, 1.0), (64, 3.0, 1.0)]:
        assert avq.eta(d, T, norm, avq.ETA_LIMIT) == pytest.approx(oracle.eta_limit(d, T, norm), rel=1e-12)
        assert avq.eta(d, T, norm, avq.ETA_EXACT) == pytest.approx(oracle.eta_exact(d, T, norm), rel=1e-8)
    assert avq.eta(100, 0.2) == pytest.approx(4.125, abs=1e-12)   # the constant Section 5.1 prints
    assert avq.eta(100, 0.2, 0.0) == 1.0


@pytest.mark.parametrize("kw", [
    dict(d=1, M=1), dict(d=100, M=7), dict(d=100, M=0), dict(d=100, M=50, bits=5),
    dict(d=100, M=50, T=-0.1), dict(d=100, M=50, eta_mode=3),
    dict(d=100, M=50, eta_mode=2, eta_explicit=0.5), dict(d=100, M=50, kmeans_iters=-1),
    dict(d=100, M=50, n_leaves=-2), dict(d=512, M=512), dict(d=100, M=50, leaf_aniso_iters=-1),
])
def test_create_rejects_bad_config_without_a_gpu(kw):
    base = dict(d=100, M=50, bits=4, T=0.2, eta_mode=0, eta_explicit=1.0, kmeans_iters=1,
                encode_passes=1, n_leaves=0, leaf_kmeans_iters=1, borrow_x=1, seed=0, leaf_aniso_iters=0)
    base.update(kw)
    cfg = avq.AvqConfig(*[base[f[0]] for f in avq.AvqConfig._fields_])
    h = C.c_void_p()
    rc = avq.lib().avq_create(C.byref(cfg), C.byref(h))
    assert rc == avq.AVQ_EINVAL
    assert h.value is None
    assert len(avq.lib().avq_last_error()) > 0


def test_null_arguments_are_errors_not_crashes():
    L = avq.lib()
    assert L.avq_create(None, None) == avq.AVQ_EINVAL
    assert L.avq_search(None, None, 1, 1, 0, 0, 0, None, None, None) == avq.AVQ_EINVAL
    assert L.avq_set_tuning(None, b"scan_qt", 1) == avq.AVQ_EINVAL
    assert L.avq_size(None) == 0
    L.avq_destroy(None)
    assert L.avq_eta(100, 0.2, 1.0, 7) == -1.0


def test_product_package_does_not_import_the_oracle():
    # the HIP path and the oracle share no code
    pkg = os.path.join(ROOT, "paper_1908_10396_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                with open(os.path.join(dirpath, fn)) as f:
                    src = f.read()
                assert "oracle" not in src.replace("no oracle", ""), fn


def _shell_index(d=100, M=50, bits=4, n_leaves=0):
    """An Index object with its shape attributes but no library handle: the binding must refuse a wrong shape
    before it passes any pointer on (no GPU is needed to see that)."""
    idx = avq.Index.__new__(avq.Index)
    idx.d, idx.M, idx.bits, idx.n_leaves = d, M, bits, n_leaves
    idx.kc, idx.ds, idx.nb = 1 << bits, d // M, (M * bits + 7) // 8
    idx.cfg = avq.AvqConfig(d, M, bits, 0.2, 0, 1.0, 1, 1, n_leaves, 1, 1, 0, 0)
    idx._h = None
    idx._keep = []
    return idx


def test_binding_refuses_wrong_shapes_before_any_pointer_is_passed():
    import numpy as np
    import torch
    idx = _shell_index()
    f32 = lambda *shape: torch.zeros(shape, dtype=torch.float32)
    i32 = lambda *shape: torch.zeros(shape, dtype=torch.int32)
    with pytest.raises(ValueError):
        idx.search(f32(4, 99), 10, 100)                                  # queries of the wrong dimension
    with pytest.raises(ValueError):
        idx.search(f32(4, 100), 10, 100, out=(i32(4, 9), f32(4, 10)))    # ids too narrow
    with pytest.raises(ValueError):
        idx.search(f32(4, 100), 10, 100, out=(i32(4, 10), f32(3, 10)))   # scores too short
    with pytest.raises(ValueError):
        idx.search_noalloc(f32(2, 100), 10, 100, out=(i32(2, 10), f32(2, 11)))
    with pytest.raises(ValueError):
        idx.brute_force(f32(4, 101), 10)
    with pytest.raises(ValueError):
        idx.train(f32(1000, 64))
    with pytest.raises(ValueError):
        idx.encode(f32(1000))
    with pytest.raises(ValueError):
        idx.update_codebooks(f32(1000, 50))
    with pytest.raises(ValueError):
        idx.set_codebooks(np.zeros((50, 16, 3), np.float32))
    with pytest.raises(ValueError):
        idx.set_database(None, np.zeros((100, 24), np.uint8))            # 25 code bytes per point expected
    with pytest.raises(ValueError):
        idx.set_database(f32(99, 100), np.zeros((100, 25), np.uint8))    # x and codes disagree on n
    with pytest.raises(ValueError):
        idx.debug_lut(f32(4, 10), 0)
    with pytest.raises(ValueError):
        idx.debug_adc_scores(f32(4, 10), 0)
    ivf = _shell_index(n_leaves=8)
    with pytest.raises(ValueError):
        ivf.set_leaf_centers(np.zeros((8, 99), np.float32))
    with pytest.raises(ValueError):
        ivf.set_database(None, np.zeros((100, 25), np.uint8), np.zeros(99, np.int32))
    with pytest.raises(ValueError):
        ivf.debug_leaf_select(f32(2, 7), 4)
    # right shapes but host tensors: the device check still refuses them
    with pytest.raises(TypeError):
        idx.search(f32(4, 100), 10, 100)
