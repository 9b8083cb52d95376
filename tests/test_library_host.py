"""Host-side checks that need no GPU: the library loads, exports the declared symbols, rejects bad arguments."""
import ctypes as C
import os
import re

import pytest

import paper_2412_07017_amd as pkg
from paper_2412_07017_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pkg.library_path()):
        from paper_2412_07017_amd.build import build_library
        build_library()
    return pkg.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "asynclm.h")).read()
    declared = sorted(set(re.findall(r"\b(asynclm_[a-z_]+)\s*\(", header)))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(pkg.API_SYMBOLS) == declared


def test_version_and_strerror(lib):
    assert re.match(rb"\d+\.\d+\.\d+", lib.asynclm_version())
    assert lib.asynclm_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert lib.asynclm_strerror(code)


def test_create_rejects_bad_arguments_without_touching_a_device(lib):
    h = C.c_void_p()
    assert lib.asynclm_create(C.byref(h), None, None, None) == pkg.E_INVAL
    cfg = binding._Config(2, 256, 4, 4, 64, 688, 1024, 1e-5, 10000.0, 0, 1, 128, 0)
    w = binding._Weights()
    assert lib.asynclm_create(C.byref(h), C.byref(cfg), C.byref(w), None) == pkg.E_INVAL   # null weights
    assert not h
    for field, bad in (("head_dim", 48), ("n_kv_heads", 3), ("d_model", 250), ("dtype", 7), ("max_seqs", 0),
                       ("max_positions", 0), ("n_layers", 0), ("vocab", -1), ("kv_format", 1), ("kv_format", 5)):
        c2 = binding._Config(2, 256, 4, 4, 64, 688, 1024, 1e-5, 10000.0, 0, 1, 128, 0)
        setattr(c2, field, bad)
        assert lib.asynclm_create(C.byref(h), C.byref(c2), C.byref(w), None) == pkg.E_INVAL, field


def test_null_context_is_rejected(lib):
    n = C.c_int32()
    assert lib.asynclm_seq_len(None, 0, C.byref(n)) == pkg.E_INVAL
    assert lib.asynclm_decode_step(None, 0, -1, None) == pkg.E_INVAL
    assert lib.asynclm_destroy(None) == 0
    assert lib.asynclm_set_option(None, b"graph", 1) == pkg.E_INVAL
