"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
derives the same integer constants as the oracle, and turns bad arguments into error codes.
No GPU compute is called here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2604_25306_amd as qf
from paper_2604_25306_amd.binding import EXPORTS, QFlashParams

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(qf.library_path()):
        from paper_2604_25306_amd.build import build
        build(verbose=False)
    return qf.load_library()


def test_header_symbols_are_exported(lib):
    with open(os.path.join(ROOT, "include", "qflash.h")) as f:
        header = f.read()
    declared = set(re.findall(r"\b(qflash_[a-z_]+)\s*\(", header))
    assert declared == set(EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror(lib):
    assert qf.qflash_strerror(0) == "success"
    for code in qf.ERR.values():
        assert "unknown" not in qf.qflash_strerror(code)
    assert "unknown" in qf.qflash_strerror(-99)


def test_params_agree_with_oracle_on_random_scales(lib):
    """Two independent derivations (C++ in the library, Python in the oracle) give the same integers."""
    rng = np.random.default_rng(2024)
    n_ok = 0
    for _ in range(10000):
        sQ = float(10 ** rng.uniform(-2.3, 1.0))
        sK = float(10 ** rng.uniform(-2.3, 1.0))
        d = int(rng.choice([32, 64]))
        try:
            po = oracle.derive_params(sQ, sK, d)
        except ValueError:
            with pytest.raises(qf.QFlashError):
                qf.qflash_params_from_scales(sQ, sK, 1.0, d)
            continue
        pl = qf.qflash_params_from_scales(sQ, sK, 1.0, d)
        assert pl.astuple() == po.astuple(), (sQ, sK, d)
        n_ok += 1
    assert n_ok > 5000


def test_params_from_scales_errors(lib):
    p = QFlashParams()
    f = lib.qflash_params_from_scales
    assert f(0.1, 0.1, 0.1, 64, None) == qf.ERR["NULL"]
    assert f(0.1, 0.1, 0.1, 48, ctypes.byref(p)) == qf.ERR["SHAPE"]
    assert f(0.0, 0.1, 0.1, 64, ctypes.byref(p)) == qf.ERR["PARAM"]
    assert f(float("nan"), 0.1, 0.1, 64, ctypes.byref(p)) == qf.ERR["PARAM"]
    assert f(0.1, float("inf"), 0.1, 64, ctypes.byref(p)) == qf.ERR["PARAM"]
    assert f(1e-4, 1e-4, 0.1, 64, ctypes.byref(p)) == qf.ERR["PARAM"]
    assert f(3000.0, 3000.0, 0.1, 64, ctypes.byref(p)) == qf.ERR["PARAM"]


def test_context_errors_without_gpu(lib):
    assert lib.qflash_create(None, 0) == qf.ERR["NULL"]
    assert lib.qflash_destroy(None) == 0
    bogus = ctypes.c_void_p(0x1234)
    assert lib.qflash_destroy(bogus) == qf.ERR["CTX"]
    p = qf.qflash_params_from_scales(0.04, 0.04, 0.04, 64)
    one = ctypes.c_void_p(16)
    assert lib.qflash_attention(None, one, one, one, one, None, 0, 0, 1, 1, 1, 64, 64,
                                ctypes.byref(p), None) == qf.ERR["NULL"]
    assert lib.qflash_attention(bogus, one, one, one, one, None, 0, 0, 1, 1, 1, 64, 64,
                                ctypes.byref(p), None) == qf.ERR["CTX"]
    assert lib.qflash_attention_per_head(None, one, one, one, one, None, 0, 0, 1, 1, 1, 64, 64,
                                         ctypes.byref(p), None) == qf.ERR["NULL"]
    assert lib.qflash_attention_per_head(bogus, one, one, one, one, None, 0, 0, 1, 1, 1, 64, 64,
                                         ctypes.byref(p), None) == qf.ERR["CTX"]
    assert lib.qflash_attention_packed_bias(None, one, one, one, one, one, 1, 1, 1, 1, 1, 64, 64,
                                            ctypes.byref(p), 1, None) == qf.ERR["NULL"]
    assert lib.qflash_attention_packed_bias(bogus, one, one, one, one, one, 1, 1, 1, 1, 1, 64, 64,
                                            ctypes.byref(p), 1, None) == qf.ERR["CTX"]
    assert lib.qflash_pack_bias(None, one, 1, 1, 1, one, 4096, None) == qf.ERR["NULL"]
    assert lib.qflash_pack_bias(bogus, one, 1, 1, 1, one, 4096, None) == qf.ERR["CTX"]
    # size of the packed bias: ceil(N/32)^2 blocks of 4 KiB per matrix; 0 for unsupported extents
    assert lib.qflash_packed_bias_bytes(64, 3, 49) == 64 * 3 * 4 * 4096
    assert lib.qflash_packed_bias_bytes(1, 1, 197) == 49 * 4096
    assert lib.qflash_packed_bias_bytes(1, 1, 0) == 0
    assert lib.qflash_packed_bias_bytes(1 << 20, 1 << 10, 64) == 0
    h = ctypes.c_void_p()
    rc = lib.qflash_create(ctypes.byref(h), 9999)
    assert rc == qf.ERR["DEVICE"] and not h.value
    assert lib.qflash_configure(None, qf.CFG_EXP_TABLE, 1) == qf.ERR["NULL"]
    assert lib.qflash_configure(bogus, qf.CFG_EXP_TABLE, 1) == qf.ERR["CTX"]
