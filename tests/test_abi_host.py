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
from paper_2604_25306_amd.binding import EXPORTS, PEAKS_EXPORTS, QFlashParams

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
    # the measurement kernels of the benchmark have a header of their own
    with open(os.path.join(ROOT, "include", "qflash_peaks.h")) as f:
        declared = set(re.findall(r"\b(qflash_peaks_[a-z0-9_]+)\s*\(", f.read()))
    assert declared == set(PEAKS_EXPORTS)
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
        if po.x_shift > 13:       # the oracle covers the whole range of the method, the library stops at k = 13
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


def _units_taken(plan):
    return [qf.qflash_plan_unit(plan, wg) for wg in range(plan.workgroups)]


def test_plan_covers_every_unit_exactly_once(lib):
    """Whatever the decomposition, the workgroups of a launch take every unit of work exactly once
    (idle workgroups report -1): shapes of every kernel family, with and without the bias-period
    placement, whole and partial periods."""
    import numpy as np
    rng = np.random.default_rng(5)
    cases = [(64, 12, 197, 64, 64, 0, 0), (32, 12, 577, 64, 64, 0, 0), (32, 12, 577, 64, 128, 0, 0),
             (16, 16, 577, 64, 64, 0, 0), (4096, 3, 49, 32, 64, 64, 3), (80, 3, 49, 32, 64, 64, 3),
             (20, 2, 197, 64, 64, 8, 2), (16, 1, 300, 64, 128, 8, 1), (8, 1, 1200, 64, 64, 8, 1),
             (1, 1, 4096, 32, 128, 0, 0), (1, 1, 1, 32, 64, 0, 0), (3, 5, 33, 64, 64, 3, 1)]
    for _ in range(60):
        B, H = int(rng.integers(1, 300)), int(rng.integers(1, 25))
        N = int(rng.choice([rng.integers(1, 65), rng.integers(65, 400), rng.integers(400, 4097)]))
        d, tile = int(rng.choice([32, 64])), int(rng.choice([64, 128]))
        if B * H * N * d >= 1 << 31:
            continue
        bB, bH = (0, 0) if rng.integers(0, 2) else (int(rng.choice([1, 2, 8, 16, 64, B])), int(rng.choice([1, H])))
        cases.append((B, H, N, d, tile, bB, bH))
    for c in cases:
        plan = qf.qflash_plan_query(None, *c)
        taken = [u for u in _units_taken(plan) if u >= 0]
        assert sorted(taken) == list(range(plan.units)), c
        pairs = c[0] * c[1]
        if plan.kernel == 3:        # one workgroup per compute unit, several whole pairs each
            assert plan.units == plan.workgroups == -(-pairs // plan.pairs_per_workgroup) <= 256, c
            assert c[3] == 64 and c[4] == 64 and c[2] <= 256 and c[5] == 0, c
            assert 1 <= plan.wavefronts_per_pair <= 16 and plan.query_blocks * 32 >= c[2], c
            continue
        if plan.kernel == 4:        # windowed attention: persistent workgroups, runs of pairs per wavefront pair
            assert plan.units == plan.workgroups <= 256 and plan.workgroups * plan.pairs_per_workgroup >= pairs, c
            assert c[3] == 32 and 32 < c[2] <= 64 and plan.wavefronts_per_pair == 2, c
            assert c[5] == 0 or (c[0] % c[5] == 0 and c[1] % c[6] == 0), c
            continue
        assert plan.workgroups % 8 == 0 and plan.workgroups >= plan.units, c
        assert plan.bias_period_units % 8 == 0, c
        pairs = c[0] * c[1]
        if plan.pairs_per_workgroup > 1:
            assert plan.query_blocks == 1 and plan.units == -(-pairs // plan.pairs_per_workgroup), c
        else:
            assert plan.units == pairs * plan.query_blocks, c
            assert plan.query_blocks * plan.wavefronts_per_pair * 32 >= c[2], c     # every query row has a lane
    assert qf.qflash_plan_unit(plan, -1) == -1 and qf.qflash_plan_unit(plan, plan.workgroups) == -1


def test_plan_of_the_benchmark_shapes(lib):
    """The decompositions the measured figures belong to."""
    p = qf.qflash_plan_query(None, 64, 12, 197, 64, 64)       # three pairs per compute unit, 16 wavefronts
    assert (p.kernel, p.pairs_per_workgroup, p.wavefronts_per_pair, p.units, p.query_blocks) == (3, 3, 16, 256, 7)
    p = qf.qflash_plan_query(None, 1024, 6, 197, 64, 64)     # too many pairs for one round: a workgroup per pair
    assert (p.kernel, p.wavefronts_per_pair, p.units, p.tile_by_tile) == (1, 7, 6144, 1)
    p = qf.qflash_plan_query(None, 32, 12, 577, 64, 64)        # two-tile ring fed by direct loads: 4 wavefronts per workgroup
    assert (p.kernel, p.wavefronts_per_pair, p.query_blocks) == (2, 4, 5)
    p = qf.qflash_plan_query(None, 16, 16, 577, 64, 128)
    assert (p.kernel, p.wavefronts_per_pair, p.query_blocks) == (2, 4, 5)
    p = qf.qflash_plan_query(None, 16, 16, 577, 64, 64, 16, 16)  # with a bias: the ring staged by the wavefronts; same turns
    assert (p.kernel, p.wavefronts_per_pair, p.query_blocks) == (2, 7, 3)   # either way, so the larger workgroup
    p = qf.qflash_plan_query(None, 4, 4, 300, 64, 64)          # every long sequence without a bias takes the ring
    assert (p.kernel, p.wavefronts_per_pair, p.query_blocks) == (2, 4, 3)
    p = qf.qflash_plan_query(None, 4096, 3, 49, 32, 64, 64, 3)  # windowed: 256 persistent workgroups, 8 runs of 6 pairs each
    assert (p.kernel, p.pairs_per_workgroup, p.wavefronts_per_pair, p.workgroups) == (4, 48, 2, 256)
    p = qf.qflash_plan_query(None, 4097, 3, 49, 32, 64, 64, 3)  # the bias extents do not divide the batch: the resident kernel,
    assert (p.kernel, p.pairs_per_workgroup, p.wavefronts_per_pair, p.bias_period_units) == (1, 4, 2, 48)   # four windows per workgroup
    # XCD x = workgroup % 8 only ever meets an eighth of the bias slices
    for x in range(8):
        slices = {(qf.qflash_plan_unit(p, wg) * 4 + s) % 192 for wg in range(x, p.workgroups, 8) for s in range(4)
                  if qf.qflash_plan_unit(p, wg) >= 0}
        assert len(slices) == 24, x
    p = qf.qflash_plan_query(None, 1, 1, 4096, 32, 64)           # too long for LDS at d = 32: streamed
    assert p.kernel == 0
    assert lib.qflash_plan_query(None, 1, 1, 64, 64, 64, 0, 0, None) == qf.ERR["NULL"]
    info = qf.PlanInfo()
    assert lib.qflash_plan_query(None, 1, 1, 64, 48, 64, 0, 0, ctypes.byref(info)) == qf.ERR["SHAPE"]
    assert lib.qflash_plan_query(None, 1, 1, 64, 64, 96, 0, 0, ctypes.byref(info)) == qf.ERR["TILE"]
    assert lib.qflash_plan_query(ctypes.c_void_p(0x1234), 1, 1, 64, 64, 64, 0, 0, ctypes.byref(info)) == qf.ERR["CTX"]
