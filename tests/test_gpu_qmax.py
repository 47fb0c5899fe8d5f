"""GPU parity of the quantised-maximum variant (QFLASH_CFG_QUANTISED_MAX; NOT the paper's Algorithm 1)
against its own oracle, bit for bit, through the C ABI.  Needs an MI355X (``-m gpu``).
"""
import numpy as np
import pytest

import oracle
from oracle.params import OracleParams
from workloads import make_workload, quantize_per_tensor, EXCLUDED

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", params=["table", "arith"])
def gpu(request):
    import torch
    import paper_2604_25306_amd as qf
    assert torch.cuda.is_available(), "these tests need a GPU"
    qf.load_library()
    ctx = qf.Context(0)
    ctx.configure(qf.CFG_EXP_TABLE, 1 if request.param == "table" else 0)
    ctx.configure(qf.CFG_QUANTISED_MAX, 1)
    yield torch, qf, ctx
    ctx.close()


def run_gpu(gpu, Q, K, V, p, tile, bias=None, packed=False):
    torch, qf, ctx = gpu
    dev = torch.device("cuda:0")
    tQ, tK, tV = (torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (Q, K, V))
    tO = torch.full(Q.shape, 0x55, dtype=torch.int8, device=dev)
    tB = torch.from_numpy(np.ascontiguousarray(bias)).to(dev) if bias is not None else None
    lp = qf.QFlashParams(*p.astuple()) if isinstance(p, OracleParams) else [qf.QFlashParams(*x.astuple()) for x in p]
    if packed:
        tP = ctx.pack_bias(tB)
        ctx.attention_packed_bias(tQ, tK, tV, tO, lp, tile, tP, bias.shape[0], bias.shape[1])
    else:
        ctx.attention(tQ, tK, tV, tO, lp, tile, bias=tB)
    torch.cuda.synchronize()
    return tO.cpu().numpy()


def assert_same(out, ref, label):
    bad = np.argwhere(out != ref)
    assert bad.size == 0, "%s: %d mismatches, first at %s: gpu %d oracle %d" % (
        label, len(bad), bad[0], out[tuple(bad[0])], ref[tuple(bad[0])])


def check(gpu, Q, K, V, p, tile, bias=None, label=""):
    print("qmax case", label, Q.shape, "tile", tile, "bias", bias is not None, flush=True)
    ref = oracle.qflash_attention_qmax(Q, K, V, p, tile, bias=bias)
    assert_same(run_gpu(gpu, Q, K, V, p, tile, bias=bias), ref, label)
    if bias is not None:
        assert_same(run_gpu(gpu, Q, K, V, p, tile, bias=bias, packed=True), ref, label + " (packed bias)")


def rand_case(shape, seed, sigma=1.0, q_gain=1.0):
    rng = np.random.default_rng(seed)
    Qf = rng.standard_normal(shape).astype(np.float32) * np.float32(sigma * q_gain)
    Kf = rng.standard_normal(shape).astype(np.float32) * np.float32(sigma)
    Vf = rng.standard_normal(shape).astype(np.float32)
    (Q, sQ), (K, sK), (V, sV) = (quantize_per_tensor(x) for x in (Qf, Kf, Vf))
    return Q, K, V, sQ, sK, sV


# resident (all at once, tile by tile, two-tile ring) and streamed kernels, both tile sizes, ragged tails
SHAPES = [
    ((1, 1, 1, 64), 64), ((1, 2, 5, 32), 64), ((2, 2, 31, 64), 64), ((1, 2, 33, 32), 64), ((1, 2, 65, 64), 64),
    ((1, 3, 127, 32), 64), ((1, 2, 129, 64), 128), ((2, 3, 197, 64), 64), ((1, 2, 197, 64), 128),
    ((1, 2, 200, 32), 128), ((1, 2, 257, 64), 64), ((1, 2, 300, 32), 64), ((1, 1, 577, 64), 64),
    ((1, 1, 577, 64), 128), ((1, 1, 1030, 64), 64), ((3, 5, 49, 32), 64), ((1, 2, 256, 64), 64),
    ((1, 1, 2100, 32), 64), ((1, 1, 4096, 64), 128), ((64, 12, 197, 64), 64),
]


@pytest.mark.parametrize("idx", range(len(SHAPES)))
def test_random_shapes(gpu, idx):
    shape, tile = SHAPES[idx]
    Q, K, V, sQ, sK, _ = rand_case(shape, 900 + idx, q_gain=1.5 if shape[2] < 2000 else 1.0)
    p = oracle.derive_params(sQ, sK, shape[-1])
    assert p.x_shift == 0
    check(gpu, Q, K, V, p, tile, label="random")


@pytest.mark.parametrize("order", ["up", "down"])
def test_levels_that_move_in_every_tile_or_never(gpu, order):
    """Keys sorted so that the row maximum keeps rising (the level moves by one or more octaves in
    most tiles) or falls (settled in the first tile: later tiles skip the rescale altogether)."""
    shape = (1, 2, 330, 64)
    rng = np.random.default_rng(3)
    Qf = np.abs(rng.standard_normal(shape)).astype(np.float32) * 2.5
    Kf = np.abs(rng.standard_normal(shape)).astype(np.float32)
    ramp = np.linspace(0.1, 1.0, shape[2], dtype=np.float32)[None, None, :, None]
    Kf = Kf * (ramp if order == "up" else ramp[:, :, ::-1])
    Vf = rng.standard_normal(shape).astype(np.float32)
    (Q, sQ), (K, sK), (V, _) = (quantize_per_tensor(x) for x in (Qf, Kf, Vf))
    p = oracle.derive_params(sQ, sK, 64)
    for tile in (64, 128):
        check(gpu, Q, K, V, p, tile, label="levels " + order)


def test_extreme_values_and_large_level_jumps(gpu):
    rng = np.random.default_rng(1)
    shape = (1, 2, 197, 64)
    p = oracle.derive_params(0.04, 0.04, 64)
    Q = rng.integers(-127, 128, size=shape).astype(np.int8)
    V = rng.integers(-128, 128, size=shape).astype(np.int8)
    check(gpu, Q, np.zeros(shape, np.int8), V, p, 64, label="K=0")
    for qv, kv, vv in ((127, 127, 127), (127, -127, -128), (-128, -128, -128)):
        check(gpu, np.full(shape, qv, np.int8), np.full(shape, kv, np.int8), np.full(shape, vv, np.int8), p, 64,
              label="const %d %d %d" % (qv, kv, vv))
    # a huge score late in the sequence: the level jumps by hundreds of octaves at once (every
    # earlier contribution is shifted out), with fine and with coarse octaves
    Q, K, V, sQ, sK, _ = rand_case((1, 2, 260, 64), 5, q_gain=2.0)
    K2 = K.copy()
    K2[:, :, 200] = np.sign(Q[:, :, 7]) * 127
    for s_inv in (1024, 3000, 200000):
        pm, ps = oracle.params.requant_constants(s_inv)
        pp = OracleParams(0, s_inv, -round(2 ** 32 / s_inv), 32, pm, ps, -((-(1 << 30)) // s_inv), 0)
        check(gpu, Q, K2, V, pp, 64, label="late outlier s_inv=%d" % s_inv)
    # most negative numerators through the shifts
    shape = (1, 1, 512, 64)
    check(gpu, np.zeros(shape, np.int8), np.zeros(shape, np.int8), np.full(shape, -128, np.int8), p, 64, label="max |O|")


def test_bias_exclusion_and_windows(gpu):
    shape = (3, 2, 100, 64)
    Q, K, V, sQ, sK, _ = rand_case(shape, 8)
    p = oracle.derive_params(sQ, sK, 64)
    rng = np.random.default_rng(4)
    bias = rng.integers(-3000, 3000, size=(3, 1, 100, 100)).astype(np.int32)
    bias[rng.random(bias.shape) < 0.2] = EXCLUDED
    bias[1, 0, 5, :] = EXCLUDED                        # a fully excluded row
    bias[2, 0, :, 64:] = EXCLUDED                      # a fully excluded tile
    check(gpu, Q, K, V, p, 64, bias=bias, label="bias + exclusion")
    w = make_workload("swin_t_s1_b64", batch=2)
    B, H, N, d = w.shape
    check(gpu, w.Q, w.K, w.V, oracle.derive_params(w.sQ, w.sK, d), 64, bias=w.bias, label="windows")


@pytest.mark.parametrize("out_round", [0, 1])
def test_out_round_and_per_head(gpu, out_round):
    shape = (2, 3, 150, 64)
    Q, K, V, sQ, sK, _ = rand_case(shape, 77)
    ps = [oracle.derive_params(sQ * g, sK, 64, out_round=out_round) for g in (1.0, 0.6, 1.7)]
    check(gpu, Q, K, V, ps[0], 64, label="out_round=%d" % out_round)
    check(gpu, Q, K, V, ps, 64, label="per head, out_round=%d" % out_round)


@pytest.mark.parametrize("name,tile", [("deit_b384_b32", 64), ("deit_b384_b32", 128), ("swin_t_s1_b64", 64)])
def test_benchmark_workloads_full_size(gpu, name, tile):
    w = make_workload(name)
    B, H, N, d = w.shape
    p = oracle.derive_params(w.sQ, w.sK, d)
    print("qmax workload", name, tile, flush=True)
    ref = oracle.qflash_attention_qmax(w.Q, w.K, w.V, p, tile, bias=w.bias)
    assert_same(run_gpu(gpu, w.Q, w.K, w.V, p, tile, bias=w.bias, packed=w.bias is not None), ref, name)


def test_variant_differs_from_algorithm_1_and_is_refused_where_unsupported(gpu):
    torch, qf, ctx = gpu
    Q, K, V, sQ, sK, _ = rand_case((1, 2, 197, 64), 2, q_gain=1.5)
    p = oracle.derive_params(sQ, sK, 64)
    out = run_gpu(gpu, Q, K, V, p, 64)
    assert not np.array_equal(out, oracle.qflash_attention(Q, K, V, p, 64))       # it is another function
    info = qf.qflash_plan_query(ctx.handle, 1, 2, 197, 64, 64)
    assert info.kernel != 3                      # the whole-compute-unit kernel is Algorithm 1 only
    # coarse scales (x_shift > 0) are refused, and so are the entry points that do not offer the variant
    pc = oracle.derive_params(sQ * 40, sK * 40, 64)
    assert pc.x_shift > 0
    dev = torch.device("cuda:0")
    t = [torch.from_numpy(x).to(dev) for x in (Q, K, V)]
    o = torch.zeros(Q.shape, dtype=torch.int8, device=dev)
    with pytest.raises(qf.QFlashError) as e:
        ctx.attention(*t, o, qf.QFlashParams(*pc.astuple()), 64)
    assert e.value.code == qf.ERR["PARAM"]
    with pytest.raises(qf.QFlashError) as e:
        ctx.attention_static(*t, o, qf.QFlashParams(*p.astuple()), 64)
    assert e.value.code == qf.ERR["PARAM"]
    # switching the variant off again restores Algorithm 1 on the same context
    ctx.configure(qf.CFG_QUANTISED_MAX, 0)
    try:
        ctx.attention(*t, o, qf.QFlashParams(*p.astuple()), 64)
        torch.cuda.synchronize()
        assert np.array_equal(o.cpu().numpy(), oracle.qflash_attention(Q, K, V, p, 64))
    finally:
        ctx.configure(qf.CFG_QUANTISED_MAX, 1)
