"""GPU parity: the HIP library behind the C ABI must reproduce the CPU oracle bit for bit.

All tests here need an MI355X (``-m gpu``).  Inputs are seeded and synthetic; expected values come
from the oracle run in the same process.  Integer work: the bar is exact equality of every byte.
"""
import ctypes

import numpy as np
import pytest

import oracle
from oracle.params import OracleParams
from workloads import make_workload, quantize_per_tensor, EXCLUDED

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", params=["table", "arith"])
def gpu(request):
    """Every parity case runs twice: with the LDS weight table allowed (the default; the library
    still computes arithmetically where no table fits) and with it switched off."""
    import torch
    import paper_2604_25306_amd as qf
    assert torch.cuda.is_available(), "these tests need a GPU"
    qf.load_library()                      # raises if the HIP library has not been built
    ctx = qf.Context(0)
    ctx.configure(qf.CFG_EXP_TABLE, 1 if request.param == "table" else 0)
    yield torch, qf, ctx
    ctx.close()


def lib_params(qf, p: OracleParams):
    return qf.QFlashParams(*p.astuple())


def run_gpu(gpu, Q, K, V, p, tile, bias=None, stream=None, packed=False):
    """p: one OracleParams or a list of H.  packed: hand the bias over in the lane-major layout."""
    torch, qf, ctx = gpu
    dev = torch.device("cuda:0")
    tQ, tK, tV = (torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (Q, K, V))
    tO = torch.full(Q.shape, 0x55, dtype=torch.int8, device=dev)
    tB = torch.from_numpy(np.ascontiguousarray(bias)).to(dev) if bias is not None else None
    lp = lib_params(qf, p) if isinstance(p, OracleParams) else [lib_params(qf, x) for x in p]
    if packed:
        tP = ctx.pack_bias(tB, stream=stream)
        ctx.attention_packed_bias(tQ, tK, tV, tO, lp, tile, tP, bias.shape[0], bias.shape[1], stream=stream)
    else:
        ctx.attention(tQ, tK, tV, tO, lp, tile, bias=tB, stream=stream)
    torch.cuda.synchronize()
    return tO.cpu().numpy()


def assert_same(out, ref, label):
    bad = np.argwhere(out != ref)
    assert bad.size == 0, "%s: %d mismatches, first at %s: gpu %d oracle %d" % (
        label, len(bad), bad[0], out[tuple(bad[0])], ref[tuple(bad[0])])


def check(gpu, Q, K, V, p, tile, bias=None, label=""):
    """Every case with a bias runs twice on the GPU: plain bias, and the same bias packed."""
    print("case", label, Q.shape, "tile", tile, "bias", bias is not None, flush=True)
    ref = oracle.qflash_attention(Q, K, V, p, tile, bias=bias)
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


# ------------------------------------------------ shapes: several tiles, ragged tails, extremes

SHAPES = [
    ((1, 1, 1, 64), 64), ((1, 2, 5, 32), 64), ((2, 2, 31, 64), 64), ((1, 2, 32, 64), 64),
    ((1, 2, 33, 32), 64), ((2, 1, 64, 64), 64), ((1, 2, 65, 64), 64), ((1, 3, 127, 32), 64),
    ((1, 2, 128, 64), 128), ((1, 2, 129, 64), 128), ((2, 3, 197, 64), 64), ((1, 2, 197, 64), 128),
    ((1, 2, 200, 32), 128), ((1, 2, 257, 64), 64), ((1, 2, 300, 32), 64), ((1, 1, 577, 64), 64),
    ((1, 1, 577, 64), 128), ((1, 1, 1030, 64), 64), ((3, 5, 49, 32), 64), ((3, 5, 49, 32), 128),
    # tile-by-tile staging: the fewest wavefronts that allow it, full tiles only, one odd row
    ((1, 2, 100, 64), 64), ((1, 2, 128, 64), 64), ((2, 2, 160, 64), 64), ((1, 2, 256, 64), 64),
    ((1, 2, 193, 64), 64), ((1, 2, 384, 64), 128), ((1, 1, 640, 64), 64),
]


@pytest.mark.parametrize("idx", range(len(SHAPES)))
def test_random_shapes(gpu, idx):
    shape, tile = SHAPES[idx]
    Q, K, V, sQ, sK, _ = rand_case(shape, 500 + idx, q_gain=1.5)
    p = oracle.derive_params(sQ, sK, shape[-1])
    check(gpu, Q, K, V, p, tile, label="random")


@pytest.mark.parametrize("out_round", [0, 1])
def test_out_round(gpu, out_round):
    Q, K, V, sQ, sK, _ = rand_case((2, 2, 150, 64), 77)
    p = oracle.derive_params(sQ, sK, 64, out_round=out_round)
    check(gpu, Q, K, V, p, 64, label="out_round=%d" % out_round)


def test_max_n(gpu):
    Q, K, V, sQ, sK, _ = rand_case((1, 1, 4096, 64), 4096)
    p = oracle.derive_params(sQ, sK, 64)
    check(gpu, Q, K, V, p, 128, label="N=4096")


# ------------------------------------------------------------------------- adversarial values


def test_uniform_scores_and_extreme_values(gpu):
    rng = np.random.default_rng(1)
    shape = (1, 2, 197, 64)
    p = oracle.derive_params(0.04, 0.04, 64)
    Q = rng.integers(-127, 128, size=shape).astype(np.int8)
    V = rng.integers(-128, 128, size=shape).astype(np.int8)
    check(gpu, Q, np.zeros(shape, np.int8), V, p, 64, label="K=0")
    for qv, kv, vv in ((127, 127, 127), (127, -127, -128), (-128, -128, -128), (-128, 127, 127)):
        check(gpu, np.full(shape, qv, np.int8), np.full(shape, kv, np.int8),
              np.full(shape, vv, np.int8), p, 64, label="const %d %d %d" % (qv, kv, vv))
    signs = rng.choice(np.array([-127, 127], dtype=np.int8), size=(3,) + shape)
    check(gpu, signs[0], signs[1], signs[2], p, 64, label="all +-127")
    # worst case for the accumulators at the largest N the 24-bit paths must carry
    shape = (1, 1, 512, 64)
    check(gpu, np.zeros(shape, np.int8), np.zeros(shape, np.int8), np.full(shape, -128, np.int8),
          p, 64, label="max |O| N=512")
    shape = (1, 1, 4096, 32)
    check(gpu, np.zeros(shape, np.int8), np.zeros(shape, np.int8), np.full(shape, -128, np.int8),
          oracle.derive_params(0.04, 0.04, 32), 128, label="max |O| N=4096")


def test_outliers_and_sorted_maxima(gpu):
    Q, K, V, sQ, sK, _ = rand_case((1, 2, 260, 64), 5, q_gain=2.0)
    p = oracle.derive_params(sQ, sK, 64)
    K2 = K.copy()
    K2[:, :, 200] = np.sign(Q[:, :, 7]) * 127            # one huge score late in the sequence
    check(gpu, Q, K2, V, p, 64, label="late outlier")
    Qp = np.clip(Q[:, :, :1].astype(np.int64) + np.random.default_rng(2).integers(-3, 4, Q.shape),
                 -127, 127).astype(np.int8)
    s0 = Qp[0, 0, 0].astype(np.int64) @ K[0, 0].astype(np.int64).T
    for name, perm in (("ascending", np.argsort(s0)), ("descending", np.argsort(-s0))):
        check(gpu, Qp, K[:, :, perm], V[:, :, perm], p, 64, label=name)


def test_coarse_and_fine_scales(gpu):
    """x_shift > 0 (coarse scores) and the largest supported s_inv."""
    rng = np.random.default_rng(8)
    shape = (1, 2, 150, 64)
    Q = rng.integers(-127, 128, size=shape).astype(np.int8)
    K = rng.integers(-127, 128, size=shape).astype(np.int8)
    V = rng.integers(-127, 128, size=shape).astype(np.int8)
    for sQ, sK in ((3.0, 4.0), (0.9, 1.1), (6.0, 7.0), (0.0048, 0.0048), (0.2, 0.2)):
        p = oracle.derive_params(sQ, sK, 64)
        check(gpu, Q, K, V, p, 64, label="scales %g %g k=%d s_inv=%d" % (sQ, sK, p.x_shift, p.s_inv))
    # scaling identity on the GPU as well: forced x_shift
    base = oracle.derive_params(0.02, 0.02, 64)
    Ks = rng.integers(-15, 16, size=shape).astype(np.int8)
    check(gpu, Q, Ks, V, OracleParams(3, *base.astuple()[1:]), 64, label="forced k=3")


# ------------------------------------------------------------------------------ bias and mask


def packed_layout(bias):
    """The packed layout as the header defines it, element by element (NumPy indexing only)."""
    bB, bH, N, _ = bias.shape
    R = (N + 31) // 32
    s, rb, cb, a, l, b = np.meshgrid(np.arange(bB * bH), np.arange(R), np.arange(R), np.arange(4),
                                     np.arange(64), np.arange(4), indexing="ij")
    row = np.minimum(32 * rb + l % 32, N - 1)
    col = 32 * cb + 8 * a + 4 * (l // 32) + b
    flat = bias.reshape(bB * bH, N, N)
    return np.where(col < N, flat[s, row, np.minimum(col, N - 1)], np.int32(EXCLUDED)).astype(np.int32)


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 3, 49, 49), (1, 2, 64, 64), (3, 1, 197, 197), (1, 1, 577, 577)])
def test_pack_bias_layout(gpu, shape):
    torch, qf, ctx = gpu
    rng = np.random.default_rng(shape[2])
    bias = rng.integers(-(1 << 30), 1 << 30, size=shape).astype(np.int32)
    want = packed_layout(bias)
    assert qf.qflash_packed_bias_bytes(*shape[:3]) == want.size * 4
    got = ctx.pack_bias(torch.from_numpy(bias).to("cuda:0"))
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), want.ravel())



def test_bias_and_exclusion(gpu):
    Q, K, V, sQ, sK, _ = rand_case((4, 3, 49, 32), 43, q_gain=1.5)
    p = oracle.derive_params(sQ, sK, 32)
    rng = np.random.default_rng(3)
    bias = rng.integers(-20000, 20000, size=(2, 3, 49, 49)).astype(np.int32)
    check(gpu, Q, K, V, p, 64, bias=bias, label="bias [2,3]")
    check(gpu, Q, K, V, p, 64, bias=bias[:1, :1], label="bias [1,1]")
    mask = rng.random((2, 3, 49, 49)) < 0.3
    bias_m = np.where(mask, np.int32(EXCLUDED), bias)
    bias_m[0, 0, 5, :] = EXCLUDED                      # a row with nothing to attend to
    check(gpu, Q, K, V, p, 64, bias=bias_m, label="bias + mask")
    # several tiles, d = 64, whole tiles excluded for some rows
    Q, K, V, sQ, sK, _ = rand_case((2, 2, 200, 64), 44)
    p = oracle.derive_params(sQ, sK, 64)
    bias = rng.integers(-3000, 3000, size=(1, 2, 200, 200)).astype(np.int32)
    bias[0, 0, 10, :64] = EXCLUDED
    bias[0, 0, 11, 64:128] = EXCLUDED
    bias[0, 1, 12, :192] = EXCLUDED
    bias[0, 1, 13, :] = EXCLUDED
    bias[0, :, :, 199] = EXCLUDED
    for tile in (64, 128):
        check(gpu, Q, K, V, p, tile, bias=bias, label="multi-tile mask")


# -------------------------------------------- the five benchmark workloads at their full size


@pytest.mark.parametrize("name", ["deit_tiny_b1", "vit_b16_b64", "deit_b384_b32", "swin_t_s1_b64",
                                  "vit_l384_heavy"])
def test_benchmark_workloads_full_size(gpu, name):
    """Same launch configuration as bench.py; every output byte is compared (the oracle needs a few
    seconds per workload on the host cores)."""
    wl = make_workload(name)
    p = oracle.derive_params(wl.sQ, wl.sK, wl.shape[-1])
    if name == "vit_l384_heavy":
        assert p.x_shift > 0
    for tile in wl.kv_tiles:
        check(gpu, wl.Q, wl.K, wl.V, p, tile, bias=wl.bias, label=name)


# ------------------------------- the paper's own workload table at batch 1 and 8 (small launches)


from workloads import TABLE1_CONFIGS  # noqa: E402


@pytest.mark.parametrize("name", TABLE1_CONFIGS)
def test_table1_workloads(gpu, name):
    """Table 1 (A1-A7) at batch 1 and 8: few workgroups, windowed ones with relative-position bias
    and shifted-window exclusion, several windows per workgroup."""
    wl = make_workload(name)
    p = oracle.derive_params(wl.sQ, wl.sK, wl.shape[-1])
    for tile in wl.kv_tiles:
        check(gpu, wl.Q, wl.K, wl.V, p, tile, bias=wl.bias, label=name)


@pytest.mark.parametrize("shape,bias_bh,tile", [
    ((80, 3, 49, 32), (64, 3), 64),      # four windows per workgroup, 1.25 bias periods
    ((128, 3, 49, 32), (64, 3), 64),     # whole periods
    ((20, 2, 197, 64), (8, 2), 64),      # one pair per workgroup, 2.5 periods
    ((16, 1, 300, 64), (8, 1), 128),     # two query tiles per pair
    ((8, 1, 1200, 64), (8, 1), 64),      # streamed kernel
    # last tile more than half full: with a packed bias it runs as a full tile
    ((4, 2, 120, 64), (1, 2), 64), ((2, 2, 250, 32), (2, 1), 64), ((2, 2, 230, 64), (1, 1), 128),
    ((3, 2, 33, 32), (1, 1), 64), ((3, 2, 97, 32), (3, 2), 128),
])
def test_bias_period_mapping(gpu, shape, bias_bh, tile):
    """Launches whose bias repeats every 8k units of work take the bias-aware placement of
    workgroups; the result must not depend on placement."""
    B, H, N, d = shape
    Q, K, V, sQ, sK, _ = rand_case(shape, 300 + N)
    p = oracle.derive_params(sQ, sK, d)
    rng = np.random.default_rng(N)
    bias = rng.integers(-4000, 4000, size=bias_bh + (N, N)).astype(np.int32)
    bias[rng.random(bias.shape) < 0.1] = EXCLUDED
    check(gpu, Q, K, V, p, tile, bias=bias, label="bias period %s" % (bias_bh,))


@pytest.mark.parametrize("shape,with_bias", [
    ((2, 3, 331, 64), False),    # shortest sequences that keep two KV tiles in LDS: ragged last tile
    ((1, 2, 353, 64), True),     # one row into a new row block; bias, plain and packed
    ((3, 2, 384, 64), False),    # whole tiles only
    ((40, 13, 400, 64), False),  # enough pairs for the 4-wavefront workgroups
    ((1, 2, 640, 64), True),
    ((1, 2, 1089, 64), False),   # beyond what fits LDS as a whole
    ((1, 1, 2500, 64), False),
    ((2, 2, 257, 64), True),     # shortest sequence of the kv_tile 128 ring: 2 tiles, the second one row
    ((2, 2, 300, 64), False),
])
@pytest.mark.parametrize("tile", [64, 128])
def test_two_tile_ring(gpu, shape, with_bias, tile):
    """d = 64 and N > 330 or so (kv_tile 64) or N > 256 (kv_tile 128): the kernel keeps two KV tiles
    in LDS and reuses the slots; with kv_tile 128 every staging thread carries two items."""
    B, H, N, d = shape
    Q, K, V, sQ, sK, _ = rand_case(shape, 700 + N, q_gain=1.3)
    p = oracle.derive_params(sQ, sK, d)
    bias = None
    if with_bias:
        rng = np.random.default_rng(N)
        bias = rng.integers(-3000, 3000, size=(1, H, N, N)).astype(np.int32)
        bias[rng.random(bias.shape) < 0.2] = EXCLUDED
        bias[0, 0, 7, :] = EXCLUDED
    check(gpu, Q, K, V, p, tile, bias=bias, label="ring")


# (batch, heads, N): several pairs per workgroup, a last workgroup with fewer pairs than the others,
# every number of 8-key groups in the ragged tile, single tiles, a sequence of a single row, sequences
# that end exactly on a 16-row block and on a tile, four pairs per workgroup
WHOLE_CU_SHAPES = [(103, 5, 197), (86, 3, 70), (64, 5, 1), (300, 1, 16), (301, 1, 17), (70, 4, 64), (50, 6, 65),
                   (257, 1, 128), (43, 6, 129), (90, 3, 200), (33, 8, 208), (40, 7, 224), (37, 7, 225), (32, 9, 249),
                   (100, 3, 256), (1, 3, 197), (8, 6, 197), (128, 8, 33), (51, 5, 73), (51, 5, 81), (51, 5, 89),
                   (51, 5, 97), (51, 5, 105), (51, 5, 113), (51, 5, 121),
                   # four pairs per workgroup fit only without the weight table: arithmetic weights, and the
                   # fourth pair has no wavefronts of its own at the start (its loads ride with the third's)
                   (84, 12, 197)]


@pytest.mark.parametrize("bhn", WHOLE_CU_SHAPES)
def test_whole_compute_unit_kernel(gpu, bhn):
    """Short sequences with 64 features, tile 64 and no bias, few enough pairs for one round of
    workgroups: the kernel in which one workgroup per compute unit holds Q, K, V of several pairs in
    LDS (direct loads, per-tile counters, units of 32 query rows handed out dynamically)."""
    torch, qf, ctx = gpu
    B, H, N = bhn
    plan = qf.qflash_plan_query(ctx.handle, B, H, N, 64, 64)       # (the plan assumes a 32 KiB table)
    assert plan.kernel == 3 or B * H > 768, (bhn, plan.kernel)
    Q, K, V, sQ, sK, _ = rand_case((B, H, N, 64), 900 + B + N, q_gain=1.0 + (N % 3) * 0.4)
    p = oracle.derive_params(sQ, sK, 64)
    check(gpu, Q, K, V, p, 64, label="whole CU %s pairs/wg %d" % (bhn, plan.pairs_per_workgroup))
    if N in (197, 70):          # the coarse-score variant (x_shift > 0) and rounding to nearest
        p2 = oracle.derive_params(sQ * 40.0, sK * 40.0, 64, out_round=1)
        assert p2.x_shift > 0
        check(gpu, Q, K, V, p2, 64, label="whole CU, x_shift %d" % p2.x_shift)


# (B, H, N, bias_B, bias_H, tile): runs that end inside a slice, slices that change inside a run, more
# heads than bias heads, one bias for everything, fewer pairs than compute units, no bias at all
WINDOWED_SHAPES = [(4096 // 16, 3, 49, 64, 3, 64), (70, 3, 49, 10, 3, 64), (2315, 1, 49, 5, 1, 64), (36, 6, 49, 12, 2, 128),
                   (1000, 3, 33, 1, 1, 64), (64, 4, 64, 64, 4, 64), (9, 24, 49, 1, 24, 64), (2, 2, 40, 2, 1, 64),
                   (700, 3, 49, 0, 0, 64), (3, 5, 57, 0, 0, 128), (1, 1, 63, 1, 1, 64)]


@pytest.mark.parametrize("shape", WINDOWED_SHAPES)
def test_windowed_kernel(gpu, shape):
    """Windows of 33 to 64 tokens with 32 features: the persistent kernel in which every wavefront
    works through a run of pairs of one bias slice with the bias in registers.  The packed-bias
    call (and the call without a bias) must take it, the plain-bias call the resident kernel; all
    three equal the oracle."""
    torch, qf, ctx = gpu
    B, H, N, bB, bH, tile = shape
    Q, K, V, sQ, sK, _ = rand_case((B, H, N, 32), 1300 + B + N, q_gain=1.0 + (N % 3) * 0.3)
    rng = np.random.default_rng(B + N)
    bias = None
    if bB:
        bias = rng.integers(-2500, 2500, size=(bB, bH, N, N)).astype(np.int32)
        bias[rng.random(bias.shape) < 0.25] = EXCLUDED
        bias[..., 0] = 17                       # every row keeps a key ...
        bias[0, 0, N // 2, :] = EXCLUDED        # ... but one, which is excluded altogether
    for out_round in ((0, 1) if N == 49 and B < 100 else (0,)):
        p = oracle.derive_params(sQ, sK, 32, out_round=out_round)
        ref = oracle.qflash_attention(Q, K, V, p, tile, bias=bias)
        out = run_gpu(gpu, Q, K, V, p, tile, bias=bias, packed=bias is not None)
        assert qf.qflash_cache_query(ctx.handle).last_kernel == 4, shape
        assert_same(out, ref, "windowed %s" % (shape,))
        if bias is not None and B * H <= 1000:
            out = run_gpu(gpu, Q, K, V, p, tile, bias=bias, packed=False)
            assert qf.qflash_cache_query(ctx.handle).last_kernel == 1, shape
            assert_same(out, ref, "windowed, plain bias %s" % (shape,))
    # coarse scores (x_shift > 0): the arithmetic variant with the left shift
    if N in (49, 40):
        p2 = oracle.derive_params(sQ * 40.0, sK * 40.0, 32)
        assert p2.x_shift > 0
        b2 = None if bias is None else np.where(bias == EXCLUDED, bias, bias // 1500).astype(np.int32)
        assert_same(run_gpu(gpu, Q, K, V, p2, tile, bias=b2, packed=b2 is not None),
                    oracle.qflash_attention(Q, K, V, p2, tile, bias=b2), "windowed, x_shift %d" % p2.x_shift)


def test_windowed_kernel_is_not_taken_when_the_bias_does_not_divide_the_batch(gpu):
    torch, qf, ctx = gpu
    Q, K, V, sQ, sK, _ = rand_case((7, 3, 49, 32), 1401)
    p = oracle.derive_params(sQ, sK, 32)
    bias = np.random.default_rng(1).integers(-2000, 2000, size=(2, 3, 49, 49)).astype(np.int32)
    out = run_gpu(gpu, Q, K, V, p, 64, bias=bias, packed=True)
    assert qf.qflash_cache_query(ctx.handle).last_kernel == 1
    assert_same(out, oracle.qflash_attention(Q, K, V, p, 64, bias=bias), "7 images, 2 bias slices")


# long sequences without a bias: the two-tile ring fed by direct loads, both tile sizes, ragged last tiles,
# one to five row blocks in the last workgroup of a pair, fewer than four wavefronts per workgroup
DIRECT_RING_SHAPES = [(2, 3, 257, 64), (3, 2, 288, 128), (1, 5, 320, 64), (2, 2, 383, 128), (1, 3, 449, 64),
                      (4, 12, 577, 64), (4, 12, 577, 128), (1, 2, 640, 64), (1, 1, 1030, 128), (1, 2, 2049, 64),
                      (1, 1, 4096, 64)]


@pytest.mark.parametrize("shape", DIRECT_RING_SHAPES)
def test_direct_load_ring(gpu, shape):
    torch, qf, ctx = gpu
    B, H, N, tile = shape
    plan = qf.qflash_plan_query(ctx.handle, B, H, N, 64, tile)
    assert plan.kernel == 2 and plan.wavefronts_per_pair <= 4, (shape, plan.kernel, plan.wavefronts_per_pair)
    Q, K, V, sQ, sK, _ = rand_case((B, H, N, 64), 1500 + N, sigma=1.0 + (N % 2) * 0.5)
    p = oracle.derive_params(sQ, sK, 64, out_round=N % 2)
    check(gpu, Q, K, V, p, tile, label="direct ring %s" % (shape,))
    if N in (257, 577):
        # per-head constants (tables of different sizes, one head coarse), and a late outlier key
        ps = [oracle.derive_params(sQ * gq, sK, 64) for gq in ([1.0, 0.5, 40.0] + [1.3] * H)[:H]]
        check(gpu, Q, K, V, ps, tile, label="direct ring per head %s" % (shape,))
        K2 = K.copy()
        K2[:, :, N - 3] = np.sign(Q[:, :, 5]) * 127
        check(gpu, Q, K2, V, p, tile, label="direct ring, late outlier %s" % (shape,))


@pytest.mark.parametrize("tile", [64, 128])
def test_streamed_kernel_with_bias(gpu, tile):
    """d = 32 and a sequence too long for LDS: the kernel that streams KV tiles, with a bias in both
    layouts, exclusions across whole tiles and a ragged last tile."""
    shape = (1, 2, 2100, 32)
    assert paper_plan(shape, tile).kernel == 0
    Q, K, V, sQ, sK, _ = rand_case(shape, 2100 + tile)
    p = oracle.derive_params(sQ, sK, 32)
    rng = np.random.default_rng(tile)
    bias = rng.integers(-3000, 3000, size=(1, 2, 2100, 2100)).astype(np.int32)
    bias[rng.random(bias.shape) < 0.05] = EXCLUDED
    bias[0, 0, 17, :1024] = EXCLUDED
    bias[0, 1, 18, :] = EXCLUDED
    check(gpu, Q, K, V, p, tile, bias=bias, label="streamed + bias")
    ps = [p, oracle.derive_params(sQ * 1.7, sK, 32)]
    check_per_head(gpu, Q, K, V, ps, tile, bias=bias, label="streamed + bias, per head")


def paper_plan(shape, tile, bias_bh=(0, 0)):
    import paper_2604_25306_amd as qf
    return qf.qflash_plan_query(None, shape[0], shape[1], shape[2], shape[3], tile, *bias_bh)


# ------------------------------------------------------------- per-head constants (Appendix C3)


def run_gpu_per_head(gpu, Q, K, V, ps, tile, bias=None, packed=False):
    return run_gpu(gpu, Q, K, V, list(ps), tile, bias=bias, packed=packed)


def check_per_head(gpu, Q, K, V, ps, tile, bias=None, label=""):
    print("per-head case", label, Q.shape, "tile", tile, "bias", bias is not None, flush=True)
    ref = oracle.qflash_attention(Q, K, V, ps, tile, bias=bias)
    assert_same(run_gpu_per_head(gpu, Q, K, V, ps, tile, bias=bias), ref, label)
    if bias is not None:
        assert_same(run_gpu_per_head(gpu, Q, K, V, ps, tile, bias=bias, packed=True), ref, label + " (packed bias)")


@pytest.mark.parametrize("shape,tile", [((2, 4, 197, 64), 64), ((3, 5, 49, 32), 64), ((1, 3, 300, 64), 128),
                                        ((2, 6, 70, 32), 64), ((1, 2, 1200, 64), 64), ((1, 64, 40, 32), 64)])
def test_per_head_constants(gpu, shape, tile):
    """Heads with scales a factor 200 apart (some need x_shift > 0, so the launch mixes shifts),
    every kernel family: one head per workgroup with and without tile-by-tile staging, several
    windows per workgroup, the streamed kernel, the largest head count; with and without bias."""
    from workloads import quantize_per_head
    B, H, N, d = shape
    rng = np.random.default_rng(900 + N + H)
    gain = np.exp2(np.linspace(-2.5, 5.3, H))[None, :, None, None]
    Qf = rng.standard_normal(shape) * gain
    Kf = rng.standard_normal(shape) * gain
    Vf = rng.standard_normal(shape)
    (Q, sQ), (K, sK), (V, sV) = (quantize_per_head(x.astype(np.float32)) for x in (Qf, Kf, Vf))
    ps = [oracle.derive_params(sQ[h], sK[h], d) for h in range(H)]
    if H >= 4:
        assert len({p.x_shift for p in ps}) > 1
    check_per_head(gpu, Q, K, V, ps, tile, label="random")
    bias = rng.integers(-3000, 3000, size=(2, H, N, N)).astype(np.int32)
    bias[:, :, :, ::7] = EXCLUDED
    bias[1, 0, 3, :] = EXCLUDED
    check_per_head(gpu, Q, K, V, ps, tile, bias=bias, label="bias")


def test_per_head_equal_constants_match_per_tensor_call(gpu):
    wl = make_workload("a2_deit_s_b8")
    p = oracle.derive_params(wl.sQ, wl.sK, wl.shape[-1])
    a = run_gpu(gpu, wl.Q, wl.K, wl.V, p, 64)
    b = run_gpu_per_head(gpu, wl.Q, wl.K, wl.V, [p] * wl.shape[1], 64)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("name", ["vit_b16_b64", "deit_b384_b32", "swin_t_s1_b64"])
def test_per_head_workloads_full_size(gpu, name):
    """The per-head variant of three benchmark workloads (heads of different range, one scale per
    head; the windowed one with its bias in each head's own score unit, plain and packed), at full
    size, every byte."""
    wl = make_workload(name, per_head=True)
    H, d = wl.shape[1], wl.shape[3]
    ps = [oracle.derive_params(wl.sQ[h], wl.sK[h], d) for h in range(H)]
    check_per_head(gpu, wl.Q, wl.K, wl.V, ps, wl.kv_tiles[0], bias=wl.bias, label=wl.name)


@pytest.mark.parametrize("shape,bias_bh", [((7, 3, 49, 32), (1, 3)), ((64, 3, 49, 32), (64, 3)), ((130, 6, 20, 32), (16, 6)),
                                           ((9, 24, 49, 32), (1, 1)), ((5, 2, 64, 64), None), ((33, 4, 30, 64), (3, 4))])
def test_per_head_several_pairs_per_workgroup(gpu, shape, bias_bh):
    """Short sequences with per-head constants: a workgroup then takes one head of several
    consecutive batch elements (so that one weight table serves it); batch sizes that are and are
    not multiples of the group, bias periods that do and do not fit it."""
    from workloads import quantize_per_head
    B, H, N, d = shape
    rng = np.random.default_rng(B * 1000 + N)
    gains = np.exp2(rng.uniform(-1.5, 1.5, size=H)).astype(np.float32)
    Qf = rng.standard_normal(shape).astype(np.float32) * gains[None, :, None, None]
    Kf = rng.standard_normal(shape).astype(np.float32)
    Vf = rng.standard_normal(shape).astype(np.float32)
    (Q, sQ), (K, sK), (V, sV) = (quantize_per_head(x) for x in (Qf, Kf, Vf))
    ps = [oracle.derive_params(float(sQ[h]), float(sK[h]), d) for h in range(H)]
    bias = None
    if bias_bh is not None:
        bias = rng.integers(-4000, 4000, size=bias_bh + (N, N)).astype(np.int32)
        bias[rng.random(bias.shape) < 0.1] = EXCLUDED
    check_per_head(gpu, Q, K, V, ps, 64, bias=bias, label="per-head, several pairs per workgroup")


def test_per_head_errors(gpu):
    torch, qf, ctx = gpu
    dev = torch.device("cuda:0")
    p = qf.qflash_params_from_scales(0.02, 0.02, 0.02, 32)
    q = torch.zeros((1, 65, 8, 32), dtype=torch.int8, device=dev)
    with pytest.raises(qf.QFlashError) as e:
        ctx.attention(q, q, q, torch.empty_like(q), [p] * 65, 64)
    assert e.value.code == qf.ERR["SHAPE"]
    q = torch.zeros((1, 2, 8, 32), dtype=torch.int8, device=dev)
    p2 = qf.QFlashParams(*p.astuple())
    p2.out_round = 1
    with pytest.raises(qf.QFlashError) as e:
        ctx.attention(q, q, q, torch.empty_like(q), [p, p2], 64)
    assert e.value.code == qf.ERR["PARAM"]
    with pytest.raises(ValueError):
        ctx.attention(q, q, q, torch.empty_like(q), [p], 64)


# ------------------------------------------------- dynamic quantisation in front of the kernel


def run_dynamic(gpu, Qf, Kf, Vf, tile, out_round=0, bias_real=None, excluded=None):
    torch, qf, ctx = gpu
    dev = torch.device("cuda:0")
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(dev) for x in (Qf, Kf, Vf))
    tO = torch.full(Qf.shape, 0x55, dtype=torch.int8, device=dev)
    ref = bias_real if bias_real is not None else excluded
    nbytes = qf.qflash_dynamic_workspace_bytes(*Qf.shape) if ref is None else \
        qf.qflash_dynamic_bias_workspace_bytes(*Qf.shape, ref.shape[0], ref.shape[1])
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    info = torch.zeros(ctypes.sizeof(qf.DynamicInfo), dtype=torch.uint8, device=dev)
    tb = torch.from_numpy(np.ascontiguousarray(bias_real, dtype=np.float32)).to(dev) if bias_real is not None else None
    tm = torch.from_numpy(np.ascontiguousarray(excluded, dtype=np.uint8)).to(dev) if excluded is not None else None
    ctx.attention_dynamic(tq, tk, tv, tO, tile, ws, info=info, out_round=out_round, bias_real=tb, excluded=tm)
    torch.cuda.synchronize()
    inf = qf.DynamicInfo.from_buffer_copy(info.cpu().numpy().tobytes())
    n = Qf.size
    a256 = lambda x: (x + 255) & ~255
    wsn = ws.cpu().numpy()
    qkv = [wsn[i * a256(n): i * a256(n) + n].view(np.int8).reshape(Qf.shape) for i in range(3)]
    return tO.cpu().numpy(), inf, qkv


@pytest.mark.parametrize("shape,tile,gains", [((2, 3, 197, 64), 64, (1.0, 1.0, 1.0)), ((3, 4, 49, 32), 64, (0.3, 2.0, 1e-3)),
                                              ((1, 2, 577, 64), 128, (40.0, 40.0, 5.0)), ((1, 1, 1, 32), 64, (1.0, 1.0, 1.0)),
                                              ((1, 2, 1100, 64), 64, (1.5, 1.5, 1.0))])
def test_dynamic_quantisation_pipeline(gpu, shape, tile, gains):
    """Scales, quantised tensors, derived constants and the attention output all equal the oracle's
    (float32 rounding decisions included); a heavy-gain case needs x_shift > 0 on the GPU."""
    rng = np.random.default_rng(4000 + shape[2])
    Qf, Kf, Vf = ((rng.standard_normal(shape) * g).astype(np.float32) for g in gains)
    for out_round in (0, 1):
        ref, rinfo = oracle.qflash_attention_dynamic(Qf, Kf, Vf, tile, out_round=out_round)
        out, inf, qkv = run_dynamic(gpu, Qf, Kf, Vf, tile, out_round=out_round)
        assert inf.status == 0
        assert (inf.sQ, inf.sK, inf.sV) == (rinfo["sQ"], rinfo["sK"], rinfo["sV"])
        assert inf.params.astuple() == rinfo["params"].astuple()
        for name, got in zip("QKV", qkv):
            assert np.array_equal(got, rinfo[name]), name
        assert np.array_equal(out, ref)
    if gains[0] >= 40.0:
        assert inf.params.x_shift > 0


def test_dynamic_degenerate_and_out_of_window(gpu):
    torch, qf, ctx = gpu
    shape = (1, 2, 40, 32)
    rng = np.random.default_rng(5)
    Kf, Vf = (rng.standard_normal(shape).astype(np.float32) for _ in range(2))
    # all-zero Q: scale 1, uniform weights
    ref, rinfo = oracle.qflash_attention_dynamic(np.zeros(shape, np.float32), Kf, Vf, 64)
    out, inf, _ = run_dynamic(gpu, np.zeros(shape, np.float32), Kf, Vf, 64)
    assert inf.status == 0 and inf.sQ == 1.0 and np.array_equal(out, ref)
    # scales far too fine for the integer exponent: reported, nothing crashes
    with pytest.raises(ValueError):
        oracle.qflash_attention_dynamic(Kf * 1e-6, Kf * 1e-6, Vf, 64)
    out, inf, _ = run_dynamic(gpu, Kf * 1e-6, Kf * 1e-6, Vf, 64)
    assert inf.status == qf.ERR["PARAM"]
    assert not out.any(), "scales outside the window: the output must be all zeros"
    # argument errors
    dev = torch.device("cuda:0")
    t = torch.zeros(shape, dtype=torch.float32, device=dev)
    o = torch.zeros(shape, dtype=torch.int8, device=dev)
    small = torch.empty(64, dtype=torch.uint8, device=dev)
    with pytest.raises(qf.QFlashError) as e:
        ctx.attention_dynamic(t, t, t, o, 64, small)
    assert e.value.code == qf.ERR["SHAPE"]
    ws = torch.empty(qf.qflash_dynamic_workspace_bytes(*shape), dtype=torch.uint8, device=dev)
    with pytest.raises(qf.QFlashError) as e:
        ctx.attention_dynamic(t, t, t, o, 64, ws, out_round=2)
    assert e.value.code == qf.ERR["PARAM"]
    with pytest.raises(qf.QFlashError) as e:
        ctx.attention_dynamic(t, t, t, o, 96, ws)
    assert e.value.code == qf.ERR["TILE"]


@pytest.mark.parametrize("shape,bias_bh,tile", [((6, 3, 49, 32), (2, 3), 64), ((2, 2, 197, 64), (1, 1), 64),
                                                 ((2, 2, 300, 64), (2, 1), 128), ((1, 1, 1, 32), (1, 1), 64)])
def test_dynamic_with_real_bias_and_mask(gpu, shape, bias_bh, tile):
    """A bias in real units and an exclusion mask, converted on the GPU to the score unit of the
    scales found on the fly: equal to the oracle's conversion and attention, bit for bit; mask only
    and bias only as well."""
    rng = np.random.default_rng(4100 + shape[2])
    Qf, Kf, Vf = (rng.standard_normal(shape).astype(np.float32) for _ in range(3))
    N = shape[2]
    b = (rng.standard_normal(bias_bh + (N, N)) * 0.6).astype(np.float32)
    m = (rng.random(bias_bh + (N, N)) < 0.25).astype(np.uint8)
    m[..., 0] = 0                                   # keep one key per row
    if N > 5:
        m[0, 0, 5, :] = 1                           # ... except for one fully excluded row
    for bias_real, excluded in ((b, m), (b, None), (None, m)):
        ref, rinfo = oracle.qflash_attention_dynamic(Qf, Kf, Vf, tile, bias_real=bias_real, excluded=excluded)
        out, inf, _ = run_dynamic(gpu, Qf, Kf, Vf, tile, bias_real=bias_real, excluded=excluded)
        assert inf.status == 0 and inf.params.astuple() == rinfo["params"].astuple()
        assert_same(out, ref, "dynamic bias %s %s" % (bias_real is not None, excluded is not None))


def test_dynamic_bias_windowed_workload_and_errors(gpu):
    torch, qf, ctx = gpu
    from workloads import make_float_qkv, make_float_window_bias
    Qf, Kf, Vf = make_float_qkv("swin_t_s1_b64", batch=256)
    bias_real, excluded = make_float_window_bias("swin_t_s1_b64")
    ref, _ = oracle.qflash_attention_dynamic(Qf, Kf, Vf, 64, bias_real=bias_real, excluded=excluded)
    out, inf, _ = run_dynamic(gpu, Qf, Kf, Vf, 64, bias_real=bias_real, excluded=excluded)
    assert inf.status == 0
    assert_same(out, ref, "swin stage 1 from float inputs")
    # argument errors of the new entry point
    dev = torch.device("cuda:0")
    shape = (1, 2, 40, 32)
    t = torch.zeros(shape, dtype=torch.float32, device=dev)
    o = torch.zeros(shape, dtype=torch.int8, device=dev)
    bias = torch.zeros((1, 1, 40, 40), dtype=torch.float32, device=dev)
    ws_small = torch.empty(qf.qflash_dynamic_workspace_bytes(*shape), dtype=torch.uint8, device=dev)
    with pytest.raises(qf.QFlashError) as e:           # workspace without room for the converted bias
        ctx.attention_dynamic(t, t, t, o, 64, ws_small, bias_real=bias)
    assert e.value.code == qf.ERR["SHAPE"]
    assert qf.qflash_dynamic_bias_workspace_bytes(*shape, 0, 1) == 0
    lib = qf.load_library()
    ws = torch.empty(qf.qflash_dynamic_bias_workspace_bytes(*shape, 1, 1), dtype=torch.uint8, device=dev)
    vp = ctypes.c_void_p
    args = [vp(ctx.handle), vp(t.data_ptr()), vp(t.data_ptr()), vp(t.data_ptr()), vp(o.data_ptr())]
    tail = [1, 2, 40, 32, 64, 0, None, vp(ws.data_ptr()), ws.numel(), None]
    assert lib.qflash_attention_dynamic_bias(*args, None, None, 1, 1, *tail) == qf.ERR["NULL"]
    assert lib.qflash_attention_dynamic_bias(*args, vp(bias.data_ptr()), None, 0, 1, *tail) == qf.ERR["SHAPE"]
    assert lib.qflash_attention_dynamic_bias(*args, vp(bias.data_ptr() + 2), None, 1, 1, *tail) == qf.ERR["ALIGN"]
    assert lib.qflash_attention_dynamic_bias(*args, vp(bias.data_ptr()), None, 1, 1, *tail) == 0
    torch.cuda.synchronize()


def test_dynamic_headline_shape_full_size(gpu):
    """ViT-B/16 B=64 from float32 activations, every output byte."""
    rng = np.random.default_rng(4242)
    shape = (64, 12, 197, 64)
    Qf, Kf, Vf = (rng.standard_normal(shape, dtype=np.float32) for _ in range(3))
    ref, rinfo = oracle.qflash_attention_dynamic(Qf, Kf, Vf, 64)
    out, inf, _ = run_dynamic(gpu, Qf, Kf, Vf, 64)
    assert inf.status == 0 and inf.params.astuple() == rinfo["params"].astuple()
    assert np.array_equal(out, ref)


# ------------------------------------------------------------------- seeded random sweep


@pytest.mark.parametrize("seed", range(40))
def test_random_configurations(gpu, seed):
    """Shapes, tile size, scales, bias, exclusion, rounding mode and scale granularity drawn from a
    seed: every kernel family and staging mode meets combinations no hand-written case lists."""
    from workloads import quantize_per_head
    rng = np.random.default_rng(70000 + seed)
    d = int(rng.choice([32, 64]))
    tile = int(rng.choice([64, 128]))
    N = int(rng.choice([rng.integers(1, 65), rng.integers(65, 257), rng.integers(257, 700), rng.integers(700, 1400)]))
    B, H = int(rng.integers(1, 4)), int(rng.integers(1, 6))
    shape = (B, H, N, d)
    per_head = bool(rng.integers(0, 3) == 0)
    out_round = int(rng.integers(0, 2))
    q_gain = float(np.exp2(rng.uniform(-1.0, 3.0)))
    Qf = (rng.standard_normal(shape) * q_gain).astype(np.float32)
    Kf = rng.standard_normal(shape).astype(np.float32)
    Vf = rng.standard_normal(shape).astype(np.float32)
    if per_head:
        gain = np.exp2(rng.uniform(-1.5, 2.5, size=H))[None, :, None, None].astype(np.float32)
        Qf, Kf = Qf * gain, Kf * gain
        (Q, sQ), (K, sK), (V, sV) = (quantize_per_head(x) for x in (Qf, Kf, Vf))
        ps = [oracle.derive_params(sQ[h], sK[h], d, out_round=out_round) for h in range(H)]
    else:
        (Q, sQ), (K, sK), (V, sV) = (quantize_per_tensor(x) for x in (Qf, Kf, Vf))
        ps = oracle.derive_params(sQ, sK, d, out_round=out_round)
    bias = None
    if rng.integers(0, 3) == 0:
        bB, bH = int(rng.choice([1, B])), int(rng.choice([1, H]))
        bias = rng.integers(-5000, 5000, size=(bB, bH, N, N)).astype(np.int32)
        bias[rng.random(bias.shape) < 0.15] = EXCLUDED
        if N > 3:
            bias[0, 0, N // 2, :] = EXCLUDED           # a fully excluded row
    print("config", shape, "tile", tile, "per_head", per_head, "round", out_round, "bias", None if bias is None else bias.shape, flush=True)
    ref = oracle.qflash_attention(Q, K, V, ps, tile, bias=bias)
    out = run_gpu_per_head(gpu, Q, K, V, ps, tile, bias=bias) if per_head else run_gpu(gpu, Q, K, V, ps, tile, bias=bias)
    assert np.array_equal(out, ref)
    if bias is not None:
        out = run_gpu(gpu, Q, K, V, ps, tile, bias=bias, packed=True)
        assert np.array_equal(out, ref), "packed bias"


# ------------------------------------------------------------------------------ ABI behaviour


def test_stream_determinism_and_full_overwrite(gpu):
    torch, qf, ctx = gpu
    Q, K, V, sQ, sK, _ = rand_case((2, 3, 197, 64), 9)
    p = oracle.derive_params(sQ, sK, 64)
    ref = oracle.qflash_attention(Q, K, V, p, 64)
    a = run_gpu(gpu, Q, K, V, p, 64)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        b = run_gpu(gpu, Q, K, V, p, 64)
    c = run_gpu(gpu, Q, K, V, p, 64, stream=s.cuda_stream)
    assert np.array_equal(a, ref) and np.array_equal(b, ref) and np.array_equal(c, ref)


def test_graph_capture_and_replay(gpu):
    """The call path allocates nothing and never waits for the GPU, so a launch can be captured in a
    HIP graph: every replay (with eager work and synchronisations in between, and with the inputs
    changed in place) must give the bytes of the eager call and of the oracle."""
    torch, qf, ctx = gpu
    dev = torch.device("cuda:0")
    wl = make_workload("a2_deit_s_b8")
    p = oracle.derive_params(wl.sQ, wl.sK, wl.shape[-1])
    lp = lib_params(qf, p)
    q, k, v = (torch.from_numpy(x).to(dev) for x in (wl.Q, wl.K, wl.V))
    o = torch.zeros_like(q)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):                       # warm-up on the capture stream: table, kernel attributes
            ctx.attention(q, k, v, o, lp, 64)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ctx.attention(q, k, v, o, lp, 64)
    ref = oracle.qflash_attention(wl.Q, wl.K, wl.V, p, 64)
    for rep in range(4):
        o.fill_(0x11)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(o.cpu().numpy(), ref), "replay %d" % rep
    # new inputs in the same buffers: the graph reads what is there at replay time
    Q2 = np.ascontiguousarray(wl.Q[::-1])
    q.copy_(torch.from_numpy(Q2).to(dev))
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    assert np.array_equal(o.cpu().numpy(), oracle.qflash_attention(Q2, wl.K, wl.V, p, 64))


def test_table_cache_many_constants_and_streams(gpu):
    """Far more distinct constants than the context has table slots (a 12-layer, 12-head model with
    per-head constants has 144): the least recently used tables are rebuilt, every call keeps the
    look-up mode and every result equals the oracle's; the same constants on two streams (each
    builds its own table); eviction across streams."""
    torch, qf, _ = gpu
    ctx = qf.Context(0)                       # a cache of its own, in its initial state
    try:
        rng = np.random.default_rng(12)
        shape = (1, 2, 197, 64)
        Q = rng.integers(-127, 128, size=shape).astype(np.int8)
        K = rng.integers(-127, 128, size=shape).astype(np.int8)
        V = rng.integers(-127, 128, size=shape).astype(np.int8)
        g2 = (torch, qf, ctx)
        s2 = torch.cuda.Stream()
        for j in range(144):
            p = oracle.derive_params(0.03 + 0.0002 * j, 0.04, 64)
            out = run_gpu(g2, Q, K, V, p, 64, stream=s2.cuda_stream if j % 5 == 4 else None)
            ci = ctx.cache_info()
            assert ci.last_weight_mode == qf.WEIGHTS_TABLE, (j, ci.last_weight_mode)
            if j % 9 == 0 or j > 138:
                assert np.array_equal(out, oracle.qflash_attention(Q, K, V, p, 64)), j
        ci = ctx.cache_info()
        assert ci.slots_in_use == ci.slots_total == 32 and ci.evictions == 144 - 32 and ci.slots_pinned == 0
        # the first constants again (their table was rebuilt for others long ago), on both streams
        p = oracle.derive_params(0.03, 0.04, 64)
        ref = oracle.qflash_attention(Q, K, V, p, 64)
        assert np.array_equal(run_gpu(g2, Q, K, V, p, 64), ref)
        assert np.array_equal(run_gpu(g2, Q, K, V, p, 64, stream=s2.cuda_stream), ref)
        assert ctx.cache_info().last_weight_mode == qf.WEIGHTS_TABLE
        # per-head constants, 12 heads: one table each, all found again on the second call
        shape = (2, 12, 197, 64)
        Q, K, V = (rng.integers(-127, 128, size=shape).astype(np.int8) for _ in range(3))
        ps = [oracle.derive_params(0.05 + 0.001 * h, 0.045, 64) for h in range(12)]      # none of them seen before
        ref = oracle.qflash_attention(Q, K, V, ps, 64)
        for rep in range(2):
            assert np.array_equal(run_gpu(g2, Q, K, V, ps, 64), ref), rep
            assert ctx.cache_info().last_weight_mode == qf.WEIGHTS_TABLE
        assert ctx.cache_info().evictions == 144 - 32 + 2 + 12
        # with the table switched off the same call reports the arithmetic mode
        ctx.configure(qf.CFG_EXP_TABLE, 0)
        assert np.array_equal(run_gpu(g2, Q, K, V, ps, 64), ref)
        assert ctx.cache_info().last_weight_mode == qf.WEIGHTS_ARITHMETIC
    finally:
        ctx.close()


def test_capture_before_any_eager_call(gpu):
    """A stream is captured into a HIP graph before the context has ever seen the constants: the
    captured call must not leave a table behind that only exists once the graph has run (an eager
    call with the same constants right after the capture would read it unwritten).  Captured call:
    arithmetic; eager call afterwards: builds its table; every replay and the eager call equal the
    oracle.  A second graph captured after the eager call reads the table and pins it."""
    torch, qf, _ = gpu
    dev = torch.device("cuda:0")
    ctx = qf.Context(0)
    try:
        rng = np.random.default_rng(31)
        shape = (2, 3, 197, 64)
        Q, K, V = (rng.integers(-127, 128, size=shape).astype(np.int8) for _ in range(3))
        p = oracle.derive_params(0.031, 0.041, 64)
        lp = lib_params(qf, p)
        ref = oracle.qflash_attention(Q, K, V, p, 64)
        q, k, v = (torch.from_numpy(x).to(dev) for x in (Q, K, V))
        o_graph, o_eager = torch.zeros_like(q), torch.zeros_like(q)
        # kernel attributes are set on first use of a kernel variant: do that outside the capture,
        # with other constants and the table switched off (the arithmetic variant is what is captured)
        ctx.configure(qf.CFG_EXP_TABLE, 0)
        ctx.attention(q, k, v, o_eager, lib_params(qf, oracle.derive_params(0.05, 0.05, 64)), 64)
        ctx.configure(qf.CFG_EXP_TABLE, 1)
        torch.cuda.synchronize()
        assert ctx.cache_info().slots_in_use == 0
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            ctx.attention(q, k, v, o_graph, lp, 64)
        ci = ctx.cache_info()
        assert ci.slots_in_use == 0 and ci.last_weight_mode == qf.WEIGHTS_ARITHMETIC
        # eager call on the same stream, same constants, before the graph has ever run
        with torch.cuda.stream(side):
            ctx.attention(q, k, v, o_eager, lp, 64)
        torch.cuda.synchronize()
        assert np.array_equal(o_eager.cpu().numpy(), ref)
        ci = ctx.cache_info()
        assert ci.slots_in_use == 1 and ci.last_weight_mode == qf.WEIGHTS_TABLE and ci.slots_pinned == 0
        for rep in range(3):
            o_graph.fill_(0x22)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(o_graph.cpu().numpy(), ref), rep
        graph2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph2, stream=side):
            ctx.attention(q, k, v, o_graph, lp, 64)
        ci = ctx.cache_info()
        assert ci.last_weight_mode == qf.WEIGHTS_TABLE and ci.slots_pinned == 1
        o_graph.fill_(0x33)
        torch.cuda.synchronize()
        graph2.replay()
        torch.cuda.synchronize()
        assert np.array_equal(o_graph.cpu().numpy(), ref)
        del graph, graph2
    finally:
        ctx.close()


def test_concurrent_host_threads(gpu):
    """Several host threads call one context at once, each on its own stream and with its own
    constants (the table cache is filled concurrently); every result equals the oracle's."""
    import threading
    torch, qf, _ = gpu
    ctx = qf.Context(0)
    shape = (2, 3, 150, 64)
    rng = np.random.default_rng(99)
    Q, K, V = (rng.integers(-127, 128, size=shape).astype(np.int8) for _ in range(3))
    n_threads, rounds = 4, 6
    params = [[oracle.derive_params(0.02 + 0.003 * (t * rounds + r), 0.05, 64) for r in range(rounds)]
              for t in range(n_threads)]
    refs = [[oracle.qflash_attention(Q, K, V, p, 64) for p in row] for row in params]
    errors = []

    def worker(t):
        try:
            s = torch.cuda.Stream()
            for r in range(rounds):
                out = run_gpu((torch, qf, ctx), Q, K, V, params[t][r], 64, stream=s.cuda_stream)
                if not np.array_equal(out, refs[t][r]):
                    errors.append((t, r))
        except Exception as e:          # noqa: BLE001 - reported below
            errors.append((t, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(n_threads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    ctx.close()
    assert not errors, errors


def test_error_codes_on_gpu(gpu):
    torch, qf, ctx = gpu
    lib = qf.load_library()
    dev = torch.device("cuda:0")
    t = torch.zeros((1, 1, 64, 64), dtype=torch.int8, device=dev)
    o = torch.zeros_like(t)
    p = qf.qflash_params_from_scales(0.04, 0.04, 0.04, 64)
    h = ctypes.c_void_p(ctx.handle)
    ptr = lambda x: ctypes.c_void_p(x.data_ptr())  # noqa: E731

    def call(Qp=None, N=64, d=64, tile=64, par=p, B=1, H=1, bias=None, bB=0, bH=0):
        return lib.qflash_attention(h, Qp if Qp is not None else ptr(t), ptr(t), ptr(t), ptr(o), bias,
                                    bB, bH, B, H, N, d, tile, ctypes.byref(par) if par else None, None)

    assert call() == 0
    assert call(par=None) == qf.ERR["NULL"]
    assert call(Qp=ctypes.c_void_p(None)) == qf.ERR["NULL"]
    assert call(d=48) == qf.ERR["SHAPE"]
    assert call(N=0) == qf.ERR["SHAPE"]
    assert call(N=4097) == qf.ERR["SHAPE"]
    assert call(B=0) == qf.ERR["SHAPE"]
    assert call(tile=32) == qf.ERR["TILE"]
    assert call(Qp=ctypes.c_void_p(t.data_ptr() + 4)) == qf.ERR["ALIGN"]
    assert call(bias=ptr(t), bB=0, bH=1) == qf.ERR["SHAPE"]
    for field, val in (("s_inv", 100), ("s_inv", 1 << 18), ("x_shift", 14), ("exp_shift", 31),
                       ("exp_mul", 5), ("p_mul", 0), ("a_mul", 1), ("out_round", 2)):
        bad = qf.QFlashParams(*p.astuple())
        setattr(bad, field, val)
        assert call(par=bad) == qf.ERR["PARAM"], field
    assert lib.qflash_configure(h, 99, 1) == qf.ERR["PARAM"]
    assert lib.qflash_configure(h, qf.CFG_EXP_TABLE, 2) == qf.ERR["PARAM"]
    # packed bias: sizes, alignment, number of parameter sets
    assert qf.qflash_packed_bias_bytes(1, 1, 64) == 2 * 2 * 4 * 64 * 16
    assert qf.qflash_packed_bias_bytes(0, 1, 64) == 0 and qf.qflash_packed_bias_bytes(1, 1, 4097) == 0
    b32 = torch.zeros((1, 1, 64, 64), dtype=torch.int32, device=dev)
    pk = torch.zeros(qf.qflash_packed_bias_bytes(1, 1, 64) // 4 + 4, dtype=torch.int32, device=dev)
    nbytes = ctypes.c_size_t(pk.numel() * 4 - 16)
    assert lib.qflash_pack_bias(h, ptr(b32), 1, 1, 64, ptr(pk), nbytes, None) == 0
    assert lib.qflash_pack_bias(h, None, 1, 1, 64, ptr(pk), nbytes, None) == qf.ERR["NULL"]
    assert lib.qflash_pack_bias(h, ptr(b32), 1, 1, 64, ptr(pk), ctypes.c_size_t(1024), None) == qf.ERR["SHAPE"]
    assert lib.qflash_pack_bias(h, ptr(b32), 1, 0, 64, ptr(pk), nbytes, None) == qf.ERR["SHAPE"]
    assert lib.qflash_pack_bias(h, ptr(b32), 1, 1, 64, ctypes.c_void_p(pk.data_ptr() + 4), nbytes, None) == qf.ERR["ALIGN"]

    def call_pk(pkp, n_params=1, H=1):
        return lib.qflash_attention_packed_bias(h, ptr(t), ptr(t), ptr(t), ptr(o), pkp, 1, 1, 1, H, 64, 64, 64,
                                                ctypes.byref(p), n_params, None)

    assert call_pk(ptr(pk)) == 0
    assert call_pk(None) == qf.ERR["NULL"]
    assert call_pk(ptr(pk), n_params=2) == qf.ERR["PARAM"]
    assert call_pk(ctypes.c_void_p(pk.data_ptr() + 4)) == qf.ERR["ALIGN"]
    torch.cuda.synchronize()
    # context life cycle
    h2 = qf.qflash_create(0)
    qf.qflash_destroy(h2)
    assert lib.qflash_destroy(ctypes.c_void_p(h2)) == qf.ERR["CTX"]
    assert lib.qflash_attention(ctypes.c_void_p(h2), ptr(t), ptr(t), ptr(t), ptr(o), None, 0, 0,
                                1, 1, 64, 64, 64, ctypes.byref(p), None) == qf.ERR["CTX"]
    hh = ctypes.c_void_p()
    assert lib.qflash_create(ctypes.byref(hh), 99) == qf.ERR["DEVICE"]
