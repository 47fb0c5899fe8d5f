"""Pins for the oracle of the quantised-maximum variant (NOT the paper's Algorithm 1; no GPU).

The variant refers every score to the running maximum rounded up to a whole octave (a multiple of
s_inv in units of the scaled score), so that the rescale of past accumulators is an exact shift.

* level rule: closed form, brute force over integers, invariants (at or above the maximum, less
  than one octave above it)
* scaled exponential == Algorithm 2 on the same argument; exact powers of two at whole octaves
* single tile == whole-row definition in NumPy; state == exact int64 matmuls
* 2..10 tiles: the chain rebuilt in NumPy with plain shifts (moving, settled and random levels)
* level settled in the first tile: any tiling gives the whole-row result, bit for bit
* adding a whole number of octaves to every score of a row changes nothing, exactly
* uniform scores: floor(mean V); exclusion == deleted key; fully excluded row keeps the initial level
* exact softmax in float64 on tiny inputs (cosine), and the price against Algorithm 1
* per-head constants == head-by-head runs
"""
import math

import numpy as np
import pytest

import oracle
from oracle.params import OracleParams, derive_params, requant_constants
from workloads import quantize_per_tensor, EXCLUDED

M_INIT = -(1 << 21)


def cosine(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))


def rand_case(shape, seed, sigma=1.0, q_gain=1.0):
    rng = np.random.default_rng(seed)
    Qf = rng.standard_normal(shape).astype(np.float32) * np.float32(sigma * q_gain)
    Kf = rng.standard_normal(shape).astype(np.float32) * np.float32(sigma)
    Vf = rng.standard_normal(shape).astype(np.float32)
    (Q, sQ), (K, sK), (V, sV) = (quantize_per_tensor(x) for x in (Qf, Kf, Vf))
    return Q, K, V, sQ, sK, sV


def exact_params(s_inv=1024, k=0):
    p_mul, p_shift = requant_constants(s_inv)
    return OracleParams(k, s_inv, -((1 << 32) // s_inv), 32, p_mul, p_shift, -((-(1 << 30)) // s_inv), 0)


# ------------------------------------------------------------------ the level rule


@pytest.mark.parametrize("s_inv,k", [(1024, 0), (6161, 0), (1500, 3), (2047, 16), (262143, 0)])
def test_level_is_the_ceiling_of_the_scaled_score_in_octaves(s_inv, k):
    p = exact_params(s_inv, k)
    rng = np.random.default_rng(s_inv + k)
    ts = list(rng.integers(-(1 << 21), 1 << 21, size=300)) + [0, 1, -1, M_INIT, (1 << 21) - 1]
    if k == 0:
        ts += [s_inv, s_inv + 1, s_inv - 1, -s_inv, -s_inv + 1, -s_inv - 1, 7 * s_inv, -7 * s_inv]
    for t in ts:
        t = int(t)
        L = oracle.qmax_level(t, p)
        # Python integers: exact.  L is the smallest integer with L * s_inv >= t * 2^k
        assert L * s_inv >= t * 2 ** k > (L - 1) * s_inv
        assert L == math.ceil(t * 2 ** k / s_inv) or abs(t * 2 ** k) > 2 ** 50   # float form where it is exact


def test_level_brute_force_small():
    p = exact_params(1024, 0)
    for t in range(-5000, 5000):
        L = oracle.qmax_level(t, p)
        assert L == next(c for c in range(-6, 7) if c * 1024 >= t)


def test_scaled_exponential_is_algorithm_2_on_the_scaled_argument():
    """For k = 0 the two functions are the same; for k > 0, feeding x * 2^k gives what Algorithm 2
    gives for x.  Whole octaves give exact powers of two."""
    for p in (derive_params(0.03, 0.03, 64), exact_params(1024, 0), derive_params(0.9, 1.3, 32), exact_params(1500, 3)):
        rng = np.random.default_rng(p.s_inv)
        for x in list(rng.integers(-40 * p.s_inv >> p.x_shift, 1, size=400)) + [0, -1]:
            x = int(x)
            assert oracle.shift_exp2_scaled(x << p.x_shift, p) == oracle.shift_exp2(x, p)
    p = exact_params(1024, 3)
    for n in range(0, 11):
        assert oracle.shift_exp2_scaled(-1024 * n, p) == 1024 >> n
    # an argument between the scaled steps of Algorithm 2 (not a multiple of 2^k): hand-worked,
    # xs = -1538 -> q = 1, r = -514, y = ((-514 >> 1) + 1024) >> 1 = 383
    assert oracle.shift_exp2_scaled(-1538, p) == 383


# ------------------------------------------------------------------ single tile


@pytest.mark.parametrize("shape,tile,seed", [
    ((2, 3, 49, 32), 64, 2), ((1, 2, 64, 64), 64, 3), ((3, 1, 17, 64), 128, 4),
    ((1, 1, 1, 32), 64, 5), ((2, 2, 128, 64), 128, 6)])
def test_single_tile_equals_whole_row_definition(shape, tile, seed):
    Q, K, V, sQ, sK, _ = rand_case(shape, seed)
    p = derive_params(sQ, sK, shape[-1])
    out, st = oracle.qflash_attention_qmax(Q, K, V, p, tile, return_state=True)
    ref, rst = oracle.fullrow_int_attention_qmax(Q, K, V, p, return_state=True)
    assert st["violations"] == 0
    assert np.array_equal(st["m"], rst["m"]) and np.array_equal(st["l"], rst["l"])
    assert np.array_equal(st["O_acc"], rst["O_acc"]) and np.array_equal(out, ref)


@pytest.mark.parametrize("k_forced", [None, 2])
def test_single_tile_state_from_scalar_functions(k_forced):
    """Level, weights and sums of one tile from exact int64 matmuls and the scalar building blocks,
    element by element (Python integers)."""
    shape = (1, 2, 23, 32)
    Q, K, V, sQ, sK, _ = rand_case(shape, 11)
    p = derive_params(sQ, sK, 32) if k_forced is None else derive_params(sQ * 30, sK * 30, 32)
    if k_forced is not None:
        assert p.x_shift > 0
    out, st = oracle.qflash_attention_qmax(Q, K, V, p, 64, return_state=True)
    S = Q.astype(np.int64) @ K.astype(np.int64).transpose(0, 1, 3, 2)
    for h in range(2):
        for i in range(23):
            row = [int(v) for v in S[0, h, i]]
            L = max(oracle.qmax_level(M_INIT, p), oracle.qmax_level(max(row), p))
            assert st["m"][0, h, i] == L
            ref_level = L * p.s_inv
            assert 0 <= ref_level - (max(row) << p.x_shift) < p.s_inv
            P = [oracle.requant(oracle.shift_exp2_scaled((s << p.x_shift) - ref_level, p), p) for s in row]
            assert max(P) >= 63                        # the largest weight loses at most one bit
            assert st["l"][0, h, i] == sum(P)
            acc = [sum(P[c] * int(V[0, h, c, t]) for c in range(23)) for t in range(32)]
            assert [int(v) for v in st["O_acc"][0, h, i]] == acc
            assert [int(v) for v in out[0, h, i]] == [max(-128, min(127, a // sum(P))) for a in acc]


# ------------------------------------------------------------------ several tiles


@pytest.mark.parametrize("n_tiles,tile,order", [(2, 16, "up"), (3, 16, "up"), (5, 16, "up"), (10, 8, "up"), (4, 64, "up"),
                                                (6, 16, "down"), (7, 16, "mixed")])
def test_many_tile_chain_rebuilt_with_plain_shifts(n_tiles, tile, order):
    N = n_tiles * tile - 3
    shape = (1, 2, N, 32)
    rng = np.random.default_rng(77 + n_tiles)
    Qf = np.abs(rng.standard_normal(shape)).astype(np.float32) * 2.5
    Kf = np.abs(rng.standard_normal(shape)).astype(np.float32)
    ramp = np.linspace(0.1, 1.0, N, dtype=np.float32)[None, None, :, None]
    if order == "up":
        Kf = Kf * ramp
    elif order == "down":
        Kf = Kf * ramp[:, :, ::-1]
    else:
        Kf = rng.standard_normal(shape).astype(np.float32)
    Vf = rng.standard_normal(shape).astype(np.float32)
    (Q, sQ), (K, sK), (V, _) = (quantize_per_tensor(x) for x in (Qf, Kf, Vf))
    p = derive_params(sQ, sK, 32)
    assert p.x_shift == 0
    out, st = oracle.qflash_attention_qmax(Q, K, V, p, tile, return_state=True)
    S = Q.astype(np.int64) @ K.astype(np.int64).transpose(0, 1, 3, 2)
    Vi = V.astype(np.int64)
    L = np.full(S.shape[:-1], -((-M_INIT) // p.s_inv), dtype=np.int64)     # ceil of a negative number
    l = np.zeros_like(L)
    O = np.zeros(S.shape[:-1] + (32,), dtype=np.int64)
    moved, shifts = [], []
    for j in range(n_tiles):
        Sj, Vj = S[..., j * tile:(j + 1) * tile], Vi[:, :, j * tile:(j + 1) * tile]
        L_new = np.maximum(L, -((-Sj.max(-1)) // p.s_inv))
        n = L_new - L
        Pj = oracle.requant_np(oracle.shift_exp2_np(Sj - (L_new * p.s_inv)[..., None], p), p)   # k = 0
        l = (l >> np.minimum(n, 62)) + Pj.sum(-1)
        O = (O >> np.minimum(n, 62)[..., None]) + Pj @ Vj
        if j > 0:
            moved.append(float((n > 0).mean()))
            shifts.append(int(n.max()))
        L = L_new
    if order == "up":
        assert np.mean(moved) > 0.3 and max(shifts) >= 1, (moved, shifts)       # levels do move
    if order == "down":
        assert max(moved) < 0.2, moved
    assert np.array_equal(st["m"], L) and np.array_equal(st["l"], l) and np.array_equal(st["O_acc"], O)
    assert np.array_equal(out, np.clip(O // l[..., None], -128, 127).astype(np.int8))


@pytest.mark.parametrize("tile", [8, 16, 48, 64, 256])
def test_level_settled_in_first_tile_equals_whole_row(tile):
    """When the first tile already holds a score within the top octave, no later tile moves the
    level and the tile-wise result is the whole-row result bit for bit, whatever the tiling."""
    rng = np.random.default_rng(7)
    B, H, N, d = 2, 2, 150, 64
    Q = rng.integers(-10, 11, size=(B, H, N, d)).astype(np.int8)
    K = rng.integers(-10, 11, size=(B, H, N, d)).astype(np.int8)
    V = rng.integers(-127, 128, size=(B, H, N, d)).astype(np.int8)
    Q[..., 0] = 127
    K[..., 0] = -np.abs(K[..., 0])
    K[:, :, 3, 0] = 127
    p = exact_params(4000)
    out, st = oracle.qflash_attention_qmax(Q, K, V, p, tile, return_state=True)
    ref, rst = oracle.fullrow_int_attention_qmax(Q, K, V, p, return_state=True)
    assert (rst["P"] > 0).mean() > 0.3
    assert np.array_equal(st["O_acc"], rst["O_acc"]) and np.array_equal(st["l"], rst["l"])
    assert np.array_equal(out, ref)


def test_tiling_changes_the_result_only_through_floors():
    """With a moving level the tilings differ by floors only: a weight computed at an earlier, lower
    level and shifted down later differs from the weight computed at the final level by less than
    one unit, and every shift of a sum floors once.  So the denominators of any tiling stay within
    (keys + tiles) units of the whole-row value; the int8 outputs agree within one step on more than
    95 % of the elements (rows with a small denominator move by a few steps)."""
    Q, K, V, sQ, sK, _ = rand_case((1, 2, 160, 32), 5, q_gain=2.0)
    p = derive_params(sQ, sK, 32)
    ref, rst = oracle.fullrow_int_attention_qmax(Q, K, V, p, return_state=True)
    differs = False
    for tile in (8, 16, 40, 64):
        out, st = oracle.qflash_attention_qmax(Q, K, V, p, tile, return_state=True)
        assert np.array_equal(st["m"], rst["m"])                       # the final level is the row's
        n_t = -(-160 // tile)
        assert np.abs(st["l"] - rst["l"]).max() <= 160 + n_t
        diff = np.abs(out.astype(int) - ref.astype(int))
        assert (diff <= 1).mean() > 0.95 and diff.mean() < 0.4 and diff.max() <= 10
        differs |= not np.array_equal(st["l"], rst["l"])
    assert differs                                                      # the case does exercise moving levels


def test_whole_octave_offset_changes_nothing():
    """Adding j * s_inv (k = 0) to every score of a row moves its level by j and leaves every
    weight, sum and output unchanged, exactly -- the shift invariance of softmax survives for
    whole octaves."""
    shape = (1, 2, 70, 32)
    Q, K, V, sQ, sK, _ = rand_case(shape, 12, q_gain=1.5)
    p = derive_params(sQ, sK, 32)
    assert p.x_shift == 0
    rng = np.random.default_rng(3)
    j = rng.integers(-3, 4, size=(1, 2, 70, 1))
    bias = np.broadcast_to(j * p.s_inv, (1, 2, 70, 70)).astype(np.int32)
    for tile in (64, 16):
        o0, s0 = oracle.qflash_attention_qmax(Q, K, V, p, tile, return_state=True)
        o1, s1 = oracle.qflash_attention_qmax(Q, K, V, p, tile, bias=bias, return_state=True)
        assert np.array_equal(o0, o1) and np.array_equal(s0["l"], s1["l"]) and np.array_equal(s0["O_acc"], s1["O_acc"])
        assert np.array_equal(s1["m"] - s0["m"], j[..., 0])
    # ... and a fraction of an octave does change the weights
    bias2 = np.full((1, 1, 70, 70), p.s_inv // 2, dtype=np.int32)
    _, s2 = oracle.qflash_attention_qmax(Q, K, V, p, 64, bias=bias2, return_state=True)
    assert not np.array_equal(s2["l"], s0["l"])


def test_uniform_scores_give_floor_of_mean():
    rng = np.random.default_rng(9)
    shape = (1, 2, 197, 64)
    Q = rng.integers(-127, 128, size=shape).astype(np.int8)
    K = np.zeros(shape, dtype=np.int8)
    V = rng.integers(-127, 128, size=shape).astype(np.int8)
    p = derive_params(0.04, 0.04, 64)
    for r in (0, 1):
        pr = OracleParams(*p.astuple()[:-1], r)
        out, st = oracle.qflash_attention_qmax(Q, K, V, pr, 64, return_state=True)
        assert np.all(st["m"] == 0)                              # score 0 sits on a level
        assert np.all(st["l"] == oracle.requant(p.s_inv, p) * 197)
        sumV = V.astype(np.int64).sum(axis=2, keepdims=True)
        ref = sumV // 197 if r == 0 else (2 * sumV + 197) // (2 * 197)
        assert np.array_equal(out, np.broadcast_to(ref, shape).astype(np.int8))


def test_exclusion_equals_deleted_key_and_empty_rows_keep_the_initial_level():
    shape = (1, 2, 40, 32)
    Q, K, V, sQ, sK, _ = rand_case(shape, 5)
    p = derive_params(sQ, sK, 32)
    bias = np.zeros((1, 1, 40, 40), dtype=np.int32)
    bias[0, 0, :, 13] = EXCLUDED
    keep = [c for c in range(40) if c != 13]
    for tile in (64, 16):
        out = oracle.qflash_attention_qmax(Q, K, V, p, tile, bias=bias)
        # deleting key 13 (the queries stay): same rows
        Kd, Vd = K[:, :, keep], V[:, :, keep]
        S = Q.astype(np.int64) @ Kd.astype(np.int64).transpose(0, 1, 3, 2)
        if tile == 64:
            L = np.maximum(-((-S.max(-1)) // p.s_inv), -((-M_INIT) // p.s_inv))
            P = oracle.requant_np(oracle.shift_exp2_np(S - (L * p.s_inv)[..., None], p), p)
            ref = np.clip((P @ Vd.astype(np.int64)) // P.sum(-1)[..., None], -128, 127).astype(np.int8)
            assert np.array_equal(out, ref)
    bias[0, 0, 7, :] = EXCLUDED
    for tile in (64, 16):
        out, st = oracle.qflash_attention_qmax(Q, K, V, p, tile, bias=bias, return_state=True)
        assert np.all(st["m"][:, :, 7] == oracle.qmax_level(M_INIT, p)) and np.all(st["l"][:, :, 7] == 0)
        assert np.all(out[:, :, 7] == 0)


# ------------------------------------------------------------------ against exact softmax


@pytest.mark.parametrize("N,d,tile", [(16, 64, 8), (32, 32, 16), (48, 32, 16)])
def test_cosine_against_float_softmax_tiny(N, d, tile):
    """Tiny inputs, Q scaled by 2.  The variant gives up to one bit of the weights, so its gate is
    the paper's 0.999 on the mean of the un-rounded ratio and 0.998 on the worst case; beside it
    the figures of Algorithm 1 on the same inputs."""
    cos_v, cos_a, cos_mid = [], [], []
    for seed in range(24):
        Q, K, V, sQ, sK, sV = rand_case((1, 2, N, d), 100 + seed, q_gain=2.0)
        p = derive_params(sQ, sK, d)
        out, st = oracle.qflash_attention_qmax(Q, K, V, p, tile, return_state=True)
        assert st["violations"] == 0
        _, sa = oracle.qflash_attention(Q, K, V, p, tile, return_state=True)
        ref = oracle.float_attention_ratio(Q, K, V, sQ, sK)
        cos_v.append(cosine(st["O_acc"] / st["l"][..., None], ref))
        cos_a.append(cosine(sa["O_acc"] / sa["l"][..., None], ref))
        cos_mid.append(cosine(out.astype(np.float64) + 0.5, ref))
    assert np.mean(cos_v) >= 0.999, (np.mean(cos_v), min(cos_v))
    assert min(cos_v) >= 0.998, min(cos_v)
    assert np.mean(cos_mid) >= 0.998, np.mean(cos_mid)
    # the price: not better than Algorithm 1 on average, and not much worse
    assert np.mean(cos_a) - np.mean(cos_v) < 1e-3


def test_agreement_with_algorithm_1_on_a_benchmark_shape():
    """On a DeiT-shaped layer the variant's int8 outputs are those of Algorithm 1 in the bulk:
    within one step almost everywhere."""
    Q, K, V, sQ, sK, _ = rand_case((1, 3, 197, 64), 1)
    p = derive_params(sQ, sK, 64)
    a = oracle.qflash_attention(Q, K, V, p, 64).astype(int)
    v = oracle.qflash_attention_qmax(Q, K, V, p, 64).astype(int)
    diff = np.abs(a - v)
    assert (diff <= 1).mean() > 0.99 and diff.max() <= 4, ((diff <= 1).mean(), diff.max())


def test_per_head_constants_equal_head_by_head_runs():
    shape = (2, 3, 70, 32)
    Q, K, V, sQ, sK, _ = rand_case(shape, 8)
    ps = [derive_params(sQ * g, sK, 32) for g in (1.0, 0.6, 1.7)]
    out = oracle.qflash_attention_qmax(Q, K, V, ps, 16)
    for h in range(3):
        ref = oracle.qflash_attention_qmax(Q[:, h:h + 1], K[:, h:h + 1], V[:, h:h + 1], ps[h], 16)
        assert np.array_equal(out[:, h:h + 1], ref)
