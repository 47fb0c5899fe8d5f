"""Pins for the tile-wise CPU oracle (Algorithm 1) against definitions that do not use it (no GPU).

* exact integer matmuls and row maxima against NumPy int64
* single KV tile, and any tiling when every row maximum sits in the first tile:
  bit-equal to the brute-force full-row integer softmax
* two tiles: the composition rule of Algorithm 1 (rescale by alpha, release its
  scale, add the new tile) written out on the state of the first tile
* uniform scores: the output is floor(mean(V)) exactly
* exact softmax attention in float64 on tiny inputs (cosine >= 0.999)
* floor division at the end, the scaling identity behind x_shift, exclusion
  equals deleting the key, a per-row constant bias changes nothing
* invariants of the running state
"""
import numpy as np
import pytest

import oracle
from oracle.params import OracleParams, derive_params
from workloads import make_qkv, quantize_per_tensor, make_workload, EXCLUDED


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


# ---------------------------------------------------------------- exact pieces


@pytest.mark.parametrize("shape,tile", [((2, 2, 40, 64), 64), ((1, 3, 49, 32), 64),
                                        ((1, 1, 100, 16), 128)])
def test_single_tile_state_is_exact_matmul(shape, tile):
    Q, K, V, sQ, sK, _ = rand_case(shape, 1)
    p = derive_params(sQ, sK, shape[-1])
    out, st = oracle.qflash_attention(Q, K, V, p, tile, return_state=True)
    assert st["violations"] == 0
    S = Q.astype(np.int64) @ K.astype(np.int64).transpose(0, 1, 3, 2)
    m = S.max(axis=-1)
    assert np.array_equal(st["m"], m)
    P = oracle.requant_np(oracle.shift_exp2_np(S - m[..., None], p), p)
    assert np.array_equal(st["l"], P.sum(-1))
    assert np.array_equal(st["O_acc"], P @ V.astype(np.int64))
    # final step is Python's floor division, then saturation
    ref = np.empty(shape, dtype=np.int64)
    for idx in np.ndindex(*shape):
        ref[idx] = max(-128, min(127, int(st["O_acc"][idx]) // int(st["l"][idx[:-1]])))
    assert np.array_equal(out, ref.astype(np.int8))


@pytest.mark.parametrize("shape,tile,seed", [
    ((2, 3, 49, 32), 64, 2), ((1, 2, 64, 64), 64, 3), ((3, 1, 17, 64), 128, 4),
    ((1, 1, 1, 32), 64, 5), ((2, 2, 128, 64), 128, 6)])
def test_single_tile_equals_fullrow(shape, tile, seed):
    Q, K, V, sQ, sK, _ = rand_case(shape, seed)
    p = derive_params(sQ, sK, shape[-1])
    out = oracle.qflash_attention(Q, K, V, p, tile)
    assert np.array_equal(out, oracle.fullrow_int_attention(Q, K, V, p))


@pytest.mark.parametrize("tile", [8, 16, 48, 64])
def test_early_maximum_equals_fullrow(tile):
    """When every row's maximum lies in the first KV tile, later alphas are exactly 1.0
    and the tile-wise result is bit-equal to the full-row integer softmax."""
    rng = np.random.default_rng(7)
    B, H, N, d = 2, 2, 150, 64
    Q = rng.integers(-10, 11, size=(B, H, N, d)).astype(np.int8)
    K = rng.integers(-10, 11, size=(B, H, N, d)).astype(np.int8)
    V = rng.integers(-127, 128, size=(B, H, N, d)).astype(np.int8)
    Q[..., 0] = 127
    K[..., 0] = -np.abs(K[..., 0])
    K[:, :, 3, 0] = 127                    # key 3 wins every row: 16129 - 6300 > 6300
    S = Q.astype(np.int64) @ K.astype(np.int64).transpose(0, 1, 3, 2)
    assert np.all(S.argmax(-1) == 3)
    # about 4 octaves between the winner and the rest, so the other weights are not all zero
    p = OracleParams(0, 4000, -round(2 ** 32 / 4000), 32,
                     *oracle.params.requant_constants(4000), -((-(1 << 30)) // 4000), 0)
    out, st = oracle.qflash_attention(Q, K, V, p, tile, return_state=True)
    ref, rst = oracle.fullrow_int_attention(Q, K, V, p, return_state=True)
    assert (rst["P"] > 0).mean() > 0.3
    assert np.array_equal(st["O_acc"], rst["O_acc"]) and np.array_equal(st["l"], rst["l"])
    assert np.array_equal(out, ref)


@pytest.mark.parametrize("N,tile", [(32, 16), (70, 64), (129, 128), (40, 24)])
def test_two_tile_composition(N, tile):
    """State after tile 2 = ScaleRelease(state after tile 1, alpha) + tile 2, with alpha from
    the change of the running maximum (Algorithm 1, inner loop)."""
    assert tile < N <= 2 * tile
    shape = (2, 2, N, 32)
    Q, K, V, sQ, sK, _ = rand_case(shape, 21 + N, q_gain=1.5)
    p = derive_params(sQ, sK, 32)
    out, st = oracle.qflash_attention(Q, K, V, p, tile, return_state=True)
    # state after the first tile: run the oracle on the first `tile` keys only
    _, s1 = oracle.qflash_attention(Q[:, :, :tile], K[:, :, :tile], V[:, :, :tile], p, tile,
                                    return_state=True)
    Qi = Q.astype(np.int64)
    S2 = Qi @ K[:, :, tile:].astype(np.int64).transpose(0, 1, 3, 2)          # [B,H,N,N-tile]
    S1 = Qi @ K[:, :, :tile].astype(np.int64).transpose(0, 1, 3, 2)
    m1 = S1.max(-1)
    # rows >= tile were not part of the truncated run: rebuild their first-tile state directly
    P1 = oracle.requant_np(oracle.shift_exp2_np(S1 - m1[..., None], p), p)
    l1 = P1.sum(-1)
    O1 = P1 @ V[:, :, :tile].astype(np.int64)
    assert np.array_equal(s1["l"], l1[:, :, :tile]) and np.array_equal(s1["O_acc"], O1[:, :, :tile])
    m2 = np.maximum(m1, S2.max(-1))
    a_hat = oracle.shift_exp2_np(m1 - m2, p)
    a16 = np.minimum((a_hat * p.a_mul) >> 14, 65536)
    assert (a16 < 65536).mean() > 0.01 and (a16 == 65536).mean() > 0.2     # both branches live
    P2 = oracle.requant_np(oracle.shift_exp2_np(S2 - m2[..., None], p), p)
    l2 = ((l1 * a16) >> 16) + P2.sum(-1)
    O2 = ((O1 * a16[..., None]) >> 16) + P2 @ V[:, :, tile:].astype(np.int64)
    assert np.array_equal(st["m"], m2)
    assert np.array_equal(st["l"], l2)
    assert np.array_equal(st["O_acc"], O2)
    assert np.array_equal(out, np.clip(O2 // l2[..., None], -128, 127).astype(np.int8))


@pytest.mark.parametrize("n_tiles,tile,order", [(3, 16, "up"), (5, 16, "up"), (10, 8, "up"), (4, 64, "up"),
                                                (6, 16, "down"), (7, 16, "mixed")])
def test_many_tile_composition(n_tiles, tile, order):
    """The whole chain of Algorithm 1's inner loop, tile after tile, rebuilt in NumPy int64 from the
    scores: running maximum, alpha from its change, ScaleRelease of denominator and numerator, the
    tile's weights.  Keys are ordered so that the row maximum moves in every tile ("up"), never
    after the first ("down"), or at random ("mixed"); the last tile is ragged."""
    N = n_tiles * tile - 3
    shape = (1, 2, N, 32)
    rng = np.random.default_rng(77 + n_tiles)
    Qf = np.abs(rng.standard_normal(shape)).astype(np.float32) * 1.5
    Kf = np.abs(rng.standard_normal(shape)).astype(np.float32)
    ramp = np.linspace(0.2, 1.0, N, dtype=np.float32)[None, None, :, None]
    if order == "up":
        Kf = Kf * ramp
    elif order == "down":
        Kf = Kf * ramp[:, :, ::-1]
    else:
        Kf = rng.standard_normal(shape).astype(np.float32)
    Vf = rng.standard_normal(shape).astype(np.float32)
    (Q, sQ), (K, sK), (V, _) = (quantize_per_tensor(x) for x in (Qf, Kf, Vf))
    p = derive_params(sQ, sK, 32)
    out, st = oracle.qflash_attention(Q, K, V, p, tile, return_state=True)
    S = Q.astype(np.int64) @ K.astype(np.int64).transpose(0, 1, 3, 2)
    Vi = V.astype(np.int64)
    m = np.full(S.shape[:-1], -(1 << 21), dtype=np.int64)
    l = np.zeros_like(m)
    O = np.zeros(S.shape[:-1] + (32,), dtype=np.int64)
    moved = []
    for j in range(n_tiles):
        Sj, Vj = S[..., j * tile:(j + 1) * tile], Vi[:, :, j * tile:(j + 1) * tile]
        m_new = np.maximum(m, Sj.max(-1))
        a16 = np.minimum((oracle.shift_exp2_np(m - m_new, p) * p.a_mul) >> 14, 65536)
        Pj = oracle.requant_np(oracle.shift_exp2_np(Sj - m_new[..., None], p), p)
        l = ((l * a16) >> 16) + Pj.sum(-1)
        O = ((O * a16[..., None]) >> 16) + Pj @ Vj
        if j > 0:
            moved.append(float((m_new > m).mean()))
        m = m_new
    if order == "up":
        assert min(moved) > 0.7, moved            # the maximum moves in every tile for most rows
    if order == "down":
        assert max(moved) < 0.3, moved
    assert np.array_equal(st["m"], m) and np.array_equal(st["l"], l) and np.array_equal(st["O_acc"], O)
    assert np.array_equal(out, np.clip(O // l[..., None], -128, 127).astype(np.int8))


def test_initial_maximum_survives_in_a_fully_excluded_row():
    """Algorithm 1 starts the running maximum at -2^21; a row whose every key is excluded never
    updates it (and yields zeros), in one tile and in several."""
    shape = (1, 2, 40, 32)
    Q, K, V, sQ, sK, _ = rand_case(shape, 5)
    p = derive_params(sQ, sK, 32)
    bias = np.zeros((1, 1, 40, 40), dtype=np.int32)
    bias[0, 0, 7, :] = EXCLUDED
    bias[0, 0, 12, :39] = EXCLUDED              # one key left: an ordinary row
    for tile in (64, 16):
        out, st = oracle.qflash_attention(Q, K, V, p, tile, bias=bias, return_state=True)
        assert np.all(st["m"][:, :, 7] == -(1 << 21)) and np.all(st["l"][:, :, 7] == 0)
        assert np.all(out[:, :, 7] == 0)
        S = Q.astype(np.int64) @ K.astype(np.int64).transpose(0, 1, 3, 2)
        assert np.array_equal(st["m"][:, :, 12], S[:, :, 12, 39])
        assert np.array_equal(out[:, :, 12], V[:, :, 39])          # a single weight: the value row itself
        others = [i for i in range(40) if i not in (7, 12)]
        assert np.array_equal(st["m"][:, :, others], S[:, :, others].max(-1))


def test_uniform_scores_give_floor_of_mean():
    """K = 0: all scores equal, all weights equal, every alpha is 1.0 -> out = floor(mean V)."""
    rng = np.random.default_rng(9)
    shape = (1, 2, 197, 64)
    Q = rng.integers(-127, 128, size=shape).astype(np.int8)
    K = np.zeros(shape, dtype=np.int8)
    V = rng.integers(-127, 128, size=shape).astype(np.int8)
    p = derive_params(0.04, 0.04, 64)
    for r in (0, 1):
        pr = OracleParams(*p.astuple()[:-1], r)
        out, st = oracle.qflash_attention(Q, K, V, pr, 64, return_state=True)
        w = oracle.requant(p.s_inv, p)
        assert np.all(st["l"] == w * 197)
        sumV = V.astype(np.int64).sum(axis=2, keepdims=True)
        ref = sumV // 197 if r == 0 else (2 * sumV + 197) // (2 * 197)
        assert np.array_equal(out, np.broadcast_to(ref, shape).astype(np.int8))


def test_saturation_and_sign_of_final_division():
    """V = -128 everywhere: numerator = -128 * l exactly -> -128; V = 127 -> 127."""
    shape = (1, 1, 70, 32)
    Q, K, _, sQ, sK, _ = rand_case(shape, 31)
    p = derive_params(sQ, sK, 32)
    for v in (-128, 127, -1, 1):
        V = np.full(shape, v, dtype=np.int8)
        out, st = oracle.qflash_attention(Q, K, V, p, 64, return_state=True)
        # numerator and denominator are rescaled by separate floors, so they may differ by a
        # few units; the result stays within one step of v and inside int8
        ref = np.clip(st["O_acc"] // st["l"][..., None], -128, 127)
        assert np.array_equal(out, ref.astype(np.int8))
        assert np.all(np.abs(out.astype(np.int64) - v) <= 1)


# ------------------------------------------------------- against exact softmax


@pytest.mark.parametrize("N,d,tile", [(16, 64, 8), (32, 32, 16), (48, 32, 16)])
def test_cosine_against_float_softmax_tiny(N, d, tile):
    """Tiny inputs, Q scaled by 2: the integer path tracks exact softmax attention on the same
    dequantised inputs with cosine >= 0.999, both for the un-rounded ratio numerator/denominator
    and for the int8 output dequantised at the mid-point of its floor interval."""
    cos_ratio, cos_mid, cos_floor = [], [], []
    for seed in range(24):
        Q, K, V, sQ, sK, sV = rand_case((1, 2, N, d), 100 + seed, q_gain=2.0)
        p = derive_params(sQ, sK, d)
        out, st = oracle.qflash_attention(Q, K, V, p, tile, return_state=True)
        assert st["violations"] == 0
        ref = oracle.float_attention_ratio(Q, K, V, sQ, sK)
        ratio = st["O_acc"] / st["l"][..., None]
        cos_ratio.append(cosine(ratio, ref))
        cos_mid.append(cosine(out.astype(np.float64) + 0.5, ref))
        cos_floor.append(cosine(out, ref))
    assert min(cos_ratio) >= 0.999, cos_ratio
    assert np.mean(cos_mid) >= 0.999, cos_mid
    assert min(cos_floor) >= 0.99


def test_fullrow_bruteforce_against_float_softmax():
    """The brute-force integer reference itself is pinned to exact softmax."""
    for seed in range(8):
        Q, K, V, sQ, sK, _ = rand_case((1, 2, 32, 32), 300 + seed, q_gain=2.0)
        p = derive_params(sQ, sK, 32)
        _, st = oracle.fullrow_int_attention(Q, K, V, p, return_state=True)
        ratio = st["O_acc"] / st["l"][..., None]
        assert cosine(ratio, oracle.float_attention_ratio(Q, K, V, sQ, sK)) >= 0.999


@pytest.mark.parametrize("order", ["ascending", "descending"])
def test_maximum_moves_every_tile_or_never(order):
    """Keys sorted so that the running maximum rises at every tile (alpha < 1 every time) or is
    found at once: both must track exact softmax."""
    N, d, tile = 64, 32, 8
    Q, K, V, sQ, sK, _ = rand_case((1, 1, N, d), 55, q_gain=2.0)
    # make all queries nearly parallel so one key order sorts every row
    Q[0, 0] = np.clip(Q[0, 0, :1].astype(np.int64) + np.random.default_rng(1).integers(-3, 4, (N, d)),
                      -127, 127).astype(np.int8)
    s0 = Q[0, 0, 0].astype(np.int64) @ K[0, 0].astype(np.int64).T
    perm = np.argsort(s0) if order == "ascending" else np.argsort(-s0)
    K, V = K[:, :, perm], V[:, :, perm]
    p = derive_params(sQ, sK, d)
    out, st = oracle.qflash_attention(Q, K, V, p, tile, return_state=True)
    ref = oracle.float_attention_ratio(Q, K, V, sQ, sK)
    assert cosine(st["O_acc"] / st["l"][..., None], ref) >= 0.998
    assert st["violations"] == 0


# ------------------------------------------------------------------ identities


def test_x_shift_scaling_identity():
    """Forcing x_shift = k on (Q, K) equals x_shift = 0 on (Q, 2^k K) with the same constants."""
    rng = np.random.default_rng(77)
    k = 3
    shape = (2, 2, 90, 32)
    Q = rng.integers(-127, 128, size=shape).astype(np.int8)
    K = rng.integers(-15, 16, size=shape).astype(np.int8)
    V = rng.integers(-127, 128, size=shape).astype(np.int8)
    base = derive_params(0.02, 0.02, 32)
    pk = OracleParams(k, *base.astuple()[1:])
    p0 = OracleParams(0, *base.astuple()[1:])
    a = oracle.qflash_attention(Q, K, V, pk, 32)
    b = oracle.qflash_attention(Q, (K.astype(np.int64) << k).astype(np.int8), V, p0, 32)
    assert np.array_equal(a, b)


def test_heavy_tail_needs_and_gets_x_shift():
    """Coarse score scale (heavy-tailed activations): derive_params picks k > 0, s_inv stays in
    range and the result still tracks exact softmax."""
    rng = np.random.default_rng(5)
    shape = (1, 2, 48, 64)
    xs = []
    for _ in range(3):
        x = rng.standard_t(3.0, size=shape).astype(np.float32)
        x[..., 5] *= 8
        xs.append(quantize_per_tensor(x))
    (Q, sQ), (K, sK), (V, sV) = xs
    p = derive_params(sQ, sK, 64)
    assert p.x_shift > 0 and 1024 <= p.s_inv < 2048
    out, st = oracle.qflash_attention(Q, K, V, p, 16, return_state=True)
    assert st["violations"] == 0
    ref = oracle.float_attention_ratio(Q, K, V, sQ, sK)
    assert cosine(st["O_acc"] / st["l"][..., None], ref) >= 0.995


def test_row_constant_bias_changes_nothing():
    Q, K, V, sQ, sK, _ = rand_case((2, 2, 80, 32), 41)
    p = derive_params(sQ, sK, 32)
    rng = np.random.default_rng(2)
    rowc = rng.integers(-5000, 5000, size=(2, 2, 80, 1)).astype(np.int32)
    bias = np.broadcast_to(rowc, (2, 2, 80, 80)).copy()
    assert np.array_equal(oracle.qflash_attention(Q, K, V, p, 32, bias=bias),
                          oracle.qflash_attention(Q, K, V, p, 32))


def test_bias_enters_the_score():
    """Single tile with a random bias equals the brute force with the bias added to S, and tracks
    float softmax with the same (real) bias."""
    Q, K, V, sQ, sK, _ = rand_case((2, 3, 49, 32), 43, q_gain=1.5)
    p = derive_params(sQ, sK, 32)
    rng = np.random.default_rng(3)
    unit = sQ * sK / np.sqrt(32.0)
    bias_real = rng.standard_normal((2, 3, 49, 49)) * 0.5
    bias = np.floor(bias_real / unit + 0.5).astype(np.int32)
    out, st = oracle.qflash_attention(Q, K, V, p, 64, bias=bias, return_state=True)
    assert np.array_equal(out, oracle.fullrow_int_attention(Q, K, V, p, bias=bias))
    ref = oracle.float_attention_ratio(Q, K, V, sQ, sK, bias_real=bias * unit)
    assert cosine(st["O_acc"] / st["l"][..., None], ref) >= 0.998
    assert not np.array_equal(out, oracle.qflash_attention(Q, K, V, p, 64))
    # bias broadcasting over batch: [1,3,N,N] indexed with b % 1
    out_b = oracle.qflash_attention(Q, K, V, p, 64, bias=bias[:1])
    assert np.array_equal(out_b[0], out[0])
    assert np.array_equal(out_b[1], oracle.qflash_attention(Q[1:], K[1:], V[1:], p, 64, bias=bias[:1])[0])


def test_excluded_column_equals_deleted_key():
    """Single tile: excluding key c for all queries gives the same result as deleting key/value c."""
    Q, K, V, sQ, sK, _ = rand_case((1, 2, 49, 32), 47)
    p = derive_params(sQ, sK, 32)
    drop = [0, 17, 48]
    bias = np.zeros((1, 1, 49, 49), dtype=np.int32)
    bias[..., drop] = EXCLUDED
    keep = [c for c in range(49) if c not in drop]
    a = oracle.qflash_attention(Q, K, V, p, 64, bias=bias)
    # same queries, keys/values without the dropped ones: run the brute force on rectangular S
    Kd, Vd = K[:, :, keep], V[:, :, keep]
    S = Q.astype(np.int64) @ Kd.astype(np.int64).transpose(0, 1, 3, 2)
    P = oracle.requant_np(oracle.shift_exp2_np(S - S.max(-1, keepdims=True), p), p)
    ref = np.clip((P @ Vd.astype(np.int64)) // P.sum(-1, keepdims=True), -128, 127).astype(np.int8)
    assert np.array_equal(a, ref)


def test_excluded_multi_tile_and_fully_excluded_rows():
    """Several tiles: exclusion = weight 0 and no part in the maximum; a row with every column
    excluded returns 0; a tile with every column excluded leaves the state untouched."""
    Q, K, V, sQ, sK, _ = rand_case((1, 1, 40, 32), 49)
    p = derive_params(sQ, sK, 32)
    bias = np.zeros((1, 1, 40, 40), dtype=np.int32)
    bias[0, 0, 5, :] = EXCLUDED                    # row 5: nothing to attend to
    bias[0, 0, 6, :16] = EXCLUDED                  # row 6: first two tiles (of 8) empty
    bias[0, 0, 7, 8:16] = EXCLUDED                 # row 7: second tile empty
    bias[0, 0, 8, 39] = EXCLUDED
    out, st = oracle.qflash_attention(Q, K, V, p, 8, bias=bias, return_state=True)
    assert np.all(out[0, 0, 5] == 0) and st["l"][0, 0, 5] == 0
    # Deleting the excluded keys keeps every other tile boundary in these three rows (whole
    # leading tiles, a whole middle tile, the last column), so the results must be identical.
    for row, cols in ((6, range(16, 40)), (7, [c for c in range(40) if not 8 <= c < 16]),
                      (8, range(0, 39))):
        cols = list(cols)
        rows = [row] + [r for r in range(40) if r != row][:len(cols) - 1]   # square problem
        sub = oracle.qflash_attention(Q[:, :, rows], K[:, :, cols], V[:, :, cols], p, 8)
        assert np.array_equal(out[0, 0, row], sub[0, 0, 0])


def test_swin_workload_bias_recipe_single_tile():
    wl = make_workload("swin_t_s1_b64", batch=4)
    assert wl.bias.shape == (64, 3, 49, 49) and wl.bias.dtype == np.int32
    assert wl.excluded[0].sum() == 0 and wl.excluded[1].sum() > 0
    p = derive_params(wl.sQ, wl.sK, 32)
    out, st = oracle.qflash_attention(wl.Q, wl.K, wl.V, p, 64, bias=wl.bias, return_state=True)
    assert np.array_equal(out, oracle.fullrow_int_attention(wl.Q, wl.K, wl.V, p, bias=wl.bias))
    B = wl.Q.shape[0]
    ref = oracle.float_attention_ratio(wl.Q, wl.K, wl.V, wl.sQ, wl.sK,
                                       bias_real=wl.bias_real[np.arange(B) % 64],
                                       excluded=wl.excluded[np.arange(B) % 64])
    assert cosine(st["O_acc"] / st["l"][..., None], ref) >= 0.995


# ------------------------------------------------------------------ invariants


@pytest.mark.parametrize("name,batch", [("deit_tiny_b1", 1), ("vit_b16_b64", 1),
                                        ("deit_b384_b32", 1), ("vit_l384_heavy", 1)])
def test_invariants_on_workload_shapes(name, batch):
    wl = make_workload(name, batch=batch)
    B, H, N, d = wl.shape
    sel = slice(0, 2)                                # two heads keep this quick
    Q, K, V = wl.Q[:, sel], wl.K[:, sel], wl.V[:, sel]
    p = derive_params(wl.sQ, wl.sK, d)
    for tile in wl.kv_tiles:
        out, st = oracle.qflash_attention(Q, K, V, p, tile, return_state=True)
        assert st["violations"] == 0
        assert st["l"].min() >= 126 and st["l"].max() <= 127 * N
        assert np.abs(st["O_acc"]).max() <= 128 * 127 * N
        S = Q.astype(np.int64) @ K.astype(np.int64).transpose(0, 1, 3, 2)
        assert np.array_equal(st["m"], S.max(-1))
        assert np.array_equal(out, np.clip(st["O_acc"] // st["l"][..., None], -128, 127))
        ref = oracle.float_attention_ratio(Q, K, V, wl.sQ, wl.sK)
        assert cosine(st["O_acc"] / st["l"][..., None], ref) >= 0.99


def test_result_does_not_depend_on_thread_count_or_batching():
    Q, K, V, sQ, sK, _ = rand_case((3, 2, 70, 32), 61)
    p = derive_params(sQ, sK, 32)
    a = oracle.qflash_attention(Q, K, V, p, 32, nthreads=1)
    b = oracle.qflash_attention(Q, K, V, p, 32, nthreads=4)
    c = np.stack([oracle.qflash_attention(Q[i:i + 1], K[i:i + 1], V[i:i + 1], p, 32)[0]
                  for i in range(3)])
    assert np.array_equal(a, b) and np.array_equal(a, c)


# ------------------------------------------------------------- per-head constants (Appendix C3)


def test_per_head_constants_equal_head_by_head_runs():
    """With one set of constants per head, head h must be exactly what the per-tensor routine
    gives on the slice [:, h] with constants h: pins the head indexing (and nothing else is new).
    Heads differ strongly in scale, one of them needs x_shift > 0; bias with bias_H = H and = 1."""
    rng = np.random.default_rng(77)
    B, H, N, d, tile = 2, 4, 150, 32, 64
    Q, K, V = (rng.integers(-127, 128, size=(B, H, N, d)).astype(np.int8) for _ in range(3))
    sQ = [0.004, 0.02, 0.11, 2.5]
    ps = [derive_params(sQ[h], 0.03 * (h + 1), d) for h in range(H)]
    assert len({p.s_inv for p in ps}) == H and ps[-1].x_shift > 0 and ps[0].x_shift == 0
    for bias_H in (None, H, 1):
        bias = None
        if bias_H is not None:
            bias = rng.integers(-2000, 2000, size=(1, bias_H, N, N)).astype(np.int32)
            bias[0, :, :, 5] = EXCLUDED
        got = oracle.qflash_attention(Q, K, V, ps, tile, bias=bias)
        for h in range(H):
            bh = None if bias is None else bias[:, (h % bias_H):(h % bias_H) + 1]
            want = oracle.qflash_attention(Q[:, h:h + 1], K[:, h:h + 1], V[:, h:h + 1], ps[h], tile, bias=bh)
            assert np.array_equal(got[:, h:h + 1], want), (bias_H, h)
    # the constants really are per head: a different assignment changes the result
    other = oracle.qflash_attention(Q, K, V, ps[::-1], tile)
    assert not np.array_equal(other, oracle.qflash_attention(Q, K, V, ps, tile))


def test_per_head_with_equal_constants_is_the_per_tensor_result():
    wl = make_workload("deit_tiny_b1")
    p = derive_params(wl.sQ, wl.sK, wl.shape[-1])
    a = oracle.qflash_attention(wl.Q, wl.K, wl.V, p, 64)
    b = oracle.qflash_attention(wl.Q, wl.K, wl.V, [p] * wl.shape[1], 64)
    assert np.array_equal(a, b)
    with pytest.raises(ValueError):
        oracle.qflash_attention(wl.Q, wl.K, wl.V, [p] * (wl.shape[1] - 1), 64)


def test_per_head_quantisation_improves_fidelity_when_heads_differ():
    """The point of per-head scales: heads of different range, quantised per tensor, lose the
    quiet heads; per head they keep them.  Cosine against float softmax attention on the
    dequantised per-head inputs, worst head."""
    from oracle.bruteforce import float_attention
    from workloads import make_qkv, head_gains
    shape = (1, 4, 48, 32)
    Qh, Kh, Vh, sQ, sK, sV, _ = make_qkv(shape, 5, per_head=True, head_gain=head_gains(4))
    ps = [derive_params(sQ[h], sK[h], 32) for h in range(4)]
    out = oracle.qflash_attention(Qh, Kh, Vh, ps, 16)
    for h in range(4):
        ref = float_attention(Qh[:, h:h + 1], Kh[:, h:h + 1], Vh[:, h:h + 1], sQ[h], sK[h], sV[h])[0, 0]
        got = (out[0, h].astype(np.float64) + 0.5) * sV[h]
        cos = float((ref * got).sum() / np.sqrt((ref * ref).sum() * (got * got).sum()))
        assert cos > 0.995, (h, cos)
