"""Pins of the dynamic quantiser (Eq. 1-2 evaluated on the fly) and of the pipeline built on it.

The quantiser is pinned against what Eq. 1-2 fix mathematically (nearest level of the grid
s_X * Z, symmetric range, scale = max|x| / 127) and against the double-precision quantiser the
static workloads use; the pipeline reduces to already pinned functions.
"""
import numpy as np
import pytest

import oracle
from workloads import quantize_per_tensor


def _cases():
    rng = np.random.default_rng(11)
    yield rng.standard_normal(20000).astype(np.float32)
    yield (rng.standard_normal(20000) * 1e-3).astype(np.float32)
    yield (rng.standard_t(3.0, size=20000) * 40.0).astype(np.float32)
    yield np.linspace(-5.0, 5.0, 10001, dtype=np.float32)
    yield np.array([3.0, -3.0, 1.5, -1.5, 0.0], dtype=np.float32)


@pytest.mark.parametrize("x", list(_cases()))
def test_quantiser_is_nearest_level_of_eq2(x):
    q, amax, s = oracle.dynamic_quantize(x)
    assert amax == np.max(np.abs(x)) and s == float(np.float64(amax) / 127.0)
    assert q.dtype == np.int8 and q.min() >= -127 and q.max() <= 127
    assert np.abs(q).max() == 127 and abs(int(q[np.argmax(np.abs(x))])) == 127
    # nearest level: |x - q s| <= s/2, up to the float32 rounding of x * r (relative 2^-23 of 127)
    err = np.abs(x.astype(np.float64) - q.astype(np.float64) * s)
    assert err.max() <= s * (0.5 + 127.0 * 2.0 ** -22)
    # odd symmetry (round half to even is symmetric) and monotonicity
    qn, _, _ = oracle.dynamic_quantize(-x)
    assert np.array_equal(qn, -q)
    order = np.argsort(x, kind="stable")
    assert np.all(np.diff(q[order].astype(np.int32)) >= 0)


def test_quantiser_against_the_double_precision_one():
    """Same levels as the float64 evaluation of Eq. 2 except within float32 rounding of a tie."""
    rng = np.random.default_rng(12)
    x = rng.standard_normal((4, 3, 50, 32)).astype(np.float32)
    q, _, s = oracle.dynamic_quantize(x)
    q64, s64 = quantize_per_tensor(x)
    assert s == s64
    diff = q.astype(np.int32) - q64.astype(np.int32)
    assert np.abs(diff).max() <= 1 and np.mean(diff != 0) < 1e-4


def test_quantiser_hand_values_and_degenerate_input():
    x = np.array([1.0, 0.5, -0.25, 0.0039, -1.0], dtype=np.float32)
    q, amax, s = oracle.dynamic_quantize(x)
    assert list(q) == [127, 64, -32, 0, -127]        # 63.5 -> 64 and -31.75 -> -32 (half to even: 63.5 -> 64)
    q, amax, s = oracle.dynamic_quantize(np.zeros((2, 3), dtype=np.float32))
    assert not q.any() and s == 1.0
    with pytest.raises(ValueError):
        oracle.dynamic_quantize(np.array([1.0, np.inf], dtype=np.float32))


def test_dynamic_pipeline_is_quantise_derive_attend():
    rng = np.random.default_rng(13)
    shape = (2, 3, 90, 32)
    Qf, Kf, Vf = (rng.standard_normal(shape).astype(np.float32) * g for g in (1.0, 1.7, 0.3))
    O, info = oracle.qflash_attention_dynamic(Qf, Kf, Vf, 64)
    Q, _, sQ = oracle.dynamic_quantize(Qf)
    K, _, sK = oracle.dynamic_quantize(Kf)
    V, _, sV = oracle.dynamic_quantize(Vf)
    p = oracle.derive_params(sQ, sK, 32)
    assert info["params"] == p and (info["sQ"], info["sK"], info["sV"]) == (sQ, sK, sV)
    assert np.array_equal(O, oracle.qflash_attention(Q, K, V, p, 64))
    # fidelity of the whole integer pipeline against float softmax attention on the real inputs
    from oracle.bruteforce import float_attention
    ref = float_attention(Qf.astype(np.float64), Kf.astype(np.float64), Vf.astype(np.float64), 1.0, 1.0, 1.0)
    got = (O.astype(np.float64) + 0.5) * sV
    cos = float((ref * got).sum() / np.sqrt((ref * ref).sum() * (got * got).sum()))
    assert cos > 0.99, cos


# ------------------------------------------------- a bias in real units in front of Algorithm 1


def test_bias_conversion_hand_values():
    """sQ = sK = 0.25, d = 64: one integer score unit is 0.0625 / 8 = 2^-7, so b_hat = b * 128
    rounded half up -- exact in binary."""
    b = np.array([[[[0.0, 1.0, -1.0, 0.00390625, -0.00390625, 0.01171875, -0.01171875, 3.3]]]], dtype=np.float32)
    got = oracle.dynamic_bias_to_int(np.broadcast_to(b, (1, 1, 8, 8)).copy(), None, 0.25, 0.25, 64)[0, 0, 0]
    # 0.00390625 * 128 = 0.5 -> 1 (half up), -0.5 -> 0 (half up), 1.5 -> 2, -1.5 -> -1; float32(3.3) * 128 = 422.4
    assert list(got) == [0, 128, -128, 1, 0, 2, -1, 422]
    # the exclusion mask wins over any value; the range is clipped to +-(2^20 - 1)
    big = np.full((1, 1, 2, 2), 1e9, dtype=np.float32)
    big[0, 0, 1, 1] = -1e9
    mask = np.zeros((1, 1, 2, 2), dtype=np.uint8)
    mask[0, 0, 0, 1] = 1
    got = oracle.dynamic_bias_to_int(big, mask, 0.25, 0.25, 64)
    assert got[0, 0, 0, 0] == (1 << 20) - 1 and got[0, 0, 1, 1] == -((1 << 20) - 1)
    assert got[0, 0, 0, 1] == np.iinfo(np.int32).min
    # a mask alone is a bias of zeros with exclusions; nothing at all is no bias
    got = oracle.dynamic_bias_to_int(None, mask, 0.25, 0.25, 64)
    assert got[0, 0, 0, 1] == np.iinfo(np.int32).min and np.count_nonzero(got) == 1
    assert oracle.dynamic_bias_to_int(None, None, 0.25, 0.25, 64) is None


@pytest.mark.parametrize("sQ,sK,d", [(0.031, 0.027, 32), (0.0123, 0.045, 64), (1e-3, 2e-3, 32)])
def test_bias_conversion_is_the_nearest_score_unit(sQ, sK, d):
    rng = np.random.default_rng(5)
    b = (rng.standard_normal((2, 3, 20, 20)) * 0.7).astype(np.float32)
    unit = sQ * sK / np.sqrt(float(d))
    got = oracle.dynamic_bias_to_int(b, None, sQ, sK, d).astype(np.float64)
    if np.abs(b).max() / unit < (1 << 20) - 2:
        assert np.abs(got * unit - b.astype(np.float64)).max() <= unit * (0.5 + 1e-9)
    # the host recipe of the static windowed workloads (same formula on float64 values)
    ref = np.floor(b.astype(np.float64) / unit + 0.5)
    assert np.array_equal(got, np.clip(ref, -(2 ** 20 - 1), 2 ** 20 - 1))


def test_dynamic_pipeline_with_bias_and_mask():
    """Windowed workload from float inputs: the pipeline is quantise -> derive -> convert the bias
    with the scales just found -> Algorithm 1; an excluded key equals a deleted key; the result
    tracks float softmax attention with the real bias."""
    from workloads import make_float_qkv, make_float_window_bias
    Qf, Kf, Vf = make_float_qkv("swin_t_s1_b64", batch=6)
    bias_real, excluded = make_float_window_bias("swin_t_s1_b64", n_windows=2)
    O, info = oracle.qflash_attention_dynamic(Qf, Kf, Vf, 64, bias_real=bias_real, excluded=excluded)
    Q, _, sQ = oracle.dynamic_quantize(Qf)
    K, _, sK = oracle.dynamic_quantize(Kf)
    V, _, sV = oracle.dynamic_quantize(Vf)
    p = oracle.derive_params(sQ, sK, 32)
    bias = oracle.dynamic_bias_to_int(bias_real, excluded, sQ, sK, 32)
    assert np.array_equal(info["bias"], bias) and (bias == np.iinfo(np.int32).min).mean() > 0.1
    assert np.array_equal(O, oracle.qflash_attention(Q, K, V, p, 64, bias=bias))
    from oracle.bruteforce import float_attention
    B, H = Qf.shape[:2]
    br = np.broadcast_to(bias_real[np.arange(B) % 2], (B, H, 49, 49)).astype(np.float64)
    ex = np.broadcast_to(excluded[np.arange(B) % 2], (B, H, 49, 49)) != 0
    ref = float_attention(Qf.astype(np.float64), Kf.astype(np.float64), Vf.astype(np.float64), 1.0, 1.0, 1.0,
                          bias_real=br, excluded=ex)
    got = (O.astype(np.float64) + 0.5) * sV
    cos = float((ref * got).sum() / np.sqrt((ref * ref).sum() * (got * got).sum()))
    assert cos > 0.99, cos
    # without the bias the result is a different one (the bias does enter)
    O0, _ = oracle.qflash_attention_dynamic(Qf, Kf, Vf, 64)
    assert not np.array_equal(O, O0)
