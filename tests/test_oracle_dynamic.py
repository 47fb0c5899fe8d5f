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
