"""Pins for the scalar building blocks of the CPU oracle (no GPU).

Each test ties a function of the oracle to something fixed by the paper or by
mathematics: the closed form 2^x and the error of its linear fraction (Eq. 5-8),
the division form of the quotient (Appendix B.2), the requantisation range
(Eq. 9-10), floor semantics of ">>".
"""
import math

import numpy as np
import pytest

import oracle
from oracle.params import OracleParams, derive_params, score_scale, requant_constants

# (1 + f/2) / 2^f is largest at f = 1/ln2 - 2: the linear fraction of Eq. 7 never
# undershoots 2^f on (-1, 0] and overshoots by at most this factor.
LIN_MAX = (1 + (1 / math.log(2) - 2) / 2) / 2 ** (1 / math.log(2) - 2)


def exact_params(s_inv=1024, k=0):
    """Constants for a score scale of exactly 2^k / s_inv (no rounding anywhere)."""
    p_mul, p_shift = requant_constants(s_inv)
    return OracleParams(k, s_inv, -((1 << 32) // s_inv), 32, p_mul, p_shift,
                        -((-(1 << 30)) // s_inv), 0)


SCALE_CASES = [(0.037, 0.036, 64), (0.05, 0.06, 64), (0.04, 0.035, 32), (0.02, 0.025, 64),
               (3.1, 4.2, 64), (0.9, 1.3, 32), (0.011, 0.012, 64)]


def test_lin_max_constant():
    assert abs(LIN_MAX - 1.0615) < 1e-4


def test_hand_worked_shift_exp2():
    # s = 1/1024: x = -1536 is the exponent -1.5 = -1 + (-0.5).
    # q = 1, r = -1536 + 1024 = -512, y = ((-512 >> 1) + 1024) >> 1 = 384 = 1024 * (1 - 0.25) / 2.
    p = exact_params(1024)
    assert oracle.shift_exp2_quotient(-1536, p) == 1
    assert oracle.shift_exp2(-1536, p) == 384
    # exact powers of two: x = -n * 1024 -> 1024 >> n
    for n in range(0, 11):
        assert oracle.shift_exp2(-1024 * n, p) == 1024 >> n
    # x = -1 : q = 0 (product 2^22 < 2^32), r = -1, (r >> 1) = -1 (floor), y = 1023
    assert oracle.shift_exp2(-1, p) == 1023
    # far below: y = 0, and the q > 31 rule
    assert oracle.shift_exp2(-1024 * 31, p) == 0
    assert oracle.shift_exp2(-1024 * 40, p) == 0
    assert oracle.shift_exp2(-(1 << 22), p) == 0


def test_hand_worked_with_x_shift():
    # k = 3: x is multiplied by 8 first; x = -192 -> x' = -1536, same as above.
    p = exact_params(1024, k=3)
    assert oracle.shift_exp2(-192, p) == 384
    assert oracle.shift_exp2(0, p) == 1024


@pytest.mark.parametrize("sQ,sK,d", SCALE_CASES)
def test_params_closed_form(sQ, sK, d):
    p = derive_params(sQ, sK, d)
    s = sQ * sK / math.sqrt(d) * math.log2(math.e)
    assert abs(score_scale(sQ, sK, d) - s) < 1e-15 * max(1.0, s)
    s_k = s / 2 ** p.x_shift
    # s_inv is 1/s' to the nearest integer, inside the supported window, k minimal
    assert abs(p.s_inv - 1 / s_k) <= 0.5
    assert 1024 <= p.s_inv < (1 << 18)
    if p.x_shift > 0:
        assert math.floor(2 ** (p.x_shift - 1) / s + 0.5) < 1024
    # M is -s' * 2^32 to the nearest integer
    assert p.exp_shift == 32
    assert abs(p.exp_mul + s_k * 2 ** 32) <= 0.5 and p.exp_mul < 0
    # Eq. 9-10 with ratio 127/s_inv and b = 8
    rho = 127 / p.s_inv
    n = math.floor(math.log2(rho))
    assert p.p_shift == 8 - n
    assert abs(p.p_mul - rho * 2 ** p.p_shift) <= 0.5
    assert 256 <= p.p_mul <= 512
    assert 2 ** p.p_shift > 2 * p.s_inv
    # alpha multiplier
    assert p.a_mul == math.ceil(2 ** 30 / p.s_inv)


def test_params_reject_out_of_range():
    with pytest.raises(ValueError):
        derive_params(1e-4, 1e-4, 64)          # s_inv far above 2^18
    with pytest.raises(ValueError):
        derive_params(0.0, 1.0, 64)
    with pytest.raises(ValueError):
        derive_params(3000.0, 3000.0, 64)      # needs x_shift > 16


@pytest.mark.parametrize("sQ,sK,d", SCALE_CASES)
def test_shift_exp2_against_two_to_the_x(sQ, sK, d):
    """y / s_inv lies between 2^u and LIN_MAX * 2^u (u = s x), up to floors and constant rounding."""
    p = derive_params(sQ, sK, d)
    s = score_scale(sQ, sK, d)
    span = int(14 / s) + 2                      # down to 2^-14
    xs = np.unique(np.concatenate([
        -np.arange(0, min(span, 20000)),
        -np.linspace(0, span, 4000).astype(np.int64)]))
    ys = np.array([oracle.shift_exp2(int(x), p) for x in xs], dtype=np.float64)
    true = p.s_inv * np.exp2(s * xs.astype(np.float64))
    assert np.all(ys >= true * (1 - 0.01) - 2.0)
    assert np.all(ys <= true * LIN_MAX * (1 + 0.01) + 2.0)
    assert oracle.shift_exp2(0, p) == p.s_inv
    assert ys.min() >= 0 and ys.max() == p.s_inv
    # the approximation really is the chord: at the midpoint of an octave the value
    # is close to 0.75 * 2^-n, not to 2^-0.5 * 2^-n
    if 1.5 / s > 200:                           # needs an integer x close to the midpoint
        x_mid = -int(round(1.5 / s))
        assert abs(oracle.shift_exp2(x_mid, p) / p.s_inv - 0.375) < 0.004


@pytest.mark.parametrize("sQ,sK,d", SCALE_CASES)
def test_quotient_against_division_form(sQ, sK, d):
    """mul+shift quotient vs q = floor(x' / -s_inv): never more than 1 apart, nearly always equal."""
    p = derive_params(sQ, sK, d)
    rng = np.random.default_rng(5)
    hi = 20 * p.s_inv >> p.x_shift
    xs = -rng.integers(0, hi + 1, size=6000)
    q_ms = np.array([oracle.shift_exp2_quotient(int(x), p) for x in xs])
    q_div = np.array([(int(x) << p.x_shift) // -p.s_inv if x != 0 else 0 for x in xs])
    assert np.all(q_ms >= 0)
    assert np.all(np.abs(q_ms - q_div) <= 1)
    assert np.mean(q_ms == q_div) > 0.99
    # where the two agree the remainder is a true remainder and the result is the I-ViT form
    for x, q in zip(xs[:500], q_ms[:500]):
        xs_ = int(x) << p.x_shift
        if q == xs_ // -p.s_inv and q <= 31:
            r = xs_ + int(q) * p.s_inv
            assert -p.s_inv < r <= 0
            assert oracle.shift_exp2(int(x), p) == ((r >> 1) + p.s_inv) >> int(q)


@pytest.mark.parametrize("sQ,sK,d", SCALE_CASES[:4])
def test_shift_exp2_monotone_inside_octaves(sQ, sK, d):
    p = derive_params(sQ, sK, d)
    xs = -np.arange(0, 9 * p.s_inv >> p.x_shift)
    q = np.array([oracle.shift_exp2_quotient(int(x), p) for x in xs])
    y = np.array([oracle.shift_exp2(int(x), p) for x in xs])
    same = q[1:] == q[:-1]
    assert np.all(y[1:][same] <= y[:-1][same])
    # and over octave boundaries it never rises by more than the rounding wobble
    assert np.all(y[1:] <= y[:-1] + 2)


@pytest.mark.parametrize("sQ,sK,d", SCALE_CASES)
def test_numpy_and_c_shift_exp2_agree(sQ, sK, d):
    p = derive_params(sQ, sK, d)
    rng = np.random.default_rng(11)
    xs = -rng.integers(0, 1 << 22, size=3000)
    xs[:64] = -np.arange(64)
    y_c = np.array([oracle.shift_exp2(int(x), p) for x in xs])
    assert np.array_equal(y_c, oracle.shift_exp2_np(xs, p))


@pytest.mark.parametrize("sQ,sK,d", SCALE_CASES)
def test_requant_range(sQ, sK, d):
    p = derive_params(sQ, sK, d)
    ys = np.arange(0, p.s_inv + 1)
    P = np.array([oracle.requant(int(y), p) for y in ys])
    assert P[0] == 0 and P[-1] in (126, 127)
    assert P.min() >= 0 and P.max() <= 127
    assert np.all(np.diff(P) >= 0)
    # 1.0 <-> 127: P = floor(y*rho +- y/2^(r+1)) with y/2^(r+1) < 1/4
    d = P - ys * 127.0 / p.s_inv
    assert np.all(d > -1.25) and np.all(d <= 0.25)
    assert np.array_equal(P, oracle.requant_np(ys, p))
    assert oracle.requant(10 * p.s_inv, p) == 127          # saturates


@pytest.mark.parametrize("sQ,sK,d", SCALE_CASES)
def test_alpha16(sQ, sK, d):
    p = derive_params(sQ, sK, d)
    assert oracle.alpha16(p.s_inv, p) == 65536             # unchanged maximum: exact identity
    assert oracle.alpha16(0, p) == 0
    a = np.array([oracle.alpha16(int(v), p) for v in range(0, p.s_inv + 1)])
    assert np.all(np.diff(a) >= 0)
    ideal = np.arange(0, p.s_inv + 1) * 65536.0 / p.s_inv
    assert np.all(a >= np.floor(ideal) - 1e-9) and np.all(a <= ideal + 65536.0 / 16384 + 1)
    assert p.s_inv * p.a_mul < 2 ** 31


def test_scale_release_is_floor():
    assert oracle.scale_release(1000, 65536) == 1000
    assert oracle.scale_release(-1000, 65536) == -1000
    assert oracle.scale_release(-1, 32768) == -1            # floor(-0.5), not truncation
    assert oracle.scale_release(1, 32768) == 0
    assert oracle.scale_release(-3, 32768) == -2
    assert oracle.scale_release(12345, 0) == 0
    rng = np.random.default_rng(3)
    for acc, a in zip(rng.integers(-2 ** 26, 2 ** 26, 200), rng.integers(0, 65537, 200)):
        assert oracle.scale_release(int(acc), int(a)) == (int(acc) * int(a)) // 65536
