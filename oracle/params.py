"""Host-side integer constants of the QFlash kernel (oracle side; test infrastructure).

Everything the kernel consumes is an integer that depends only on the real
scales, so it is computed once outside the kernel (Section 4.3 after Eq. 7,
Section 4.4 after Eq. 10, Algorithm 1 "Require").

Readings of open points (R-numbers as in the design document):

R1   the fixed-point width N of ``M = round(-s * 2^N)`` (Appendix B.2) is 32.
R5   when the score scale ``s`` is coarse, ``round(1/s)`` collapses towards 0
     and Algorithm 2 loses all resolution.  Scores are therefore multiplied by
     ``2^k`` first and ``s`` divided by ``2^k``; ``k`` is the smallest value
     >= 0 with ``round(2^k / s) >= 1024``.  The function approximated,
     ``2^(s x)``, is unchanged.  ``k = 0`` is the paper as printed.
R6   ScaleRelease needs alpha (1.0 <-> s_inv) brought to a fixed scale; it is
     requantised to 16 fractional bits with the multiplier ``ceil(2^30/s_inv)``.
R7   the int8 weight P has 1.0 <-> 127: Eq. 9-10 with s_X/s_Y = 127/s_inv, b = 8.
R13  ``round`` on real numbers is ``floor(x + 0.5)``.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, astuple

LOG2_E = 1.4426950408889634  # log2(e) in IEEE double
EXP_SHIFT = 32
S_INV_MIN = 1 << 10
S_INV_MAX = 1 << 18          # exclusive
X_SHIFT_MAX = 16          # the range of k the interface of the method allows (the HIP library stops at 13)


@dataclass(frozen=True)
class OracleParams:
    x_shift: int
    s_inv: int
    exp_mul: int
    exp_shift: int
    p_mul: int
    p_shift: int
    a_mul: int
    out_round: int = 0

    def astuple(self):
        return astuple(self)


def _round_half_up(x: float) -> int:
    return int(math.floor(x + 0.5))


def score_scale(sQ: float, sK: float, d: int) -> float:
    """s of Algorithm 1: sQ * sK * d^(-1/2) * log2(e), evaluated left to right in double."""
    return ((sQ * sK) / math.sqrt(float(d))) * LOG2_E


def requant_constants(s_inv: int):
    """(M_r, r) of Eq. 9-10 for the ratio rho = 127 / s_inv and b = 8.

    n = floor(log2(rho)) is found with integers only: 2^n <= 127/s_inv < 2^(n+1).
    M_r = round(rho * 2^r) is also evaluated exactly in integers.
    """
    if s_inv <= 127:
        raise ValueError("s_inv must exceed 127")
    # rho < 1, so n = -e with e > 0 and 2^-e <= 127/s_inv < 2^-(e-1),
    # i.e. e is the smallest integer with 127 * 2^e >= s_inv.
    e = 0
    while 127 * (1 << e) < s_inv:
        e += 1
    n = -e
    r = 8 - n
    m_r = (2 * 127 * (1 << r) + s_inv) // (2 * s_inv)   # floor(127*2^r/s_inv + 1/2)
    return m_r, r


def derive_params(sQ: float, sK: float, d: int, out_round: int = 0, x_shift=None) -> OracleParams:
    """All integer constants of one call from the real scales of Q and K and the head size.

    ``x_shift`` forces k (used by the scaling-identity pin); by default k follows R5.
    Raises ValueError when the scales fall outside what the 32-bit kernel supports.
    """
    if not (sQ > 0.0 and sK > 0.0 and math.isfinite(sQ) and math.isfinite(sK)) or d < 1:
        raise ValueError("scales must be positive and finite, d >= 1")
    s = score_scale(sQ, sK, d)
    if x_shift is None:
        k = 0
        while _round_half_up((2.0 ** k) / s) < S_INV_MIN:
            k += 1
            if k > X_SHIFT_MAX:
                raise ValueError("score scale too coarse: needs x_shift > %d" % X_SHIFT_MAX)
    else:
        k = int(x_shift)
    s_k = s / (2.0 ** k)
    s_inv = _round_half_up(1.0 / s_k)
    if not (S_INV_MIN <= s_inv < S_INV_MAX):
        raise ValueError("s_inv=%d outside [2^10, 2^18)" % s_inv)
    exp_mul = _round_half_up(-s_k * (2.0 ** EXP_SHIFT))
    p_mul, p_shift = requant_constants(s_inv)
    a_mul = -((-(1 << 30)) // s_inv)                     # ceil(2^30 / s_inv)
    return OracleParams(k, s_inv, exp_mul, EXP_SHIFT, p_mul, p_shift, a_mul, int(out_round))
