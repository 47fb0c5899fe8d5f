"""Brute-force references on whole rows (NumPy; test infrastructure).

These are the plain definitions the tile-wise algorithm is compared with on
small inputs: an integer softmax over the complete score row (no tiling, so no
rescaling of past accumulators happens), and exact softmax attention in float64
on the dequantised integer inputs.
"""
from __future__ import annotations

import numpy as np

from .params import OracleParams, score_scale

EXCLUDED = np.iinfo(np.int32).min


def _asr(v, n):
    """floor(v / 2^n) on int64 arrays (NumPy's >> on signed integers is arithmetic)."""
    return np.right_shift(v, n)


def shift_exp2_np(x, p: OracleParams):
    """Algorithm 2 on an int64 array of non-positive inputs; 1.0 <-> s_inv."""
    x = np.asarray(x, dtype=np.int64)
    xs = x * (1 << p.x_shift)
    q = _asr(xs * np.int64(p.exp_mul), p.exp_shift)
    r = xs + q * np.int64(p.s_inv)
    qc = np.minimum(q, 62)
    y = _asr(_asr(r, 1) + np.int64(p.s_inv), qc)
    return np.where(q > 31, 0, y)


def requant_np(y, p: OracleParams):
    """Eq. 10 with 1.0 <-> 127, saturated at 127."""
    return np.minimum(_asr(np.asarray(y, dtype=np.int64) * np.int64(p.p_mul), p.p_shift), 127)


def _scores(Q, K, bias):
    S = np.einsum("bhid,bhcd->bhic", Q.astype(np.int64), K.astype(np.int64))
    excl = np.zeros(S.shape, dtype=bool)
    if bias is not None:
        B, H = Q.shape[:2]
        bb = np.asarray(bias, dtype=np.int64)
        bsel = bb[np.arange(B) % bb.shape[0]][:, np.arange(H) % bb.shape[1]]
        excl = bsel == EXCLUDED
        S = S + np.where(excl, 0, bsel)
    return S, excl


def fullrow_int_attention(Q, K, V, p: OracleParams, bias=None, return_state=False):
    """Integer softmax attention with the maximum taken over the whole row.

    P = requant(ShiftExp2(S - rowmax)), out = clamp(floor(P V / sum P)).  This
    is what Algorithm 1 computes when there is a single KV tile.
    """
    S, excl = _scores(Q, K, bias)
    Sm = np.where(excl, np.int64(-(1 << 21)), S)
    m = np.maximum(Sm.max(axis=-1, keepdims=True), -(1 << 21))
    P = requant_np(shift_exp2_np(np.minimum(S - m, 0), p), p)
    P = np.where(excl, 0, P)
    l = P.sum(axis=-1, keepdims=True)
    acc = np.einsum("bhic,bhcd->bhid", P, V.astype(np.int64))
    safe_l = np.where(l == 0, 1, l)
    if p.out_round:
        out = np.floor_divide(2 * acc + safe_l, 2 * safe_l)
    else:
        out = np.floor_divide(acc, safe_l)
    out = np.where(l == 0, 0, np.clip(out, -128, 127)).astype(np.int8)
    if return_state:
        return out, {"O_acc": acc, "l": l[..., 0], "m": m[..., 0], "P": P}
    return out


def fullrow_int_attention_qmax(Q, K, V, p: OracleParams, bias=None, return_state=False):
    """The whole-row definition of the quantised-maximum variant (not the paper's): the reference
    level is the row maximum (never below the initial maximum -2^21) rounded up to a whole number
    of octaves, L = ceil(max * 2^k / s_inv); weights are Algorithm 2 (from the quotient step on)
    and Eq. 10 applied to S * 2^k - L * s_inv; out = clamp(floor(P V / sum P))."""
    S, excl = _scores(Q, K, bias)
    Sm = np.where(excl, np.int64(-(1 << 21)), S)
    m = np.maximum(Sm.max(axis=-1, keepdims=True), -(1 << 21))
    s_inv = np.int64(p.s_inv)
    L = -np.floor_divide(-(m << p.x_shift), s_inv)
    xs = np.minimum((S << p.x_shift) - L * s_inv, 0)
    q = _asr(xs * np.int64(p.exp_mul), p.exp_shift)
    y = np.where(q > 31, 0, _asr(_asr(xs + q * s_inv, 1) + s_inv, np.minimum(q, 62)))
    P = np.where(excl, 0, requant_np(y, p))
    l = P.sum(axis=-1, keepdims=True)
    acc = np.einsum("bhic,bhcd->bhid", P, V.astype(np.int64))
    safe_l = np.where(l == 0, 1, l)
    if p.out_round:
        out = np.floor_divide(2 * acc + safe_l, 2 * safe_l)
    else:
        out = np.floor_divide(acc, safe_l)
    out = np.where(l == 0, 0, np.clip(out, -128, 127)).astype(np.int8)
    if return_state:
        return out, {"O_acc": acc, "l": l[..., 0], "m": L[..., 0], "P": P}
    return out


def float_attention_ratio(Q, K, V, sQ, sK, bias_real=None, excluded=None):
    """softmax(Q K^T sQ sK / sqrt(d) [+ bias]) V in float64, in units of s_V (not rounded)."""
    d = Q.shape[-1]
    S = np.einsum("bhid,bhcd->bhic", Q.astype(np.float64), K.astype(np.float64))
    S = S * (sQ * sK / np.sqrt(float(d)))
    if bias_real is not None:
        S = S + bias_real
    if excluded is not None:
        S = np.where(excluded, -np.inf, S)
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    W = E / E.sum(axis=-1, keepdims=True)
    return np.einsum("bhic,bhcd->bhid", W, V.astype(np.float64))


def float_attention(Q, K, V, sQ, sK, sV, bias_real=None, excluded=None):
    """Exact softmax attention on the dequantised int8 inputs, in real units."""
    return float_attention_ratio(Q, K, V, sQ, sK, bias_real, excluded) * sV


__all__ = ["shift_exp2_np", "requant_np", "fullrow_int_attention", "fullrow_int_attention_qmax", "float_attention",
           "float_attention_ratio", "score_scale"]
