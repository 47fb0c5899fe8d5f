"""Dynamic per-tensor quantisation in front of Algorithm 1 (oracle side; test infrastructure).

The paper quantises activations on the fly (Section 5, evaluation set-up) with Eq. 1-2:
``s_X = max|X| / (2^(b-1) - 1)`` and ``X_hat = round(X / s_X)``, b = 8.  It fixes no arithmetic
precision for this step.  Reading frozen here (both sides take the rounding decision in the
same precision, float32, the type the activations arrive in):

    amax = max |x|                          exact in any order
    r    = float32(127) / amax              one correctly rounded float32 division
    x_hat = clip(rint(x * r), -127, 127)    one float32 multiplication, round-half-to-even
    s_X  = double(amax) / 127.0             the scale handed to the constant derivation

An all-zero tensor gives x_hat = 0 and s_X = 1.  Inputs are finite.

A bias given in real units (windowed attention: relative-position bias, exclusion mask) has to be
brought to the unit of the integer score Q_hat K_hat^T, which with on-the-fly scales is only known
after the abs-max step.  The paper adds the bias to S inside Algorithm 1 without fixing how it is
quantised; reading frozen here (float64, the precision the scales are held in):

    unit  = (s_Q * s_K) / sqrt(d)                    real value of one integer score unit
    b_hat = clip(floor(double(b) / unit + 0.5), -(2^20 - 1), 2^20 - 1)     round half up
    excluded pairs (mask != 0) take no part (the exclusion mark of Algorithm 1's bias)

which is what the static workloads do on the host with their known scales.
"""
from __future__ import annotations

import numpy as np

import math

from .params import derive_params
from .cbinding import qflash_attention

EXCLUDED = np.iinfo(np.int32).min
BIAS_LIMIT = (1 << 20) - 1


def dynamic_quantize(x):
    """Eq. 1-2 on a float32 array: returns (int8 array, amax as float32, scale as Python float)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    amax = np.float32(np.max(np.abs(x))) if x.size else np.float32(0.0)
    if not np.isfinite(amax):
        raise ValueError("inputs must be finite")
    if amax == np.float32(0.0):
        return np.zeros(x.shape, dtype=np.int8), amax, 1.0
    r = np.float32(127.0) / amax                       # float32 division
    y = np.rint(x * r)                                 # float32 multiply, then round half to even
    q = np.clip(y, np.float32(-127.0), np.float32(127.0)).astype(np.int8)
    return q, amax, float(np.float64(amax) / 127.0)


def dynamic_bias_to_int(bias_real, excluded, sQ: float, sK: float, d: int):
    """Real bias (float32 [bias_B,bias_H,N,N] or None) and exclusion mask (same shape, nonzero =
    excluded, or None) -> int32 bias of Algorithm 1 in units of the integer score, for the scales
    sQ, sK (Python floats, i.e. float64) and head size d."""
    if bias_real is None and excluded is None:
        return None
    shape = (bias_real if bias_real is not None else excluded).shape
    unit = (float(sQ) * float(sK)) / math.sqrt(float(d))
    if bias_real is None:
        b = np.zeros(shape, dtype=np.float64)
    else:
        b = np.asarray(bias_real, dtype=np.float32).astype(np.float64)
        if not np.all(np.isfinite(b)):
            raise ValueError("bias must be finite")
    t = np.floor(b / unit + 0.5)
    out = np.clip(t, -float(BIAS_LIMIT), float(BIAS_LIMIT)).astype(np.int32)
    if excluded is not None:
        out = np.where(np.asarray(excluded) != 0, np.int32(EXCLUDED), out)
    return np.ascontiguousarray(out, dtype=np.int32)


def qflash_attention_dynamic(Qf, Kf, Vf, kv_tile: int, out_round: int = 0, nthreads: int = 0,
                             bias_real=None, excluded=None):
    """Quantise Q, K, V per tensor, derive the integer constants from the scales, bring the real
    bias (if any) to the integer score unit of those scales, run Algorithm 1.

    Returns (O int8 [B,H,N,d], dict(sQ, sK, sV, params, Q, K, V, bias)); O has scale sV.
    Raises ValueError when the scales fall outside the supported window (see derive_params).
    """
    Q, _, sQ = dynamic_quantize(Qf)
    K, _, sK = dynamic_quantize(Kf)
    V, _, sV = dynamic_quantize(Vf)
    p = derive_params(sQ, sK, Q.shape[-1], out_round=out_round)
    bias = dynamic_bias_to_int(bias_real, excluded, sQ, sK, Q.shape[-1])
    O = qflash_attention(Q, K, V, p, kv_tile, bias=bias, nthreads=nthreads)
    return O, {"sQ": sQ, "sK": sK, "sV": sV, "params": p, "Q": Q, "K": K, "V": V, "bias": bias}
