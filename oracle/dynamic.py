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
"""
from __future__ import annotations

import numpy as np

from .params import derive_params
from .cbinding import qflash_attention


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


def qflash_attention_dynamic(Qf, Kf, Vf, kv_tile: int, out_round: int = 0, nthreads: int = 0):
    """Quantise Q, K, V per tensor, derive the integer constants from the scales, run Algorithm 1.

    Returns (O int8 [B,H,N,d], dict(sQ, sK, sV, params, Q, K, V)); O has scale sV.
    Raises ValueError when the scales fall outside the supported window (see derive_params).
    """
    Q, _, sQ = dynamic_quantize(Qf)
    K, _, sK = dynamic_quantize(Kf)
    V, _, sV = dynamic_quantize(Vf)
    p = derive_params(sQ, sK, Q.shape[-1], out_round=out_round)
    O = qflash_attention(Q, K, V, p, kv_tile, nthreads=nthreads)
    return O, {"sQ": sQ, "sK": sK, "sV": sV, "params": p, "Q": Q, "K": K, "V": V}
