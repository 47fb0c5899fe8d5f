"""ctypes wrapper around the plain-C oracle (test infrastructure)."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .params import OracleParams

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qflash_oracle.c")
_LIB = os.path.join(_HERE, "libqflash_oracle.so")
_lib = None


class _CParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "x_shift", "s_inv", "exp_mul", "exp_shift", "p_mul", "p_shift", "a_mul", "out_round")]


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP over (batch, head) only)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
             "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        pp = ctypes.POINTER(_CParams)
        lib.oracle_shift_exp2.restype = i64
        lib.oracle_shift_exp2.argtypes = [i64, pp]
        lib.oracle_shift_exp2_quotient.restype = i64
        lib.oracle_shift_exp2_quotient.argtypes = [i64, pp]
        lib.oracle_requant.restype = i64
        lib.oracle_requant.argtypes = [i64, pp]
        lib.oracle_alpha16.restype = i64
        lib.oracle_alpha16.argtypes = [i64, pp]
        lib.oracle_scale_release.restype = i64
        lib.oracle_scale_release.argtypes = [i64, i64]
        lib.oracle_num_threads.restype = ci
        lib.oracle_qflash_attention.restype = ci
        lib.oracle_qflash_attention.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci,
                                                pp, vp, vp, vp, vp, ci]
        lib.oracle_qflash_attention_per_head.restype = ci
        lib.oracle_qflash_attention_per_head.argtypes = lib.oracle_qflash_attention.argtypes
        for name in ("oracle_qflash_attention_qmax", "oracle_qflash_attention_qmax_per_head"):
            getattr(lib, name).restype = ci
            getattr(lib, name).argtypes = lib.oracle_qflash_attention.argtypes
        lib.oracle_qmax_level.restype = i64
        lib.oracle_qmax_level.argtypes = [i64, pp]
        lib.oracle_shift_exp2_scaled.restype = i64
        lib.oracle_shift_exp2_scaled.argtypes = [i64, pp]
        _lib = lib
    return _lib


def _cp(p: OracleParams) -> _CParams:
    return _CParams(*p.astuple())


def shift_exp2(x: int, p: OracleParams) -> int:
    return int(_load().oracle_shift_exp2(int(x), ctypes.byref(_cp(p))))


def shift_exp2_quotient(x: int, p: OracleParams) -> int:
    return int(_load().oracle_shift_exp2_quotient(int(x), ctypes.byref(_cp(p))))


def requant(y: int, p: OracleParams) -> int:
    return int(_load().oracle_requant(int(y), ctypes.byref(_cp(p))))


def alpha16(alpha_hat: int, p: OracleParams) -> int:
    return int(_load().oracle_alpha16(int(alpha_hat), ctypes.byref(_cp(p))))


def scale_release(acc: int, a16: int) -> int:
    return int(_load().oracle_scale_release(int(acc), int(a16)))


def qmax_level(t: int, p: OracleParams) -> int:
    """Quantised-maximum variant (not the paper's): smallest L with L * s_inv >= t * 2^k."""
    return int(_load().oracle_qmax_level(int(t), ctypes.byref(_cp(p))))


def shift_exp2_scaled(xs: int, p: OracleParams) -> int:
    """Algorithm 2 from the quotient step on, for an argument already multiplied by 2^k."""
    return int(_load().oracle_shift_exp2_scaled(int(xs), ctypes.byref(_cp(p))))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def qflash_attention_qmax(Q, K, V, p, kv_tile: int, bias=None, nthreads: int = 0,
                          return_state: bool = False):
    """The quantised-maximum variant (NOT the paper's Algorithm 1: the reference level of the
    softmax is the maximum rounded up to a whole octave, so that the rescale of past
    accumulators is an exact shift).  Arguments and results as qflash_attention; the state's
    ``m`` holds the final level L of each row (reference = L * s_inv in scaled-score units)."""
    return qflash_attention(Q, K, V, p, kv_tile, bias=bias, nthreads=nthreads,
                            return_state=return_state, _variant="_qmax")


def qflash_attention(Q, K, V, p, kv_tile: int, bias=None, nthreads: int = 0,
                     return_state: bool = False, _variant: str = ""):
    """Algorithm 1 on int8 arrays of shape [B,H,N,d]; returns int8 [B,H,N,d].

    ``p``: one OracleParams (per-tensor scales) or a sequence of H of them (per-head scales).
    ``bias``: None or int32 [bias_B, bias_H, N, N] (INT32_MIN excludes a column).
    With ``return_state`` also returns dict(O_acc, l, m, violations) of int64 arrays.
    """
    Q = np.ascontiguousarray(Q, dtype=np.int8)
    K = np.ascontiguousarray(K, dtype=np.int8)
    V = np.ascontiguousarray(V, dtype=np.int8)
    if Q.ndim != 4 or K.shape != Q.shape or V.shape != Q.shape:
        raise ValueError("Q, K, V must share the shape [B,H,N,d]")
    B, H, N, d = Q.shape
    O = np.empty_like(Q)
    bias_ptr, bias_B, bias_H = None, 0, 0
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.int32)
        if bias.ndim != 4 or bias.shape[2:] != (N, N):
            raise ValueError("bias must be [bias_B,bias_H,N,N]")
        bias_B, bias_H = bias.shape[:2]
        bias_ptr = bias.ctypes.data
    O_acc = np.zeros((B, H, N, d), dtype=np.int64) if return_state else None
    l = np.zeros((B, H, N), dtype=np.int64) if return_state else None
    m = np.zeros((B, H, N), dtype=np.int64) if return_state else None
    viol = np.zeros(1, dtype=np.int64)
    if isinstance(p, OracleParams):
        fn, cparams = getattr(_load(), "oracle_qflash_attention" + _variant), _cp(p)
    else:
        p = list(p)
        if len(p) != H:
            raise ValueError("per-head constants: need one OracleParams per head")
        fn, cparams = getattr(_load(), "oracle_qflash_attention%s_per_head" % _variant), (_CParams * H)(*[_cp(x) for x in p])
    rc = fn(
        Q.ctypes.data, K.ctypes.data, V.ctypes.data, O.ctypes.data, bias_ptr, bias_B, bias_H,
        B, H, N, d, int(kv_tile), ctypes.cast(ctypes.byref(cparams), ctypes.POINTER(_CParams)),
        O_acc.ctypes.data if return_state else None,
        l.ctypes.data if return_state else None,
        m.ctypes.data if return_state else None,
        viol.ctypes.data, int(nthreads))
    if rc != 0:
        raise ValueError("oracle_qflash_attention rejected its arguments")
    if return_state:
        return O, {"O_acc": O_acc, "l": l, "m": m, "violations": int(viol[0])}
    if viol[0] != 0:
        raise OverflowError("%d intermediates exceed 32 bits" % int(viol[0]))
    return O
