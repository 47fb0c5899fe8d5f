"""QFlash CPU oracle -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It imports nothing from the GPU library
and the GPU library imports nothing from it.

Contents
--------
* ``derive_params``          host constants of Algorithm 1 / 2 / Eq. 9-10 from the real scales
* ``qflash_attention``       Algorithm 1 (tile-wise integer attention), plain C via ctypes
* ``shift_exp2`` etc.        the scalar building blocks of the C oracle, exposed for pins
* ``fullrow_int_attention``  brute force: integer softmax over the whole row at once (NumPy)
* ``float_attention``        exact softmax attention in float64 on dequantised inputs (NumPy)
* ``qflash_attention_qmax``  the quantised-maximum variant (not the paper's; rescale by exact shifts)
* ``dynamic_quantize``, ``qflash_attention_dynamic``  Eq. 1-2 on the fly in front of Algorithm 1
"""
from .params import OracleParams, derive_params
from .cbinding import (
    build_oracle,
    qflash_attention,
    qflash_attention_qmax,
    qmax_level,
    shift_exp2_scaled,
    shift_exp2,
    shift_exp2_quotient,
    requant,
    alpha16,
    scale_release,
    num_threads,
)
from .bruteforce import (
    shift_exp2_np,
    requant_np,
    fullrow_int_attention,
    fullrow_int_attention_qmax,
    float_attention,
    float_attention_ratio,
)

from .dynamic import dynamic_quantize, qflash_attention_dynamic, dynamic_bias_to_int

__all__ = [
    "dynamic_quantize", "qflash_attention_dynamic", "dynamic_bias_to_int",
    "OracleParams", "derive_params", "build_oracle", "qflash_attention", "shift_exp2",
    "shift_exp2_quotient", "requant", "alpha16", "scale_release", "num_threads",
    "shift_exp2_np", "requant_np", "fullrow_int_attention", "float_attention",
    "qflash_attention_qmax", "qmax_level", "shift_exp2_scaled", "fullrow_int_attention_qmax",
    "float_attention_ratio",
]
