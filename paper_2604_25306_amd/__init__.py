"""MI355X-native integer-only fused attention (QFlash, arxiv 2604.25306): thin Python binding.

The package is argument marshalling only: every step of the attention runs in the hand-written
gfx950 kernels of ``libqflash.so`` behind the C ABI declared in ``include/qflash.h``.  There is no
CPU or PyTorch fallback; if the library has not been built, importing ``binding`` functions raises.
"""
from .binding import (  # noqa: F401
    QFlashError, QFlashParams, Context, library_path, load_library,
    qflash_params_from_scales, qflash_create, qflash_configure, qflash_attention,
    qflash_attention_static,
    qflash_attention_per_head, qflash_dynamic_workspace_bytes, qflash_attention_dynamic, DynamicInfo,
    qflash_dynamic_bias_workspace_bytes,
    qflash_destroy, qflash_strerror, EXCLUDED, ERR, CFG_EXP_TABLE, CFG_QUANTISED_MAX,
    MAX_PARAM_HEADS, qflash_packed_bias_bytes, qflash_pack_bias, qflash_attention_packed_bias,
    params_array, PlanInfo, qflash_plan_query, qflash_plan_unit, CacheInfo, qflash_cache_query,
    WEIGHTS_ARITHMETIC, WEIGHTS_TABLE, WEIGHTS_MIXED, qflash_peaks_mfma_i8, qflash_peaks_copy, qflash_peaks_valu,
)
