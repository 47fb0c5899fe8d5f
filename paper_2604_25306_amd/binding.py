"""ctypes binding of the C ABI in include/qflash.h (same names, argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libqflash.so")
_lib = None

EXCLUDED = -(1 << 31)

ERR = {"OK": 0, "NULL": -1, "SHAPE": -2, "TILE": -3, "PARAM": -4, "DEVICE": -5, "LAUNCH": -6,
       "CTX": -7, "ALIGN": -8, "SCRATCH": -9}

EXPORTS = ["qflash_params_from_scales", "qflash_create", "qflash_configure", "qflash_attention",
           "qflash_attention_static",
           "qflash_attention_per_head", "qflash_dynamic_workspace_bytes", "qflash_attention_dynamic",
           "qflash_dynamic_bias_workspace_bytes", "qflash_attention_dynamic_bias",
           "qflash_packed_bias_bytes", "qflash_pack_bias", "qflash_attention_packed_bias",
           "qflash_plan_query", "qflash_plan_unit", "qflash_cache_query",
           "qflash_destroy", "qflash_strerror"]

PEAKS_EXPORTS = ["qflash_peaks_mfma_i8", "qflash_peaks_mfma_i8_ops", "qflash_peaks_copy",
                 "qflash_peaks_valu", "qflash_peaks_valu_lane_ops"]   # include/qflash_peaks.h

MAX_PARAM_HEADS = 64

CFG_EXP_TABLE = 1
CFG_QUANTISED_MAX = 2     # a variant that is not the paper's Algorithm 1 (see qflash.h)


class QFlashError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %d (%s)" % (where, code, qflash_strerror(code)))


class QFlashParams(ctypes.Structure):
    """Mirror of ``qflash_params``."""
    _fields_ = [(n, ctypes.c_int32) for n in (
        "x_shift", "s_inv", "exp_mul", "exp_shift", "p_mul", "p_shift", "a_mul", "out_round")]

    def astuple(self):
        return tuple(getattr(self, n) for n, _ in self._fields_)

    def __repr__(self):
        return "QFlashParams(%s)" % ", ".join("%s=%d" % (n, getattr(self, n)) for n, _ in self._fields_)


class DynamicInfo(ctypes.Structure):
    """Mirror of ``qflash_dynamic_info`` (what the dynamic entry point reports, in device memory)."""
    _fields_ = [("sQ", ctypes.c_double), ("sK", ctypes.c_double), ("sV", ctypes.c_double),
                ("params", QFlashParams), ("status", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class CacheInfo(ctypes.Structure):
    """Mirror of ``qflash_cache_info`` (state of a context's table cache, mode of its last launch)."""
    _fields_ = [(n, ctypes.c_int32) for n in (
        "slots_total", "slots_in_use", "slots_pinned", "evictions", "last_weight_mode", "last_kernel")] + \
        [("reserved", ctypes.c_int32 * 2)]


WEIGHTS_ARITHMETIC, WEIGHTS_TABLE, WEIGHTS_MIXED = 0, 1, 2


class PlanInfo(ctypes.Structure):
    """Mirror of ``qflash_plan_info`` (how a call would be laid out on the GPU)."""
    _fields_ = [(n, ctypes.c_int32) for n in (
        "kernel", "pairs_per_workgroup", "wavefronts_per_pair", "query_blocks", "units", "workgroups",
        "tile_by_tile", "bias_period_units", "units_per_xcd")] + [("reserved", ctypes.c_int32 * 3)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libqflash.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                "libqflash.so is missing: build it with `python -m paper_2604_25306_amd.build` "
                "(hipcc, gfx950). There is no CPU fallback.")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, ci, dbl = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        pp = ctypes.POINTER(QFlashParams)
        lib.qflash_params_from_scales.restype = ci
        lib.qflash_params_from_scales.argtypes = [dbl, dbl, dbl, ci, pp]
        lib.qflash_create.restype = ci
        lib.qflash_create.argtypes = [ctypes.POINTER(vp), ci]
        lib.qflash_attention.restype = ci
        lib.qflash_attention_per_head.restype = ci
        lib.qflash_dynamic_workspace_bytes.restype = ctypes.c_size_t
        lib.qflash_dynamic_workspace_bytes.argtypes = [ci, ci, ci, ci]
        lib.qflash_dynamic_bias_workspace_bytes.restype = ctypes.c_size_t
        lib.qflash_dynamic_bias_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
        lib.qflash_attention_dynamic_bias.restype = ci
        lib.qflash_attention_dynamic_bias.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp, vp,
                                                      ctypes.c_size_t, vp]
        lib.qflash_attention_dynamic.restype = ci
        lib.qflash_attention_dynamic.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp,
                                                 ctypes.c_size_t, vp]
        lib.qflash_attention_per_head.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, pp, vp]
        lib.qflash_attention.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, pp, vp]
        lib.qflash_attention_static.restype = ci
        lib.qflash_attention_static.argtypes = lib.qflash_attention.argtypes
        lib.qflash_packed_bias_bytes.restype = ctypes.c_size_t
        lib.qflash_packed_bias_bytes.argtypes = [ci, ci, ci]
        lib.qflash_pack_bias.restype = ci
        lib.qflash_pack_bias.argtypes = [vp, vp, ci, ci, ci, vp, ctypes.c_size_t, vp]
        lib.qflash_attention_packed_bias.restype = ci
        lib.qflash_attention_packed_bias.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, pp, ci, vp]
        lib.qflash_plan_query.restype = ci
        lib.qflash_plan_query.argtypes = [vp, ci, ci, ci, ci, ci, ci, ci, ctypes.POINTER(PlanInfo)]
        lib.qflash_plan_unit.restype = ci
        lib.qflash_plan_unit.argtypes = [ctypes.POINTER(PlanInfo), ci]
        lib.qflash_configure.restype = ci
        lib.qflash_configure.argtypes = [vp, ci, ci]
        lib.qflash_cache_query.restype = ci
        lib.qflash_cache_query.argtypes = [vp, ctypes.POINTER(CacheInfo)]
        lib.qflash_destroy.restype = ci
        lib.qflash_destroy.argtypes = [vp]
        lib.qflash_peaks_mfma_i8.restype = ci
        lib.qflash_peaks_mfma_i8.argtypes = [ci, ci, vp, ctypes.c_size_t, vp]
        lib.qflash_peaks_mfma_i8_ops.restype = dbl
        lib.qflash_peaks_mfma_i8_ops.argtypes = [ci, ci]
        lib.qflash_peaks_valu.restype = ci
        lib.qflash_peaks_valu.argtypes = [ci, ci, vp, ctypes.c_size_t, vp]
        lib.qflash_peaks_valu_lane_ops.restype = dbl
        lib.qflash_peaks_valu_lane_ops.argtypes = [ci, ci]
        lib.qflash_peaks_copy.restype = ci
        lib.qflash_peaks_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.qflash_strerror.restype = ctypes.c_char_p
        lib.qflash_strerror.argtypes = [ci]
        _lib = lib
    return _lib


def qflash_strerror(code: int) -> str:
    return load_library().qflash_strerror(int(code)).decode()


def qflash_params_from_scales(sQ: float, sK: float, sV: float, d: int) -> QFlashParams:
    p = QFlashParams()
    rc = load_library().qflash_params_from_scales(float(sQ), float(sK), float(sV), int(d),
                                                  ctypes.byref(p))
    if rc != 0:
        raise QFlashError(rc, "qflash_params_from_scales")
    return p


def qflash_create(device_id: int = 0) -> int:
    """Returns the opaque context handle (an integer address)."""
    h = ctypes.c_void_p()
    rc = load_library().qflash_create(ctypes.byref(h), int(device_id))
    if rc != 0:
        raise QFlashError(rc, "qflash_create")
    return h.value


def qflash_configure(ctx: int, key: int, value: int) -> None:
    rc = load_library().qflash_configure(ctypes.c_void_p(ctx), int(key), int(value))
    if rc != 0:
        raise QFlashError(rc, "qflash_configure")


def qflash_destroy(ctx: Optional[int]) -> None:
    rc = load_library().qflash_destroy(ctypes.c_void_p(ctx))
    if rc != 0:
        raise QFlashError(rc, "qflash_destroy")


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _marshal(Q, K, V, O, bias, stream):
    import torch
    for name, t in (("Q", Q), ("K", K), ("V", V), ("O", O)):
        if t.dtype != torch.int8 or not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError("%s must be a contiguous int8 CUDA tensor [B,H,N,d]" % name)
        if t.shape != Q.shape:
            raise ValueError("Q, K, V, O must share one shape")
    B, H, N, d = Q.shape
    bias_B = bias_H = 0
    if bias is not None:
        if bias.dtype != torch.int32 or not bias.is_cuda or not bias.is_contiguous() \
                or bias.dim() != 4 or tuple(bias.shape[2:]) != (N, N):
            raise ValueError("bias must be a contiguous int32 CUDA tensor [bias_B,bias_H,N,N]")
        bias_B, bias_H = int(bias.shape[0]), int(bias.shape[1])
    if stream is None:
        stream = torch.cuda.current_stream(Q.device).cuda_stream
    return (_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(bias), bias_B, bias_H,
            int(B), int(H), int(N), int(d)), ctypes.c_void_p(stream)


def qflash_attention(ctx: int, Q, K, V, O, params: QFlashParams, kv_tile: int, bias=None,
                     stream: Optional[int] = None) -> None:
    """Enqueue one forward pass.  Q, K, V, O: contiguous int8 CUDA tensors [B,H,N,d];
    bias: None or contiguous int32 CUDA tensor [bias_B,bias_H,N,N].  ``stream`` is a raw
    hipStream_t value (default: torch's current stream on the tensors' device)."""
    args, st = _marshal(Q, K, V, O, bias, stream)
    rc = load_library().qflash_attention(ctypes.c_void_p(ctx), *args, int(kv_tile), ctypes.byref(params), st)
    if rc != 0:
        raise QFlashError(rc, "qflash_attention")


def qflash_attention_static(ctx: int, Q, K, V, O, params: QFlashParams, kv_tile: int, bias=None,
                            stream: Optional[int] = None) -> None:
    """``qflash_attention`` through the entry point that allocates no device memory."""
    args, st = _marshal(Q, K, V, O, bias, stream)
    rc = load_library().qflash_attention_static(ctypes.c_void_p(ctx), *args, int(kv_tile),
                                                ctypes.byref(params), st)
    if rc != 0:
        raise QFlashError(rc, "qflash_attention_static")


def params_array(params):
    """A C array of ``QFlashParams`` from a sequence of them: what the per-head entry points take.
    Callers in a loop build it once and pass it instead of the sequence."""
    params = list(params)
    return (QFlashParams * len(params))(*params)


def qflash_attention_per_head(ctx: int, Q, K, V, O, params, kv_tile: int, bias=None,
                              stream: Optional[int] = None) -> None:
    """The same with one ``QFlashParams`` per head (a sequence of H of them, or ``params_array`` of it)."""
    args, st = _marshal(Q, K, V, O, bias, stream)
    arr = params if isinstance(params, ctypes.Array) else params_array(params)
    if len(arr) != args[8]:
        raise ValueError("need one QFlashParams per head")
    rc = load_library().qflash_attention_per_head(
        ctypes.c_void_p(ctx), *args, int(kv_tile), ctypes.cast(arr, ctypes.POINTER(QFlashParams)), st)
    if rc != 0:
        raise QFlashError(rc, "qflash_attention_per_head")


def qflash_packed_bias_bytes(bias_B: int, bias_H: int, N: int) -> int:
    return int(load_library().qflash_packed_bias_bytes(int(bias_B), int(bias_H), int(N)))


def qflash_pack_bias(ctx: int, bias, packed, stream: Optional[int] = None) -> None:
    """Rewrite ``bias`` (contiguous int32 CUDA tensor [bias_B,bias_H,N,N]) into ``packed`` (contiguous
    int32 CUDA tensor of at least ``qflash_packed_bias_bytes`` bytes) for ``qflash_attention_packed_bias``."""
    import torch
    if bias.dtype != torch.int32 or not bias.is_cuda or not bias.is_contiguous() or bias.dim() != 4 \
            or bias.shape[2] != bias.shape[3]:
        raise ValueError("bias must be a contiguous int32 CUDA tensor [bias_B,bias_H,N,N]")
    if packed.dtype != torch.int32 or not packed.is_cuda or not packed.is_contiguous():
        raise ValueError("packed must be a contiguous int32 CUDA tensor")
    if stream is None:
        stream = torch.cuda.current_stream(bias.device).cuda_stream
    rc = load_library().qflash_pack_bias(
        ctypes.c_void_p(ctx), _ptr(bias), int(bias.shape[0]), int(bias.shape[1]), int(bias.shape[2]),
        _ptr(packed), int(packed.numel()) * 4, ctypes.c_void_p(stream))
    if rc != 0:
        raise QFlashError(rc, "qflash_pack_bias")


def qflash_attention_packed_bias(ctx: int, Q, K, V, O, params, kv_tile: int, packed, bias_B: int,
                                 bias_H: int, stream: Optional[int] = None) -> None:
    """The forward pass with a bias packed by ``qflash_pack_bias`` for the same bias_B, bias_H, N.
    ``params``: one QFlashParams or a sequence of H."""
    import torch
    args, st = _marshal(Q, K, V, O, None, stream)
    if packed.dtype != torch.int32 or not packed.is_cuda or not packed.is_contiguous():
        raise ValueError("packed must be a contiguous int32 CUDA tensor")
    # same figure as qflash_packed_bias_bytes, without a call into the library per launch
    if packed.numel() < int(bias_B) * int(bias_H) * ((args[9] + 31) // 32) ** 2 * 1024:
        raise ValueError("packed is smaller than qflash_packed_bias_bytes(bias_B, bias_H, N)")
    if isinstance(params, QFlashParams):
        pp, n_p = ctypes.byref(params), 1
    else:
        arr = params if isinstance(params, ctypes.Array) else params_array(params)
        pp, n_p = ctypes.cast(arr, ctypes.POINTER(QFlashParams)), len(arr)
    rc = load_library().qflash_attention_packed_bias(
        ctypes.c_void_p(ctx), args[0], args[1], args[2], args[3], _ptr(packed), int(bias_B), int(bias_H),
        args[7], args[8], args[9], args[10], int(kv_tile), pp, n_p, st)
    if rc != 0:
        raise QFlashError(rc, "qflash_attention_packed_bias")


def qflash_plan_query(ctx: Optional[int], B: int, H: int, N: int, d: int, kv_tile: int,
                      bias_B: int = 0, bias_H: int = 0) -> PlanInfo:
    """The launch plan of such a call (host only; ``ctx`` None assumes an MI355X)."""
    info = PlanInfo()
    rc = load_library().qflash_plan_query(ctypes.c_void_p(ctx), int(B), int(H), int(N), int(d), int(kv_tile),
                                          int(bias_B), int(bias_H), ctypes.byref(info))
    if rc != 0:
        raise QFlashError(rc, "qflash_plan_query")
    return info


def qflash_cache_query(ctx: int) -> CacheInfo:
    info = CacheInfo()
    rc = load_library().qflash_cache_query(ctypes.c_void_p(ctx), ctypes.byref(info))
    if rc != 0:
        raise QFlashError(rc, "qflash_cache_query")
    return info


def qflash_plan_unit(plan: PlanInfo, workgroup: int) -> int:
    return int(load_library().qflash_plan_unit(ctypes.byref(plan), int(workgroup)))


def qflash_dynamic_workspace_bytes(B: int, H: int, N: int, d: int) -> int:
    return int(load_library().qflash_dynamic_workspace_bytes(int(B), int(H), int(N), int(d)))


def qflash_dynamic_bias_workspace_bytes(B: int, H: int, N: int, d: int, bias_B: int, bias_H: int) -> int:
    return int(load_library().qflash_dynamic_bias_workspace_bytes(int(B), int(H), int(N), int(d), int(bias_B), int(bias_H)))


def qflash_attention_dynamic(ctx: int, Qf, Kf, Vf, O, kv_tile: int, workspace, info=None,
                             out_round: int = 0, stream: Optional[int] = None, bias_real=None, excluded=None) -> None:
    """Quantise float32 CUDA tensors Qf, Kf, Vf [B,H,N,d] on the GPU and run the forward pass.
    ``workspace``: uint8 CUDA tensor of at least ``qflash_dynamic_workspace_bytes`` bytes
    (``qflash_dynamic_bias_workspace_bytes`` with a bias);
    ``info``: None or a uint8 CUDA tensor of ``ctypes.sizeof(DynamicInfo)`` bytes;
    ``bias_real`` / ``excluded``: None, or float32 / uint8 CUDA tensors [bias_B,bias_H,N,N] (a bias in
    real units and an exclusion mask: qflash_attention_dynamic_bias)."""
    import torch
    ref = bias_real if bias_real is not None else excluded
    if ref is not None:
        if bias_real is not None and (bias_real.dtype != torch.float32 or not bias_real.is_cuda
                                      or not bias_real.is_contiguous() or bias_real.dim() != 4):
            raise ValueError("bias_real must be a contiguous float32 CUDA tensor [bias_B,bias_H,N,N]")
        if excluded is not None and (excluded.dtype != torch.uint8 or not excluded.is_cuda
                                     or not excluded.is_contiguous() or excluded.shape != ref.shape):
            raise ValueError("excluded must be a contiguous uint8 CUDA tensor of the bias shape")
        if tuple(ref.shape[2:]) != (Qf.shape[2], Qf.shape[2]):
            raise ValueError("bias must be [bias_B,bias_H,N,N]")
    for name, t in (("Qf", Qf), ("Kf", Kf), ("Vf", Vf)):
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or t.dim() != 4 \
                or t.shape != Qf.shape:
            raise ValueError("%s must be a contiguous float32 CUDA tensor [B,H,N,d]" % name)
    if O.dtype != torch.int8 or not O.is_cuda or not O.is_contiguous() or O.shape != Qf.shape:
        raise ValueError("O must be a contiguous int8 CUDA tensor [B,H,N,d]")
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous uint8 CUDA tensor")
    if info is not None and (info.dtype != torch.uint8 or not info.is_cuda
                             or info.numel() < ctypes.sizeof(DynamicInfo)):
        raise ValueError("info must be a uint8 CUDA tensor of sizeof(DynamicInfo) bytes")
    B, H, N, d = Qf.shape
    if stream is None:
        stream = torch.cuda.current_stream(Qf.device).cuda_stream
    if ref is not None:
        rc = load_library().qflash_attention_dynamic_bias(
            ctypes.c_void_p(ctx), _ptr(Qf), _ptr(Kf), _ptr(Vf), _ptr(O), _ptr(bias_real), _ptr(excluded),
            int(ref.shape[0]), int(ref.shape[1]), int(B), int(H), int(N), int(d), int(kv_tile), int(out_round),
            _ptr(info), _ptr(workspace), int(workspace.numel()), ctypes.c_void_p(stream))
        if rc != 0:
            raise QFlashError(rc, "qflash_attention_dynamic_bias")
        return
    rc = load_library().qflash_attention_dynamic(
        ctypes.c_void_p(ctx), _ptr(Qf), _ptr(Kf), _ptr(Vf), _ptr(O), int(B), int(H), int(N), int(d),
        int(kv_tile), int(out_round), _ptr(info), _ptr(workspace), int(workspace.numel()),
        ctypes.c_void_p(stream))
    if rc != 0:
        raise QFlashError(rc, "qflash_attention_dynamic")


def qflash_peaks_mfma_i8(workgroups: int, iters: int, out, stream: Optional[int] = None) -> float:
    """Enqueue the int8 matrix-rate kernel; ``out``: uint8/int64 CUDA tensor of at least
    16 * workgroups + 16 bytes.  Returns the number of int8 operations the launch executes."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(out.device).cuda_stream
    rc = load_library().qflash_peaks_mfma_i8(int(workgroups), int(iters), _ptr(out),
                                             int(out.numel() * out.element_size()), ctypes.c_void_p(stream))
    if rc != 0:
        raise RuntimeError("qflash_peaks_mfma_i8 failed: %d" % rc)
    return float(load_library().qflash_peaks_mfma_i8_ops(int(workgroups), int(iters)))


def qflash_peaks_valu(workgroups: int, iters: int, out, stream: Optional[int] = None) -> float:
    """Enqueue the vector-integer issue-rate kernel; ``out`` as for qflash_peaks_mfma_i8.  Returns the
    number of lane-operations the launch executes."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(out.device).cuda_stream
    rc = load_library().qflash_peaks_valu(int(workgroups), int(iters), _ptr(out),
                                          int(out.numel() * out.element_size()), ctypes.c_void_p(stream))
    if rc != 0:
        raise RuntimeError("qflash_peaks_valu failed: %d" % rc)
    return float(load_library().qflash_peaks_valu_lane_ops(int(workgroups), int(iters)))


def qflash_peaks_copy(src, dst, stream: Optional[int] = None) -> None:
    """Enqueue the device-to-device copy kernel over two CUDA tensors of equal byte size."""
    import torch
    n = int(src.numel() * src.element_size())
    if n != int(dst.numel() * dst.element_size()):
        raise ValueError("src and dst must have the same size")
    if stream is None:
        stream = torch.cuda.current_stream(src.device).cuda_stream
    rc = load_library().qflash_peaks_copy(_ptr(src), _ptr(dst), n, ctypes.c_void_p(stream))
    if rc != 0:
        raise RuntimeError("qflash_peaks_copy failed: %d" % rc)


class Context:
    """RAII wrapper: ``with Context(0) as ctx: ctx.attention(...)``."""

    def __init__(self, device_id: int = 0):
        self.handle = qflash_create(device_id)

    def configure(self, key: int, value: int):
        qflash_configure(self.handle, key, value)

    def cache_info(self) -> CacheInfo:
        return qflash_cache_query(self.handle)

    def attention(self, Q, K, V, O, params, kv_tile, bias=None, stream=None):
        """``params``: one QFlashParams (per-tensor scales) or a sequence of H (per-head scales)."""
        if isinstance(params, QFlashParams):
            qflash_attention(self.handle, Q, K, V, O, params, kv_tile, bias, stream)
        else:
            qflash_attention_per_head(self.handle, Q, K, V, O, params, kv_tile, bias, stream)

    def attention_static(self, Q, K, V, O, params, kv_tile, bias=None, stream=None):
        qflash_attention_static(self.handle, Q, K, V, O, params, kv_tile, bias, stream)

    def pack_bias(self, bias, stream=None):
        """Returns the packed copy of ``bias`` (a new int32 CUDA tensor) for ``attention_packed_bias``."""
        import torch
        n = qflash_packed_bias_bytes(bias.shape[0], bias.shape[1], bias.shape[2])
        if n == 0:
            raise ValueError("bias extents are not supported")
        packed = torch.empty(n // 4, dtype=torch.int32, device=bias.device)
        qflash_pack_bias(self.handle, bias, packed, stream)
        return packed

    def attention_packed_bias(self, Q, K, V, O, params, kv_tile, packed, bias_B, bias_H, stream=None):
        qflash_attention_packed_bias(self.handle, Q, K, V, O, params, kv_tile, packed, bias_B, bias_H, stream)

    def attention_dynamic(self, Qf, Kf, Vf, O, kv_tile, workspace, info=None, out_round=0, stream=None,
                          bias_real=None, excluded=None):
        qflash_attention_dynamic(self.handle, Qf, Kf, Vf, O, kv_tile, workspace, info, out_round, stream,
                                 bias_real, excluded)

    def close(self):
        if self.handle is not None:
            qflash_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
