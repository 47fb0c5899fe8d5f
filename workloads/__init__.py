"""Seeded synthetic attention inputs (shared by tests, smoke and bench).

This module holds no arithmetic of the attention method itself: it draws real
tensors from a seed, quantises them per tensor to int8 (Eq. 1-2: symmetric,
scale = max|x| / 127) and, for the windowed workload, builds the additive
integer bias / exclusion mask.  Both the CPU oracle and the GPU library are fed
the arrays made here; neither imports this module.

The five named workloads stand in for the attention layers of ViT / DeiT / Swin
models (shapes of Table 1, scaled to the batch sizes of the benchmark): real
activations would need ImageNet and trained weights, which are not available.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

EXCLUDED = np.iinfo(np.int32).min


@dataclass
class Workload:
    name: str
    Q: np.ndarray                 # int8 [B,H,N,d]
    K: np.ndarray
    V: np.ndarray
    sQ: float                     # per-tensor scale, or array [H] in the per-head variant
    sK: float
    sV: float
    kv_tiles: tuple               # KV tile sizes this workload is run with
    bias: Optional[np.ndarray] = None        # int32 [bias_B,bias_H,N,N] or None
    bias_real: Optional[np.ndarray] = None   # float64, same shape, 0 where excluded
    excluded: Optional[np.ndarray] = None    # bool, same shape
    meta: dict = field(default_factory=dict)

    @property
    def shape(self):
        return self.Q.shape


def quantize_per_tensor(x: np.ndarray):
    """Eq. 1-2 with b = 8: s = max|x| / 127 (double), x_hat = clip(rint(x / s), -127, 127)."""
    amax = float(np.max(np.abs(x)))
    if amax == 0.0:
        return np.zeros(x.shape, dtype=np.int8), 1.0
    s = amax / 127.0
    q = np.clip(np.rint(x.astype(np.float64) / s), -127, 127).astype(np.int8)
    return q, s


def quantize_per_head(x: np.ndarray):
    """Eq. 1-2 with one scale per head (axis 1 of [B,H,N,d]): returns int8 array and scales [H]."""
    H = x.shape[1]
    q = np.zeros(x.shape, dtype=np.int8)
    s = np.ones(H, dtype=np.float64)
    for h in range(H):
        q[:, h], s[h] = quantize_per_tensor(x[:, h])
    return q, s


def _draw(rng, shape, dist, sigma=1.0, outlier_frac=0.0, outlier_gain=8.0):
    if dist == "normal":
        x = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(sigma)
    elif dist == "student_t3":
        x = rng.standard_t(3.0, size=shape).astype(np.float32)
    else:
        raise ValueError(dist)
    if outlier_frac > 0.0:
        B, H, N, d = shape
        n_out = int(np.ceil(outlier_frac * H * d))
        ch = rng.choice(H * d, size=n_out, replace=False)
        xv = x.transpose(0, 2, 1, 3).reshape(B, N, H * d)    # channel = h*d + t
        xv[:, :, ch] *= np.float32(outlier_gain)
        x = xv.reshape(B, N, H, d).transpose(0, 2, 1, 3).copy()
    return x


def make_qkv(shape, seed, dist="normal", sigma=1.0, outlier_frac=0.0, per_head=False, head_gain=None):
    """Q, K, V drawn in that order from one generator, each quantised per tensor (or per head:
    the scales are then arrays [H]; ``head_gain`` [H] multiplies the real values of each head
    first, so that heads differ in range the way trained heads do)."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(3):
        x = _draw(rng, shape, dist, sigma, outlier_frac)
        if head_gain is not None:
            x = x * np.asarray(head_gain, dtype=np.float32)[None, :, None, None]
        out.append(quantize_per_head(x) if per_head else quantize_per_tensor(x))
    (Q, sQ), (K, sK), (V, sV) = out
    return Q, K, V, sQ, sK, sV, rng


def swin_window_bias(rng, heads, d, sQ, sK, n_windows=64, win=7):
    """Relative-position bias plus shifted-window exclusion mask, in units of the int32 score.

    Table [heads, (2*win-1)^2] ~ N(0, 0.5^2), gathered with index
    (dy + win-1) * (2*win-1) + (dx + win-1).  Windows with an odd index carry the
    shifted-window mask: the window is split into four regions at row/column
    win - win//2; a query and a key in different regions exclude each other.
    Real bias -> integer: round(bias * sqrt(d) / (sQ*sK)), the unit of Q_hat K_hat^T.
    """
    n = win * win
    table = rng.standard_normal(size=(heads, (2 * win - 1) ** 2)) * 0.5
    ys, xs = np.divmod(np.arange(n), win)
    dy = ys[:, None] - ys[None, :] + (win - 1)
    dx = xs[:, None] - xs[None, :] + (win - 1)
    rel = table[:, dy * (2 * win - 1) + dx]                       # [heads, n, n]
    split = win - win // 2
    label = (ys >= split).astype(np.int64) * 2 + (xs >= split).astype(np.int64)
    differ = label[:, None] != label[None, :]
    excluded = np.zeros((n_windows, heads, n, n), dtype=bool)
    excluded[1::2] = differ[None, None]
    bias_real = np.broadcast_to(rel[None], (n_windows, heads, n, n)).copy()
    # one score unit for the tensor, or one per head (per-head scales: arrays [heads])
    unit = (np.asarray(sQ, dtype=np.float64) * np.asarray(sK, dtype=np.float64)) / np.sqrt(float(d))
    if unit.ndim == 1:
        unit = unit.reshape(1, heads, 1, 1)
    bias_int = np.floor(bias_real / unit + 0.5).astype(np.int64)
    assert np.abs(bias_int).max() < (1 << 20)
    bias = np.where(excluded, np.int64(EXCLUDED), bias_int).astype(np.int32)
    bias_real = np.where(excluded, 0.0, bias_int * unit)
    return bias, bias_real, excluded


# name -> (shape [B,H,N,d], dist, sigma, outlier_frac, kv_tiles, windowed: False, True (64 windows) or the window count)
CONFIGS = {
    "deit_tiny_b1":   ((1, 3, 197, 64),   "normal",     1.0, 0.0,  (64,),     False),
    "vit_b16_b64":    ((64, 12, 197, 64), "normal",     1.0, 0.0,  (64,),     False),
    "deit_b384_b32":  ((32, 12, 577, 64), "normal",     1.5, 0.0,  (64, 128), False),
    "swin_t_s1_b64":  ((4096, 3, 49, 32), "normal",     1.0, 0.0,  (64,),     True),
    "vit_l384_heavy": ((16, 16, 577, 64), "student_t3", 1.0, 0.01, (64,),     False),
}
# The attention workloads of Table 1 at the paper's own batch sizes 1 and 8 (small, latency-bound
# launches).  Windowed ones give the number of windows per image: B = batch * windows, and the
# bias holds one [H,N,N] slice per window position.  The last stage has a single window per image,
# hence no shifted-window mask.
#   name -> (heads, N, d, windows per image or 0)
TABLE1 = {
    "a1_deit_t": (3, 197, 64, 0),
    "a2_deit_s": (6, 197, 64, 0),
    "a3_vit_b":  (12, 197, 64, 0),
    "a4_swin_s1": (3, 49, 32, 64),
    "a5_swin_s2": (6, 49, 32, 16),
    "a6_swin_s3": (12, 49, 32, 4),
    "a7_swin_s4": (24, 49, 32, 1),
}
for _name, (_h, _n, _d, _win) in TABLE1.items():
    for _b in (1, 8):
        CONFIGS["%s_b%d" % (_name, _b)] = ((_b * max(_win, 1), _h, _n, _d), "normal", 1.0, 0.0, (64,), _win)
CONFIG_ORDER = list(CONFIGS)
# A shape outside the paper's workloads, for measuring the corner where a d = 32 sequence no longer
# fits LDS and the streamed kernel takes over (appended after CONFIG_ORDER is fixed: seeds unchanged).
CONFIGS["long_d32_n2100"] = ((8, 8, 2100, 32), "normal", 1.0, 0.0, (64, 128), False)
CONFIG_ORDER.append("long_d32_n2100")
HEADLINE = "vit_b16_b64"
BASELINE_CONFIGS = CONFIG_ORDER[:5]           # the five benchmark configurations
TABLE1_CONFIGS = CONFIG_ORDER[5:5 + 2 * len(TABLE1)]   # Table 1 at batch 1 and 8


def make_float_qkv(name: str, batch: Optional[int] = None):
    """The float32 Q, K, V a workload is quantised from (same seed, same draws): input of the
    dynamic-quantisation path."""
    shape, dist, sigma, ofrac, _, windowed = CONFIGS[name]
    if batch is not None:
        shape = (int(batch),) + tuple(shape[1:])
    rng = np.random.default_rng(1000 + CONFIG_ORDER.index(name) + 1)
    return tuple(_draw(rng, shape, dist, sigma, ofrac) for _ in range(3))


def make_float_window_bias(name: str, n_windows: Optional[int] = None):
    """Real-valued bias of a windowed workload for the dynamic-quantisation path: relative-position
    bias (float32 [windows, heads, N, N], table ~ N(0, 0.5^2) gathered as in swin_window_bias) and
    the shifted-window exclusion mask (uint8, same shape, 1 = excluded; odd windows carry it)."""
    shape, _, _, _, _, windowed = CONFIGS[name]
    if not windowed:
        raise ValueError("not a windowed workload")
    n_win = int(n_windows) if n_windows is not None else (64 if windowed is True else int(windowed))
    heads, n = shape[1], shape[2]
    win = int(round(np.sqrt(n)))
    rng = np.random.default_rng(2000 + CONFIG_ORDER.index(name) + 1)
    table = rng.standard_normal(size=(heads, (2 * win - 1) ** 2)) * 0.5
    ys, xs = np.divmod(np.arange(n), win)
    dy = ys[:, None] - ys[None, :] + (win - 1)
    dx = xs[:, None] - xs[None, :] + (win - 1)
    rel = table[:, dy * (2 * win - 1) + dx].astype(np.float32)
    split = win - win // 2
    label = (ys >= split).astype(np.int64) * 2 + (xs >= split).astype(np.int64)
    differ = label[:, None] != label[None, :]
    excluded = np.zeros((n_win, heads, n, n), dtype=np.uint8)
    excluded[1::2] = differ[None, None]
    bias_real = np.ascontiguousarray(np.broadcast_to(rel[None], (n_win, heads, n, n)))
    return bias_real, excluded


def head_gains(H: int) -> np.ndarray:
    """Deterministic spread of per-head ranges, 1/4 .. 4 (geometric), used by the per-head variant."""
    return np.exp2(np.linspace(-2.0, 2.0, H)) if H > 1 else np.ones(1)


def make_workload(name: str, batch: Optional[int] = None, per_head: bool = False) -> Workload:
    """Build one of the named workloads; ``batch`` overrides B (tests use smaller ones).

    Seed = 1000 + position of the workload in CONFIG_ORDER (1-based).
    """
    shape, dist, sigma, ofrac, kv_tiles, windowed = CONFIGS[name]
    if batch is not None:
        shape = (int(batch),) + tuple(shape[1:])
    seed = 1000 + CONFIG_ORDER.index(name) + 1
    if per_head:
        # per-head variant (Appendix C3): heads get different ranges and their own scales;
        # sQ, sK, sV are arrays [H].  The integer bias of a windowed workload is then expressed
        # head by head in that head's score unit.
        Q, K, V, sQ, sK, sV, rng = make_qkv(shape, seed, dist, sigma, ofrac, per_head=True,
                                            head_gain=head_gains(shape[1]))
        wl = Workload(name + "/per_head", Q, K, V, sQ, sK, sV, kv_tiles,
                      meta={"seed": seed, "dist": dist, "per_head": True})
        if windowed:
            n_windows = 64 if windowed is True else int(windowed)
            wl.bias, wl.bias_real, wl.excluded = swin_window_bias(rng, shape[1], shape[3], sQ, sK, n_windows=n_windows)
        return wl
    Q, K, V, sQ, sK, sV, rng = make_qkv(shape, seed, dist, sigma, ofrac)
    wl = Workload(name, Q, K, V, sQ, sK, sV, kv_tiles, meta={"seed": seed, "dist": dist})
    if windowed:
        n_windows = 64 if windowed is True else int(windowed)
        wl.bias, wl.bias_real, wl.excluded = swin_window_bias(rng, shape[1], shape[3], sQ, sK, n_windows=n_windows)
    return wl
