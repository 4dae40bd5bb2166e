"""Variance-increment indicator of one operator from device-side tensor statistics.

Paper: Indicator section, Prop. 3 (Omega = gamma^2 d_o sigma_fp + (d_L - d_o) sigma_bp) and the two case
equations for sigma_fp / sigma_bp of unary computation-intensive operators.  The statistics (squared
norm, absmax) come out of the same pass that computes the quantization scale (`qsync_absmax_scale`
with `sumsq_opt`); this module only gathers the handful of scalars and evaluates the closed form on the
host, as the paper does after profiling.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch

from . import qsync as Q


@dataclass
class TensorStats:
    sumsq: float
    amax: float
    D: int

    @property
    def e(self) -> int:
        """Effective exponent: 2^e <= amax < 2^(e+1); -126 for an all-zero tensor."""
        return int(math.floor(math.log2(self.amax))) if self.amax > 0 else -126


def tensor_stats(x: torch.Tensor, stream=None) -> TensorStats:
    """One pass of `qsync_absmax_scale` over a 2-D (or flattened) device tensor: squared norm and absmax."""
    x2 = x.reshape(x.shape[0], -1) if x.dim() > 1 else x.reshape(1, -1)
    rows, cols = x2.shape
    f = lambda: torch.empty(1, dtype=torch.float32, device=x.device)
    scale, inv, amax, sumsq = f(), f(), f(), f()
    ws = torch.zeros(max(Q.qsync_absmax_workspace_bytes(rows, cols, Q.PER_TENSOR), 256), dtype=torch.uint8, device=x.device)
    Q.qsync_absmax_scale(x2, rows, cols, cols, Q.PER_TENSOR, 8, scale, inv, amax, None, ws, stream, sumsq_opt=sumsq)
    both = torch.cat([sumsq, amax]).tolist()          # one device-to-host copy
    return TensorStats(sumsq=both[0], amax=both[1], D=rows * cols)


def variance_increment(kind: str, x: TensorStats, v: TensorStats, gv: TensorStats, q_x: float = 0.0, q_v: float = 0.0,
                       eps: float = 2.0 ** -9, gamma: float = 1.0, d_o: int = 1, d_L: int = 1) -> dict:
    """Omega of one operator; `kind` is "fixed" (q_x, q_v: the fixed-point scales of parameter and
    activation) or "float" (eps = 2^-k of the floating-point format)."""
    if kind == "fixed":
        s_fp = (x.sumsq * q_v ** 2 * v.D + v.sumsq * q_x ** 2 * x.D) / 6.0
        s_bp = (gv.sumsq * q_v ** 2 * v.D + v.sumsq * 4.0 ** gv.e * eps ** 2 * gv.D) / 6.0
    elif kind == "float":
        s_fp = eps ** 2 * (x.sumsq * 4.0 ** v.e * v.D + v.sumsq * 4.0 ** x.e * x.D) / 6.0
        s_bp = eps ** 2 * (gv.sumsq * 4.0 ** v.e * v.D + v.sumsq * 4.0 ** gv.e * gv.D) / 6.0
    else:
        raise ValueError(kind)
    return dict(sigma_fp=s_fp, sigma_bp=s_bp, omega=gamma ** 2 * d_o * s_fp + (d_L - d_o) * s_bp)
