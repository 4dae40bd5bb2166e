"""Gathers the tensor statistics the variance-increment indicator needs from the device.

Paper: Indicator section, Prop. 3.  The statistics (squared norm, absmax) come out of the same pass that
computes the quantization scale (`qsync_absmax_scale` with `sumsq_opt`); this module copies the two scalars
to the host.  The indicator itself is evaluated by libqsync (`qsync_variance_increment`, a host function of
the C ABI); nothing here computes.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import qsync as Q


@dataclass
class TensorStats:
    sumsq: float
    amax: float
    D: int


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
                       k: int = 9, gamma: float = 1.0, d_o: int = 1, d_L: int = 1) -> dict:
    """Omega of one operator through `qsync_variance_increment`; `kind` is "fixed" (q_x, q_v: the fixed-point
    scales of parameter and activation) or "float"; k: mantissa bits of the floating-point format."""
    kinds = {"fixed": Q.QUANT_FIXED, "float": Q.QUANT_FLOAT}
    if kind not in kinds:
        raise ValueError(kind)
    return Q.qsync_variance_increment(kinds[kind], x, v, gv, q_x, q_v, k, gamma, d_o, d_L)
