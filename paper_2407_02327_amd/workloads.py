"""Seeded synthetic inputs for the quantized-operator hot path.

This module holds input recipes only: tensor shapes, value distributions and
seeds that stand in for the CNN and transformer layers the method was evaluated
on (the paper's Benchmarks paragraph names ResNet/VGG on ImageNet and BERT/RoBERTa
fine-tuning; none of that data is used here).  It contains none of the method's
arithmetic, so the CPU oracle and the HIP path can both be fed from it.

Every tensor is drawn on the host from ``numpy.random.default_rng(seed)`` in a
fixed order, so that the oracle and the GPU always see identical bits.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

INT8, FP16, FP32 = 8, 16, 32          # per-operator precision tags (paper, problem (1): b_io)


@dataclass
class LinearCase:
    """One linear operator: Y = X W^T + b, with the upstream gradient dY."""
    name: str
    x: np.ndarray                      # [M, K]
    w: np.ndarray                      # [N, K]
    bias: np.ndarray                   # [N] fp32
    dy: np.ndarray                     # [M, N]
    w_gran: str = "tensor"             # "tensor" | "row" (per output channel)
    dy_round: str = "nearest"          # "nearest" | "stochastic"
    philox_seed: int = 0
    tags: List[int] = field(default_factory=lambda: [INT8])
    nhwc: Optional[np.ndarray] = None  # convolution cases: the [B,H,W,C] activation whose 3x3 im2col is x

    @property
    def mnk(self):
        return self.x.shape[0], self.w.shape[0], self.x.shape[1]


def _normal(rng, shape, sigma, dtype):
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    return a.astype(dtype, copy=False)


def config1() -> LinearCase:
    """Small INT8 linear, everything per-tensor and round-to-nearest (seed 0)."""
    rng = np.random.default_rng(0)
    x = _normal(rng, (64, 128), 1.0, np.float32)
    w = _normal(rng, (128, 128), 0.02, np.float32)
    dy = _normal(rng, (64, 128), 1e-2, np.float32)
    return LinearCase("c1_small_int8", x, w, np.zeros(128, np.float32), dy,
                      w_gran="tensor", dy_round="nearest", philox_seed=0, tags=[INT8])


def config2(tokens: int = 4096) -> LinearCase:
    """BERT-base FFN up-projection: 768 -> 3072, fp16 activations and gradients."""
    rng = np.random.default_rng(1)
    x = _normal(rng, (tokens, 768), 1.0, np.float16)
    w = _normal(rng, (3072, 768), 0.02, np.float32)
    dy = _normal(rng, (tokens, 3072), 1e-3, np.float16)
    return LinearCase("c2_bert_base_ffn", x, w, np.zeros(3072, np.float32), dy,
                      w_gran="row", dy_round="stochastic", philox_seed=1, tags=[INT8])


def im2col_nhwc_3x3(act: np.ndarray) -> np.ndarray:
    """[B,H,W,C] -> [B*H*W, 9*C] patches of a 3x3, stride-1, pad-1 convolution.

    The k index runs (kh, kw, c_in), matching weights reshaped from
    [C_out, C_in, 3, 3] to [C_out, 3, 3, C_in].
    """
    b, h, w, c = act.shape
    padded = np.zeros((b, h + 2, w + 2, c), dtype=act.dtype)
    padded[:, 1:-1, 1:-1, :] = act
    out = np.empty((b, h, w, 9, c), dtype=act.dtype)
    for kh in range(3):
        for kw in range(3):
            out[:, :, :, kh * 3 + kw, :] = padded[:, kh:kh + h, kw:kw + w, :]
    return out.reshape(b * h * w, 9 * c)


def config3(batch: int = 64) -> LinearCase:
    """ResNet-50 stage-2 3x3 convolution lowered to an im2col GEMM (M=B*56*56, K=576, N=64)."""
    rng = np.random.default_rng(3)
    act = np.abs(rng.standard_normal(size=(batch, 56, 56, 64), dtype=np.float32)).astype(np.float16)
    wconv = _normal(rng, (64, 64, 3, 3), float(np.sqrt(2.0 / 576.0)), np.float32)   # Kaiming normal, fan_in 576
    w = np.ascontiguousarray(wconv.transpose(0, 2, 3, 1)).reshape(64, 576)
    dy = _normal(rng, (batch * 56 * 56, 64), 1e-3, np.float16)
    x = im2col_nhwc_3x3(act)
    return LinearCase("c3_resnet50_conv3x3", x, w, np.zeros(64, np.float32), dy,
                      w_gran="row", dy_round="stochastic", philox_seed=3, tags=[INT8, FP16], nhwc=act)


@dataclass
class ChainCase:
    name: str
    x: np.ndarray                      # [tokens, width]
    weights: List[np.ndarray]          # layer l: [out_l, in_l]
    tags: List[int]
    dy_last: np.ndarray
    philox_seed: int = 4


def config4(tokens: int = 8192, width: int = 1024, hidden: int = 4096, layers: int = 12) -> ChainCase:
    """Mixed-precision MLP stack: (width->hidden, GELU, hidden->width) repeated, tags per layer."""
    seed = 4
    while True:
        tags = [(INT8, FP16, FP32)[i] for i in np.random.default_rng(seed).integers(0, 3, size=layers)]
        if len(set(tags)) == 3 or layers < 3:
            break
        seed += 1
    rng = np.random.default_rng(4)
    x = _normal(rng, (tokens, width), 1.0, np.float32)
    weights = []
    for l in range(layers):
        shape = (hidden, width) if l % 2 == 0 else (width, hidden)
        weights.append(_normal(rng, shape, 0.02, np.float32))
    out_w = width if layers % 2 == 0 else hidden
    dy_last = _normal(rng, (tokens, out_w), 1e-2, np.float32)
    return ChainCase("c4_mixed_mlp", x, weights, tags, dy_last, philox_seed=4)


def config5(tokens: int = 16384) -> Dict[str, LinearCase]:
    """BERT-large-scale linears: 1024 -> 4096 ("up") and 4096 -> 1024 ("down")."""
    rng = np.random.default_rng(7)
    x_up = _normal(rng, (tokens, 1024), 1.0, np.float16)
    w_up = _normal(rng, (4096, 1024), 0.02, np.float32)
    dy_up = _normal(rng, (tokens, 4096), 1e-3, np.float16)
    x_dn = _normal(rng, (tokens, 4096), 1.0, np.float16)
    w_dn = _normal(rng, (1024, 4096), 0.02, np.float32)
    dy_dn = _normal(rng, (tokens, 1024), 1e-3, np.float16)
    mk = lambda n, x, w, dy: LinearCase(n, x, w, np.zeros(w.shape[0], np.float32), dy, w_gran="row",
                                        dy_round="stochastic", philox_seed=7, tags=[INT8, FP16])
    return {"up": mk("c5_bert_large_up", x_up, w_up, dy_up),
            "down": mk("c5_bert_large_down", x_dn, w_dn, dy_dn)}


def ragged_case(m: int, n: int, k: int, seed: int, dtype=np.float32, sigma_dy: float = 1e-2) -> LinearCase:
    """Arbitrary-shape case for tile-boundary and ragged-tail tests."""
    rng = np.random.default_rng(seed)
    x = _normal(rng, (m, k), 1.0, dtype)
    w = _normal(rng, (n, k), 0.02, np.float32)
    dy = _normal(rng, (m, n), sigma_dy, dtype)
    bias = _normal(rng, (n,), 0.1, np.float32)
    return LinearCase(f"ragged_{m}x{n}x{k}", x, w, bias, dy, w_gran="row",
                      dy_round="stochastic", philox_seed=seed, tags=[INT8, FP16, FP32])
