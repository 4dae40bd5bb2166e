"""Thin Python binding of libqsync.so: argument marshalling only.

Every function has the name and argument order of its C counterpart in
``include/qsync.h`` and takes torch tensors (for their device pointers) where the
C function takes pointers.  No arithmetic happens here.  The library is loaded
from the package directory; if it is missing the import of this module fails
loudly -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

INT8, FP16, FP32 = 8, 16, 32                       # qsync_prec_t
QUANT_FIXED, QUANT_FLOAT = 0, 1                    # qsync_quant_kind_t
F32, F16, I8, I32 = 0, 1, 2, 3                     # qsync_dtype_t
PER_TENSOR, PER_ROW, PER_COL = 0, 1, 2             # qsync_gran_t
ROUND_NEAREST, ROUND_STOCHASTIC, ROUND_FLOOR = 0, 1, 2
OK, ERR_NULL, ERR_BAD_ENUM, ERR_BAD_SHAPE, ERR_UNSUPPORTED, ERR_ALIGN, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4, -5, -6, -7

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libqsync.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2407_02327_amd.build`")
lib = ctypes.CDLL(LIB_PATH)

_vp, _i, _i64, _u64, _sz, _f = (ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64,
                                 ctypes.c_size_t, ctypes.c_float)
SIGNATURES = {
    "qsync_absmax_scale": (_i, [_vp, _i, _i64, _i64, _i64, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "qsync_absmax_workspace_bytes": (_sz, [_i64, _i64, _i]),
    "qsync_absmax_scale_static": (_i, [_vp, _i, _i64, _i64, _i64, _i, _vp, _vp, _vp, _vp, _vp, _vp]),
    "qsync_quantize": (_i, [_vp, _i, _i64, _i64, _i64, _i, _i, _i, _i, _u64, _u64, _vp, _vp, _vp, _vp]),
    "qsync_qlinear_fwd": (_i, [_i, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _i, _vp, _vp, _i, _vp, _vp, _sz, _vp]),
    "qsync_absmax_quantize": (_i, [_vp, _i, _i64, _i64, _i, _i, ctypes.c_uint64, ctypes.c_uint64, _vp, _vp, _vp, _vp, _vp,
                                   _vp, _sz, _i, _vp]),
    "qsync_absmax_quantize_workspace_bytes": (_sz, [_i64, _i64]),
    "qsync_qlinear_fwd_amax": (_i, [_i, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _i, _vp, _vp, _i, _vp, _vp, _vp, _sz, _vp]),
    "qsync_scale_from_amax": (_i, [_vp, _i, _vp, _vp, _i, _vp]),
    "qsync_qlinear_fwd_codes": (_i, [_i, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _i, _vp, _vp, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]),
    "qsync_transpose_i8": (_i, [_vp, _i64, _i64, _vp, _vp]),
    "qsync_qlinear_bwd": (_i, [_i, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _vp, _i, _vp, _i,
                               _vp, _vp, _i, _vp, _vp, _vp, _sz, _vp]),
    "qsync_qlinear_workspace_bytes": (_sz, [_i, _i64, _i64, _i64]),
    "qsync_qlinear_bwd_rm": (_i, [_i, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _i, _vp, _i, _vp, _i, _vp, _vp, _i, _vp, _vp,
                                 _vp, _sz, _vp]),
    "qsync_qlinear_bwd_rm_workspace_bytes": (_sz, [_i, _i64, _i64, _i64]),
    "qsync_qlinear_bwd_fp16_of_int8": (_i, [_i64, _i64, _i64, _vp, _i, _vp, _i, _vp, _vp, _vp, _i, _vp, _i, _vp, _i, _vp, _vp, _sz,
                                           ctypes.POINTER(ctypes.c_size_t), _vp]),
    "qsync_qlinear_bwd_fp16_of_int8_workspace_bytes": (_sz, [_i64, _i64, _i64, _i]),
    "qsync_qlinear_bwd_workspace_bytes": (_sz, [_i, _i64, _i64, _i64]),
    "qsync_im2col3x3_i8": (_i, [_vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp]),
    "qsync_conv3x3_fwd": (_i, [_i, _i64, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _i, _vp, _vp, _i, _vp, _vp]),
    "qsync_conv3x3_fwd_amax": (_i, [_i, _i64, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _i, _vp, _vp, _i, _vp, _vp, _vp]),
    "qsync_debug_set_gemm_tile": (None, [_i]),
    "qsync_debug_set_gemm_persistent": (None, [_i]),
    "qsync_conv3x3_wgrad": (_i, [_i, _i64, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _i, _vp, _vp, _sz, _vp]),
    "qsync_conv3x3_wgrad_workspace_bytes": (_sz, [_i, _i64, _i64, _i64, _i64, _i64]),
    "qsync_conv3x3_prepare_weights": (_i, [_vp, _i, _i64, _i64, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "qsync_conv3x3_prepare_weights_workspace_bytes": (_sz, [_i64, _i64]),
    "qsync_probe_mfma": (_i, [_i, _i, _i, _vp, ctypes.POINTER(ctypes.c_double), _vp]),
    "qsync_prepare_weights": (_i, [_vp, _i, _i64, _i64, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "qsync_conv3x3_wflip": (_i, [_vp, _i, _i64, _i64, _vp, _vp]),
    "qsync_dequantize": (_i, [_vp, _i, _i64, _i64, _i64, _vp, _vp, _f, _vp, _vp, _vp, _i, _vp]),
    "qsync_variance_increment": (_i, [_i, _vp, _vp, _vp, ctypes.c_double, ctypes.c_double, _i, ctypes.c_double, _i64, _i64,
                                      ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double)]),
    "qsync_last_hip_error": (_i, []),
    "qsync_strerror": (ctypes.c_char_p, [_i]),
    "qsync_version": (_i, []),
}
for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(lib, _name)
    _fn.restype, _fn.argtypes = _res, _args

_DTYPE_OF = {torch.float32: F32, torch.float16: F16, torch.int8: I8, torch.int32: I32}


class QsyncError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        msg = lib.qsync_strerror(status).decode()
        if status == ERR_HIP:
            msg += f" (hipError_t {lib.qsync_last_hip_error()})"
        super().__init__(f"qsync status {status}: {msg}")


def _check(status: int) -> None:
    if status != OK:
        raise QsyncError(status)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def dtype_code(t: torch.Tensor) -> int:
    return _DTYPE_OF[t.dtype]


def _bytes(ws: Optional[torch.Tensor]) -> int:
    return 0 if ws is None else ws.numel() * ws.element_size()


def qsync_absmax_workspace_bytes(rows: int, cols: int, gran: int) -> int:
    return lib.qsync_absmax_workspace_bytes(rows, cols, gran)


def qsync_qlinear_workspace_bytes(tag: int, M: int, N: int, K: int) -> int:
    return lib.qsync_qlinear_workspace_bytes(tag, M, N, K)


def qsync_qlinear_bwd_workspace_bytes(tag: int, M: int, N: int, K: int) -> int:
    return lib.qsync_qlinear_bwd_workspace_bytes(tag, M, N, K)


def qsync_absmax_scale(x, rows, cols, ld, gran, bits, scale, inv_scale, amax_opt, colsum_opt, workspace,
                       stream=None, sumsq_opt=None) -> None:
    _check(lib.qsync_absmax_scale(_ptr(x), dtype_code(x), rows, cols, ld, gran, bits, _ptr(scale), _ptr(inv_scale),
                                  _ptr(amax_opt), _ptr(colsum_opt), _ptr(sumsq_opt), _ptr(workspace),
                                  _bytes(workspace), _stream(stream)))


def qsync_absmax_scale_static(x, rows, cols, ld, bits, scale, inv_scale, amax_opt, colsum_opt, sumsq_opt,
                              stream=None) -> None:
    _check(lib.qsync_absmax_scale_static(_ptr(x), dtype_code(x), rows, cols, ld, bits, _ptr(scale), _ptr(inv_scale),
                                         _ptr(amax_opt), _ptr(colsum_opt), _ptr(sumsq_opt), _stream(stream)))


def qsync_quantize(x, rows, cols, ld, tag, bits, gran, rnd, philox_seed, philox_offset, inv_scale, q_opt, qT_opt,
                   stream=None) -> None:
    _check(lib.qsync_quantize(_ptr(x), dtype_code(x), rows, cols, ld, tag, bits, gran, rnd, philox_seed,
                              philox_offset, _ptr(inv_scale), _ptr(q_opt), _ptr(qT_opt), _stream(stream)))


def qsync_qlinear_fwd(tag, M, N, K, xq, sx, wq, sw, wgran, bias_opt, y, acc_dump_opt, workspace, stream=None) -> None:
    _check(lib.qsync_qlinear_fwd(tag, M, N, K, _ptr(xq), _ptr(sx), _ptr(wq), _ptr(sw), wgran, _ptr(bias_opt),
                                 _ptr(y), dtype_code(y), _ptr(acc_dump_opt), _ptr(workspace), _bytes(workspace),
                                 _stream(stream)))


def qsync_absmax_quantize_workspace_bytes(rows, cols) -> int:
    return int(lib.qsync_absmax_quantize_workspace_bytes(rows, cols))


def qsync_absmax_quantize(x, rows, cols, bits, rnd, seed, offset, scale, inv_scale, amax_opt, q_opt, qT_opt, workspace,
                          poll_limit=-1, stream=None) -> None:
    _check(lib.qsync_absmax_quantize(_ptr(x), dtype_code(x), rows, cols, bits, rnd, seed, offset, _ptr(scale),
                                     _ptr(inv_scale), _ptr(amax_opt), _ptr(q_opt), _ptr(qT_opt), _ptr(workspace),
                                     _bytes(workspace), poll_limit, _stream(stream)))


def qsync_qlinear_fwd_amax(tag, M, N, K, xq, sx, wq, sw, wgran, bias_opt, y, acc_dump_opt, y_amax, workspace,
                           stream=None) -> None:
    _check(lib.qsync_qlinear_fwd_amax(tag, M, N, K, _ptr(xq), _ptr(sx), _ptr(wq), _ptr(sw), wgran, _ptr(bias_opt),
                                      _ptr(y), dtype_code(y), _ptr(acc_dump_opt), _ptr(y_amax), _ptr(workspace),
                                      _bytes(workspace), _stream(stream)))


def qsync_qlinear_fwd_codes(tag, M, N, K, xq, sx, wq, sw, wgran, bias_opt, y, bits, next_inv_scale, yq, y_amax_opt, workspace,
                            stream=None) -> None:
    _check(lib.qsync_qlinear_fwd_codes(tag, M, N, K, _ptr(xq), _ptr(sx), _ptr(wq), _ptr(sw), wgran, _ptr(bias_opt), _ptr(y),
                                       dtype_code(y), bits, _ptr(next_inv_scale), _ptr(yq), _ptr(y_amax_opt), _ptr(workspace),
                                       _bytes(workspace), _stream(stream)))


def qsync_transpose_i8(a, rows, cols, out, stream=None) -> None:
    _check(lib.qsync_transpose_i8(_ptr(a), rows, cols, _ptr(out), _stream(stream)))


def qsync_scale_from_amax(amax, bits, scale, inv_scale, consume=True, stream=None) -> None:
    _check(lib.qsync_scale_from_amax(_ptr(amax), bits, _ptr(scale), _ptr(inv_scale), 1 if consume else 0,
                                     _stream(stream)))


def qsync_qlinear_bwd(tag, M, N, K, dyq, dyqT, sdy, xqT, sx, wqbT, swb, wbgran, dx_opt, dw_opt, db_opt, dy_float_opt,
                      acc_dx_dump_opt, acc_dw_dump_opt, workspace, stream=None) -> None:
    _check(lib.qsync_qlinear_bwd(tag, M, N, K, _ptr(dyq), _ptr(dyqT), _ptr(sdy), _ptr(xqT), _ptr(sx), _ptr(wqbT),
                                 _ptr(swb), wbgran,
                                 _ptr(dx_opt), F32 if dx_opt is None else dtype_code(dx_opt),
                                 _ptr(dw_opt), F32 if dw_opt is None else dtype_code(dw_opt),
                                 _ptr(db_opt), _ptr(dy_float_opt),
                                 F32 if dy_float_opt is None else dtype_code(dy_float_opt),
                                 _ptr(acc_dx_dump_opt), _ptr(acc_dw_dump_opt), _ptr(workspace), _bytes(workspace),
                                 _stream(stream)))


def qsync_qlinear_bwd_rm_workspace_bytes(tag: int, M: int, N: int, K: int) -> int:
    return int(lib.qsync_qlinear_bwd_rm_workspace_bytes(tag, M, N, K))


def qsync_qlinear_bwd_rm(tag, M, N, K, dyq, sdy, xq, sx, wqbT, swb, wbgran, dx_opt, dw_opt, db_opt, dy_float_opt, acc_dx_dump_opt,
                         acc_dw_dump_opt, workspace, stream=None) -> None:
    _check(lib.qsync_qlinear_bwd_rm(tag, M, N, K, _ptr(dyq), _ptr(sdy), _ptr(xq), _ptr(sx), _ptr(wqbT), _ptr(swb), wbgran,
                                    _ptr(dx_opt), dtype_code(dx_opt) if dx_opt is not None else F32,
                                    _ptr(dw_opt), dtype_code(dw_opt) if dw_opt is not None else F32, _ptr(db_opt),
                                    _ptr(dy_float_opt), dtype_code(dy_float_opt) if dy_float_opt is not None else F32,
                                    _ptr(acc_dx_dump_opt), _ptr(acc_dw_dump_opt), _ptr(workspace), _bytes(workspace),
                                    _stream(stream)))


def qsync_qlinear_bwd_fp16_of_int8_workspace_bytes(M: int, N: int, K: int, dy_dtype_code: int) -> int:
    return int(lib.qsync_qlinear_bwd_fp16_of_int8_workspace_bytes(M, N, K, dy_dtype_code))


def qsync_qlinear_bwd_fp16_of_int8(M, N, K, dy, xq_or_xqT, x_rowmajor, sx, wq, sw, wgran, dx_opt, dw_opt, db_opt, workspace,
                                   stream=None):
    """Returns the five byte offsets of the binary16 operands inside the workspace (x_hat^T -- x_hat when x_rowmajor --,
    w_hat, w_hat^T, dY16, dY16^T)."""
    offs = (ctypes.c_size_t * 5)()
    _check(lib.qsync_qlinear_bwd_fp16_of_int8(M, N, K, _ptr(dy), dtype_code(dy), _ptr(xq_or_xqT), int(bool(x_rowmajor)), _ptr(sx),
                                              _ptr(wq), _ptr(sw), wgran,
                                              _ptr(dx_opt), dtype_code(dx_opt) if dx_opt is not None else F32,
                                              _ptr(dw_opt), dtype_code(dw_opt) if dw_opt is not None else F32, _ptr(db_opt),
                                              _ptr(workspace), _bytes(workspace), offs, _stream(stream)))
    return [int(o) for o in offs]


def qsync_conv3x3_fwd(tag, nimg, H, W, C, N, xq, sx, wq, sw, wgran, bias_opt, y, acc_dump_opt=None, stream=None) -> None:
    _check(lib.qsync_conv3x3_fwd(tag, nimg, H, W, C, N, _ptr(xq), _ptr(sx), _ptr(wq), _ptr(sw), wgran, _ptr(bias_opt),
                                 _ptr(y), dtype_code(y), _ptr(acc_dump_opt), _stream(stream)))


def qsync_conv3x3_fwd_amax(tag, nimg, H, W, C, N, xq, sx, wq, sw, wgran, bias_opt, y, acc_dump_opt, y_amax, stream=None) -> None:
    _check(lib.qsync_conv3x3_fwd_amax(tag, nimg, H, W, C, N, _ptr(xq), _ptr(sx), _ptr(wq), _ptr(sw), wgran, _ptr(bias_opt),
                                      _ptr(y), dtype_code(y), _ptr(acc_dump_opt), _ptr(y_amax), _stream(stream)))


def qsync_prepare_weights(w, N, K, bits, sw, iw, aw_opt, wq, swb, iwb, wqbT, workspace, stream=None) -> None:
    _check(lib.qsync_prepare_weights(_ptr(w), dtype_code(w), N, K, bits, _ptr(sw), _ptr(iw), _ptr(aw_opt), _ptr(wq),
                                     _ptr(swb), _ptr(iwb), _ptr(wqbT), _ptr(workspace), _bytes(workspace), _stream(stream)))


def qsync_probe_mfma(tag: int, random_operands: int, iters: int, out, stream=None) -> float:
    """Launches the probe on `stream` and returns the operation count of the launch (the caller times it)."""
    ops = ctypes.c_double(0.0)
    _check(lib.qsync_probe_mfma(tag, int(random_operands), iters, _ptr(out), ctypes.byref(ops), _stream(stream)))
    return ops.value


def qsync_conv3x3_prepare_weights_workspace_bytes(N: int, C: int) -> int:
    return lib.qsync_conv3x3_prepare_weights_workspace_bytes(N, C)


def qsync_conv3x3_prepare_weights(w, N, C, bits, sw, iw, wq, swb, iwb, wflip, workspace, stream=None) -> None:
    _check(lib.qsync_conv3x3_prepare_weights(_ptr(w), dtype_code(w), N, C, bits, _ptr(sw), _ptr(iw), _ptr(wq), _ptr(swb),
                                             _ptr(iwb), _ptr(wflip), _ptr(workspace), _bytes(workspace), _stream(stream)))


def qsync_conv3x3_wgrad_workspace_bytes(tag: int, nimg: int, H: int, W: int, C: int, N: int) -> int:
    return lib.qsync_conv3x3_wgrad_workspace_bytes(tag, nimg, H, W, C, N)


def qsync_conv3x3_wgrad(tag, nimg, H, W, C, N, xq, sx, dyq, sdy, dw, acc_dump_opt, workspace, stream=None) -> None:
    _check(lib.qsync_conv3x3_wgrad(tag, nimg, H, W, C, N, _ptr(xq), _ptr(sx), _ptr(dyq), _ptr(sdy), _ptr(dw), dtype_code(dw),
                                   _ptr(acc_dump_opt), _ptr(workspace), _bytes(workspace), _stream(stream)))


def qsync_debug_set_gemm_tile(tile: int) -> None:
    lib.qsync_debug_set_gemm_tile(tile)


def qsync_debug_set_gemm_persistent(mode: int) -> None:
    lib.qsync_debug_set_gemm_persistent(mode)


def qsync_conv3x3_wflip(w, N, C, wflip, stream=None) -> None:
    _check(lib.qsync_conv3x3_wflip(_ptr(w), dtype_code(w), N, C, _ptr(wflip), _stream(stream)))


def qsync_im2col3x3_i8(xq, nimg, H, W, C, a_opt, aT_opt, stream=None) -> None:
    _check(lib.qsync_im2col3x3_i8(_ptr(xq), nimg, H, W, C, _ptr(a_opt), _ptr(aT_opt), _stream(stream)))


def qsync_dequantize(a, rows, cols, ld, row_scale_opt, col_scale_opt, tensor_scale, col_bias_opt, y,
                     stream=None, tensor_scale_dev_opt=None) -> None:
    _check(lib.qsync_dequantize(_ptr(a), dtype_code(a), rows, cols, ld, _ptr(row_scale_opt), _ptr(col_scale_opt),
                                float(tensor_scale), _ptr(tensor_scale_dev_opt), _ptr(col_bias_opt), _ptr(y),
                                dtype_code(y), _stream(stream)))


class TensorStatsC(ctypes.Structure):
    """qsync_tensor_stats_t"""
    _fields_ = [("sumsq", ctypes.c_double), ("amax", ctypes.c_double), ("D", ctypes.c_int64)]


def qsync_variance_increment(kind: int, x, v, grad_v, q_x: float, q_v: float, k: int, gamma: float, d_o: int,
                             d_L: int) -> dict:
    """x, v, grad_v: objects with fields sumsq, amax, D.  Returns dict(sigma_fp, sigma_bp, omega) (host doubles)."""
    c = [TensorStatsC(float(t.sumsq), float(t.amax), int(t.D)) for t in (x, v, grad_v)]
    out = [ctypes.c_double() for _ in range(3)]
    _check(lib.qsync_variance_increment(kind, ctypes.byref(c[0]), ctypes.byref(c[1]), ctypes.byref(c[2]), float(q_x),
                                        float(q_v), int(k), float(gamma), int(d_o), int(d_L), ctypes.byref(out[0]),
                                        ctypes.byref(out[1]), ctypes.byref(out[2])))
    return dict(sigma_fp=out[0].value, sigma_bp=out[1].value, omega=out[2].value)
