"""Buffer plumbing for one quantized linear operator on the GPU.

`QLinear` owns the device buffers of one operator (codes, scales, transposed copies,
outputs, workspace) and sequences the C-ABI calls of ``qsync.py`` for a forward and a
backward pass.  All arithmetic runs inside libqsync's kernels; nothing here computes.
Buffers are allocated once in the constructor, so `forward` / `backward` allocate nothing
and can be timed or replayed.

Call order per step (paper: Cost Mapper paragraph, casting cost in the forward pass for
inputs and weights, extra casting in the backward pass; Backend section):
  forward : absmax+quantize X (codes and transposed codes), absmax+quantize W
            (per output channel for the forward, per input feature and transposed for dX),
            GEMM with fused dequantize + bias
  backward: absmax+quantize dY (stochastic rounding; codes and transposed codes),
            dX GEMM, dW GEMM, bias gradient
  backward, bwd_tag = FP16 on an INT8 operator (the pairing the paper itself runs, footnote in the
            Cost Mapper paragraph): dequantize the saved codes to binary16, cast dY, FP16 GEMMs
"""
from __future__ import annotations

from typing import Optional

import torch

from . import qsync as Q

_TORCH_OF_TAG = {Q.INT8: torch.int8, Q.FP16: torch.float16, Q.FP32: torch.float32}


def _ws(nbytes: int, device) -> Optional[torch.Tensor]:
    # zero-filled once: qsync_absmax_scale keeps block arrival counters at the start of its workspace
    return torch.zeros(max(nbytes, 256), dtype=torch.uint8, device=device)


class QLinear:
    def __init__(self, tag: int, M: int, N: int, K: int, x_dtype=torch.float16, w_dtype=torch.float32,
                 dy_dtype=None, y_dtype=torch.float32, dx_dtype=torch.float16, dw_dtype=torch.float32,
                 w_gran: int = Q.PER_ROW, dy_round: int = Q.ROUND_STOCHASTIC, philox_seed: int = 0,
                 bias: bool = True, dump_acc: bool = False, bits: int = 8, device="cuda",
                 bwd_tag: Optional[int] = None, collect_y_amax: bool = False, transposed_copies: Optional[bool] = None):
        """transposed_copies: INT8 and FP16 tags.  False: the activation and gradient operands are kept row-major only
        and the weight-gradient GEMM reads them as they are (qsync_qlinear_bwd_rm; needs M % 128 == 0 and N, K
        multiples of 16 -- 8 for FP16); True: the conversion also writes the transposed copies xqT / dyqT for
        qsync_qlinear_bwd.
        None picks False when the shape allows it and the copies are large enough to be worth it: the row-major
        weight-gradient GEMM is 6-8 % slower on 256-wide tiles and loses the 64-wide tile, the quantizer saves one
        byte written per element (measured on MI355X: 16384x4096x1024 operators 0.803 -> 0.749 ms per step,
        4096x768x3072 operators 0.129 -> 0.132 ms)."""
        self.tag, self.M, self.N, self.K = tag, M, N, K
        # max |Y| collected by the forward GEMM's epilogue, for a consumer that quantizes Y as it is
        self.y_amax = torch.zeros(1, dtype=torch.float32, device=device) if collect_y_amax else None
        self.bwd_tag = tag if bwd_tag is None else bwd_tag
        if self.bwd_tag != tag and not (tag == Q.INT8 and self.bwd_tag == Q.FP16):
            raise ValueError("bwd_tag: only the FP16 backward of an INT8 forward differs from the forward tag")
        self.w_gran, self.dy_round, self.seed, self.bits = w_gran, dy_round, philox_seed, bits
        self.offset = 0
        mult = 16 if tag == Q.INT8 else 8
        rm_ok = tag in (Q.INT8, Q.FP16) and M % 128 == 0 and N % mult == 0 and K % mult == 0      # (either backward tag)
        if transposed_copies is False and not rm_ok:
            raise ValueError("transposed_copies=False needs tag INT8 or FP16 with the same backward tag, M % 128 == 0, "
                             "N and K multiples of 16 (FP16: 8)")
        self.rowmajor_bwd = (rm_ok and M * (N + K) >= (32 << 20)) if transposed_copies is None else not transposed_copies
        dy_dtype = dy_dtype or x_dtype
        dev = device
        e = lambda *s, dt: torch.empty(*s, dtype=dt, device=dev)
        qd = _TORCH_OF_TAG[tag]
        f32 = torch.float32
        # operands in the layouts the GEMMs consume (contraction axis contiguous)
        self.xq, self.xqT = e(M, K, dt=qd), (e(K, M, dt=qd) if not self.rowmajor_bwd else None)
        self.wq, self.wqbT = e(N, K, dt=qd), e(K, N, dt=qd)
        fp16_bwd = self.bwd_tag != tag           # that backward converts dY itself: no gradient operands are kept here
        self.dyq = e(M, N, dt=qd) if not fp16_bwd else None
        self.dyqT = e(N, M, dt=qd) if not (self.rowmajor_bwd or fp16_bwd) else None
        # scales (amax/qmax), inverse scales, and the raw maxima
        self.sx, self.ix, self.ax = e(1, dt=f32), e(1, dt=f32), e(1, dt=f32)
        nsw = N if w_gran == Q.PER_ROW else 1
        nswb = K if w_gran == Q.PER_ROW else 1
        self.sw, self.iw, self.aw = e(nsw, dt=f32), e(nsw, dt=f32), e(nsw, dt=f32)
        self.swb, self.iwb = e(nswb, dt=f32), e(nswb, dt=f32)
        self.sdy, self.idy, self.ady = e(1, dt=f32), e(1, dt=f32), e(1, dt=f32)
        self.bias = torch.zeros(N, dtype=f32, device=dev) if bias else None
        self.y, self.dx, self.dw = e(M, N, dt=y_dtype), e(M, K, dt=dx_dtype), e(N, K, dt=dw_dtype)
        self.db = e(N, dt=f32)
        self.acc = self.acc_dx = self.acc_dw = None
        if dump_acc and tag == Q.INT8:
            i32 = torch.int32
            self.acc, self.acc_dx, self.acc_dw = e(M, N, dt=i32), e(M, K, dt=i32), e(N, K, dt=i32)
        nws = max(Q.qsync_absmax_workspace_bytes(M, K, Q.PER_TENSOR), Q.qsync_absmax_workspace_bytes(M, N, Q.PER_TENSOR))
        self.ws_absmax = _ws(nws, dev)
        # the weight conversion may run on a second stream beside the activation conversion: own scratch
        self.ws_absmax_w = _ws(max(Q.qsync_absmax_workspace_bytes(N, K, Q.PER_COL),
                                   Q.qsync_absmax_workspace_bytes(N, K, Q.PER_TENSOR)), dev)
        self.ws_fwd = _ws(Q.qsync_qlinear_workspace_bytes(tag, M, N, K), dev)
        self.ws_bwd = _ws(max(Q.qsync_qlinear_bwd_workspace_bytes(self.bwd_tag, M, N, K),
                              Q.qsync_qlinear_bwd_rm_workspace_bytes(tag, M, N, K) if self.rowmajor_bwd else 0), dev)
        if self.bwd_tag != tag:
            # FP16 backward of the INT8 forward: one C-ABI call; its workspace receives the binary16 operands
            # (dequantized X^T, dequantized W and its transpose, cast dY and its transpose)
            self.dy_dtype = dy_dtype
            nb = Q.qsync_qlinear_bwd_fp16_of_int8_workspace_bytes(M, N, K, Q._DTYPE_OF[dy_dtype])
            self.ws_bwd16 = torch.zeros(max(nb, 256), dtype=torch.uint8, device=dev)

    # ---- precision conversion -----------------------------------------------------------
    def convert_x(self, x: torch.Tensor, stream=None, x_amax: Optional[torch.Tensor] = None) -> None:
        """x_amax: device float holding max |x| already (the producer's `y_amax`); it replaces the pass over x
        that finds the maximum and is left at zero for the producer's next step."""
        M, K = self.M, self.K
        if self.tag == Q.INT8:
            if x_amax is not None:
                Q.qsync_scale_from_amax(x_amax, self.bits, self.sx, self.ix, True, stream)
            else:
                # maximum, scale and codes: one launch for small activations, the two separate passes otherwise
                Q.qsync_absmax_quantize(x, M, K, self.bits, Q.ROUND_NEAREST, 0, 0, self.sx, self.ix, self.ax, self.xq,
                                        self.xqT, self.ws_absmax, -1, stream)
                return
            Q.qsync_quantize(x, M, K, K, Q.INT8, self.bits, Q.PER_TENSOR, Q.ROUND_NEAREST, 0, 0, self.ix, self.xq,
                             self.xqT, stream)
        elif x.dtype == _TORCH_OF_TAG[self.tag] and x.is_contiguous():
            # already in the operand type: the tensor itself is the saved operand, only its transpose (if kept) is written
            self.xq = x
            if self.xqT is not None:
                Q.qsync_quantize(x, M, K, K, self.tag, 0, 0, 0, 0, 0, None, None, self.xqT, stream)
        else:
            Q.qsync_quantize(x, M, K, K, self.tag, 0, 0, 0, 0, 0, None, self.xq, self.xqT, stream)

    def convert_x_nhwc(self, act: torch.Tensor, stream=None) -> None:
        """3x3 / stride 1 / pad 1 convolution lowered to this operator (K = 9*C): the NHWC activation is
        quantized once and its codes are expanded into the patch matrix and its transpose, instead of
        quantizing a nine times larger fp16 patch matrix (INT8 tag only)."""
        b, h, w, c = act.shape
        assert self.tag == Q.INT8 and b * h * w == self.M and 9 * c == self.K
        if not hasattr(self, "xq_nhwc"):
            self.xq_nhwc = torch.empty(b * h * w, c, dtype=torch.int8, device=act.device)
        Q.qsync_absmax_scale(act, self.M, c, c, Q.PER_TENSOR, self.bits, self.sx, self.ix, self.ax, None, self.ws_absmax,
                             stream)
        Q.qsync_quantize(act, self.M, c, c, Q.INT8, self.bits, Q.PER_TENSOR, Q.ROUND_NEAREST, 0, 0, self.ix, self.xq_nhwc,
                         None, stream)
        Q.qsync_im2col3x3_i8(self.xq_nhwc, b, h, w, c, self.xq, self.xqT, stream)

    def convert_w(self, w: torch.Tensor, stream=None) -> None:
        N, K = self.N, self.K
        if self.tag != Q.INT8:
            Q.qsync_quantize(w, N, K, K, self.tag, 0, 0, 0, 0, 0, None, self.wq, self.wqbT, stream)
            return
        if self.w_gran == Q.PER_TENSOR:       # one quantization serves the forward and dX
            Q.qsync_absmax_scale(w, N, K, K, Q.PER_TENSOR, self.bits, self.sw, self.iw, self.aw, None, self.ws_absmax_w,
                                 stream)
            Q.qsync_quantize(w, N, K, K, Q.INT8, self.bits, Q.PER_TENSOR, Q.ROUND_NEAREST, 0, 0, self.iw, self.wq,
                             self.wqbT, stream)
            self.swb = self.sw
            return
        # per-output-channel codes for the forward; dX contracts over the output channels, so its weight codes
        # carry one scale per input feature (second quantization, stored transposed): one fused call
        Q.qsync_prepare_weights(w, N, K, self.bits, self.sw, self.iw, self.aw, self.wq, self.swb, self.iwb, self.wqbT,
                                self.ws_absmax_w, stream)

    def convert_dy(self, dy: torch.Tensor, stream=None) -> None:
        M, N, K = self.M, self.N, self.K
        if self.bwd_tag != self.tag:
            return          # the FP16 backward converts its operands inside its own call (gemm_bwd)
        if self.tag == Q.INT8:
            # the same pass over dY yields its absmax and the bias gradient db (column sums)
            Q.qsync_absmax_scale(dy, M, N, N, Q.PER_TENSOR, self.bits, self.sdy, self.idy, self.ady, self.db,
                                 self.ws_absmax, stream)
            Q.qsync_quantize(dy, M, N, N, Q.INT8, self.bits, Q.PER_TENSOR, self.dy_round, self.seed, self.offset,
                             self.idy, self.dyq, self.dyqT, stream)
            self.last_dy_offset = self.offset
            self.offset += (M * N + 7) // 8
        elif dy.dtype == _TORCH_OF_TAG[self.tag] and dy.is_contiguous():
            self.dyq = dy
            if self.dyqT is not None:
                Q.qsync_quantize(dy, M, N, N, self.tag, 0, 0, 0, 0, 0, None, None, self.dyqT, stream)
        else:
            Q.qsync_quantize(dy, M, N, N, self.tag, 0, 0, 0, 0, 0, None, self.dyq, self.dyqT, stream)

    # ---- GEMMs ---------------------------------------------------------------------------
    def gemm_fwd(self, stream=None) -> None:
        if self.y_amax is not None:
            Q.qsync_qlinear_fwd_amax(self.tag, self.M, self.N, self.K, self.xq, self.sx, self.wq, self.sw, self.w_gran,
                                     self.bias, self.y, self.acc, self.y_amax, self.ws_fwd, stream)
            return
        Q.qsync_qlinear_fwd(self.tag, self.M, self.N, self.K, self.xq, self.sx, self.wq, self.sw, self.w_gran,
                            self.bias, self.y, self.acc, self.ws_fwd, stream)

    def gemm_fwd_codes(self, consumer: "QLinear", stream=None) -> None:
        """Forward GEMM whose epilogue also writes the INT8 codes of Y straight into `consumer.xq`, quantized with
        the inverse scale the consumer holds (`consumer.ix`, e.g. from the previous step); max |Y| of this step
        goes to `self.y_amax` when that is collected."""
        Q.qsync_qlinear_fwd_codes(self.tag, self.M, self.N, self.K, self.xq, self.sx, self.wq, self.sw, self.w_gran,
                                  self.bias, self.y, consumer.bits, consumer.ix, consumer.xq, self.y_amax, self.ws_fwd,
                                  stream)

    def forward_from_codes(self, w: torch.Tensor, stream=None) -> torch.Tensor:
        """Forward of an INT8 operator whose activation codes (`xq`, scale `sx`/`ix`) were written by its
        producer's epilogue: only the transposed copy for the weight gradient is still to be made."""
        self.convert_w(w, stream)
        if self.xqT is not None:
            Q.qsync_transpose_i8(self.xq, self.M, self.K, self.xqT, stream)
        self.gemm_fwd(stream)
        return self.y

    def gemm_bwd(self, dy: Optional[torch.Tensor], stream=None) -> None:
        if self.bwd_tag != self.tag:
            self._fp16_backward(dy, self.dx, self.dw, self.db, stream)
            return
        want_db = dy is not None and self.tag != Q.INT8      # INT8: db already came out of the absmax pass over dY
        if self.rowmajor_bwd:
            Q.qsync_qlinear_bwd_rm(self.tag, self.M, self.N, self.K, self.dyq, self.sdy, self.xq, self.sx, self.wqbT, self.swb,
                                   self.w_gran if self.w_gran == Q.PER_TENSOR else Q.PER_ROW, self.dx, self.dw,
                                   self.db if want_db else None, dy if want_db else None,
                                   self.acc_dx, self.acc_dw, self.ws_bwd, stream)
            return
        Q.qsync_qlinear_bwd(self.tag, self.M, self.N, self.K, self.dyq, self.dyqT, self.sdy, self.xqT, self.sx,
                            self.wqbT, self.swb, self.w_gran if self.w_gran == Q.PER_TENSOR else Q.PER_ROW,
                            self.dx, self.dw, self.db if want_db else None, dy if want_db else None, self.acc_dx,
                            self.acc_dw, self.ws_bwd, stream)

    def _fp16_backward(self, dy, dx, dw, db, stream) -> None:
        M, N, K = self.M, self.N, self.K
        if not dy.is_contiguous():
            dy = dy.contiguous()
        rm = self.rowmajor_bwd
        offs = Q.qsync_qlinear_bwd_fp16_of_int8(M, N, K, dy, self.xq if rm else self.xqT, rm, self.sx, self.wq, self.sw,
                                                self.w_gran, dx, dw, db, self.ws_bwd16, stream)
        h = torch.float16
        view = lambda off, r, c: self.ws_bwd16[off:off + 2 * r * c].view(h).view(r, c)
        # the binary16 operands as the call left them in its workspace (for inspection and tests)
        self.xh, self.xhT = (view(offs[0], M, K), None) if rm else (None, view(offs[0], K, M))
        self.wh, self.whT = view(offs[1], N, K), view(offs[2], K, N)
        self.dyh = dy if dy.dtype == h else view(offs[3], M, N)
        self.dyhT = None if rm else view(offs[4], N, M)

    def gemm_bwd_part(self, which: str, dy: Optional[torch.Tensor], stream=None) -> None:
        """One of the two independent backward GEMMs ("dx" or "dw", the latter with the bias gradient when the tag
        needs it from here), so that a caller can run them on different streams."""
        dx = self.dx if which == "dx" else None
        dw = self.dw if which == "dw" else None
        if self.bwd_tag != self.tag:
            self._fp16_backward(dy, dx, dw, self.db if dw is not None else None, stream)
            return
        want_db = dy is not None and self.tag != Q.INT8 and dw is not None
        if self.rowmajor_bwd:
            Q.qsync_qlinear_bwd_rm(self.tag, self.M, self.N, self.K, self.dyq, self.sdy, self.xq, self.sx, self.wqbT, self.swb,
                                   self.w_gran if self.w_gran == Q.PER_TENSOR else Q.PER_ROW, dx, dw,
                                   self.db if want_db else None, dy if want_db else None,
                                   self.acc_dx if dx is not None else None, self.acc_dw if dw is not None else None,
                                   self.ws_bwd, stream)
            return
        Q.qsync_qlinear_bwd(self.tag, self.M, self.N, self.K, self.dyq, self.dyqT, self.sdy, self.xqT, self.sx,
                            self.wqbT, self.swb, self.w_gran if self.w_gran == Q.PER_TENSOR else Q.PER_ROW,
                            dx, dw, self.db if want_db else None, dy if want_db else None,
                            self.acc_dx if dx is not None else None, self.acc_dw if dw is not None else None,
                            self.ws_bwd, stream)

    # ---- whole passes ----------------------------------------------------------------------
    def forward(self, x: torch.Tensor, w: torch.Tensor, stream=None, side_stream=None,
                x_amax: Optional[torch.Tensor] = None) -> torch.Tensor:
        """With `side_stream` (a torch stream of default priority) the small, latency-bound weight
        conversion kernels run beside the HBM-bound activation conversion and join before the GEMM."""
        if side_stream is None:
            self.convert_x(x, stream, x_amax)
            self.convert_w(w, stream)
        else:
            main = stream if stream is not None else torch.cuda.current_stream()
            side_stream.wait_stream(main)
            self.convert_w(w, side_stream)
            self.convert_x(x, main, x_amax)
            main.wait_stream(side_stream)
        self.gemm_fwd(stream)
        return self.y

    def backward(self, dy: torch.Tensor, stream=None):
        self.convert_dy(dy, stream)
        self.gemm_bwd(dy, stream)
        return self.dx, self.dw, self.db


class QConv3x3:
    """One 3x3 / stride 1 / pad 1 NHWC convolution as quantized operator (paper: Backend section, low-precision
    convolution on NHWC tensors).  Forward and data gradient run as implicit GEMMs over the codes (the patch
    matrix is never stored); the weight gradient contracts over the pixels and reads the transposed patch
    matrix, expanded from the int8 codes.  Buffers are allocated once; nothing here computes.

    INT8 and FP16: all three passes (the patch-matrix form of the weight gradient is INT8 only).
    The weight gradient reads both operands transposed over a zero-padded pixel axis (qsync_conv3x3_wgrad);
    wgrad_via_patches=True materialises the transposed patch matrix instead (qsync_im2col3x3_i8 + the linear
    operator's dW GEMM).
    """

    def __init__(self, tag: int, nimg: int, H: int, W: int, C: int, N: int, x_dtype=torch.float16, w_dtype=torch.float32,
                 dy_dtype=None, y_dtype=torch.float32, dx_dtype=torch.float16, dw_dtype=torch.float32,
                 w_gran: int = Q.PER_ROW, dy_round: int = Q.ROUND_STOCHASTIC, philox_seed: int = 0,
                 bias: bool = True, dump_acc: bool = False, bits: int = 8, device="cuda", wgrad_via_patches: bool = False,
                 collect_y_amax: bool = False):
        if tag not in (Q.INT8, Q.FP16):
            raise ValueError("QConv3x3: tag INT8 or FP16")
        # max |Y| collected by the forward GEMM's epilogue, for a convolution that quantizes Y as it is
        self.y_amax = torch.zeros(1, dtype=torch.float32, device=device) if collect_y_amax else None
        self.wgrad_via_patches = wgrad_via_patches
        self.tag, self.nimg, self.H, self.W, self.C, self.N = tag, nimg, H, W, C, N
        M, K = nimg * H * W, 9 * C
        self.M, self.K = M, K
        self.w_gran, self.dy_round, self.seed, self.bits, self.offset = w_gran, dy_round, philox_seed, bits, 0
        e = lambda *s, dt: torch.empty(*s, dtype=dt, device=device)
        qd, f32 = _TORCH_OF_TAG[tag], torch.float32
        self.xq = e(M, C, dt=qd)
        self.xqTp = e(K, M, dt=qd) if (tag == Q.INT8 and wgrad_via_patches) else None   # transposed patch matrix
        self.wq, self.wflip = e(N, K, dt=qd), e(C, 9 * N, dt=qd)
        self.dyq = e(M, N, dt=qd)
        self.dyqT = e(N, M, dt=qd) if wgrad_via_patches else None
        self.sx, self.ix, self.ax = e(1, dt=f32), e(1, dt=f32), e(1, dt=f32)
        nsw, nswb = (N, C) if w_gran == Q.PER_ROW else (1, 1)
        self.sw, self.iw, self.aw = e(nsw, dt=f32), e(nsw, dt=f32), e(nsw, dt=f32)
        self.swb, self.iwb = e(nswb, dt=f32), e(nswb, dt=f32)
        self.sdy, self.idy, self.ady = e(1, dt=f32), e(1, dt=f32), e(1, dt=f32)
        self.bias = torch.zeros(N, dtype=f32, device=device) if bias else None
        self.y, self.dx, self.dw = e(M, N, dt=y_dtype), e(M, C, dt=dx_dtype), e(N, K, dt=dw_dtype)
        self.db = e(N, dt=f32)
        self.acc = self.acc_dx = self.acc_dw = None
        if dump_acc and tag == Q.INT8:
            i32 = torch.int32
            self.acc, self.acc_dx, self.acc_dw = e(M, N, dt=i32), e(M, C, dt=i32), e(N, K, dt=i32)
        self.ws_absmax = _ws(max(Q.qsync_absmax_workspace_bytes(M, C, Q.PER_TENSOR),
                                 Q.qsync_absmax_workspace_bytes(M, N, Q.PER_TENSOR)), device)
        self.ws_absmax_w = _ws(max(Q.qsync_conv3x3_prepare_weights_workspace_bytes(N, C),
                                   Q.qsync_absmax_workspace_bytes(N, K, Q.PER_TENSOR)), device)
        if wgrad_via_patches and tag != Q.INT8:
            raise ValueError("QConv3x3: the patch-matrix weight gradient exists for INT8 only")
        self.ws_bwd = _ws(Q.qsync_qlinear_bwd_workspace_bytes(tag, M, N, K) if wgrad_via_patches
                          else Q.qsync_conv3x3_wgrad_workspace_bytes(tag, nimg, H, W, C, N), device)

    def convert_x(self, act: torch.Tensor, stream=None, x_amax: Optional[torch.Tensor] = None) -> None:
        """x_amax: device float holding max |act| already (the producer's `y_amax`); it replaces the pass over the
        activation that finds the maximum and is left at zero for the producer's next step."""
        M, C = self.M, self.C
        if self.tag == Q.INT8 and x_amax is not None:
            Q.qsync_scale_from_amax(x_amax, self.bits, self.sx, self.ix, True, stream)
            Q.qsync_quantize(act, M, C, C, Q.INT8, self.bits, Q.PER_TENSOR, Q.ROUND_NEAREST, 0, 0, self.ix, self.xq, None,
                             stream)
        elif self.tag == Q.INT8:
            Q.qsync_absmax_quantize(act, M, C, self.bits, Q.ROUND_NEAREST, 0, 0, self.sx, self.ix, self.ax, self.xq, None,
                                    self.ws_absmax, -1, stream)
        elif act.dtype == _TORCH_OF_TAG[self.tag] and act.is_contiguous():
            self.xq = act.view(M, C)           # already in the operand type: used in place
        else:
            Q.qsync_quantize(act, M, C, C, self.tag, 0, 0, 0, 0, 0, None, self.xq, None, stream)

    def convert_w(self, w: torch.Tensor, stream=None) -> None:
        N, K, C = self.N, self.K, self.C
        if self.tag != Q.INT8:
            Q.qsync_quantize(w, N, K, K, self.tag, 0, 0, 0, 0, 0, None, self.wq, None, stream)
            Q.qsync_conv3x3_wflip(self.wq, N, C, self.wflip, stream)
            return
        if self.w_gran == Q.PER_TENSOR:
            Q.qsync_absmax_scale(w, N, K, K, Q.PER_TENSOR, self.bits, self.sw, self.iw, self.aw, None, self.ws_absmax_w, stream)
            Q.qsync_quantize(w, N, K, K, Q.INT8, self.bits, Q.PER_TENSOR, Q.ROUND_NEAREST, 0, 0, self.iw, self.wq, None, stream)
            self.swb = self.sw
            Q.qsync_conv3x3_wflip(self.wq, N, C, self.wflip, stream)
            return
        # the output channel is the data gradient's contraction axis: second set of codes with one scale per
        # input channel c (per column of the weights viewed as [9*N, C]), mirrored and channel-exchanged
        Q.qsync_conv3x3_prepare_weights(w, N, C, self.bits, self.sw, self.iw, self.wq, self.swb, self.iwb, self.wflip,
                                        self.ws_absmax_w, stream)

    def conv_fwd(self, stream=None) -> None:
        if self.y_amax is not None:
            Q.qsync_conv3x3_fwd_amax(self.tag, self.nimg, self.H, self.W, self.C, self.N, self.xq, self.sx, self.wq, self.sw,
                                     self.w_gran, self.bias, self.y, self.acc, self.y_amax, stream)
            return
        Q.qsync_conv3x3_fwd(self.tag, self.nimg, self.H, self.W, self.C, self.N, self.xq, self.sx, self.wq, self.sw,
                            self.w_gran, self.bias, self.y, self.acc, stream)

    def convert_dy(self, dy: torch.Tensor, stream=None) -> None:
        M, N = self.M, self.N
        if self.tag == Q.INT8:
            Q.qsync_absmax_scale(dy, M, N, N, Q.PER_TENSOR, self.bits, self.sdy, self.idy, self.ady, self.db, self.ws_absmax, stream)
            Q.qsync_quantize(dy, M, N, N, Q.INT8, self.bits, Q.PER_TENSOR, self.dy_round, self.seed, self.offset,
                             self.idy, self.dyq, self.dyqT, stream)
            self.offset += (M * N + 7) // 8
        elif dy.dtype == _TORCH_OF_TAG[self.tag] and dy.is_contiguous():
            self.dyq = dy
        else:
            Q.qsync_quantize(dy, M, N, N, self.tag, 0, 0, 0, 0, 0, None, self.dyq, None, stream)

    def conv_dgrad(self, stream=None) -> None:
        # dX = conv3x3(dY, mirrored weights with the channel roles exchanged)
        Q.qsync_conv3x3_fwd(self.tag, self.nimg, self.H, self.W, self.N, self.C, self.dyq, self.sdy, self.wflip, self.swb,
                            self.w_gran, None, self.dx, self.acc_dx, stream)

    def conv_wgrad(self, stream=None) -> None:
        if not self.wgrad_via_patches:
            Q.qsync_conv3x3_wgrad(self.tag, self.nimg, self.H, self.W, self.C, self.N, self.xq, self.sx, self.dyq, self.sdy, self.dw,
                                  self.acc_dw, self.ws_bwd, stream)
            return
        Q.qsync_im2col3x3_i8(self.xq, self.nimg, self.H, self.W, self.C, None, self.xqTp, stream)
        Q.qsync_qlinear_bwd(Q.INT8, self.M, self.N, self.K, None, self.dyqT, self.sdy, self.xqTp, self.sx, None, None,
                            Q.PER_TENSOR, None, self.dw, None, None, None, self.acc_dw, self.ws_bwd, stream)

    def forward(self, act: torch.Tensor, w: torch.Tensor, stream=None, x_amax: Optional[torch.Tensor] = None) -> torch.Tensor:
        self.convert_w(w, stream)
        self.convert_x(act, stream, x_amax)
        self.conv_fwd(stream)
        return self.y

    def backward(self, dy: torch.Tensor, stream=None):
        self.convert_dy(dy, stream)
        self.conv_dgrad(stream)
        self.conv_wgrad(stream)
        return self.dx, self.dw, (self.db if self.tag == Q.INT8 else None)     # db comes out of the INT8 absmax pass
