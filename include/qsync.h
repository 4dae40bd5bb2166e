/*
 * qsync.h - C ABI of the MI355X (gfx950) quantized training operators.
 *
 * The library implements the low-precision operator backend of QSync (arXiv 2407.02327,
 * section "Backend Optimization and Implementation"): for a linear operator Y = X W^T + b
 * with a per-operator precision tag b in {INT8, FP16, FP32} (problem (1) of the paper),
 * it finds the absolute maximum of a tensor, derives a symmetric fixed-point scale,
 * quantizes to INT8 codes (or casts to FP16), runs the forward GEMM and the two backward
 * GEMMs dX = dY W and dW = dY^T X with int32 / fp32 accumulation, and dequantizes with the
 * scales and the bias fused into the GEMM epilogue.
 *
 * Conventions that hold for every entry point
 *  - All data pointers are DEVICE pointers (HIP global memory) unless a parameter says
 *    "host".  The library never allocates, frees or keeps device memory: every buffer,
 *    including scratch ("workspace"), is owned by the caller.
 *  - Matrices are row-major.  Inputs that take a leading dimension `ld` count it in
 *    elements; every other matrix is packed (leading dimension = number of columns).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    enqueue work; they never synchronise and never copy to the host.  Scales stay on the
 *    device.
 *  - Return value: QSYNC_OK (0) or a negative qsync_status_t.  Arguments are validated
 *    before any HIP call; nothing is launched when validation fails.  The library never
 *    throws, aborts or prints.  After QSYNC_ERR_HIP, qsync_last_hip_error() returns the
 *    hipError_t of the failing call on this thread.
 *  - A tensor with rows*cols == 0 (or a GEMM with M*N == 0) is a successful no-op.
 *    A GEMM with K == 0 writes the bias (or zeros).
 *  - Inputs must be finite; behaviour on NaN/Inf is unspecified.
 *  - Calls on different streams may run concurrently as long as their buffers are disjoint.
 */
#ifndef QSYNC_H
#define QSYNC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Per-operator precision tag b_io (paper: problem (1); evaluation uses INT8, FP16, FP32). */
typedef enum { QSYNC_INT8 = 8, QSYNC_FP16 = 16, QSYNC_FP32 = 32 } qsync_prec_t;

/* Element type of a buffer. */
typedef enum { QSYNC_F32 = 0, QSYNC_F16 = 1, QSYNC_I8 = 2, QSYNC_I32 = 3 } qsync_dtype_t;

/* Granularity of a scale: one per tensor ("layer-wise"), one per row, or one per column
 * ("channel-wise"; paper, Cost Mapper paragraph on quantization methods). */
typedef enum { QSYNC_PER_TENSOR = 0, QSYNC_PER_ROW = 1, QSYNC_PER_COL = 2 } qsync_gran_t;

/* Rounding of the fixed-point quantizer: ties-to-even, stochastic (the unbiased quantizer
 * of the Indicator section), or floor (Discussion, "Quantization by Floor"). */
typedef enum { QSYNC_ROUND_NEAREST = 0, QSYNC_ROUND_STOCHASTIC = 1, QSYNC_ROUND_FLOOR = 2 } qsync_round_t;

typedef enum {
    QSYNC_OK              = 0,
    QSYNC_ERR_NULL        = -1, /* a required pointer is NULL */
    QSYNC_ERR_BAD_ENUM    = -2, /* an enum argument holds no enumerator */
    QSYNC_ERR_BAD_SHAPE   = -3, /* negative dimension, ld < cols, or element count overflow */
    QSYNC_ERR_UNSUPPORTED = -4, /* valid but not implemented combination (bits, tag/dtype) */
    QSYNC_ERR_ALIGN       = -5, /* pointer or dimension violates a kernel's alignment rule */
    QSYNC_ERR_WORKSPACE   = -6, /* workspace NULL or smaller than the matching *_workspace_bytes */
    QSYNC_ERR_HIP         = -7  /* a HIP runtime call failed */
} qsync_status_t;

/*
 * qsync_absmax_scale - absolute maximum and symmetric fixed-point scale.
 * Paper: Backend section, "Minmax Optimization" (two-step reduction: block partials, then a
 * small second step; here the last block to finish performs that step inside the same launch);
 * scale of the fixed-point quantizer x_bar = (x - z)/q with z = 0.
 *
 *   amax  = max |x| over the tensor (PER_TENSOR), each row (PER_ROW) or each column (PER_COL)
 *   scale = amax / qmax,  inv_scale = qmax / amax,   qmax = 2^(bits-1) - 1   (one fp32 division each)
 *   amax == 0  ->  scale = inv_scale = 1
 *
 * x         [rows, ld] of xdt (QSYNC_F32 or QSYNC_F16), ld >= cols.
 * scale, inv_scale   out, 1 / rows / cols floats according to gran.  Both required.
 * amax_opt  out, same shape, may be NULL.
 * colsum_opt out, cols floats or NULL; PER_TENSOR only and cols <= 2^19 (QSYNC_ERR_UNSUPPORTED otherwise).  When
 *           given, the same pass over x also produces colsum[c] = sum_r x[r,c] in fp32: for x = dY
 *           this is the bias gradient db (paper: Appendix, proof of Prop. 1, gradient of a linear
 *           operator), obtained without reading dY a third time.
 * sumsq_opt out, one float or NULL; PER_TENSOR only.  When given, the same pass also yields the squared
 *           Euclidean norm sum x[r,c]^2 (fp32 per lane and block, block results folded in double in block
 *           order): with amax it is what the variance indicator needs from a tensor (paper: Indicator
 *           section, Prop. 3: norms, scaling factors and effective bits "collected through profiling").
 * workspace scratch of at least qsync_absmax_workspace_bytes(rows, cols, gran) bytes, 16-byte aligned.
 *           PER_TENSOR: its first 256 bytes hold a block arrival counter: ZERO THEM ONCE after
 *           allocating the buffer (hipMemset); every call that completes leaves them zero again, so
 *           the buffer can be reused by later calls without clearing.  The rest needs no
 *           initialisation.  Two calls that may run concurrently (different streams) need separate
 *           workspaces.  A counter that is not zero yields an undefined scale (no fault).
 * bits      2..8.
 * Any alignment of x and ld is accepted (vector loads are used when x and ld*sizeof(elem)
 * are multiples of 16 bytes).
 */
int qsync_absmax_scale(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld,
                       int gran, int bits, float* scale, float* inv_scale, float* amax_opt,
                       float* colsum_opt, float* sumsq_opt, void* workspace, size_t workspace_bytes,
                       void* stream);
size_t qsync_absmax_workspace_bytes(int64_t rows, int64_t cols, int gran);

/*
 * qsync_absmax_scale_static - qsync_absmax_scale for callers that cannot allocate device memory and have no
 * workspace to pass: code under HIP graph capture, tight serving loops, harnesses that forbid allocation.
 * Per-tensor granularity only; same results as qsync_absmax_scale(..., QSYNC_PER_TENSOR, ...), bit for bit.
 * The scratch (arrival counter, block partials, column-sum partials) is a device array inside the library,
 * about 8.4 MB per GPU, held until the process ends; its device address is looked up on the first call on each
 * device.  The call allocates and frees nothing and clears its counter with a kernel (no memset node).
 * Limit: with colsum_opt, cols <= 4096 (QSYNC_ERR_WORKSPACE beyond: the partials would not fit); without it any
 * size.  All calls on one GPU share that GPU's scratch: calls that may overlap (different streams, or
 * different threads) race and give undefined results; serialise them or use qsync_absmax_scale with separate
 * workspaces.  Other arguments and errors as for qsync_absmax_scale.
 */
int qsync_absmax_scale_static(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int bits,
                              float* scale, float* inv_scale, float* amax_opt, float* colsum_opt,
                              float* sumsq_opt, void* stream);

/*
 * qsync_quantize - precision conversion of one tensor under a precision tag.
 * Paper: Indicator section (x_bar = (x - z)/q, x_hat = round(x_bar) q + z, stochastic
 * rounding as the unbiased quantizer), Cost Mapper (casting kernels), Backend section.
 *
 *   tag INT8: code = clamp(round(x * inv_scale), -qmax, qmax) as int8; the product is one
 *             fp32 multiply.  Stochastic rounding: with f = x*inv - floor(x*inv), round up
 *             iff u < floor(f * 2^16), where u is the 16-bit draw of the element:
 *             Philox4x32-10, key = (seed low word, seed high word), counter = the 128-bit
 *             integer offset + i/8 (i = row*cols + col, independent of ld), output words
 *             cut into eight 16-bit draws, element takes draw i%8 (word (i%8)/2, low half
 *             first).  A call consumes ceil(rows*cols/8) counters.
 *   tag FP16: IEEE round-to-nearest-even narrowing to binary16 (copy if x is binary16).
 *             With rnd = QSYNC_ROUND_STOCHASTIC and fp32 input: the floating-point stochastic
 *             quantizer of the paper (Appendix, Proposition 2): the mantissa is truncated to k bits
 *             (k = bits, 7..10; bits = 0 means 9, the value the paper states for float16; 10 keeps the full
 *             binary16 mantissa) and
 *             the value moves up by one spacing 2^(max(e,-14)-k) with probability dropped/spacing,
 *             decided as u < floor(p * 2^16) with the same per-element Philox draw u as tag INT8.
 *             Values that reach 2^16 become infinity, as in IEEE narrowing.
 *   tag FP32: copy as fp32 (widening from binary16 is exact).
 *
 * x         [rows, ld] of xdt (QSYNC_F32 or QSYNC_F16).
 * inv_scale from qsync_absmax_scale with the same gran (1 / rows / cols floats); ignored
 *           (may be NULL) for FP16 and FP32.
 * q_opt     out, packed [rows, cols] of int8 / binary16 / fp32 according to tag, or NULL.
 * qT_opt    out, packed [cols, rows], the transpose of q (identical codes), or NULL.
 *           At least one of q_opt, qT_opt is required.  The GEMM entry points take some
 *           operands in transposed form; this is where those copies are made.
 * bits, gran, rnd, seed, offset are ignored for FP16 / FP32 (except the stochastic FP16 case above).
 * Any shape and alignment is accepted; the vectorised path needs cols % 8 == 0, x and ld*sizeof(elem)
 * multiples of 16 bytes, q 16-byte aligned (and rows % 16 == 0 for qT).
 */
int qsync_quantize(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld,
                   int tag, int bits, int gran, int rnd,
                   uint64_t philox_seed, uint64_t philox_offset, const float* inv_scale,
                   void* q_opt, void* qT_opt, void* stream);

/*
 * qsync_absmax_quantize - qsync_absmax_scale (PER_TENSOR) followed by qsync_quantize (tag INT8, PER_TENSOR) on a
 * packed tensor (ld == cols), with identical results, in one launch where that pays: for a small tensor (up to
 * 4M elements, 1M with stochastic rounding) that meets the vector path's rules (cols % 8 == 0, 16-byte aligned x
 * and outputs, rows % 16 == 0 with a transposed copy) every workgroup finds the maximum of its share, they meet
 * once, and each quantizes the part it has just read; other tensors take the two launches.  Paper: Backend section, "Minimum and Maximum
 * Optimization" (the collection of the maximum is the casting cost the paper trims); Cost Mapper, cvt_cost.
 *
 * scale, inv_scale, amax_opt, q_opt, qT_opt, bits, rnd, philox_seed, philox_offset: as in the two calls.
 * workspace   at least qsync_absmax_quantize_workspace_bytes(rows, cols) bytes, 16-byte aligned; its first 4 bytes
 *             must be zero before the first use and are zero again after every call (the same rule, and the same
 *             buffer if wanted, as qsync_absmax_scale).  Calls that overlap in time need separate workspaces.
 * poll_limit  how many times a workgroup polls for the others before it finds the maximum by reading the whole
 *             tensor itself (same result; this bounds every wait, so the call cannot hang when its workgroups
 *             are not all resident at once, e.g. beside another stream's kernel).  < 0: library default.
 */
int qsync_absmax_quantize(const void* x, int xdt, int64_t rows, int64_t cols, int bits, int rnd,
                          uint64_t philox_seed, uint64_t philox_offset,
                          float* scale, float* inv_scale, float* amax_opt, void* q_opt, void* qT_opt,
                          void* workspace, size_t workspace_bytes, int poll_limit, void* stream);
size_t qsync_absmax_quantize_workspace_bytes(int64_t rows, int64_t cols);

/*
 * qsync_qlinear_fwd - forward GEMM with the dequantizer and bias fused into the epilogue.
 * Paper: proof of Prop. 2 (y = q_v q_w sum(v_q w_q) + b), Backend section "Dequantization
 * Fusion" (int32 accumulation, INT32 -> FP32 conversion with the scale in the epilogue),
 * Cost Mapper (layer-wise input with channel-wise weight -> channel-wise dequantizer).
 *
 *   INT8: acc[m,n] = sum_k xq[m,k] wq[n,k]  (int32, wraps mod 2^32)
 *         Y[m,n]   = float(acc) * (sx * sw[n or 0]) + bias[n]
 *   FP16: Y = X W^T + bias with binary16 operands, fp32 accumulation.
 *   FP32: Y = X W^T + bias in fp32.
 *
 * xq  [M,K], wq [N,K] packed, element type int8 / binary16 / fp32 by tag, 16-byte aligned.
 * sx  1 float (per-tensor activation scale); sw 1 float (wgran PER_TENSOR) or N floats
 *     (PER_ROW of wq, i.e. per output channel).  Both ignored (may be NULL) unless tag is INT8.
 * bias_opt  N floats or NULL.
 * y   out, packed [M,N] of ydt (QSYNC_F32 or QSYNC_F16).
 * acc_dump_opt  INT8 only: if non-NULL, also receives the raw int32 accumulators [M,N]
 *     (verification aid; NULL in production).
 * workspace     at least qsync_qlinear_workspace_bytes(tag, M, N, K) bytes, 16-byte aligned
 *     (may be NULL if that is 0).
 * INT8 needs K % 16 == 0 and FP16 needs K % 8 == 0 (rows of 16-byte vectors feed the matrix
 * cores); otherwise QSYNC_ERR_ALIGN.  M and N are arbitrary.  A row of K elements may take at most
 * 16 MiB (QSYNC_ERR_UNSUPPORTED beyond; the same bound holds for N in the dX GEMM and M in the dW GEMM
 * of qsync_qlinear_bwd).
 */
int qsync_qlinear_fwd(int tag, int64_t M, int64_t N, int64_t K,
                      const void* xq, const float* sx,
                      const void* wq, const float* sw, int wgran,
                      const float* bias_opt, void* y, int ydt, int32_t* acc_dump_opt,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * qsync_qlinear_fwd_amax - qsync_qlinear_fwd that also collects max |Y| in its epilogue, so that an
 * operator fed directly by Y can skip its own minimum/maximum pass.  Paper: the Backend section counts the
 * collection of the minimum/maximum as part of the casting cost ("Minimum and Maximum Optimization");
 * the Cost Mapper's cvt_cost of the consumer shrinks by that pass.
 *
 * y_amax  device float, read and written: on return of the kernel it holds max(previous value, max |Y|),
 *         where Y is taken as stored (after rounding to ydt).  Set it to 0 before the first collection
 *         (qsync_scale_from_amax with consume != 0 leaves it at 0).  4-byte aligned.  NaN outputs are not
 *         ordered; finite outputs are assumed.
 * The maximum is taken where the output is written: in the GEMM's epilogue, or in the reduction pass when K is split.
 * All other arguments and errors as qsync_qlinear_fwd (same workspace).
 */
int qsync_qlinear_fwd_amax(int tag, int64_t M, int64_t N, int64_t K,
                           const void* xq, const float* sx,
                           const void* wq, const float* sw, int wgran,
                           const float* bias_opt, void* y, int ydt, int32_t* acc_dump_opt,
                           float* y_amax, void* workspace, size_t workspace_bytes, void* stream);

/*
 * qsync_qlinear_fwd_codes - qsync_qlinear_fwd whose epilogue also writes the fixed-point codes of Y for the
 * operator that consumes Y, so that the consumer's quantization pass (read Y, write codes) disappears.
 * Paper: Cost Mapper paragraph (cvt_cost, the casting of an operator's input, is "non-negligible for all
 * cases"; the output scaling factor is part of runtime fixed-point quantization); Backend section (work fused
 * into the epilogue before the result leaves the kernel).
 *
 *   yq[m,n] = clamp(round(Y[m,n] * next_inv_scale[0]), -qmax, qmax),  qmax = 2^(bits-1) - 1
 *   with Y as stored (after rounding to ydt), one fp32 multiply, ties to even: the same bits as
 *   qsync_quantize(Y, ..., QSYNC_INT8, bits, QSYNC_PER_TENSOR, QSYNC_ROUND_NEAREST, ..., next_inv_scale, yq).
 *
 * A per-tensor scale needs the maximum of the whole of Y, which is not known while Y is being produced: the
 * caller supplies the inverse scale (for instance from the maximum this call collected on the previous
 * step) and may collect max |Y| of this step in y_amax_opt (semantics of qsync_qlinear_fwd_amax) to check
 * that nothing was clamped (max |Y| * inv_scale <= qmax + 0.5) and to derive the next scale.
 * next_inv_scale  device float.   yq  out [M,N] int8, packed.   bits 2..8.
 * The consumer's transposed copy (needed for its weight gradient only) is qsync_transpose_i8 of yq.
 * No accumulator dump; tag FP32 needs 16-byte aligned operands with K % 4 == 0 (QSYNC_ERR_UNSUPPORTED
 * otherwise).  All other arguments, the workspace and errors as qsync_qlinear_fwd.
 */
int qsync_qlinear_fwd_codes(int tag, int64_t M, int64_t N, int64_t K,
                            const void* xq, const float* sx,
                            const void* wq, const float* sw, int wgran,
                            const float* bias_opt, void* y, int ydt, int bits, const float* next_inv_scale,
                            void* yq, float* y_amax_opt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * qsync_transpose_i8 - out[c, r] = in[r, c] for int8 codes (the K-contiguous operand layout of the backward
 * GEMMs from row-major codes, see qsync_qlinear_bwd).  in [rows, cols], out [cols, rows], both packed, distinct.
 */
int qsync_transpose_i8(const void* in, int64_t rows, int64_t cols, void* out, void* stream);

/*
 * qsync_scale_from_amax - scale = amax / qmax, inv_scale = qmax / amax (1 and 1 for amax == 0) from a
 * maximum already on the device, with the arithmetic of qsync_absmax_scale (PER_TENSOR); qmax = 2^(bits-1) - 1.
 * amax       device float (read; set to 0 afterwards if consume != 0).
 * scale, inv_scale  device floats, out.
 * bits       2..8, otherwise QSYNC_ERR_UNSUPPORTED.
 */
int qsync_scale_from_amax(float* amax, int bits, float* scale, float* inv_scale, int consume, void* stream);

/*
 * qsync_qlinear_bwd - both backward GEMMs of a linear operator, plus the bias gradient.
 * Paper: Appendix proof of Prop. 1 ((dW, dX) = G[dY, C(v, x)]); Backend section (dW is
 * produced in FP32, dX in FP16, dequantization fused in the epilogue).
 *
 *   dX[m,k] = sum_n dY[m,n] W[n,k]      dW[n,k] = sum_m dY[m,n] X[m,k]      db[n] = sum_m dY[m,n]
 *   INT8: dX = float(accX) * (sdy * swb[k or 0]),  dW = float(accW) * (sdy * sx), int32 accumulators.
 *
 * Every operand is handed over with its contraction axis contiguous:
 *   dyq   [M,N]  and  dyqT [N,M]   the quantized / cast gradient and its transpose
 *   xqT   [K,M]                    transpose of the forward's activation operand
 *   wqbT  [K,N]                    transpose of the weight operand.  For INT8 its scale swb is
 *                                  1 float (wbgran PER_TENSOR) or K floats (PER_ROW of wqbT, one
 *                                  per input feature k): a scale along n would lie on the
 *                                  contraction axis of dX and could not leave the integer sum.
 * sdy, sx  1 float each (INT8 only).
 * dx_opt  out [M,K] of dxdt; dw_opt out [N,K] of dwdt (QSYNC_F32 or QSYNC_F16); either may be
 *         NULL to skip that GEMM (then its operands may be NULL too).
 * db_opt  out N floats or NULL; needs dy_float_opt, the unquantized gradient [M,N] of dydt
 *         (QSYNC_F32 or QSYNC_F16, packed), summed in fp32.
 * acc_dx_dump_opt [M,K], acc_dw_dump_opt [N,K]: raw int32 accumulators (INT8 only), or NULL.
 * workspace  at least qsync_qlinear_bwd_workspace_bytes(tag, M, N, K) bytes.
 * Alignment: INT8 needs N % 16 == 0 (for dX) and M % 16 == 0 (for dW); FP16 needs % 8.
 */
int qsync_qlinear_bwd(int tag, int64_t M, int64_t N, int64_t K,
                      const void* dyq, const void* dyqT, const float* sdy,
                      const void* xqT, const float* sx,
                      const void* wqbT, const float* swb, int wbgran,
                      void* dx_opt, int dxdt, void* dw_opt, int dwdt,
                      float* db_opt, const void* dy_float_opt, int dydt,
                      int32_t* acc_dx_dump_opt, int32_t* acc_dw_dump_opt,
                      void* workspace, size_t workspace_bytes, void* stream);

size_t qsync_qlinear_workspace_bytes(int tag, int64_t M, int64_t N, int64_t K);
size_t qsync_qlinear_bwd_workspace_bytes(int tag, int64_t M, int64_t N, int64_t K);

/*
 * qsync_qlinear_bwd_rm - qsync_qlinear_bwd for INT8 or FP16 operands without transposed copies of the activation
 * and gradient operands: the weight gradient dW = dY^T X contracts over the rows of both operands, and its GEMM
 * reads the row-major dyq [M,N] and xq [M,K] directly (transposing LDS reads feed the matrix instructions), so
 * qsync_quantize has to write one copy of X and of dY only -- none at all for a binary16 tensor under the FP16 tag,
 * which is its own operand.  Paper: Cost Mapper paragraph (cvt_cost and bp_cost,
 * the casting costs of the forward and backward pass); Appendix, proof of Prop. 1 (the two gradient contractions).
 *
 *   dX[m,k] = sum_n dyq[m,n] wqbT[k,n] * (sdy swb[k or 0])      dW[n,k] = sum_m dyq[m,n] xq[m,k] * (sdy sx)
 *   db[n] = sum_m dY[m,n]                                          same bits as qsync_qlinear_bwd
 *
 * tag  QSYNC_INT8 or QSYNC_FP16 (QSYNC_ERR_UNSUPPORTED otherwise).
 * dyq [M,N], xq [M,K] int8 / binary16 row-major (the forward's own operand), wqbT [K,N]; scales as in
 * qsync_qlinear_bwd (INT8 only; ignored for FP16, whose sums carry no scale).
 * The weight gradient needs M % 128 == 0, N and K multiples of 16 (INT8) or 8 (FP16) and N, K < 2^24
 * (QSYNC_ERR_ALIGN / QSYNC_ERR_UNSUPPORTED otherwise: use qsync_qlinear_bwd with transposed copies then).
 * workspace  at least qsync_qlinear_bwd_rm_workspace_bytes(tag, M, N, K) bytes.
 */
int qsync_qlinear_bwd_rm(int tag, int64_t M, int64_t N, int64_t K, const void* dyq, const float* sdy,
                         const void* xq, const float* sx, const void* wqbT, const float* swb, int wbgran,
                         void* dx_opt, int dxdt, void* dw_opt, int dwdt, float* db_opt,
                         const void* dy_float_opt, int dydt, int32_t* acc_dx_dump_opt, int32_t* acc_dw_dump_opt,
                         void* workspace, size_t workspace_bytes, void* stream);
size_t qsync_qlinear_bwd_rm_workspace_bytes(int tag, int64_t M, int64_t N, int64_t K);

/*
 * qsync_qlinear_bwd_fp16_of_int8 - backward of an INT8 operator the way the paper runs it: in FP16, on the
 * dequantized codes the forward saved.  Paper: footnote of the Cost Mapper paragraph (integer backward is
 * inefficient, the backward of fixed-point kernels is executed in FP16 and incurs additional casting);
 * Indicator section (x_hat = code * q); Backend section (dW in FP32, dX in FP16).
 *
 *   x_hat^T = binary16(xqT * sx)            w_hat = binary16(wq * sw[n or 0])      dY16 = binary16(dY)
 *   dX = dY16 w_hat      dW = dY16^T x_hat      db = sum_m dY         (fp32 accumulation)
 *   Each binary16 operand is the exact product (or value) rounded once to nearest even.
 *
 * One call runs the dequantizers, the casts / transposes and both FP16 GEMMs (the per-operator tag of the
 * backward is thereby a parameter of the C boundary, not of the caller's sequencing).
 * dy    [M,N] of dydt (QSYNC_F32 or QSYNC_F16), 16-byte aligned; a binary16 gradient is used in place.
 * xq_or_xqT, x_rowmajor   the activation codes the forward kept; sx 1 float.
 *        x_rowmajor 0: xqT [K,M], the transposed codes; x_hat^T and dY16^T are formed and the weight gradient is
 *        the NT GEMM of qsync_qlinear_bwd.
 *        x_rowmajor 1: xq [M,K], the forward's own operand; x_hat [M,K] is formed, no transpose of dY is written
 *        and the weight gradient reads the row-major operands (qsync_qlinear_bwd_rm): needs M % 128 == 0 and
 *        N, K multiples of 8 (QSYNC_ERR_ALIGN otherwise).  Same dW up to the order of the fp32 sums.
 * wq    [N,K] int8: the forward's weight codes; sw 1 float (wgran PER_TENSOR) or N floats (PER_ROW).
 * dx_opt [M,K] of dxdt, dw_opt [N,K] of dwdt, db_opt N floats; each may be NULL (its inputs may then be NULL).
 * workspace  at least qsync_qlinear_bwd_fp16_of_int8_workspace_bytes(M, N, K, dydt) bytes, 256-byte aligned
 *        (QSYNC_ERR_WORKSPACE / QSYNC_ERR_ALIGN otherwise); it receives the binary16 operands.
 * operand_offsets_opt  HOST array of 5 or NULL: byte offsets in the workspace of x_hat^T [K,M] (x_hat [M,K] when
 *        x_rowmajor), w_hat [N,K], w_hat^T [K,N], dY16 [M,N] (unused when dy is binary16) and dY16^T [N,M] (unused
 *        when x_rowmajor) (verification aid).
 * FP16 alignment rules as for qsync_qlinear_bwd: N % 8 == 0 for dX, M % 8 == 0 for dW.
 */
int qsync_qlinear_bwd_fp16_of_int8(int64_t M, int64_t N, int64_t K, const void* dy, int dydt,
                                   const void* xq_or_xqT, int x_rowmajor, const float* sx,
                                   const void* wq, const float* sw, int wgran,
                                   void* dx_opt, int dxdt, void* dw_opt, int dwdt, float* db_opt,
                                   void* workspace, size_t workspace_bytes, size_t* operand_offsets_opt, void* stream);
size_t qsync_qlinear_bwd_fp16_of_int8_workspace_bytes(int64_t M, int64_t N, int64_t K, int dydt);

/*
 * qsync_prepare_weights - every weight operand of one INT8 linear operator with per-output-channel
 * scales, from one call (paper: Cost Mapper paragraph, casting cost of the weights in the forward pass;
 * channel-wise weight quantization).  Equivalent to, and bit-identical with, the sequence
 *   qsync_absmax_scale(w, PER_ROW) -> sw, iw;   qsync_quantize(w, PER_ROW, nearest) -> wq [N,K]
 *   qsync_absmax_scale(w, PER_COL) -> swb, iwb; qsync_quantize(w, PER_COL, nearest) -> wqbT [K,N] (transposed only)
 * but reads w twice instead of four times (row and column maxima come from one pass, both sets of codes
 * from another).  wqbT / swb are the operand and scales qsync_qlinear_bwd takes for dX.
 *
 * w        [N,K] packed, wdt QSYNC_F32 or QSYNC_F16, device.
 * sw, iw   out, N floats each (scale, inverse scale per output channel); aw_opt out, N raw maxima or NULL.
 * swb, iwb out, K floats each (per input feature).
 * wq       out, [N,K] int8;  wqbT out, [K,N] int8.
 * workspace  at least qsync_absmax_workspace_bytes(N, K, QSYNC_PER_COL) bytes, 16-byte aligned.
 */
int qsync_prepare_weights(const void* w, int wdt, int64_t N, int64_t K, int bits,
                          float* sw, float* iw, float* aw_opt, void* wq,
                          float* swb, float* iwb, void* wqbT,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * qsync_conv3x3_wgrad - weight gradient of the 3x3 / stride 1 / pad 1 convolution on int8 codes or binary16
 * (paper: Appendix, proof of Prop. 1, backward of an operator from the saved, compressed context):
 *   dw[n, (kh*3+kw)*C + c] = sdy * sx * sum_{b,h,w} dyq[b,h,w,n] * xq[b, h+kh-1, w+kw-1, c]   (0 outside the image)
 * (tag FP16: the same sum over binary16 operands with fp32 accumulation, no scales).
 * The contraction runs over the pixels.  When nimg*H*W is a multiple of 128 (and nimg*H*W*C*element size < 2^31)
 * the GEMM reads both operands as they are: the row-major gradient, and the patch matrix [pixels, 9*C] formed by
 * its own loads from the NHWC activation (padding taps read a zero block); transposing LDS reads feed the matrix
 * instructions, no copy of either operand is made, and the workspace holds split-K partials only.
 * Otherwise both operands are written to the workspace transposed over a zero-padded pixel axis (a zero row in
 * front of every image, rows padded with zeros to a multiple of 16 pixels) on which every window offset is a plain
 * displacement: the gradient once, the activation three times (displaced by -1, 0, +1 pixel, so that every tap
 * reads 16-byte aligned rows), about 3.5 elements per activation element instead of the 9 of a materialised patch
 * matrix, and the GEMM reads the nine taps as displaced rows of those copies.  Same int32 accumulators either way.
 *
 * tag  QSYNC_INT8 or QSYNC_FP16 (QSYNC_FP32: QSYNC_ERR_UNSUPPORTED).
 * xq   [nimg, H, W, C] and dyq [nimg*H*W, N], int8 or binary16, device, 16-byte aligned; C and N times the
 *      element size must be multiples of 16 bytes (QSYNC_ERR_ALIGN); (W + 16) * element size <= 1024
 *      (QSYNC_ERR_BAD_SHAPE).  sx, sdy: one float each (device; INT8 only).
 * dw   out, [N, 9*C] of dwdt (QSYNC_F32 or QSYNC_F16); acc_dump_opt: raw int32 accumulators [N, 9*C] or NULL
 *      (INT8 only).
 * workspace  at least qsync_conv3x3_wgrad_workspace_bytes(...) bytes, 256-byte aligned; no part of it needs
 *            to be initialised.
 */
int qsync_conv3x3_wgrad(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N,
                        const void* xq, const float* sx, const void* dyq, const float* sdy,
                        void* dw, int dwdt, int32_t* acc_dump_opt,
                        void* workspace, size_t workspace_bytes, void* stream);
size_t qsync_conv3x3_wgrad_workspace_bytes(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N);

/*
 * qsync_conv3x3_prepare_weights - every weight operand of one INT8 3x3 convolution with per-output-channel
 * scales (paper: channel-wise weight quantization; casting cost of the weights in the forward pass).
 * Bit-identical with the sequence
 *   qsync_absmax_scale(w [N,9C], PER_ROW) -> sw, iw;          qsync_quantize(PER_ROW, nearest) -> wq [N,9C]
 *   qsync_absmax_scale(w as [9N,C], PER_COL) -> swb, iwb;     qsync_quantize(PER_COL, nearest) -> codes [N,9C]
 *   qsync_conv3x3_wflip(codes) -> wflip [C,9N]
 * wflip with swb (QSYNC_PER_ROW of wflip) is the weight operand of the data gradient, see qsync_conv3x3_fwd.
 * Three launches and two reads of w when N % 16 == 0 (row and column maxima in one pass, both sets of codes
 * from one read, written straight to their final places), the five separate passes otherwise.
 * w [N, 9*C] packed (k = (kh, kw, c)), wdt QSYNC_F32 or QSYNC_F16; sw, iw: N floats; swb, iwb: C floats.
 * workspace  at least qsync_conv3x3_prepare_weights_workspace_bytes(N, C) bytes, 16-byte aligned, its first
 *            256 bytes zeroed once by the caller (as for qsync_absmax_scale).
 */
int qsync_conv3x3_prepare_weights(const void* w, int wdt, int64_t N, int64_t C, int bits,
                                  float* sw, float* iw, void* wq, float* swb, float* iwb, void* wflip,
                                  void* workspace, size_t workspace_bytes, void* stream);
size_t qsync_conv3x3_prepare_weights_workspace_bytes(int64_t N, int64_t C);

/*
 * qsync_conv3x3_fwd - 3x3 / stride 1 / pad 1 convolution over an NHWC tensor as an implicit GEMM.
 * Paper: Backend section (low-precision convolution kernels run on NHWC tensors; dequantization is
 * fused into the kernel's epilogue); Appendix, proof of Prop. 2 (forward flow of a fixed-point
 * kernel).  The patch matrix is never stored: the GEMM's loads gather it from the NHWC codes.
 *
 *   y[m, n] = sx * sw[n] * sum_{kh,kw,c} xq[b, h+kh-1, w+kw-1, c] * wq[n, (kh*3+kw)*C + c] + bias[n]
 *   m = (b*H + h)*W + w; terms outside the image are zero.  FP16: the same sum over binary16 operands
 *   with fp32 accumulation, no scales.
 *
 * tag     QSYNC_INT8 or QSYNC_FP16 (QSYNC_FP32: QSYNC_ERR_UNSUPPORTED).
 * xq      [nimg, H, W, C] codes (int8) or binary16, device, 16-byte aligned; C * element size must be a
 *         multiple of 16 bytes (QSYNC_ERR_ALIGN) and nimg*H*W*C*element size < 2^31 (QSYNC_ERR_BAD_SHAPE).
 * wq      [N, 9*C], k = (kh, kw, c), same element type, 16-byte aligned.
 * sx, sw, wgran, bias_opt, y [nimg*H*W, N], ydt, acc_dump_opt: as in qsync_qlinear_fwd.
 *
 * The data gradient of the convolution is this same entry point with the roles of the channels
 * swapped: dX[m, c] = conv3x3(dyq [nimg,H,W,N], wflip [C, 9*N]) with wflip from qsync_conv3x3_wflip
 * (C and N exchanged in the call).  The weight gradient is qsync_qlinear_bwd (dx_opt = NULL) on the
 * transposed patch matrix of qsync_im2col3x3_i8.
 */
int qsync_conv3x3_fwd(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N,
                      const void* xq, const float* sx, const void* wq, const float* sw, int wgran,
                      const float* bias_opt, void* y, int ydt, int32_t* acc_dump_opt, void* stream);

/*
 * qsync_conv3x3_fwd_amax - qsync_conv3x3_fwd that also collects max |Y| in its epilogue (as qsync_qlinear_fwd_amax
 * does for the linear operator; paper: Backend section, "Minimum and Maximum Optimization"), so that a convolution
 * fed directly by Y takes its activation scale from that word (qsync_scale_from_amax) and quantizes Y without a
 * pass of its own for the maximum.
 * y_amax  device float, read and written: max(previous value, max |Y| as stored); 4-byte aligned; see
 *         qsync_qlinear_fwd_amax.  All other arguments and errors as qsync_conv3x3_fwd.
 */
int qsync_conv3x3_fwd_amax(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N,
                           const void* xq, const float* sx, const void* wq, const float* sw, int wgran,
                           const float* bias_opt, void* y, int ydt, int32_t* acc_dump_opt, float* y_amax, void* stream);

/*
 * qsync_conv3x3_wflip - weights of the data-gradient convolution:
 *   wflip[c, ((2-kh)*3 + (2-kw))*N + n] = w[n, (kh*3+kw)*C + c]
 * (window mirrored, channel roles exchanged), so that dX = conv3x3(dY, wflip).
 * w [N, 9*C] and wflip [C, 9*N] of wdt (QSYNC_I8 or QSYNC_F16), device, distinct buffers.
 */
int qsync_conv3x3_wflip(const void* w, int wdt, int64_t N, int64_t C, void* wflip, void* stream);

/*
 * qsync_im2col3x3_i8 - patches of a 3x3, stride-1, pad-1 convolution, built from int8 codes.
 * Paper: Backend section (low-precision convolution runs on NHWC tensors; the convolution is
 * lowered to the GEMM of the linear operator).  The activation is quantized once as an NHWC
 * tensor (qsync_absmax_scale + qsync_quantize on [nimg*H*W, C]) and expanded afterwards; the
 * codes equal those of quantizing the fp16 patch matrix with the same per-tensor scale.
 *
 *   a [m, (kh*3+kw)*C + c] = xq[n, h+kh-1, w+kw-1, c]   (0 outside the image),  m = (n*H + h)*W + w
 *   aT[k, m]               = a[m, k]
 *
 * xq      [nimg, H, W, C] int8, 16-byte aligned.  C % 16 == 0 (QSYNC_ERR_UNSUPPORTED otherwise).
 * a_opt   out, [nimg*H*W, 9*C] int8, 16-byte aligned, or NULL.
 * aT_opt  out, [9*C, nimg*H*W] int8, 16-byte aligned, or NULL; needs nimg*H*W % 16 == 0 (QSYNC_ERR_ALIGN).
 */
int qsync_im2col3x3_i8(const void* xq, int64_t nimg, int64_t H, int64_t W, int64_t C,
                       void* a_opt, void* aT_opt, void* stream);

/*
 * qsync_dequantize - standalone dequantizer (used when it is not fused into a GEMM).
 * Paper: Indicator section (x_hat = code * q), Cost Mapper (layer-wise / channel-wise
 * dequantizers as element-wise kernels).
 *
 *   y[r,c] = float(a[r,c]) * (tensor_scale * tensor_scale_dev[0]) * row_scale[r] * col_scale[c] + col_bias[c]
 *   (absent factors are 1, absent bias is 0; evaluated in fp32 in that order)
 *
 * a  [rows, ld] of adt (QSYNC_I32 or QSYNC_I8).  tensor_scale is a HOST float;
 * tensor_scale_dev_opt is a DEVICE pointer to one float or NULL (the per-tensor scale that
 * qsync_absmax_scale left on the device: no host round trip is needed to dequantize saved
 * codes, e.g. for the FP16 backward of an INT8 forward, paper: footnote in the Cost Mapper paragraph).
 * row_scale_opt rows floats, col_scale_opt / col_bias_opt cols floats, or NULL.
 * y  out, packed [rows, cols] of ydt (QSYNC_F32 or QSYNC_F16).
 */
int qsync_dequantize(const void* a, int adt, int64_t rows, int64_t cols, int64_t ld,
                     const float* row_scale_opt, const float* col_scale_opt, float tensor_scale,
                     const float* tensor_scale_dev_opt, const float* col_bias_opt, void* y, int ydt,
                     void* stream);

/*
 * qsync_variance_increment - HOST function (no GPU work, every pointer is a host pointer): the indicator
 * of one unary computation-intensive operator (linear, convolution) from tensor statistics.
 * Paper: Indicator section, Prop. 2 (a stochastic-rounding grid of spacing d adds a variance of
 * d^2 D / 6 to a tensor of D elements; d = q on a fixed-point grid, d = 2^e eps with eps = 2^-k and
 * 2^e <= max|t| < 2^(e+1) on a floating-point one) and Prop. 3 with its two case equations:
 *
 *   sigma_fp = |x|^2 Var[v] + |v|^2 Var[x]            x: parameter, v: activation, in the operator's format
 *   sigma_bp = |grad_v|^2 Var[v] + |v|^2 Var[grad_v]   the activation gradient always on the floating-point grid
 *   Omega    = gamma^2 d_o sigma_fp + (d_L - d_o) sigma_bp
 *
 * The statistics are what qsync_absmax_scale delivers in one pass (sumsq_opt, amax_opt) plus the element
 * count.  kind QSYNC_QUANT_FIXED uses the fixed-point scales q_x, q_v for x and v; QSYNC_QUANT_FLOAT ignores
 * them.  k: mantissa bits kept by the floating-point format (the paper states 9 for float16).
 * sigma_fp / sigma_bp may be NULL.  Errors: QSYNC_ERR_NULL, _BAD_ENUM, _BAD_SHAPE (negative or non-finite
 * statistics, d_L < d_o), _UNSUPPORTED (k outside 1..52, negative or non-finite scales or gamma).
 */
typedef enum { QSYNC_QUANT_FIXED = 0, QSYNC_QUANT_FLOAT = 1 } qsync_quant_kind_t;
typedef struct { double sumsq; double amax; int64_t D; } qsync_tensor_stats_t;
int qsync_variance_increment(int kind, const qsync_tensor_stats_t* x, const qsync_tensor_stats_t* v,
                             const qsync_tensor_stats_t* grad_v, double q_x, double q_v, int k, double gamma,
                             int64_t d_o, int64_t d_L, double* sigma_fp, double* sigma_bp, double* omega);

/* hipError_t (as int) of the last failing HIP call made by this thread, 0 if none. */
int qsync_last_hip_error(void);
/* Static description of a qsync_status_t. */
const char* qsync_strerror(int status);
/* Library version, major*100 + minor. */
int qsync_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QSYNC_H */
