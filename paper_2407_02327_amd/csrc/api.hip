// C ABI of libqsync: argument validation (the "front-end security wrapper" the paper's backend
// puts around its tensorized kernels) and dispatch to the gfx950 kernels.  Validation never
// touches the HIP runtime, so every argument error is reported even on a machine with no GPU.
#include "../../include/qsync.h"
#include "../../include/qsync_debug.h"
#include "kernels.h"

#include <limits>

using namespace qsync;

namespace {

thread_local int g_last_hip_error = 0;

int hip_status(hipError_t e)
{
    if(e == hipSuccess) return QSYNC_OK;
    g_last_hip_error = static_cast<int>(e);
    (void)hipGetLastError();   // clear the sticky launch error
    return QSYNC_ERR_HIP;
}

bool is_float_dtype(int dt) { return dt == QSYNC_F32 || dt == QSYNC_F16; }
bool is_tag(int t) { return t == QSYNC_INT8 || t == QSYNC_FP16 || t == QSYNC_FP32; }
bool is_gran(int g) { return g == QSYNC_PER_TENSOR || g == QSYNC_PER_ROW || g == QSYNC_PER_COL; }
bool is_round(int r) { return r == QSYNC_ROUND_NEAREST || r == QSYNC_ROUND_STOCHASTIC || r == QSYNC_ROUND_FLOOR; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// rows*cols (and a few multiples of it) must fit comfortably in int64
bool count_ok(int64_t a, int64_t b)
{
    if(a < 0 || b < 0) return false;
    if(a == 0 || b == 0) return true;
    return a <= (std::numeric_limits<int64_t>::max() / 64) / b;
}

// the contraction axis of an MFMA GEMM: rows of at most 16 MiB (32-bit lane offsets inside an operand panel)
bool gemm_row_ok(int tag, int64_t k)
{
    const int64_t esz = tag == QSYNC_INT8 ? 1 : (tag == QSYNC_FP16 ? 2 : 4);
    return k <= kGemmMaxRowBytes / esz;
}

size_t round256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

}  // namespace

extern "C" {

int qsync_version(void) { return 100; }

int qsync_last_hip_error(void) { return g_last_hip_error; }

const char* qsync_strerror(int status)
{
    switch(status)
    {
    case QSYNC_OK: return "ok";
    case QSYNC_ERR_NULL: return "a required pointer is NULL";
    case QSYNC_ERR_BAD_ENUM: return "an enum argument holds no enumerator";
    case QSYNC_ERR_BAD_SHAPE: return "bad shape: negative dimension, ld < cols, or element count overflow";
    case QSYNC_ERR_UNSUPPORTED: return "unsupported combination of arguments";
    case QSYNC_ERR_ALIGN: return "pointer or dimension violates an alignment rule";
    case QSYNC_ERR_WORKSPACE: return "workspace missing or too small";
    case QSYNC_ERR_HIP: return "a HIP runtime call failed (see qsync_last_hip_error)";
    default: return "unknown status";
    }
}

size_t qsync_absmax_workspace_bytes(int64_t rows, int64_t cols, int gran)
{
    if(rows < 0 || cols < 0 || !is_gran(gran)) return 0;
    return round256(absmax_workspace_bytes(rows, cols, gran));
}

int qsync_absmax_scale(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int gran, int bits,
                       float* scale, float* inv_scale, float* amax_opt, float* colsum_opt, float* sumsq_opt,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    if(!x || !scale || !inv_scale) return QSYNC_ERR_NULL;
    if(!is_float_dtype(xdt) || !is_gran(gran)) return QSYNC_ERR_BAD_ENUM;
    if(!count_ok(rows, cols) || ld < cols || !count_ok(rows, ld)) return QSYNC_ERR_BAD_SHAPE;
    if(bits < 2 || bits > 8) return QSYNC_ERR_UNSUPPORTED;
    if((colsum_opt || sumsq_opt) && gran != QSYNC_PER_TENSOR) return QSYNC_ERR_UNSUPPORTED;
    if(colsum_opt && cols > (int64_t(1) << 19)) return QSYNC_ERR_UNSUPPORTED;   // one block-maximum slot per column strip
    if(rows == 0 || cols == 0) return QSYNC_OK;
    const size_t need = qsync_absmax_workspace_bytes(rows, cols, gran);
    if(need > 0)
    {
        if(!workspace || workspace_bytes < need) return QSYNC_ERR_WORKSPACE;
        if(!aligned16(workspace)) return QSYNC_ERR_ALIGN;
    }
    const float qmax = static_cast<float>((1 << (bits - 1)) - 1);
    return hip_status(launch_absmax_scale(x, xdt, rows, cols, ld, gran, qmax, scale, inv_scale, amax_opt, colsum_opt,
                                          sumsq_opt, workspace, static_cast<hipStream_t>(stream)));
}

int qsync_absmax_scale_static(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int bits, float* scale,
                              float* inv_scale, float* amax_opt, float* colsum_opt, float* sumsq_opt, void* stream)
{
    if(!x || !scale || !inv_scale) return QSYNC_ERR_NULL;
    if(!is_float_dtype(xdt)) return QSYNC_ERR_BAD_ENUM;
    if(!count_ok(rows, cols) || ld < cols || !count_ok(rows, ld)) return QSYNC_ERR_BAD_SHAPE;
    if(bits < 2 || bits > 8) return QSYNC_ERR_UNSUPPORTED;
    // the library's own scratch holds the column-sum partials of at most kStaticMaxCols columns
    if(colsum_opt && cols > kStaticMaxCols) return QSYNC_ERR_WORKSPACE;
    if(rows == 0 || cols == 0) return QSYNC_OK;
    if(absmax_workspace_bytes(rows, colsum_opt ? cols : 0, kPerTensor) > kStaticScratchBytes) return QSYNC_ERR_WORKSPACE;
    void*      ws = nullptr;
    hipError_t e  = static_scratch(&ws);
    if(e != hipSuccess) return hip_status(e);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the arrival counter must start at zero whatever an earlier call left behind (cleared by a kernel, not by a
    // memset node, so that the call can be captured into a graph)
    e = launch_zero_f32(static_cast<float*>(ws), 64, st);
    if(e != hipSuccess) return hip_status(e);
    const float qmax = static_cast<float>((1 << (bits - 1)) - 1);
    return hip_status(launch_absmax_scale(x, xdt, rows, cols, ld, kPerTensor, qmax, scale, inv_scale, amax_opt, colsum_opt,
                                          sumsq_opt, ws, st));
}

int qsync_quantize(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int tag, int bits, int gran,
                   int rnd, uint64_t philox_seed, uint64_t philox_offset, const float* inv_scale, void* q_opt,
                   void* qT_opt, void* stream)
{
    if(!x || (!q_opt && !qT_opt)) return QSYNC_ERR_NULL;
    if(!is_tag(tag) || !is_float_dtype(xdt)) return QSYNC_ERR_BAD_ENUM;
    if(tag == QSYNC_INT8)
    {
        if(!inv_scale) return QSYNC_ERR_NULL;
        if(!is_gran(gran) || !is_round(rnd)) return QSYNC_ERR_BAD_ENUM;
    }
    if(!count_ok(rows, cols) || ld < cols || !count_ok(rows, ld)) return QSYNC_ERR_BAD_SHAPE;
    if(tag == QSYNC_INT8 && (bits < 2 || bits > 8)) return QSYNC_ERR_UNSUPPORTED;
    const bool fp_sr = tag == QSYNC_FP16 && rnd == QSYNC_ROUND_STOCHASTIC && xdt == QSYNC_F32;
    if(fp_sr && bits != 0 && (bits < 7 || bits > 10)) return QSYNC_ERR_UNSUPPORTED;
    if(rows == 0 || cols == 0) return QSYNC_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if(fp_sr)
        return hip_status(launch_convert_sr(static_cast<const float*>(x), rows, cols, ld, bits == 0 ? 9 : bits,
                                            philox_seed, philox_offset, q_opt, qT_opt, st));
    if(tag == QSYNC_INT8)
    {
        const int qmax = (1 << (bits - 1)) - 1;
        return hip_status(launch_quantize_int8(x, xdt, rows, cols, ld, qmax, gran, rnd, philox_seed, philox_offset,
                                               inv_scale, static_cast<int8_t*>(q_opt), static_cast<int8_t*>(qT_opt),
                                               st));
    }
    return hip_status(launch_convert(x, xdt, rows, cols, ld, tag == QSYNC_FP16 ? kF16 : kF32, q_opt, qT_opt, st));
}

size_t qsync_absmax_quantize_workspace_bytes(int64_t rows, int64_t cols)
{
    return qsync_absmax_workspace_bytes(rows, cols, QSYNC_PER_TENSOR);
}

int qsync_absmax_quantize(const void* x, int xdt, int64_t rows, int64_t cols, int bits, int rnd, uint64_t philox_seed,
                          uint64_t philox_offset, float* scale, float* inv_scale, float* amax_opt, void* q_opt,
                          void* qT_opt, void* workspace, size_t workspace_bytes, int poll_limit, void* stream)
{
    if(!x || !scale || !inv_scale || (!q_opt && !qT_opt)) return QSYNC_ERR_NULL;
    if(!is_float_dtype(xdt) || !is_round(rnd)) return QSYNC_ERR_BAD_ENUM;
    if(!count_ok(rows, cols)) return QSYNC_ERR_BAD_SHAPE;
    if(bits < 2 || bits > 8) return QSYNC_ERR_UNSUPPORTED;
    if(rows == 0 || cols == 0) return QSYNC_OK;
    const size_t need = qsync_absmax_quantize_workspace_bytes(rows, cols);
    if(!workspace || workspace_bytes < need) return QSYNC_ERR_WORKSPACE;
    if(!aligned16(workspace)) return QSYNC_ERR_ALIGN;
    const int          qmax  = (1 << (bits - 1)) - 1;
    const unsigned int polls = poll_limit < 0 ? (1u << 14) : static_cast<unsigned int>(poll_limit);
    return hip_status(launch_absmax_quantize(x, xdt, rows, cols, qmax, rnd, philox_seed, philox_offset, scale, inv_scale,
                                             amax_opt, static_cast<int8_t*>(q_opt), static_cast<int8_t*>(qT_opt),
                                             workspace, polls, static_cast<hipStream_t>(stream)));
}

size_t qsync_qlinear_workspace_bytes(int tag, int64_t M, int64_t N, int64_t K)
{
    if(!is_tag(tag) || M < 0 || N < 0 || K < 0) return 0;
    return round256(plan_gemm(tag, M, N, K).workspace);
}

size_t qsync_qlinear_bwd_workspace_bytes(int tag, int64_t M, int64_t N, int64_t K)
{
    if(!is_tag(tag) || M < 0 || N < 0 || K < 0) return 0;
    return round256(plan_gemm(tag, M, K, N).workspace) + round256(plan_gemm(tag, N, K, M).workspace)
         + round256(colsum_workspace_bytes(M, N));
}

static int qlinear_fwd_impl(int tag, int64_t M, int64_t N, int64_t K, const void* xq, const float* sx, const void* wq,
                            const float* sw, int wgran, const float* bias_opt, void* y, int ydt, int32_t* acc_dump_opt,
                            float* y_amax_opt, void* workspace, size_t workspace_bytes, void* stream,
                            void* yq_opt = nullptr, const float* yq_inv = nullptr, int yq_qmax = 127)
{
    if(!xq || !wq || !y) return QSYNC_ERR_NULL;
    if(!is_tag(tag) || !is_float_dtype(ydt)) return QSYNC_ERR_BAD_ENUM;
    if(tag == QSYNC_INT8)
    {
        if(!sx || !sw) return QSYNC_ERR_NULL;
        if(!is_gran(wgran)) return QSYNC_ERR_BAD_ENUM;
    }
    if(!count_ok(M, N) || !count_ok(M, K) || !count_ok(N, K)) return QSYNC_ERR_BAD_SHAPE;
    if(!gemm_row_ok(tag, K)) return QSYNC_ERR_UNSUPPORTED;
    if(tag == QSYNC_INT8 && wgran == QSYNC_PER_COL) return QSYNC_ERR_UNSUPPORTED;
    if(tag != QSYNC_INT8 && acc_dump_opt) return QSYNC_ERR_UNSUPPORTED;
    if(tag != QSYNC_FP32)
    {
        if(K % (tag == QSYNC_INT8 ? 16 : 8) != 0) return QSYNC_ERR_ALIGN;
        if(!aligned16(xq) || !aligned16(wq)) return QSYNC_ERR_ALIGN;
    }
    if(M == 0 || N == 0) return QSYNC_OK;
    const GemmPlan plan = plan_gemm(tag, M, N, K);
    if(plan.workspace > 0)
    {
        if(!workspace || workspace_bytes < plan.workspace) return QSYNC_ERR_WORKSPACE;
        if(!aligned16(workspace)) return QSYNC_ERR_ALIGN;
    }
    GemmProblem p{};
    p.prec = tag; p.M = M; p.N = N; p.K = K;
    p.A = xq; p.B = wq; p.C = y; p.c_dtype = ydt;
    if(tag == QSYNC_INT8)
    {
        p.s0 = sx;
        if(wgran == QSYNC_PER_TENSOR) p.s1 = sw; else p.col_scale = sw;
        p.acc_dump = acc_dump_opt;
    }
    p.col_bias = bias_opt;
    p.out_amax_bits = reinterpret_cast<unsigned int*>(y_amax_opt);
    p.out_codes = yq_opt; p.out_code_inv = yq_inv; p.out_code_qmax = yq_qmax;
    return hip_status(launch_gemm(p, plan, workspace, static_cast<hipStream_t>(stream)));
}

int qsync_qlinear_fwd(int tag, int64_t M, int64_t N, int64_t K, const void* xq, const float* sx, const void* wq,
                      const float* sw, int wgran, const float* bias_opt, void* y, int ydt, int32_t* acc_dump_opt,
                      void* workspace, size_t workspace_bytes, void* stream)
{
    return qlinear_fwd_impl(tag, M, N, K, xq, sx, wq, sw, wgran, bias_opt, y, ydt, acc_dump_opt, nullptr, workspace,
                            workspace_bytes, stream);
}

int qsync_qlinear_fwd_amax(int tag, int64_t M, int64_t N, int64_t K, const void* xq, const float* sx, const void* wq,
                           const float* sw, int wgran, const float* bias_opt, void* y, int ydt, int32_t* acc_dump_opt,
                           float* y_amax, void* workspace, size_t workspace_bytes, void* stream)
{
    if(!y_amax) return QSYNC_ERR_NULL;
    if((reinterpret_cast<uintptr_t>(y_amax) & 3u) != 0) return QSYNC_ERR_ALIGN;
    return qlinear_fwd_impl(tag, M, N, K, xq, sx, wq, sw, wgran, bias_opt, y, ydt, acc_dump_opt, y_amax, workspace,
                            workspace_bytes, stream);
}

int qsync_qlinear_fwd_codes(int tag, int64_t M, int64_t N, int64_t K, const void* xq, const float* sx, const void* wq,
                            const float* sw, int wgran, const float* bias_opt, void* y, int ydt, int bits,
                            const float* next_inv_scale, void* yq, float* y_amax_opt, void* workspace,
                            size_t workspace_bytes, void* stream)
{
    if(!yq || !next_inv_scale) return QSYNC_ERR_NULL;
    if(bits < 2 || bits > 8) return QSYNC_ERR_UNSUPPORTED;
    if(y_amax_opt && (reinterpret_cast<uintptr_t>(y_amax_opt) & 3u) != 0) return QSYNC_ERR_ALIGN;
    // fp32 operands whose rows are not 16-byte multiples run the any-shape kernel, which has no code output
    if(tag == QSYNC_FP32 && ((K * 4) % 16 != 0 || !aligned16(xq) || !aligned16(wq))) return QSYNC_ERR_UNSUPPORTED;
    return qlinear_fwd_impl(tag, M, N, K, xq, sx, wq, sw, wgran, bias_opt, y, ydt, nullptr, y_amax_opt, workspace,
                            workspace_bytes, stream, yq, next_inv_scale, (1 << (bits - 1)) - 1);
}

int qsync_transpose_i8(const void* in, int64_t rows, int64_t cols, void* out, void* stream)
{
    if(!in || !out) return QSYNC_ERR_NULL;
    if(!count_ok(rows, cols)) return QSYNC_ERR_BAD_SHAPE;
    if(in == out) return QSYNC_ERR_UNSUPPORTED;
    return hip_status(launch_transpose_i8(static_cast<const int8_t*>(in), rows, cols, static_cast<int8_t*>(out),
                                          static_cast<hipStream_t>(stream)));
}

int qsync_scale_from_amax(float* amax, int bits, float* scale, float* inv_scale, int consume, void* stream)
{
    if(!amax || !scale || !inv_scale) return QSYNC_ERR_NULL;
    if(bits < 2 || bits > 8) return QSYNC_ERR_UNSUPPORTED;
    const float qmax = static_cast<float>((1 << (bits - 1)) - 1);
    return hip_status(launch_scale_from_amax(amax, qmax, scale, inv_scale, consume != 0, static_cast<hipStream_t>(stream)));
}

int qsync_qlinear_bwd(int tag, int64_t M, int64_t N, int64_t K, const void* dyq, const void* dyqT, const float* sdy,
                      const void* xqT, const float* sx, const void* wqbT, const float* swb, int wbgran, void* dx_opt,
                      int dxdt, void* dw_opt, int dwdt, float* db_opt, const void* dy_float_opt, int dydt,
                      int32_t* acc_dx_dump_opt, int32_t* acc_dw_dump_opt, void* workspace, size_t workspace_bytes,
                      void* stream)
{
    if(dx_opt && (!dyq || !wqbT)) return QSYNC_ERR_NULL;
    if(dw_opt && (!dyqT || !xqT)) return QSYNC_ERR_NULL;
    if(db_opt && !dy_float_opt) return QSYNC_ERR_NULL;
    if(!is_tag(tag)) return QSYNC_ERR_BAD_ENUM;
    if(dx_opt && !is_float_dtype(dxdt)) return QSYNC_ERR_BAD_ENUM;
    if(dw_opt && !is_float_dtype(dwdt)) return QSYNC_ERR_BAD_ENUM;
    if(db_opt && !is_float_dtype(dydt)) return QSYNC_ERR_BAD_ENUM;
    if(tag == QSYNC_INT8)
    {
        if((dx_opt || dw_opt) && !sdy) return QSYNC_ERR_NULL;
        if(dx_opt && !swb) return QSYNC_ERR_NULL;
        if(dw_opt && !sx) return QSYNC_ERR_NULL;
        if(dx_opt && !is_gran(wbgran)) return QSYNC_ERR_BAD_ENUM;
    }
    if(!count_ok(M, N) || !count_ok(M, K) || !count_ok(N, K)) return QSYNC_ERR_BAD_SHAPE;
    if((dx_opt && !gemm_row_ok(tag, N)) || (dw_opt && !gemm_row_ok(tag, M))) return QSYNC_ERR_UNSUPPORTED;
    if(tag == QSYNC_INT8 && dx_opt && wbgran == QSYNC_PER_COL) return QSYNC_ERR_UNSUPPORTED;
    if(tag != QSYNC_INT8 && (acc_dx_dump_opt || acc_dw_dump_opt)) return QSYNC_ERR_UNSUPPORTED;
    if(tag != QSYNC_FP32)
    {
        const int64_t mult = tag == QSYNC_INT8 ? 16 : 8;
        if(dx_opt && (N % mult != 0 || !aligned16(dyq) || !aligned16(wqbT))) return QSYNC_ERR_ALIGN;
        if(dw_opt && (M % mult != 0 || !aligned16(dyqT) || !aligned16(xqT))) return QSYNC_ERR_ALIGN;
    }
    const GemmPlan plan_dx = plan_gemm(tag, M, K, N);
    const GemmPlan plan_dw = plan_gemm(tag, N, K, M);
    const size_t   off_dw  = round256(plan_dx.workspace);
    const size_t   off_db  = off_dw + round256(plan_dw.workspace);
    const size_t   need    = (dx_opt ? plan_dx.workspace : 0) + (dw_opt ? plan_dw.workspace : 0)
                        + ((db_opt && M > 0 && N > 0) ? colsum_workspace_bytes(M, N) : 0);
    if(need > 0)
    {
        if(!workspace || workspace_bytes < qsync_qlinear_bwd_workspace_bytes(tag, M, N, K)) return QSYNC_ERR_WORKSPACE;
        if(!aligned16(workspace)) return QSYNC_ERR_ALIGN;
    }
    hipStream_t st  = static_cast<hipStream_t>(stream);
    char*       wsb = static_cast<char*>(workspace);
    if(dx_opt && M > 0 && K > 0)
    {
        GemmProblem p{};
        p.prec = tag; p.M = M; p.N = K; p.K = N;
        p.A = dyq; p.B = wqbT; p.C = dx_opt; p.c_dtype = dxdt;
        if(tag == QSYNC_INT8)
        {
            p.s0 = sdy;
            if(wbgran == QSYNC_PER_TENSOR) p.s1 = swb; else p.col_scale = swb;
            p.acc_dump = acc_dx_dump_opt;
        }
        const int rc = hip_status(launch_gemm(p, plan_dx, wsb, st));
        if(rc != QSYNC_OK) return rc;
    }
    if(dw_opt && N > 0 && K > 0)
    {
        GemmProblem p{};
        p.prec = tag; p.M = N; p.N = K; p.K = M;
        p.A = dyqT; p.B = xqT; p.C = dw_opt; p.c_dtype = dwdt;
        if(tag == QSYNC_INT8)
        {
            p.s0 = sdy; p.s1 = sx;
            p.acc_dump = acc_dw_dump_opt;
        }
        const int rc = hip_status(launch_gemm(p, plan_dw, wsb ? wsb + off_dw : nullptr, st));
        if(rc != QSYNC_OK) return rc;
    }
    if(db_opt && N > 0 && M == 0)
    {   // no rows to sum: the bias gradient is zero (the column-sum kernels need their workspace, which an
        // empty batch does not have to bring)
        const int rc = hip_status(launch_zero_f32(db_opt, N, st));
        if(rc != QSYNC_OK) return rc;
    }
    else if(db_opt && N > 0)
    {
        const int rc = hip_status(launch_colsum(dy_float_opt, dydt, M, N, db_opt,
                                                reinterpret_cast<float*>(wsb + off_db), st));
        if(rc != QSYNC_OK) return rc;
    }
    return QSYNC_OK;
}

size_t qsync_qlinear_bwd_rm_workspace_bytes(int tag, int64_t M, int64_t N, int64_t K)
{
    if((tag != QSYNC_INT8 && tag != QSYNC_FP16) || M < 0 || N < 0 || K < 0) return 0;
    // the data gradient (and bias gradient) go through qsync_qlinear_bwd, which asks for its own full size
    const size_t nt = qsync_qlinear_bwd_workspace_bytes(tag, M, N, K);
    const size_t rm = round256(plan_gemm(tag, M, K, N).workspace)
                    + round256(plan_gemm(tag, N, K, M, -1, -1, true, /*tn=*/true).workspace);
    return nt > rm ? nt : rm;
}

int qsync_qlinear_bwd_rm(int tag, int64_t M, int64_t N, int64_t K, const void* dyq, const float* sdy, const void* xq, const float* sx,
                         const void* wqbT, const float* swb, int wbgran, void* dx_opt, int dxdt, void* dw_opt, int dwdt,
                         float* db_opt, const void* dy_float_opt, int dydt, int32_t* acc_dx_dump_opt,
                         int32_t* acc_dw_dump_opt, void* workspace, size_t workspace_bytes, void* stream)
{
    if(!is_tag(tag)) return QSYNC_ERR_BAD_ENUM;
    if(tag != QSYNC_INT8 && tag != QSYNC_FP16) return QSYNC_ERR_UNSUPPORTED;
    const bool i8 = tag == QSYNC_INT8;
    if((dx_opt || dw_opt) && (!dyq || (i8 && !sdy))) return QSYNC_ERR_NULL;
    if(dx_opt && (!wqbT || (i8 && !swb))) return QSYNC_ERR_NULL;
    if(dw_opt && (!xq || (i8 && !sx))) return QSYNC_ERR_NULL;
    if(db_opt && !dy_float_opt) return QSYNC_ERR_NULL;
    if(!i8 && (acc_dx_dump_opt || acc_dw_dump_opt)) return QSYNC_ERR_UNSUPPORTED;
    if(dx_opt && (!is_float_dtype(dxdt) || !is_gran(wbgran))) return QSYNC_ERR_BAD_ENUM;
    if(dw_opt && !is_float_dtype(dwdt)) return QSYNC_ERR_BAD_ENUM;
    if(db_opt && !is_float_dtype(dydt)) return QSYNC_ERR_BAD_ENUM;
    if(!count_ok(M, N) || !count_ok(M, K) || !count_ok(N, K)) return QSYNC_ERR_BAD_SHAPE;
    if(dx_opt && wbgran == QSYNC_PER_COL) return QSYNC_ERR_UNSUPPORTED;
    if((dx_opt && !gemm_row_ok(tag, N)) || (dw_opt && (N >= (int64_t(1) << 24) || K >= (int64_t(1) << 24))))
        return QSYNC_ERR_UNSUPPORTED;
    const int64_t mult = i8 ? 16 : 8;                           // elements per 16-byte chunk
    if(dx_opt && (N % mult != 0 || !aligned16(dyq) || !aligned16(wqbT))) return QSYNC_ERR_ALIGN;
    // the weight gradient reads both operands row-major: whole K tiles of contraction rows, 16-byte column chunks
    if(dw_opt && (M % 128 != 0 || N % mult != 0 || K % mult != 0 || !aligned16(dyq) || !aligned16(xq))) return QSYNC_ERR_ALIGN;
    // the data gradient is the NT GEMM of qsync_qlinear_bwd; it also owns the bias gradient
    if(dx_opt || db_opt)
    {
        const int rc = qsync_qlinear_bwd(tag, M, N, K, dyq, nullptr, sdy, nullptr, nullptr, wqbT, swb, wbgran, dx_opt, dxdt,
                                         nullptr, dwdt, db_opt, dy_float_opt, dydt, acc_dx_dump_opt, nullptr, workspace,
                                         workspace_bytes, stream);
        if(rc != QSYNC_OK) return rc;
    }
    if(!dw_opt || N == 0 || K == 0) return QSYNC_OK;
    const GemmPlan plan   = plan_gemm(tag, N, K, M, -1, -1, true, /*tn=*/M > 0);
    const size_t   off_dw = round256(plan_gemm(tag, M, K, N).workspace);
    if(plan.workspace > 0)
    {
        if(!workspace || workspace_bytes < qsync_qlinear_bwd_rm_workspace_bytes(tag, M, N, K)) return QSYNC_ERR_WORKSPACE;
        if(!aligned16(workspace)) return QSYNC_ERR_ALIGN;
    }
    GemmProblem p{};
    p.prec = tag; p.M = N; p.N = K; p.K = M;
    p.A = dyq; p.B = xq; p.C = dw_opt; p.c_dtype = dwdt;
    p.s0 = i8 ? sdy : nullptr; p.s1 = i8 ? sx : nullptr; p.acc_dump = acc_dw_dump_opt;
    p.tn = true;
    if(M == 0)
    {   // empty contraction: the NT form writes the zeros (no operand is read)
        p.tn = false;
    }
    return hip_status(launch_gemm(p, plan, workspace ? static_cast<char*>(workspace) + off_dw : nullptr,
                                  static_cast<hipStream_t>(stream)));
}

// Workspace of qsync_qlinear_bwd_fp16_of_int8: binary16 operands of the FP16 backward, then the GEMMs' own scratch;
// every part starts on a 256-byte boundary.
namespace {
struct Fp16BwdLayout { size_t off_xhT, off_wh, off_whT, off_dyh, off_dyhT, off_gemm, total; };
Fp16BwdLayout fp16_bwd_layout(int64_t M, int64_t N, int64_t K, int dydt)
{
    Fp16BwdLayout l;
    size_t at = 0;
    auto take = [&](int64_t elems) { const size_t o = at; at += round256(static_cast<size_t>(elems) * 2); return o; };
    l.off_xhT  = take(K * M);
    l.off_wh   = take(N * K);
    l.off_whT  = take(K * N);
    l.off_dyh  = take(dydt == QSYNC_F16 ? 0 : M * N);          // a binary16 gradient is used in place
    l.off_dyhT = take(N * M);
    l.off_gemm = at;
    const size_t nt = qsync_qlinear_bwd_workspace_bytes(QSYNC_FP16, M, N, K), rm = qsync_qlinear_bwd_rm_workspace_bytes(QSYNC_FP16, M, N, K);
    l.total    = at + (nt > rm ? nt : rm);
    return l;
}
}  // namespace

size_t qsync_qlinear_bwd_fp16_of_int8_workspace_bytes(int64_t M, int64_t N, int64_t K, int dydt)
{
    if(M < 0 || N < 0 || K < 0 || !is_float_dtype(dydt) || !count_ok(M, N) || !count_ok(M, K) || !count_ok(N, K)) return 0;
    return fp16_bwd_layout(M, N, K, dydt).total;
}

int qsync_qlinear_bwd_fp16_of_int8(int64_t M, int64_t N, int64_t K, const void* dy, int dydt, const void* xqT,
                                   int x_rowmajor, const float* sx, const void* wq, const float* sw, int wgran, void* dx_opt, int dxdt,
                                   void* dw_opt, int dwdt, float* db_opt, void* workspace, size_t workspace_bytes,
                                   size_t* operand_offsets_opt, void* stream)
{
    if(!dy || !workspace) return !dy ? QSYNC_ERR_NULL : QSYNC_ERR_WORKSPACE;
    if(dx_opt && (!wq || !sw)) return QSYNC_ERR_NULL;
    if(dw_opt && (!xqT || !sx)) return QSYNC_ERR_NULL;
    if(!is_float_dtype(dydt)) return QSYNC_ERR_BAD_ENUM;
    if(dx_opt && (!is_float_dtype(dxdt) || (wgran != QSYNC_PER_TENSOR && wgran != QSYNC_PER_ROW))) return QSYNC_ERR_BAD_ENUM;
    if(dw_opt && !is_float_dtype(dwdt)) return QSYNC_ERR_BAD_ENUM;
    if(!count_ok(M, N) || !count_ok(M, K) || !count_ok(N, K)) return QSYNC_ERR_BAD_SHAPE;
    if(x_rowmajor != 0 && x_rowmajor != 1) return QSYNC_ERR_BAD_ENUM;
    if((dx_opt && N % 8 != 0) || (dw_opt && M % 8 != 0) || !aligned16(dy)) return QSYNC_ERR_ALIGN;
    if(dw_opt && x_rowmajor && (M % 128 != 0 || N % 8 != 0 || K % 8 != 0)) return QSYNC_ERR_ALIGN;
    const Fp16BwdLayout l = fp16_bwd_layout(M, N, K, dydt);
    if(workspace_bytes < l.total) return QSYNC_ERR_WORKSPACE;
    if((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return QSYNC_ERR_ALIGN;
    if(operand_offsets_opt)
    {   // where the binary16 operands lie in the workspace (host array of 5: xhT, wh, whT, dyh, dyhT)
        const size_t offs[5] = {l.off_xhT, l.off_wh, l.off_whT, l.off_dyh, l.off_dyhT};
        for(int i = 0; i < 5; ++i) operand_offsets_opt[i] = offs[i];
    }
    if(M == 0 || N == 0 || K == 0)
        return qsync_qlinear_bwd(QSYNC_FP16, M, N, K, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                 QSYNC_PER_TENSOR, nullptr, dxdt, nullptr, dwdt, db_opt, dy, dydt, nullptr, nullptr,
                                 static_cast<char*>(workspace) + l.off_gemm, workspace_bytes - l.off_gemm, stream);
    hipStream_t st   = static_cast<hipStream_t>(stream);
    char*       base = static_cast<char*>(workspace);
    void *xhT = base + l.off_xhT, *wh = base + l.off_wh, *whT = base + l.off_whT, *dyhT = base + l.off_dyhT;
    const void* dyh = dydt == QSYNC_F16 ? dy : base + l.off_dyh;
    hipError_t e = hipSuccess;
    if(dw_opt && x_rowmajor)      // x_hat = code * q_x narrowed to binary16, [M,K] like the codes (xqT holds xq here)
        e = launch_dequantize(xqT, kI8, M, K, K, nullptr, nullptr, 1.0f, sx, nullptr, xhT, kF16, st);
    else if(dw_opt)      // x_hat^T, straight from the saved transposed codes
        e = launch_dequantize(xqT, kI8, K, M, M, nullptr, nullptr, 1.0f, sx, nullptr, xhT, kF16, st);
    if(e == hipSuccess && dx_opt)
    {   // w_hat with the forward's scales (one per output channel, or one), then its transpose for dX
        e = launch_dequantize(wq, kI8, N, K, K, wgran == QSYNC_PER_ROW ? sw : nullptr, nullptr, 1.0f,
                              wgran == QSYNC_PER_ROW ? nullptr : sw, nullptr, wh, kF16, st);
        if(e == hipSuccess) e = launch_convert(wh, kF16, N, K, K, kF16, nullptr, whT, st);
    }
    void* const dyh_out  = dydt == QSYNC_F16 ? nullptr : const_cast<void*>(dyh);
    void* const dyhT_out = (dw_opt && !x_rowmajor) ? dyhT : nullptr;
    if(e == hipSuccess && (dyh_out || dyhT_out))      // dY narrowed to binary16 (or used in place) and transposed
        e = launch_convert(dy, dydt == QSYNC_F16 ? kF16 : kF32, M, N, N, kF16, dyh_out, dyhT_out, st);
    if(e != hipSuccess) return hip_status(e);
    if(x_rowmajor)
        return qsync_qlinear_bwd_rm(QSYNC_FP16, M, N, K, dyh, nullptr, xhT, nullptr, whT, nullptr, QSYNC_PER_TENSOR, dx_opt, dxdt,
                                    dw_opt, dwdt, db_opt, dy, dydt, nullptr, nullptr, base + l.off_gemm,
                                    workspace_bytes - l.off_gemm, stream);
    return qsync_qlinear_bwd(QSYNC_FP16, M, N, K, dyh, dyhT, nullptr, xhT, nullptr, whT, nullptr, QSYNC_PER_TENSOR, dx_opt, dxdt,
                             dw_opt, dwdt, db_opt, dy, dydt, nullptr, nullptr, base + l.off_gemm, workspace_bytes - l.off_gemm,
                             stream);
}

int qsync_prepare_weights(const void* w, int wdt, int64_t N, int64_t K, int bits, float* sw, float* iw, float* aw_opt,
                          void* wq, float* swb, float* iwb, void* wqbT, void* workspace, size_t workspace_bytes,
                          void* stream)
{
    if(!w || !sw || !iw || !wq || !swb || !iwb || !wqbT) return QSYNC_ERR_NULL;
    if(!is_float_dtype(wdt)) return QSYNC_ERR_BAD_ENUM;
    if(!count_ok(N, K)) return QSYNC_ERR_BAD_SHAPE;
    if(bits < 2 || bits > 8) return QSYNC_ERR_UNSUPPORTED;
    if(N == 0 || K == 0) return QSYNC_OK;
    if(!workspace || workspace_bytes < absmax_workspace_bytes(N, K, kPerCol)) return QSYNC_ERR_WORKSPACE;
    if(!aligned16(workspace)) return QSYNC_ERR_ALIGN;
    const float qmax = static_cast<float>((1 << (bits - 1)) - 1);
    return hip_status(launch_prepare_weights(w, wdt == QSYNC_F32 ? kF32 : kF16, N, K, qmax, sw, iw, aw_opt,
                                             static_cast<int8_t*>(wq), swb, iwb, static_cast<int8_t*>(wqbT), workspace,
                                             static_cast<hipStream_t>(stream)));
}

// Workspace of qsync_conv3x3_wgrad: [margin][three displaced copies of the activation, C x Mp each][margin]
// [gradient operand, N x Mp][split-K partials]; every part starts on a 256-byte boundary.
namespace {
struct WgradLayout { ConvPaddedAxis ax; size_t margin, off_x, off_dy, off_part, total; GemmPlan plan; };
WgradLayout wgrad_layout(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N)
{
    const size_t esz = tag == QSYNC_INT8 ? 1 : 2;
    WgradLayout  l;
    l.ax       = conv_padded_axis(nimg, static_cast<int>(H), static_cast<int>(W));
    l.margin   = round256(static_cast<size_t>(l.ax.Wp) * esz);
    l.off_x    = l.margin;
    l.off_dy   = l.off_x + round256(static_cast<size_t>(3 * C * l.ax.Mp) * esz) + l.margin;
    l.off_part = l.off_dy + round256(static_cast<size_t>(N * l.ax.Mp) * esz);
    l.plan     = plan_gemm(tag, N, 9 * C, l.ax.Mp);
    l.total    = l.off_part + l.plan.workspace;
    return l;
}
// The gathering form: the weight-gradient GEMM reads the row-major gradient and the NHWC activation themselves (TN
// form, patches formed by its loads).  Needs whole K tiles of 128 pixels and 32-bit byte offsets into the activation.
bool wgrad_gathers(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N)
{
    const int64_t esz = tag == QSYNC_INT8 ? 1 : 2, M = nimg * H * W;
    return M > 0 && M % 128 == 0 && M * C * esz < (int64_t(1) << 31) && N < (int64_t(1) << 24) && 9 * C < (int64_t(1) << 24)
           && H <= 65535 && W <= 65535;
}
bool wgrad_shape_ok(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N)
{
    const int64_t esz = tag == QSYNC_INT8 ? 1 : 2;
    if(nimg < 0 || H < 0 || W < 0 || C < 0 || N < 0 || H > 65535 || (W + 16) * esz > 1024 || C > (1 << 20)
       || N > (int64_t(1) << 31))
        return false;
    if(H > 0 && W > 0 && nimg > ((int64_t(1) << 31) - 1) / ((H + 1) * (W + 16))) return false;
    const ConvPaddedAxis ax = conv_padded_axis(nimg, static_cast<int>(H), static_cast<int>(W));
    return 3 * C * ax.Mp * esz < (int64_t(1) << 32) - (1 << 20) && count_ok(N, ax.Mp) && count_ok(N, 9 * C);
}
}  // namespace

size_t qsync_conv3x3_wgrad_workspace_bytes(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N)
{
    if((tag != QSYNC_INT8 && tag != QSYNC_FP16) || nimg <= 0 || H <= 0 || W <= 0 || C <= 0 || N <= 0
       || !wgrad_shape_ok(tag, nimg, H, W, C, N))
        return 0;
    if(wgrad_gathers(tag, nimg, H, W, C, N))
    {   // split-K partials only (the largest over the tile shapes, so that a pinned tile fits too)
        size_t need = plan_gemm(tag, N, 9 * C, nimg * H * W, -1, -1, true, true).workspace;
        for(int t = 0; t < 3; ++t)
        {
            const size_t w = plan_gemm(tag, N, 9 * C, nimg * H * W, t, 0, true, true).workspace;
            need = w > need ? w : need;
        }
        return round256(need);
    }
    return wgrad_layout(tag, nimg, H, W, C, N).total;
}

int qsync_conv3x3_wgrad(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N, const void* xq, const float* sx,
                        const void* dyq, const float* sdy, void* dw, int dwdt, int32_t* acc_dump_opt, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    if(!xq || !dyq || !dw) return QSYNC_ERR_NULL;
    if(!is_tag(tag) || !is_float_dtype(dwdt)) return QSYNC_ERR_BAD_ENUM;
    if(tag == QSYNC_FP32) return QSYNC_ERR_UNSUPPORTED;
    if(tag == QSYNC_INT8 && (!sx || !sdy)) return QSYNC_ERR_NULL;
    if(tag != QSYNC_INT8 && acc_dump_opt) return QSYNC_ERR_UNSUPPORTED;
    if(!wgrad_shape_ok(tag, nimg, H, W, C, N)) return QSYNC_ERR_BAD_SHAPE;
    if(nimg == 0 || H == 0 || W == 0 || C == 0 || N == 0) return QSYNC_OK;
    const int esz = tag == QSYNC_INT8 ? 1 : 2;
    if((C * esz) % 16 != 0 || (N * esz) % 16 != 0 || !aligned16(xq) || !aligned16(dyq)) return QSYNC_ERR_ALIGN;
    hipStream_t st  = static_cast<hipStream_t>(stream);
    if(wgrad_gathers(tag, nimg, H, W, C, N))
    {
        const int64_t  M    = nimg * H * W;
        const GemmPlan plan = plan_gemm(tag, N, 9 * C, M, -1, -1, true, /*tn=*/true);
        if(plan.workspace > 0)
        {
            if(!workspace || workspace_bytes < plan.workspace) return QSYNC_ERR_WORKSPACE;
            if((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return QSYNC_ERR_ALIGN;
        }
        GemmProblem p{};
        p.prec = tag; p.M = N; p.N = 9 * C; p.K = M;
        p.A = dyq; p.B = xq; p.C = dw; p.c_dtype = dwdt; p.tn = true;
        p.conv_H = static_cast<int>(H); p.conv_W = static_cast<int>(W); p.conv_C = C;
        if(tag == QSYNC_INT8) { p.s0 = sdy; p.s1 = sx; p.acc_dump = acc_dump_opt; }
        return hip_status(launch_gemm(p, plan, workspace, st));
    }
    const WgradLayout l = wgrad_layout(tag, nimg, H, W, C, N);
    if(!workspace || workspace_bytes < l.total) return QSYNC_ERR_WORKSPACE;
    if((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return QSYNC_ERR_ALIGN;
    uint8_t*    xT  = static_cast<uint8_t*>(workspace) + l.off_x;
    uint8_t*    dyT = static_cast<uint8_t*>(workspace) + l.off_dy;
    hipError_t  e   = launch_conv_padded_transpose(xq, esz, nimg, static_cast<int>(H), static_cast<int>(W), static_cast<int>(C), 3, xT, static_cast<int>(l.margin), st);
    if(e != hipSuccess) return hip_status(e);
    e = launch_conv_padded_transpose(dyq, esz, nimg, static_cast<int>(H), static_cast<int>(W), static_cast<int>(N), 1, dyT, 0, st);
    if(e != hipSuccess) return hip_status(e);
    GemmProblem p{};
    p.prec = tag; p.M = N; p.N = 9 * C; p.K = l.ax.Mp;
    p.A = dyT; p.B = xT; p.C = dw; p.c_dtype = dwdt;
    if(tag == QSYNC_INT8) { p.s0 = sdy; p.s1 = sx; p.acc_dump = acc_dump_opt; }
    p.b_remap_C = C; p.b_remap_shift = static_cast<int64_t>(l.ax.Wp) * esz;
    return hip_status(launch_gemm(p, l.plan, static_cast<uint8_t*>(workspace) + l.off_part, st));
}

size_t qsync_conv3x3_prepare_weights_workspace_bytes(int64_t N, int64_t C)
{
    if(N <= 0 || C <= 0) return 0;
    return absmax_workspace_bytes(N, 9 * C, kPerCol) + static_cast<size_t>(9 * N * C);
}

int qsync_conv3x3_prepare_weights(const void* w, int wdt, int64_t N, int64_t C, int bits, float* sw, float* iw, void* wq,
                                  float* swb, float* iwb, void* wflip, void* workspace, size_t workspace_bytes,
                                  void* stream)
{
    if(!w || !sw || !iw || !wq || !swb || !iwb || !wflip) return QSYNC_ERR_NULL;
    if(!is_float_dtype(wdt)) return QSYNC_ERR_BAD_ENUM;
    if(N < 0 || C < 0 || C > (1 << 20) || !count_ok(N, 9 * C)) return QSYNC_ERR_BAD_SHAPE;
    if(bits < 2 || bits > 8) return QSYNC_ERR_UNSUPPORTED;
    if(N == 0 || C == 0) return QSYNC_OK;
    if(!workspace || workspace_bytes < qsync_conv3x3_prepare_weights_workspace_bytes(N, C)) return QSYNC_ERR_WORKSPACE;
    if(!aligned16(workspace)) return QSYNC_ERR_ALIGN;
    const float qmax = static_cast<float>((1 << (bits - 1)) - 1);
    return hip_status(launch_conv3x3_prepare_weights(w, wdt == QSYNC_F32 ? kF32 : kF16, N, C, qmax, sw, iw, swb, iwb,
                                                     static_cast<int8_t*>(wq), static_cast<int8_t*>(wflip), workspace,
                                                     static_cast<hipStream_t>(stream)));
}

int qsync_probe_mfma(int tag, int random_operands, int iters, void* out, double* ops_out, void* stream)
{
    if(!out) return QSYNC_ERR_NULL;
    if(tag != QSYNC_INT8 && tag != QSYNC_FP16) return QSYNC_ERR_BAD_ENUM;
    if(iters < 1 || iters > (1 << 24)) return QSYNC_ERR_BAD_SHAPE;
    iters = (iters + 3) / 4 * 4;               // the kernel runs whole groups of four iterations
    if(random_operands < 0 || random_operands > 2) return QSYNC_ERR_BAD_ENUM;
    if(ops_out)   // a 32x32x32 int8 instruction is 2*32*32*32 operations, the 32x32x16 binary16 one half of that
        *ops_out = static_cast<double>(kProbeBlocks) * 4.0 * 4.0 * iters * (tag == QSYNC_INT8 ? 65536.0 : 32768.0);
    return hip_status(launch_probe_mfma(tag, random_operands, iters, out, static_cast<hipStream_t>(stream)));
}

void qsync_debug_set_gemm_tile(int tile) { set_gemm_tile_override(tile); }
void qsync_debug_set_gemm_persistent(int mode) { set_gemm_persistent_mode(mode); }

static int conv3x3_fwd_impl(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N, const void* xq,
                            const float* sx, const void* wq, const float* sw, int wgran, const float* bias_opt, void* y,
                            int ydt, int32_t* acc_dump_opt, float* y_amax_opt, void* stream)
{
    if(!xq || !wq || !y) return QSYNC_ERR_NULL;
    if(!is_tag(tag) || !is_float_dtype(ydt)) return QSYNC_ERR_BAD_ENUM;
    if(tag == QSYNC_INT8)
    {
        if(!sx || !sw) return QSYNC_ERR_NULL;
        if(!is_gran(wgran)) return QSYNC_ERR_BAD_ENUM;
    }
    if(nimg < 0 || H < 0 || W < 0 || C < 0 || N < 0 || H > 65535 || W > 65535 || C > (1 << 20) || N > (int64_t(1) << 31))
        return QSYNC_ERR_BAD_SHAPE;
    if(tag == QSYNC_FP32) return QSYNC_ERR_UNSUPPORTED;
    if(tag == QSYNC_INT8 && wgran == QSYNC_PER_COL) return QSYNC_ERR_UNSUPPORTED;
    if(tag != QSYNC_INT8 && acc_dump_opt) return QSYNC_ERR_UNSUPPORTED;
    const int64_t esz = tag == QSYNC_INT8 ? 1 : 2;
    if(H > 0 && W > 0 && C > 0 && nimg > ((int64_t(1) << 31) - 1) / (H * W * C * esz)) return QSYNC_ERR_BAD_SHAPE;
    const int64_t M = nimg * H * W;
    if(!count_ok(M, N) || !count_ok(N, 9 * C)) return QSYNC_ERR_BAD_SHAPE;
    if((C * esz) % 16 != 0 || !aligned16(xq) || !aligned16(wq)) return QSYNC_ERR_ALIGN;
    if(M == 0 || N == 0) return QSYNC_OK;
    const GemmPlan plan = plan_gemm(tag, M, N, 9 * C, -1, -1, /*allow_split=*/false);
    GemmProblem p{};
    p.prec = tag; p.M = M; p.N = N; p.K = 9 * C;
    p.A = xq; p.B = wq; p.C = y; p.c_dtype = ydt;
    p.conv_H = static_cast<int>(H); p.conv_W = static_cast<int>(W); p.conv_C = C;
    if(tag == QSYNC_INT8)
    {
        p.s0 = sx;
        if(wgran == QSYNC_PER_TENSOR) p.s1 = sw; else p.col_scale = sw;
        p.acc_dump = acc_dump_opt;
    }
    p.col_bias = bias_opt;
    p.out_amax_bits = reinterpret_cast<unsigned int*>(y_amax_opt);
    return hip_status(launch_gemm(p, plan, nullptr, static_cast<hipStream_t>(stream)));
}

int qsync_conv3x3_fwd(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N, const void* xq,
                      const float* sx, const void* wq, const float* sw, int wgran, const float* bias_opt, void* y,
                      int ydt, int32_t* acc_dump_opt, void* stream)
{
    return conv3x3_fwd_impl(tag, nimg, H, W, C, N, xq, sx, wq, sw, wgran, bias_opt, y, ydt, acc_dump_opt, nullptr, stream);
}

int qsync_conv3x3_fwd_amax(int tag, int64_t nimg, int64_t H, int64_t W, int64_t C, int64_t N, const void* xq,
                           const float* sx, const void* wq, const float* sw, int wgran, const float* bias_opt, void* y,
                           int ydt, int32_t* acc_dump_opt, float* y_amax, void* stream)
{
    if(!y_amax) return QSYNC_ERR_NULL;
    if((reinterpret_cast<uintptr_t>(y_amax) & 3u) != 0) return QSYNC_ERR_ALIGN;
    return conv3x3_fwd_impl(tag, nimg, H, W, C, N, xq, sx, wq, sw, wgran, bias_opt, y, ydt, acc_dump_opt, y_amax, stream);
}

int qsync_conv3x3_wflip(const void* w, int wdt, int64_t N, int64_t C, void* wflip, void* stream)
{
    if(!w || !wflip) return QSYNC_ERR_NULL;
    if(wdt != QSYNC_I8 && wdt != QSYNC_F16) return QSYNC_ERR_BAD_ENUM;
    if(N < 0 || C < 0 || !count_ok(N, 9 * C)) return QSYNC_ERR_BAD_SHAPE;
    if(w == wflip) return QSYNC_ERR_UNSUPPORTED;
    return hip_status(launch_conv3x3_wflip(w, wdt == QSYNC_I8 ? 1 : 2, N, C, wflip, static_cast<hipStream_t>(stream)));
}

int qsync_im2col3x3_i8(const void* xq, int64_t nimg, int64_t H, int64_t W, int64_t C, void* a_opt, void* aT_opt,
                       void* stream)
{
    if(!xq || (!a_opt && !aT_opt)) return QSYNC_ERR_NULL;
    if(nimg < 0 || H < 0 || W < 0 || C < 0 || H > (1 << 15) || W > (1 << 15) || C > (1 << 15)) return QSYNC_ERR_BAD_SHAPE;
    if(nimg > 0 && H > 0 && W > 0 && nimg > (int64_t(1) << 40) / (H * W)) return QSYNC_ERR_BAD_SHAPE;
    const int64_t M = nimg * H * W;
    if(M == 0 || C == 0) return QSYNC_OK;
    if(C % 16 != 0) return QSYNC_ERR_UNSUPPORTED;
    if(((M + 511) / 512) * ((9 * C / 16 + 7) / 8) >= (int64_t(1) << 31)) return QSYNC_ERR_BAD_SHAPE;
    if(!aligned16(xq) || (a_opt && !aligned16(a_opt)) || (aT_opt && (!aligned16(aT_opt) || M % 16 != 0))) return QSYNC_ERR_ALIGN;
    return hip_status(launch_im2col3x3_i8(static_cast<const int8_t*>(xq), nimg, static_cast<int>(H), static_cast<int>(W),
                                          static_cast<int>(C), static_cast<int8_t*>(a_opt), static_cast<int8_t*>(aT_opt),
                                          static_cast<hipStream_t>(stream)));
}

int qsync_dequantize(const void* a, int adt, int64_t rows, int64_t cols, int64_t ld, const float* row_scale_opt,
                     const float* col_scale_opt, float tensor_scale, const float* tensor_scale_dev_opt,
                     const float* col_bias_opt, void* y, int ydt, void* stream)
{
    if(!a || !y) return QSYNC_ERR_NULL;
    if((adt != QSYNC_I32 && adt != QSYNC_I8) || !is_float_dtype(ydt)) return QSYNC_ERR_BAD_ENUM;
    if(!count_ok(rows, cols) || ld < cols || !count_ok(rows, ld)) return QSYNC_ERR_BAD_SHAPE;
    if(rows == 0 || cols == 0) return QSYNC_OK;
    return hip_status(launch_dequantize(a, adt == QSYNC_I32 ? kI32 : kI8, rows, cols, ld, row_scale_opt, col_scale_opt,
                                        tensor_scale, tensor_scale_dev_opt, col_bias_opt, y, ydt,
                                        static_cast<hipStream_t>(stream)));
}

}  // extern "C"
