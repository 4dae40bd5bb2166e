// Internal launch interface between the C ABI (api.hip) and the gfx950 kernels.
// Every launcher assumes its arguments were validated by the caller; each returns the
// hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace qsync {

enum Dtype { kF32 = 0, kF16 = 1, kI8 = 2, kI32 = 3 };
enum Gran { kPerTensor = 0, kPerRow = 1, kPerCol = 2 };
enum Round { kNearest = 0, kStochastic = 1, kFloor = 2 };

// ---- absmax / scale -------------------------------------------------------------------
constexpr int kAbsmaxMaxBlocks = 2048;  // per-tensor stage-1 partials
constexpr int kColParts = 512;          // most stage-1 partials per column of a per-column reduction
size_t absmax_workspace_bytes(int64_t rows, int64_t cols, int gran);
// Library-owned scratch (a file-scope device array, one copy per GPU) for qsync_absmax_scale_static: large enough
// for a per-tensor pass with fused column sums over kStaticMaxCols columns.
constexpr int64_t kStaticMaxCols      = 4096;
constexpr size_t  kStaticScratchBytes = 256 + sizeof(float) * (2 * kAbsmaxMaxBlocks + static_cast<size_t>(kColParts) * kStaticMaxCols);
// device address of the calling thread's current GPU's copy (looked up on first use per device)
hipError_t static_scratch(void** ptr_out);
hipError_t launch_scale_from_amax(float* amax, float qmax, float* scale, float* inv_scale, int consume, hipStream_t st);
hipError_t launch_absmax_scale(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int gran,
                               float qmax, float* scale, float* inv_scale, float* amax_opt,
                               float* colsum_opt /* per-tensor only: fused column sums */,
                               float* sumsq_opt /* per-tensor only: squared norm */,
                               void* workspace /* zero before first use; left zero where it must be */,
                               hipStream_t stream);

// ---- quantize / cast / copy (+ transpose) ---------------------------------------------
hipError_t launch_absmax_quantize(const void* x, int xdt, int64_t rows, int64_t cols, int qmax, int rnd, uint64_t seed,
                                  uint64_t offset, float* scale, float* inv_scale, float* amax_opt, int8_t* q, int8_t* qT,
                                  void* workspace, unsigned int poll_limit, hipStream_t stream);
hipError_t launch_quantize_int8(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int qmax,
                                int gran, int rnd, uint64_t seed, uint64_t offset, const float* inv_scale,
                                int8_t* q, int8_t* qT, hipStream_t stream);
hipError_t launch_convert(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int outdt,
                          void* q, void* qT, hipStream_t stream);
// binary32 -> binary16 with stochastic rounding of the mantissa to `mantissa_bits` (7..10) bits
hipError_t launch_convert_sr(const float* x, int64_t rows, int64_t cols, int64_t ld, int mantissa_bits,
                             uint64_t seed, uint64_t offset, void* q, void* qT, hipStream_t stream);

// ---- standalone dequantize, column sums -----------------------------------------------
hipError_t launch_dequantize(const void* a, int adt, int64_t rows, int64_t cols, int64_t ld,
                             const float* row_scale, const float* col_scale, float tensor_scale,
                             const float* tensor_scale_dev, const float* col_bias, void* y, int ydt,
                             hipStream_t stream);
// 3x3 / stride 1 / pad 1 patches of an int8 NHWC tensor: a [M, 9C] and/or aT [9C, M], M = nimg*H*W
hipError_t launch_prepare_weights(const void* w, int wdt, int64_t N, int64_t K, float qmax, float* sw, float* iw,
                                  float* aw_opt, int8_t* wq, float* swb, float* iwb, int8_t* wqbT, void* workspace,
                                  hipStream_t stream);
hipError_t launch_conv3x3_prepare_weights(const void* w, int wdt, int64_t N, int64_t C, float qmax, float* sw, float* iw,
                                          float* swb, float* iwb, int8_t* wq, int8_t* wflip, void* workspace,
                                          hipStream_t stream);
hipError_t launch_conv3x3_wflip(const void* w, int elem_bytes, int64_t N, int64_t C, void* wflip, hipStream_t stream);
// padded pixel axis of the convolution's weight-gradient operands (see conv_padded_transpose_kernel)
struct ConvPaddedAxis { int Wp; int64_t Mp; };
ConvPaddedAxis conv_padded_axis(int64_t nimg, int H, int W);
// in [nimg*H*W, Ch] of 1- or 2-byte elements (Ch * elem_bytes % 16 == 0) -> out [copies][Ch][Mp];
// copies 3 (displaced by -1, 0, +1 pixel) or 1; margin_bytes > 0 (a multiple of 16): that many bytes in front of
// and behind `out` are cleared as well
hipError_t launch_conv_padded_transpose(const void* in, int elem_bytes, int64_t nimg, int H, int W, int Ch, int copies,
                                        void* out, int margin_bytes, hipStream_t stream);
hipError_t launch_im2col3x3_i8(const int8_t* xq, int64_t nimg, int H, int W, int C, int8_t* a, int8_t* aT,
                               hipStream_t stream);
hipError_t launch_zero_f32(float* p, int64_t n, hipStream_t stream);
// out[c, r] = in[r, c] for int8 codes, any shape (16-byte patches when rows and cols are multiples of 16)
hipError_t launch_transpose_i8(const int8_t* in, int64_t rows, int64_t cols, int8_t* out, hipStream_t stream);
size_t colsum_workspace_bytes(int64_t rows, int64_t cols);
hipError_t launch_colsum(const void* x, int xdt, int64_t rows, int64_t cols, float* out, float* workspace,
                         hipStream_t stream);

// ---- GEMM  C[M,N] = epilogue( sum_k A[M,k] B[N,k] ) ------------------------------------
// epilogue(acc) = float(acc) * (s0 * s1 * col_scale[n]) + col_bias[n]; absent factors are 1 / 0.
struct GemmProblem {
    int         prec;       // 8: int8 operands, int32 accumulate; 16: binary16, fp32; 32: fp32
    int64_t     M, N, K;    // K in elements
    const void* A;          // [M,K] packed
    const void* B;          // [N,K] packed
    void*       C;          // [M,N] packed, fp32 or binary16
    int         c_dtype;    // kF32 | kF16
    const float* s0;        // device scalars or nullptr
    const float* s1;
    const float* col_scale; // [N] or nullptr
    const float* col_bias;  // [N] or nullptr
    int32_t*    acc_dump;   // [M,N] raw int32 accumulators (prec 8 only) or nullptr
    // conv_H > 0: A is an NHWC tensor [M = images*conv_H*conv_W, conv_C] and the GEMM runs over its
    // 3x3 / stride 1 / pad 1 patch matrix [M, K = 9*conv_C] (k = (kh, kw, c)), formed on the fly.
    int         conv_H = 0, conv_W = 0;
    int64_t     conv_C = 0;
    // b_remap_C > 0 (int8 and binary16): N = 9*b_remap_C logical rows (tap, c) of B are the rows (tap%3)*b_remap_C + c of a
    // [3*b_remap_C, K] matrix, read with the K axis displaced by (tap/3 - 1)*b_remap_shift bytes (a multiple of
    // 16, at most 1024); that many bytes in front of and behind the matrix must be readable.
    int64_t     b_remap_C = 0, b_remap_shift = 0;
    // tn (int8 only): A is [K, M] and B is [K, N], row-major with the contraction axis as rows (K % 128 == 0,
    // M % 16 == 0, N % 16 == 0): C[m,n] = sum_k A[k,m] B[k,n] without transposed copies of the operands
    bool        tn = false;
    // optional device word holding a running maximum of |C| as stored (bit pattern of a non-negative fp32);
    // raised by the epilogue (by the reduction pass when K is split)
    unsigned int* out_amax_bits = nullptr;
    // optional int8 codes of C as stored, [M][N]: clamp(round(C * out_code_inv[0]), -out_code_qmax, out_code_qmax)
    // with the quantizer's arithmetic (round to nearest even); out_code_inv is a device scalar
    void*        out_codes = nullptr;
    const float* out_code_inv = nullptr;
    int          out_code_qmax = 127;
};

// longest operand row (contraction axis) in bytes the MFMA GEMM addresses: 32-bit lane offsets span 255 rows
constexpr int64_t kGemmMaxRowBytes = int64_t(16) << 20;

struct GemmPlan {
    int     tile;          // index into the tile table (see gemm_mfma.hip)
    int     splits;        // split-K factor (1 = epilogue fused in the GEMM kernel)
    size_t  workspace;     // bytes needed for split-K partials
};
// force_tile / force_splits < 0 leave the choice to the heuristic; tn: plan for GemmProblem::tn operands.
GemmPlan plan_gemm(int prec, int64_t M, int64_t N, int64_t K, int force_tile = -1, int force_splits = -1,
                   bool allow_split = true, bool tn = false);
// tile >= 0 pins the tile shape of every later plan (tests, tuning); -1 returns the choice to the planner.
void set_gemm_tile_override(int tile);
// 1: launch the persistent 256x256 kernel whenever a problem is eligible; anything else: never (the default)
void set_gemm_persistent_mode(int mode);
hipError_t launch_gemm(const GemmProblem& p, const GemmPlan& plan, void* workspace, hipStream_t stream);

// ---- measurement probe (probe.hip): matrix instructions on register operands, no memory traffic
constexpr int kProbeBlocks = 512;       // workgroups of 4 wavefronts, 4 matrix instructions per wavefront and iteration
hipError_t launch_probe_mfma(int prec, int operand_mode, int iters, void* out, hipStream_t stream);

}  // namespace qsync
