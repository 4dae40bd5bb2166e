/*
 * qsync_debug.h - measurement and test hooks of libqsync.  NOT part of the operator ABI (qsync.h): nothing
 * here is needed to run the operators, and a production caller has no reason to include this file.
 */
#ifndef QSYNC_DEBUG_H
#define QSYNC_DEBUG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * qsync_probe_mfma - measurement probe, not part of the operator path: launches a kernel that issues
 * `iters` x 4 back-to-back 32x32 matrix instructions per wavefront on register operands (512 workgroups
 * of 4 wavefronts, no memory traffic), so that a caller can time the matrix-instruction rate this GPU
 * sustains: with constant operands (random_operands = 0) and with pseudo-random operand values
 * (random_operands = 1; power management lowers the clock when operand bits toggle); random_operands = 2
 * is mode 1 with the second binary16 operand drawn from the subnormal range (same as 1 for QSYNC_INT8).
 * tag QSYNC_INT8 (v_mfma_i32_32x32x32_i8) or QSYNC_FP16 (v_mfma_f32_32x32x16_f16); 1 <= iters <= 2^24,
 * rounded up to a multiple of 4.
 * out      device scratch, at least 512 KiB (one 4-byte word per thread).
 * ops_out  host pointer or NULL: receives the number of arithmetic operations the launch performs.
 * The caller times the launch on `stream`.
 */
int qsync_probe_mfma(int tag, int random_operands, int iters, void* out, double* ops_out, void* stream);

/*
 * qsync_debug_set_gemm_tile - for tests and tuning runs: pin the tile shape of the MFMA GEMM
 * (0: 256x256, 1: 128x128, 2: 64x64) for every later call made by the calling thread, -1 (or any other value)
 * returns the choice to the planner.  Workspace sizes reported afterwards follow the pinned tile.
 * The override is per calling thread (a thread sees only its own setting), so it never races with other
 * threads that use the library; it is the only state the library keeps besides a per-process note of which
 * kernels already had their dynamic-LDS limit raised.
 */
void qsync_debug_set_gemm_tile(int tile);

/*
 * qsync_debug_set_gemm_persistent - for tests and tuning runs, per calling thread: 0 = never launch the
 * persistent 256x256 GEMM kernel, 1 = launch it whenever a problem is eligible (binary16 output, M and N
 * multiples of 256, operand rows multiples of 256 bytes, no accumulator dump, no output maximum), any other
 * value = the default, which is 0 as well: the kernel is opt-in.  Results are the same bits either way for
 * int8 operands; binary16 operands sum in the same order, too.
 */
void qsync_debug_set_gemm_persistent(int mode);

#ifdef __cplusplus
}
#endif
#endif /* QSYNC_DEBUG_H */
