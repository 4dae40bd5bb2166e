// Measurement probe: the matrix-instruction rate this GPU sustains with no memory traffic at all.
// 512 workgroups of 4 wavefronts issue back-to-back 32x32 matrix instructions on register operands
// (four independent accumulators per wavefront).  The sustained rate depends on the operand values:
// with constant operands the instruction stream runs at the clock the published peak assumes, with
// varying operands (random codes, as in a quantized GEMM) power management lowers the clock.  The
// benchmark reports both beside the GEMM's own rate.
#include "kernels.h"

namespace qsync {

namespace {

typedef int      v4i32 __attribute__((ext_vector_type(4)));
typedef int      v16i32 __attribute__((ext_vector_type(16)));
typedef float    v16f32 __attribute__((ext_vector_type(16)));
typedef _Float16 v8f16 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ unsigned mix(unsigned h)
{
    h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15; h *= 2654435761u; h ^= h >> 16;
    return h;
}

template <bool RANDOM>
__global__ __launch_bounds__(256) void probe_i8_kernel(int iters, int* out)
{
    v16i32 acc[4];
    v4i32  a[4], b[4];
#pragma unroll
    for(int i = 0; i < 4; ++i)
    {
#pragma unroll
        for(int v = 0; v < 16; ++v) acc[i][v] = 0;
#pragma unroll
        for(int j = 0; j < 4; ++j)
        {
            a[i][j] = RANDOM ? static_cast<int>(mix(threadIdx.x * 131u + i * 17u + j * 3u + blockIdx.x * 7919u)) : 0x01010101;
            b[i][j] = RANDOM ? static_cast<int>(mix(threadIdx.x * 733u + i * 19u + j * 5u + blockIdx.x * 104729u + 99u)) : 0x01010101;
        }
    }
    for(int it = 0; it < iters; it += 4)      // four iterations per trip: every operand index is static
#pragma unroll
        for(int r = 0; r < 4; ++r)
#pragma unroll
            for(int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[(i + r) & 3], acc[i], 0, 0, 0);
    int s = 0;
#pragma unroll
    for(int i = 0; i < 4; ++i)
#pragma unroll
        for(int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

template <bool RANDOM>
__global__ __launch_bounds__(256) void probe_f16_kernel(int iters, float* out, float b_step)
{
    v16f32 acc[4];
    v8f16  a[4], b[4];
#pragma unroll
    for(int i = 0; i < 4; ++i)
    {
#pragma unroll
        for(int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
#pragma unroll
        for(int j = 0; j < 8; ++j)
        {
            const unsigned ha = mix(threadIdx.x * 131u + i * 17u + j * 3u + blockIdx.x * 7919u);
            const unsigned hb = mix(threadIdx.x * 733u + i * 19u + j * 5u + 99u);
            a[i][j] = RANDOM ? static_cast<_Float16>((static_cast<int>(ha % 2001u) - 1000) * 0.001f) : static_cast<_Float16>(1.0f);
            b[i][j] = RANDOM ? static_cast<_Float16>((static_cast<int>(hb % 2001u) - 1000) * b_step) : static_cast<_Float16>(1.0f);
        }
    }
    for(int it = 0; it < iters; it += 4)
#pragma unroll
        for(int r = 0; r < 4; ++r)
#pragma unroll
            for(int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[(i + r) & 3], acc[i], 0, 0, 0);
    float s = 0.0f;
#pragma unroll
    for(int i = 0; i < 4; ++i)
#pragma unroll
        for(int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_probe_mfma(int prec, int operand_mode, int iters, void* out, hipStream_t st)
{
    const bool  random_operands = operand_mode != 0;
    // binary16 second operand: multiples of b_step up to 1000 steps; mode 2 keeps most of them below the
    // smallest normal binary16 (6.1e-5)
    const float b_step = operand_mode == 2 ? 2e-8f : 1e-3f;
    const dim3 grid(kProbeBlocks), block(256);
    if(prec == 8)
    {
        if(random_operands) probe_i8_kernel<true><<<grid, block, 0, st>>>(iters, static_cast<int*>(out));
        else                probe_i8_kernel<false><<<grid, block, 0, st>>>(iters, static_cast<int*>(out));
    }
    else
    {
        if(random_operands) probe_f16_kernel<true><<<grid, block, 0, st>>>(iters, static_cast<float*>(out), b_step);
        else                probe_f16_kernel<false><<<grid, block, 0, st>>>(iters, static_cast<float*>(out), b_step);
    }
    return hipGetLastError();
}

}  // namespace qsync
