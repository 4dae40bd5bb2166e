// FP32 GEMM for the FP32 precision tag:  C[M,N] = sum_k A[m,k] * B[n,k] (* scale) + bias.
// The paper leaves FP32 operators untouched; this is the plain fp32 product (k ascending,
// fp32 fused multiply-add) on the vector ALUs, LDS-tiled 64x64x16 with a 4x4 register block per
// lane.  It is a correctness path: the matrix cores are used by the INT8 and FP16 tags.
#include "device_utils.h"
#include "kernels.h"

namespace qsync {

namespace {

constexpr int kT  = 64;   // tile edge
constexpr int kBK = 16;   // K step

__global__ __launch_bounds__(256) void gemm_f32_nt_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                          int64_t M, int64_t N, int64_t K, void* C, int c_is_f16,
                                                          const float* s0, const float* s1,
                                                          const float* __restrict__ col_scale,
                                                          const float* __restrict__ col_bias, int64_t tiles_n,
                                                          unsigned int* amax_bits)
{
    __shared__ float As[kBK][kT + 1];
    __shared__ float Bs[kBK][kT + 1];
    const int64_t tm = blockIdx.x / tiles_n, tn = blockIdx.x - tm * tiles_n;
    const int64_t m0 = tm * kT, n0 = tn * kT;
    const int     tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    float         acc[4][4] = {};
    for(int64_t k0 = 0; k0 < K; k0 += kBK)
    {
#pragma unroll
        for(int i = 0; i < 4; ++i)
        {
            const int     idx = tid + 256 * i, row = idx / kBK, kk = idx % kBK;
            const int64_t k   = k0 + kk;
            As[kk][row] = (m0 + row < M && k < K) ? A[(m0 + row) * K + k] : 0.0f;
            Bs[kk][row] = (n0 + row < N && k < K) ? B[(n0 + row) * K + k] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for(int kk = 0; kk < kBK; ++kk)
        {
            float a[4], b[4];
#pragma unroll
            for(int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for(int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for(int i = 0; i < 4; ++i)
#pragma unroll
                for(int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    unsigned int run = 0u;     // maximum of |C| as stored, as fp32 bits
    const unsigned int seen = amax_bits ? __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
    float alpha = 1.0f;
    if(s0) alpha *= *s0;
    if(s1) alpha *= *s1;
#pragma unroll
    for(int i = 0; i < 4; ++i)
    {
        const int64_t row = m0 + ty * 4 + i;
        if(row >= M) continue;
#pragma unroll
        for(int j = 0; j < 4; ++j)
        {
            const int64_t col = n0 + tx * 4 + j;
            if(col >= N) continue;
            const float f = alpha * (col_scale ? col_scale[col] : 1.0f);
            const float y = acc[i][j] * f + (col_bias ? col_bias[col] : 0.0f);
            float stored = y;
            if(c_is_f16)
            {
                const __half h = __float2half_rn(y);
                static_cast<__half*>(C)[row * N + col] = h;
                stored = __half2float(h);
            }
            else
                static_cast<float*>(C)[row * N + col] = y;
            const unsigned int u = __float_as_uint(stored) & 0x7FFFFFFFu;
            run = run > u ? run : u;
        }
    }
    if(amax_bits)
    {   // one atomic maximum per workgroup (As is free: the K loop ended with a barrier)
        unsigned int* slots = reinterpret_cast<unsigned int*>(&As[0][0]);
        slots[tid] = run;
        __syncthreads();
        for(int w = 128; w >= 1; w >>= 1)
        {
            if(tid < w) slots[tid] = slots[tid] > slots[tid + w] ? slots[tid] : slots[tid + w];
            __syncthreads();
        }
        if(tid == 0 && slots[0] > seen) atomicMax(amax_bits, slots[0]);      // `seen` may be stale, never too large
    }
}

}  // namespace

hipError_t launch_gemm_f32(const GemmProblem& p, hipStream_t stream)
{
    const int64_t tiles_m = (p.M + kT - 1) / kT, tiles_n = (p.N + kT - 1) / kT;
    gemm_f32_nt_kernel<<<dim3(static_cast<unsigned>(tiles_m * tiles_n)), dim3(256), 0, stream>>>(
        static_cast<const float*>(p.A), static_cast<const float*>(p.B), p.M, p.N, p.K, p.C, p.c_dtype == kF16, p.s0,
        p.s1, p.col_scale, p.col_bias, tiles_n, p.out_amax_bits);
    return hipGetLastError();
}

}  // namespace qsync
