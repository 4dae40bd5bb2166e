// Device helpers shared by the gfx950 kernels: wave reductions, 16-byte vector access,
// the Philox4x32-10 block function and the scalar fixed-point quantizer.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace qsync {

constexpr int kWaveSize = 64;

__device__ __forceinline__ float wave_reduce_max(float v)
{
#pragma unroll
    for(int off = kWaveSize / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWaveSize));
    return v;
}

__device__ __forceinline__ float wave_reduce_sum(float v)
{
#pragma unroll
    for(int off = kWaveSize / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWaveSize);
    return v;
}

// Block-wide maximum for blocks of up to 1024 threads; the result is valid in thread 0.
__device__ __forceinline__ float block_reduce_max(float v, float* lds /* >= 16 floats */)
{
    v = wave_reduce_max(v);
    const int lane = threadIdx.x % kWaveSize, wave = threadIdx.x / kWaveSize;
    if(lane == 0) lds[wave] = v;
    __syncthreads();
    if(threadIdx.x == 0)
    {
        const int nw = (blockDim.x + kWaveSize - 1) / kWaveSize;
        for(int i = 1; i < nw; ++i) v = fmaxf(v, lds[i]);
    }
    return v;
}

// Block-wide sum in a fixed order (wave shuffles, then the wave sums in order); valid in thread 0.
__device__ __forceinline__ float block_reduce_sum(float v, float* lds /* >= 16 floats */)
{
    v = wave_reduce_sum(v);
    const int lane = threadIdx.x % kWaveSize, wave = threadIdx.x / kWaveSize;
    if(lane == 0) lds[wave] = v;
    __syncthreads();
    if(threadIdx.x == 0)
    {
        const int nw = (blockDim.x + kWaveSize - 1) / kWaveSize;
        for(int i = 1; i < nw; ++i) v += lds[i];
    }
    return v;
}

// Element access that widens to fp32 (binary16 -> fp32 is exact).
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(__half v) { return __half2float(v); }

// 16 bytes of T as fp32 values.
template <typename T> struct Vec16;
template <> struct Vec16<float>
{
    static constexpr int N = 4;
    __device__ static __forceinline__ void decode(const uint4& r, float (&out)[4])
    {
        out[0] = __uint_as_float(r.x); out[1] = __uint_as_float(r.y);
        out[2] = __uint_as_float(r.z); out[3] = __uint_as_float(r.w);
    }
    __device__ static __forceinline__ void load(const float* p, float (&out)[4])
    {
        decode(*reinterpret_cast<const uint4*>(p), out);
    }
};
template <> struct Vec16<__half>
{
    static constexpr int N = 8;
    __device__ static __forceinline__ void load(const __half* p, float (&out)[8])
    {
        decode(*reinterpret_cast<const uint4*>(p), out);
    }
    __device__ static __forceinline__ void decode(const uint4& raw, float (&out)[8])
    {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for(int i = 0; i < 4; ++i)
        {
            out[2 * i]     = __half2float(__ushort_as_half(static_cast<unsigned short>(w[i] & 0xFFFFu)));
            out[2 * i + 1] = __half2float(__ushort_as_half(static_cast<unsigned short>(w[i] >> 16)));
        }
    }
};

// Philox4x32 with ten rounds (Salmon et al., SC'11).  One round maps
// (c0,c1,c2,c3) -> (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)); the key
// advances by the Weyl constants.  The key is wave-uniform here, so its schedule runs on
// the scalar unit.
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for(int r = 0; r < 10; ++r)
    {
        const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c.x;
        const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c.z;
        uint4 n;
        n.x = static_cast<uint32_t>(p1 >> 32) ^ c.y ^ k0;
        n.y = static_cast<uint32_t>(p1);
        n.z = static_cast<uint32_t>(p0 >> 32) ^ c.w ^ k1;
        n.w = static_cast<uint32_t>(p0);
        c = n;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c;
}

// The Philox block of the 8-element group `group` of a tensor: counter = offset + group as a
// 128-bit integer (offset and group are 64-bit, so only a carry reaches word 2).
__device__ __forceinline__ uint4 philox_group(uint64_t seed, uint64_t offset, uint64_t group)
{
    const uint64_t lo = offset + group;
    uint4 c;
    c.x = static_cast<uint32_t>(lo);
    c.y = static_cast<uint32_t>(lo >> 32);
    c.z = lo < group ? 1u : 0u;
    c.w = 0u;
    return philox4x32_10(c, static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32));
}

// 16-bit draw number `slot` (0..7) of a Philox block: word slot/2, low half first.
__device__ __forceinline__ uint32_t philox_draw16(const uint4& blk, int slot)
{
    const uint32_t w = (slot >> 1) == 0 ? blk.x : (slot >> 1) == 1 ? blk.y : (slot >> 1) == 2 ? blk.z : blk.w;
    return (slot & 1) ? (w >> 16) : (w & 0xFFFFu);
}

// Fixed-point code of one value: clamp(round(x * inv), -qmax, qmax).  RND is a qsync::Round.
// The product is a single fp32 multiply.  Stochastic rounding: the value rounds up iff
// u16 < floor(residual * 2^16) with residual = x*inv - floor(x*inv).  It is evaluated in 16.16 fixed point:
// t = floor(x*inv * 2^16) is exact (a power-of-two scaling), floor(x*inv) = t >> 16 and floor(residual * 2^16) =
// t & 0xFFFF, so "floor + (u16 < low half)" is the carry of t + (65535 - u16) into bit 16.  Clamping t to
// +-qmax * 2^16 first is the clamp of the code (a clamped t has a zero low half) and keeps the sum inside 32 bits.
template <int RND>
__device__ __forceinline__ int quantize_code(float x, float inv, int qmax, uint32_t u16)
{
    const float v = __fmul_rn(x, inv);
    int         c;
    if(RND == 0) c = static_cast<int>(rintf(v));
    else if(RND == 2) c = static_cast<int>(floorf(v));
    else
    {
        int       t   = static_cast<int>(floorf(__fmul_rn(v, 65536.0f)));     // saturates; NaN -> 0
        const int lim = qmax << 16;
        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(t) : "v"(t), "v"(-lim), "v"(lim));
        return (t + static_cast<int>(65535u - u16)) >> 16;
    }
    return min(max(c, -qmax), qmax);
}

}  // namespace qsync
