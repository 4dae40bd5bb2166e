// HBM-bound kernels of the quantized-operator path for gfx950: absmax + scale (two-stage
// reduction), INT8 quantize with optional transposed copy, precision cast / copy with
// optional transpose, standalone dequantize, and column sums (bias gradient).
//
// All of them stream their input once with 16-byte loads per lane when alignment allows,
// reduce at wavefront level with cross-lane shuffles and at block level through LDS, and
// fall back to scalar element access for shapes or pointers that do not meet the vector
// path's alignment rule.
#include "device_utils.h"
#include "kernels.h"

#include <mutex>

#include <type_traits>

namespace qsync {

namespace {

constexpr int kBlock = 256;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

__device__ __forceinline__ void write_scale(float amax, float qmax, float* scale, float* inv_scale,
                                            float* amax_opt, int64_t i)
{
    float s = 1.0f, iv = 1.0f;
    if(amax != 0.0f)
    {
        s  = __fdiv_rn(amax, qmax);
        iv = __fdiv_rn(qmax, amax);
    }
    scale[i]     = s;
    inv_scale[i] = iv;
    if(amax_opt) amax_opt[i] = amax;
}

// Running maximum of |x| over 16-byte vectors.  binary16 magnitudes order like their bit
// patterns with the sign bit cleared, so for binary16 the maximum runs on packed 16-bit
// integers (two elements per VALU operation) and is widened to fp32 once at the end.
typedef unsigned short us2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_absmax_u16(uint32_t m, uint32_t w)
{
    const us2_t a = __builtin_bit_cast(us2_t, m), b = __builtin_bit_cast(us2_t, w & 0x7FFF7FFFu);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, b));
}
__device__ __forceinline__ float half_bits_to_f32(uint32_t h) { return __half2float(__ushort_as_half(static_cast<unsigned short>(h))); }

template <typename T> struct RunMax;
template <> struct RunMax<float>
{
    float m = 0.0f;
    __device__ __forceinline__ void add(const uint4& r)
    {
        m = fmaxf(fmaxf(m, fmaxf(fabsf(__uint_as_float(r.x)), fabsf(__uint_as_float(r.y)))),
                  fmaxf(fabsf(__uint_as_float(r.z)), fabsf(__uint_as_float(r.w))));
    }
    __device__ __forceinline__ void add_scalar(float v) { m = fmaxf(m, fabsf(v)); }
    __device__ __forceinline__ float get() const { return m; }
};
template <> struct RunMax<__half>
{
    uint32_t pk = 0u;
    float    s  = 0.0f;
    __device__ __forceinline__ void add(const uint4& r)
    {
        pk = pk_absmax_u16(pk_absmax_u16(pk, r.x), r.y);
        pk = pk_absmax_u16(pk_absmax_u16(pk, r.z), r.w);
    }
    __device__ __forceinline__ void add_scalar(__half v) { s = fmaxf(s, fabsf(__half2float(v))); }
    __device__ __forceinline__ float get() const
    {
        return fmaxf(s, fmaxf(half_bits_to_f32(pk & 0xFFFFu), half_bits_to_f32(pk >> 16)));
    }
};

// Running sum of squares in fp32 (the squared norm of the indicator statistics).
template <typename T> struct RunSq
{
    float s = 0.0f;
    __device__ __forceinline__ void add(const uint4& r)
    {
        float v[Vec16<T>::N];
        Vec16<T>::decode(r, v);
#pragma unroll
        for(int e = 0; e < Vec16<T>::N; ++e) s = fmaf(v[e], v[e], s);
    }
    __device__ __forceinline__ void add_scalar(T x) { const float v = to_f32(x); s = fmaf(v, v, s); }
};

// The last block folds the per-block sums of squares in block order, in double.  The first `cap`
// partials are fetched by the whole block into LDS, any further ones straight from memory.
__device__ __forceinline__ void fold_sumsq(const float* partial_sq, unsigned int nblocks, float* sumsq, double* lds_d,
                                           unsigned int cap)
{
    for(unsigned int i = threadIdx.x; i < nblocks && i < cap; i += blockDim.x)
        lds_d[i] = static_cast<double>(__hip_atomic_load(partial_sq + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    __syncthreads();
    if(threadIdx.x == 0)
    {
        double t = 0.0;
        for(unsigned int i = 0; i < nblocks; ++i)
            t += i < cap ? lds_d[i]
                         : static_cast<double>(__hip_atomic_load(partial_sq + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        *sumsq = static_cast<float>(t);
    }
}

// ------------------------------------------------------------------ arrival counter
// The per-tensor maximum finishes inside one launch: every block publishes its partial maximum,
// then takes a ticket from an arrival counter; the block that draws the last ticket folds the
// partials (a maximum: the result does not depend on which block that is) and resets the counter
// to zero for the next launch.  The counter lives at the start of the caller's workspace, which
// must be zero before its first use.  Tickets to one address cost about 10 ns each on this
// part, so these kernels run few, large blocks (at most a few hundred).
// Partials are written and read with device-scope atomic accesses (write-through stores, loads
// that bypass the non-coherent cache levels), so no cache-wide flush is needed: a block waits
// until its own partial store has completed, joins its barrier, and only then draws its ticket;
// the last block reads the partials after its ticket has returned.
__device__ __forceinline__ void st_partial(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_partial(const float* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool last_arrival(unsigned int* ctr, unsigned int expected, bool* flag_lds)
{
    __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0): this wavefront's partial stores have completed
    __syncthreads();
    if(threadIdx.x == 0)
    {
        const unsigned int t = atomicAdd(ctr, 1u);
        *flag_lds            = (t == expected - 1u);
    }
    __syncthreads();
    return *flag_lds;
}

// ------------------------------------------------------------------ absmax, per tensor
// Each block folds contiguous pieces of the tensor (BLOCK * 8 sixteen-byte vectors each) into one
// partial maximum; the last block to arrive folds the partials and writes amax, scale and
// inverse scale.  With ctr == nullptr only the partials are written (a second launch folds them).
template <typename T, bool VEC, int BLOCK>
__global__ __launch_bounds__(BLOCK) void absmax_tensor_kernel(const T* __restrict__ x, int64_t rows,
                                                              int64_t cols, int64_t ld, float* partial,
                                                              unsigned int* ctr, float qmax, float* scale,
                                                              float* inv_scale, float* amax_opt, float* partial_sq,
                                                              float* sumsq_opt)
{
    __shared__ float  lds[16];
    __shared__ double lds_d[1024];
    __shared__ bool   flag;
    RunMax<T>         rm;
    RunSq<T>          sq;                 // only when sumsq_opt is given
    const bool        want_sq = sumsq_opt != nullptr;
    const int64_t     n = rows * cols;
    if(VEC)
    {   // contiguous tensor, 16-byte aligned base
        constexpr int E    = Vec16<T>::N;
        constexpr int U    = 8;                       // 16-byte loads in flight per lane
        const int64_t nvec = n / E;
        const int64_t step = static_cast<int64_t>(gridDim.x) * BLOCK * U;
        const uint4*  xv   = reinterpret_cast<const uint4*>(x);
        for(int64_t c = static_cast<int64_t>(blockIdx.x) * BLOCK * U + threadIdx.x; c < nvec; c += step)
        {
            uint4 v[U];
#pragma unroll
            for(int u = 0; u < U; ++u)
            {
                const int64_t idx = c + static_cast<int64_t>(u) * BLOCK;
                v[u] = idx < nvec ? xv[idx] : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for(int u = 0; u < U; ++u) rm.add(v[u]);
            if(want_sq)
            {
#pragma unroll
                for(int u = 0; u < U; ++u) sq.add(v[u]);
            }
        }
        if(blockIdx.x == 0)
            for(int64_t j = nvec * E + threadIdx.x; j < n; j += BLOCK)
            {
                rm.add_scalar(x[j]);
                if(want_sq) sq.add_scalar(x[j]);
            }
    }
    else
    {
        const int64_t stride = static_cast<int64_t>(gridDim.x) * BLOCK;
        for(int64_t i = static_cast<int64_t>(blockIdx.x) * BLOCK + threadIdx.x; i < n; i += stride)
        {
            const int64_t r = i / cols, c = i - r * cols;
            rm.add_scalar(x[r * ld + c]);
            if(want_sq) sq.add_scalar(x[r * ld + c]);
        }
    }
    const float m = block_reduce_max(rm.get(), lds);
    if(threadIdx.x == 0) st_partial(partial + blockIdx.x, m);
    if(want_sq)
    {
        __syncthreads();
        const float bs = block_reduce_sum(sq.s, lds);
        if(threadIdx.x == 0) st_partial(partial_sq + blockIdx.x, bs);
    }
    if(!ctr) return;
    if(!last_arrival(ctr, gridDim.x, &flag)) return;
    if(want_sq)
    {
        fold_sumsq(partial_sq, gridDim.x, sumsq_opt, lds_d, 1024u);
        __syncthreads();
    }
    float mm = 0.0f;
    for(int i = threadIdx.x; i < static_cast<int>(gridDim.x); i += BLOCK) mm = fmaxf(mm, ld_partial(partial + i));
    mm = block_reduce_max(mm, lds);
    if(threadIdx.x == 0)
    {
        write_scale(mm, qmax, scale, inv_scale, amax_opt, 0);
        *ctr = 0u;
    }
}

// Second launch of the two-launch form: one block folds the partials.
__global__ __launch_bounds__(kBlock) void absmax_tensor_finalize_kernel(const float* __restrict__ partial, int n,
                                                                        float qmax, float* scale, float* inv_scale,
                                                                        float* amax_opt)
{
    __shared__ float lds[16];
    float            m = 0.0f;
    for(int i = threadIdx.x; i < n; i += kBlock) m = fmaxf(m, partial[i]);
    m = block_reduce_max(m, lds);
    if(threadIdx.x == 0) write_scale(m, qmax, scale, inv_scale, amax_opt, 0);
}

// Scale and inverse scale from a maximum some other kernel has collected (a GEMM epilogue); `consume` clears the
// word for the next collection.
__global__ void scale_from_amax_kernel(float* amax, float qmax, float* scale, float* inv_scale, int consume)
{
    if(threadIdx.x != 0 || blockIdx.x != 0) return;
    const float m = __hip_atomic_load(amax, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    write_scale(m, qmax, scale, inv_scale, nullptr, 0);
    if(consume) *amax = 0.0f;
}

// ------------------------------------------------------------------ absmax, per row
// WPR wavefronts per row (1 when there are many rows, 4 = the whole block when there are few),
// four 16-byte loads in flight per lane; no second stage.
template <typename T, bool VEC, int WPR>
__global__ __launch_bounds__(kBlock) void absmax_rows_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                             int64_t ld, float qmax, float* scale, float* inv_scale,
                                                             float* amax_opt)
{
    constexpr int RPB = kBlock / kWaveSize / WPR;       // rows per block
    constexpr int TPR = WPR * kWaveSize;                // threads per row
    __shared__ float lds[kBlock / kWaveSize];
    const int     lane = threadIdx.x % kWaveSize, t = threadIdx.x % TPR;
    const int64_t r    = static_cast<int64_t>(blockIdx.x) * RPB + threadIdx.x / TPR;
    RunMax<T>     rm;
    if(r < rows)
    {
        const T* row  = x + r * ld;
        int64_t  done = 0;
        if(VEC)
        {
            constexpr int E    = Vec16<T>::N;
            const int64_t nvec = cols / E;
            const uint4*  rv   = reinterpret_cast<const uint4*>(row);
            for(int64_t i = t; i < nvec; i += 4 * TPR)
            {
                uint4 v[4];
#pragma unroll
                for(int u = 0; u < 4; ++u) v[u] = i + u * TPR < nvec ? rv[i + u * TPR] : make_uint4(0, 0, 0, 0);
#pragma unroll
                for(int u = 0; u < 4; ++u) rm.add(v[u]);
            }
            done = nvec * E;
        }
        for(int64_t c = done + t; c < cols; c += TPR) rm.add_scalar(row[c]);
    }
    float m = wave_reduce_max(rm.get());
    if(WPR > 1)
    {
        if(lane == 0) lds[threadIdx.x / kWaveSize] = m;
        __syncthreads();
        if(t == 0)
        {
            const int w0 = (threadIdx.x / TPR) * WPR;
            for(int w = 1; w < WPR; ++w) m = fmaxf(m, lds[w0 + w]);
        }
    }
    if(t == 0 && r < rows) write_scale(m, qmax, scale, inv_scale, amax_opt, r);
}

// ------------------------------------------------------------------ per-column reductions
// Shared by the per-column absmax (OP_MAX), the column sums of the bias gradient (OP_SUM) and
// their fusion with the tensor-wide absmax (OP_SUMMAX: one pass yields both).
// Stage 1: block (bx, by) reduces rows by*rpb + tr, + gridDim.y*rpb, ... of a strip of tpr*E
// columns, four rows in flight per lane.  Lanes own adjacent columns (one 16-byte vector each
// when VEC); the block's row lanes are folded through LDS, so partial[by][c] holds one value
// per block row; a second launch folds those.  The tensor-wide maximum of OP_SUMMAX is folded
// by the last block of the grid to arrive (ctr != nullptr).
enum { OP_MAX = 0, OP_SUM = 1, OP_SUMMAX = 2 };

struct TensorFinal          // OP_SUMMAX: where the tensor-wide result goes
{
    unsigned int* ctr;      // arrival counter; nullptr: a second launch folds the block maxima
    float         qmax;
    float*        scale;
    float*        inv_scale;
    float*        amax_opt;
    float*        partial_sq;   // per-block sums of squares and their total (indicator statistics), or nullptr
    float*        sumsq_opt;
};

template <typename T, bool VEC, int OP, int BLOCK>
__global__ __launch_bounds__(BLOCK) void colreduce_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                          int64_t ld, int tpr, float* partial, float* partial_max,
                                                          const TensorFinal fin)
{
    constexpr int E = VEC ? Vec16<T>::N : 1;
    constexpr int U = 4;                                    // rows in flight per lane
    __shared__ float lds[BLOCK * E];
    __shared__ float lds_max[16];
    __shared__ bool  flag;
    RunMax<T>        rm;                                    // OP_SUMMAX only
    float            sqv     = 0.0f;                        // OP_SUMMAX with fin.sumsq_opt: sum of squares
    const bool       want_sq = OP == OP_SUMMAX && fin.sumsq_opt != nullptr;
    const int     rpb = BLOCK / tpr;                       // row lanes per block
    const int     tc = threadIdx.x % tpr, tr = threadIdx.x / tpr;
    const int64_t c0  = (static_cast<int64_t>(blockIdx.x) * tpr + tc) * E;
    const int64_t S   = static_cast<int64_t>(gridDim.y) * rpb;
    float    acc[E];
    uint32_t pk[4] = {0u, 0u, 0u, 0u};                      // packed binary16 maxima (VEC, OP_MAX, binary16)
    constexpr bool kPacked = VEC && OP == OP_MAX && sizeof(T) == 2;
#pragma unroll
    for(int e = 0; e < E; ++e) acc[e] = 0.0f;
    if(c0 < cols)
    {
        for(int64_t r = static_cast<int64_t>(blockIdx.y) * rpb + tr; r < rows; r += S * U)
        {
            if(VEC)
            {
                uint4 raw[U];
#pragma unroll
                for(int u = 0; u < U; ++u)
                {
                    const int64_t rr = r + u * S;        // rows past the end contribute zeros (neutral for sum and max)
                    raw[u] = rr < rows ? *reinterpret_cast<const uint4*>(x + rr * ld + c0) : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
                for(int u = 0; u < U; ++u)
                {
                    if(kPacked)
                    {
                        pk[0] = pk_absmax_u16(pk[0], raw[u].x); pk[1] = pk_absmax_u16(pk[1], raw[u].y);
                        pk[2] = pk_absmax_u16(pk[2], raw[u].z); pk[3] = pk_absmax_u16(pk[3], raw[u].w);
                    }
                    else
                    {
                        float v[Vec16<T>::N];
                        Vec16<T>::decode(raw[u], v);
#pragma unroll
                        for(int e = 0; e < E; ++e) acc[e] = OP == OP_MAX ? fmaxf(acc[e], fabsf(v[e])) : acc[e] + v[e];
                        if(OP == OP_SUMMAX) rm.add(raw[u]);
                        if(want_sq)
                        {
#pragma unroll
                            for(int e = 0; e < E; ++e) sqv = fmaf(v[e], v[e], sqv);
                        }
                    }
                }
            }
            else
            {
#pragma unroll
                for(int u = 0; u < U; ++u)
                {
                    const int64_t rr = r + u * S;
                    if(rr < rows)
                    {
                        const T     xv = x[rr * ld + c0];
                        const float v  = to_f32(xv);
                        acc[0] = OP == OP_MAX ? fmaxf(acc[0], fabsf(v)) : acc[0] + v;
                        if(OP == OP_SUMMAX) rm.add_scalar(xv);
                        if(want_sq) sqv = fmaf(v, v, sqv);
                    }
                }
            }
        }
    }
    if(kPacked)
    {
#pragma unroll
        for(int e = 0; e < E; ++e) acc[e] = half_bits_to_f32((pk[e / 2] >> (16 * (e % 2))) & 0xFFFFu);
    }
    if(OP == OP_SUMMAX)
    {   // every thread of the block takes part (threads beyond the last column carry 0)
        const float bm = block_reduce_max(rm.get(), lds_max);
        if(threadIdx.x == 0) st_partial(partial_max + blockIdx.y * gridDim.x + blockIdx.x, bm);
        if(want_sq)
        {
            __syncthreads();
            const float bs = block_reduce_sum(sqv, lds_max);
            if(threadIdx.x == 0) st_partial(fin.partial_sq + blockIdx.y * gridDim.x + blockIdx.x, bs);
        }
    }
    // fold the block's row lanes in order 0, 1, ... through LDS
    auto fold_rows = [&]() {
#pragma unroll
        for(int e = 0; e < E; ++e) lds[(tr * tpr + tc) * E + e] = acc[e];
        __syncthreads();
        if(tr == 0)
            for(int q = 1; q < rpb; ++q)
#pragma unroll
                for(int e = 0; e < E; ++e)
                {
                    const float o = lds[(q * tpr + tc) * E + e];
                    acc[e] = OP == OP_MAX ? fmaxf(acc[e], o) : acc[e] + o;
                }
    };
    fold_rows();
    if(tr == 0 && c0 < cols)
    {
#pragma unroll
        for(int e = 0; e < E; ++e) partial[static_cast<int64_t>(blockIdx.y) * cols + c0 + e] = acc[e];
    }
    if(OP != OP_SUMMAX || !fin.ctr) return;

    // ---- tensor-wide maximum: the last block of the whole grid
    const unsigned int nblocks = gridDim.x * gridDim.y;
    if(last_arrival(fin.ctr, nblocks, &flag))
    {
        if(want_sq)
        {   // the strip buffer is free by now: borrow it for the fold
            fold_sumsq(fin.partial_sq, nblocks, fin.sumsq_opt, reinterpret_cast<double*>(lds), BLOCK * E / 2);
            __syncthreads();
        }
        float mm = 0.0f;
        for(unsigned int i = threadIdx.x; i < nblocks; i += BLOCK) mm = fmaxf(mm, ld_partial(partial_max + i));
        mm = block_reduce_max(mm, lds_max);
        if(threadIdx.x == 0)
        {
            write_scale(mm, fin.qmax, fin.scale, fin.inv_scale, fin.amax_opt, 0);
            *fin.ctr = 0u;
        }
    }
}

// Second launch of the two-launch form: 16 columns per block; sixteen threads per column fold a
// sixteenth of the partials each (fixed assignment, fixed order), then the sixteen are folded in order.
template <int OP>
__global__ __launch_bounds__(kBlock) void colreduce_finalize_kernel(const float* __restrict__ partial, int S,
                                                                    int64_t cols, float qmax, float* out,
                                                                    float* inv_scale, float* amax_opt)
{
    __shared__ float lds[kBlock];
    const int     tc = threadIdx.x % 16, q = threadIdx.x / 16;
    const int64_t c  = static_cast<int64_t>(blockIdx.x) * 16 + tc;
    float         acc = 0.0f;
    if(c < cols)
    {
#pragma unroll 8                              // independent loads in flight; the fold keeps its order
        for(int s = q; s < S; s += 16)
        {
            const float o = partial[static_cast<int64_t>(s) * cols + c];
            acc = OP == OP_MAX ? fmaxf(acc, o) : acc + o;
        }
    }
    lds[threadIdx.x] = acc;
    __syncthreads();
    if(q == 0 && c < cols)
    {
        float t = 0.0f;
        for(int i = 0; i < 16; ++i) t = OP == OP_MAX ? fmaxf(t, lds[i * 16 + tc]) : t + lds[i * 16 + tc];
        if(OP == OP_MAX)
            write_scale(t, qmax, out, inv_scale, amax_opt, c);
        else
            out[c] = t;
    }
}

// ------------------------------------------------------------------ weights: row and column maxima in one pass
// Block b owns rows b*R .. b*R+R-1 in full: a thread sweeps its 16-byte column vectors with the R
// row loads of a vector in flight together, keeps the running maximum of every row in registers and
// writes the column maxima of its row group to partial[b][c] (folded by colreduce_finalize_kernel).
// Row maxima are complete inside the block: wave shuffles, one LDS exchange, then scale and inverse.
// Maxima are order independent, so the results equal those of the separate per-row and per-column passes.
template <typename T, int R, int U>
__global__ __launch_bounds__(kBlock) void absmax_rowcol_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                               int64_t ld, float qmax, float* row_scale, float* row_inv,
                                                               float* row_amax_opt, float* __restrict__ col_partial)
{
    constexpr int E = Vec16<T>::N;
    __shared__ float lds[R][kBlock / kWaveSize];
    const int64_t r0  = static_cast<int64_t>(blockIdx.x) * R;
    const int64_t ncv = cols / E;                    // cols % E == 0 on this path
    float         rowm[R];
#pragma unroll
    for(int i = 0; i < R; ++i) rowm[i] = 0.0f;
    for(int64_t cv0 = threadIdx.x; cv0 < ncv; cv0 += static_cast<int64_t>(kBlock) * U)
    {
        uint4 raw[U][R];                             // R x U loads in flight
#pragma unroll
        for(int u = 0; u < U; ++u)
#pragma unroll
            for(int i = 0; i < R; ++i)
            {
                const int64_t cv = cv0 + u * kBlock;
                raw[u][i] = (r0 + i < rows && cv < ncv) ? *reinterpret_cast<const uint4*>(x + (r0 + i) * ld + cv * E)
                                                         : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
        for(int u = 0; u < U; ++u)
        {
            const int64_t cv = cv0 + u * kBlock;
            float         cm[E];
#pragma unroll
            for(int e = 0; e < E; ++e) cm[e] = 0.0f;
#pragma unroll
            for(int i = 0; i < R; ++i)
            {
                float v[E];
                Vec16<T>::decode(raw[u][i], v);
#pragma unroll
                for(int e = 0; e < E; ++e)
                {
                    const float a = fabsf(v[e]);
                    cm[e]   = fmaxf(cm[e], a);
                    rowm[i] = fmaxf(rowm[i], a);
                }
            }
            if(cv < ncv)
            {
                float* dst = col_partial + static_cast<int64_t>(blockIdx.x) * cols + cv * E;
#pragma unroll
                for(int e = 0; e < E; e += 4)
                    *reinterpret_cast<float4*>(dst + e) = make_float4(cm[e], cm[e + 1], cm[e + 2], cm[e + 3]);
            }
        }
    }
    const int lane = threadIdx.x % kWaveSize, wave = threadIdx.x / kWaveSize;
#pragma unroll
    for(int i = 0; i < R; ++i)
    {
        const float m = wave_reduce_max(rowm[i]);
        if(lane == 0) lds[i][wave] = m;
    }
    __syncthreads();
    if(threadIdx.x < R && r0 + threadIdx.x < rows)
    {
        float m = lds[threadIdx.x][0];
#pragma unroll
        for(int w = 1; w < kBlock / kWaveSize; ++w) m = fmaxf(m, lds[threadIdx.x][w]);
        write_scale(m, qmax, row_scale, row_inv, row_amax_opt, r0 + threadIdx.x);
    }
}

// ------------------------------------------------------------------ INT8 quantize, vector path
// Each lane owns a patch of 16 (or 8) rows x 32 input bytes (16 binary16 or 8 fp32 columns) and
// requests the eight 16-byte loads of four rows together before it converts them.  A wavefront is up
// to 8 patches wide (fewer for narrow matrices, so that no lane idles) and the rest of its lanes
// stack patches downwards, so every load instruction covers whole 256-byte row segments; the int8
// codes of a patch row leave as one 16-byte (8-byte for fp32 input) store, and -- after a byte
// transpose held entirely in registers -- each column of the patch leaves as one 16-byte (8-byte)
// store to the transposed copy, lanes side by side.  No LDS, no barrier.
// Needs cols % 8 == 0 (Philox groups of 8 never straddle a row), rows % 16 == 0 when the
// transposed copy is written, and 16-byte aligned rows.

__device__ __forceinline__ uint32_t byte_of(uint32_t w, int b) { return (w >> (8 * b)) & 0xFFu; }

// `block` is the workgroup's index in the patch grid; GIVEN: the per-tensor inverse scale arrives as a value
// (a kernel that has just computed it) instead of through inv_scale.
template <typename T, int RND, bool PERCOL, int PR, bool DUAL, bool GIVEN>
__device__ __forceinline__ void quantize_patch_body(int64_t block, float inv_given, const T* __restrict__ x, int64_t rows,
                                                    int64_t cols, int64_t ld, int qmax, int gran, uint64_t seed,
                                                    uint64_t offset, const float* __restrict__ inv_scale,
                                                    int8_t* __restrict__ q, int8_t* __restrict__ qT, int64_t grid_x,
                                                    int lpr_log2, const float* __restrict__ inv_scale_T, int flip_C)
{
    // DUAL (weights): q takes the scales of `gran` (per row), the transposed copy takes one scale per column
    // from inv_scale_T -- two quantizations of the same values from one read.  flip_C > 0 (3x3 convolution
    // weights [N, 9*C]): the column scale belongs to the input channel c = column % C and column (tap, c)
    // lands in row c*9 + (8 - tap) of the transposed copy, i.e. the mirrored, channel-exchanged weights.
    static_assert(!DUAL || (!PERCOL && RND != kStochastic), "dual scales: nearest/floor, row scales for q");
    // A lane converts a patch of PR rows x PCOLS columns; the 2^lpr_log2 lanes of a wavefront that share
    // rows cover a contiguous row segment, the other lane bits stack patches downwards.  Narrow matrices
    // use fewer lanes per row (no idle lanes), small ones shorter patches (more wavefronts in flight).
    constexpr int E     = Vec16<T>::N;            // elements per 16-byte load (8 or 4)
    constexpr int PCOLS = 2 * E;                  // patch width: 16 (binary16) or 8 (fp32) columns
    constexpr int NH    = PCOLS / 8;              // 8-column halves per patch row (one Philox block each)
    constexpr int CW    = PCOLS / 4;              // code dwords per patch row
    const int     wtile_r = (kWaveSize >> lpr_log2) * PR, wtile_c = PCOLS << lpr_log2;
    const int     lane = threadIdx.x % kWaveSize, wave = threadIdx.x / kWaveSize;
    const int64_t by   = block / grid_x, bx = block - by * grid_x;
    const int64_t r0   = (by * (kBlock / kWaveSize) + wave) * wtile_r + (lane >> lpr_log2) * PR;
    const int64_t c0   = bx * wtile_c + (lane & ((1 << lpr_log2) - 1)) * PCOLS;
    if(r0 >= rows || c0 >= cols) return;
    const bool second_ok = NH == 1 || c0 + 8 < cols;      // binary16: the patch's second 8 columns exist

    float fcol[PCOLS];
    if(PERCOL || DUAL)
    {
        const float* cs = DUAL ? inv_scale_T : inv_scale;
#pragma unroll
        for(int j = 0; j < PCOLS; ++j)
            fcol[j] = (j < 8 || second_ok) ? cs[(DUAL && flip_C > 0) ? (c0 + j) % flip_C : (c0 + j)] : 1.0f;
    }
    const float ftensor = GIVEN ? inv_given : ((!PERCOL && gran == kPerTensor) ? inv_scale[0] : 1.0f);

    uint32_t code[PR][CW];   // row i, columns 4w..4w+3 in dword w
    uint32_t codeT[DUAL ? PR : 1][CW];   // DUAL: the codes of the transposed copy
    constexpr int RB = 4;                // rows per batch
#pragma unroll
    for(int batch = 0; batch < PR / RB; ++batch)
    {   // four rows at a time: their 8 loads are requested together, then converted
        uint4 raw[RB][2];
#pragma unroll
        for(int ii = 0; ii < RB; ++ii)
        {
            const int64_t r = r0 + batch * RB + ii;
#pragma unroll
            for(int l = 0; l < 2; ++l)
            {
                const bool ok = r < rows && (l == 0 || second_ok);
                raw[ii][l] = ok ? *reinterpret_cast<const uint4*>(x + r * ld + c0 + l * E) : make_uint4(0, 0, 0, 0);
            }
        }
#pragma unroll
        for(int ii = 0; ii < RB; ++ii)
        {
            const int     i    = batch * RB + ii;
            const int64_t r    = r0 + i;
            const float   frow = PERCOL ? 1.0f : ((gran == kPerRow && r < rows) ? inv_scale[r] : ftensor);
            float         v[PCOLS];
            float         t0[E], t1[E];
            Vec16<T>::decode(raw[ii][0], t0);
            Vec16<T>::decode(raw[ii][1], t1);
#pragma unroll
            for(int e = 0; e < E; ++e)
            {
                v[e]     = t0[e];
                v[E + e] = t1[e];
            }
#pragma unroll
            for(int w = 0; w < CW; ++w) code[i][w] = 0u;
            if constexpr(DUAL)
            {
#pragma unroll
                for(int w = 0; w < CW; ++w) codeT[i][w] = 0u;
#pragma unroll
                for(int col = 0; col < PCOLS; ++col)
                {
                    const int c = quantize_code<RND>(v[col], fcol[col], qmax, 0u);
                    codeT[i][col / 4] |= (static_cast<uint32_t>(c) & 0xFFu) << (8 * (col % 4));
                }
            }
#pragma unroll
            for(int h = 0; h < NH; ++h)
            {
                uint4 blk = {0u, 0u, 0u, 0u};
                if(RND == kStochastic)
                    blk = philox_group(seed, offset, static_cast<uint64_t>(r * cols + c0 + 8 * h) >> 3);
#pragma unroll
                for(int j = 0; j < 8; ++j)
                {
                    const int   col = 8 * h + j;
                    const float f   = PERCOL ? fcol[col] : frow;
                    const int   c   = quantize_code<RND>(v[col], f, qmax, philox_draw16(blk, j));
                    code[i][col / 4] |= (static_cast<uint32_t>(c) & 0xFFu) << (8 * (col % 4));
                }
            }
        }
        // Pin the batch's codes here: otherwise the compiler sinks all conversions behind the last
        // batch's loads and keeps every raw vector of the patch alive (register budget).
#pragma unroll
        for(int ii = 0; ii < RB; ++ii)
#pragma unroll
            for(int w = 0; w < CW; ++w) asm volatile("" : "+v"(code[batch * RB + ii][w]));
    }

    if(q)
    {
#pragma unroll
        for(int i = 0; i < PR; ++i)
        {
            const int64_t r = r0 + i;
            if(r >= rows) continue;
            int8_t* dst = q + r * cols + c0;
            if(NH == 1)
                *reinterpret_cast<uint2*>(dst) = make_uint2(code[i][0], code[i][1]);
            else if(cols % 16 == 0)
                *reinterpret_cast<uint4*>(dst) = make_uint4(code[i][0], code[i][1], code[i][CW - 2], code[i][CW - 1]);
            else
            {
                *reinterpret_cast<uint2*>(dst) = make_uint2(code[i][0], code[i][1]);
                if(second_ok) *reinterpret_cast<uint2*>(dst + 8) = make_uint2(code[i][CW - 2], code[i][CW - 1]);
            }
        }
    }
    if(qT)
    {   // rows % 16 == 0 here, so every row of the patch exists
#pragma unroll
        for(int col = 0; col < PCOLS; ++col)
        {
            if(col >= 8 && !second_ok) continue;
            uint32_t t[PR / 4];
#pragma unroll
            for(int g = 0; g < PR / 4; ++g)
            {
                auto pick = [&](int r, int w) -> uint32_t {
                    if constexpr(DUAL) return codeT[r][w]; else return code[r][w];
                };
                t[g] = byte_of(pick(4 * g + 0, col / 4), col % 4) | (byte_of(pick(4 * g + 1, col / 4), col % 4) << 8)
                     | (byte_of(pick(4 * g + 2, col / 4), col % 4) << 16)
                     | (byte_of(pick(4 * g + 3, col / 4), col % 4) << 24);
            }
            int64_t trow = c0 + col;
            if(DUAL && flip_C > 0)
            {
                const int64_t tap = trow / flip_C;
                trow = (trow - tap * flip_C) * 9 + (8 - tap);
            }
            int8_t* dst = qT + trow * rows + r0;
            if constexpr(PR == 16)
                *reinterpret_cast<uint4*>(dst) = make_uint4(t[0], t[1], t[2], t[3]);
            else if constexpr(PR == 8)
                *reinterpret_cast<uint2*>(dst) = make_uint2(t[0], t[1]);
            else
                *reinterpret_cast<uint32_t*>(dst) = t[0];
        }
    }
}

template <typename T, int RND, bool PERCOL, int PR, bool DUAL = false>
__global__ __launch_bounds__(kBlock, 3) void quantize_patch_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                                int64_t ld, int qmax, int gran, uint64_t seed,
                                                                uint64_t offset, const float* __restrict__ inv_scale,
                                                                int8_t* __restrict__ q, int8_t* __restrict__ qT,
                                                                int64_t grid_x, int lpr_log2,
                                                                const float* __restrict__ inv_scale_T = nullptr,
                                                                int flip_C = 0)
{
    quantize_patch_body<T, RND, PERCOL, PR, DUAL, false>(blockIdx.x, 1.0f, x, rows, cols, ld, qmax, gran, seed, offset,
                                                         inv_scale, q, qT, grid_x, lpr_log2, inv_scale_T, flip_C);
}

// ------------------------------------------------------------------ INT8 quantize, row-major codes only
// Contiguous tensor, one scale, no transposed copy: nothing ties a lane to a patch, so the lanes of a wavefront take
// adjacent groups of 8 elements (one Philox block each; a load instruction of a wavefront covers 1 KB of consecutive
// memory for binary16 input) with U groups in flight per lane, and the 8 codes of a group leave as one 8-byte store.
template <typename T, int RND>
__global__ __launch_bounds__(kBlock) void quantize_stream_kernel(const T* __restrict__ x, int64_t ngroups, int qmax,
                                                                 uint64_t seed, uint64_t offset,
                                                                 const float* __restrict__ inv_scale, int8_t* __restrict__ q)
{
    constexpr int E  = Vec16<T>::N;       // elements per 16-byte load (8 or 4)
    constexpr int VG = 8 / E;             // loads per group
    constexpr int U  = 4;
    const float   f  = inv_scale[0];
    const uint4*  xv = reinterpret_cast<const uint4*>(x);
    const int64_t g0 = static_cast<int64_t>(blockIdx.x) * (kBlock * U) + threadIdx.x;
    uint4         raw[U][VG];
#pragma unroll
    for(int u = 0; u < U; ++u)
    {
        const int64_t g = g0 + u * kBlock;
#pragma unroll
        for(int l = 0; l < VG; ++l) raw[u][l] = g < ngroups ? xv[g * VG + l] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for(int u = 0; u < U; ++u)
    {
        const int64_t g = g0 + u * kBlock;
        if(g >= ngroups) continue;
        float v[8];
#pragma unroll
        for(int l = 0; l < VG; ++l)
        {
            float t[E];
            Vec16<T>::decode(raw[u][l], t);
#pragma unroll
            for(int e = 0; e < E; ++e) v[l * E + e] = t[e];
        }
        uint4 blk = {0u, 0u, 0u, 0u};
        if(RND == kStochastic) blk = philox_group(seed, offset, static_cast<uint64_t>(g));
        uint32_t w[2] = {0u, 0u};
#pragma unroll
        for(int j = 0; j < 8; ++j)
        {
            const int c = quantize_code<RND>(v[j], f, qmax, philox_draw16(blk, j));
            w[j / 4] |= (static_cast<uint32_t>(c) & 0xFFu) << (8 * (j % 4));
        }
        *reinterpret_cast<uint2*>(q + g * 8) = make_uint2(w[0], w[1]);
    }
}

// ------------------------------------------------------------------ maximum and quantize in one launch
// Per-tensor scale, contiguous tensor.  Every workgroup (1) folds its share of the tensor into a partial
// maximum and publishes it, (2) takes a ticket; the last one to arrive clears the ticket counter and advances a
// generation word, the others poll that word, (3) folds all partials (the same maximum in every workgroup),
// forms the scale with the arithmetic of the separate pass, and (4) quantizes its patches, which it has just
// read and which therefore mostly still sit in cache.  The wait in (2) is bounded: a workgroup whose polls run
// out (the grid does not fit the device at once, or shares it with another kernel) finds the maximum by reading
// the whole tensor itself -- slower, same result, and no workgroup ever depends on one that has not started.
// `sync`: two 32-bit words, [0] tickets (zero before first use, zero again afterwards), [1] generation (any
// value); `partial`: one float per workgroup.
template <typename T, int RND, int PR>
__global__ __launch_bounds__(kBlock, 3) void absmax_quantize_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                                     int qmax, uint64_t seed, uint64_t offset,
                                                                     unsigned int* sync, float* partial, float* scale,
                                                                     float* inv_scale,
                                                                     float* amax_opt, int8_t* __restrict__ q,
                                                                     int8_t* __restrict__ qT, int64_t grid_x, int lpr_log2,
                                                                     int64_t patch_blocks, unsigned int poll_limit)
{
    __shared__ float lds[16];
    __shared__ int   timed_out;
    __shared__ float amax_all;
    constexpr int E = Vec16<T>::N;
    constexpr int U = 8;
    const int64_t nvec = rows * cols / E;                  // cols % 8 == 0: no scalar tail
    const uint4*  xv   = reinterpret_cast<const uint4*>(x);
    unsigned int  gen = 0u;
    if(threadIdx.x == 0) gen = __hip_atomic_load(sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // before the ticket
    auto fold_range = [&](int64_t first, int64_t step) {
        RunMax<T> rm;
        for(int64_t c = first + threadIdx.x; c < nvec; c += step)
        {
            uint4 v[U];
#pragma unroll
            for(int u = 0; u < U; ++u)
            {
                const int64_t idx = c + static_cast<int64_t>(u) * kBlock;
                v[u] = idx < nvec ? xv[idx] : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for(int u = 0; u < U; ++u) rm.add(v[u]);
        }
        return block_reduce_max(rm.get(), lds);
    };
    // (1) this workgroup's share: pieces of kBlock * U vectors, dealt round-robin
    const float mine = fold_range(static_cast<int64_t>(blockIdx.x) * kBlock * U, static_cast<int64_t>(gridDim.x) * kBlock * U);
    // (2)
    if(threadIdx.x == 0)
    {
        st_partial(partial + blockIdx.x, mine);
        __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): the partial has been written
        const unsigned int t = atomicAdd(sync, 1u);
        int late = 0;
        if(t == gridDim.x - 1u)
        {
            __hip_atomic_store(sync, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __hip_atomic_store(sync + 1, gen + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        else
        {
            unsigned int polls = 0u;
            while(__hip_atomic_load(sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gen)
            {
                if(++polls > poll_limit) { late = 1; break; }
                __builtin_amdgcn_s_sleep(4);
            }
        }
        timed_out = late;
    }
    __syncthreads();
    // (3)
    float folded;                                           // valid in thread 0
    if(!timed_out)
    {
        float m = 0.0f;
        for(int i = threadIdx.x; i < static_cast<int>(gridDim.x); i += kBlock) m = fmaxf(m, ld_partial(partial + i));
        folded = block_reduce_max(m, lds);
    }
    else
        folded = fold_range(0, static_cast<int64_t>(kBlock) * U);
    if(threadIdx.x == 0) amax_all = folded;
    __syncthreads();
    const float amax = amax_all;
    float inv = 1.0f;
    if(amax != 0.0f) inv = __fdiv_rn(static_cast<float>(qmax), amax);
    if(blockIdx.x == 0 && threadIdx.x == 0) write_scale(amax, static_cast<float>(qmax), scale, inv_scale, amax_opt, 0);
    // (4)
    for(int64_t b = blockIdx.x; b < patch_blocks; b += gridDim.x)
        quantize_patch_body<T, RND, false, PR, false, true>(b, inv, x, rows, cols, cols, qmax, kPerTensor, seed, offset,
                                                            nullptr, q, qT, grid_x, lpr_log2, nullptr, 0);
}

// Any shape, any alignment: one element per thread.
template <typename T>
__global__ __launch_bounds__(kBlock) void quantize_generic_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                                  int64_t ld, int qmax, int gran, int rnd,
                                                                  uint64_t seed, uint64_t offset,
                                                                  const float* __restrict__ inv_scale,
                                                                  int8_t* __restrict__ q, int8_t* __restrict__ qT)
{
    const int64_t n      = rows * cols;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for(int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n; i += stride)
    {
        const int64_t r = i / cols, c = i - r * cols;
        const float   f = inv_scale[gran == kPerTensor ? 0 : (gran == kPerRow ? r : c)];
        const float   v = to_f32(x[r * ld + c]);
        int           code;
        if(rnd == kStochastic)
        {
            const uint4 blk = philox_group(seed, offset, static_cast<uint64_t>(i) >> 3);
            code            = quantize_code<kStochastic>(v, f, qmax, philox_draw16(blk, static_cast<int>(i & 7)));
        }
        else if(rnd == kFloor)
            code = quantize_code<kFloor>(v, f, qmax, 0u);
        else
            code = quantize_code<kNearest>(v, f, qmax, 0u);
        if(q) q[i] = static_cast<int8_t>(code);
        if(qT) qT[c * rows + r] = static_cast<int8_t>(code);
    }
}

// ------------------------------------------------------------------ 3x3 im2col on int8 codes
// Patches of a 3x3, stride-1, pad-1 convolution built from the already quantized NHWC activation:
// A[m, (kh*3+kw)*C + c] = xq[n, h+kh-1, w+kw-1, c] (0 outside the image), m = (n*H + h)*W + w.
// The codes of the patch matrix equal the codes of the quantized fp16 patch matrix (per-tensor
// scale, zeros map to zero), but the activation is read and quantized once instead of nine times.
// Same lane geometry as the quantizer: a lane owns 16 output pixels x 16 K bytes (one tap, 16
// channels; needs C % 16 == 0), a wavefront 128 pixels x 128 K bytes; row-major rows leave as
// 16-byte stores, the transposed copy after a byte transpose in registers (needs M % 16 == 0).
__global__ __launch_bounds__(kBlock) void im2col3x3_i8_kernel(const int8_t* __restrict__ xq, int64_t nimg, int H, int W,
                                                              int C, int8_t* __restrict__ a, int8_t* __restrict__ aT,
                                                              int64_t grid_x)
{
    const int64_t M  = nimg * H * W;
    const int     K  = 9 * C, nchunk = K / 16;
    const int     lane = threadIdx.x % kWaveSize, wave = threadIdx.x / kWaveSize;
    const int64_t by = blockIdx.x / grid_x, bx = blockIdx.x - by * grid_x;
    const int64_t m0 = (by * (kBlock / kWaveSize) + wave) * 128 + (lane / 8) * 16;
    const int     ch = static_cast<int>(bx) * 8 + (lane % 8);             // 16-byte chunk of the K axis
    if(m0 >= M || ch >= nchunk) return;
    const int k0  = ch * 16;
    const int tap = k0 / C, c0 = k0 - tap * C;
    const int dh  = tap / 3 - 1, dw = tap % 3 - 1;
    uint32_t  code[16][4];
#pragma unroll
    for(int i = 0; i < 16; ++i)
    {
        const int64_t m = m0 + i;
        uint4         v = make_uint4(0, 0, 0, 0);
        if(m < M)
        {
            const int64_t hw = m % (static_cast<int64_t>(H) * W), n = m / (static_cast<int64_t>(H) * W);
            const int     h = static_cast<int>(hw / W) + dh, w = static_cast<int>(hw % W) + dw;
            if(h >= 0 && h < H && w >= 0 && w < W)
                v = *reinterpret_cast<const uint4*>(xq + ((n * H + h) * W + w) * C + c0);
        }
        code[i][0] = v.x; code[i][1] = v.y; code[i][2] = v.z; code[i][3] = v.w;
    }
    if(a)
    {
#pragma unroll
        for(int i = 0; i < 16; ++i)
            if(m0 + i < M)
                *reinterpret_cast<uint4*>(a + (m0 + i) * K + k0) = make_uint4(code[i][0], code[i][1], code[i][2], code[i][3]);
    }
    if(aT)
    {   // M % 16 == 0 here, so the 16 pixels all exist
#pragma unroll
        for(int col = 0; col < 16; ++col)
        {
            uint32_t t[4];
#pragma unroll
            for(int g = 0; g < 4; ++g)
                t[g] = byte_of(code[4 * g + 0][col / 4], col % 4) | (byte_of(code[4 * g + 1][col / 4], col % 4) << 8)
                     | (byte_of(code[4 * g + 2][col / 4], col % 4) << 16)
                     | (byte_of(code[4 * g + 3][col / 4], col % 4) << 24);
            *reinterpret_cast<uint4*>(aT + (static_cast<int64_t>(k0) + col) * M + m0) = make_uint4(t[0], t[1], t[2], t[3]);
        }
    }
}

// ------------------------------------------------------------------ padded, transposed pixel layout
// Operands of the convolution's weight gradient, which contracts over the pixels.  The codes [M, Ch] of an
// NHWC tensor are transposed to [Ch, Mp] over a padded pixel axis: every image is preceded by a zero row,
// rows are Wp >= W + 1 pixels long (a multiple of 16, the excess zero), one more zero row closes the axis:
//   p = (img * (H + 1) + 1 + h) * Wp + w.
// On this axis a window offset (dh, dw) is the plain displacement dh * Wp + dw and every out-of-image
// neighbour is a stored zero.  NS = 3 writes the three copies displaced by dw = -1, 0, +1
// (out[s][ch][q] = padded[ch][q + s - 1]), so that the GEMM reads 16-byte aligned rows for every tap;
// NS = 1 writes the undisplaced copy (the gradient operand).  A lane gathers 18 (16) pixels x 16 channels
// and leaves with one 16-byte store per channel and copy; pads are written, nothing is assumed zero.
// ES = element size in bytes (1: int8 codes, 2: binary16); `in`/`out` are byte pointers, Ch counts elements.
template <int NS, int ES>
__global__ __launch_bounds__(kBlock) void conv_padded_transpose_kernel(const int8_t* __restrict__ in, int64_t nimg, int H,
                                                                       int W, int Ch, int Wp, int64_t Mp,
                                                                       int8_t* __restrict__ out, int cw_log2,
                                                                       int margin_bytes)
{
    constexpr int NP  = NS == 3 ? 18 : 16;
    constexpr int CPC = 16 / ES;                  // channels per 16-byte chunk
    // margin_bytes > 0: `out` sits between two margins of that many bytes which the GEMM's displaced rows reach
    // into (multiplied by zeros of the other operand); they are cleared here so that no stale NaN pattern can
    // meet a binary16 zero
    if(margin_bytes > 0 && blockIdx.x == 0)
        for(int t = threadIdx.x * 16; t < margin_bytes; t += kBlock * 16)
        {
            *reinterpret_cast<uint4*>(out - margin_bytes + t) = make_uint4(0, 0, 0, 0);
            *reinterpret_cast<uint4*>(out + static_cast<int64_t>(NS) * Ch * Mp * ES + t) = make_uint4(0, 0, 0, 0);
        }
    const int64_t lin  = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    const int     ncc  = Ch / CPC, cw = 1 << cw_log2;
    const int64_t nq   = Mp / 16, rest = lin >> cw_log2;
    const int64_t qb   = rest % nq, ccg = rest / nq;
    const int     cc   = static_cast<int>(ccg) * cw + static_cast<int>(lin & (cw - 1));
    if(cc >= ncc) return;
    const int64_t q0 = qb * 16;
    const int     c0 = cc * CPC;
    // first gathered pixel: q0 - 1 (NS = 3) or q0; position -1 is written as the last column of a row "-1"
    int64_t p0 = q0 - (NS == 3 ? 1 : 0);
    int     col, hrow;
    int64_t img;
    if(p0 < 0) { col = Wp - 1; hrow = H; img = -1; }
    else
    {
        const int64_t r = p0 / Wp;
        col  = static_cast<int>(p0 - r * Wp);
        img  = r / (H + 1);
        hrow = static_cast<int>(r - img * (H + 1));
    }
    uint32_t code[NP][4];
#pragma unroll
    for(int i = 0; i < NP; ++i)
    {
        uint4 v = make_uint4(0, 0, 0, 0);
        if(col < W && hrow >= 1 && img >= 0 && img < nimg)
            v = *reinterpret_cast<const uint4*>(in + (((img * H + (hrow - 1)) * W + col) * Ch + c0) * ES);
        code[i][0] = v.x; code[i][1] = v.y; code[i][2] = v.z; code[i][3] = v.w;
        if(++col == Wp)
        {
            col = 0;
            if(++hrow == H + 1) { hrow = 0; ++img; }
        }
    }
#pragma unroll
    for(int s = 0; s < NS; ++s)
#pragma unroll
        for(int ch = 0; ch < CPC; ++ch)
        {
            int8_t* dst = out + ((static_cast<int64_t>(s) * Ch + c0 + ch) * Mp + q0) * ES;
            if constexpr(ES == 1)
            {
                uint32_t t[4];
#pragma unroll
                for(int g = 0; g < 4; ++g)
                    t[g] = byte_of(code[4 * g + 0 + s][ch / 4], ch % 4) | (byte_of(code[4 * g + 1 + s][ch / 4], ch % 4) << 8)
                         | (byte_of(code[4 * g + 2 + s][ch / 4], ch % 4) << 16)
                         | (byte_of(code[4 * g + 3 + s][ch / 4], ch % 4) << 24);
                *reinterpret_cast<uint4*>(dst) = make_uint4(t[0], t[1], t[2], t[3]);
            }
            else
            {
                uint32_t t[8];
#pragma unroll
                for(int g = 0; g < 8; ++g)
                {
                    const uint32_t lo = code[2 * g + 0 + s][ch / 2], hi = code[2 * g + 1 + s][ch / 2];
                    t[g] = (ch % 2 == 0) ? ((lo & 0xFFFFu) | (hi << 16)) : ((lo >> 16) | (hi & 0xFFFF0000u));
                }
                reinterpret_cast<uint4*>(dst)[0] = make_uint4(t[0], t[1], t[2], t[3]);
                reinterpret_cast<uint4*>(dst)[1] = make_uint4(t[4], t[5], t[6], t[7]);
            }
        }
}

// ------------------------------------------------------------------ cast / copy (+ transpose)
template <typename To, typename Ti> __device__ __forceinline__ To convert_elem(Ti v);
template <> __device__ __forceinline__ float  convert_elem<float, float>(float v) { return v; }
template <> __device__ __forceinline__ float  convert_elem<float, __half>(__half v) { return __half2float(v); }
template <> __device__ __forceinline__ __half convert_elem<__half, float>(float v) { return __float2half_rn(v); }
template <> __device__ __forceinline__ __half convert_elem<__half, __half>(__half v) { return v; }

// Floating-point stochastic quantization of one binary32 value to binary16 (Appendix, Proposition 2:
// truncate the mantissa to k bits, move up by one spacing with probability dropped / spacing).
// Integer arithmetic on the significand: sig * 2^(e-23) = |x|; D = (23-k) + max(0, -14-e) low bits are
// dropped (below the binary16 normal range the spacing stays 2^(-14-k)); up iff u16 < floor(rem * 2^16 / 2^D).
// The result is exact in binary16 (or reaches 2^16 and narrows to infinity).
__device__ __forceinline__ __half sr_narrow(float xv, int k, uint32_t u16)
{
    const uint32_t bits = __float_as_uint(xv);
    const uint32_t eb   = (bits >> 23) & 0xFFu;
    const uint32_t mant = bits & 0x7FFFFFu;
    const uint64_t sig  = eb == 0 ? mant : (mant | 0x800000u);
    const int      e    = eb == 0 ? -126 : static_cast<int>(eb) - 127;
    int            D    = (23 - k) + (e < -14 ? -14 - e : 0);
    D                   = D > 40 ? 40 : D;
    const uint64_t kept = sig >> D;
    const uint64_t rem  = sig & ((uint64_t(1) << D) - 1);
    const uint64_t thr  = D >= 16 ? (rem >> (D - 16)) : (rem << (16 - D));
    const uint32_t res  = static_cast<uint32_t>(kept) + (u16 < thr ? 1u : 0u);       // <= 2^(k+1)
    float          val  = ldexpf(static_cast<float>(res), e - 23 + D);                // exact
    val                 = (bits >> 31) ? -val : val;
    return __float2half_rn(val);                                                     // exact, or overflow to infinity
}

// 64x64 tile; the transposed copy goes through a padded LDS tile so that both copies are
// written with lanes along the contiguous axis.  SR (binary32 -> binary16 only) draws the element's
// 16-bit number from the Philox block of its row-major index, as the fixed-point quantizer does.
template <typename Ti, typename To, bool SR>
__global__ __launch_bounds__(kBlock) void convert_kernel(const Ti* __restrict__ x, int64_t rows, int64_t cols,
                                                         int64_t ld, To* __restrict__ q, To* __restrict__ qT,
                                                         int64_t grid_x, uint64_t seed, uint64_t offset, int k)
{
    __shared__ To tile[64][65];
    const int64_t by = blockIdx.x / grid_x, bx = blockIdx.x - by * grid_x;
    const int     tx = threadIdx.x % 64, ty = threadIdx.x / 64;
#pragma unroll 4
    for(int i = 0; i < 16; ++i)
    {
        const int     lr = ty + 4 * i;
        const int64_t r = by * 64 + lr, c = bx * 64 + tx;
        if(r < rows && c < cols)
        {
            To v;
            if constexpr(SR)
            {
                const uint64_t idx = static_cast<uint64_t>(r) * static_cast<uint64_t>(cols) + static_cast<uint64_t>(c);
                const uint4    blk = philox_group(seed, offset, idx >> 3);
                v = sr_narrow(x[r * ld + c], k, philox_draw16(blk, static_cast<int>(idx & 7)));
            }
            else
                v = convert_elem<To, Ti>(x[r * ld + c]);
            if(q) q[r * cols + c] = v;
            tile[lr][tx] = v;
        }
    }
    if(!qT) return;      // uniform over the block
    __syncthreads();
#pragma unroll 4
    for(int i = 0; i < 16; ++i)
    {
        const int     lc = ty + 4 * i;
        const int64_t c = bx * 64 + lc, r = by * 64 + tx;
        if(r < rows && c < cols) qT[c * rows + r] = tile[tx][lc];
    }
}

// Vector path of the cast to binary16 (and of the plain binary16 copy/transpose): each lane owns an
// 8 x 8 patch (8 rows x 16 bytes of binary16 output), a wavefront is 8 x 8 patches, so every load and
// every store instruction covers 128-byte (binary16) or 256-byte (fp32 input) row segments.  The patch
// is transposed in registers by pairing 16-bit halves; no LDS, no barrier.  Needs cols % 8 == 0, 16-byte
// aligned rows, and rows % 8 == 0 when the transposed copy is written.
template <typename Ti>
__global__ __launch_bounds__(kBlock) void cast_f16_patch_kernel(const Ti* __restrict__ x, int64_t rows, int64_t cols,
                                                                int64_t ld, __half* __restrict__ q,
                                                                __half* __restrict__ qT, int64_t grid_x)
{
    const int     lane = threadIdx.x % kWaveSize, wave = threadIdx.x / kWaveSize;
    const int64_t by = blockIdx.x / grid_x, bx = blockIdx.x - by * grid_x;
    const int64_t r0 = (by * (kBlock / kWaveSize) + wave) * 64 + (lane / 8) * 8;
    const int64_t c0 = bx * 64 + (lane % 8) * 8;
    if(r0 >= rows || c0 >= cols) return;
    uint32_t w[8][4];                           // row i of the patch as four pairs of binary16
#pragma unroll
    for(int i = 0; i < 8; ++i)
    {
        const int64_t r  = r0 + i;
        const bool    ok = r < rows;
        if constexpr(sizeof(Ti) == 2)
        {
            const uint4 v = ok ? *reinterpret_cast<const uint4*>(x + r * ld + c0) : make_uint4(0, 0, 0, 0);
            w[i][0] = v.x; w[i][1] = v.y; w[i][2] = v.z; w[i][3] = v.w;
        }
        else
        {
            const uint4 a = ok ? *reinterpret_cast<const uint4*>(x + r * ld + c0) : make_uint4(0, 0, 0, 0);
            const uint4 b = ok ? *reinterpret_cast<const uint4*>(x + r * ld + c0 + 4) : make_uint4(0, 0, 0, 0);
            const uint32_t f[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for(int j = 0; j < 4; ++j)
                w[i][j] = static_cast<uint32_t>(__half_as_ushort(__float2half_rn(__uint_as_float(f[2 * j]))))
                        | (static_cast<uint32_t>(__half_as_ushort(__float2half_rn(__uint_as_float(f[2 * j + 1])))) << 16);
        }
    }
    if(q)
    {
#pragma unroll
        for(int i = 0; i < 8; ++i)
            if(r0 + i < rows)
                *reinterpret_cast<uint4*>(q + (r0 + i) * cols + c0) = make_uint4(w[i][0], w[i][1], w[i][2], w[i][3]);
    }
    if(qT)
    {   // rows % 8 == 0 here: all eight rows exist.  Column c of the patch = halves c%2 of pair c/2 of every row.
#pragma unroll
        for(int c = 0; c < 8; ++c)
        {
            uint32_t t[4];
#pragma unroll
            for(int g = 0; g < 4; ++g)
            {
                const uint32_t lo = w[2 * g][c / 2], hi = w[2 * g + 1][c / 2];
                t[g] = (c % 2 == 0) ? ((lo & 0xFFFFu) | (hi << 16)) : ((lo >> 16) | (hi & 0xFFFF0000u));
            }
            *reinterpret_cast<uint4*>(qT + (c0 + c) * rows + r0) = make_uint4(t[0], t[1], t[2], t[3]);
        }
    }
}

// ------------------------------------------------------------------ standalone dequantize
// code * scale (+ bias) in the output type.  The dequantized scalar is the exact product of a code and a scale
// (Indicator section: x_hat = round(x_bar) * q_x); for an 8-bit code and one binary32 scale that product has at
// most 32 significant bits.  The binary16 result is that exact value rounded once: the binary32 product is
// brought to round-to-odd with the exact residual of the multiplication (fused multiply-add), and a value
// rounded to odd at 24 bits narrows to 11 bits like the exact one.  With a bias the sum is formed in binary32.
template <typename To> __device__ __forceinline__ To scaled_code(float a, float g, float bias, bool has_bias);
template <> __device__ __forceinline__ float scaled_code<float>(float a, float g, float bias, bool has_bias)
{
    const float v = a * g;
    return has_bias ? v + bias : v;
}
template <> __device__ __forceinline__ __half scaled_code<__half>(float a, float g, float bias, bool has_bias)
{
    const float p = a * g;
    if(has_bias) return __float2half_rn(p + bias);
    const float e = fmaf(a, g, -p);                         // exact residual of a normal product
    uint32_t    b = __float_as_uint(p);
    if(e != 0.0f && (b & 1u) == 0u && (b & 0x7F800000u) != 0u)
        b += ((e > 0.0f) == (p > 0.0f)) ? 1u : 0xFFFFFFFFu;       // the neighbour on the residual's side is the odd one
    return __float2half_rn(__uint_as_float(b));
}

template <typename Ti, typename To, int V>
__global__ __launch_bounds__(kBlock) void dequantize_kernel(const Ti* __restrict__ a, int64_t rows, int64_t cols,
                                                            int64_t ld, const float* __restrict__ rs,
                                                            const float* __restrict__ cs, float ts_host,
                                                            const float* __restrict__ ts_dev,
                                                            const float* __restrict__ cb, To* __restrict__ y)
{
    const float   ts     = ts_dev ? ts_host * ts_dev[0] : ts_host;      // one fp32 product (exact when ts_host is 1)
    const int64_t cv     = cols / V;          // V divides cols on this path (V == 1 otherwise)
    const int64_t n      = rows * cv;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for(int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n; i += stride)
    {
        const int64_t r = i / cv, c = (i - r * cv) * V;
        alignas(16) Ti in[V];
        if(V == 4 && sizeof(Ti) == 4)
            *reinterpret_cast<uint4*>(in) = *reinterpret_cast<const uint4*>(a + r * ld + c);
        else if(V == 4 && sizeof(Ti) == 1)
            *reinterpret_cast<uint32_t*>(in) = *reinterpret_cast<const uint32_t*>(a + r * ld + c);
        else
            in[0] = a[r * ld + c];
        // the scales are multiplied together first: with a single scale in use that product is the scale itself
        const float grow = ts * (rs ? rs[r] : 1.0f);
        alignas(16) To out[V];
#pragma unroll
        for(int e = 0; e < V; ++e)
            out[e] = scaled_code<To>(static_cast<float>(in[e]), cs ? grow * cs[c + e] : grow, cb ? cb[c + e] : 0.0f,
                                     cb != nullptr);
        To* dst = y + r * cols + c;
        if(V == 4 && sizeof(To) == 4)
            *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(out);
        else if(V == 4 && sizeof(To) == 2)
            *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(out);
        else
            dst[0] = out[0];
    }
}

// Vector path: a thread owns V = 16 / sizeof(Ti) adjacent columns (one 16-byte load) and walks down the
// rows, four loads in flight; its column scales and biases are fetched once.  2^tx_log2 threads of a
// block lie side by side along a row (the whole block, 4 KB, when the matrix is wide enough), the
// rest of the block stacks rows.  Same arithmetic per element as dequantize_kernel.
template <typename Ti, typename To>
__global__ __launch_bounds__(kBlock) void dequantize_cols_kernel(const Ti* __restrict__ a, int64_t rows, int64_t cols,
                                                                 int64_t ld, const float* __restrict__ rs,
                                                                 const float* __restrict__ cs, float ts_host,
                                                                 const float* __restrict__ ts_dev,
                                                                 const float* __restrict__ cb, To* __restrict__ y,
                                                                 int tx_log2)
{
    constexpr int V = 16 / sizeof(Ti);
    constexpr int U = 4;
    const float   ts = ts_dev ? ts_host * ts_dev[0] : ts_host;
    const int     tx = threadIdx.x & ((1 << tx_log2) - 1), ty = threadIdx.x >> tx_log2, TY = kBlock >> tx_log2;
    const int64_t c  = ((static_cast<int64_t>(blockIdx.x) << tx_log2) + tx) * V;
    if(c >= cols) return;
    float fcs[V], fcb[V];
#pragma unroll
    for(int e = 0; e < V; e += 4)
    {
        const float4 s4 = cs ? *reinterpret_cast<const float4*>(cs + c + e) : make_float4(1.0f, 1.0f, 1.0f, 1.0f);
        const float4 b4 = cb ? *reinterpret_cast<const float4*>(cb + c + e) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        fcs[e] = s4.x; fcs[e + 1] = s4.y; fcs[e + 2] = s4.z; fcs[e + 3] = s4.w;
        fcb[e] = b4.x; fcb[e + 1] = b4.y; fcb[e + 2] = b4.z; fcb[e + 3] = b4.w;
    }
    // a block works on TY * U adjacent rows at a time
    for(int64_t base = static_cast<int64_t>(blockIdx.y) * (TY * U); base < rows; base += static_cast<int64_t>(gridDim.y) * (TY * U))
    {
        uint4 raw[U];
#pragma unroll
        for(int u = 0; u < U; ++u)
        {
            const int64_t r = base + u * TY + ty;
            raw[u] = r < rows ? *reinterpret_cast<const uint4*>(a + r * ld + c) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for(int u = 0; u < U; ++u)
        {
            const int64_t r = base + u * TY + ty;
            if(r >= rows) continue;
            const float grow = ts * (rs ? rs[r] : 1.0f);
            alignas(16) Ti in[V];
            *reinterpret_cast<uint4*>(in) = raw[u];
            alignas(16) To out[V];
#pragma unroll
            for(int e = 0; e < V; ++e)
                out[e] = scaled_code<To>(static_cast<float>(in[e]), cs ? grow * fcs[e] : grow, fcb[e], cb != nullptr);
            To* dst = y + r * cols + c;
#pragma unroll
            for(int e = 0; e < V * static_cast<int>(sizeof(To)) / 16; ++e)
                reinterpret_cast<uint4*>(dst)[e] = reinterpret_cast<const uint4*>(out)[e];
            if(V * sizeof(To) == 8) *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(out);
        }
    }
}

int next_pow2(int64_t v)
{
    int p = 1;
    while(p < v) p <<= 1;
    return p;
}

// Launch shape of a per-column reduction with `block` threads per block: threads per row (a power
// of two, at most one wavefront so that a wavefront reads 1 KB of a row) and block rows
// (gridDim.y, at most kColParts).  Large inputs run 1024-thread blocks, about one per compute
// unit: sixteen wavefronts with four loads in flight each keep the memory pipeline full, and a
// strip then has few enough partials for one block to fold them.
void colreduce_shape(int64_t rows, int64_t cols, int E, int block, int& tpr, int& gy)
{
    const int64_t ncv = (cols + E - 1) / E;
    tpr               = ncv >= kWaveSize ? kWaveSize : (next_pow2(ncv) < 2 ? 2 : next_pow2(ncv));
    if(ncv > static_cast<int64_t>(kWaveSize) * 1000) tpr = kBlock;     // very wide: keep the strip count small
    const int64_t gx  = (ncv + tpr - 1) / tpr;
    const int     rpb = block / tpr;
    const int64_t target = block >= 1024 ? 256 : 1024;
    int64_t       g   = (target + gx - 1) / gx;
    const int64_t maxg = (rows + rpb - 1) / rpb;              // no more block rows than row groups
    if(g > maxg) g = maxg;
    if(g > kColParts) g = kColParts;
    if(g < 1) g = 1;
    gy = static_cast<int>(g);
}

// Workspace of the per-tensor reductions: the arrival counter first (a 256-byte slot), partials behind it.
constexpr size_t kCtrBytes = 256;

template <typename T, int OP>
hipError_t colreduce_launch(const T* x, int64_t rows, int64_t cols, int64_t ld, float qmax, float* out,
                            float* inv_scale, float* amax_opt, float* partial, float* partial_max, TensorFinal tfin,
                            hipStream_t st)
{
    constexpr int E     = Vec16<T>::N;
    const bool    vec   = aligned16(x) && (ld * sizeof(T)) % 16 == 0 && cols % E == 0;
    const int     block = rows * cols >= (int64_t(1) << 20) ? 1024 : kBlock;
    int           tpr, gy;
    colreduce_shape(rows, cols, vec ? E : 1, block, tpr, gy);
    const int64_t ncv = (cols + (vec ? E : 1) - 1) / (vec ? E : 1);
    const int64_t gx  = (ncv + tpr - 1) / tpr;
    if(partial_max)
        while(gx * gy > kAbsmaxMaxBlocks && gy > 1) gy = (gy + 1) / 2;  // block maxima must fit their slots
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(gy));
    if(vec)
    {
        if(block == 1024)
            colreduce_kernel<T, true, OP, 1024><<<grid, dim3(1024), 0, st>>>(x, rows, cols, ld, tpr, partial, partial_max, tfin);
        else
            colreduce_kernel<T, true, OP, kBlock><<<grid, dim3(kBlock), 0, st>>>(x, rows, cols, ld, tpr, partial, partial_max, tfin);
    }
    else
    {
        if(block == 1024)
            colreduce_kernel<T, false, OP, 1024><<<grid, dim3(1024), 0, st>>>(x, rows, cols, ld, tpr, partial, partial_max, tfin);
        else
            colreduce_kernel<T, false, OP, kBlock><<<grid, dim3(kBlock), 0, st>>>(x, rows, cols, ld, tpr, partial, partial_max, tfin);
    }
    constexpr int FOP = OP == OP_MAX ? OP_MAX : OP_SUM;
    colreduce_finalize_kernel<FOP><<<dim3((cols + 15) / 16), dim3(kBlock), 0, st>>>(partial, gy, cols, qmax, out, inv_scale,
                                                                                amax_opt);
    if(OP == OP_SUMMAX && !tfin.ctr)
        absmax_tensor_finalize_kernel<<<dim3(1), dim3(kBlock), 0, st>>>(partial_max, static_cast<int>(gx * gy), tfin.qmax,
                                                                        tfin.scale, tfin.inv_scale, tfin.amax_opt);
    return hipGetLastError();
}

}  // namespace

// ======================================================================== launchers
size_t absmax_workspace_bytes(int64_t rows, int64_t cols, int gran)
{
    (void)rows;
    const size_t c = static_cast<size_t>(cols > 0 ? cols : 0);
    if(gran == kPerTensor)   // counter, block maxima, block sums of squares; with fused column sums also their partials
        return kCtrBytes + sizeof(float) * (2 * kAbsmaxMaxBlocks + static_cast<size_t>(kColParts) * c);
    if(gran == kPerCol) return kCtrBytes + sizeof(float) * kColParts * c;   // same layout: the counter slot stays untouched
    return 0;
}

template <typename T>
static hipError_t absmax_typed(const T* x, int64_t rows, int64_t cols, int64_t ld, int gran, float qmax, float* scale,
                               float* inv_scale, float* amax_opt, float* colsum_opt, float* sumsq_opt, void* workspace,
                               hipStream_t st)
{
    constexpr int E       = Vec16<T>::N;
    const bool    rows_ok = aligned16(x) && (ld * sizeof(T)) % 16 == 0;
    (void)E;
    if(gran == kPerTensor)
    {
        unsigned int* ctr = static_cast<unsigned int*>(workspace);
        float*        ws  = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + kCtrBytes);
        float*        wsq = ws + kAbsmaxMaxBlocks;          // block sums of squares
        if(colsum_opt)
        {   // per-tensor absmax fused with column sums: one pass over x
            TensorFinal tfin{ctr, qmax, scale, inv_scale, amax_opt, wsq, sumsq_opt};
            return colreduce_launch<T, OP_SUMMAX>(x, rows, cols, ld, 0.0f, colsum_opt, nullptr, nullptr,
                                                  ws + 2 * kAbsmaxMaxBlocks, ws, tfin, st);
        }
        const bool    vec  = aligned16(x) && ld == cols;
        const int64_t work = vec ? (rows * cols) / E : rows * cols;
        const bool    big  = work >= (int64_t(1) << 19);
        const int     blk  = big ? 1024 : kBlock;
        int64_t       nb   = (work + blk * 8 - 1) / (blk * 8);
        nb                 = nb < 1 ? 1 : (nb > 256 ? 256 : nb);       // few blocks: the tickets are serialised
        if(vec)
        {
            if(big)
                absmax_tensor_kernel<T, true, 1024><<<dim3(nb), dim3(1024), 0, st>>>(x, rows, cols, ld, ws, ctr, qmax, scale, inv_scale, amax_opt, wsq, sumsq_opt);
            else
                absmax_tensor_kernel<T, true, kBlock><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, ws, ctr, qmax, scale, inv_scale, amax_opt, wsq, sumsq_opt);
        }
        else
        {
            if(big)
                absmax_tensor_kernel<T, false, 1024><<<dim3(nb), dim3(1024), 0, st>>>(x, rows, cols, ld, ws, ctr, qmax, scale, inv_scale, amax_opt, wsq, sumsq_opt);
            else
                absmax_tensor_kernel<T, false, kBlock><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, ws, ctr, qmax, scale, inv_scale, amax_opt, wsq, sumsq_opt);
        }
    }
    else if(gran == kPerRow)
    {
        const bool few = rows < 4096;         // too few rows to fill the chip with one wavefront per row
        const int64_t nb = few ? rows : (rows + 3) / 4;
        if(rows_ok)
        {
            if(few)
                absmax_rows_kernel<T, true, 4><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, qmax, scale, inv_scale, amax_opt);
            else
                absmax_rows_kernel<T, true, 1><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, qmax, scale, inv_scale, amax_opt);
        }
        else
        {
            if(few)
                absmax_rows_kernel<T, false, 4><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, qmax, scale, inv_scale, amax_opt);
            else
                absmax_rows_kernel<T, false, 1><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, qmax, scale, inv_scale, amax_opt);
        }
    }
    else
    {
        TensorFinal none{nullptr, qmax, nullptr, nullptr, nullptr, nullptr, nullptr};
        return colreduce_launch<T, OP_MAX>(x, rows, cols, ld, qmax, scale, inv_scale, amax_opt,
                                           reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + kCtrBytes), nullptr,
                                           none, st);
    }
    return hipGetLastError();
}

hipError_t launch_scale_from_amax(float* amax, float qmax, float* scale, float* inv_scale, int consume, hipStream_t st)
{
    scale_from_amax_kernel<<<dim3(1), dim3(64), 0, st>>>(amax, qmax, scale, inv_scale, consume);
    return hipGetLastError();
}

// ---- scratch that the library owns: for the entry point that may not allocate ---------------------------------
// One array per GPU (every device that loads this code object holds its own copy at its own address), kept
// until the process ends.  Host code must never pass the array's name to a kernel: that name is a host-side
// stand-in.  The device address is looked up once per device and handed to the kernels like any workspace.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t static_scratch(void** ptr_out)
{
    constexpr int      kMaxDevices = 64;
    static std::mutex  lock;
    static void*       per_device[kMaxDevices] = {};
    int                dev = -1;
    hipError_t         e   = hipGetDevice(&dev);
    if(e != hipSuccess) return e;
    if(dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(lock);
    if(!per_device[dev])
    {
        void* p = nullptr;
        e       = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if(e != hipSuccess) return e;
        if(!p) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr_out = per_device[dev];
    return hipSuccess;
}

hipError_t launch_absmax_scale(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int gran, float qmax,
                               float* scale, float* inv_scale, float* amax_opt, float* colsum_opt, float* sumsq_opt,
                               void* workspace, hipStream_t stream)
{
    if(xdt == kF32)
        return absmax_typed(static_cast<const float*>(x), rows, cols, ld, gran, qmax, scale, inv_scale, amax_opt,
                            colsum_opt, sumsq_opt, workspace, stream);
    return absmax_typed(static_cast<const __half*>(x), rows, cols, ld, gran, qmax, scale, inv_scale, amax_opt,
                        colsum_opt, sumsq_opt, workspace, stream);
}

// Launch shape of the patch kernel: lanes per row (as a power of two) and patch height.
struct PatchShape { int lpr_log2, pr; int64_t gx, gy; };
template <typename T> static PatchShape patch_shape(int64_t rows, int64_t cols, bool transposed_copy)
{
    constexpr int PCOLS = 2 * Vec16<T>::N;
    PatchShape    p{3, 16, 0, 0};
    const int64_t pc = (cols + PCOLS - 1) / PCOLS;                 // patches per row
    while(p.lpr_log2 > 0 && (int64_t(1) << (p.lpr_log2 - 1)) >= pc) --p.lpr_log2;
    // 8-row patches put twice the wavefronts in flight (measured: faster whenever no transposed copy is
    // written, and below about eight wavefronts of 16-row patches per compute unit); the transposed copy
    // of a large tensor prefers 16-byte stores
    if(!transposed_copy || (rows / 16) * pc < int64_t(kWaveSize) * 2048) p.pr = 8;
    p.gx = (pc + (int64_t(1) << p.lpr_log2) - 1) >> p.lpr_log2;
    const int64_t rows_per_block = static_cast<int64_t>(kBlock / kWaveSize) * (kWaveSize >> p.lpr_log2) * p.pr;
    p.gy = (rows + rows_per_block - 1) / rows_per_block;
    return p;
}

template <typename T, int RND>
static void quantize_patch_launch(const T* x, int64_t rows, int64_t cols, int64_t ld, int qmax, int gran,
                                  uint64_t seed, uint64_t offset, const float* inv, int8_t* q, int8_t* qT,
                                  hipStream_t st)
{
    const PatchShape ps = patch_shape<T>(rows, cols, qT != nullptr);
    const dim3       grid(static_cast<unsigned>(ps.gx * ps.gy));
    auto go = [&](auto percol, auto pr) {
        quantize_patch_kernel<T, RND, decltype(percol)::value, decltype(pr)::value><<<grid, dim3(kBlock), 0, st>>>(
            x, rows, cols, ld, qmax, gran, seed, offset, inv, q, qT, ps.gx, ps.lpr_log2);
    };
    typedef std::integral_constant<int, 16> P16;
    typedef std::integral_constant<int, 8>  P8;
    if(gran == kPerCol) { if(ps.pr == 16) go(std::true_type{}, P16{}); else go(std::true_type{}, P8{}); }
    else                { if(ps.pr == 16) go(std::false_type{}, P16{}); else go(std::false_type{}, P8{}); }
}

template <typename T>
static hipError_t quantize_typed(const T* x, int64_t rows, int64_t cols, int64_t ld, int qmax, int gran, int rnd,
                                 uint64_t seed, uint64_t offset, const float* inv, int8_t* q, int8_t* qT,
                                 hipStream_t st)
{
    const PatchShape ps = patch_shape<T>(rows, cols, qT != nullptr);
    const int64_t    gx = ps.gx, gy = ps.gy;
    const bool    fast = cols % 8 == 0 && aligned16(x) && (ld * sizeof(T)) % 16 == 0 && (!q || aligned16(q))
                      && (!qT || (aligned16(qT) && rows % 16 == 0)) && gx * gy < (int64_t(1) << 31);
    if(fast && q && !qT && gran == kPerTensor && ld == cols && rows * cols / 8 < (int64_t(1) << 40))
    {   // row-major codes of a contiguous tensor with one scale: the streaming form
        const int64_t ngroups = rows * cols / 8;
        const dim3    grid(static_cast<unsigned>((ngroups + kBlock * 4 - 1) / (kBlock * 4)));
        if(rnd == kStochastic)
            quantize_stream_kernel<T, kStochastic><<<grid, dim3(kBlock), 0, st>>>(x, ngroups, qmax, seed, offset, inv, q);
        else if(rnd == kFloor)
            quantize_stream_kernel<T, kFloor><<<grid, dim3(kBlock), 0, st>>>(x, ngroups, qmax, seed, offset, inv, q);
        else
            quantize_stream_kernel<T, kNearest><<<grid, dim3(kBlock), 0, st>>>(x, ngroups, qmax, seed, offset, inv, q);
    }
    else if(fast)
    {
        if(rnd == kStochastic)
            quantize_patch_launch<T, kStochastic>(x, rows, cols, ld, qmax, gran, seed, offset, inv, q, qT, st);
        else if(rnd == kFloor)
            quantize_patch_launch<T, kFloor>(x, rows, cols, ld, qmax, gran, seed, offset, inv, q, qT, st);
        else
            quantize_patch_launch<T, kNearest>(x, rows, cols, ld, qmax, gran, seed, offset, inv, q, qT, st);
    }
    else
    {
        int64_t nb = (rows * cols + kBlock - 1) / kBlock;
        nb         = nb > 65536 ? 65536 : nb;
        quantize_generic_kernel<T><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, qmax, gran, rnd, seed, offset,
                                                                     inv, q, qT);
    }
    return hipGetLastError();
}

hipError_t launch_quantize_int8(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int qmax, int gran,
                                int rnd, uint64_t seed, uint64_t offset, const float* inv_scale, int8_t* q, int8_t* qT,
                                hipStream_t stream)
{
    if(xdt == kF32)
        return quantize_typed(static_cast<const float*>(x), rows, cols, ld, qmax, gran, rnd, seed, offset, inv_scale,
                              q, qT, stream);
    return quantize_typed(static_cast<const __half*>(x), rows, cols, ld, qmax, gran, rnd, seed, offset, inv_scale, q,
                          qT, stream);
}

// Per-tensor maximum, scales and codes with one launch where that pays (a small contiguous tensor: the second
// read comes from cache and one dependent launch is saved), otherwise the two separate launches.  The single
// launch runs one workgroup per compute unit at most (few tickets), a third of what the separate quantize kernel
// keeps in flight, so it stops paying at about 4M elements (measured: 2048x1024 14 vs 17 us, 8192x1024 22 vs 18
// us) and, with the arithmetic-heavy stochastic rounding, at about 1M (1024x1024 13 vs 17 us, 2048x1024 17 vs 17 us).
constexpr int64_t kOneLaunchMaxElems = int64_t(1) << 22, kOneLaunchMaxElemsStochastic = int64_t(1) << 20;

template <typename T>
static hipError_t absmax_quantize_typed(const T* x, int64_t rows, int64_t cols, int qmax, int rnd, uint64_t seed,
                                        uint64_t offset, float* scale, float* inv_scale, float* amax_opt, int8_t* q,
                                        int8_t* qT, void* workspace, unsigned int poll_limit, hipStream_t st)
{
    const PatchShape ps = patch_shape<T>(rows, cols, qT != nullptr);
    const int64_t    patch_blocks = ps.gx * ps.gy;
    const bool one_launch = cols % 8 == 0 && aligned16(x) && (!q || aligned16(q)) && (!qT || (aligned16(qT) && rows % 16 == 0))
                         && patch_blocks < (int64_t(1) << 31)
                         && rows * cols <= (rnd == kStochastic ? kOneLaunchMaxElemsStochastic : kOneLaunchMaxElems);
    if(!one_launch)
    {
        hipError_t e = absmax_typed(x, rows, cols, cols, kPerTensor, static_cast<float>(qmax), scale, inv_scale, amax_opt,
                                    nullptr, nullptr, workspace, st);
        if(e != hipSuccess) return e;
        return quantize_typed(x, rows, cols, cols, qmax, kPerTensor, rnd, seed, offset, inv_scale, q, qT, st);
    }
    // one workgroup per compute unit at most: all of them resident at once on an otherwise idle device, and few
    // tickets on the counter
    static int cus = 0;
    if(cus == 0)
    {
        int dev = 0, n = 0;
        if(hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 64;
        cus = n;
    }
    const int64_t g = patch_blocks < cus ? patch_blocks : cus;
    unsigned int* sync    = static_cast<unsigned int*>(workspace);
    float*        partial = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + kCtrBytes);
    auto go = [&](auto rnd_tag, auto pr) {
        absmax_quantize_kernel<T, decltype(rnd_tag)::value, decltype(pr)::value><<<dim3(static_cast<unsigned>(g)), dim3(kBlock), 0, st>>>(
            x, rows, cols, qmax, seed, offset, sync, partial, scale, inv_scale, amax_opt, q, qT, ps.gx, ps.lpr_log2,
            patch_blocks, poll_limit);
    };
    typedef std::integral_constant<int, 16> P16;
    typedef std::integral_constant<int, 8>  P8;
    auto by_pr = [&](auto rnd_tag) { if(ps.pr == 16) go(rnd_tag, P16{}); else go(rnd_tag, P8{}); };
    if(rnd == kStochastic) by_pr(std::integral_constant<int, kStochastic>{});
    else if(rnd == kFloor) by_pr(std::integral_constant<int, kFloor>{});
    else                   by_pr(std::integral_constant<int, kNearest>{});
    return hipGetLastError();
}

hipError_t launch_absmax_quantize(const void* x, int xdt, int64_t rows, int64_t cols, int qmax, int rnd, uint64_t seed,
                                  uint64_t offset, float* scale, float* inv_scale, float* amax_opt, int8_t* q, int8_t* qT,
                                  void* workspace, unsigned int poll_limit, hipStream_t stream)
{
    if(xdt == kF32)
        return absmax_quantize_typed(static_cast<const float*>(x), rows, cols, qmax, rnd, seed, offset, scale, inv_scale,
                                     amax_opt, q, qT, workspace, poll_limit, stream);
    return absmax_quantize_typed(static_cast<const __half*>(x), rows, cols, qmax, rnd, seed, offset, scale, inv_scale,
                                 amax_opt, q, qT, workspace, poll_limit, stream);
}

// Weights of one linear operator in one go: per-row scales and codes for the forward, per-column scales
// and transposed codes for dX.  Fused form: row + column maxima in one pass, the column fold, one dual
// quantize (3 launches, W read twice); otherwise the five separate launches.  Same results either way.
template <typename T>
static hipError_t prepare_weights_typed(const T* w, int64_t N, int64_t K, float qmax, float* sw, float* iw,
                                        float* aw_opt, int8_t* wq, float* swb, float* iwb, int8_t* wqbT,
                                        void* workspace, hipStream_t st, int64_t conv_C = 0)
{
    // conv_C > 0: w is [N, 9*conv_C]; the second scales are per input channel (conv_C of them) and wqbT is the
    // mirrored, channel-exchanged copy [conv_C, 9*N]; only the fused form serves this case.
    constexpr int E = Vec16<T>::N;
    float*        partial = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + kCtrBytes);
    const bool    fused = aligned16(w) && K % (2 * E) == 0 && K % 8 == 0 && N % 16 == 0 && N <= 16 * kColParts
                       && aligned16(wq) && aligned16(wqbT) && aligned16(partial);
    if(!fused && conv_C > 0) return hipErrorInvalidValue;      // the caller tests the same conditions before choosing this form
    if(!fused)
    {
        hipError_t e = absmax_typed(w, N, K, K, kPerRow, qmax, sw, iw, aw_opt, nullptr, nullptr, workspace, st);
        if(e != hipSuccess) return e;
        e = quantize_typed(w, N, K, K, static_cast<int>(qmax), kPerRow, kNearest, 0, 0, iw, wq, nullptr, st);
        if(e != hipSuccess) return e;
        e = absmax_typed(w, N, K, K, kPerCol, qmax, swb, iwb, nullptr, nullptr, nullptr, workspace, st);
        if(e != hipSuccess) return e;
        return quantize_typed(w, N, K, K, static_cast<int>(qmax), kPerCol, kNearest, 0, 0, iwb, nullptr, wqbT, st);
    }
    int gy;          // row groups = partial rows per column (at most kColParts); 16 loads in flight per thread
    if(N <= 2 * kColParts)
    {
        gy = static_cast<int>((N + 1) / 2);
        absmax_rowcol_kernel<T, 2, 8><<<dim3(gy), dim3(kBlock), 0, st>>>(w, N, K, K, qmax, sw, iw, aw_opt, partial);
    }
    else if(N <= 4 * kColParts)
    {
        gy = static_cast<int>((N + 3) / 4);
        absmax_rowcol_kernel<T, 4, 4><<<dim3(gy), dim3(kBlock), 0, st>>>(w, N, K, K, qmax, sw, iw, aw_opt, partial);
    }
    else if(N <= 8 * kColParts)
    {
        gy = static_cast<int>((N + 7) / 8);
        absmax_rowcol_kernel<T, 8, 2><<<dim3(gy), dim3(kBlock), 0, st>>>(w, N, K, K, qmax, sw, iw, aw_opt, partial);
    }
    else
    {
        gy = static_cast<int>((N + 15) / 16);
        absmax_rowcol_kernel<T, 16, 1><<<dim3(gy), dim3(kBlock), 0, st>>>(w, N, K, K, qmax, sw, iw, aw_opt, partial);
    }
    if(conv_C > 0)      // partial[gy][9][C] read as gy*9 rows of C columns: maxima per input channel
        colreduce_finalize_kernel<OP_MAX><<<dim3((conv_C + 15) / 16), dim3(kBlock), 0, st>>>(partial, gy * 9, conv_C, qmax, swb, iwb, nullptr);
    else
        colreduce_finalize_kernel<OP_MAX><<<dim3((K + 15) / 16), dim3(kBlock), 0, st>>>(partial, gy, K, qmax, swb, iwb, nullptr);
    // 4-row patches: weights are small, more wavefronts in flight matter more than wide transposed stores
    PatchShape ps = patch_shape<T>(N, K, false);
    ps.gy = (N + 4 * (kWaveSize >> ps.lpr_log2) * 4 - 1) / (4 * (kWaveSize >> ps.lpr_log2) * 4);
    quantize_patch_kernel<T, kNearest, false, 4, true><<<dim3(static_cast<unsigned>(ps.gx * ps.gy)), dim3(kBlock), 0, st>>>(
        w, N, K, K, static_cast<int>(qmax), kPerRow, 0, 0, iw, wq, wqbT, ps.gx, ps.lpr_log2, iwb, static_cast<int>(conv_C));
    return hipGetLastError();
}

hipError_t launch_prepare_weights(const void* w, int wdt, int64_t N, int64_t K, float qmax, float* sw, float* iw,
                                  float* aw_opt, int8_t* wq, float* swb, float* iwb, int8_t* wqbT, void* workspace,
                                  hipStream_t stream)
{
    if(wdt == kF32)
        return prepare_weights_typed(static_cast<const float*>(w), N, K, qmax, sw, iw, aw_opt, wq, swb, iwb, wqbT, workspace, stream);
    return prepare_weights_typed(static_cast<const __half*>(w), N, K, qmax, sw, iw, aw_opt, wq, swb, iwb, wqbT, workspace, stream);
}

template <typename Ti, typename To>
static hipError_t convert_typed(const void* x, int64_t rows, int64_t cols, int64_t ld, void* q, void* qT,
                                hipStream_t st)
{
    if constexpr(std::is_same<To, __half>::value)
    {
        const int64_t bx = (cols + 63) / 64, by = (rows + 255) / 256;
        if(cols % 8 == 0 && aligned16(x) && (ld * sizeof(Ti)) % 16 == 0 && (!q || aligned16(q))
           && (!qT || (aligned16(qT) && rows % 8 == 0)) && bx * by < (int64_t(1) << 31))
        {
            cast_f16_patch_kernel<Ti><<<dim3(static_cast<unsigned>(bx * by)), dim3(kBlock), 0, st>>>(
                static_cast<const Ti*>(x), rows, cols, ld, static_cast<__half*>(q), static_cast<__half*>(qT), bx);
            return hipGetLastError();
        }
    }
    const int64_t gx = (cols + 63) / 64, gy = (rows + 63) / 64;
    convert_kernel<Ti, To, false><<<dim3(static_cast<unsigned>(gx * gy)), dim3(kBlock), 0, st>>>(
        static_cast<const Ti*>(x), rows, cols, ld, static_cast<To*>(q), static_cast<To*>(qT), gx, 0, 0, 0);
    return hipGetLastError();
}

hipError_t launch_convert(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int outdt, void* q, void* qT,
                          hipStream_t stream)
{
    if(xdt == kF32 && outdt == kF16) return convert_typed<float, __half>(x, rows, cols, ld, q, qT, stream);
    if(xdt == kF32 && outdt == kF32) return convert_typed<float, float>(x, rows, cols, ld, q, qT, stream);
    if(xdt == kF16 && outdt == kF16) return convert_typed<__half, __half>(x, rows, cols, ld, q, qT, stream);
    return convert_typed<__half, float>(x, rows, cols, ld, q, qT, stream);
}

hipError_t launch_convert_sr(const float* x, int64_t rows, int64_t cols, int64_t ld, int mantissa_bits, uint64_t seed,
                             uint64_t offset, void* q, void* qT, hipStream_t stream)
{
    const int64_t gx = (cols + 63) / 64, gy = (rows + 63) / 64;
    convert_kernel<float, __half, true><<<dim3(static_cast<unsigned>(gx * gy)), dim3(kBlock), 0, stream>>>(
        x, rows, cols, ld, static_cast<__half*>(q), static_cast<__half*>(qT), gx, seed, offset, mantissa_bits);
    return hipGetLastError();
}

template <typename Ti, typename To>
static hipError_t dequantize_typed(const void* a, int64_t rows, int64_t cols, int64_t ld, const float* rs,
                                   const float* cs, float ts, const float* tsd, const float* cb, void* y, hipStream_t st)
{
    constexpr int V16 = 16 / sizeof(Ti);
    const bool    wide = cols % V16 == 0 && (ld * sizeof(Ti)) % 16 == 0 && aligned16(a) && aligned16(y)
                      && (!cs || aligned16(cs)) && (!cb || aligned16(cb));
    // (without per-column parameters the flat kernel below streams 32-bit inputs a little faster: measured)
    if(wide && (cs || cb || sizeof(Ti) == 1))
    {
        const int64_t cv = cols / V16;
        int           tx_log2 = 8;                                   // the whole block along the row when possible
        while(tx_log2 > 0 && (int64_t(1) << (tx_log2 - 1)) >= cv) --tx_log2;
        const int64_t gx = (cv + (int64_t(1) << tx_log2) - 1) >> tx_log2;
        const int64_t ty = kBlock >> tx_log2;
        int64_t       gy = (rows + ty * 4 - 1) / (ty * 4);           // four rows in flight per thread
        if(gy > 65535) gy = 65535;
        if(gy < 1) gy = 1;
        if(gx < (int64_t(1) << 31))
        {
            dequantize_cols_kernel<Ti, To><<<dim3(static_cast<unsigned>(gx), static_cast<unsigned>(gy)), dim3(kBlock), 0, st>>>(
                static_cast<const Ti*>(a), rows, cols, ld, rs, cs, ts, tsd, cb, static_cast<To*>(y), tx_log2);
            return hipGetLastError();
        }
    }
    const bool vec = cols % 4 == 0 && ld % 4 == 0 && (reinterpret_cast<uintptr_t>(a) % (4 * sizeof(Ti))) == 0
                  && (reinterpret_cast<uintptr_t>(y) % (4 * sizeof(To))) == 0;
    const int64_t work = vec ? rows * (cols / 4) : rows * cols;
    int64_t       nb   = (work + kBlock - 1) / kBlock;
    nb                 = nb > (1 << 20) ? (1 << 20) : nb;
    if(vec)
        dequantize_kernel<Ti, To, 4><<<dim3(nb), dim3(kBlock), 0, st>>>(static_cast<const Ti*>(a), rows, cols, ld, rs,
                                                                       cs, ts, tsd, cb, static_cast<To*>(y));
    else
        dequantize_kernel<Ti, To, 1><<<dim3(nb), dim3(kBlock), 0, st>>>(static_cast<const Ti*>(a), rows, cols, ld, rs,
                                                                       cs, ts, tsd, cb, static_cast<To*>(y));
    return hipGetLastError();
}

hipError_t launch_dequantize(const void* a, int adt, int64_t rows, int64_t cols, int64_t ld, const float* row_scale,
                             const float* col_scale, float tensor_scale, const float* tensor_scale_dev,
                             const float* col_bias, void* y, int ydt, hipStream_t stream)
{
    if(adt == kI32 && ydt == kF32)
        return dequantize_typed<int32_t, float>(a, rows, cols, ld, row_scale, col_scale, tensor_scale, tensor_scale_dev, col_bias, y, stream);
    if(adt == kI32 && ydt == kF16)
        return dequantize_typed<int32_t, __half>(a, rows, cols, ld, row_scale, col_scale, tensor_scale, tensor_scale_dev, col_bias, y, stream);
    if(adt == kI8 && ydt == kF32)
        return dequantize_typed<int8_t, float>(a, rows, cols, ld, row_scale, col_scale, tensor_scale, tensor_scale_dev, col_bias, y, stream);
    return dequantize_typed<int8_t, __half>(a, rows, cols, ld, row_scale, col_scale, tensor_scale, tensor_scale_dev, col_bias, y, stream);
}

// wflip[c, (8 - tap)*N + n] = w[n, tap*C + c]: a few kilobytes of weights, one element per thread.
template <typename T>
__global__ __launch_bounds__(256) void conv3x3_wflip_kernel(const T* __restrict__ w, int64_t N, int64_t C, T* __restrict__ wflip)
{
    const int64_t total = 9 * N * C;
    for(int64_t o = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; o < total; o += static_cast<int64_t>(gridDim.x) * 256)
    {
        const int64_t c = o / (9 * N), r = o - c * 9 * N, tap = r / N, n = r - tap * N;
        wflip[o] = w[n * 9 * C + (8 - tap) * C + c];
    }
}

hipError_t launch_conv3x3_wflip(const void* w, int elem_bytes, int64_t N, int64_t C, void* wflip, hipStream_t stream)
{
    const int64_t total = 9 * N * C;
    if(total <= 0) return hipSuccess;
    int64_t nb = (total + 255) / 256;
    nb         = nb > 4096 ? 4096 : nb;
    if(elem_bytes == 1)
        conv3x3_wflip_kernel<int8_t><<<dim3(static_cast<unsigned>(nb)), dim3(256), 0, stream>>>(
            static_cast<const int8_t*>(w), N, C, static_cast<int8_t*>(wflip));
    else
        conv3x3_wflip_kernel<uint16_t><<<dim3(static_cast<unsigned>(nb)), dim3(256), 0, stream>>>(
            static_cast<const uint16_t*>(w), N, C, static_cast<uint16_t*>(wflip));
    return hipGetLastError();
}

hipError_t launch_conv3x3_prepare_weights(const void* w, int wdt, int64_t N, int64_t C, float qmax, float* sw, float* iw,
                                          float* swb, float* iwb, int8_t* wq, int8_t* wflip, void* workspace,
                                          hipStream_t st)
{
    const int64_t K = 9 * C;
    const int64_t e2 = wdt == kF32 ? 8 : 16;
    float*        partial = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + kCtrBytes);
    const bool    fused = aligned16(w) && K % e2 == 0 && N % 16 == 0 && N <= 16 * kColParts && C <= (1 << 20)
                       && aligned16(wq) && aligned16(wflip) && aligned16(partial);
    if(fused)
    {
        if(wdt == kF32)
            return prepare_weights_typed(static_cast<const float*>(w), N, K, qmax, sw, iw, nullptr, wq, swb, iwb, wflip, workspace, st, C);
        return prepare_weights_typed(static_cast<const __half*>(w), N, K, qmax, sw, iw, nullptr, wq, swb, iwb, wflip, workspace, st, C);
    }
    // large weights: the separate passes; the per-c codes go through the workspace (behind the absmax scratch)
    int8_t*    wqb = static_cast<int8_t*>(workspace) + absmax_workspace_bytes(N, K, kPerCol);
    hipError_t e   = launch_absmax_scale(w, wdt, N, K, K, kPerRow, qmax, sw, iw, nullptr, nullptr, nullptr, workspace, st);
    if(e != hipSuccess) return e;
    e = launch_quantize_int8(w, wdt, N, K, K, static_cast<int>(qmax), kPerRow, kNearest, 0, 0, iw, wq, nullptr, st);
    if(e != hipSuccess) return e;
    e = launch_absmax_scale(w, wdt, 9 * N, C, C, kPerCol, qmax, swb, iwb, nullptr, nullptr, nullptr, workspace, st);
    if(e != hipSuccess) return e;
    e = launch_quantize_int8(w, wdt, 9 * N, C, C, static_cast<int>(qmax), kPerCol, kNearest, 0, 0, iwb, wqb, nullptr, st);
    if(e != hipSuccess) return e;
    return launch_conv3x3_wflip(wqb, 1, N, C, wflip, st);
}


hipError_t launch_im2col3x3_i8(const int8_t* xq, int64_t nimg, int H, int W, int C, int8_t* a, int8_t* aT,
                               hipStream_t stream)
{
    const int64_t M  = nimg * H * W;
    const int64_t gx = (9 * C / 16 + 7) / 8, gy = (M + 511) / 512;
    im2col3x3_i8_kernel<<<dim3(static_cast<unsigned>(gx * gy)), dim3(kBlock), 0, stream>>>(xq, nimg, H, W, C, a, aT, gx);
    return hipGetLastError();
}

ConvPaddedAxis conv_padded_axis(int64_t nimg, int H, int W)
{
    ConvPaddedAxis a;
    a.Wp = (W + 1 + 15) / 16 * 16;
    a.Mp = (nimg * (H + 1) + 1) * a.Wp;          // a multiple of 16
    return a;
}

hipError_t launch_conv_padded_transpose(const void* in, int elem_bytes, int64_t nimg, int H, int W, int Ch, int copies,
                                        void* out, int margin_bytes, hipStream_t stream)
{
    const ConvPaddedAxis ax = conv_padded_axis(nimg, H, W);
    const int     ncc = Ch / (16 / elem_bytes);
    int           cw_log2 = 2;                                   // four channel chunks side by side when there are that many
    while(cw_log2 > 0 && (1 << (cw_log2 - 1)) >= ncc) --cw_log2;
    const int64_t groups = (ncc + (1 << cw_log2) - 1) >> cw_log2;
    const int64_t lanes  = (ax.Mp / 16) * groups << cw_log2;
    const int64_t nb     = (lanes + kBlock - 1) / kBlock;
    if(nb >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    const dim3    grid(static_cast<unsigned>(nb)), block(kBlock);
    const int8_t* src = static_cast<const int8_t*>(in);
    int8_t*       dst = static_cast<int8_t*>(out);
    if(elem_bytes == 1)
    {
        if(copies == 3) conv_padded_transpose_kernel<3, 1><<<grid, block, 0, stream>>>(src, nimg, H, W, Ch, ax.Wp, ax.Mp, dst, cw_log2, margin_bytes);
        else            conv_padded_transpose_kernel<1, 1><<<grid, block, 0, stream>>>(src, nimg, H, W, Ch, ax.Wp, ax.Mp, dst, cw_log2, margin_bytes);
    }
    else
    {
        if(copies == 3) conv_padded_transpose_kernel<3, 2><<<grid, block, 0, stream>>>(src, nimg, H, W, Ch, ax.Wp, ax.Mp, dst, cw_log2, margin_bytes);
        else            conv_padded_transpose_kernel<1, 2><<<grid, block, 0, stream>>>(src, nimg, H, W, Ch, ax.Wp, ax.Mp, dst, cw_log2, margin_bytes);
    }
    return hipGetLastError();
}

size_t colsum_workspace_bytes(int64_t rows, int64_t cols)
{
    (void)rows;
    return sizeof(float) * static_cast<size_t>(kColParts) * static_cast<size_t>(cols > 0 ? cols : 0);
}

// ------------------------------------------------------------------ transpose of int8 codes
// out[c, r] = in[r, c].  A lane owns a 16 x 16 byte patch: sixteen 16-byte loads, a byte transpose in registers,
// sixteen 16-byte stores; a wavefront is 8 patches wide (128-byte row segments) and 8 patches high.
__global__ __launch_bounds__(kBlock) void transpose_i8_patch_kernel(const int8_t* __restrict__ in, int64_t rows, int64_t cols,
                                                                   int8_t* __restrict__ out, int64_t grid_x)
{
    const int     lane = threadIdx.x % kWaveSize, wave = threadIdx.x / kWaveSize;
    const int64_t by = blockIdx.x / grid_x, bx = blockIdx.x - by * grid_x;
    const int64_t r0 = (by * (kBlock / kWaveSize) + wave) * 128 + (lane / 8) * 16;
    const int64_t c0 = bx * 128 + (lane % 8) * 16;
    if(r0 >= rows || c0 >= cols) return;                   // rows and cols are multiples of 16: patches are whole
    uint4 raw[16];
#pragma unroll
    for(int i = 0; i < 16; ++i) raw[i] = *reinterpret_cast<const uint4*>(in + (r0 + i) * cols + c0);
#pragma unroll
    for(int c = 0; c < 16; ++c)
    {
        uint32_t t[4];
#pragma unroll
        for(int g = 0; g < 4; ++g)
        {
            auto word = [&](int r) -> uint32_t {
                const uint4& v = raw[r];
                return (c / 4) == 0 ? v.x : (c / 4) == 1 ? v.y : (c / 4) == 2 ? v.z : v.w;
            };
            t[g] = byte_of(word(4 * g + 0), c % 4) | (byte_of(word(4 * g + 1), c % 4) << 8)
                 | (byte_of(word(4 * g + 2), c % 4) << 16) | (byte_of(word(4 * g + 3), c % 4) << 24);
        }
        *reinterpret_cast<uint4*>(out + (c0 + c) * rows + r0) = make_uint4(t[0], t[1], t[2], t[3]);
    }
}

__global__ __launch_bounds__(kBlock) void transpose_i8_generic_kernel(const int8_t* __restrict__ in, int64_t rows, int64_t cols,
                                                                     int8_t* __restrict__ out)
{
    const int64_t n = rows * cols, stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for(int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n; i += stride)
    {
        const int64_t r = i / cols, c = i - r * cols;
        out[c * rows + r] = in[i];
    }
}

hipError_t launch_transpose_i8(const int8_t* in, int64_t rows, int64_t cols, int8_t* out, hipStream_t stream)
{
    if(rows <= 0 || cols <= 0) return hipSuccess;
    const int64_t gx = (cols + 127) / 128, gy = (rows + 128 * (kBlock / kWaveSize) - 1) / (128 * (kBlock / kWaveSize));
    if(rows % 16 == 0 && cols % 16 == 0 && aligned16(in) && aligned16(out) && gx * gy < (int64_t(1) << 31))
        transpose_i8_patch_kernel<<<dim3(static_cast<unsigned>(gx * gy)), dim3(kBlock), 0, stream>>>(in, rows, cols, out, gx);
    else
    {
        int64_t nb = (rows * cols + kBlock - 1) / kBlock;
        nb         = nb > 65536 ? 65536 : nb;
        transpose_i8_generic_kernel<<<dim3(static_cast<unsigned>(nb)), dim3(kBlock), 0, stream>>>(in, rows, cols, out);
    }
    return hipGetLastError();
}

// Clears n floats with a kernel (a memset node recorded into a captured graph is avoided on purpose).
__global__ __launch_bounds__(256) void zero_f32_kernel(float* __restrict__ p, int64_t n)
{
    for(int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += static_cast<int64_t>(gridDim.x) * 256)
        p[i] = 0.0f;
}

hipError_t launch_zero_f32(float* p, int64_t n, hipStream_t stream)
{
    if(n <= 0) return hipSuccess;
    int64_t nb = (n + 255) / 256;
    nb         = nb > 1024 ? 1024 : nb;
    zero_f32_kernel<<<dim3(static_cast<unsigned>(nb)), dim3(256), 0, stream>>>(p, n);
    return hipGetLastError();
}

hipError_t launch_colsum(const void* x, int xdt, int64_t rows, int64_t cols, float* out, float* workspace,
                         hipStream_t stream)
{
    TensorFinal none{nullptr, 0.0f, nullptr, nullptr, nullptr, nullptr, nullptr};
    if(xdt == kF32)
        return colreduce_launch<float, OP_SUM>(static_cast<const float*>(x), rows, cols, cols, 0.0f, out, nullptr, nullptr,
                                               workspace, nullptr, none, stream);
    return colreduce_launch<__half, OP_SUM>(static_cast<const __half*>(x), rows, cols, cols, 0.0f, out, nullptr, nullptr,
                                            workspace, nullptr, none, stream);
}

}  // namespace qsync
