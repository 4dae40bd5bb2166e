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

// ------------------------------------------------------------------ absmax, per tensor
// Stage 1: each block folds a strided share of the tensor into one partial maximum.
template <typename T, bool VEC>
__global__ __launch_bounds__(kBlock) void absmax_tensor_kernel(const T* __restrict__ x, int64_t rows,
                                                               int64_t cols, int64_t ld,
                                                               float* __restrict__ partial)
{
    __shared__ float lds[16];
    float            m      = 0.0f;
    const int64_t    n      = rows * cols;
    const int64_t    stride = static_cast<int64_t>(gridDim.x) * kBlock;
    int64_t          i      = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if(VEC)
    {   // contiguous tensor, 16-byte aligned base: every block streams contiguous 32 KB pieces
        constexpr int E    = Vec16<T>::N;
        constexpr int U    = 8;                       // 16-byte loads in flight per lane
        const int64_t nvec = n / E;
        const int64_t step = static_cast<int64_t>(gridDim.x) * kBlock * U;
        for(int64_t c = static_cast<int64_t>(blockIdx.x) * kBlock * U + threadIdx.x; c < nvec; c += step)
        {
            float v[U][E];
#pragma unroll
            for(int u = 0; u < U; ++u)
            {
                const int64_t idx = c + static_cast<int64_t>(u) * kBlock;
                if(idx < nvec)
                    Vec16<T>::load(x + idx * E, v[u]);
                else
                {
#pragma unroll
                    for(int e = 0; e < E; ++e) v[u][e] = 0.0f;
                }
            }
#pragma unroll
            for(int u = 0; u < U; ++u)
#pragma unroll
                for(int e = 0; e < E; ++e) m = fmaxf(m, fabsf(v[u][e]));
        }
        if(blockIdx.x == 0)
            for(int64_t j = nvec * E + threadIdx.x; j < n; j += kBlock) m = fmaxf(m, fabsf(to_f32(x[j])));
    }
    else
    {
        for(; i < n; i += stride)
        {
            const int64_t r = i / cols, c = i - r * cols;
            m = fmaxf(m, fabsf(to_f32(x[r * ld + c])));
        }
    }
    m = block_reduce_max(m, lds);
    if(threadIdx.x == 0) partial[blockIdx.x] = m;
}

// Stage 2: one block folds the partials and writes amax, scale and inverse scale.
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

// ------------------------------------------------------------------ absmax, per row
// One wavefront per row; the row maximum needs no second stage.
template <typename T, bool VEC>
__global__ __launch_bounds__(kBlock) void absmax_rows_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                             int64_t ld, float qmax, float* scale, float* inv_scale,
                                                             float* amax_opt)
{
    const int     lane = threadIdx.x % kWaveSize;
    const int64_t r    = static_cast<int64_t>(blockIdx.x) * (kBlock / kWaveSize) + threadIdx.x / kWaveSize;
    if(r >= rows) return;
    const T* row = x + r * ld;
    float    m   = 0.0f;
    int64_t  done = 0;
    if(VEC)
    {
        constexpr int E    = Vec16<T>::N;
        const int64_t nvec = cols / E;
        float         v[E];
        for(int64_t i = lane; i < nvec; i += kWaveSize)
        {
            Vec16<T>::load(row + i * E, v);
#pragma unroll
            for(int e = 0; e < E; ++e) m = fmaxf(m, fabsf(v[e]));
        }
        done = nvec * E;
    }
    for(int64_t c = done + lane; c < cols; c += kWaveSize) m = fmaxf(m, fabsf(to_f32(row[c])));
    m = wave_reduce_max(m);
    if(lane == 0) write_scale(m, qmax, scale, inv_scale, amax_opt, r);
}

// ------------------------------------------------------------------ absmax, per column
// Stage 1: lanes own adjacent columns (one 16-byte vector each when VEC), wavefronts own
// interleaved row subsets; partial[s][c] holds the maximum of subset s.
template <typename T, bool VEC>
__global__ __launch_bounds__(kBlock) void absmax_cols_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                             int64_t ld, float* __restrict__ partial)
{
    constexpr int E    = VEC ? Vec16<T>::N : 1;
    const int     lane = threadIdx.x % kWaveSize;
    const int64_t c0   = (static_cast<int64_t>(blockIdx.x) * kWaveSize + lane) * E;
    const int     s    = blockIdx.y * (kBlock / kWaveSize) + threadIdx.x / kWaveSize;
    const int     S    = gridDim.y * (kBlock / kWaveSize);
    if(c0 >= cols) return;
    float m[E];
#pragma unroll
    for(int e = 0; e < E; ++e) m[e] = 0.0f;
    for(int64_t r = s; r < rows; r += S)
    {
        if(VEC)
        {
            float v[Vec16<T>::N];
            Vec16<T>::load(x + r * ld + c0, v);
#pragma unroll
            for(int e = 0; e < E; ++e) m[e] = fmaxf(m[e], fabsf(v[e]));
        }
        else
            m[0] = fmaxf(m[0], fabsf(to_f32(x[r * ld + c0])));
    }
#pragma unroll
    for(int e = 0; e < E; ++e) partial[static_cast<int64_t>(s) * cols + c0 + e] = m[e];
}

__global__ __launch_bounds__(kBlock) void absmax_cols_finalize_kernel(const float* __restrict__ partial, int S,
                                                                      int64_t cols, float qmax, float* scale,
                                                                      float* inv_scale, float* amax_opt)
{
    const int64_t c = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if(c >= cols) return;
    float m = 0.0f;
    for(int s = 0; s < S; ++s) m = fmaxf(m, partial[static_cast<int64_t>(s) * cols + c]);
    write_scale(m, qmax, scale, inv_scale, amax_opt, c);
}

// ------------------------------------------------------------------ INT8 quantize, vector path
// Each lane owns a 16x16 patch of the tensor.  A wavefront is 8 patches wide and 8 tall, so
// every load instruction covers 8 rows of 128 contiguous columns, the int8 codes of a row
// leave as one 16-byte store (8 lanes = 128 contiguous bytes), and -- after a 16x16 byte
// transpose held entirely in registers -- each column of the patch leaves as one 16-byte
// store to the transposed copy (8 lanes = 128 contiguous bytes there, too).  No LDS, no
// barrier.  Needs cols % 8 == 0 (Philox groups of 8 never straddle a row), rows % 16 == 0 when
// the transposed copy is written, and 16-byte aligned rows.
constexpr int kPatch      = 16;
constexpr int kWaveTile   = 8 * kPatch;                       // 128 x 128 elements per wavefront
constexpr int kBlockRows  = (kBlock / kWaveSize) * kWaveTile; // wavefronts stacked along rows

__device__ __forceinline__ uint32_t byte_of(uint32_t w, int b) { return (w >> (8 * b)) & 0xFFu; }

template <typename T, int RND, bool PERCOL>
__global__ __launch_bounds__(kBlock) void quantize_patch_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                                int64_t ld, float qmax, int gran, uint64_t seed,
                                                                uint64_t offset, const float* __restrict__ inv_scale,
                                                                int8_t* __restrict__ q, int8_t* __restrict__ qT,
                                                                int64_t grid_x)
{
    constexpr int E    = Vec16<T>::N;        // elements per 16-byte load
    constexpr int LPH  = 8 / E;              // loads per 8-column half-row (1 for binary16, 2 for fp32)
    const int     lane = threadIdx.x % kWaveSize, wave = threadIdx.x / kWaveSize;
    const int64_t by   = blockIdx.x / grid_x, bx = blockIdx.x - by * grid_x;
    const int64_t r0   = by * kBlockRows + wave * kWaveTile + (lane / 8) * kPatch;
    const int64_t c0   = bx * kWaveTile + (lane % 8) * kPatch;
    if(r0 >= rows || c0 >= cols) return;
    const bool half_ok[2] = {true, c0 + 8 < cols};

    float fcol[kPatch];
    if(PERCOL)
    {
#pragma unroll
        for(int j = 0; j < kPatch; ++j) fcol[j] = (j < 8 || half_ok[1]) ? inv_scale[c0 + j] : 1.0f;
    }
    const float ftensor = (!PERCOL && gran == kPerTensor) ? inv_scale[0] : 1.0f;

    uint32_t code[kPatch][4];   // row i, columns 4w..4w+3 in dword w
#pragma unroll
    for(int i = 0; i < kPatch; ++i)
    {
        const int64_t r = r0 + i;
#pragma unroll
        for(int w = 0; w < 4; ++w) code[i][w] = 0u;
        if(r < rows)
        {
            const float frow = PERCOL ? 1.0f : (gran == kPerRow ? inv_scale[r] : ftensor);
#pragma unroll
            for(int h = 0; h < 2; ++h)
            {
                if(!half_ok[h]) continue;
                float v[8];
#pragma unroll
                for(int l = 0; l < LPH; ++l)
                {
                    float t[E];
                    Vec16<T>::load(x + r * ld + c0 + 8 * h + l * E, t);
#pragma unroll
                    for(int e = 0; e < E; ++e) v[l * E + e] = t[e];
                }
                uint4 blk = {0u, 0u, 0u, 0u};
                if(RND == kStochastic)
                    blk = philox_group(seed, offset, static_cast<uint64_t>(r * cols + c0 + 8 * h) >> 3);
#pragma unroll
                for(int j = 0; j < 8; ++j)
                {
                    const int   col = 8 * h + j;
                    const float f   = PERCOL ? fcol[col] : frow;
                    const int   c   = quantize_code<RND>(v[j], f, qmax, philox_draw16(blk, j));
                    code[i][col / 4] |= (static_cast<uint32_t>(c) & 0xFFu) << (8 * (col % 4));
                }
            }
        }
    }

    if(q)
    {
        const bool wide = (cols % 16 == 0);
#pragma unroll
        for(int i = 0; i < kPatch; ++i)
        {
            const int64_t r = r0 + i;
            if(r >= rows) continue;
            int8_t* dst = q + r * cols + c0;
            if(wide)
                *reinterpret_cast<uint4*>(dst) = make_uint4(code[i][0], code[i][1], code[i][2], code[i][3]);
            else
            {
                *reinterpret_cast<uint2*>(dst) = make_uint2(code[i][0], code[i][1]);
                if(half_ok[1]) *reinterpret_cast<uint2*>(dst + 8) = make_uint2(code[i][2], code[i][3]);
            }
        }
    }
    if(qT)
    {   // rows % 16 == 0 here, so the patch's 16 rows all exist
#pragma unroll
        for(int col = 0; col < kPatch; ++col)
        {
            if(col >= 8 && !half_ok[1]) continue;
            uint32_t t[4];
#pragma unroll
            for(int g = 0; g < 4; ++g)
                t[g] = byte_of(code[4 * g + 0][col / 4], col % 4) | (byte_of(code[4 * g + 1][col / 4], col % 4) << 8)
                     | (byte_of(code[4 * g + 2][col / 4], col % 4) << 16)
                     | (byte_of(code[4 * g + 3][col / 4], col % 4) << 24);
            *reinterpret_cast<uint4*>(qT + (c0 + col) * rows + r0) = make_uint4(t[0], t[1], t[2], t[3]);
        }
    }
}

// Any shape, any alignment: one element per thread.
template <typename T>
__global__ __launch_bounds__(kBlock) void quantize_generic_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                                  int64_t ld, float qmax, int gran, int rnd,
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

// ------------------------------------------------------------------ cast / copy (+ transpose)
template <typename To, typename Ti> __device__ __forceinline__ To convert_elem(Ti v);
template <> __device__ __forceinline__ float  convert_elem<float, float>(float v) { return v; }
template <> __device__ __forceinline__ float  convert_elem<float, __half>(__half v) { return __half2float(v); }
template <> __device__ __forceinline__ __half convert_elem<__half, float>(float v) { return __float2half_rn(v); }
template <> __device__ __forceinline__ __half convert_elem<__half, __half>(__half v) { return v; }

// 64x64 tile; the transposed copy goes through a padded LDS tile so that both copies are
// written with lanes along the contiguous axis.
template <typename Ti, typename To>
__global__ __launch_bounds__(kBlock) void convert_kernel(const Ti* __restrict__ x, int64_t rows, int64_t cols,
                                                         int64_t ld, To* __restrict__ q, To* __restrict__ qT,
                                                         int64_t grid_x)
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
            const To v = convert_elem<To, Ti>(x[r * ld + c]);
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

// ------------------------------------------------------------------ standalone dequantize
template <typename To> __device__ __forceinline__ To from_f32(float v);
template <> __device__ __forceinline__ float  from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ __half from_f32<__half>(float v) { return __float2half_rn(v); }

template <typename Ti, typename To, int V>
__global__ __launch_bounds__(kBlock) void dequantize_kernel(const Ti* __restrict__ a, int64_t rows, int64_t cols,
                                                            int64_t ld, const float* __restrict__ rs,
                                                            const float* __restrict__ cs, float ts,
                                                            const float* __restrict__ cb, To* __restrict__ y)
{
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
        const float frow = rs ? rs[r] : 1.0f;
        alignas(16) To out[V];
#pragma unroll
        for(int e = 0; e < V; ++e)
        {
            float v = static_cast<float>(in[e]) * ts;
            v       = v * frow;
            if(cs) v = v * cs[c + e];
            if(cb) v = v + cb[c + e];
            out[e] = from_f32<To>(v);
        }
        To* dst = y + r * cols + c;
        if(V == 4 && sizeof(To) == 4)
            *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(out);
        else if(V == 4 && sizeof(To) == 2)
            *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(out);
        else
            dst[0] = out[0];
    }
}

// ------------------------------------------------------------------ column sums (bias gradient)
// Stage 1: block (bx, by) sums rows by, by+gridDim.y, ... of a strip of columns.  Lanes own
// adjacent columns (one 16-byte vector each when VEC); the block's row lanes are folded
// through LDS, so partial[by][c] holds one value per block row.
template <typename T, bool VEC>
__global__ __launch_bounds__(kBlock) void colsum_kernel(const T* __restrict__ x, int64_t rows, int64_t cols, int tpr,
                                                        float* __restrict__ partial)
{
    constexpr int E   = VEC ? Vec16<T>::N : 1;
    __shared__ float lds[kBlock * E];
    const int     rpb = kBlock / tpr;                       // row lanes per block
    const int     tc = threadIdx.x % tpr, tr = threadIdx.x / tpr;
    const int64_t c0  = (static_cast<int64_t>(blockIdx.x) * tpr + tc) * E;
    const int64_t S   = static_cast<int64_t>(gridDim.y) * rpb;
    float acc[E];
#pragma unroll
    for(int e = 0; e < E; ++e) acc[e] = 0.0f;
    if(c0 < cols)
    {
        for(int64_t r = static_cast<int64_t>(blockIdx.y) * rpb + tr; r < rows; r += S)
        {
            if(VEC)
            {
                float v[Vec16<T>::N];
                Vec16<T>::load(x + r * cols + c0, v);
#pragma unroll
                for(int e = 0; e < E; ++e) acc[e] += v[e];
            }
            else
                acc[0] += to_f32(x[r * cols + c0]);
        }
    }
#pragma unroll
    for(int e = 0; e < E; ++e) lds[(tr * tpr + tc) * E + e] = acc[e];
    __syncthreads();
    if(tr == 0 && c0 < cols)
    {
        for(int q = 1; q < rpb; ++q)
#pragma unroll
            for(int e = 0; e < E; ++e) acc[e] += lds[(q * tpr + tc) * E + e];
#pragma unroll
        for(int e = 0; e < E; ++e) partial[static_cast<int64_t>(blockIdx.y) * cols + c0 + e] = acc[e];
    }
}

// Stage 2: 16 columns per block; sixteen threads per column fold a sixteenth of the partials
// each (fixed assignment, fixed order), then the sixteen are added in order.
__global__ __launch_bounds__(kBlock) void colsum_finalize_kernel(const float* __restrict__ partial, int S, int64_t cols,
                                                                 float* __restrict__ out)
{
    __shared__ float lds[kBlock];
    const int     tc = threadIdx.x % 16, q = threadIdx.x / 16;
    const int64_t c  = static_cast<int64_t>(blockIdx.x) * 16 + tc;
    float         acc = 0.0f;
    if(c < cols)
        for(int s = q; s < S; s += 16) acc += partial[static_cast<int64_t>(s) * cols + c];
    lds[threadIdx.x] = acc;
    __syncthreads();
    if(q == 0 && c < cols)
    {
        float t = 0.0f;
        for(int i = 0; i < 16; ++i) t += lds[i * 16 + tc];
        out[c] = t;
    }
}

int next_pow2(int64_t v)
{
    int p = 1;
    while(p < v) p <<= 1;
    return p;
}

// Column-sum launch shape: threads per row (power of two) and block rows (gridDim.y, at most
// kColsumSplits), aiming at about five hundred blocks.
void colsum_shape(int64_t rows, int64_t cols, int E, int& tpr, int& gy)
{
    const int64_t ncv = (cols + E - 1) / E;
    tpr               = ncv >= kBlock ? kBlock : (next_pow2(ncv) < 2 ? 2 : next_pow2(ncv));
    const int64_t gx  = (ncv + tpr - 1) / tpr;
    const int     rpb = kBlock / tpr;
    int64_t       g   = (512 + gx - 1) / gx;
    const int64_t maxg = (rows + rpb - 1) / rpb;              // no more block rows than row groups
    if(g > maxg) g = maxg;
    if(g > kColsumSplits) g = kColsumSplits;
    if(g < 1) g = 1;
    gy = static_cast<int>(g);
}

}  // namespace

// ======================================================================== launchers
size_t absmax_workspace_bytes(int64_t rows, int64_t cols, int gran)
{
    (void)rows;
    if(gran == kPerTensor) return sizeof(float) * kAbsmaxMaxBlocks;
    if(gran == kPerCol) return sizeof(float) * kAbsmaxColSplits * static_cast<size_t>(cols > 0 ? cols : 0);
    return 0;
}

template <typename T>
static hipError_t absmax_typed(const T* x, int64_t rows, int64_t cols, int64_t ld, int gran, float qmax, float* scale,
                               float* inv_scale, float* amax_opt, float* ws, hipStream_t st)
{
    constexpr int E       = Vec16<T>::N;
    const bool    rows_ok = aligned16(x) && (ld * sizeof(T)) % 16 == 0;
    if(gran == kPerTensor)
    {
        const bool    vec  = aligned16(x) && ld == cols;
        const int64_t work = vec ? (rows * cols) / E : rows * cols;
        int64_t       nb   = (work + kBlock * 8 - 1) / (kBlock * 8);
        nb                 = nb < 1 ? 1 : (nb > kAbsmaxMaxBlocks ? kAbsmaxMaxBlocks : nb);
        if(vec)
            absmax_tensor_kernel<T, true><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, ws);
        else
            absmax_tensor_kernel<T, false><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, ws);
        absmax_tensor_finalize_kernel<<<dim3(1), dim3(kBlock), 0, st>>>(ws, static_cast<int>(nb), qmax, scale,
                                                                        inv_scale, amax_opt);
    }
    else if(gran == kPerRow)
    {
        const int64_t nb = (rows + 3) / 4;
        if(rows_ok)
            absmax_rows_kernel<T, true><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, qmax, scale, inv_scale,
                                                                          amax_opt);
        else
            absmax_rows_kernel<T, false><<<dim3(nb), dim3(kBlock), 0, st>>>(x, rows, cols, ld, qmax, scale, inv_scale,
                                                                           amax_opt);
    }
    else
    {
        const bool    vec = rows_ok && cols % E == 0;
        const int64_t per = static_cast<int64_t>(kWaveSize) * (vec ? E : 1);
        const dim3    grid(static_cast<unsigned>((cols + per - 1) / per), kAbsmaxColSplits / (kBlock / kWaveSize));
        if(vec)
            absmax_cols_kernel<T, true><<<grid, dim3(kBlock), 0, st>>>(x, rows, cols, ld, ws);
        else
            absmax_cols_kernel<T, false><<<grid, dim3(kBlock), 0, st>>>(x, rows, cols, ld, ws);
        absmax_cols_finalize_kernel<<<dim3((cols + kBlock - 1) / kBlock), dim3(kBlock), 0, st>>>(
            ws, kAbsmaxColSplits, cols, qmax, scale, inv_scale, amax_opt);
    }
    return hipGetLastError();
}

hipError_t launch_absmax_scale(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, int gran, float qmax,
                               float* scale, float* inv_scale, float* amax_opt, float* workspace, hipStream_t stream)
{
    if(xdt == kF32)
        return absmax_typed(static_cast<const float*>(x), rows, cols, ld, gran, qmax, scale, inv_scale, amax_opt,
                            workspace, stream);
    return absmax_typed(static_cast<const __half*>(x), rows, cols, ld, gran, qmax, scale, inv_scale, amax_opt,
                        workspace, stream);
}

template <typename T, int RND>
static void quantize_patch_launch(const T* x, int64_t rows, int64_t cols, int64_t ld, float qmax, int gran,
                                  uint64_t seed, uint64_t offset, const float* inv, int8_t* q, int8_t* qT,
                                  hipStream_t st)
{
    const int64_t gx = (cols + kWaveTile - 1) / kWaveTile, gy = (rows + kBlockRows - 1) / kBlockRows;
    const dim3    grid(static_cast<unsigned>(gx * gy));
    if(gran == kPerCol)
        quantize_patch_kernel<T, RND, true><<<grid, dim3(kBlock), 0, st>>>(x, rows, cols, ld, qmax, gran, seed, offset,
                                                                          inv, q, qT, gx);
    else
        quantize_patch_kernel<T, RND, false><<<grid, dim3(kBlock), 0, st>>>(x, rows, cols, ld, qmax, gran, seed,
                                                                           offset, inv, q, qT, gx);
}

template <typename T>
static hipError_t quantize_typed(const T* x, int64_t rows, int64_t cols, int64_t ld, float qmax, int gran, int rnd,
                                 uint64_t seed, uint64_t offset, const float* inv, int8_t* q, int8_t* qT,
                                 hipStream_t st)
{
    const int64_t gx   = (cols + kWaveTile - 1) / kWaveTile, gy = (rows + kBlockRows - 1) / kBlockRows;
    const bool    fast = cols % 8 == 0 && aligned16(x) && (ld * sizeof(T)) % 16 == 0 && (!q || aligned16(q))
                      && (!qT || (aligned16(qT) && rows % 16 == 0)) && gx * gy < (int64_t(1) << 31);
    if(fast)
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

hipError_t launch_quantize_int8(const void* x, int xdt, int64_t rows, int64_t cols, int64_t ld, float qmax, int gran,
                                int rnd, uint64_t seed, uint64_t offset, const float* inv_scale, int8_t* q, int8_t* qT,
                                hipStream_t stream)
{
    if(xdt == kF32)
        return quantize_typed(static_cast<const float*>(x), rows, cols, ld, qmax, gran, rnd, seed, offset, inv_scale,
                              q, qT, stream);
    return quantize_typed(static_cast<const __half*>(x), rows, cols, ld, qmax, gran, rnd, seed, offset, inv_scale, q,
                          qT, stream);
}

template <typename Ti, typename To>
static hipError_t convert_typed(const void* x, int64_t rows, int64_t cols, int64_t ld, void* q, void* qT,
                                hipStream_t st)
{
    const int64_t gx = (cols + 63) / 64, gy = (rows + 63) / 64;
    convert_kernel<Ti, To><<<dim3(static_cast<unsigned>(gx * gy)), dim3(kBlock), 0, st>>>(
        static_cast<const Ti*>(x), rows, cols, ld, static_cast<To*>(q), static_cast<To*>(qT), gx);
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

template <typename Ti, typename To>
static hipError_t dequantize_typed(const void* a, int64_t rows, int64_t cols, int64_t ld, const float* rs,
                                   const float* cs, float ts, const float* cb, void* y, hipStream_t st)
{
    const bool vec = cols % 4 == 0 && ld % 4 == 0 && (reinterpret_cast<uintptr_t>(a) % (4 * sizeof(Ti))) == 0
                  && (reinterpret_cast<uintptr_t>(y) % (4 * sizeof(To))) == 0;
    const int64_t work = vec ? rows * (cols / 4) : rows * cols;
    int64_t       nb   = (work + kBlock - 1) / kBlock;
    nb                 = nb > (1 << 20) ? (1 << 20) : nb;
    if(vec)
        dequantize_kernel<Ti, To, 4><<<dim3(nb), dim3(kBlock), 0, st>>>(static_cast<const Ti*>(a), rows, cols, ld, rs,
                                                                       cs, ts, cb, static_cast<To*>(y));
    else
        dequantize_kernel<Ti, To, 1><<<dim3(nb), dim3(kBlock), 0, st>>>(static_cast<const Ti*>(a), rows, cols, ld, rs,
                                                                       cs, ts, cb, static_cast<To*>(y));
    return hipGetLastError();
}

hipError_t launch_dequantize(const void* a, int adt, int64_t rows, int64_t cols, int64_t ld, const float* row_scale,
                             const float* col_scale, float tensor_scale, const float* col_bias, void* y, int ydt,
                             hipStream_t stream)
{
    if(adt == kI32 && ydt == kF32)
        return dequantize_typed<int32_t, float>(a, rows, cols, ld, row_scale, col_scale, tensor_scale, col_bias, y, stream);
    if(adt == kI32 && ydt == kF16)
        return dequantize_typed<int32_t, __half>(a, rows, cols, ld, row_scale, col_scale, tensor_scale, col_bias, y, stream);
    if(adt == kI8 && ydt == kF32)
        return dequantize_typed<int8_t, float>(a, rows, cols, ld, row_scale, col_scale, tensor_scale, col_bias, y, stream);
    return dequantize_typed<int8_t, __half>(a, rows, cols, ld, row_scale, col_scale, tensor_scale, col_bias, y, stream);
}

size_t colsum_workspace_bytes(int64_t rows, int64_t cols)
{
    (void)rows;
    return sizeof(float) * static_cast<size_t>(kColsumSplits) * static_cast<size_t>(cols > 0 ? cols : 0);
}

template <typename T>
static hipError_t colsum_typed(const T* x, int64_t rows, int64_t cols, float* out, float* ws, hipStream_t st)
{
    constexpr int E   = Vec16<T>::N;
    const bool    vec = aligned16(x) && cols % E == 0;
    int           tpr, gy;
    colsum_shape(rows, cols, vec ? E : 1, tpr, gy);
    const int64_t ncv = (cols + (vec ? E : 1) - 1) / (vec ? E : 1);
    const dim3    grid(static_cast<unsigned>((ncv + tpr - 1) / tpr), static_cast<unsigned>(gy));
    if(vec)
        colsum_kernel<T, true><<<grid, dim3(kBlock), 0, st>>>(x, rows, cols, tpr, ws);
    else
        colsum_kernel<T, false><<<grid, dim3(kBlock), 0, st>>>(x, rows, cols, tpr, ws);
    colsum_finalize_kernel<<<dim3((cols + 15) / 16), dim3(kBlock), 0, st>>>(ws, gy, cols, out);
    return hipGetLastError();
}

hipError_t launch_colsum(const void* x, int xdt, int64_t rows, int64_t cols, float* out, float* workspace,
                         hipStream_t stream)
{
    if(xdt == kF32) return colsum_typed(static_cast<const float*>(x), rows, cols, out, workspace, stream);
    return colsum_typed(static_cast<const __half*>(x), rows, cols, out, workspace, stream);
}

}  // namespace qsync
