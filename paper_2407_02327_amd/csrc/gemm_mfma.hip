// LDS-tiled MFMA GEMM for gfx950 (CDNA4):  C[M,N] = epilogue( sum_k A[m,k] * B[n,k] ).
//
// Both operands are K-contiguous ("NT"), which is exactly the operand shape of the gfx950
// 32x32 matrix instructions: every lane feeds 16 contiguous K-bytes of one row of A and of
// one row of B (v_mfma_i32_32x32x32_i8: 16 int8; v_mfma_f32_32x32x16_f16: 8 binary16).  The
// INT8 and FP16 kernels therefore move identical bytes and share one tiling:
//
//   * block tile BM x BN, K step of 128 bytes per row; WGM x WGN wavefronts, each owning a
//     (BM/WGM) x (BN/WGN) sub-tile as 32x32 accumulator fragments.  The large tile is
//     256x256 with 8 wavefronts (2 per SIMD, 128 accumulator registers each), so that one
//     wavefront's LDS reads and barrier waits hide behind the other's matrix instructions;
//   * global -> LDS with direct 16-byte loads (global_load_lds_dwordx4), bypassing the VGPRs;
//     LDS rows are 128 bytes.  The LDS of gfx950 serves a 16-byte read in groups of 16 lanes,
//     one 256-byte bank row per group, so the chunk position is XOR-swizzled with (row/2)%8
//     (applied on the global-address side of the direct load): the 16 lanes that read one
//     chunk index of 16 consecutive rows then touch 16 different 16-byte bank groups;
//   * two LDS stages: the next K step streams in while the current one feeds the matrix
//     cores; fragments for the next 32-byte K chunk are requested before the current chunk's
//     matrix instructions; one barrier per K step;
//   * the dequantizer (scalar scales, per-column scale vector, per-column bias) runs on the
//     accumulator registers (the paper fuses dequantization at the same point: before the
//     accumulators are copied to shared memory); the B fragment is fed as the instruction's
//     first operand so that a lane holds four consecutive output columns per register quad,
//     which are packed, passed through the wavefront's private LDS slice and stored to C as
//     16-byte vectors along the rows;
//   * workgroup ids are remapped so that consecutive tiles stay on one XCD (ids are dealt
//     round-robin to the 8 XCDs, each with its own L2) and walk the tile grid in groups of
//     rows, which keeps the A and B panels of neighbouring tiles in that L2;
//   * split-K (for outputs with too few tiles to fill 256 CUs) writes raw partial
//     accumulators to a workspace; a second kernel adds them in a fixed order and applies
//     the epilogue, so results do not depend on scheduling.
#include "device_utils.h"
#include "kernels.h"

#include <cmath>
#include <type_traits>
#include <utility>

namespace qsync {

namespace {

typedef int      v4i32 __attribute__((ext_vector_type(4)));
typedef int      v16i32 __attribute__((ext_vector_type(16)));
typedef float    v16f32 __attribute__((ext_vector_type(16)));
typedef _Float16 v8f16 __attribute__((ext_vector_type(8)));
typedef unsigned v4u32 __attribute__((ext_vector_type(4)));

constexpr int kRowBytes   = 128;  // K bytes per tile row and per LDS row
constexpr int kChunks     = 8;    // 16-byte chunks per LDS row
constexpr int kNumXcd     = 8;
constexpr int kNumCu      = 256;  // compute units of the target: one persistent workgroup each
constexpr int kPersistentLdsBytes = 159744;   // two 64 KB stages, hand-over area, column parameters
constexpr int kGroupM     = 8;    // tile rows walked together (default; GemmKernelArgs::group_m)

struct I8Traits
{
    typedef int32_t acc_t;
    typedef v16i32  accv_t;
    static constexpr int kElemBytes = 1;
    __device__ static __forceinline__ accv_t mfma(const v4i32& a, const v4i32& b, const accv_t& c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    }
};
struct F16Traits
{
    typedef float  acc_t;
    typedef v16f32 accv_t;
    static constexpr int kElemBytes = 2;
    __device__ static __forceinline__ accv_t mfma(const v4i32& a, const v4i32& b, const accv_t& c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8f16, a), __builtin_bit_cast(v8f16, b), c, 0,
                                                      0, 0);
    }
};

// fp32 operands: a lane's 16 K-bytes are four floats of one row; the 32x32x2 instruction takes one float per
// lane (rows lane%32, K index lane/32), so the four components feed four instructions.  Every instruction pairs
// the same components of A and B, i.e. the same K indices: the K axis is merely visited in a different order.
struct F32Traits
{
    typedef float  acc_t;
    typedef v16f32 accv_t;
    static constexpr int kElemBytes = 4;
    __device__ static __forceinline__ accv_t mfma(const v4i32& a, const v4i32& b, const accv_t& c)
    {
        typedef float v4f32 __attribute__((ext_vector_type(4)));
        const v4f32 fa = __builtin_bit_cast(v4f32, a), fb = __builtin_bit_cast(v4f32, b);
        accv_t      r  = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.x, fb.x, c, 0, 0, 0);
        r              = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.y, fb.y, r, 0, 0, 0);
        r              = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.z, fb.z, r, 0, 0, 0);
        return __builtin_amdgcn_mfma_f32_32x32x2f32(fa.w, fb.w, r, 0, 0, 0);
    }
};

struct GemmKernelArgs
{
    const uint8_t* A;
    const uint8_t* B;
    int64_t        M, N;
    int64_t        Kb;           // bytes per operand row (K * element size), multiple of 16
    void*          C;
    int            c_is_f16;
    const float*   s0;
    const float*   s1;
    const float*   col_scale;
    const float*   col_bias;
    int32_t*       acc_dump;
    void*          partial;      // split-K: [splits][M][N] raw accumulators
    int            ktiles_per_split;
    int            tiles_m, tiles_n;
    int            group_m;      // tile rows that the tile walk keeps together (see item_of_block)
    int            conv_H, conv_W, conv_Cb;   // implicit 3x3 patch matrix: image height, width, bytes per pixel
    // B rows remapped (weight gradient of a 3x3 convolution): logical row (tap, c) = tap*remap_C + c is physical
    // row (tap%3)*remap_C + c of B, read with its K axis displaced by (tap/3 - 1)*remap_shift bytes
    int            remap_C, remap_shift;
    // optional: running maximum of |C| as stored (bit pattern of a non-negative fp32), raised with one atomic
    // maximum per workgroup
    unsigned int*  amax_bits;
    // optional: fixed-point codes of C as stored, clamp(round(C * code_inv[0]), -code_qmax, code_qmax), [M][N] int8
    int8_t*        codes;
    const float*   code_inv;
    int            code_qmax;
};

// Work item (K split, tile) of a workgroup.  Workgroups are dealt round-robin to the eight XCDs
// in launch order, each with its own L2, so XCD x takes the x-th contiguous eighth of the item
// list (split-major, tiles in grouped row-major order inside a split): the workgroups that share
// an L2 then read neighbouring operand panels, and with split K also the same K range.
__device__ __forceinline__ void item_of_block(int lin, int tiles_m, int tiles_n, int splits, int group_m, int& split,
                                              int& tm, int& tn)
{
    const int tiles = tiles_m * tiles_n, total = tiles * splits;
    const int per = total / kNumXcd, rem = total % kNumXcd;
    const int xcd = lin % kNumXcd, loc = lin / kNumXcd;
    const int item  = xcd * per + (xcd < rem ? xcd : rem) + loc;
    split           = item / tiles;
    const int L     = item - split * tiles;
    const int width = group_m * tiles_n;
    const int group = L / width, first = group * group_m;
    const int gsz   = (tiles_m - first) < group_m ? (tiles_m - first) : group_m;
    const int in    = L - group * width;
    // the divisions run on the vector unit; hand the (uniform) results back as scalars
    split = __builtin_amdgcn_readfirstlane(split);
    tm    = __builtin_amdgcn_readfirstlane(first + in % gsz);
    tn    = __builtin_amdgcn_readfirstlane(in / gsz);
}

// Output value a*s + b of the fused epilogues.  fp32: the fused multiply-add.  binary16: the same sum rounded ONCE
// to binary16, by the mixed-precision fused multiply-add (fp32 sources, binary16 result) -- written as an
// instruction so that every epilogue (per-tile staged and element-wise, persistent) produces the same bits; left to
// the compiler, fmaf + conversion becomes that instruction in some places and a fp32 result converted afterwards
// (two roundings, different at binary16 ties) in others.
template <typename T> __device__ __forceinline__ T fma_out(float a, float s, float b);
template <> __device__ __forceinline__ float fma_out<float>(float a, float s, float b) { return fmaf(a, s, b); }
template <> __device__ __forceinline__ __half fma_out<__half>(float a, float s, float b)
{
    uint32_t r;
    asm("v_fma_mixlo_f16 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(s), "v"(b));
    return __ushort_as_half(static_cast<unsigned short>(r & 0xFFFFu));
}
// two of them packed in one word (first value in the low half)
__device__ __forceinline__ uint32_t fma_out_half2(float a0, float s0, float b0, float a1, float s1, float b1)
{
    uint32_t r;
    asm("v_fma_mixlo_f16 %0, %1, %2, %3\n\tv_fma_mixhi_f16 %0, %4, %5, %6"
        : "=&v"(r) : "v"(a0), "v"(s0), "v"(b0), "v"(a1), "v"(s1), "v"(b1));
    return r;
}

// One direct global->LDS load of 16 bytes per lane.  D selects the wavefront's D-th 1 KB slot
// relative to the shared LDS base `lds_mid` (which points DPW/2 KB into the wavefront's slice).
// The hardware adds the instruction's immediate offset to the LDS address and to the global
// address alike.  The global address is formed as uniform base + 32-bit lane offset (scalar base
// addressing), so the K loop spends no vector instructions on addresses: `sbase` is the
// operand panel's address at this K tile minus kDmaBias, and `voff` already contains
// + kDmaBias - IMM.
constexpr int kDmaBias = 4096;
// A wavefront's DPW loads are issued in groups of at most 8 that share one LDS base (the immediate reaches
// +-4 KB); a wavefront with 16 loads per K tile changes the base once in between.
template <int DPW> constexpr int dma_group() { return DPW > 8 ? 8 : DPW; }
template <int D, int DPW> constexpr int dma_imm() { return (D % dma_group<DPW>() - dma_group<DPW>() / 2) * 1024; }   // -4096 .. 3072
template <int D, int DPW> constexpr int dma_lds_shift() { return (D / dma_group<DPW>()) * dma_group<DPW>() * 1024; }
template <int D, int DPW>
__device__ __forceinline__ void dma_issue(const uint8_t* sbase, uint32_t voff, uint8_t* lds_mid)
{
    constexpr int IMM = dma_imm<D, DPW>();
    static_assert(IMM >= -4096 && IMM <= 4095, "immediate offset out of range");
    asm volatile("" : "+v"(voff));      // keep the widening of the lane offset next to the load (scalar-base form)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(sbase + voff),
                                     (__attribute__((address_space(3))) void*)(lds_mid + dma_lds_shift<D, DPW>()), 16, IMM, 0);
}

template <int DPW, int... Ds>
__device__ __forceinline__ void dma_sequence(std::integer_sequence<int, Ds...>, const uint8_t* sbase,
                                             const uint32_t (&voff)[DPW], uint8_t* lds_mid)
{
    (dma_issue<Ds, DPW>(sbase, voff[Ds], lds_mid), ...);
}

// Last, partial K tile: a chunk past the end of K is fetched from the row's first chunk instead
// (and overwritten with zeros once landed).
template <int DPW, int... Ds>
__device__ __forceinline__ void dma_sequence_tail(std::integer_sequence<int, Ds...>, const uint8_t* sbase,
                                                  const uint32_t (&voff)[DPW], const int (&gchunk)[2], int64_t kb,
                                                  int64_t Kb, uint8_t* lds_mid)
{
    (dma_issue<Ds, DPW>(sbase, voff[Ds] - ((kb + gchunk[Ds & 1] >= Kb) ? gchunk[Ds & 1] : 0), lds_mid), ...);
}

// Implicit patch matrix of a 3x3 / stride 1 / pad 1 convolution over an NHWC tensor: row m of A is
// output pixel m, its K axis runs (kh, kw, c).  A 16-byte chunk lies inside one tap because the
// pixel size is a multiple of 16 bytes, so the direct load of a lane either reads 16 bytes of the
// neighbouring pixel (same image, inside the border) or, for padding and for chunks past the end
// of K, 16 zero bytes from a constant block.
__device__ uint4 g_zero_chunk;     // never written: static storage starts at zero

struct ConvTap { int delta[2]; int dh[2]; int dw[2]; bool valid[2]; };     // per chunk parity of the lane

template <int D, int DPW>
__device__ __forceinline__ void conv_issue(const uint8_t* a, const uint8_t* zero, uint32_t pix_off, uint32_t hw,
                                           const ConvTap& t, int H, int W, uint8_t* lds_mid)
{
    constexpr int IMM = dma_imm<D, DPW>();
    constexpr int par = D & 1;
    const int  hh  = static_cast<int>(hw >> 16) + t.dh[par], ww = static_cast<int>(hw & 0xffffu) + t.dw[par];
    const bool inb = t.valid[par] && static_cast<unsigned>(hh) < static_cast<unsigned>(H)
                     && static_cast<unsigned>(ww) < static_cast<unsigned>(W);
    const uint8_t* src = inb ? a + static_cast<int64_t>(static_cast<int32_t>(pix_off) + t.delta[par]) : zero;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src - IMM),
                                     (__attribute__((address_space(3))) void*)(lds_mid + dma_lds_shift<D, DPW>()), 16, IMM, 0);
}

template <int DPW, int... Ds>
__device__ __forceinline__ void conv_sequence(std::integer_sequence<int, Ds...>, const uint8_t* a, const uint8_t* zero,
                                              const uint32_t (&pix_off)[DPW], const uint32_t (&hw)[DPW],
                                              const ConvTap& t, int H, int W, uint8_t* lds_mid)
{
    (conv_issue<Ds, DPW>(a, zero, pix_off[Ds], hw[Ds], t, H, W, lds_mid), ...);
}

// TN form with the B operand gathered from an NHWC tensor (weight gradient of the 3x3 convolution): stage row r of
// K tile kt is pixel m = kt * KR + r, and a lane's 16-byte chunk lies in one tap (dh, dw) at channel offset c0, both
// fixed per load slot; what changes from K tile to K tile is the pixel, i.e. (h, w).  `delta` holds the slot's whole
// constant part ((dh W + dw) Cb + c0 + r Cb); `code` = (dh + 1) | (dw + 1) << 2 | valid << 4; `hw` = h << 16 | w of the
// pixel of the NEXT K tile to be requested and is advanced by KR pixels here (dr = KR % W, hq = (KR / W) % H).
template <int D, int DPW>
__device__ __forceinline__ void conv_tn_issue(const uint8_t* x, const uint8_t* zero, int64_t pix_base, int delta, int code,
                                              uint32_t& hw, int H, int W, int dr, int hq, uint8_t* lds_mid)
{
    constexpr int IMM = dma_imm<D, DPW>();
    int        h = static_cast<int>(hw >> 16), w = static_cast<int>(hw & 0xffffu);
    const int  hh = h + (code & 3) - 1, ww = w + ((code >> 2) & 3) - 1;
    const bool inb = (code >> 4) != 0 && static_cast<unsigned>(hh) < static_cast<unsigned>(H)
                     && static_cast<unsigned>(ww) < static_cast<unsigned>(W);
    const uint8_t* src = inb ? x + (pix_base + delta) : zero;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src - IMM),
                                     (__attribute__((address_space(3))) void*)(lds_mid + dma_lds_shift<D, DPW>()), 16, IMM, 0);
    w += dr;
    const int carry = w >= W ? 1 : 0;
    w -= carry ? W : 0;
    h += hq + carry;
    h -= h >= H ? H : 0;
    hw = (static_cast<uint32_t>(h) << 16) | static_cast<uint32_t>(w);
}

template <int DPW, int... Ds>
__device__ __forceinline__ void conv_tn_sequence(std::integer_sequence<int, Ds...>, const uint8_t* x, const uint8_t* zero,
                                                 int64_t pix_base, const int (&delta)[DPW], const int (&code)[DPW],
                                                 uint32_t (&hw)[DPW], int H, int W, int dr, int hq, uint8_t* lds_mid)
{
    (conv_tn_issue<Ds, DPW>(x, zero, pix_base, delta[Ds], code[Ds], hw[Ds], H, W, dr, hq, lds_mid), ...);
}

template <int DPW, int... Ds>
__device__ __forceinline__ void fill_dma_imms(int (&imm)[DPW], std::integer_sequence<int, Ds...>)
{
    ((imm[Ds] = dma_imm<Ds, DPW>()), ...);
}

__device__ __forceinline__ int swizzle(int row, int chunk) { return (chunk ^ ((row >> 1) & 7)) << 4; }

// Maximum magnitude of the 16 output bytes in `v`, folded into `run`: binary16 magnitudes order like their bit
// patterns without the sign (two per dword), fp32 magnitudes likewise (one per dword).
typedef unsigned short gus2_t __attribute__((ext_vector_type(2)));
template <int OS> __device__ __forceinline__ uint32_t fold_abs_bits(uint32_t run, const v4u32& v)
{
#pragma unroll
    for(int k = 0; k < 4; ++k)
    {
        if(OS == 2)
            run = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(gus2_t, run),
                                                                         __builtin_bit_cast(gus2_t, v[k] & 0x7FFF7FFFu)));
        else
        {
            const uint32_t u = v[k] & 0x7FFFFFFFu;
            run = run > u ? run : u;
        }
    }
    return run;
}
// the folded maximum as the bit pattern of an fp32
template <int OS> __device__ __forceinline__ uint32_t abs_bits_as_f32(uint32_t run)
{
    if(OS == 4) return run;
    const uint32_t h = (run & 0xFFFFu) > (run >> 16) ? (run & 0xFFFFu) : (run >> 16);
    return __float_as_uint(__half2float(__ushort_as_half(static_cast<unsigned short>(h))));
}

// One 16-byte LDS read per fragment of a set, as explicit instructions (the waits are placed by hand in the
// K loop): fragment I lies I * 32 rows further, which fits the instruction's immediate offset.
template <int I>
__device__ __forceinline__ void frag_read(v4i32& dst, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(I * 32 * kRowBytes) : "memory");
}
typedef unsigned v2u32 __attribute__((ext_vector_type(2)));
// compile-time loop: f(std::integral_constant<int, 0>), ..., f(std::integral_constant<int, N - 1>)
template <typename F, int... Is> __device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}
// Transposing 8-byte reads, sixteen lanes at a time.  ESZ 1: the lanes read 8 rows x 16 bytes (lane s: half s%2 of
// row s/2) and lane j receives the eight bytes of column j.  ESZ 2: they read 4 rows x 32 bytes (lane s: quarter
// s%4 of row s/4) and lane j receives the four 16-bit elements of column j.
template <int ESZ, int OFF> __device__ __forceinline__ void frag_read_tr(v2u32& dst, uint32_t addr)
{
    static_assert(OFF >= 0 && OFF < 65536, "immediate offset");
    if constexpr(ESZ == 1)
        asm volatile("ds_read_b64_tr_b8 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
    else
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}
// XOR term (in 16-byte chunks) of stage row `row` of a TN operand region whose rows are RB bytes long: the rows that
// one pass of a transposing read touches (8 rows x 32 bytes for ESZ 1, 4 rows x 64 bytes for ESZ 2) land in
// different bank groups.  Unchanged by the row steps between the reads of one lane (multiples of 8, resp. 4).
template <int ESZ, int RB> __device__ __forceinline__ int tn_swizzle(int row)
{
    constexpr int CPR = RB / 16;                                    // chunks per row
    if constexpr(ESZ == 1) return 2 * ((row / (16 / CPR)) % (CPR / 2));
    else                   return RB >= 256 ? 4 * (row % 4) : 4 * ((row / 2) % 2);
}
template <int F, int... Is>
__device__ __forceinline__ void frag_reads(v4i32 (&dst)[F], uint32_t addr, std::integer_sequence<int, Is...>)
{
    (frag_read<Is>(dst[Is], addr), ...);
}

// TN (int8 and binary16): both operands are handed over with the contraction axis as their ROW axis, A [P, M] and
// B [P, N] row-major (C[m,n] = sum_p A[p,m] B[p,n]): the weight gradient dW = dY^T X straight from the row-major
// operands, no transposed copies.  A stage then holds 128 (int8) or 64 (binary16) contraction rows of each operand
// (rows of BM / BN elements), and the fragments come out of LDS through the transposing reads of gfx950
// (ds_read_b64_tr_b8 / _b16): sixteen lanes read 8 rows x 16 bytes (4 rows x 32 bytes) and receive, lane j, the
// eight (four) elements of column j -- consecutive contraction indices of one output row, which is what the
// matrix instruction wants; two reads make a lane's 16 operand bytes.  16-byte chunks are XOR-swizzled per row so
// that the lanes of one access pass touch all banks once.  Everything behind the fragments
// (matrix instructions, epilogue, split K) is shared with the NT form.  Kb is the contraction length P here.
template <typename TR, int BM, int BN, int WGM, int WGN, bool SPLIT, bool CONV = false, bool TN = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_nt_kernel(const GemmKernelArgs p)
{
    static_assert(!(SPLIT && CONV && !TN), "the implicit patch matrix of the forward is not combined with split K");
    static_assert(!TN || (TR::kElemBytes <= 2 && BM == BN && BM >= 64), "TN: int8 or binary16 operands, square tiles");
    constexpr bool CONVA  = CONV && !TN;       // NT form: the A operand is the implicit patch matrix (forward, data gradient)
    constexpr bool CONVTN = CONV && TN;        // TN form: the B operand is gathered from the NHWC tensor (weight gradient)
    constexpr int ESZ = TR::kElemBytes;
    typedef typename TR::accv_t accv_t;
    typedef typename TR::acc_t  acc_t;
    constexpr int kThreads = 64 * WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;   // wavefront sub-tile
    constexpr int FM = WTM / 32, FN = WTN / 32;     // 32x32 fragments per wavefront
    constexpr int STAGE_BYTES = (BM + BN) * kRowBytes;
    constexpr int DPW = (BM + BN) / 8 / (WGM * WGN);    // direct-load instructions per wavefront per K tile
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wavefront sub-tiles are made of 32x32 fragments");
    static_assert((BM + BN) % (8 * WGM * WGN) == 0 && BM % 16 == 0, "stage rows must split evenly over the wavefronts");

    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

    int split, tm, tn;
    item_of_block(static_cast<int>(blockIdx.y * gridDim.x + blockIdx.x), p.tiles_m, p.tiles_n, SPLIT ? static_cast<int>(gridDim.y) : 1, p.group_m,
                  split, tm, tn);
    const int64_t m0 = static_cast<int64_t>(tm) * BM, n0 = static_cast<int64_t>(tn) * BN;
    const int     tid = threadIdx.x, lane = tid % kWaveSize;
    const int     wave = __builtin_amdgcn_readfirstlane(tid / kWaveSize);     // wavefront index, held in an SGPR
    const int     wm = wave / WGN, wn = wave % WGN;

    // K-tile indices are 32-bit so that the loop control stays on the scalar unit
    const int ktiles_all = static_cast<int>((p.Kb + kRowBytes - 1) / kRowBytes);
    const int tail_kt    = (p.Kb % kRowBytes) ? ktiles_all - 1 : -1;     // index of a partial last tile, if any
    int       kt_begin = 0, kt_end = ktiles_all;
    if(SPLIT)
    {
        kt_begin = split * p.ktiles_per_split;
        kt_end   = kt_begin + p.ktiles_per_split < ktiles_all ? kt_begin + p.ktiles_per_split : ktiles_all;
    }

    // Global -> LDS with direct loads (global_load_lds_dwordx4): the data never passes through
    // VGPRs and no LDS store instruction is issued.  One such instruction of a wavefront fills
    // 1 KB of LDS = 8 consecutive stage rows (A rows first, then B rows): lane l lands at row l/8,
    // chunk position l%8, so it fetches the logical chunk (l%8) ^ ((row/2)%8) of that row.
    // Rows beyond M (or N) are clamped to the last row: they only feed accumulators of outputs
    // that are never stored.  Chunks beyond the end of K (last, partial K tile only) are
    // fetched from the row's first chunk of that tile and overwritten with zeros once landed.
    // A wavefront's DPW instructions cover 8*DPW consecutive stage rows, all of A or all of B, so
    // its source is one uniform base pointer plus a 32-bit lane offset per instruction.
    constexpr bool kUniformSide = (BM / 8) % DPW == 0;
    static_assert(kUniformSide, "a wavefront must not straddle the A/B boundary of a stage");
    const bool     is_a      = wave * DPW < BM / 8;
    // TN: the panel starts at the tile's first column of the operand (its rows are contraction indices)
    const uint8_t* gbase     = TN ? (is_a ? p.A + m0 * ESZ : (CONVTN ? p.B : p.B + n0 * ESZ))
                                  : (is_a ? p.A + m0 * p.Kb : ((!CONV && p.remap_C > 0) ? p.B : p.B + n0 * p.Kb));
    const int64_t  rows_left = is_a ? p.M - m0 : p.N - n0;           // >= 1
    uint32_t       voff[DPW];                                         // lane offset + kDmaBias - immediate
    uint32_t       hw[CONV ? DPW : 1];                                // CONV: (h << 16) | w of the lane's pixels
    int            tnc_delta[CONVTN ? DPW : 1], tnc_code[CONVTN ? DPW : 1];      // CONVTN, B side (see conv_tn_issue)
    int            gchunk[2];                                         // the swizzle term depends on d%2 only
    {
        int imm[DPW];
        fill_dma_imms<DPW>(imm, std::make_integer_sequence<int, DPW>{});
        if constexpr(TN)
        {   // instruction q of the stage fills LDS bytes [1024 q, 1024 q + 1024) of the A region (128 / ESZ rows of
            // BM elements), then of the B region; a lane's 16 bytes are chunk (position ^ swizzle(row)) of its row
            constexpr int RB = BM * ESZ;                                   // bytes per region row
            const int64_t ld    = (is_a ? p.M : p.N) * ESZ;                // operand row length in bytes
            const int64_t width = (is_a ? p.M - m0 : p.N - n0) * ESZ;      // valid bytes of this tile's columns (>= 16)
#pragma unroll
            for(int d = 0; d < DPW; ++d)
            {
                const int q     = wave * DPW + d - (is_a ? 0 : BM / 8);
                const int o     = q * 1024 + lane * 16;
                const int row   = o / RB, pos = (o % RB) / 16;
                int       chunk = pos ^ tn_swizzle<ESZ, RB>(row);
                if constexpr(CONVTN)
                    if(!is_a)
                    {   // B side: column byte (n0 * ESZ + 16 chunk) of the implicit [pixels, 9 C] matrix = tap, channel offset
                        constexpr int KR = kRowBytes / ESZ;                       // pixels per K tile
                        const int64_t colb  = n0 * ESZ + static_cast<int64_t>(chunk) * 16;
                        const bool    valid = colb < static_cast<int64_t>(9) * p.conv_Cb;      // tile columns past 9 C: zeros, never stored
                        const int     tap   = valid ? static_cast<int>(colb / p.conv_Cb) : 0;
                        const int     c0    = valid ? static_cast<int>(colb - static_cast<int64_t>(tap) * p.conv_Cb) : 0;
                        const int     kh = (tap * 11) >> 5, kw = tap - 3 * kh;          // tap / 3 for tap < 12
                        tnc_delta[d] = ((kh - 1) * p.conv_W + (kw - 1)) * p.conv_Cb + c0 + row * p.conv_Cb;
                        tnc_code[d]  = kh | (kw << 2) | (valid ? 16 : 0);
                        const uint32_t m  = static_cast<uint32_t>(kt_begin) * KR + static_cast<uint32_t>(row);
                        const uint32_t qq = m / static_cast<uint32_t>(p.conv_W);
                        hw[d]   = ((qq % static_cast<uint32_t>(p.conv_H)) << 16) | (m - qq * static_cast<uint32_t>(p.conv_W));
                        voff[d] = 0u;
                        continue;
                    }
                if(static_cast<int64_t>(chunk) * 16 >= width) chunk = 0;    // columns past the matrix: any valid chunk, never stored
                voff[d] = static_cast<uint32_t>(static_cast<int64_t>(row) * ld + chunk * 16 + kDmaBias - imm[d]);
            }
            gchunk[0] = gchunk[1] = 0;
        }
        else
#pragma unroll
        for(int d = 0; d < DPW; ++d)
        {
            const int srow  = (wave * DPW + d) * 8 + lane / 8;            // row inside the stage
            const int chunk = (lane % 8) ^ ((srow >> 1) & 7);             // BM % 16 == 0: same term for A and B rows
            int64_t   lrow  = srow - (is_a ? 0 : BM);
            if(lrow >= rows_left) lrow = rows_left - 1;
            voff[d] = static_cast<uint32_t>(lrow * p.Kb + chunk * 16 + kDmaBias - imm[d]);
            if(!CONV && p.remap_C > 0 && !is_a)
            {   // offset from p.B itself (the base below is not advanced to this tile's rows)
                const int64_t row = n0 + lrow;
                const int     tap = static_cast<int>(row / p.remap_C), c = static_cast<int>(row - static_cast<int64_t>(tap) * p.remap_C);
                const int     kh = (tap * 11) >> 5, kw = tap - 3 * kh;          // tap / 3 for tap < 12
                voff[d] = static_cast<uint32_t>(static_cast<int64_t>(kw * p.remap_C + c) * p.Kb + (kh - 1) * p.remap_shift
                                                + chunk * 16 + kDmaBias - imm[d]);
            }
            if constexpr(CONVA)
                if(is_a)
                {   // A side: voff holds the byte offset of output pixel m in the NHWC tensor instead
                    const uint32_t m = static_cast<uint32_t>(m0 + lrow), q = m / static_cast<uint32_t>(p.conv_W);
                    voff[d] = m * static_cast<uint32_t>(p.conv_Cb);
                    hw[d]   = ((q % static_cast<uint32_t>(p.conv_H)) << 16) | (m - q * static_cast<uint32_t>(p.conv_W));
                }
            if(d < 2) gchunk[d] = chunk * 16;
        }
    }
    // the panel base as two scalar registers (the wavefront index is uniform, so is the choice of panel)
    const uint64_t gbits = reinterpret_cast<uint64_t>(gbase) - kDmaBias;
    // (the builtin returns a signed int: widen each half through uint32_t, never by sign extension)
    const uint32_t glo    = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(gbits))));
    const uint32_t ghi    = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(gbits >> 32))));
    const uint8_t* sbase0 = reinterpret_cast<const uint8_t*>((static_cast<uint64_t>(ghi) << 32) | static_cast<uint64_t>(glo));
    // All DPW instructions of a wavefront share one LDS base (M0): instruction d reaches its 1 KB
    // slot through the instruction's immediate offset (d - DPW/2) KB.  Rewriting M0 between direct
    // loads would stall the wavefront until the previous load has left the issue queue
    // (measured: +20 % GEMM throughput without it).
    // CONVTN: pixels per K tile, and how far (h, w) of a stage row move from one K tile to the next
    constexpr int tnc_KR = kRowBytes / ESZ;
    const int     tnc_dr = CONVTN ? tnc_KR % p.conv_W : 0, tnc_hq = CONVTN ? (tnc_KR / p.conv_W) % p.conv_H : 0;
    auto dma = [&](int stage, int kt) {
        const int64_t  kb    = static_cast<int64_t>(kt) * kRowBytes;
        uint8_t*       lbase = lds + stage * STAGE_BYTES + wave * (DPW * 1024) + (dma_group<DPW>() / 2) * 1024;
        if constexpr(CONVTN)
            if(!is_a)
            {   // (requested for consecutive K tiles only, starting at kt_begin: hw is advanced by every call)
                conv_tn_sequence<DPW>(std::make_integer_sequence<int, DPW>{}, p.B, reinterpret_cast<const uint8_t*>(&g_zero_chunk),
                                      static_cast<int64_t>(kt) * tnc_KR * p.conv_Cb, tnc_delta, tnc_code, hw, p.conv_H, p.conv_W,
                                      tnc_dr, tnc_hq, lbase);
                return;
            }
        if constexpr(CONVA)
            if(is_a)
            {
                ConvTap t;
#pragma unroll
                for(int par = 0; par < 2; ++par)
                {
                    const uint32_t koff = static_cast<uint32_t>(kb) + static_cast<uint32_t>(gchunk[par]);
                    const uint32_t tap  = koff / static_cast<uint32_t>(p.conv_Cb);
                    const int      c0   = static_cast<int>(koff - tap * static_cast<uint32_t>(p.conv_Cb));
                    const int      kh   = static_cast<int>((tap * 11u) >> 5);         // tap / 3 for tap < 12
                    const int      kw   = static_cast<int>(tap) - 3 * kh;
                    t.dh[par]    = kh - 1;
                    t.dw[par]    = kw - 1;
                    t.delta[par] = ((kh - 1) * p.conv_W + (kw - 1)) * p.conv_Cb + c0;
                    t.valid[par] = static_cast<int64_t>(koff) < p.Kb;
                }
                conv_sequence<DPW>(std::make_integer_sequence<int, DPW>{}, p.A,
                                   reinterpret_cast<const uint8_t*>(&g_zero_chunk), voff, hw, t, p.conv_H, p.conv_W, lbase);
                return;
            }
        const uint8_t* sb    = TN ? sbase0 + kb * (is_a ? p.M : p.N) : sbase0 + kb;      // TN: 128 operand rows further
        asm volatile("" : "+s"(sb));      // keep base + K offset a scalar pair: the lane offsets stay loop-invariant 32-bit values
        if(!TN && kt == tail_kt)
            dma_sequence_tail<DPW>(std::make_integer_sequence<int, DPW>{}, sb, voff, gchunk, kb, p.Kb, lbase);
        else
            dma_sequence<DPW>(std::make_integer_sequence<int, DPW>{}, sb, voff, lbase);
    };
    // Waits for this wavefront's direct loads and for its outstanding fragment reads (the barrier hands the
    // stage they read to the next direct load, and the compiler does not see those reads), zero-fills its
    // out-of-K chunks, then joins the block.
    auto land = [&](int stage, int kt) {
        __builtin_amdgcn_s_waitcnt(0x0070);                       // vmcnt(0), lgkmcnt(0)
        if(!TN && kt == tail_kt)
        {
            const int64_t kb = static_cast<int64_t>(kt) * kRowBytes;
#pragma unroll
            for(int d = 0; d < DPW; ++d)
                if(kb + gchunk[d & 1] >= p.Kb)
                    *reinterpret_cast<uint4*>(lds + stage * STAGE_BYTES + (wave * DPW + d) * 1024 + lane * 16)
                        = make_uint4(0, 0, 0, 0);
        }
        __syncthreads();
    };

    accv_t acc[FM][FN];
#pragma unroll
    for(int i = 0; i < FM; ++i)
#pragma unroll
        for(int j = 0; j < FN; ++j)
#pragma unroll
            for(int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    // Fragment reads: lane -> row lane%32 of a fragment, K chunk 2*ks + lane/32.  The swizzle term
    // (row/2)%8 is the same for every fragment of a lane because fragments start at multiples of 32.
    const int frag_row = lane & 31, khalf = lane >> 5;
    int       roff[4];
#pragma unroll
    for(int ks = 0; ks < 4; ++ks) roff[ks] = frag_row * kRowBytes + swizzle(frag_row, ks * 2 + khalf);
    const int a_base = (wm * WTM) * kRowBytes, b_base = BM * kRowBytes + (wn * WTN) * kRowBytes;

    // The fragment reads are written as instructions with hand-placed waits.  The compiler's own wait
    // insertion treats a direct global->LDS load as an access that may return through either counter, and
    // while one is in flight (always, here) every wait it places on an LDS read becomes "all LDS reads
    // done", including the reads just issued for a later chunk: the wavefront would then sit out a full LDS
    // latency twice per K tile.  LDS reads of a wavefront return in order, so "at most FM + FN outstanding"
    // is exactly "the older of two fragment sets has arrived".
    v4i32          af[2][FM], bf[2][FN];
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) uint8_t*)lds));
    // TN: lane (kb = lane/32, g = (lane%32)/16, s = lane%16) receives row 16 g + s of a fragment.
    // int8: it supplies the 8-byte half s%2 of chunk (first chunk of the sub-tile + 2f + g) of contraction row
    // 32 ks + 16 kb + 8 r + s/2 (r = 0, 1: the two reads of a fragment) and receives contraction indices
    // 32 ks + 16 kb + 8 r + 0..7.  binary16: the 8-byte half s%2 of chunk (first chunk + 4f + 2g + (s%4)/2) of
    // contraction row 16 ks + 8 kb + 4 r + s/4; it receives contraction indices 16 ks + 8 kb + 4 r + 0..3.
    uint32_t tn_a[TN ? FM : 1], tn_b[TN ? FN : 1];
    if constexpr(TN)
    {
        constexpr int RB = BM * ESZ;
        const int s16 = lane & 15, g = (lane >> 4) & 1, kb16 = lane >> 5;
        const int prow = ESZ == 1 ? 16 * kb16 + s16 / 2 : 8 * kb16 + s16 / 4;   // + ks and r steps through the immediate
        const int swz  = tn_swizzle<ESZ, RB>(prow);
        const int lch  = ESZ == 1 ? g : 2 * g + (s16 & 3) / 2;                   // chunk inside the fragment's columns
        constexpr int CPF = 2 * ESZ;                                            // chunks per 32-column fragment
#pragma unroll
        for(int f = 0; f < FM; ++f)
            tn_a[f] = static_cast<uint32_t>(prow * RB + ((((wm * WTM * ESZ) / 16 + CPF * f + lch) ^ swz) * 16) + 8 * (s16 & 1));
#pragma unroll
        for(int f = 0; f < FN; ++f)
            tn_b[f] = static_cast<uint32_t>(128 * BM + prow * RB + ((((wn * WTN * ESZ) / 16 + CPF * f + lch) ^ swz) * 16) + 8 * (s16 & 1));
    }
    auto           load_frags = [&](auto buf_tag, int stage, int ks) {
        constexpr int  buf = decltype(buf_tag)::value;
        if constexpr(TN)
        {
            const uint32_t sb = lds0 + static_cast<uint32_t>(stage * STAGE_BYTES + ks * 32 * BM);
            static_for<FM>([&](auto ft) {
                constexpr int f = decltype(ft)::value;
                v2u32 lo, hi;
                frag_read_tr<ESZ, 0>(lo, sb + tn_a[f]);
                frag_read_tr<ESZ, 8 * BM>(hi, sb + tn_a[f]);
                af[buf][f] = v4i32{static_cast<int>(lo.x), static_cast<int>(lo.y), static_cast<int>(hi.x), static_cast<int>(hi.y)};
            });
            static_for<FN>([&](auto ft) {
                constexpr int f = decltype(ft)::value;
                v2u32 lo, hi;
                frag_read_tr<ESZ, 0>(lo, sb + tn_b[f]);
                frag_read_tr<ESZ, 8 * BN>(hi, sb + tn_b[f]);
                bf[buf][f] = v4i32{static_cast<int>(lo.x), static_cast<int>(lo.y), static_cast<int>(hi.x), static_cast<int>(hi.y)};
            });
            return;
        }
        const uint32_t fa  = lds0 + static_cast<uint32_t>(stage * STAGE_BYTES + a_base + roff[ks]);
        const uint32_t fb  = lds0 + static_cast<uint32_t>(stage * STAGE_BYTES + b_base + roff[ks]);
        frag_reads<FM>(af[buf], fa, std::make_integer_sequence<int, FM>{});
        frag_reads<FN>(bf[buf], fb, std::make_integer_sequence<int, FN>{});
    };
    // lgkmcnt(reads of one fragment set), other counters untouched.  TN issues two reads per fragment (at most 12
    // per set; the counter holds 15 and a wavefront's further LDS instructions wait while it is full).
    constexpr int kReadsPerSet  = TN ? 2 * (FM + FN) : FM + FN;
    static_assert(kReadsPerSet <= 15, "the LDS counter holds 15");
    constexpr int kWaitOlderSet = 0xC07F | (kReadsPerSet << 8);
    constexpr int kWaitAllLds   = 0xC07F;                         // lgkmcnt(0)
    static_assert(FM + FN <= 15, "the LDS counter holds 15");
    auto mma = [&](auto buf_tag) {
        constexpr int buf = decltype(buf_tag)::value;
        __builtin_amdgcn_sched_barrier(0);           // fences: the matrix instructions stay behind the wait in front of them
#pragma unroll
        for(int i = 0; i < FM; ++i)
#pragma unroll
            for(int j = 0; j < FN; ++j) acc[i][j] = TR::mfma(bf[buf][j], af[buf][i], acc[i][j]);
        __builtin_amdgcn_sched_barrier(0);
    };
    const std::integral_constant<int, 0> set0{};
    const std::integral_constant<int, 1> set1{};

    // K pipeline.  A tile has four 32-byte K chunks whose fragments alternate between two
    // register sets: the reads for chunk ks+2 are issued right behind the matrix instructions of
    // chunk ks (into the set those instructions have just consumed), so they complete while
    // chunk ks+1 keeps the matrix cores busy, and every wait in front of a chunk leaves the
    // younger set's reads in flight.  At the tile boundary the wavefront (1) joins the barrier
    // that publishes the next stage (every wavefront's reads of the current stage have returned
    // by then: the barrier's fence waits for them), (2) requests the direct load of the tile
    // after next into the stage just drained (half of the wavefronts: behind step 4 instead, see
    // below), (3) reads chunk 0 of the next tile, (4) issues chunk 3, whose operands are already
    // in registers, and (5) reads chunk 1 of the next tile: barrier release, LDS latency and a
    // whole K tile of memory latency hide behind matrix work.
    // Per-column epilogue parameters of this tile (alpha * column scale, column bias) are parked
    // in LDS behind the stages while the first direct loads are in flight; the epilogue reads them
    // back with a few 16-byte LDS reads instead of waiting on global memory.
    // The direct loads of a K tile are not requested by all wavefronts at once.  A compute unit takes such an
    // instruction (1 KB) at about 64 bytes per clock, and a wavefront issues nothing else while its loads
    // queue up: with every wavefront requesting right behind the barrier, both wavefronts of every SIMD sit
    // in that queue together and the matrix pipeline idles until the unit has taken all (BM + BN) / 8 of them.
    // The upper half of the wavefronts (the second wavefront of each SIMD) therefore requests behind its chunk
    // 3 instead: while one wavefront of a SIMD queues loads, its sibling issues matrix instructions
    // (launched alone: 4-10 % fewer cycles per launch on every tile shape, int8 and binary16).
    const bool late_loader = wave >= WGM * WGN / 2;
    float* colp = reinterpret_cast<float*>(lds + 2 * STAGE_BYTES);       // [2][BN]: scale, bias
    float  alpha = 1.0f, cp_scale = 1.0f, cp_bias = 0.0f;
    if(!SPLIT)
    {
        if(p.s0) alpha *= *p.s0;
        if(p.s1) alpha *= *p.s1;
        const int64_t col = n0 + tid;
        const bool    cok = tid < BN && col < p.N;
        cp_scale = alpha * ((p.col_scale && cok) ? p.col_scale[col] : 1.0f);
        cp_bias  = (p.col_bias && cok) ? p.col_bias[col] : 0.0f;
    }
    const uint32_t amax_seen = (!SPLIT && p.amax_bits) ? __hip_atomic_load(p.amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
    const float    code_inv  = (!SPLIT && p.codes) ? *p.code_inv : 0.0f;
    const bool any_k = kt_begin < kt_end;
    if(any_k) dma(0, kt_begin);
    if(!SPLIT && tid < BN)
    {
        colp[tid]      = cp_scale;
        colp[BN + tid] = cp_bias;
    }
    if(any_k)
    {
        land(0, kt_begin);
        if(kt_begin + 1 < kt_end) dma(1, kt_begin + 1);
        load_frags(set0, 0, 0);
        load_frags(set1, 0, 1);
        for(int kt = kt_begin; kt < kt_end; ++kt)
        {
            const int  stage = (kt - kt_begin) & 1;
            const bool more  = kt + 1 < kt_end;
            __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
            mma(set0);
            load_frags(set0, stage, 2);
            __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
            mma(set1);
            load_frags(set1, stage, 3);
            __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
            mma(set0);
            if(more) land(stage ^ 1, kt + 1);
            // without a next tile the reads below fetch chunks 0 and 1 of the current stage again: in bounds, unused
            const int  nstage  = more ? (stage ^ 1) : stage;
            const bool request = kt + 2 < kt_end;
            if(request && !late_loader) dma(stage, kt + 2);
            load_frags(set0, nstage, 0);
            __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
            mma(set1);
            if(request && late_loader) dma(stage, kt + 2);
            load_frags(set1, nstage, 1);
        }
        __builtin_amdgcn_s_waitcnt(kWaitAllLds);     // the unused reads of the last trip land before the registers are reused
    }

    // ---- epilogue.  The B fragment is the matrix instruction's first operand, so a lane holds
    //      C^T fragments: lane -> output row m = lane%32 of the fragment; register v -> output
    //      column n = 8*(v/4) + 4*(lane/32) + v%4, i.e. four consecutive columns per register quad.
    const int64_t wrow0 = m0 + wm * WTM, wcol0 = n0 + wn * WTN;
    // Staged stores: pass the wavefront's sub-tile through its private slice of LDS (the K
    // pipeline is drained, so the stages are free) and leave with 16-byte stores whose lanes run
    // along the rows of the destination: every store instruction writes whole 128-byte (or
    // longer) row segments.  RAW writes the accumulators themselves (split-K partials); otherwise
    // they are dequantized in registers first.
    constexpr int STG_BYTES = 2 * STAGE_BYTES / (WGM * WGN);
    uint8_t*      stg       = lds + wave * STG_BYTES;
    uint32_t out_run = 0u;     // running maximum of |C| of this lane (packed like the output type)
    // one atomic maximum per workgroup at most: lanes -> wavefront (shuffles) -> workgroup (LDS slots behind the
    // column parameters).  Atomics on one word retire about 10 ns apart, so a workgroup skips its own when the
    // word, as read at the start of the kernel (`amax_seen`: possibly stale, never too large), already covers it.
    auto publish_amax = [&](uint32_t bits_f32) {
#pragma unroll
        for(int off = 32; off >= 1; off >>= 1)
        {
            const uint32_t o = static_cast<uint32_t>(__shfl_xor(static_cast<int>(bits_f32), off));
            bits_f32 = bits_f32 > o ? bits_f32 : o;
        }
        uint32_t* slots = reinterpret_cast<uint32_t*>(colp + 2 * BN);
        if(lane == 0) slots[wave] = bits_f32;
        __syncthreads();
        if(tid == 0)
        {
            uint32_t m = slots[0];
#pragma unroll
            for(int w = 1; w < WGM * WGN; ++w) m = m > slots[w] ? m : slots[w];
            if(m > amax_seen) atomicMax(p.amax_bits, m);
        }
    };
    auto staged_store = [&](auto out_tag, auto raw_tag, uint8_t* dst_base) {
        typedef decltype(out_tag) out_t;
        constexpr bool RAW   = decltype(raw_tag)::value;
        constexpr int  OS    = sizeof(out_t);
        constexpr int  PITCH = WTN * OS + 16;                     // padded row pitch in the staging slice
        constexpr int  CPITCH = WTN + 16;                         // the same for the optional int8 codes of the rows
        constexpr int  FITS  = STG_BYTES / (32 * (PITCH + CPITCH));
        constexpr int  FPP   = FITS >= FM ? FM : (FITS >= 2 ? 2 : 1);
        static_assert(32 * (PITCH + CPITCH) <= STG_BYTES && FM % FPP == 0, "staging slice too small");
        uint8_t* const cstg  = stg + FPP * 32 * PITCH;            // codes behind the output rows
        constexpr int LPR   = WTN * OS / 16;                     // lanes per output row in the store phase
        constexpr int RPI   = 64 / LPR;                          // rows per store instruction
        __syncthreads();                                  // all wavefronts are done reading the stages
#pragma unroll
        for(int pass = 0; pass < FM / FPP; ++pass)
        {
#pragma unroll
            for(int ii = 0; ii < FPP; ++ii)
            {
                const int i = pass * FPP + ii;
#pragma unroll
                for(int j = 0; j < FN; ++j)
#pragma unroll
                    for(int vq = 0; vq < 4; ++vq)
                    {
                        out_t o[4];
                        float f4[4] = {1.0f, 1.0f, 1.0f, 1.0f}, b4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                        if constexpr(!RAW)
                        {   // column scale and bias of these four columns, parked in LDS by the prologue
                            const int    c  = wn * WTN + j * 32 + 8 * vq + 4 * khalf;          // column inside the tile
                            const float4 fs = *reinterpret_cast<const float4*>(colp + c);
                            const float4 bs = *reinterpret_cast<const float4*>(colp + BN + c);
                            f4[0] = fs.x; f4[1] = fs.y; f4[2] = fs.z; f4[3] = fs.w;
                            b4[0] = bs.x; b4[1] = bs.y; b4[2] = bs.z; b4[3] = bs.w;
                        }
#pragma unroll
                        for(int e = 0; e < 4; ++e)
                        {
                            if constexpr(RAW)
                                o[e] = acc[i][j][vq * 4 + e];
                            else
                            {
                                o[e] = fma_out<out_t>(static_cast<float>(acc[i][j][vq * 4 + e]), f4[e], b4[e]);
                            }
                        }
                        uint8_t* dst = stg + (ii * 32 + frag_row) * PITCH + (j * 32 + 8 * vq + 4 * khalf) * OS;
                        if(OS == 2)
                            *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(o);
                        else
                            *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(o);
                        if constexpr(!RAW)
                            if(p.codes)
                            {   // the quantizer's arithmetic on the value as stored (one fp32 multiply, ties to even, clamp)
                                uint32_t cw = 0u;
#pragma unroll
                                for(int e = 0; e < 4; ++e)
                                {
                                    float stored;
                                    if constexpr(OS == 2) stored = __half2float(o[e]); else stored = o[e];
                                    cw |= (static_cast<uint32_t>(quantize_code<kNearest>(stored, code_inv, p.code_qmax, 0u)) & 0xFFu) << (8 * e);
                                }
                                *reinterpret_cast<uint32_t*>(cstg + (ii * 32 + frag_row) * CPITCH + (j * 32 + 8 * vq + 4 * khalf)) = cw;
                            }
                    }
            }
            // Lanes read what other lanes of the wavefront have just written: the hardware keeps a
            // wavefront's LDS operations in order, and the wavefront-scope fence tells the compiler
            // that these loads may not be satisfied from values a lane has seen before.
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
#pragma unroll
            for(int r0 = 0; r0 < FPP * 32; r0 += RPI)
            {
                const int     lr  = r0 + lane / LPR, seg = lane % LPR;
                const v4u32   val = *reinterpret_cast<const v4u32*>(stg + lr * PITCH + seg * 16);
                const int64_t row = wrow0 + pass * FPP * 32 + lr;
                const int64_t col = wcol0 + seg * (16 / OS);
                if(row < p.M && col < p.N)
                {
                    if constexpr(!RAW)
                        if(p.amax_bits) out_run = fold_abs_bits<OS>(out_run, val);
                    v4u32* dst = reinterpret_cast<v4u32*>(dst_base + (row * p.N + col) * OS);
                    if constexpr(RAW)
                        *dst = val;      // read back soon by the reduction: ordinary store
                    else                 // streaming store: C is not read again here, keep the operand panels in L2
                        __builtin_nontemporal_store(val, dst);
                }
            }
            if constexpr(!RAW)
                if(p.codes)
                {   // rows of WTN code bytes leave as 16-byte vectors too
                    constexpr int CLPR = WTN / 16, CRPI = 64 / CLPR;
#pragma unroll
                    for(int r0 = 0; r0 < FPP * 32; r0 += CRPI)
                    {
                        const int     lr  = r0 + lane / CLPR, seg = lane % CLPR;
                        const v4u32   val = *reinterpret_cast<const v4u32*>(cstg + lr * CPITCH + seg * 16);
                        const int64_t row = wrow0 + pass * FPP * 32 + lr;
                        const int64_t col = wcol0 + seg * 16;
                        if(lr < FPP * 32 && row < p.M && col < p.N)
                            *reinterpret_cast<v4u32*>(p.codes + row * p.N + col) = val;      // read next by the consumer's GEMM
                    }
                }
        }
    };

    if(SPLIT)
    {
        acc_t* part = static_cast<acc_t*>(p.partial) + static_cast<int64_t>(split) * p.M * p.N;
        if((p.N * 4) % 16 == 0 && (reinterpret_cast<uintptr_t>(part) & 15) == 0)
        {
            staged_store(acc_t{}, std::true_type{}, reinterpret_cast<uint8_t*>(part));
            return;
        }
#pragma unroll
        for(int i = 0; i < FM; ++i)
        {
            const int64_t row = wrow0 + i * 32 + frag_row;
#pragma unroll
            for(int j = 0; j < FN; ++j)
#pragma unroll
                for(int v = 0; v < 16; ++v)
                {
                    const int64_t col = wcol0 + j * 32 + 8 * (v / 4) + 4 * khalf + (v % 4);
                    if(row < p.M && col < p.N) part[row * p.N + col] = acc[i][j][v];
                }
        }
        return;
    }

    const int osize = p.c_is_f16 ? 2 : 4;
    const bool fast = !p.acc_dump && (p.N * osize) % 16 == 0 && (reinterpret_cast<uintptr_t>(p.C) & 15) == 0
                   && (!p.codes || (p.N % 16 == 0 && (reinterpret_cast<uintptr_t>(p.codes) & 15) == 0));
    if(!fast)
    {   // element-wise stores: any N, any alignment, optional raw accumulator dump
#pragma unroll
        for(int j = 0; j < FN; ++j)
#pragma unroll
            for(int v = 0; v < 16; ++v)
            {
                const int64_t col = wcol0 + j * 32 + 8 * (v / 4) + 4 * khalf + (v % 4);
                const bool    cok = col < p.N;
                const float   f   = alpha * ((p.col_scale && cok) ? p.col_scale[col] : 1.0f);
                const float   b   = (p.col_bias && cok) ? p.col_bias[col] : 0.0f;
#pragma unroll
                for(int i = 0; i < FM; ++i)
                {
                    const int64_t row = wrow0 + i * 32 + frag_row;
                    if(row < p.M && cok)
                    {
                        // (the same arithmetic as the vector path: a binary16 output is the fused multiply-add rounded
                        // once to binary16)
                        float stored;
                        if(p.c_is_f16)
                        {
                            const __half h = fma_out<__half>(static_cast<float>(acc[i][j][v]), f, b);
                            static_cast<__half*>(p.C)[row * p.N + col] = h;
                            stored = __half2float(h);
                        }
                        else
                        {
                            stored = fmaf(static_cast<float>(acc[i][j][v]), f, b);
                            static_cast<float*>(p.C)[row * p.N + col] = stored;
                        }
                        const uint32_t u = __float_as_uint(stored) & 0x7FFFFFFFu;
                        out_run = out_run > u ? out_run : u;
                        if(p.codes)
                            p.codes[row * p.N + col] = static_cast<int8_t>(quantize_code<kNearest>(stored, code_inv, p.code_qmax, 0u));
                        if(sizeof(acc_t) == 4 && p.acc_dump)
                            p.acc_dump[row * p.N + col] = static_cast<int32_t>(acc[i][j][v]);
                    }
                }
            }
        if(p.amax_bits) publish_amax(out_run);
        return;
    }

    if(p.c_is_f16)
    {
        staged_store(__half{}, std::false_type{}, static_cast<uint8_t*>(p.C));
        if(p.amax_bits) publish_amax(abs_bits_as_f32<2>(out_run));
    }
    else
    {
        staged_store(float{}, std::false_type{}, static_cast<uint8_t*>(p.C));
        if(p.amax_bits) publish_amax(abs_bits_as_f32<4>(out_run));
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Persistent variant of the 256x256 kernel for binary16 outputs whose M, N are multiples of 256 and whose operand
// rows are multiples of two K tiles.  One workgroup per compute unit walks its tiles; three things differ from
// gemm_nt_kernel:
//   * the wavefronts split the vector-memory roles.  Loads and stores of a wavefront share one in-flight counter
//     that retires in issue order, so a wavefront that has just stored its part of C cannot see a later load
//     land before those stores have reached the cache, microseconds later.  Wavefronts 0-3 (one per SIMD, the
//     upper half of the tile) therefore issue every direct global->LDS load and never store; wavefronts 4-7 (the
//     lower half) issue every store of C and never load.  The loaders pass their dequantized half through LDS;
//   * the next tile's first K tile is requested while the last K tile of the current one is still being
//     multiplied (its stage is free by then), the second one as soon as the storers have drained the hand-over
//     area (which is the other stage plus the spare LDS behind the stages); nobody waits for a store, so the
//     write-back of a tile overlaps the next tile's K loop;
//   * barriers are bare s_barrier instructions behind an LDS wait (the compiler's __syncthreads would wait for
//     every vector-memory operation of the wavefront, stores included), and every LDS access behind the first
//     store is written as an instruction for the same reason.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void wait_lds_all() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); __builtin_amdgcn_sched_barrier(0); }
// LDS accesses as instructions; OFF is the instruction's immediate byte offset (16 bits)
template <int OFF> __device__ __forceinline__ void lds_write_b64(uint32_t addr, const v2u32& v)
{
    static_assert(OFF >= 0 && OFF < 65536, "immediate offset");
    asm volatile("ds_write_b64 %0, %1 offset:%2" ::"v"(addr), "v"(v), "n"(OFF) : "memory");
}
__device__ __forceinline__ void lds_write_b32(uint32_t addr, uint32_t v) { asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(v) : "memory"); }
template <int OFF> __device__ __forceinline__ void lds_read_b128(v4u32& d, uint32_t addr)
{
    static_assert(OFF >= 0 && OFF < 65536, "immediate offset");
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFF) : "memory");
}
// bit patterns by value (a vector element is not an object a bit cast could be applied to directly)
template <typename T> __device__ __forceinline__ T word_as(uint32_t u);
template <> __device__ __forceinline__ int32_t word_as<int32_t>(uint32_t u) { return static_cast<int32_t>(u); }
template <> __device__ __forceinline__ float   word_as<float>(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t as_word(int32_t v) { return static_cast<uint32_t>(v); }
__device__ __forceinline__ uint32_t as_word(float v) { return __float_as_uint(v); }

template <typename TR>
__global__ __launch_bounds__(512) void gemm_nt_persistent_kernel(const GemmKernelArgs p, const int total_tiles)
{
    typedef typename TR::accv_t accv_t;
    constexpr int BM = 256, BN = 256, WGN = 4, WTM = 128, WTN = 64, FM = 4, FN = 2;
    constexpr int STAGE_BYTES = (BM + BN) * kRowBytes;        // 64 KB
    constexpr int DPW         = 16;                           // direct loads per loader wavefront and K tile
    constexpr int PITCH       = WTN * 2 + 16;                 // padded row of 64 binary16 outputs in the hand-over area
    constexpr int L_STG       = WTM * PITCH;                  // a loader's whole sub-tile
    constexpr int S_STG       = 32 * PITCH;                   // a storer's private slice: one row of fragments
    constexpr int STG_BASE    = STAGE_BYTES;                  // the hand-over area starts where stage 1 starts
    constexpr int S_BASE      = STG_BASE + 4 * L_STG;
    constexpr int COLP_BASE   = S_BASE + 4 * S_STG;           // [2][BN] floats: alpha * column scale, column bias
    static_assert(COLP_BASE + 2 * BN * 4 <= kPersistentLdsBytes, "LDS layout");

    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) uint8_t*)lds));
    const int  tid = threadIdx.x, lane = tid % kWaveSize;
    const int  wave = __builtin_amdgcn_readfirstlane(tid / kWaveSize);
    const int  wm = wave / WGN, wn = wave % WGN;
    const bool loader = wave < 4;                              // uniform per wavefront
    const int  KT = static_cast<int>(p.Kb / kRowBytes);        // even, >= 2 (checked by the launcher)
    const int  G  = static_cast<int>(gridDim.x);

    // ---- loader set-up: wavefront l covers stage rows [128 l, 128 l + 128): l = 0, 1 rows of A, l = 2, 3 rows of B
    const int  lw   = wave & 3;
    const bool is_a = lw < 2;
    uint32_t   voff[DPW];
    {
        int imm[DPW];
        fill_dma_imms<DPW>(imm, std::make_integer_sequence<int, DPW>{});
#pragma unroll
        for(int d = 0; d < DPW; ++d)
        {
            const int srow  = (lw * DPW + d) * 8 + lane / 8;
            const int chunk = (lane % 8) ^ ((srow >> 1) & 7);
            const int lrow  = srow - (is_a ? 0 : BM);
            voff[d] = static_cast<uint32_t>(static_cast<int64_t>(lrow) * p.Kb + chunk * 16 + kDmaBias - imm[d]);
        }
    }
    auto panel_base = [&](int tm, int tn) -> const uint8_t* {
        const uint8_t* g = is_a ? p.A + static_cast<int64_t>(tm) * BM * p.Kb : p.B + static_cast<int64_t>(tn) * BN * p.Kb;
        const uint64_t bits = reinterpret_cast<uint64_t>(g) - kDmaBias;
        const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(bits))));
        const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(bits >> 32))));
        return reinterpret_cast<const uint8_t*>((static_cast<uint64_t>(hi) << 32) | static_cast<uint64_t>(lo));
    };
    auto dma = [&](int stage, const uint8_t* sbase, int kt) {
        const uint8_t* sb    = sbase + static_cast<int64_t>(kt) * kRowBytes;
        uint8_t*       lbase = lds + stage * STAGE_BYTES + lw * (DPW * 1024) + (dma_group<DPW>() / 2) * 1024;
        asm volatile("" : "+s"(sb));
        dma_sequence<DPW>(std::make_integer_sequence<int, DPW>{}, sb, voff, lbase);
    };
    auto park_column_parameters = [&](int tn) {               // threads 0..255 are exactly the loaders
        float alpha = 1.0f;
        if(p.s0) alpha *= *p.s0;
        if(p.s1) alpha *= *p.s1;
        const int64_t col = static_cast<int64_t>(tn) * BN + tid;
        const float   sc  = alpha * (p.col_scale ? p.col_scale[col] : 1.0f);
        const float   bi  = p.col_bias ? p.col_bias[col] : 0.0f;
        lds_write_b32(lds0 + COLP_BASE + tid * 4, __float_as_uint(sc));
        lds_write_b32(lds0 + COLP_BASE + (BN + tid) * 4, __float_as_uint(bi));
    };

    // ---- fragment reads (as in gemm_nt_kernel)
    const int frag_row = lane & 31, khalf = lane >> 5;
    int       roff[4];
#pragma unroll
    for(int ks = 0; ks < 4; ++ks) roff[ks] = frag_row * kRowBytes + swizzle(frag_row, ks * 2 + khalf);
    const int a_base = (wm * WTM) * kRowBytes, b_base = BM * kRowBytes + (wn * WTN) * kRowBytes;
    v4i32     af[2][FM], bf[2][FN];
    auto      load_frags = [&](auto buf_tag, int stage, int ks) {
        constexpr int  buf = decltype(buf_tag)::value;
        const uint32_t fa  = lds0 + static_cast<uint32_t>(stage * STAGE_BYTES + a_base + roff[ks]);
        const uint32_t fb  = lds0 + static_cast<uint32_t>(stage * STAGE_BYTES + b_base + roff[ks]);
        frag_reads<FM>(af[buf], fa, std::make_integer_sequence<int, FM>{});
        frag_reads<FN>(bf[buf], fb, std::make_integer_sequence<int, FN>{});
    };
    constexpr int kWaitOlderSet = 0xC07F | ((FM + FN) << 8);
    accv_t        acc[FM][FN];
    auto          mma = [&](auto buf_tag) {
        constexpr int buf = decltype(buf_tag)::value;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for(int i = 0; i < FM; ++i)
#pragma unroll
            for(int j = 0; j < FN; ++j) acc[i][j] = TR::mfma(bf[buf][j], af[buf][i], acc[i][j]);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto clear_acc = [&]() {
#pragma unroll
        for(int i = 0; i < FM; ++i)
#pragma unroll
            for(int j = 0; j < FN; ++j)
#pragma unroll
                for(int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    };
    const std::integral_constant<int, 0> set0{};
    const std::integral_constant<int, 1> set1{};

    // ---- first tile: both stages requested, column parameters parked, first K tile awaited
    int lin = static_cast<int>(blockIdx.x);
    int split_unused, tm, tn;
    item_of_block(lin, p.tiles_m, p.tiles_n, 1, p.group_m, split_unused, tm, tn);
    const uint8_t* cur = panel_base(tm, tn);
    if(loader)
    {
        dma(0, cur, 0);
        dma(1, cur, 1);
        park_column_parameters(tn);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    wg_barrier();

    while(true)
    {
        __builtin_amdgcn_sched_barrier(0);     // the accumulators' live range starts here, not before the last tile's stores
        clear_acc();
        const int  nlin     = lin + G;
        const bool has_next = nlin < total_tiles;
        int        ntm = 0, ntn = 0;
        if(has_next) item_of_block(nlin, p.tiles_m, p.tiles_n, 1, p.group_m, split_unused, ntm, ntn);
        const uint8_t* nxt = has_next ? panel_base(ntm, ntn) : cur;

        // ---- K loop.  On entry K tile 0 is in stage 0 and published, K tile 1 is in flight towards stage 1.
        load_frags(set0, 0, 0);
        load_frags(set1, 0, 1);
        for(int kt = 0; kt < KT; ++kt)
        {
            const int stage = kt & 1;
            __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
            mma(set0);
            load_frags(set0, stage, 2);
            __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
            mma(set1);
            load_frags(set1, stage, 3);
            __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
            mma(set0);
            const bool more = kt + 1 < KT;
            if(more)
            {
                // the loaders' K tile kt+1 has landed, everybody's reads of this stage have returned
                if(loader) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                wg_barrier();
                if(loader)
                {
                    if(kt + 2 < KT) dma(stage, cur, kt + 2);
                    else if(has_next) dma(stage, nxt, 0);        // kt + 2 == KT: stage 0, first K tile of the next tile
                }
            }
            // on the last K tile the reads below fetch chunks 0 and 1 of the current stage again: in bounds, unused
            const int nstage = more ? (stage ^ 1) : stage;
            load_frags(set0, nstage, 0);
            __builtin_amdgcn_s_waitcnt(kWaitOlderSet);
            mma(set1);
            load_frags(set1, nstage, 1);
        }

        // ---- epilogue.  Stage 1 (last K tile) is drained once everybody passes this barrier.
        wg_barrier();
        const int64_t m0 = static_cast<int64_t>(tm) * BM, n0 = static_cast<int64_t>(tn) * BN;
        // where this wavefront's dequantized rows go: a loader fills its whole 128-row region, a storer its
        // private 32-row slice, pass by pass (the storer's base steps back by one pass per pass, so that both
        // use the same immediates)
        const uint32_t my_stg  = lds0 + (loader ? STG_BASE + wave * L_STG : S_BASE + (wave - 4) * S_STG);
        const uint32_t wr_lane = my_stg + static_cast<uint32_t>(frag_row * PITCH + 8 * khalf);
        const uint32_t cp_lane = lds0 + COLP_BASE + static_cast<uint32_t>((wn * WTN + 4 * khalf) * 4);
        const int      lr8 = lane / 8, seg = lane % 8;
        const uint32_t rd_lane = static_cast<uint32_t>(lr8 * PITCH + seg * 16);
        const int64_t  wcol0 = n0 + wn * WTN;
        __half* const  cbase = static_cast<__half*>(p.C) + wcol0 + seg * 8;
        // alpha * column scale and bias of this lane's 2 x 16 columns, read once per tile
        v4u32 rs[FN][4], rb[FN][4];
        static_for<FN>([&](auto jt) {                         // (a batch of 8 reads per fragment column: the LDS counter holds 15)
            constexpr int j = decltype(jt)::value;
            static_for<4>([&](auto vt) {
                constexpr int vq = decltype(vt)::value;
                lds_read_b128<(j * 32 + 8 * vq) * 4>(rs[j][vq], cp_lane);
                lds_read_b128<(BN + j * 32 + 8 * vq) * 4>(rb[j][vq], cp_lane);
            });
            wait_lds_all();
        });
        static_for<FM>([&](auto it) {
            constexpr int  i       = decltype(it)::value;
            const uint32_t wr_base = loader ? wr_lane : wr_lane - static_cast<uint32_t>(i * 32 * PITCH);
            static_for<FN>([&](auto jt) {
                constexpr int j = decltype(jt)::value;
                static_for<4>([&](auto vt) {
                    constexpr int vq = decltype(vt)::value;
                    // the per-tile kernel's arithmetic: each value one fused multiply-add rounded once to binary16
                    auto pair = [&](int e) {
                        return fma_out_half2(static_cast<float>(acc[i][j][vq * 4 + e]), __uint_as_float(rs[j][vq][e]),
                                             __uint_as_float(rb[j][vq][e]),
                                             static_cast<float>(acc[i][j][vq * 4 + e + 1]), __uint_as_float(rs[j][vq][e + 1]),
                                             __uint_as_float(rb[j][vq][e + 1]));
                    };
                    const v2u32 packed = {pair(0), pair(2)};
                    lds_write_b64<i * 32 * PITCH + (j * 32 + 8 * vq) * 2>(wr_base, packed);
                });
            });
            if(!loader)
            {   // the storer's own rows leave right away: written by this wavefront, read back transposed
                wait_lds_all();
                v4u32 val[4];
                static_for<4>([&](auto qt) { lds_read_b128<decltype(qt)::value * 8 * PITCH>(val[decltype(qt)::value], my_stg + rd_lane); });
                wait_lds_all();
#pragma unroll
                for(int q = 0; q < 4; ++q)
                {
                    const int64_t row = m0 + WTM + i * 32 + q * 8 + lr8;
                    __builtin_nontemporal_store(val[q], reinterpret_cast<v4u32*>(cbase + row * p.N));
                }
            }
        });
        wg_barrier();                                        // the loaders' rows are in the hand-over area
        // The storers take the partner's sub-tile (same columns, the upper half of the tile) out of the hand-over
        // area into registers, so that the area is free again after one more barrier and the loaders' request for
        // the next tile's second K tile enters the memory pipeline ahead of the stores that follow.
        // (The 64 registers are those of the accumulators, dead by now: a separate array would raise the kernel's
        // register demand and the compiler would spill the results of the LDS instructions before they arrive.)
        if(!loader)
        {
            const uint32_t src = lds0 + STG_BASE + static_cast<uint32_t>((wave - 4) * L_STG) + rd_lane;
            static_for<2>([&](auto bt) {                       // two batches: the LDS counter of a wavefront holds 15
                constexpr int b = decltype(bt)::value;
                v4u32 t[8];
                static_for<8>([&](auto rt) { lds_read_b128<(b * 8 + decltype(rt)::value) * 8 * PITCH>(t[decltype(rt)::value], src); });
                wait_lds_all();
                static_for<8>([&](auto rt) {
                    constexpr int r = b * 8 + decltype(rt)::value;
#pragma unroll
                    for(int e = 0; e < 4; ++e)
                        {
                        const uint32_t word = t[decltype(rt)::value][e];
                        acc[r / 4][0][4 * (r % 4) + e] = word_as<typename TR::acc_t>(word);
                    }
                });
            });
        }
        if(loader && has_next)
        {
            park_column_parameters(ntn);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the next tile's first K tile has landed
        }
        wg_barrier();                                        // hand-over area drained, stage 0 and parameters published
        if(loader && has_next) dma(1, nxt, 1);
        if(!loader)
        {
#pragma unroll
            for(int r = 0; r < 16; ++r)
            {
                const int64_t row = m0 + r * 8 + lr8;
                v4u32         val;
#pragma unroll
                for(int e = 0; e < 4; ++e)
                {
                    const typename TR::acc_t a = acc[r / 4][0][4 * (r % 4) + e];
                    val[e] = as_word(a);
                }
                __builtin_nontemporal_store(val, reinterpret_cast<v4u32*>(cbase + row * p.N));
            }
        }
        if(!has_next) break;
        lin = nlin; tm = ntm; tn = ntn; cur = nxt;
    }
}


// Adds the split-K partials in split order and applies the epilogue.
constexpr int kThreads = 256;   // split-K reduction

template <typename ACC, bool VEC4>
__global__ __launch_bounds__(kThreads) void splitk_reduce_kernel(const ACC* __restrict__ partial, int splits,
                                                                 int64_t M, int64_t N, void* C, int c_is_f16,
                                                                 const float* s0, const float* s1,
                                                                 const float* __restrict__ col_scale,
                                                                 const float* __restrict__ col_bias, int32_t* acc_dump,
                                                                 unsigned int* amax_bits, int8_t* codes,
                                                                 const float* code_inv_p, int code_qmax)
{
    const float code_inv = codes ? *code_inv_p : 0.0f;
    constexpr int V      = VEC4 ? 4 : 1;       // VEC4: N % 4 == 0 and 16-byte aligned buffers
    uint32_t      run    = 0u;                 // maximum of |C| as stored (fp32 bits), when amax_bits is given
    const uint32_t seen  = amax_bits ? __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
    const int64_t n      = M * N;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads * V;
    float         alpha  = 1.0f;
    if(s0) alpha *= *s0;
    if(s1) alpha *= *s1;
    for(int64_t i = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * V; i < n; i += stride)
    {
        ACC acc[V];
#pragma unroll
        for(int e = 0; e < V; ++e) acc[e] = 0;
#pragma unroll 8                                  // eight independent partial loads in flight; the sum keeps its order
        for(int s = 0; s < splits; ++s)
        {
            ACC part[V];
            if(VEC4)
                *reinterpret_cast<uint4*>(part) = *reinterpret_cast<const uint4*>(partial + static_cast<int64_t>(s) * n + i);
            else
                part[0] = partial[static_cast<int64_t>(s) * n + i];
#pragma unroll
            for(int e = 0; e < V; ++e) acc[e] += part[e];
        }
        const int64_t col = i % N;
        float         y[V];
#pragma unroll
        for(int e = 0; e < V; ++e)
        {
            const float f = alpha * (col_scale ? col_scale[col + e] : 1.0f);
            y[e] = static_cast<float>(acc[e]) * f + (col_bias ? col_bias[col + e] : 0.0f);
        }
        if(c_is_f16)
        {   // what is stored is the rounded value: take the maximum of that
#pragma unroll
            for(int e = 0; e < V; ++e) y[e] = __half2float(__float2half_rn(y[e]));
        }
        if(amax_bits)
        {
#pragma unroll
            for(int e = 0; e < V; ++e)
            {
                const uint32_t u = __float_as_uint(y[e]) & 0x7FFFFFFFu;
                run = run > u ? run : u;
            }
        }
        if(codes)
        {   // codes of the values as stored (y holds the rounded value when the output is binary16)
            uint32_t cw = 0u;
#pragma unroll
            for(int e = 0; e < V; ++e)
                cw |= (static_cast<uint32_t>(quantize_code<kNearest>(y[e], code_inv, code_qmax, 0u)) & 0xFFu) << (8 * e);
            if(VEC4 && (reinterpret_cast<uintptr_t>(codes) & 3) == 0)
                *reinterpret_cast<uint32_t*>(codes + i) = cw;
            else
#pragma unroll
                for(int e = 0; e < V; ++e) codes[i + e] = static_cast<int8_t>((cw >> (8 * e)) & 0xFFu);
        }
        if(VEC4)
        {
            if(c_is_f16)
            {
                __half h[4];
#pragma unroll
                for(int e = 0; e < 4; ++e) h[e] = __float2half_rn(y[e]);      // exact: y is a binary16 value
                *reinterpret_cast<uint2*>(static_cast<__half*>(C) + i) = *reinterpret_cast<const uint2*>(h);
            }
            else
                *reinterpret_cast<uint4*>(static_cast<float*>(C) + i) = *reinterpret_cast<const uint4*>(y);
        }
        else if(c_is_f16)
            static_cast<__half*>(C)[i] = __float2half_rn(y[0]);
        else
            static_cast<float*>(C)[i] = y[0];
        if(acc_dump)
#pragma unroll
            for(int e = 0; e < V; ++e) acc_dump[i + e] = static_cast<int32_t>(acc[e]);
    }
    if(amax_bits)
    {   // one atomic maximum per workgroup
        __shared__ uint32_t slots[kThreads / 64];
#pragma unroll
        for(int off = 32; off >= 1; off >>= 1)
        {
            const uint32_t o = static_cast<uint32_t>(__shfl_xor(static_cast<int>(run), off));
            run = run > o ? run : o;
        }
        if(threadIdx.x % 64 == 0) slots[threadIdx.x / 64] = run;
        __syncthreads();
        if(threadIdx.x == 0)
        {
            uint32_t m = slots[0];
#pragma unroll
            for(int w = 1; w < kThreads / 64; ++w) m = m > slots[w] ? m : slots[w];
            if(m > seen) atomicMax(amax_bits, m);      // `seen` may be stale but never too large: skipping is safe
        }
    }
}

struct TileShape { int bm, bn; };
// 0: 256x256, 8 wavefronts (2x4, 128x64 each)   1: 128x128, 4 wavefronts (2x2, 64x64 each)
// 2: 64x64, 4 wavefronts (2x2, 32x32 each)
// (256x256 with 4 wavefronts of 128x128 -- a third fewer LDS fragment reads per matrix instruction, 256
//  accumulator registers per lane -- needs matrix instructions written as inline assembly on accumulator
//  registers, one loop body without branches around them, and fragment reads and direct loads placed one by one
//  between them; the compiler's own allocation keeps the accumulators in scratch memory.  Built that way it is
//  bit-identical and as fast as the 8-wavefront tile at 8192^3 but 7-14 % slower on 16384x4096x1024 and
//  16384x1024x4096, where its longer epilogue counts: not kept.)
constexpr TileShape kTiles[] = {{256, 256}, {128, 128}, {64, 64}};
constexpr int       kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

// The dynamic-LDS attribute of a kernel is set once per device: flags indexed by the current device (a process
// that drives several GPUs sets it on each; beyond kMaxDevices it is set before every launch).
constexpr int kMaxDevices = 16;
inline int current_device_slot()
{
    int dev = 0;
    return (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices) ? dev : -1;
}

template <typename TR, int BM, int BN, int WGM, int WGN>
hipError_t launch_tile(const GemmKernelArgs& a, int splits, hipStream_t st, bool tn = false)
{
    constexpr size_t lds_bytes = 2 * static_cast<size_t>(BM + BN) * kRowBytes + 2 * BN * sizeof(float) + 64;   // + amax slots
    const dim3       grid(static_cast<unsigned>(a.tiles_m * a.tiles_n), static_cast<unsigned>(splits));
    const dim3       block(64 * WGM * WGN);
    static bool      attr_set[kMaxDevices][7] = {};   // per instantiation and device; benign if set twice
    const int        slot = current_device_slot();
    const bool       conv  = a.conv_H > 0;
    const int        which = tn ? (conv ? (splits > 1 ? 6 : 5) : (splits > 1 ? 4 : 3)) : (conv ? 2 : (splits > 1 ? 1 : 0));
    if(conv && !tn && splits > 1) return hipErrorInvalidValue;
    if(tn && TR::kElemBytes > 2) return hipErrorInvalidValue;
    const void* fn = nullptr;
    if constexpr(TR::kElemBytes <= 2)
        if(tn)
        {
            if(conv)
                fn = splits > 1 ? reinterpret_cast<const void*>(&gemm_nt_kernel<TR, BM, BN, WGM, WGN, true, true, true>)
                                : reinterpret_cast<const void*>(&gemm_nt_kernel<TR, BM, BN, WGM, WGN, false, true, true>);
            else
                fn = splits > 1 ? reinterpret_cast<const void*>(&gemm_nt_kernel<TR, BM, BN, WGM, WGN, true, false, true>)
                                : reinterpret_cast<const void*>(&gemm_nt_kernel<TR, BM, BN, WGM, WGN, false, false, true>);
        }
    if(!fn)
        fn = conv ? reinterpret_cast<const void*>(&gemm_nt_kernel<TR, BM, BN, WGM, WGN, false, true>)
           : splits > 1 ? reinterpret_cast<const void*>(&gemm_nt_kernel<TR, BM, BN, WGM, WGN, true>)
                        : reinterpret_cast<const void*>(&gemm_nt_kernel<TR, BM, BN, WGM, WGN, false>);
    if(slot < 0 || !attr_set[slot][which])
    {
        const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 static_cast<int>(lds_bytes));
        if(e != hipSuccess) return e;
        if(slot >= 0) attr_set[slot][which] = true;
    }
    if constexpr(TR::kElemBytes <= 2)
        if(tn)
        {
            if(conv && splits > 1)
                gemm_nt_kernel<TR, BM, BN, WGM, WGN, true, true, true><<<grid, block, lds_bytes, st>>>(a);
            else if(conv)
                gemm_nt_kernel<TR, BM, BN, WGM, WGN, false, true, true><<<grid, block, lds_bytes, st>>>(a);
            else if(splits > 1)
                gemm_nt_kernel<TR, BM, BN, WGM, WGN, true, false, true><<<grid, block, lds_bytes, st>>>(a);
            else
                gemm_nt_kernel<TR, BM, BN, WGM, WGN, false, false, true><<<grid, block, lds_bytes, st>>>(a);
            return hipGetLastError();
        }
    if(conv)
        gemm_nt_kernel<TR, BM, BN, WGM, WGN, false, true><<<grid, block, lds_bytes, st>>>(a);
    else if(splits > 1)
        gemm_nt_kernel<TR, BM, BN, WGM, WGN, true><<<grid, block, lds_bytes, st>>>(a);
    else
        gemm_nt_kernel<TR, BM, BN, WGM, WGN, false><<<grid, block, lds_bytes, st>>>(a);
    return hipGetLastError();
}

template <typename TR>
hipError_t launch_traits(int tile, const GemmKernelArgs& a, int splits, hipStream_t st, bool tn = false)
{
    switch(tile)
    {
    case 0: return launch_tile<TR, 256, 256, 2, 4>(a, splits, st, tn);
    case 1: return launch_tile<TR, 128, 128, 2, 2>(a, splits, st, tn);
    default: return launch_tile<TR, 64, 64, 2, 2>(a, splits, st, tn);
    }
}

// The persistent kernel serves full 256x256 tiles with binary16 output and nothing optional in the epilogue.
bool persistent_eligible(const GemmKernelArgs& a, int prec, int tile, int splits)
{
    return (prec == 8 || prec == 16) && tile == 0 && splits == 1 && a.c_is_f16 && !a.acc_dump && !a.amax_bits && !a.codes && a.conv_H == 0
        && a.remap_C == 0 && a.M % 256 == 0 && a.N % 256 == 0 && a.Kb % (2 * kRowBytes) == 0 && a.Kb >= 2 * kRowBytes
        && (reinterpret_cast<uintptr_t>(a.C) & 15) == 0;
}

template <typename TR> hipError_t launch_persistent(const GemmKernelArgs& a, hipStream_t st)
{
    static bool      attr_set[kMaxDevices] = {};      // per instantiation and device; benign if set twice
    const int        slot = current_device_slot();
    const void*      fn = reinterpret_cast<const void*>(&gemm_nt_persistent_kernel<TR>);
    if(slot < 0 || !attr_set[slot])
    {
        const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kPersistentLdsBytes);
        if(e != hipSuccess) return e;
        if(slot >= 0) attr_set[slot] = true;
    }
    const int total = a.tiles_m * a.tiles_n;
    const int grid  = total < kNumCu ? total : kNumCu;
    gemm_nt_persistent_kernel<TR><<<dim3(static_cast<unsigned>(grid)), dim3(512), kPersistentLdsBytes, st>>>(a, total);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_f32(const GemmProblem& p, hipStream_t stream);   // gemm_f32.hip

static thread_local int g_tile_override = -1;     // set by tests and tuning runs only; per calling thread
void set_gemm_tile_override(int tile) { g_tile_override = (tile >= 0 && tile < kNumTiles) ? tile : -1; }
static thread_local int g_persistent_mode = -1;   // 1: whenever eligible; anything else: never (the default, see launch_gemm)
void set_gemm_persistent_mode(int mode) { g_persistent_mode = (mode == 0 || mode == 1) ? mode : -1; }

GemmPlan plan_gemm(int prec, int64_t M, int64_t N, int64_t K, int force_tile, int force_splits, bool allow_split, bool tn)
{
    if(force_tile < 0 && g_tile_override >= 0)
    {   // a forced tile keeps the planner's split choice for that tile
        GemmPlan forced = plan_gemm(prec, M, N, K, g_tile_override, force_splits >= 1 ? force_splits : 0, allow_split, tn);
        return forced;
    }
    GemmPlan plan{1, 1, 0};
    if(M <= 0 || N <= 0) return plan;
    const int64_t kb     = K * (prec == 8 ? 1 : (prec == 16 ? 2 : 4));
    if(prec == 32 && kb % 16 != 0) return plan;                   // the any-shape fp32 kernel: no tiles to plan
    // a K tile of fp32 operands takes the matrix cores eight times as long as one of int8 or binary16 operands
    const double  kwork  = prec == 32 ? 8.0 : 1.0;
    const int64_t ktiles = (kb + kRowBytes - 1) / kRowBytes;
    auto ntiles = [&](int t) { return ((M + kTiles[t].bm - 1) / kTiles[t].bm) * ((N + kTiles[t].bn - 1) / kTiles[t].bn); };
    // Plan = (tile, K splits) with the smallest estimated time.  The estimate is a small model fitted to gfx950
    // measurements of this kernel (int8, the step's code distribution, 17 shapes x up to 10 plans, launched alone;
    // rms error 6 %; binary16 scales alike):
    //   a compute unit retires `r1` Mop/us per resident workgroup of a tile shape, up to `rmax` with `occ` of them
    //   sharing it; the chip as a whole retires at most `cap` Mop/us (the power limit: 256 busy units do not
    //   each reach `rmax`); every round of co-resident workgroups costs `ovh` us of launch, first-load latency
    //   and epilogue; split K adds its reduction pass.
    struct TileModel { double r1, rmax, ovh, cap; int occ; };
    const TileModel model[kNumTiles] = {{14.9, 15.5, 9.2, 2555.0, 1}, {6.56, 8.42, 4.4, 2000.0, 2}, {2.89, 5.03, 2.5, 2035.0, 4}};
    // Row-major (TN) operands: a K tile takes twice the LDS fragment reads, and a 64-wide tile of int8 operands
    // loads 64-byte row pieces (binary16: 128 bytes, no penalty); fitted slow-down of the main loop per tile shape.
    const double    tn_rate[kNumTiles] = {0.89, 0.99, prec == 8 ? 0.66 : 0.95};
    const double    cus = 256.0;
    auto estimate = [&](int t, int64_t s) {
        const TileModel& m    = model[t];
        const double     tnf  = tn ? tn_rate[t] : 1.0;
        const double     wgs  = static_cast<double>(ntiles(t)) * static_cast<double>(s);
        const double     per  = std::ceil(wgs / cus);                                    // workgroups of the busiest unit
        const double     share = per < m.occ ? per : m.occ;                              // co-resident ones
        const double     rate = (m.r1 * share < m.rmax ? m.r1 * share : m.rmax) * tnf;
        const double     kt   = std::ceil(static_cast<double>(ktiles) / static_cast<double>(s));
        const double     mop  = 2.0 * kTiles[t].bm * kTiles[t].bn * kRowBytes * 1e-6 * kwork;    // per K tile (int8 ops)
        const double     unit = per * kt * mop / rate, chip = wgs * kt * mop / (m.cap * tnf);
        double           us   = (unit > chip ? unit : chip) + m.ovh * std::ceil(wgs / (cus * m.occ));
        if(s > 1) us += 4.2 + static_cast<double>(s + 1) * static_cast<double>(M) * static_cast<double>(N) * 4.0 / 6.35e6;
        return us;
    };
    // Candidates: no split, and the split counts that fill the units once, twice or up to their co-residency.  Tiles are
    // visited from large to small and splits from few to many; a later candidate must win by 5 % (the larger tile
    // moves fewer bytes per operation, and estimates that close are inside the model's error) -- unless the
    // incumbent's tiles overhang the output by a quarter more than the candidate's: padding is where the model
    // errs in the larger tile's favour.
    int     tile = 0, splits = 1;
    double  best = -1.0, best_area = 0.0;
    for(int t = 0; t < kNumTiles; ++t)
    {
        if(force_tile >= 0 && force_tile < kNumTiles && t != force_tile) continue;
        int64_t cand[4] = {1, 1, 1, 1};
        int     ncand   = 1;
        if(allow_split && !(force_tile >= 0 && force_splits < 0))
            for(int f = 0; f < 3; ++f)
            {
                const int64_t fill = f == 0 ? 256 : (f == 1 ? 512 : 256 * model[t].occ);
                if(fill > 256 * model[t].occ) continue;
                int64_t       s    = fill / ntiles(t);
                if(s > ktiles / 8) s = ktiles / 8;                // keep at least 8 K tiles per split
                if(s > 128) s = 128;
                if(s >= 2 && s != cand[ncand - 1]) cand[ncand++] = s;
            }
        const double area = static_cast<double>(ntiles(t)) * kTiles[t].bm * kTiles[t].bn;
        for(int c = 0; c < ncand; ++c)
        {
            const double us     = estimate(t, cand[c]);
            const double margin = best_area > 1.25 * area ? 1.0 : 0.95;
            if(best < 0.0 || us < margin * best) { best = us; best_area = area; tile = t; splits = static_cast<int>(cand[c]); }
        }
    }
    if(force_splits >= 1 && allow_split) splits = force_splits;
    if(splits > ktiles) splits = static_cast<int>(ktiles < 1 ? 1 : ktiles);
    plan.tile      = tile;
    plan.splits    = splits;
    plan.workspace = splits > 1 ? static_cast<size_t>(splits) * M * N * 4 : 0;
    return plan;
}

hipError_t launch_gemm(const GemmProblem& p, const GemmPlan& plan, void* workspace, hipStream_t stream)
{
    if(p.M <= 0 || p.N <= 0) return hipSuccess;
    if(p.prec == 32 && (p.conv_H > 0 || p.b_remap_C > 0)) return hipErrorInvalidValue;
    // fp32 on the matrix cores needs 16-byte aligned, 16-byte multiple operand rows; anything else takes the
    // any-shape kernel
    if(p.prec == 32 && ((p.K * 4) % 16 != 0 || ((reinterpret_cast<uintptr_t>(p.A) | reinterpret_cast<uintptr_t>(p.B)) & 15) != 0))
        return launch_gemm_f32(p, stream);
    const int      esz = p.prec == 8 ? 1 : (p.prec == 16 ? 2 : 4);
    // lane offsets inside an operand panel are 32-bit: 255 rows of K bytes (plus the load immediates) must fit
    if(p.K > kGemmMaxRowBytes / esz) return hipErrorInvalidValue;
    GemmKernelArgs a;
    a.A = static_cast<const uint8_t*>(p.A);
    a.B = static_cast<const uint8_t*>(p.B);
    a.M = p.M; a.N = p.N; a.Kb = p.K * esz;
    a.C = p.C; a.c_is_f16 = p.c_dtype == kF16;
    a.s0 = p.s0; a.s1 = p.s1; a.col_scale = p.col_scale; a.col_bias = p.col_bias;
    a.acc_dump = p.prec == 8 ? p.acc_dump : nullptr;
    a.partial  = workspace;
    a.conv_H = a.conv_W = a.conv_Cb = 0;
    a.remap_C = a.remap_shift = 0;
    if(p.tn)
    {   // A [K, M], B [K, N] row-major int8 or binary16: rows are contraction indices (128 bytes' worth per K tile),
        // 16-byte column chunks
        if((p.prec != 8 && p.prec != 16) || p.b_remap_C > 0 || (p.K * esz) % kRowBytes != 0
           || (p.M * esz) % 16 != 0 || (p.N * esz) % 16 != 0
           || p.M >= (int64_t(1) << 24) || p.N >= (int64_t(1) << 24)
           || ((reinterpret_cast<uintptr_t>(p.A) | reinterpret_cast<uintptr_t>(p.B)) & 15) != 0)
            return hipErrorInvalidValue;
    }
    a.amax_bits = plan.splits > 1 ? nullptr : p.out_amax_bits;      // with K splits the reduction pass takes the maximum
    a.codes     = plan.splits > 1 ? nullptr : static_cast<int8_t*>(p.out_codes);      // ... and writes the codes
    a.code_inv  = p.out_code_inv;
    a.code_qmax = p.out_code_qmax;
    if(p.b_remap_C > 0)
    {   // B is [3*remap_C, K] with a margin of |remap_shift| readable bytes in front of it and behind it
        if(p.conv_H > 0 || p.N != 9 * p.b_remap_C || p.b_remap_shift % 16 != 0 || p.b_remap_shift < 0
           || p.b_remap_shift > 1024 || 3 * p.b_remap_C * a.Kb >= (int64_t(1) << 32) - (1 << 20))
            return hipErrorInvalidValue;
        a.remap_C = static_cast<int>(p.b_remap_C); a.remap_shift = static_cast<int>(p.b_remap_shift);
    }
    if(p.conv_H > 0 && p.tn)
    {   // B is the NHWC tensor [K = images*H*W pixels, C]; the [pixels, 9*C] patch matrix is formed by the loads
        if(p.N != 9 * p.conv_C || p.K * p.conv_C * esz >= (int64_t(1) << 31) || p.conv_H > 65535 || p.conv_W > 65535
           || (p.conv_C * esz) % 16 != 0 || p.K % (static_cast<int64_t>(p.conv_H) * p.conv_W) != 0)
            return hipErrorInvalidValue;
        a.conv_H = p.conv_H; a.conv_W = p.conv_W; a.conv_Cb = static_cast<int>(p.conv_C * esz);
    }
    else if(p.conv_H > 0)
    {   // A is the NHWC tensor [M = images*H*W, C]; its 3x3 patch matrix [M, 9*C] is formed by the loads
        if(p.K != 9 * p.conv_C || plan.splits > 1 || p.M * p.conv_C * esz >= (int64_t(1) << 31)
           || p.conv_H > 65535 || p.conv_W > 65535 || (p.conv_C * esz) % 16 != 0
           || p.M % (static_cast<int64_t>(p.conv_H) * p.conv_W) != 0)
            return hipErrorInvalidValue;
        a.conv_H = p.conv_H; a.conv_W = p.conv_W; a.conv_Cb = static_cast<int>(p.conv_C * esz);
    }
    const int64_t ktiles = (a.Kb + kRowBytes - 1) / kRowBytes;
    int splits = plan.splits < 1 ? 1 : plan.splits;
    a.ktiles_per_split = static_cast<int>((ktiles + splits - 1) / splits);
    if(a.ktiles_per_split < 1) a.ktiles_per_split = 1;
    const TileShape ts = kTiles[plan.tile];
    a.tiles_m = static_cast<int>((p.M + ts.bm - 1) / ts.bm);
    a.tiles_n = static_cast<int>((p.N + ts.bn - 1) / ts.bn);
    a.group_m = kGroupM;      // (2, 4, 16 and 32 measured within noise of 8 on config 5's shapes, int8 and binary16)
    // The persistent kernel is opt-in.  Launched alone and back to back it beats the per-tile kernel by 7-20 % (the
    // write-back of a tile overlaps the next tile's K loop), but inside an operator sequence its fixed tile
    // assignment loses what it gains: workgroups that start late, behind the tail of the previous kernel, still
    // walk their full share of tiles, while the per-tile grid is balanced by the hardware dispatcher.
    if(!p.tn && persistent_eligible(a, p.prec, plan.tile, splits)
       && g_persistent_mode == 1)
        return p.prec == 8 ? launch_persistent<I8Traits>(a, stream) : launch_persistent<F16Traits>(a, stream);
    hipError_t e = p.prec == 8    ? launch_traits<I8Traits>(plan.tile, a, splits, stream, p.tn)
                   : p.prec == 16 ? launch_traits<F16Traits>(plan.tile, a, splits, stream, p.tn)
                                  : launch_traits<F32Traits>(plan.tile, a, splits, stream);
    if(e != hipSuccess || splits == 1) return e;
    const bool vec4 = p.N % 4 == 0 && ((reinterpret_cast<uintptr_t>(workspace) | reinterpret_cast<uintptr_t>(p.C)) & 15) == 0;
    int64_t    nb   = (p.M * p.N / (vec4 ? 4 : 1) + kThreads - 1) / kThreads;
    nb              = nb > 65536 ? 65536 : nb;
    if(p.out_amax_bits && nb > 1024) nb = 1024;    // at most one atomic per workgroup on one word: keep them few
    auto reduce = [&](auto acc_tag, auto vec_tag, const void* ws, int32_t* dump) {
        typedef decltype(acc_tag) acc_t;
        splitk_reduce_kernel<acc_t, decltype(vec_tag)::value><<<dim3(nb), dim3(kThreads), 0, stream>>>(
            static_cast<const acc_t*>(ws), splits, p.M, p.N, p.C, a.c_is_f16, p.s0, p.s1, p.col_scale, p.col_bias, dump,
            p.out_amax_bits, static_cast<int8_t*>(p.out_codes), p.out_code_inv, p.out_code_qmax);
    };
    if(p.prec == 8)
    {
        if(vec4) reduce(int32_t{}, std::true_type{}, workspace, a.acc_dump);
        else     reduce(int32_t{}, std::false_type{}, workspace, a.acc_dump);
    }
    else
    {
        if(vec4) reduce(float{}, std::true_type{}, workspace, nullptr);
        else     reduce(float{}, std::false_type{}, workspace, nullptr);
    }
    return hipGetLastError();
}

}  // namespace qsync
