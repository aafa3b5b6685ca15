// Matrix-core GEMM core shared by every product of the library (internal header).
//
//   C[M x N] = scale * sum_k A(m,k) * B(n,k)
//
// Operands are fetched through small "loader" functors (one per tensor layout: plain matrices for
// the fully connected layer, implicit-im2col index maps for convolutions), converted while they are
// staged into LDS, and multiplied by MFMA 32x32 tiles.  Three arithmetic modes:
//
//   MODE_BF16  the dithered products, Eqs. (qda)/(qdw).  NSD codes are integers in [-127,127] and
//              therefore EXACT in bf16 (8 significant bits).  The fp32 operand (W or X) is cut into
//              three bf16 planes hi+mid+lo that add up to the fp32 value exactly, so every product
//              code*plane is exact in the fp32 accumulator and the result has plain fp32-accumulate
//              accuracy at bf16 matrix-core rate: 3 bf16 MFMAs replace 1 fp32 MFMA that is 16x slower.
//              Fragments of codes that are entirely zero skip their MFMAs (structured sparsity).
//   MODE_I8    the 8-bit mode: int8 codes x int8 activations, exact int32 accumulation.
//   MODE_F32   the dense baseline, Eqs. (da)/(dw): fp32 MFMA on the unquantised gradient.
//
// Tiling: 256 threads = 4 wavefronts per 256x128 output tile; each wavefront owns 128x64 =
// 4x2 MFMA blocks (128 accumulator registers).  K advances in steps of four 16-byte chunks per
// row (32 bf16 / 64 int8 / 16 fp32).  LDS layout per plane: [chunk][row] of 16-byte cells, so both
// the staging writes (lanes = consecutive rows) and the fragment reads (lanes = consecutive rows)
// are conflict-free 128-bit accesses.  Global loads for step k+1 are issued before the MFMAs of
// step k.  Split-K partials go to a workspace and are summed by reduce_kernel (deterministic).
#pragma once
#include <type_traits>
#include "common.h"

namespace dbp {

enum { MODE_BF16 = 0, MODE_I8 = 1, MODE_F32 = 2, MODE_BF16X2 = 3 };   // MODE_BF16X2: kernels with prepared operands only (two planes, below)

constexpr int TM = 256, TN = 128, NCHUNK = 4;

template <int MODE> struct ModeTraits;
template <> struct ModeTraits<MODE_BF16> { static constexpr int KCH = 8;  using Acc = float;   using AccV = f32x16; };
template <> struct ModeTraits<MODE_I8>   { static constexpr int KCH = 16; using Acc = int32_t; using AccV = i32x16; };
template <> struct ModeTraits<MODE_F32>  { static constexpr int KCH = 4;  using Acc = float;   using AccV = f32x16; };

// ----------------------------------------------------------------------------------------------
// Raw register images of one 16-byte LDS cell before conversion
// ----------------------------------------------------------------------------------------------
struct RawCodes8 { uint32_t w[2]; };      // 8 int8 codes
struct RawF32x8  { float v[8]; };         // 8 fp32 values (become 3 bf16 planes)
struct RawI8x16  { u32x4 w; };            // 16 int8
struct RawF32x4  { f32x4 v; };            // 4 fp32

__device__ __forceinline__ uint32_t bf16_pair_from_i8(int a, int b)
{
    // small integers are exact in bf16: the upper 16 bits of their fp32 image (one byte permute packs the two upper halves)
    return __builtin_amdgcn_perm(__float_as_uint((float)b), __float_as_uint((float)a), 0x07060302u);
}

__device__ __forceinline__ void convert(const RawCodes8 &r, u32x4 (&out)[1])
{
    u32x4 c;
    c.x = bf16_pair_from_i8((int8_t)(r.w[0]), (int8_t)(r.w[0] >> 8));
    c.y = bf16_pair_from_i8((int8_t)(r.w[0] >> 16), (int8_t)(r.w[0] >> 24));
    c.z = bf16_pair_from_i8((int8_t)(r.w[1]), (int8_t)(r.w[1] >> 8));
    c.w = bf16_pair_from_i8((int8_t)(r.w[1] >> 16), (int8_t)(r.w[1] >> 24));
    out[0] = c;
}

// x = hi + mid + lo exactly, each piece the top 16 bits of an fp32 (a bf16): truncation split,
// 8 + 8 + 8 significant bits cover the 24-bit significand.
__device__ __forceinline__ void split3(float x, uint32_t &hi, uint32_t &mid, uint32_t &lo)
{
    hi = __float_as_uint(x) & 0xFFFF0000u;
    float r1 = x - __uint_as_float(hi);
    mid = __float_as_uint(r1) & 0xFFFF0000u;
    float r2 = r1 - __uint_as_float(mid);
    lo = __float_as_uint(r2) & 0xFFFF0000u;
}

// Two-plane form of an fp32 operand, for callers that ask for it: x ~ hi + lo, hi the bf16 nearest to x, lo the bf16 nearest
// to the rest; |x - hi - lo| <= 2^-16 |x| (two round-to-nearest-even steps of 2^-8 each: a bf16 has 8 significant bits).
// Two values at a time with the hardware's packed conversion (v_cvt_pk_bf16_f32): `a` lands in the low half of each result,
// which is also the order of a fragment's elements.  Values beyond the bf16 range (|x| > 3.39e38) round to infinity, as
// IEEE conversion does, and their products are not finite.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float  f32x2_t  __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pack_nearest(float a, float b)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
}
__device__ __forceinline__ void split2_pk(float a, float b, uint32_t &hi, uint32_t &lo)
{
    hi = bf16_pack_nearest(a, b);
    lo = bf16_pack_nearest(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xFFFF0000u));
}

// The same split for callers that pack the pieces with a byte permute of the upper halves: `lo` keeps its lower 16 bits
// (the permute drops them), which saves the last mask.
__device__ __forceinline__ void split3_upper(float x, uint32_t &hi, uint32_t &mid, uint32_t &lo)
{
    hi = __float_as_uint(x) & 0xFFFF0000u;
    float r1 = x - __uint_as_float(hi);
    mid = __float_as_uint(r1) & 0xFFFF0000u;
    lo = __float_as_uint(r1 - __uint_as_float(mid));
}

__device__ __forceinline__ void convert(const RawF32x8 &r, u32x4 (&out)[3])
{
    uint32_t h[8], m[8], l[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) split3(r.v[j], h[j], m[j], l[j]);
    // plane order: 0 = lo, 1 = mid, 2 = hi (small terms are accumulated first)
    out[0] = u32x4{(l[0] >> 16) | l[1], (l[2] >> 16) | l[3], (l[4] >> 16) | l[5], (l[6] >> 16) | l[7]};
    out[1] = u32x4{(m[0] >> 16) | m[1], (m[2] >> 16) | m[3], (m[4] >> 16) | m[5], (m[6] >> 16) | m[7]};
    out[2] = u32x4{(h[0] >> 16) | h[1], (h[2] >> 16) | h[3], (h[4] >> 16) | h[5], (h[6] >> 16) | h[7]};
}

__device__ __forceinline__ void convert(const RawI8x16 &r, u32x4 (&out)[1]) { out[0] = r.w; }
__device__ __forceinline__ void convert(const RawF32x4 &r, u32x4 (&out)[1])
{
    out[0] = u32x4{__float_as_uint(r.v.x), __float_as_uint(r.v.y), __float_as_uint(r.v.z), __float_as_uint(r.v.w)};
}

// ----------------------------------------------------------------------------------------------
// Element access helpers: KCH consecutive reduction indices of one row
// ----------------------------------------------------------------------------------------------
// contiguous int8 run (reduction index is the fast axis in memory); n_valid may be < 8/16
__device__ __forceinline__ RawCodes8 load_i8_run8(const int8_t *p, int n_valid)
{
    RawCodes8 r = {{0u, 0u}};
    if (n_valid >= 8 && (((uintptr_t)p) & 3) == 0) {
        r.w[0] = *(const uint32_t *)p;
        r.w[1] = *(const uint32_t *)(p + 4);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (j < n_valid) r.w[j >> 2] |= (uint32_t)(uint8_t)p[j] << (8 * (j & 3));
    }
    return r;
}

__device__ __forceinline__ RawI8x16 load_i8_run16(const int8_t *p, int n_valid)
{
    RawI8x16 r;
    if (n_valid >= 16 && (((uintptr_t)p) & 3) == 0) {
        const uint32_t *q = (const uint32_t *)p;
        r.w = u32x4{q[0], q[1], q[2], q[3]};
    } else {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (j < n_valid) w[j >> 2] |= (uint32_t)(uint8_t)p[j] << (8 * (j & 3));
        r.w = u32x4{w[0], w[1], w[2], w[3]};
    }
    return r;
}

// strided runs (reduction index is the slow axis in memory)
__device__ __forceinline__ RawCodes8 load_i8_strided8(const int8_t *p, int64_t stride, int n_valid)
{
    RawCodes8 r = {{0u, 0u}};
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (j < n_valid) r.w[j >> 2] |= (uint32_t)(uint8_t)p[j * stride] << (8 * (j & 3));
    return r;
}
__device__ __forceinline__ RawI8x16 load_i8_strided16(const int8_t *p, int64_t stride, int n_valid)
{
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 16; ++j)
        if (j < n_valid) w[j >> 2] |= (uint32_t)(uint8_t)p[j * stride] << (8 * (j & 3));
    RawI8x16 r; r.w = u32x4{w[0], w[1], w[2], w[3]};
    return r;
}
__device__ __forceinline__ RawF32x8 load_f32_strided8(const float *p, int64_t stride, int n_valid)
{
    RawF32x8 r;
#pragma unroll
    for (int j = 0; j < 8; ++j) r.v[j] = j < n_valid ? p[j * stride] : 0.0f;
    return r;
}
__device__ __forceinline__ RawF32x4 load_f32_strided4(const float *p, int64_t stride, int n_valid)
{
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = j < n_valid ? p[j * stride] : 0.0f;
    RawF32x4 r; r.v = f32x4{v[0], v[1], v[2], v[3]};
    return r;
}
__device__ __forceinline__ RawF32x4 load_f32_run4(const float *p, int n_valid)
{
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = j < n_valid ? p[j] : 0.0f;
    RawF32x4 r; r.v = f32x4{v[0], v[1], v[2], v[3]};
    return r;
}

template <class Raw> __device__ __forceinline__ Raw raw_zero()
{
    Raw r;
    __builtin_memset(&r, 0, sizeof(Raw));
    return r;
}

// ----------------------------------------------------------------------------------------------
// Plain-matrix loaders.  Element (row, k) lives at base[row*row_stride + k*k_stride]; exactly one of
// the strides is 1.  KFAST = reduction index contiguous in memory.
// ----------------------------------------------------------------------------------------------
template <int MODE, bool IS_CODES_OR_I8, bool KFAST> struct MatrixLoader;

// int8 codes feeding the bf16 path
template <bool KFAST> struct MatrixLoader<MODE_BF16, true, KFAST> {
    using Raw = RawCodes8;
    static constexpr int PLANES = 1;
    static constexpr bool SPARSE = true;
    const int8_t *base; int64_t ld; int rows; int K;
    struct Row { const int8_t *p; bool ok; };
    __device__ Row row(int r) const { return Row{base + (KFAST ? (int64_t)r * ld : (int64_t)r), r < rows}; }
    __device__ Raw fetch(const Row &rw, int k0) const
    {
        const int nv = K - k0;
        if (!rw.ok || nv <= 0) return raw_zero<Raw>();
        return KFAST ? load_i8_run8(rw.p + k0, nv) : load_i8_strided8(rw.p + (int64_t)k0 * ld, ld, nv);
    }
};
// fp32 operand feeding the bf16 path as three planes
template <bool KFAST> struct MatrixLoader<MODE_BF16, false, KFAST> {
    using Raw = RawF32x8;
    static constexpr int PLANES = 3;
    static constexpr bool SPARSE = false;
    const float *base; int64_t ld; int rows; int K;
    struct Row { const float *p; bool ok; };
    __device__ Row row(int r) const { return Row{base + (KFAST ? (int64_t)r * ld : (int64_t)r), r < rows}; }
    __device__ Raw fetch(const Row &rw, int k0) const
    {
        const int nv = K - k0;
        if (!rw.ok || nv <= 0) return raw_zero<Raw>();
        return KFAST ? load_f32_strided8(rw.p + k0, 1, nv) : load_f32_strided8(rw.p + (int64_t)k0 * ld, ld, nv);
    }
};
// int8 x int8
template <bool ANY, bool KFAST> struct MatrixLoader<MODE_I8, ANY, KFAST> {
    using Raw = RawI8x16;
    static constexpr int PLANES = 1;
    static constexpr bool SPARSE = ANY;
    const int8_t *base; int64_t ld; int rows; int K;
    struct Row { const int8_t *p; bool ok; };
    __device__ Row row(int r) const { return Row{base + (KFAST ? (int64_t)r * ld : (int64_t)r), r < rows}; }
    __device__ Raw fetch(const Row &rw, int k0) const
    {
        const int nv = K - k0;
        if (!rw.ok || nv <= 0) return raw_zero<Raw>();
        return KFAST ? load_i8_run16(rw.p + k0, nv) : load_i8_strided16(rw.p + (int64_t)k0 * ld, ld, nv);
    }
};
// dense fp32
template <bool ANY, bool KFAST> struct MatrixLoader<MODE_F32, ANY, KFAST> {
    using Raw = RawF32x4;
    static constexpr int PLANES = 1;
    static constexpr bool SPARSE = false;
    const float *base; int64_t ld; int rows; int K;
    struct Row { const float *p; bool ok; };
    __device__ Row row(int r) const { return Row{base + (KFAST ? (int64_t)r * ld : (int64_t)r), r < rows}; }
    __device__ Raw fetch(const Row &rw, int k0) const
    {
        const int nv = K - k0;
        if (!rw.ok || nv <= 0) return raw_zero<Raw>();
        return KFAST ? load_f32_run4(rw.p + k0, nv) : load_f32_strided4(rw.p + (int64_t)k0 * ld, ld, nv);
    }
};

// Output index maps
struct RowMajorOut {
    int64_t ld;
    __device__ int64_t operator()(int row, int col) const { return (int64_t)row * ld + col; }
};

// ----------------------------------------------------------------------------------------------
// MFMA wrappers
// ----------------------------------------------------------------------------------------------
template <int MODE> struct Mma;
template <> struct Mma<MODE_BF16> {
    static __device__ __forceinline__ void run(const u32x4 &a, const u32x4 &b, f32x16 &c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<MODE_BF16X2> : Mma<MODE_BF16> {};
template <> struct Mma<MODE_I8> {
    static __device__ __forceinline__ void run(const u32x4 &a, const u32x4 &b, i32x16 &c)
    {
        c = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b), c, 0, 0, 0);
    }
};
template <> struct Mma<MODE_F32> {
    static __device__ __forceinline__ void run(const u32x4 &a, const u32x4 &b, f32x16 &c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

struct GemmShape {
    int M, N, K;            // K = full reduction length
    int k_per_split;        // multiple of the K step; gridDim.z splits
    int tiles_m, tiles_n;
};

// ----------------------------------------------------------------------------------------------
// The kernel
// ----------------------------------------------------------------------------------------------
template <int MODE, class AL, class BL, class OM>
__global__ __launch_bounds__(256, 2) void gemm_kernel(AL al, BL bl, OM om, GemmShape sh, Scale scale_arg,
                                                       typename ModeTraits<MODE>::Acc *out,
                                                       typename ModeTraits<MODE>::Acc *partial)
{
    using MT = ModeTraits<MODE>;
    using Acc = typename MT::Acc;
    using AccV = typename MT::AccV;
    constexpr int KCH = MT::KCH, KT = NCHUNK * KCH;
    constexpr int PA = AL::PLANES, PB = BL::PLANES;

    __shared__ u32x4 sA[PA][NCHUNK][TM];
    __shared__ u32x4 sB[PB][NCHUNK][TN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    // tile order: consecutive workgroups walk down M first, so neighbours share the B (N) tile
    const int tile_m = (blockIdx.x % sh.tiles_m) * TM;
    const int tile_n = (blockIdx.x / sh.tiles_m) * TN;
    const int k_begin = blockIdx.z * sh.k_per_split;
    const int k_end = min(sh.K, k_begin + sh.k_per_split);

    // staging ownership: A row = tid (all 4 chunks); B row = tid % 128, chunks 2*(tid/128) + {0,1}
    const typename AL::Row a_row = al.row(tile_m + tid);
    const int b_r = tid & (TN - 1), b_c0 = (tid >> 7) * 2;
    const typename BL::Row b_row = bl.row(tile_n + b_r);

    typename AL::Raw a_raw[NCHUNK];
    typename BL::Raw b_raw[2];
    auto prefetch = [&](int k0) {
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c) a_raw[c] = al.fetch(a_row, k0 + c * KCH);
#pragma unroll
        for (int c = 0; c < 2; ++c) b_raw[c] = bl.fetch(b_row, k0 + (b_c0 + c) * KCH);
    };

    AccV acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    // blocks of this wavefront that lie inside the matrix (wave-uniform)
    bool m_live[4], n_live[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) m_live[i] = tile_m + wr * 128 + i * 32 < sh.M;
#pragma unroll
    for (int j = 0; j < 2; ++j) n_live[j] = tile_n + wc * 64 + j * 32 < sh.N;

    if (k_begin < k_end) prefetch(k_begin);
    for (int k0 = k_begin; k0 < k_end; k0 += KT) {
        // registers -> LDS (with conversion)
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c) {
            u32x4 cell[PA];
            convert(a_raw[c], cell);
#pragma unroll
            for (int p = 0; p < PA; ++p) sA[p][c][tid] = cell[p];
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            u32x4 cell[PB];
            convert(b_raw[c], cell);
#pragma unroll
            for (int p = 0; p < PB; ++p) sB[p][b_c0 + c][b_r] = cell[p];
        }
        __syncthreads();
        if (k0 + KT < k_end) prefetch(k0 + KT);

#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int ch = 2 * kk + (lane >> 5);
            u32x4 bf[PB][2];
#pragma unroll
            for (int p = 0; p < PB; ++p)
#pragma unroll
                for (int j = 0; j < 2; ++j) bf[p][j] = sB[p][ch][wc * 64 + j * 32 + (lane & 31)];
            bool b_nz[2] = {true, true};
            if (BL::SPARSE) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    b_nz[j] = __builtin_amdgcn_ballot_w64((bf[0][j].x | bf[0][j].y | bf[0][j].z | bf[0][j].w) != 0u) != 0ull;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (!m_live[i]) continue;
                u32x4 af[PA];
#pragma unroll
                for (int p = 0; p < PA; ++p) af[p] = sA[p][ch][wr * 128 + i * 32 + (lane & 31)];
                if (AL::SPARSE) {
                    // all 32 rows x 16/32 reduction indices of codes are zero: nothing to add
                    if (__builtin_amdgcn_ballot_w64((af[0].x | af[0].y | af[0].z | af[0].w) != 0u) == 0ull) continue;
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (!n_live[j] || !b_nz[j]) continue;
#pragma unroll
                    for (int pa = 0; pa < PA; ++pa)
#pragma unroll
                        for (int pb = 0; pb < PB; ++pb) Mma<MODE>::run(af[pa], bf[pb][j], acc[i][j]);
                }
            }
        }
        __syncthreads();
    }

    // epilogue: D[i][j] of a 32x32 block sits in lane (j, i%8/4) register 4*(i/8) + i%4
    const bool direct = gridDim.z == 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = tile_n + wc * 64 + j * 32 + (lane & 31);
            if (col >= sh.N) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = tile_m + wr * 128 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row >= sh.M) continue;
                if (direct) {
                    if (MODE == MODE_I8) out[om(row, col)] = acc[i][j][v];
                    else out[om(row, col)] = (Acc)(scale_arg.get() * (float)acc[i][j][v]);
                } else {
                    partial[((int64_t)blockIdx.z * sh.M + row) * sh.N + col] = acc[i][j][v];
                }
            }
        }
    }
}

// Sum the split-K partials in a fixed order, scale, and scatter through the output map.
template <class Acc, class OM>
__global__ __launch_bounds__(256) void reduce_kernel(const Acc *partial, Acc *out, OM om, int M, int N, int nsplit, Scale scale_arg)
{
    const int64_t total = (int64_t)M * N;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        // eight running sums (splits z = 0..7 mod 8, each in split order, combined pairwise in a fixed order): eight loads
        // in flight per thread; small outputs with hundreds of splits were latency bound with one
        Acc t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = 0;
        int z = 0;
        for (; z + 8 <= nsplit; z += 8) {
            Acc v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(z + u) * total + idx];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] += v[u];
        }
        for (int u = 0; z < nsplit; ++z, ++u) t[u] += partial[(int64_t)z * total + idx];
        const Acc s = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
        const int row = (int)(idx / N), col = (int)(idx - (int64_t)row * N);
        if constexpr (std::is_same<Acc, float>::value) out[om(row, col)] = scale_arg.get() * s;
        else out[om(row, col)] = s;
    }
}

}  // namespace dbp
