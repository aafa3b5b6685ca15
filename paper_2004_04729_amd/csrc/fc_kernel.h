// Fast matrix-core kernel for the two fully connected products, Eqs. (qda)/(qdw) (internal header).
//
//   dX[b,i] = Delta * sum_o code[b,o] W[o,i]      A = codes, reduction index contiguous  (A_KFAST)
//   dW[o,i] = Delta * sum_b code[b,o] X[b,i]      A = codes^T, reduction index strided    (!A_KFAST)
//
// In both products the fp32 operand is stored [reduction][column] with columns contiguous, so one B
// path serves both: 16-byte loads along the columns, a 3-way exact bf16 split in registers, and
// 8-byte LDS writes that assemble the [chunk][column] cells the MFMA fragments read.  Codes are
// widened to bf16 (exact) on the way into LDS.  Arithmetic, tile shape and LDS cell layout are those
// of gemm_core.h; what differs is the data movement: no per-element predicates in the main loop
// (rows/columns outside the matrix are clamped to valid addresses and discarded at the store, only
// the last K step masks), and a column/row permutation inside the tile that makes every LDS write
// and read conflict-free and gives each lane adjacent output columns (8-byte stores).
#pragma once
#include "gemm_core.h"

namespace dbp {

struct FcArgs {
    const int8_t *A; int64_t lda;     // A_KFAST: A[m*lda + k]   else: A[k*lda + m]
    const float  *B; int64_t ldb;     // B[k*ldb + n]
    float *out; int64_t ldc;          // out[m*ldc + n]
    float *partial;                   // split-K partials [z][M][N]
    int M, N, K, k_per_split, tiles_m;
    float scale;
};

__device__ __forceinline__ uint32_t bf16x2_from_codes(int a, int b)
{
    // integers up to 127 in magnitude are exact in bf16 = the upper half of their fp32 image
    return __builtin_amdgcn_perm(__float_as_uint((float)b), __float_as_uint((float)a), 0x07060302u);
}

__device__ __forceinline__ uint32_t upper_halves(uint32_t hi_word, uint32_t lo_word)
{
    return __builtin_amdgcn_perm(hi_word, lo_word, 0x07060302u);    // {hi_word[31:16], lo_word[31:16]}
}

template <bool A_KFAST, int AVEC>
__global__ __launch_bounds__(256, 2) void fc_bf16_kernel(FcArgs p)
{
    constexpr int KT = 32;
    __shared__ u32x4 sA[NCHUNK][TM];               // [chunk][row position]          16 KiB
    __shared__ uint2 sB[3][NCHUNK][TN][2];         // [plane][chunk][col position][half]  24 KiB

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int tile_m = (blockIdx.x % p.tiles_m) * TM;
    const int tile_n = (blockIdx.x / p.tiles_m) * TN;
    const int k_begin = blockIdx.z * p.k_per_split;
    const int k_end = min(p.K, k_begin + p.k_per_split);

    // ---- B staging: thread owns columns 4*nq..4*nq+3 and reduction rows 4*kq..4*kq+3 of each step
    const int nq = tid & 31, kq = tid >> 5;
    const float *b_ptr = p.B + min(tile_n + 4 * nq, p.N - 4) + (int64_t)(4 * kq) * p.ldb;
    // ---- A staging
    //   A_KFAST: thread owns row tid, all 32 reduction indices (32 contiguous bytes)
    //   else   : thread owns rows 4*mq..4*mq+3 and reduction rows 8*wave..8*wave+7 (8 dwords)
    const int mq = tid & 63;
    const int8_t *a_ptr = A_KFAST ? p.A + (int64_t)min(tile_m + tid, p.M - 1) * p.lda
                                  : p.A + min(tile_m + 4 * mq, p.M - 4) + (int64_t)(8 * wave) * p.lda;

    f32x4 b_raw[4];
    uint32_t a_raw[8];

    auto prefetch = [&](int k0) {
        if (k0 + KT <= k_end) {
#pragma unroll
            for (int r = 0; r < 4; ++r) b_raw[r] = *(const f32x4 *)(b_ptr + (int64_t)(k0 + r) * p.ldb);
            if (A_KFAST) {
                const int8_t *q = a_ptr + k0;
                if (AVEC == 16) {
                    const u32x4 v0 = *(const u32x4 *)q, v1 = *(const u32x4 *)(q + 16);
                    a_raw[0] = v0.x; a_raw[1] = v0.y; a_raw[2] = v0.z; a_raw[3] = v0.w;
                    a_raw[4] = v1.x; a_raw[5] = v1.y; a_raw[6] = v1.z; a_raw[7] = v1.w;
                } else if (AVEC == 8) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) { const uint2 v = *(const uint2 *)(q + 8 * r); a_raw[2 * r] = v.x; a_raw[2 * r + 1] = v.y; }
                } else {
#pragma unroll
                    for (int r = 0; r < 8; ++r) a_raw[r] = *(const uint32_t *)(q + 4 * r);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 8; ++r) a_raw[r] = *(const uint32_t *)(a_ptr + (int64_t)(k0 + r) * p.lda);
            }
        } else {
            // last, partial K step: mask by reduction index (zero codes and zero weights add exactly 0)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                b_raw[r] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (k0 + 4 * kq + r < k_end) b_raw[r] = *(const f32x4 *)(b_ptr + (int64_t)(k0 + r) * p.ldb);
            }
            if (A_KFAST) {
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    uint32_t w = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (k0 + 4 * r + b < k_end) w |= (uint32_t)(uint8_t)a_ptr[k0 + 4 * r + b] << (8 * b);
                    a_raw[r] = w;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    a_raw[r] = 0u;
                    if (k0 + 8 * wave + r < k_end) a_raw[r] = *(const uint32_t *)(a_ptr + (int64_t)(k0 + r) * p.lda);
                }
            }
        }
    };

    auto stage = [&]() {
        // ---- codes -> bf16 cells
        if (A_KFAST) {
#pragma unroll
            for (int c = 0; c < NCHUNK; ++c) {
                const uint32_t w0 = a_raw[2 * c], w1 = a_raw[2 * c + 1];
                u32x4 cell;
                cell.x = bf16x2_from_codes((int8_t)w0, (int8_t)(w0 >> 8));
                cell.y = bf16x2_from_codes((int8_t)(w0 >> 16), (int8_t)(w0 >> 24));
                cell.z = bf16x2_from_codes((int8_t)w1, (int8_t)(w1 >> 8));
                cell.w = bf16x2_from_codes((int8_t)(w1 >> 16), (int8_t)(w1 >> 24));
                sA[c][tid] = cell;
            }
        } else {
            // byte j of the 8 dwords = 8 consecutive reduction indices of row 4*mq+j -> position j*64+mq
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                u32x4 cell;
                cell.x = bf16x2_from_codes((int8_t)(a_raw[0] >> (8 * j)), (int8_t)(a_raw[1] >> (8 * j)));
                cell.y = bf16x2_from_codes((int8_t)(a_raw[2] >> (8 * j)), (int8_t)(a_raw[3] >> (8 * j)));
                cell.z = bf16x2_from_codes((int8_t)(a_raw[4] >> (8 * j)), (int8_t)(a_raw[5] >> (8 * j)));
                cell.w = bf16x2_from_codes((int8_t)(a_raw[6] >> (8 * j)), (int8_t)(a_raw[7] >> (8 * j)));
                sA[wave][j * 64 + mq] = cell;
            }
        }
        // ---- fp32 -> three exact bf16 planes; column 4*nq+j -> position j*32+nq
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t h[4], m[4], l[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) split3(b_raw[r][j], h[r], m[r], l[r]);
            const int pos = j * 32 + nq;
            sB[0][kq >> 1][pos][kq & 1] = uint2{upper_halves(l[1], l[0]), upper_halves(l[3], l[2])};
            sB[1][kq >> 1][pos][kq & 1] = uint2{upper_halves(m[1], m[0]), upper_halves(m[3], m[2])};
            sB[2][kq >> 1][pos][kq & 1] = uint2{upper_halves(h[1], h[0]), upper_halves(h[3], h[2])};
        }
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    if (k_begin < k_end) prefetch(k_begin);
    for (int k0 = k_begin; k0 < k_end; k0 += KT) {
        stage();
        __syncthreads();
        if (k0 + KT < k_end) prefetch(k0 + KT);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int ch = 2 * kk + (lane >> 5);
            u32x4 bf[3][2];
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    bf[pl][j] = *(const u32x4 *)&sB[pl][ch][wc * 64 + j * 32 + (lane & 31)][0];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const u32x4 af = sA[ch][wr * 128 + i * 32 + (lane & 31)];
                // 32 rows x 16 reduction indices of codes all zero: nothing to add (structured sparsity)
                if (__builtin_amdgcn_ballot_w64((af.x | af.y | af.z | af.w) != 0u) == 0ull) continue;
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int pl = 0; pl < 3; ++pl) Mma<MODE_BF16>::run(af, bf[pl][j], acc[i][j]);
            }
        }
        __syncthreads();
    }

    // ---- epilogue.  Block (i,j) of this wavefront covers row positions (4*wr+i)*32.. and column
    // positions (2*wc+j)*32..; D[ii][jj] of a block sits in lane (jj, ii%8/4), register 4*(ii/8)+ii%4.
    const bool direct = gridDim.z == 1;
    const int col = tile_n + 4 * (lane & 31) + 2 * wc;          // columns col, col+1 (j = 0, 1)
    if (col < p.N) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int mbg = wr * 4 + i;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int ii = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int row = A_KFAST ? tile_m + mbg * 32 + ii : tile_m + 128 * (mbg & 1) + 4 * ii + (mbg >> 1);
                if (row >= p.M) continue;
                if (direct) {
                    *(float2 *)(p.out + (int64_t)row * p.ldc + col) = float2{p.scale * acc[i][0][v], p.scale * acc[i][1][v]};
                } else {
                    *(float2 *)(p.partial + ((int64_t)blockIdx.z * p.M + row) * p.N + col) = float2{acc[i][0][v], acc[i][1][v]};
                }
            }
        }
    }
}

// float4 reduction of split-K partials for plain row-major outputs (N % 4 == 0, ldc % 4 == 0)
__global__ __launch_bounds__(256) void reduce4_kernel(const f32x4 *partial, float *out, int64_t ldc, int M, int N4, int nsplit, float scale)
{
    const int64_t total = (int64_t)M * N4;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        f32x4 s = partial[idx];
        for (int z = 1; z < nsplit; ++z) s += partial[(int64_t)z * total + idx];
        const int row = (int)(idx / N4), c4 = (int)(idx - (int64_t)row * N4);
        *(f32x4 *)(out + (int64_t)row * ldc + 4 * c4) = s * scale;
    }
}

}  // namespace dbp
