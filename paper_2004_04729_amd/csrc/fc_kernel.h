// Fast matrix-core kernel for the two fully connected products, Eqs. (qda)/(qdw) (internal header).
//
//   dX[b,i] = Delta * sum_o code[b,o] W[o,i]      A = codes, reduction index contiguous  (a_kfast)
//   dW[o,i] = Delta * sum_b code[b,o] X[b,i]      A = codes^T, reduction index strided    (!a_kfast)
//
// In both products the fp32 operand is stored [reduction][column] with columns contiguous, so one B
// path serves both: 16-byte loads along the columns, a 3-way exact bf16 split in registers, and
// 8-byte LDS writes that assemble the [chunk][column] cells the MFMA fragments read.  Codes are
// widened to bf16 (exact) on the way into LDS.  Arithmetic and LDS cell layout are those of
// gemm_core.h; what differs is the data movement (no per-element predicates in the main loop: rows and
// columns outside the matrix are clamped to valid addresses and discarded at the store, only the last
// K step masks; a column/row permutation inside the tile makes every LDS access conflict-free) and
// the schedule:
//
//   * 128x128 tiles, 64 accumulator registers per wavefront, 32 KiB LDS per workgroup: three to four
//     workgroups share a CU and fill each other's wait states.
//   * ONE launch computes BOTH products.  Work items (tile, K-split) of the two products are dealt
//     alternately to persistent workgroups; a workgroup's stores of one item drain while it loads the
//     next.  dX streams W from HBM and writes little, dW reads little and writes its whole output,
//     so mixing the two keeps loads, matrix cores and stores busy at the same time instead of in
//     three chip-wide bursts.
//   * Split-K partials are written in thread order and summed in split order by one small second
//     launch for both products (deterministic).
#pragma once
#include "gemm_core.h"

namespace dbp {

constexpr int FC_TM = 128, FC_TN = 128, FC_KT = 32;

struct FcProblem {
    const int8_t *A; int64_t lda;     // a_kfast: A[m*lda + k]   else: A[k*lda + m]
    const float  *B; int64_t ldb;     // B[k*ldb + n]
    float *out; int64_t ldc;          // out[m*ldc + n]
    float *partial;                   // [tile][split][128*128] in thread order (n_split > 1)
    int M, N, K, k_per_split, n_split, tiles_m, n_items;
    Scale scale;
    int a_kfast;
    // Batched form of the kernel of fc2_kernel.h (both operands reduction-contiguous, one pair per image, accumulated):
    // A_img[m*lda + k], B_img[n*ldb + k], k < nt_pq; image i at A + i*nt_a_img, B + i*nt_b_img (elements); the
    // reduction axis K counts nt_spi windows of 32 per image.  nt_pq == 0: the plain form above.
    int nt_pq, nt_spi;
    int64_t nt_a_img, nt_b_img;
};
// gx > 0 (kernels of fc2_kernel.h / fc2_i8_kernel.h): the first gx workgroups of the launch take the items of problem 0, the
// others those of problem 1, each group dealing its items round robin; gx == 0: one list for both, dealt in a serpentine.
struct FcPairArgs { FcProblem prob[2]; StatsJob stats; int gx = 0; Gate gate; };

__device__ __forceinline__ uint32_t bf16x2_from_codes(int a, int b)
{
    // integers up to 127 in magnitude are exact in bf16 = the upper half of their fp32 image
    return __builtin_amdgcn_perm(__float_as_uint((float)b), __float_as_uint((float)a), 0x07060302u);
}

__device__ __forceinline__ uint32_t upper_halves(uint32_t hi_word, uint32_t lo_word)
{
    return __builtin_amdgcn_perm(hi_word, lo_word, 0x07060302u);    // {hi_word[31:16], lo_word[31:16]}
}

struct FcSmem {
    uint2 a[NCHUNK][FC_TM][2];        // [chunk][row position][half]          8 KiB
    uint2 b[3][NCHUNK][FC_TN][2];     // [plane][chunk][col position][half]  24 KiB
};

template <bool A_KFAST>
__device__ __forceinline__ void fc_item(const FcProblem &p, int item, FcSmem &sm)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int tile = item / p.n_split, z = item - tile * p.n_split;
    const int tile_m = (tile % p.tiles_m) * FC_TM;
    const int tile_n = (tile / p.tiles_m) * FC_TN;
    const int k_begin = z * p.k_per_split;
    const int k_end = min(p.K, k_begin + p.k_per_split);

    // B staging: thread owns columns 4*nq..4*nq+3 and reduction rows 4*kq..4*kq+3 of each step
    const int nq = tid & 31, kq = tid >> 5;
    const float *b_ptr = p.B + min(tile_n + 4 * nq, p.N - 4) + (int64_t)(4 * kq) * p.ldb;
    // A staging
    //   A_KFAST: thread owns row tid/2 and reduction indices 16*(tid&1) .. +15 (16 contiguous bytes)
    //   else   : thread owns rows 4*nq..4*nq+3 and reduction rows 4*kq..4*kq+3 (4 dwords), like B
    const int8_t *a_ptr = A_KFAST ? p.A + (int64_t)min(tile_m + (tid >> 1), p.M - 1) * p.lda + 16 * (tid & 1)
                                  : p.A + min(tile_m + 4 * nq, p.M - 4) + (int64_t)(4 * kq) * p.lda;

    f32x4 b_raw[4];
    uint32_t a_raw[4];

    auto prefetch = [&](int k0) {
        if (k0 + FC_KT <= k_end) {
#pragma unroll
            for (int r = 0; r < 4; ++r) b_raw[r] = *(const f32x4 *)(b_ptr + (int64_t)(k0 + r) * p.ldb);
            if (A_KFAST) {
#pragma unroll
                for (int r = 0; r < 4; ++r) a_raw[r] = *(const uint32_t *)(a_ptr + k0 + 4 * r);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) a_raw[r] = *(const uint32_t *)(a_ptr + (int64_t)(k0 + r) * p.lda);
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
                for (int r = 0; r < 4; ++r) {
                    uint32_t w = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (k0 + 16 * (tid & 1) + 4 * r + b < k_end) w |= (uint32_t)(uint8_t)a_ptr[k0 + 4 * r + b] << (8 * b);
                    a_raw[r] = w;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    a_raw[r] = 0u;
                    if (k0 + 4 * kq + r < k_end) a_raw[r] = *(const uint32_t *)(a_ptr + (int64_t)(k0 + r) * p.lda);
                }
            }
        }
    };

    auto stage = [&]() {
        if (A_KFAST) {
            // 16 codes = chunks 2*(tid&1), 2*(tid&1)+1 of row tid/2
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const uint32_t w0 = a_raw[2 * c], w1 = a_raw[2 * c + 1];
                sm.a[2 * (tid & 1) + c][tid >> 1][0] = uint2{bf16x2_from_codes((int8_t)w0, (int8_t)(w0 >> 8)),
                                                             bf16x2_from_codes((int8_t)(w0 >> 16), (int8_t)(w0 >> 24))};
                sm.a[2 * (tid & 1) + c][tid >> 1][1] = uint2{bf16x2_from_codes((int8_t)w1, (int8_t)(w1 >> 8)),
                                                             bf16x2_from_codes((int8_t)(w1 >> 16), (int8_t)(w1 >> 24))};
            }
        } else {
            // byte j of the 4 dwords = 4 consecutive reduction indices of row 4*nq+j -> position j*32+nq
#pragma unroll
            for (int j = 0; j < 4; ++j)
                sm.a[kq >> 1][j * 32 + nq][kq & 1] =
                    uint2{bf16x2_from_codes((int8_t)(a_raw[0] >> (8 * j)), (int8_t)(a_raw[1] >> (8 * j))),
                          bf16x2_from_codes((int8_t)(a_raw[2] >> (8 * j)), (int8_t)(a_raw[3] >> (8 * j)))};
        }
        // fp32 -> three exact bf16 planes; column 4*nq+j -> position j*32+nq
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t h[4], m[4], l[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) split3_upper(b_raw[r][j], h[r], m[r], l[r]);
            const int pos = j * 32 + nq;
            sm.b[0][kq >> 1][pos][kq & 1] = uint2{upper_halves(l[1], l[0]), upper_halves(l[3], l[2])};
            sm.b[1][kq >> 1][pos][kq & 1] = uint2{upper_halves(m[1], m[0]), upper_halves(m[3], m[2])};
            sm.b[2][kq >> 1][pos][kq & 1] = uint2{upper_halves(h[1], h[0]), upper_halves(h[3], h[2])};
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    if (k_begin < k_end) prefetch(k_begin);
    for (int k0 = k_begin; k0 < k_end; k0 += FC_KT) {
        stage();
        __syncthreads();
        if (k0 + FC_KT < k_end) prefetch(k0 + FC_KT);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int ch = 2 * kk + (lane >> 5);
            u32x4 bf[3][2], af[2];
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    bf[pl][j] = *(const u32x4 *)&sm.b[pl][ch][wc * 64 + j * 32 + (lane & 31)][0];
#pragma unroll
            for (int i = 0; i < 2; ++i) af[i] = *(const u32x4 *)&sm.a[ch][wr * 64 + i * 32 + (lane & 31)][0];
            // planes outermost: consecutive MFMAs accumulate into different blocks
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) Mma<MODE_BF16>::run(af[i], bf[pl][j], acc[i][j]);
        }
        __syncthreads();
    }

    // ---- split-K: park the partial tile in thread order; fc_reduce_kernel sums the splits in a fixed
    // order.  (Summing in the last workgroup to arrive was tried: it needs device-scope fences, and on
    // this multi-XCD part each such fence writes back a whole L2 -- 10x slower than a second launch.)
    if (p.n_split > 1) {
        float2 *mine = (float2 *)(p.partial + ((int64_t)tile * p.n_split + z) * (FC_TM * FC_TN));
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) mine[(i * 16 + v) * 256 + tid] = float2{acc[i][0][v], acc[i][1][v]};
        return;
    }

    // ---- epilogue: block (i,j) covers row positions (2*wr+i)*32.. and column positions (2*wc+j)*32..;
    // D[ii][jj] of a block sits in lane (jj, ii%8/4), register 4*(ii/8)+ii%4.
    const int col = tile_n + 4 * (lane & 31) + 2 * wc;          // columns col, col+1 (j = 0, 1)
    const float sc = p.scale.get();
    if (col < p.N) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int mbg = wr * 2 + i;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int ii = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int row = A_KFAST ? tile_m + mbg * 32 + ii : tile_m + 4 * ii + mbg;
                if (row < p.M)
                    *(float2 *)(p.out + (int64_t)row * p.ldc + col) = float2{sc * acc[i][0][v], sc * acc[i][1][v]};
            }
        }
    }
}

// Sum of the quantiser's per-workgroup statistics records by one workgroup of 256 threads (integer
// sums and a maximum: the result does not depend on the order).
__device__ __forceinline__ void fc_sum_stats(const StatsJob &j, uint64_t *lds)
{
    uint64_t nnz = 0, sat = 0, nf = 0, mx = 0;
    for (int i = threadIdx.x; i < j.n; i += 256) {
        const u32x4 q = j.partials[i];
        nnz += q.x; sat += q.y; nf += q.z; mx = mx > q.w ? mx : q.w;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        nnz += __shfl_xor((unsigned long long)nnz, off); sat += __shfl_xor((unsigned long long)sat, off);
        nf += __shfl_xor((unsigned long long)nf, off);
        const uint64_t o = __shfl_xor((unsigned long long)mx, off);
        mx = mx > o ? mx : o;
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { lds[4 * wave] = nnz; lds[4 * wave + 1] = sat; lds[4 * wave + 2] = nf; lds[4 * wave + 3] = mx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t m = 0;
        for (int w = 0; w < 4; ++w) m = m > lds[4 * w + 3] ? m : lds[4 * w + 3];
        j.out->nnz = lds[0] + lds[4] + lds[8] + lds[12];
        j.out->n_saturated = lds[1] + lds[5] + lds[9] + lds[13];
        j.out->n_nonfinite = lds[2] + lds[6] + lds[10] + lds[14];
        j.out->max_abs_code = (int32_t)m; j.out->reserved = 0;
    }
    __syncthreads();                                        // the items reuse this LDS
}

// Persistent workgroups; items of the two problems alternate (even = problem 0, odd = problem 1) for as
// long as both have items left, so that neighbouring workgroups work on different products.
__global__ __launch_bounds__(256, 3) void fc_pair_kernel(FcPairArgs a)
{
    if (a.gate.closed()) return;
    __shared__ FcSmem sm;
    // the last workgroup has the fewest items: it also finishes the quantiser's statistics
    if (a.stats.n > 0 && blockIdx.x == gridDim.x - 1) fc_sum_stats(a.stats, (uint64_t *)&sm);
    const int n0 = a.prob[0].n_items, n1 = a.prob[1].n_items;
    const int both = 2 * min(n0, n1), total = n0 + n1;
    for (int t = blockIdx.x; t < total; t += gridDim.x) {
        int which, item;
        if (t < both) { which = t & 1; item = t >> 1; }
        else { which = n0 > n1 ? 0 : 1; item = t - both + (both >> 1); }
        const FcProblem &p = a.prob[which];
        if (p.a_kfast) fc_item<true>(p, item, sm);
        else fc_item<false>(p, item, sm);
        __syncthreads();                                    // LDS is reused by the next item
    }
}

// Second launch of a split-K run: workgroup (tile, slot) sums the partials of one of the tile's 32 accumulator slots
// over the splits and writes the output with the item's own mapping.  Four running sums (splits q = 0, 1, 2, 3 mod 4,
// each in split order, added as (s0 + s1) + (s2 + s3)): a fixed order, and four loads in flight per thread; with few
// tiles and hundreds of splits (a convolution's dW lowered to this kernel) one sum per thread was latency bound.
__global__ __launch_bounds__(256) void fc_reduce_kernel(FcPairArgs a, int tiles0)
{
    if (a.gate.closed()) return;
    const int which = (int)(blockIdx.x >> 5) < tiles0 ? 0 : 1;
    const FcProblem &p = a.prob[which];
    const int tile = (int)(blockIdx.x >> 5) - (which ? tiles0 : 0), slot = blockIdx.x & 31;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int tile_m = (tile % p.tiles_m) * FC_TM;
    const int tile_n = (tile / p.tiles_m) * FC_TN;
    const float2 *src = (const float2 *)(p.partial + (int64_t)tile * p.n_split * (FC_TM * FC_TN)) + slot * 256 + tid;
    const int64_t per_split = FC_TM * FC_TN / 2;
    float2 s4[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) s4[u] = float2{0.f, 0.f};
    int q = 0;
    for (; q + 4 <= p.n_split; q += 4) {
        float2 t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = src[(int64_t)(q + u) * per_split];
#pragma unroll
        for (int u = 0; u < 4; ++u) { s4[u].x += t[u].x; s4[u].y += t[u].y; }
    }
    for (int u = 0; q < p.n_split; ++q, ++u) {
        const float2 t = src[(int64_t)q * per_split];
        s4[u].x += t.x; s4[u].y += t.y;
    }
    const float2 sum = float2{(s4[0].x + s4[1].x) + (s4[2].x + s4[3].x), (s4[0].y + s4[1].y) + (s4[2].y + s4[3].y)};
    const int col = tile_n + 4 * (lane & 31) + 2 * wc;
    if (col >= p.N) return;
    const float sc = p.scale.get();
    const int i = slot >> 4, v = slot & 15;
    const int mbg = wr * 2 + i;
    const int ii = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    const int row = p.a_kfast ? tile_m + mbg * 32 + ii : tile_m + 4 * ii + mbg;
    if (row < p.M) *(float2 *)(p.out + (int64_t)row * p.ldc + col) = float2{sc * sum.x, sc * sum.y};
}

}  // namespace dbp
