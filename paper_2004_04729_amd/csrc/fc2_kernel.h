// Fully connected products, Eqs. (qda)/(qdw), with separate staging and multiplying wavefronts
// (internal header; arithmetic, LDS cell layout and operand conventions are those of fc_kernel.h).
//
// A workgroup has eight wavefronts and a CU to itself.  Wavefronts 0-3 (64 rows x 128 columns each) do
// nothing but read matrix-core fragments from LDS and multiply; wavefronts 4-7 do nothing but move data:
// global loads three K steps ahead into a ring of register sets, the exact bf16x3 split of the fp32
// operand and the widening of the codes on the vector ALUs, and the writes into the other half of a
// double-buffered LDS stage.  The two groups meet at one barrier per K step, so conversion, global-load
// latency and LDS writes overlap the matrix cores instead of alternating with them.
//
//   * 256x128 tiles: per K step of 32 a multiplying wavefront reads 28 fragments for 48 matrix-core
//     instructions, and owns whole 512-byte row segments of the output (16-byte stores).
//   * The workgroups are persistent; work items (tile, K-split) of the two products are dealt so that every
//     workgroup gets the same number of K steps; the stagers run ahead across item borders, so the loads of the next item are under
//     way while the multipliers store the finished tile.
//   * Split-K partials are written in thread order and summed in split order by fc2_reduce_kernel
//     (deterministic).
#pragma once
#include "fc_kernel.h"

namespace dbp {

constexpr int FC2_TM = 256, FC2_TN = 128, FC2_KT = 32;
constexpr int FC2_LDS_BYTES = 2 * (16 + 24) * 1024;

struct Fc2Stage {
    uint2 a[NCHUNK][FC2_TM][2];       // [chunk][row position][half]          16 KiB
    uint2 b[3][NCHUNK][FC2_TN][2];    // [plane][chunk][col position][half]   24 KiB
};
static_assert(sizeof(Fc2Stage) * 2 == FC2_LDS_BYTES, "two stages");

// Position of a workgroup in its sequence of (item, K step) pairs; both roles walk the same sequence.
struct Fc2Cursor {
    int t;                            // position in this workgroup's list of items
    int which, tile, z, tile_m, tile_n, k0, k_end;
};

// The i-th work item of this workgroup.  Items are numbered with those of problem 0 first (the longer
// ones in a backward pass: dX keeps the whole reduction of a layer) and dealt in a serpentine over the
// workgroups (pass p gives workgroup w item p*G + w, the next pass p*G + G-1-w), which balances the number
// of K steps; every workgroup then starts at a different place of its own list (rotation by w), so that
// the tiles of the chip are not all finished, and stored, at the same moment.
__device__ __forceinline__ bool fc2_open(const FcPairArgs &a, int i, Fc2Cursor &c)
{
    const int n0 = a.prob[0].n_items, total = n0 + a.prob[1].n_items;
    const int G = gridDim.x, w = blockIdx.x;
    const int passes = (total + G - 1) / G;
    const int last = (passes - 1) * G + (((passes - 1) & 1) ? G - 1 - w : w);
    const int mine = last < total ? passes : passes - 1;             // items of this workgroup
    if (i >= mine) return false;
    const int ps = (i + w) % mine;
    const int t = ps * G + ((ps & 1) ? G - 1 - w : w);
    c.which = t < n0 ? 0 : 1;
    const int item = t < n0 ? t : t - n0;
    const FcProblem &p = a.prob[c.which];
    c.t = i;
    c.tile = item / p.n_split; c.z = item - c.tile * p.n_split;
    c.tile_m = (c.tile % p.tiles_m) * FC2_TM;
    c.tile_n = (c.tile / p.tiles_m) * FC2_TN;
    c.k0 = c.z * p.k_per_split;
    c.k_end = min(p.K, c.k0 + p.k_per_split);
    return true;
}

// K steps of all items of this workgroup (the trip count of both roles).
__device__ __forceinline__ int fc2_total_steps(const FcPairArgs &a)
{
    int g = 0;
    Fc2Cursor c;
    for (int i = 0; fc2_open(a, i, c); ++i) g += (c.k_end - c.k0 + FC2_KT - 1) / FC2_KT;
    return g;
}

struct Fc2Raw {                       // one K step of one stager thread, as loaded
    f32x4 b[4];
    uint32_t a[8];
    int kfast, k_valid;               // operand layout of the item; reduction indices of the step that exist
};

// Sum of the quantiser's statistics records by one wavefront (integers: any order gives the same result).
__device__ __forceinline__ void fc2_sum_stats(const StatsJob &j, int lane)
{
    uint64_t nnz = 0, sat = 0, nf = 0, mx = 0;
    for (int i = lane; i < j.n; i += 64) {
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
    if (lane == 0) {
        j.out->nnz = nnz; j.out->n_saturated = sat; j.out->n_nonfinite = nf;
        j.out->max_abs_code = (int32_t)mx; j.out->reserved = 0;
    }
}

// Bias gradient of the layer from the quantiser's code sums: one fp64 product rounded to fp32 per element.
__device__ __forceinline__ void fc2_bias_grad(const StatsJob &j, int lane)
{
    const double d = j.step_dev ? (double)j.step_dev[0] : (double)j.step;
    for (int64_t i = lane; i < j.bias_len; i += 64) j.bias_grad[i] = (float)(d * (double)j.bias_sums[i]);
}

// Matrix row of element ii of row block i of multiplier wavefront `wave`: row positions are rows
// (a_kfast) or, inside each 128-row half, the interleave 4*nq + j -> position 32*j + nq of the staging.
__device__ __forceinline__ int fc2_row(int a_kfast, int tile_m, int wave, int i, int ii)
{
    return a_kfast ? tile_m + wave * 64 + i * 32 + ii
                   : tile_m + 128 * (wave >> 1) + 4 * ii + 2 * (wave & 1) + i;
}

__global__ __launch_bounds__(512, 1) void fc2_pair_kernel(FcPairArgs a)
{
    extern __shared__ uint4 fc2_lds[];
    Fc2Stage *stages = (Fc2Stage *)fc2_lds;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int G = fc2_total_steps(a);

    if (wave >= 4) {
        // ================================ stagers ================================
        const int tid = threadIdx.x & 255;
        // the last workgroup has the fewest items: one of its stager wavefronts finishes the quantiser's
        // statistics and the bias gradient
        if (blockIdx.x == gridDim.x - 1 && wave == 7) {
            if (a.stats.n > 0) fc2_sum_stats(a.stats, lane);
            if (a.stats.bias_len > 0) fc2_bias_grad(a.stats, lane);
        }
        const int nq = tid & 31, kq = tid >> 5;
        Fc2Cursor c;
        bool open = fc2_open(a, 0, c);

        // Loads of the cursor's K step; then the cursor moves on (to the next item after an item's last
        // step).  Straight-line: reduction indices past the end of the item are clamped to its last one here
        // and zeroed when the step is committed (zero weights and zero codes add exactly 0).
        auto issue = [&](Fc2Raw &r) {
            if (!open) return;
            const FcProblem &p = a.prob[c.which];
            const int k0 = c.k0, k_last = c.k_end - 1;
            r.kfast = p.a_kfast;
            r.k_valid = c.k_end - k0;
            const float *b_col = p.B + min(c.tile_n + 4 * nq, p.N - 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) r.b[i] = *(const f32x4 *)(b_col + (int64_t)min(k0 + 4 * kq + i, k_last) * p.ldb);
            if (p.a_kfast) {
                // row tid of the tile, 32 consecutive reduction indices (8 dwords; K is a multiple of 4 here)
                const int8_t *a_row = p.A + (int64_t)min(c.tile_m + tid, p.M - 1) * p.lda;
#pragma unroll
                for (int i = 0; i < 8; ++i) r.a[i] = *(const uint32_t *)(a_row + min(k0 + 4 * i, p.K - 4));
            } else {
                // rows 4*nq..4*nq+3 of each 128-row half, reduction rows 4*kq..4*kq+3 (one dword each)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int8_t *a_col = p.A + min(c.tile_m + 128 * h + 4 * nq, p.M - 4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) r.a[4 * h + i] = *(const uint32_t *)(a_col + (int64_t)min(k0 + 4 * kq + i, k_last) * p.lda);
                }
            }
            c.k0 += FC2_KT;
            if (c.k0 >= c.k_end) open = fc2_open(a, c.t + 1, c);
        };

        auto commit = [&](const Fc2Raw &r, Fc2Stage &sm) {
            const int kv = r.k_valid;                                // reduction indices of this step that exist (>= 32: all)
            if (r.kfast) {
                // dwords 2c, 2c+1 = chunk c of row tid
#pragma unroll
                for (int ch = 0; ch < 4; ++ch) {
                    uint32_t w0 = r.a[2 * ch], w1 = r.a[2 * ch + 1];
                    if (kv < FC2_KT) {
                        const int n0 = kv - 8 * ch, n1 = n0 - 4;       // valid bytes of the two dwords
                        w0 = n0 >= 4 ? w0 : n0 > 0 ? w0 & ((1u << (8 * n0)) - 1u) : 0u;
                        w1 = n1 >= 4 ? w1 : n1 > 0 ? w1 & ((1u << (8 * n1)) - 1u) : 0u;
                    }
                    sm.a[ch][tid][0] = uint2{bf16x2_from_codes((int8_t)w0, (int8_t)(w0 >> 8)),
                                             bf16x2_from_codes((int8_t)(w0 >> 16), (int8_t)(w0 >> 24))};
                    sm.a[ch][tid][1] = uint2{bf16x2_from_codes((int8_t)w1, (int8_t)(w1 >> 8)),
                                             bf16x2_from_codes((int8_t)(w1 >> 16), (int8_t)(w1 >> 24))};
                }
            } else {
                // byte j of the 4 dwords = 4 consecutive reduction indices of row 4*nq+j -> position j*32+nq of its half
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    uint32_t w[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) w[i] = 4 * kq + i < kv ? r.a[4 * h + i] : 0u;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        sm.a[kq >> 1][128 * h + j * 32 + nq][kq & 1] =
                            uint2{bf16x2_from_codes((int8_t)(w[0] >> (8 * j)), (int8_t)(w[1] >> (8 * j))),
                                  bf16x2_from_codes((int8_t)(w[2] >> (8 * j)), (int8_t)(w[3] >> (8 * j)))};
                }
            }
            // fp32 -> three exact bf16 planes; column 4*nq+j -> position j*32+nq
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t h[4], m[4], l[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) split3(4 * kq + i < kv ? r.b[i][j] : 0.0f, h[i], m[i], l[i]);
                const int pos = j * 32 + nq;
                sm.b[0][kq >> 1][pos][kq & 1] = uint2{upper_halves(l[1], l[0]), upper_halves(l[3], l[2])};
                sm.b[1][kq >> 1][pos][kq & 1] = uint2{upper_halves(m[1], m[0]), upper_halves(m[3], m[2])};
                sm.b[2][kq >> 1][pos][kq & 1] = uint2{upper_halves(h[1], h[0]), upper_halves(h[3], h[2])};
            }
        };

        // Step g lives in register set g % 3 and LDS stage g % 2.  Barriers: one after step 0 is staged, then
        // one per step; in the iteration of step g the stagers write step g + 1 and load step g + 4.
        Fc2Raw r0, r1, r2;
        issue(r0); issue(r1); issue(r2);
        if (G > 0) commit(r0, stages[0]);
        issue(r0);
        __syncthreads();
        for (int g = 0; g < G; g += 3) {
            if (g + 1 < G) { commit(r1, stages[(g + 1) & 1]); issue(r1); }
            __syncthreads();
            if (g + 1 < G) {
                if (g + 2 < G) { commit(r2, stages[(g + 2) & 1]); issue(r2); }
                __syncthreads();
            }
            if (g + 2 < G) {
                if (g + 3 < G) { commit(r0, stages[(g + 3) & 1]); issue(r0); }
                __syncthreads();
            }
        }
        return;
    }

    // ================================ multipliers ================================
    // Wavefront w owns rows 64*w .. 64*w+63 of the tile and all 128 columns: a lane then holds four
    // adjacent columns of a row (one from each column block), i.e. 16-byte stores and whole cache lines.
    const int tid = threadIdx.x;
    const int lcol = lane & 31, lhalf = lane >> 5;
    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    Fc2Cursor c;
    fc2_open(a, 0, c);
    const float scale0 = a.prob[0].scale.get(), scale1 = a.prob[1].scale.get();   // resolved once (host value or device Delta)

    __syncthreads();
    for (int g = 0; g < G; ++g) {
        const Fc2Stage &sm = stages[g & 1];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int ch = 2 * kk + lhalf;
            u32x4 af[2], bf[3][4];
#pragma unroll
            for (int i = 0; i < 2; ++i) af[i] = *(const u32x4 *)&sm.a[ch][wave * 64 + i * 32 + lcol][0];
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
#pragma unroll
                for (int j = 0; j < 4; ++j) bf[pl][j] = *(const u32x4 *)&sm.b[pl][ch][j * 32 + lcol][0];
            // planes outermost: consecutive instructions accumulate into different blocks
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) Mma<MODE_BF16>::run(af[i], bf[pl][j], acc[i][j]);
        }
        c.k0 += FC2_KT;
        if (c.k0 >= c.k_end) {
            // ---- the item is complete: store (the stagers are already loading the next one) ----
            const FcProblem &p = a.prob[c.which];
            if (p.n_split > 1) {
                // partial tile in thread order; fc2_reduce_kernel sums the splits in a fixed order
                float4 *mine = (float4 *)(p.partial + ((int64_t)c.tile * p.n_split + c.z) * (FC2_TM * FC2_TN));
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        mine[(i * 16 + v) * 256 + tid] = float4{acc[i][0][v], acc[i][1][v], acc[i][2][v], acc[i][3][v]};
            } else {
                // block (i,j) covers row positions 64*wave + 32*i.. and column positions 32*j.. (column 4*lcol + j);
                // D[ii][jj] of a block sits in lane (jj, ii%8/4), register 4*(ii/8)+ii%4.
                const int col = c.tile_n + 4 * lcol;
                const float sc = c.which ? scale1 : scale0;
                if (col < p.N) {
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int ii = 8 * (v >> 2) + 4 * lhalf + (v & 3);
                            const int row = fc2_row(p.a_kfast, c.tile_m, wave, i, ii);
                            if (row < p.M)
                                *(float4 *)(p.out + (int64_t)row * p.ldc + col) =
                                    float4{sc * acc[i][0][v], sc * acc[i][1][v], sc * acc[i][2][v], sc * acc[i][3][v]};
                        }
                }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
            fc2_open(a, c.t + 1, c);
        }
        __syncthreads();
    }
}

// Second launch of a split-K run: workgroup (tile, slot) sums one of the tile's 32 accumulator slots (four
// columns per thread) over the splits, in split order, and writes the output with the item's own mapping.
__global__ __launch_bounds__(256) void fc2_reduce_kernel(FcPairArgs a, int tiles0)
{
    const int which = (int)(blockIdx.x >> 5) < tiles0 ? 0 : 1;
    const FcProblem &p = a.prob[which];
    const int tile = (int)(blockIdx.x >> 5) - (which ? tiles0 : 0), slot = blockIdx.x & 31;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile_m = (tile % p.tiles_m) * FC2_TM;
    const int tile_n = (tile / p.tiles_m) * FC2_TN;
    const float4 *all = (const float4 *)(p.partial + (int64_t)tile * p.n_split * (FC2_TM * FC2_TN)) + slot * 256 + tid;
    const int col = tile_n + 4 * (lane & 31);
    float4 sum = float4{0.f, 0.f, 0.f, 0.f};
    for (int q = 0; q < p.n_split; ++q) {
        const float4 t = all[(int64_t)q * (FC2_TM * FC2_TN / 4)];
        sum.x += t.x; sum.y += t.y; sum.z += t.z; sum.w += t.w;
    }
    const int i = slot >> 4, v = slot & 15;
    const int ii = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    const int row = fc2_row(p.a_kfast, tile_m, wave, i, ii);
    const float sc = p.scale.get();
    if (col < p.N && row < p.M)
        *(float4 *)(p.out + (int64_t)row * p.ldc + col) = float4{sc * sum.x, sc * sum.y, sc * sum.z, sc * sum.w};
}

}  // namespace dbp
