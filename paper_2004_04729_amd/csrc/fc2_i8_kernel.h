// Fully connected products of the full 8-bit mode: int8 codes x int8 weights / activations on int8 matrix
// cores, exact int32 results (Sec. "Quantizing forward pass": every product of the backward pass is an 8-bit
// computation).  Same organisation as fc2_kernel.h: 256x128 tiles, persistent workgroups with four
// multiplying and four staging wavefronts, work items decoded once into LDS, one barrier per K step.
// What differs:
//   * a K step is 64 reduction indices (two matrix-core instructions deep, 16 indices per 16-byte cell);
//   * nothing is converted: codes whose reduction index is contiguous are copied (16-byte loads, 16-byte LDS
//     writes); operands whose reduction index is the slow one are transposed in registers, 4x4 bytes at a
//     time (eight v_perm for sixteen bytes), and leave as dwords of four reduction indices;
//   * one plane per operand: 16 matrix-core instructions per step and wavefront instead of 48.
#pragma once
#include "fc2_kernel.h"

namespace dbp {

constexpr int FC2I_KT = 64;

struct Fc2IStage {
    uint4 a[NCHUNK][FC2_TM];          // [chunk of 16 reduction indices][row position]      16 KiB
    uint4 b[NCHUNK][FC2_TN];          // [chunk][column position]                            8 KiB
};
constexpr int FC2I_LDS_BYTES = 2 * (int)sizeof(Fc2IStage) + FC2_MAX_ITEMS * (int)sizeof(Fc2Item);

struct Fc2IRaw {                      // one K step of one stager thread, as loaded
    uint32_t a[16];
    uint2 b[4];
    int kfast, k_valid, a_shift;
};

// bytes j of four words -> word j (a 4x4 byte transposition): out[j] = {r0.byte j, r1.byte j, r2.byte j, r3.byte j}
__device__ __forceinline__ void fc2i_transpose(uint32_t r0, uint32_t r1, uint32_t r2, uint32_t r3, uint32_t (&out)[4])
{
    const uint32_t x0 = __builtin_amdgcn_perm(r1, r0, 0x05010400u), x1 = __builtin_amdgcn_perm(r3, r2, 0x05010400u);
    const uint32_t y0 = __builtin_amdgcn_perm(r1, r0, 0x07030602u), y1 = __builtin_amdgcn_perm(r3, r2, 0x07030602u);
    out[0] = __builtin_amdgcn_perm(x1, x0, 0x05040100u); out[1] = __builtin_amdgcn_perm(x1, x0, 0x07060302u);
    out[2] = __builtin_amdgcn_perm(y1, y0, 0x05040100u); out[3] = __builtin_amdgcn_perm(y1, y0, 0x07060302u);
}

// NT: the batched form with both operands reduction-contiguous, as in fc2_kernel.h (weight gradient of a 1x1
// convolution with int8 activations straight from the NCHW tensors); here the dense operand's cells are plain copies too.
template <bool NT>
__global__ __launch_bounds__(512, 1) void fc2_i8_pair_kernel(FcPairArgs a)
{
    extern __shared__ uint4 fc2_lds[];
    if (a.gate.closed()) return;
    Fc2IStage *stages = (Fc2IStage *)fc2_lds;
    Fc2Item *table = (Fc2Item *)(stages + 2);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int mine = fc2_items_of_workgroup(a, (int)gridDim.x, (int)blockIdx.x);
    for (int i = threadIdx.x; i < mine; i += 512) table[i] = fc2_decode(a, i, mine, (int)gridDim.x, (int)blockIdx.x);
    __syncthreads();
    int steps = 0;                                    // K steps of all items (the trip count of both roles)
    for (int i = 0; i < mine; ++i) steps += (table[i].k_end - table[i].k0 + FC2I_KT - 1) / FC2I_KT;
    const int G = __builtin_amdgcn_readfirstlane(steps);

    if (wave >= 4) {
        // ================================ stagers ================================
        const int tid = threadIdx.x & 255;
        // dense operand B[k][n] (int8): reduction rows 4*k4 .. +3, columns 8*n8 .. +7 (one 8-byte load per row)
        const int k4 = tid >> 4, n8 = tid & 15;
        Fc2Cursor c;
        // Addresses as in fc2_kernel.h: a base that is the same for all lanes and moves with the K step, plus
        // 32-bit lane offsets fixed for the item (edges clamped inside them); a step always loads a full
        // window of 64 reduction indices, the last window of an item ends at the item's end and what it repeats
        // is zeroed when the step is committed (K >= 64).
        const char *b_step = nullptr, *b_cur = nullptr;
        const int8_t *a_step = nullptr, *a_cur = nullptr;
        int64_t b_unit = 0, a_unit = 0;                   // bytes per reduction index
        uint32_t boff[4] = {0, 0, 0, 0}, aoff[4] = {0, 0, 0, 0};
        int a_shift = 0, kv_cur = 0;
        // NT: position inside the item's run of images (window s of image `nt_a`/`nt_b`) and the image strides
        int nt_s = 0, nt_pq = 0, nt_spi = 1;
        int64_t nt_a_img = 0, nt_b_img = 0;
        const int8_t *nt_a = nullptr;
        const char *nt_b = nullptr;
        auto open_item = [&](int i) {
            if (!fc2_open(a, table, mine, i, c)) return false;
            if constexpr (NT) {
                const FcProblem &p = a.prob[c.which];
                nt_pq = p.nt_pq; nt_spi = p.nt_spi; nt_a_img = p.nt_a_img; nt_b_img = p.nt_b_img;
                const int img = c.k0 / (nt_spi * FC2I_KT);                // items start and end at image borders
                nt_s = 0;
                nt_a = c.A + (int64_t)img * nt_a_img;
                nt_b = (const char *)c.B + (int64_t)img * nt_b_img;
                // dense operand: columns tid/4 and 64 + tid/4 of the tile, reduction indices 16*(tid%4) .. +15 of the window
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    boff[j] = (uint32_t)min(c.tile_n + 64 * j + (tid >> 2), c.N - 1) * (uint32_t)c.ldb + 16u * (uint32_t)(tid & 3);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    aoff[j] = (uint32_t)min(c.tile_m + 64 * j + (tid >> 2), c.M - 1) * (uint32_t)c.lda + 16u * (uint32_t)(tid & 3);
                a_shift = 0;
                return true;
            }
            const uint32_t ldb = (uint32_t)c.ldb, lda = (uint32_t)c.lda;
            b_unit = c.ldb;
            b_step = (const char *)c.B + (int64_t)c.k0 * b_unit;
            const uint32_t b0 = 4u * (uint32_t)k4 * ldb + (uint32_t)min(c.tile_n + 8 * n8, c.N - 8);
#pragma unroll
            for (int j = 0; j < 4; ++j) boff[j] = b0 + (uint32_t)j * ldb;
            if (c.a_kfast) {
                // rows tid/4 + 64*j of the tile, reduction indices 16*(tid%4) .. +15: four lanes take a 64-byte run
                a_unit = 1;
                a_step = c.A + c.k0;
                a_shift = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    aoff[j] = (uint32_t)min(c.tile_m + 64 * j + (tid >> 2), c.M - 1) * lda + 16u * (uint32_t)(tid & 3);
            } else {
                // reduction indices 4*k4 .. +3 and 16 consecutive rows of the matrix each (M >= 16, M % 4 == 0); a run
                // that would pass the last row starts earlier and is moved back when the step is committed
                a_unit = c.lda;
                a_step = c.A + (int64_t)c.k0 * c.lda;
                const int m = c.tile_m + 16 * (tid & 15);
                a_shift = max(0, m + 16 - c.M) >> 2;
                const uint32_t a0 = 4u * (uint32_t)k4 * lda + (uint32_t)max(0, min(m, c.M - 16));
#pragma unroll
                for (int j = 0; j < 4; ++j) aoff[j] = a0 + (uint32_t)j * lda;
            }
            return true;
        };
        bool open = open_item(0);

        // Every call issues the same eight loads (also once the list is exhausted: the last window again, never
        // committed), so the compiler can wait for exactly the loads of three calls ago.
        auto issue = [&](Fc2IRaw &r) {
            if constexpr (NT) {
                if (open) {
                    // window s of the image: 64 reduction indices that end inside the image (the last window overlaps
                    // the one before it; what it repeats is zeroed when the step is committed)
                    const int win = min(FC2I_KT * nt_s, nt_pq - FC2I_KT);
                    kv_cur = min(FC2I_KT, nt_pq - FC2I_KT * nt_s);
                    b_cur = nt_b + win;
                    a_cur = nt_a + win;
                }
            } else
            if (open) {
                kv_cur = c.k_end - c.k0;
                const int back = max(0, FC2I_KT - kv_cur);
                b_cur = b_step - back * b_unit;
                a_cur = a_step - back * a_unit;
            }
            r.kfast = NT ? 1 : c.a_kfast;
            r.k_valid = kv_cur;
            r.a_shift = a_shift;
            if constexpr (NT) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const u32x4 v = *(const u32x4_dw *)(b_cur + (size_t)boff[i]);
                    r.b[2 * i] = uint2{v.x, v.y}; r.b[2 * i + 1] = uint2{v.z, v.w};
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) r.b[i] = *(const uint2 *)(b_cur + (size_t)boff[i]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const u32x4 v = *(const u32x4_dw *)(a_cur + (size_t)aoff[i]);
                r.a[4 * i] = v.x; r.a[4 * i + 1] = v.y; r.a[4 * i + 2] = v.z; r.a[4 * i + 3] = v.w;
            }
            if (open) {
                c.k0 += FC2I_KT;
                if constexpr (NT) {
                    if (++nt_s == nt_spi) { nt_s = 0; nt_a += nt_a_img; nt_b += nt_b_img; }
                } else {
                    b_step += FC2I_KT * b_unit; a_step += FC2I_KT * a_unit;
                }
                if (c.k0 >= c.k_end) open = open_item(c.t + 1);
            }
        };

        auto unshift = [](uint32_t (&w)[4], int sh) {
            const uint32_t t0 = w[0], t1 = w[1], t2 = w[2], t3 = w[3];
            w[0] = sh == 0 ? t0 : sh == 1 ? t1 : sh == 2 ? t2 : sh == 3 ? t3 : 0u;
            w[1] = sh == 0 ? t1 : sh == 1 ? t2 : sh == 2 ? t3 : 0u;
            w[2] = sh == 0 ? t2 : sh == 1 ? t3 : 0u;
            w[3] = sh == 0 ? t3 : 0u;
        };

        auto commit = [&](const Fc2IRaw &r, Fc2IStage &sm) {
            // window indices below `dup` repeat the step before (only in an item's last, shorter step)
            const int dup = FC2I_KT - r.k_valid;
            if (r.kfast) {
                // set i = the cell of chunk tid%4 of row position tid/4 + 64*i (the item's ends are multiples of 4:
                // whole dwords are in or out)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint32_t w[4] = {r.a[4 * i], r.a[4 * i + 1], r.a[4 * i + 2], r.a[4 * i + 3]};
                    if (dup > 0) {
#pragma unroll
                        for (int d = 0; d < 4; ++d) w[d] = 16 * (tid & 3) + 4 * d >= dup ? w[d] : 0u;
                    }
                    sm.a[tid & 3][64 * i + (tid >> 2)] = uint4{w[0], w[1], w[2], w[3]};
                }
            } else {
                // set i = reduction index 4*k4 + i; byte j of dword d = matrix row 16*(tid%16) + 4*d + j of the tile
                // -> position 16*(4*d + j) + tid%16, dword k4%4 of the cell of chunk k4/4
                const int m16 = tid & 15;
                uint32_t w[4][4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
#pragma unroll
                    for (int d = 0; d < 4; ++d) w[i][d] = r.a[4 * i + d];
                    if (r.a_shift) unshift(w[i], r.a_shift);
                    if (dup > 0 && 4 * k4 + i < dup) { w[i][0] = w[i][1] = w[i][2] = w[i][3] = 0u; }
                }
                uint32_t *cell = (uint32_t *)&sm.a[k4 >> 2][m16] + (k4 & 3);
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    uint32_t t[4];
                    fc2i_transpose(w[0][d], w[1][d], w[2][d], w[3][d], t);
#pragma unroll
                    for (int j = 0; j < 4; ++j) cell[64 * (4 * d + j)] = t[j];
                }
            }
            if constexpr (NT) {
                // set i = the cell of chunk tid%4 of column n = tid/4 + 64*i -> position 32*(n%4) + n/4
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    uint32_t w[4] = {r.b[2 * i].x, r.b[2 * i].y, r.b[2 * i + 1].x, r.b[2 * i + 1].y};
                    if (dup > 0) {
#pragma unroll
                        for (int d = 0; d < 4; ++d) w[d] = 16 * (tid & 3) + 4 * d >= dup ? w[d] : 0u;
                    }
                    const int n = 64 * i + (tid >> 2);
                    sm.b[tid & 3][32 * (n & 3) + (n >> 2)] = uint4{w[0], w[1], w[2], w[3]};
                }
                return;
            }
            // dense operand: column 8*n8 + e -> position 32*(e%4) + 2*n8 + e/4 (a multiplier lane then holds four
            // adjacent columns), dword k4%4 of the cell of chunk k4/4
            uint32_t bx[4], by[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool keep = !(dup > 0 && 4 * k4 + i < dup);
                bx[i] = keep ? r.b[i].x : 0u; by[i] = keep ? r.b[i].y : 0u;
            }
            uint32_t tx[4], ty[4];
            fc2i_transpose(bx[0], bx[1], bx[2], bx[3], tx);
            fc2i_transpose(by[0], by[1], by[2], by[3], ty);
            uint32_t *bcell = (uint32_t *)&sm.b[k4 >> 2][2 * n8] + (k4 & 3);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bcell[4 * (32 * j)] = tx[j];          // e = j
                bcell[4 * (32 * j + 1)] = ty[j];      // e = 4 + j
            }
        };

        if (G == 0) { __syncthreads(); if (wave == 7) fc2_side_jobs(a.stats, lane); return; }
        Fc2IRaw r0, r1, r2;
        issue(r0); issue(r1); issue(r2);
        commit(r0, stages[0]);
        issue(r0);
        __syncthreads();
        for (int g = 0; g < G; g += 3) {
            if (g + 1 < G) commit(r1, stages[(g + 1) & 1]);
            issue(r1);
            __syncthreads();
            if (g + 2 < G) commit(r2, stages[(g + 2) & 1]);
            issue(r2);
            if (g + 1 < G) __syncthreads();
            if (g + 3 < G) commit(r0, stages[(g + 3) & 1]);
            issue(r0);
            if (g + 2 < G) __syncthreads();
        }
        if (wave == 7) fc2_side_jobs(a.stats, lane);     // the statistics and the bias gradient, once the staging is over
        return;
    }

    // ================================ multipliers ================================
    const int tid = threadIdx.x;
    const int lcol = lane & 31, lhalf = lane >> 5;
    i32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    Fc2Cursor c;
    fc2_open(a, table, mine, 0, c);

    __syncthreads();
    for (int g = 0; g < G; ++g) {
        const Fc2IStage &sm = stages[g & 1];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int ch = 2 * kk + lhalf;
            u32x4 af[2], bf[4];
#pragma unroll
            for (int i = 0; i < 2; ++i) { const uint4 t = sm.a[ch][wave * 64 + i * 32 + lcol]; af[i] = u32x4{t.x, t.y, t.z, t.w}; }
#pragma unroll
            for (int j = 0; j < 4; ++j) { const uint4 t = sm.b[ch][j * 32 + lcol]; bf[j] = u32x4{t.x, t.y, t.z, t.w}; }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) Mma<MODE_I8>::run(af[i], bf[j], acc[i][j]);
        }
        c.k0 += FC2I_KT;
        if (c.k0 >= c.k_end) {
            const Fc2Cursor p = c;
            typedef int32_t i32v4 __attribute__((ext_vector_type(4)));
            if (p.n_split > 1) {
                i32v4 *mine_p = (i32v4 *)((int32_t *)p.partial + ((int64_t)c.tile * p.n_split + c.z) * (FC2_TM * FC2_TN));
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        mine_p[(i * 16 + v) * 256 + tid] = i32v4{acc[i][0][v], acc[i][1][v], acc[i][2][v], acc[i][3][v]};
            } else {
                const int col = c.tile_n + 4 * lcol;
                if (col < p.N) {
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int ii = 8 * (v >> 2) + 4 * lhalf + (v & 3);
                            const int row = fc2_row(p.a_kfast, c.tile_m, wave, i, ii);
                            if (row < p.M)
                                __builtin_nontemporal_store(i32v4{acc[i][0][v], acc[i][1][v], acc[i][2][v], acc[i][3][v]},
                                                            (i32v4 *)((int32_t *)p.out + (int64_t)row * p.ldc + col));
                        }
                }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
            fc2_open(a, table, mine, c.t + 1, c);
        }
        __syncthreads();
    }
}

// Split-K sums of the int8 kernel (integers: exact in any order; the order is fixed all the same).
__global__ __launch_bounds__(256) void fc2_i8_reduce_kernel(FcPairArgs a, int tiles0)
{
    if (a.gate.closed()) return;
    typedef int32_t i32v4 __attribute__((ext_vector_type(4)));
    const int which = (int)(blockIdx.x >> 5) < tiles0 ? 0 : 1;
    const FcProblem &p = a.prob[which];
    const int tile = (int)(blockIdx.x >> 5) - (which ? tiles0 : 0), slot = blockIdx.x & 31;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile_m = (tile % p.tiles_m) * FC2_TM;
    const int tile_n = (tile / p.tiles_m) * FC2_TN;
    const i32v4 *all = (const i32v4 *)((const int32_t *)p.partial + (int64_t)tile * p.n_split * (FC2_TM * FC2_TN)) + slot * 256 + tid;
    const int col = tile_n + 4 * (lane & 31);
    i32v4 sum = i32v4{0, 0, 0, 0};
    const int n_split = p.n_split;
    for (int q = 0; q < n_split; q += 8) {
        i32v4 t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = all[(int64_t)min(q + j, n_split - 1) * (FC2_TM * FC2_TN / 4)];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (q + j < n_split) sum += t[j];
    }
    const int i = slot >> 4, v = slot & 15;
    const int ii = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    const int row = fc2_row(p.a_kfast, tile_m, wave, i, ii);
    if (col < p.N && row < p.M) *(i32v4 *)((int32_t *)p.out + (int64_t)row * p.ldc + col) = sum;
}

}  // namespace dbp
