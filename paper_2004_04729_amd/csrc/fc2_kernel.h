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
constexpr int FC2_SETS = 3;                        // register sets of loads in flight per staging wavefront (K steps ahead; 4 .. 8 measured: no gain)
constexpr int FC2_MAX_ITEMS = 128;                 // work items of one workgroup (the host checks)
constexpr int FC2_LDS_BYTES = 2 * (16 + 24) * 1024 + FC2_MAX_ITEMS * 32;

struct Fc2Stage {
    uint2 a[NCHUNK][FC2_TM][2];       // [chunk][row position][half]          16 KiB
    uint2 b[3][NCHUNK][FC2_TN][2];    // [plane][chunk][col position][half]   24 KiB
};
// A decoded work item as the workgroup keeps it in LDS (after the two stages).
struct Fc2Item { int which, tile, z, tile_m, tile_n, k0, k_end, pad; };
static_assert(sizeof(Fc2Stage) * 2 + FC2_MAX_ITEMS * sizeof(Fc2Item) == FC2_LDS_BYTES, "two stages and the item table");

// Position of a workgroup in its sequence of (item, K step) pairs; both roles walk the same sequence.
struct Fc2Cursor {
    int t;                            // position in this workgroup's list of items
    int which, tile, z, tile_m, tile_n, k0, k_end;
    // the item's problem, copied once per item (indexing the kernel arguments by `which` at every use costs a
    // scalar load, and its latency, each time)
    const int8_t *A; const float *B; float *out, *partial;
    int64_t lda, ldb, ldc;
    int M, N, K, n_split, a_kfast;
};

// The i-th work item of this workgroup.  Items are numbered with those of problem 0 first (the longer
// ones in a backward pass: dX keeps the whole reduction of a layer) and dealt in a serpentine over the
// workgroups (pass p gives workgroup w item p*G + w, the next pass p*G + G-1-w), which balances the number
// of K steps; every workgroup then starts at a different place of its own list (rotation by w), so that
// the tiles of the chip are not all finished, and stored, at the same moment.
// With a.gx > 0 the workgroups are two groups instead, one per problem: a split product then needs fewer, longer items
// (fewer partial tiles to write and to sum) for the same balance.
// (G workgroups in the launch, w = this one: parameters, so that a host-side check can walk the same arithmetic.)
__host__ __device__ __forceinline__ int fc2_items_of_workgroup(const FcPairArgs &a, int G, int w)
{
    if (a.gx > 0) {
        const bool first = w < a.gx;
        const int n = first ? a.prob[0].n_items : a.prob[1].n_items;
        const int wi = first ? w : w - a.gx, gp = first ? a.gx : G - a.gx;
        return n > wi ? (n - wi + gp - 1) / gp : 0;
    }
    const int total = a.prob[0].n_items + a.prob[1].n_items;
    const int passes = (total + G - 1) / G;
    const int last = (passes - 1) * G + (((passes - 1) & 1) ? G - 1 - w : w);
    return last < total ? passes : passes - 1;
}

__host__ __device__ __forceinline__ Fc2Item fc2_decode(const FcPairArgs &a, int i, int mine, int G, int w)
{
    const int n0 = a.prob[0].n_items;
    const int ps = (i + w) % mine;
    Fc2Item c;
    int t, item;
    if (a.gx > 0) {
        const bool first = w < a.gx;
        c.which = first ? 0 : 1;
        item = ps * (first ? a.gx : G - a.gx) + (first ? w : w - a.gx);
        t = -1;
    } else {
        t = ps * G + ((ps & 1) ? G - 1 - w : w);
        c.which = t < n0 ? 0 : 1;
        item = t < n0 ? t : t - n0;
    }
    const FcProblem &p = a.prob[c.which];
    c.tile = item / p.n_split; c.z = item - c.tile * p.n_split;
    // Workgroup w runs on XCD w % 8, and each XCD has an L2 of its own.  Where the counts divide evenly the items
    // are renumbered so that one XCD keeps to one share of the re-read operand: the same reduction slice of
    // the codes for a split product, the same column tiles of the dense operand otherwise.
    if (t >= 0 && (G & 7) == 0 && (n0 & 7) == 0 && (p.n_items & 7) == 0) {
        const int x = ((t / G) & 1) ? 7 - (t & 7) : (t & 7), r = item >> 3;
        const int tiles_n = p.n_items / (p.n_split * p.tiles_m);
        if (p.n_split > 1 && (p.n_split & 7) == 0) {
            const int ns8 = p.n_split >> 3;
            c.tile = r / ns8; c.z = x * ns8 + (r - c.tile * ns8);
        } else if (p.n_split == 1 && (tiles_n & 7) == 0) {
            const int tn8 = tiles_n >> 3, tm = r / tn8;
            c.tile = (x * tn8 + (r - tm * tn8)) * p.tiles_m + tm;
        }
    }
    c.tile_m = (c.tile % p.tiles_m) * FC2_TM;
    c.tile_n = (c.tile / p.tiles_m) * FC2_TN;
    c.k0 = c.z * p.k_per_split;
    c.k_end = p.K < c.k0 + p.k_per_split ? p.K : c.k0 + p.k_per_split;
    c.pad = 0;
    return c;
}

// Makes item i of the workgroup's table the cursor's item (false past the end).  The table is decoded once per
// workgroup, by all threads in parallel: decoding in the K loop costs the roles, which are single wavefronts
// per SIMD and bound by the number of instructions they issue, about as much as a whole step's loads.
__device__ __forceinline__ bool fc2_open(const FcPairArgs &a, const Fc2Item *table, int mine, int i, Fc2Cursor &c)
{
    if (i >= mine) return false;
    const int4 lo = *(const int4 *)&table[i], hi = *((const int4 *)&table[i] + 1);
    c.t = i;
    c.which = __builtin_amdgcn_readfirstlane(lo.x); c.tile = __builtin_amdgcn_readfirstlane(lo.y);
    c.z = __builtin_amdgcn_readfirstlane(lo.z); c.tile_m = __builtin_amdgcn_readfirstlane(lo.w);
    c.tile_n = __builtin_amdgcn_readfirstlane(hi.x); c.k0 = __builtin_amdgcn_readfirstlane(hi.y);
    c.k_end = __builtin_amdgcn_readfirstlane(hi.z);
    const FcProblem &p = a.prob[c.which];
    c.A = p.A; c.B = p.B; c.out = p.out; c.partial = p.partial;
    c.lda = p.lda; c.ldb = p.ldb; c.ldc = p.ldc;
    c.M = p.M; c.N = p.N; c.K = p.K; c.n_split = p.n_split; c.a_kfast = p.a_kfast;
    return true;
}

struct Fc2Raw {                       // one K step of one stager thread, as loaded
    f32x4 b[4];
    uint32_t a[8];
    int kfast, k_valid;               // operand layout of the item; reduction indices of the step that exist
    int a_shift;                      // !kfast: dwords by which the loaded run of rows was moved back to stay inside the matrix
};

// 16 bytes from an address that is only known to be a multiple of 4 (one global_load_dwordx4)
typedef uint32_t u32x4_dw __attribute__((ext_vector_type(4), aligned(4)));

// Sum of the quantiser's statistics records by one wavefront (integers: any order gives the same result); four
// loads in flight per lane.
__device__ __forceinline__ void fc2_sum_stats(const StatsJob &j, int lane)
{
    uint64_t nnz = 0, sat = 0, nf = 0, mx = 0;
    for (int i = lane; i < j.n; i += 256) {
        u32x4 q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) q[u] = j.partials[min(i + 64 * u, j.n - 1)];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + 64 * u < j.n) { nnz += q[u].x; sat += q[u].y; nf += q[u].z; mx = mx > q[u].w ? mx : q[u].w; }
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

// Bias gradient of the layer from the quantiser's code sums: one fp64 product rounded to fp32 per element.  Every
// workgroup's wavefront takes every gridDim.x-th run of 64 elements.
__device__ __forceinline__ void fc2_bias_grad(const StatsJob &j, int lane)
{
    const double d = j.step_dev ? (double)j.step_dev[0] : (double)j.step;
    for (int64_t i = (int64_t)blockIdx.x * 64 + lane; i < j.bias_len; i += (int64_t)gridDim.x * 64)
        j.bias_grad[i] = (float)(d * (double)j.bias_sums[i]);
}

// What a stager wavefront does once its staging is over, while the multipliers finish the last steps and store: the last
// workgroup (it has the fewest items) sums the quantiser's statistics, every workgroup takes its share of the bias gradient.
// (Done in front of the staging loop by one wavefront, the two cost the kernel 20 us: that workgroup started late.)
__device__ __forceinline__ void fc2_side_jobs(const StatsJob &j, int lane)
{
    if (j.n > 0 && blockIdx.x == gridDim.x - 1) fc2_sum_stats(j, lane);
    if (j.bias_len > 0) fc2_bias_grad(j, lane);
}

// Matrix row of element ii of row block i of multiplier wavefront `wave`: row positions are rows (a_kfast)
// or the transposition position 16*(row % 16) + row / 16 of the staging (a stager lane holds 16 consecutive
// rows; with this order the 64 lanes of one LDS write fall into 64 different banks).
__device__ __forceinline__ int fc2_row(int a_kfast, int tile_m, int wave, int i, int ii)
{
    return a_kfast ? tile_m + wave * 64 + i * 32 + ii
                   : tile_m + 16 * (ii & 15) + 4 * wave + 2 * i + (ii >> 4);
}

// NT: the batched form with both operands reduction-contiguous (the weight gradient of a 1x1 convolution straight from
// NCHW tensors: rows = output channels, columns = input channels, reduction = the pixels of every image).  Only the
// stagers' addresses and the order in which they read the dense operand's registers differ.
// PL: bf16 planes of the fp32 operand, 3 (exact) or 2 (rounded to nearest, 16 significant bits).
template <bool NT, int PL = 3>
__global__ __launch_bounds__(512, 1) void fc2_pair_kernel(FcPairArgs a)
{
    extern __shared__ uint4 fc2_lds[];
    if (a.gate.closed()) return;
    Fc2Stage *stages = (Fc2Stage *)fc2_lds;
    Fc2Item *table = (Fc2Item *)(stages + 2);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int mine = fc2_items_of_workgroup(a, (int)gridDim.x, (int)blockIdx.x);
    for (int i = threadIdx.x; i < mine; i += 512) table[i] = fc2_decode(a, i, mine, (int)gridDim.x, (int)blockIdx.x);
    __syncthreads();
    int steps = 0;                                    // K steps of all items (the trip count of both roles)
    for (int i = 0; i < mine; ++i) steps += (table[i].k_end - table[i].k0 + FC2_KT - 1) / FC2_KT;
    const int G = __builtin_amdgcn_readfirstlane(steps);

    if (wave >= 4) {
        // ================================ stagers ================================
        const int tid = threadIdx.x & 255;
        // lane pairs share four columns of the dense operand and take neighbouring groups of four reduction
        // indices: their 8-byte LDS writes are then contiguous over the wavefront
        const int nq = (tid >> 1) & 31, kq = 2 * (tid >> 6) + (tid & 1);
        Fc2Cursor c;
        // Addresses: a base that is the same for all lanes and moves with the K step (scalar additions), plus a
        // 32-bit lane offset that is fixed for the item (the matrices are smaller than 4 GiB here).  Rows and
        // columns past the edge of a matrix are clamped once per item, inside the lane offsets.  A step always
        // loads a full window of 32 reduction indices: the last window of an item whose length is not a
        // multiple of 32 ends at the item's end and overlaps the window before it; the indices it repeats are
        // zeroed when the step is committed (K >= 32, so the window never leaves the row or column).
        const char *b_step = nullptr, *b_cur = nullptr;
        const int8_t *a_step = nullptr, *a_cur = nullptr;
        int64_t b_unit = 0, a_unit = 0;                   // bytes per reduction index
        uint32_t boff[4] = {0, 0, 0, 0}, aoff[2] = {0, 0};
        int a_shift = 0, kv_cur = 0;
        // NT: position inside the item's run of images (window s of image `nt_img`) and the image's operands
        int nt_s = 0, nt_pq = 0, nt_spi = 1;
        int64_t nt_a_img = 0, nt_b_img4 = 0;
        const int8_t *nt_a = nullptr;
        const char *nt_b = nullptr;
        auto open_item = [&](int i) {
            if (!fc2_open(a, table, mine, i, c)) return false;
            if constexpr (NT) {
                const FcProblem &p = a.prob[c.which];
                nt_pq = p.nt_pq; nt_spi = p.nt_spi; nt_a_img = p.nt_a_img; nt_b_img4 = p.nt_b_img * 4;
                const int img = c.k0 / (nt_spi * FC2_KT);                 // items start and end at image borders
                nt_s = 0;
                nt_a = c.A + (int64_t)img * nt_a_img;
                nt_b = (const char *)c.B + (int64_t)img * nt_b_img4;
                // dense operand: columns 4*nq .. +3 of the tile (one per load), reduction indices 4*kq .. +3 of the window
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    boff[j] = (uint32_t)min(c.tile_n + 4 * nq + j, c.N - 1) * (uint32_t)c.ldb * 4u + 16u * (uint32_t)kq;
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    aoff[j] = (uint32_t)min(c.tile_m + 128 * j + (tid >> 1), c.M - 1) * (uint32_t)c.lda + 16u * (uint32_t)(tid & 1);
                a_shift = 0;
                return true;
            }
            const uint32_t ldb4 = (uint32_t)c.ldb * 4u, lda = (uint32_t)c.lda;
            b_unit = (int64_t)c.ldb * 4;
            b_step = (const char *)c.B + (int64_t)c.k0 * b_unit;
            const uint32_t b0 = 4u * (uint32_t)kq * ldb4 + 4u * (uint32_t)min(c.tile_n + 4 * nq, c.N - 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) boff[j] = b0 + (uint32_t)j * ldb4;
            if (c.a_kfast) {
                // rows tid/2 and 128 + tid/2 of the tile, 16 consecutive reduction indices each (a pair of lanes
                // takes a 32-byte run of a row)
                a_unit = 1;
                a_step = c.A + c.k0;
                a_shift = 0;
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    aoff[j] = (uint32_t)min(c.tile_m + 128 * j + (tid >> 1), c.M - 1) * lda + 16u * (uint32_t)(tid & 1);
            } else {
                // reduction indices 2*(tid/16), +1 and 16 consecutive rows of the matrix each (M >= 16, M % 4 == 0);
                // a run that would pass the last row starts earlier and is moved back when the step is committed
                a_unit = c.lda;
                a_step = c.A + (int64_t)c.k0 * c.lda;
                const int m = c.tile_m + 16 * (tid & 15);
                a_shift = max(0, m + 16 - c.M) >> 2;
                aoff[0] = 2u * (uint32_t)(tid >> 4) * lda + (uint32_t)max(0, min(m, c.M - 16));
                aoff[1] = aoff[0] + lda;
            }
            return true;
        };
        bool open = open_item(0);

        // Loads of the cursor's K step; then the cursor moves on (to the next item after an item's last step).
        // Every call issues the same six 16-byte loads, also once the list is exhausted (the last window again;
        // it is never committed): with equal load counts on every path the compiler can wait for exactly the
        // loads of three calls ago instead of for all outstanding ones.
        auto issue = [&](Fc2Raw &r) {
            if constexpr (NT) {
                if (open) {
                    // window s of the image: 32 reduction indices that end inside the image (the last window overlaps the
                    // one before it; what it repeats is zeroed when the step is committed)
                    const int win = min(FC2_KT * nt_s, nt_pq - FC2_KT);
                    kv_cur = min(FC2_KT, nt_pq - FC2_KT * nt_s);
                    b_cur = nt_b + (int64_t)win * 4;
                    a_cur = nt_a + win;
                }
            } else
            if (open) {
                kv_cur = c.k_end - c.k0;
                const int back = max(0, FC2_KT - kv_cur);
                b_cur = b_step - back * b_unit;
                a_cur = a_step - back * a_unit;
            }
            r.kfast = NT ? 1 : c.a_kfast;
            r.k_valid = kv_cur;
            r.a_shift = a_shift;
#pragma unroll
            for (int i = 0; i < 4; ++i) r.b[i] = *(const f32x4 *)(b_cur + (size_t)boff[i]);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const u32x4 v = *(const u32x4_dw *)(a_cur + (size_t)aoff[i]);
                r.a[4 * i] = v.x; r.a[4 * i + 1] = v.y; r.a[4 * i + 2] = v.z; r.a[4 * i + 3] = v.w;
            }
            if (open) {
                c.k0 += FC2_KT;
                if constexpr (NT) {
                    if (++nt_s == nt_spi) { nt_s = 0; nt_a += nt_a_img; nt_b += nt_b_img4; }
                } else {
                    b_step += FC2_KT * b_unit; a_step += FC2_KT * a_unit;
                }
                if (c.k0 >= c.k_end) open = open_item(c.t + 1);
            }
        };

        // dwords of a 16-byte run moved back by `sh` dwords (what lies past the last row is zero)
        auto unshift = [](uint32_t (&w)[4], int sh) {
            const uint32_t t0 = w[0], t1 = w[1], t2 = w[2], t3 = w[3];
            w[0] = sh == 0 ? t0 : sh == 1 ? t1 : sh == 2 ? t2 : sh == 3 ? t3 : 0u;
            w[1] = sh == 0 ? t1 : sh == 1 ? t2 : sh == 2 ? t3 : 0u;
            w[2] = sh == 0 ? t2 : sh == 1 ? t3 : 0u;
            w[3] = sh == 0 ? t3 : 0u;
        };

        auto commit = [&](const Fc2Raw &r, Fc2Stage &sm) {
            // window indices below `dup` repeat the step before (only in an item's last, shorter step)
            const int dup = FC2_KT - r.k_valid;
            if (r.kfast) {
                // dwords 0..3 of set i = chunks 2q, 2q+1 (q = tid & 1) of row position 128*i + tid/2
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    uint32_t w[4] = {r.a[4 * i], r.a[4 * i + 1], r.a[4 * i + 2], r.a[4 * i + 3]};
                    if (dup > 0) {
                        // the item's ends are multiples of 4, so whole dwords are in or out
#pragma unroll
                        for (int d = 0; d < 4; ++d) w[d] = 16 * (tid & 1) + 4 * d >= dup ? w[d] : 0u;
                    }
                    const int pos = 128 * i + (tid >> 1);
#pragma unroll
                    for (int e = 0; e < 2; ++e)
                        *(u32x4 *)&sm.a[2 * (tid & 1) + e][pos][0] =
                            u32x4{bf16x2_from_codes((int8_t)w[2 * e], (int8_t)(w[2 * e] >> 8)),
                                  bf16x2_from_codes((int8_t)(w[2 * e] >> 16), (int8_t)(w[2 * e] >> 24)),
                                  bf16x2_from_codes((int8_t)w[2 * e + 1], (int8_t)(w[2 * e + 1] >> 8)),
                                  bf16x2_from_codes((int8_t)(w[2 * e + 1] >> 16), (int8_t)(w[2 * e + 1] >> 24))};
                }
            } else {
                // set i = reduction index 2*k2 + i (k2 = tid/16); byte j of dword d = matrix row 16*(tid&15) + 4*d + j
                // of the tile -> position 16*(4*d + j) + tid%16, dword k2%4 of the cell of chunk k2/4
                const int k2 = tid >> 4, m16 = tid & 15;
                uint32_t w0[4] = {r.a[0], r.a[1], r.a[2], r.a[3]}, w1[4] = {r.a[4], r.a[5], r.a[6], r.a[7]};
                if (r.a_shift) { unshift(w0, r.a_shift); unshift(w1, r.a_shift); }
                if (dup > 0) {
#pragma unroll
                    for (int d = 0; d < 4; ++d) { w0[d] = 2 * k2 >= dup ? w0[d] : 0u; w1[d] = 2 * k2 + 1 >= dup ? w1[d] : 0u; }
                }
                uint32_t *cell = (uint32_t *)&sm.a[k2 >> 2][m16][0] + (k2 & 3);
#pragma unroll
                for (int d = 0; d < 4; ++d)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        cell[64 * (4 * d + j)] = bf16x2_from_codes((int8_t)(w0[d] >> (8 * j)), (int8_t)(w1[d] >> (8 * j)));
            }
            // fp32 -> three exact bf16 planes (or two rounded ones); column 4*nq+j -> position j*32+nq
            // (NT: register i holds column 4*nq+i, its component j reduction index 4*kq+j -- the transposed arrangement)
            f32x4 bv[4] = {r.b[0], r.b[1], r.b[2], r.b[3]};
            if (dup > 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (4 * kq + i < dup) {
                        if constexpr (NT) { bv[0][i] = 0.f; bv[1][i] = 0.f; bv[2][i] = 0.f; bv[3][i] = 0.f; }
                        else bv[i] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int pos = j * 32 + nq;
                if constexpr (PL == 3) {
                    uint32_t h[4], m[4], l[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) split3_upper(NT ? bv[j][i] : bv[i][j], h[i], m[i], l[i]);
                    sm.b[0][kq >> 1][pos][kq & 1] = uint2{upper_halves(l[1], l[0]), upper_halves(l[3], l[2])};
                    sm.b[1][kq >> 1][pos][kq & 1] = uint2{upper_halves(m[1], m[0]), upper_halves(m[3], m[2])};
                    sm.b[2][kq >> 1][pos][kq & 1] = uint2{upper_halves(h[1], h[0]), upper_halves(h[3], h[2])};
                } else {
                    uint32_t h[2], l[2];
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        split2_pk(NT ? bv[j][2 * i] : bv[2 * i][j], NT ? bv[j][2 * i + 1] : bv[2 * i + 1][j], h[i], l[i]);
                    sm.b[0][kq >> 1][pos][kq & 1] = uint2{l[0], l[1]};
                    sm.b[1][kq >> 1][pos][kq & 1] = uint2{h[0], h[1]};
                }
            }
        };

        // Step g lives in register set g % FC2_SETS and LDS stage g % 2.  Barriers: one after step 0 is staged, then
        // one per step; in the iteration of step g the stagers write step g + 1 and load step g + 1 + FC2_SETS.
        // The loads are unconditional (see issue); only commits and barriers depend on the trip count.
        if (G == 0) { __syncthreads(); if (wave == 7) fc2_side_jobs(a.stats, lane); return; }
        Fc2Raw r[FC2_SETS];
#pragma unroll
        for (int j = 0; j < FC2_SETS; ++j) issue(r[j]);
        commit(r[0], stages[0]);
        issue(r[0]);
        __syncthreads();
        for (int g = 0; g < G; g += FC2_SETS) {
#pragma unroll
            for (int j = 1; j <= FC2_SETS; ++j) {                // step g + j: from set j % SETS into stage (g + j) & 1
                if (g + j < G) commit(r[j % FC2_SETS], stages[(g + j) & 1]);
                issue(r[j % FC2_SETS]);
                if (g + j - 1 < G) __syncthreads();
            }
        }
        if (wave == 7) fc2_side_jobs(a.stats, lane);
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
    fc2_open(a, table, mine, 0, c);
    const float scale0 = a.prob[0].scale.get(), scale1 = a.prob[1].scale.get();   // resolved once (host value or device Delta)

    __syncthreads();
    for (int g = 0; g < G; ++g) {
        const Fc2Stage &sm = stages[g & 1];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int ch = 2 * kk + lhalf;
            u32x4 af[2], bf[PL][4];
#pragma unroll
            for (int i = 0; i < 2; ++i) af[i] = *(const u32x4 *)&sm.a[ch][wave * 64 + i * 32 + lcol][0];
#pragma unroll
            for (int pl = 0; pl < PL; ++pl)
#pragma unroll
                for (int j = 0; j < 4; ++j) bf[pl][j] = *(const u32x4 *)&sm.b[pl][ch][j * 32 + lcol][0];
            // planes outermost: consecutive instructions accumulate into different blocks
#pragma unroll
            for (int pl = 0; pl < PL; ++pl)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) Mma<MODE_BF16>::run(af[i], bf[pl][j], acc[i][j]);
        }
        c.k0 += FC2_KT;
        if (c.k0 >= c.k_end) {
            // ---- the item is complete: store (the stagers are already loading the next one) ----
            const Fc2Cursor p = c;
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
                                // written once and read by nobody in this launch: streaming stores (the MLP step 124 -> 120 us; the partial tiles
                                // above, which the reduction reads right away, lose 4 us with them)
                                __builtin_nontemporal_store(f32x4{sc * acc[i][0][v], sc * acc[i][1][v], sc * acc[i][2][v], sc * acc[i][3][v]},
                                                            (f32x4 *)(p.out + (int64_t)row * p.ldc + col));
                        }
                }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
            fc2_open(a, table, mine, c.t + 1, c);
        }
        __syncthreads();
    }
}

// Second launch of a split-K run: workgroup (tile, slot) sums one of the tile's 32 accumulator slots (four
// columns per thread) over the splits, in split order, and writes the output with the item's own mapping.
__global__ __launch_bounds__(256) void fc2_reduce_kernel(FcPairArgs a, int tiles0)
{
    if (a.gate.closed()) return;
    const int which = (int)(blockIdx.x >> 5) < tiles0 ? 0 : 1;
    const FcProblem &p = a.prob[which];
    const int tile = (int)(blockIdx.x >> 5) - (which ? tiles0 : 0), slot = blockIdx.x & 31;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile_m = (tile % p.tiles_m) * FC2_TM;
    const int tile_n = (tile / p.tiles_m) * FC2_TN;
    const float4 *all = (const float4 *)(p.partial + (int64_t)tile * p.n_split * (FC2_TM * FC2_TN)) + slot * 256 + tid;
    const int col = tile_n + 4 * (lane & 31);
    float4 sum = float4{0.f, 0.f, 0.f, 0.f};
    // eight loads in flight at a time (the loop is bound by their latency); the additions stay in split order
    const int n_split = p.n_split;
    for (int q = 0; q < n_split; q += 8) {
        float4 t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = all[(int64_t)min(q + j, n_split - 1) * (FC2_TM * FC2_TN / 4)];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (q + j < n_split) { sum.x += t[j].x; sum.y += t[j].y; sum.z += t[j].z; sum.w += t[j].w; }
    }
    const int i = slot >> 4, v = slot & 15;
    const int ii = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    const int row = fc2_row(p.a_kfast, tile_m, wave, i, ii);
    const float sc = p.scale.get();
    if (col < p.N && row < p.M)
        *(float4 *)(p.out + (int64_t)row * p.ldc + col) = float4{sc * sum.x, sc * sum.y, sc * sum.z, sc * sum.w};
}

}  // namespace dbp
