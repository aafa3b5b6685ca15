// NSD pass: fused dither + quantise + int8 codes + tile-sparse format + statistics.
//
// Eq. (nsd) of the paper, applied elementwise to the preactivation gradient as in Eq. (qdz):
//   k = floor(x/Delta + u),  u = nu/Delta + 1/2 in (0,1)  <=>  q = Delta*floor((x+nu)/Delta + 1/2).
// The kernel is HBM-bound: 4 B read + 1 B code + 1/8 B bitmap + 2 B per nonzero per element.
//
// Work decomposition: one wavefront owns one 256-column tile of one row per loop iteration.
// Lane l holds the 4 consecutive columns 4l..4l+3 (one 16-byte load, one 4-byte code store), so a
// tile is a single fully coalesced 1 KiB read.  The nonzero flags of the four sub-columns are
// wave ballots (free by-products of the compares); their popcounts give the tile count and, via
// mbcnt, each lane's exclusive prefix, so compaction needs neither LDS nor atomics.  The four
// ballots ARE the bitmap words of the tile (word j = sub-column j), so the bitmap costs nothing.
#include "common.h"

namespace dbp {

namespace {

constexpr uint32_t kG = 0x9E3779B9u, kA = 0x6A09E667u, kC = 0xBB67AE85u;

__host__ __device__ inline uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= kA; x ^= x >> 15; x *= kC; x ^= x >> 16;
    return x;
}

// One 32-bit hash word per PAIR of elements; `k1c` already contains k1 + hi32(counter)*C.
__device__ __forceinline__ uint32_t hash_word(uint32_t counter_lo, uint32_t k0, uint32_t k1c)
{
    uint32_t h = (counter_lo ^ k0) * kG;
    h ^= h >> 16;
    h = (h + k1c) * kA;
    h ^= h >> 15;
    h *= kC;
    h ^= h >> 16;
    return h;
}

// u = (2m+1) * 2^-17 for a 16-bit m: build 1 + m*2^-16 in the mantissa, subtract (1 - 2^-17). Exact.
__device__ __forceinline__ float dither_from_m16(uint32_t m)
{
    return __uint_as_float(0x3F800000u | (m << 7)) - 0x1.ffffp-1f;
}

__device__ __forceinline__ float dither_u(uint64_t g, uint32_t k0, uint32_t k1)
{
    uint64_t c = g >> 1;
    uint32_t h = hash_word((uint32_t)c, k0, k1 + (uint32_t)(c >> 32) * kC);
    return dither_from_m16((g & 1) ? (h >> 16) : (h & 0xFFFFu));
}

constexpr int kMaxRun = 16;
struct WaveStats { uint32_t nnz, sat, nonfinite; float maxabs; };

// {byte0 of d, byte0 of c, byte0 of b, byte0 of a} -> one dword, a in the low byte
__device__ __forceinline__ uint32_t pack_low_bytes(int a, int b, int c, int d)
{
    const uint32_t ab = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);
    const uint32_t cd = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x04000c0cu);
    return ab | cd;
}

// {Delta, 1/Delta} of Algorithm 1 from the sums of the values and of their squares: Delta = s * sqrt(S2/n - (S1/n)^2) in
// fp64, rounded to fp32 once.  A degenerate tensor (constant or non-finite gradient) gives {0, 0}: everything quantises
// to zero codes and the products are zero.
__device__ __forceinline__ void step_pair_from_sums(double S1, double S2, int64_t n, float s, float &step_out, float &inv_out)
{
    double var = n > 0 ? (S2 - S1 * S1 / (double)n) / (double)n : 0.0;
    if (var < 0.0) var = 0.0;
    const double sigma = __builtin_sqrt(var);
    const float step = (float)((double)s * sigma);
    const float inv = __fdiv_rn(1.0f, step);
    const bool ok = step > 0.0f && step < __builtin_inff() && inv >= 1.17549435e-38f && inv < __builtin_inff();
    step_out = ok ? step : 0.0f;
    inv_out = ok ? inv : 0.0f;
}

// One wavefront owns one 256-column tile per loop trip; every index that is the same for the whole
// wavefront (tile, row, segment, base offsets, the high half of the dither counter) lives in SGPRs.
// EX adds what surrounds the quantiser in a layer's backward pass: the rectifier's derivative applied on load
// (delta_z = delta_a (.) f'(z)), a step size that an earlier kernel left in device memory (Algorithm 1), and the
// bias gradient's integer code sums (the bias enters z additively: delta_b = sum of q over what shares the bias).
// Magnitude of an element as an integer that orders like it: the bit pattern of |x|, 0 for a NaN.
__device__ __forceinline__ uint32_t magnitude_key(float x)
{
    const uint32_t b = __float_as_uint(x) & 0x7fffffffu;
    return b > 0x7f800000u ? 0u : b;
}

// TOPK replaces the dither by the constant 1/2 (Eq. (nsd) with nu = 0: rounding to the nearest level) and drops the elements
// whose magnitude is below their vector's threshold: the top-k sparsifier of Sec. "Comparison to meProp" in the same code
// and tile format.
// COLWALK (per-column bias sums without the format) changes the order of the tiles only: a run of a.run tiles is the same
// 256-column segment of a.run consecutive rows, so that a lane meets the same four columns on every trip and keeps their
// code sums in registers: four atomics per lane and run instead of one per nonzero code.  Tile number t then counts
// (row block, segment, row in block), and the last block's rows past the tensor are empty tiles.
template <bool VEC, bool FORMAT, bool EX, bool TOPK = false, bool COLWALK = false>
__global__ __launch_bounds__(256) void nsd_kernel(NsdArgs a)
{
    static_assert(!(EX && TOPK), "the top-k sparsifier takes none of the layer extensions");
    static_assert(!COLWALK || (EX && !FORMAT), "the column walk serves the bias sums of a pass that writes no format");
    const int lane = threadIdx.x & 63;
    const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t n_waves = (int64_t)gridDim.x * 4;
    float inv = a.inv_step;
    if constexpr (EX) {
        if (a.tree.count > 0) {
            // the step size's tree is unfinished: every workgroup adds its last two levels (groups of 16 partial sums in
            // order, then the group sums in order: the same additions as std_finish_kernel), the first one publishes it
            __shared__ double s_tree[2][16];
            __shared__ float s_pair[2];
            const int count = a.tree.count, groups = (count + 15) >> 4;
            if ((int)threadIdx.x < groups) {
                const int lo = (int)threadIdx.x * 16;
                double v1[16], v2[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) { const int i = min(lo + j, count - 1); v1[j] = a.tree.s1[i]; v2[j] = a.tree.s2[i]; }
                double t1 = v1[0], t2 = v2[0];
#pragma unroll
                for (int j = 1; j < 16; ++j) if (lo + j < count) { t1 += v1[j]; t2 += v2[j]; }
                s_tree[0][threadIdx.x] = t1; s_tree[1][threadIdx.x] = t2;
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                double S1 = s_tree[0][0], S2 = s_tree[1][0];
                for (int i = 1; i < groups; ++i) { S1 += s_tree[0][i]; S2 += s_tree[1][i]; }
                float step, inv_step;
                step_pair_from_sums(S1, S2, a.tree.n, a.tree.s, step, inv_step);
                s_pair[0] = step; s_pair[1] = inv_step;
                if (blockIdx.x == 0) { a.tree.step_out[0] = step; a.tree.step_out[1] = inv_step; }
            }
            __syncthreads();
            inv = s_pair[1];
        } else if (a.step_dev) {
            inv = a.step_dev[1];
        }
    }
    const int c_in = 4 * lane;                                        // in-tile column of this lane's first element

    __shared__ __attribute__((aligned(16))) uint16_t s_ent[4][DBP_TILE];                          // per-wavefront staging of compacted entries
    WaveStats ws = {0u, 0u, 0u, 0.0f};
    uint64_t run_words = 0;                                           // per-run bitmap words / counts, see below
    uint32_t run_cnt = 0;

    // Tiles are handed out in runs of a.run consecutive tiles per wavefront, so that the bitmap words
    // and counts a wavefront writes on consecutive trips fall into the same cache lines.
    const uint32_t block_id = blockIdx.x;
    int64_t t = ((int64_t)block_id * 4 + wave_in_block) * a.run;
    int in_run = 0;
    int64_t row = t / a.tiles_per_row;
    int64_t seg = t - row * a.tiles_per_row;
    int bias_acc[4] = {0, 0, 0, 0};                                   // COLWALK: code sums of this lane's four columns in the run
    // COLWALK: unit u = t / run is (row block u / tiles_per_row, segment u % tiles_per_row); the run walks the block's rows
    auto colwalk_place = [&](int64_t tt, int64_t &r, int64_t &sg) {
        const int64_t u = tt / a.run, rb = u / a.tiles_per_row;
        sg = u - rb * a.tiles_per_row;
        r = rb * a.run + (tt - u * a.run);
    };
    if constexpr (COLWALK) colwalk_place(t, row, seg);

    auto tile_base = [&](int64_t r, int64_t sg) { return r * a.cols + sg * DBP_TILE; };
    auto load_tile = [&](const float *tensor, int64_t base, int valid, float (&x)[4]) {
        x[0] = x[1] = x[2] = x[3] = 0.f;
        const float *src = tensor + base;
        if (VEC) {
            if (c_in < valid) {
                const f32x4 v = __builtin_nontemporal_load((const f32x4 *)(src + c_in));
                x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (c_in + j < valid) x[j] = __builtin_nontemporal_load(src + c_in + j);
        }
    };

    float x[4], x_next[4];
    float m[4] = {1.f, 1.f, 1.f, 1.f}, m_next[4] = {1.f, 1.f, 1.f, 1.f};     // EX: the activation of each element
    const bool masked = EX && a.act != nullptr;
    int64_t base = 0;
    int valid = 0;
    if (t < a.n_tiles) {
        base = tile_base(row, seg);
        valid = (int)min((int64_t)DBP_TILE, a.cols - seg * DBP_TILE);
        if (COLWALK && row >= a.rows) valid = 0;                       // a row past the tensor: an empty tile
        load_tile(a.delta, base, valid, x);
        if (masked) load_tile(a.act, base, valid, m);
    }

    while (t < a.n_tiles) {
        // ---- software pipeline: issue the next tile's load before working on this one
        const bool jump = in_run == a.run - 1;                         // wave-uniform
        const int run_pos = in_run;                                    // position of this tile in its run
        int64_t t_next, row_next, seg_next, base_next;
        if (!jump) {                                                   // next tile of the run: it starts right
            t_next = t + 1; seg_next = seg + 1; row_next = row;        // after this one, also across a row end
            if constexpr (COLWALK) {                                   // (column walk: the same segment of the next row)
                seg_next = seg; row_next = row + 1;
                base_next = base + a.cols;
            } else {
                if (seg_next == a.tiles_per_row) { seg_next = 0; ++row_next; }
                base_next = base + valid;
            }
            ++in_run;
        } else {                                                       // first tile of this wavefront's next run
            t_next = t + (n_waves - 1) * a.run + 1;
            if constexpr (COLWALK) {
                colwalk_place(t_next, row_next, seg_next);
            } else {
                row_next = row + a.wave_stride_rows; seg_next = seg + a.wave_stride_segs;
                if (seg_next >= a.tiles_per_row) { seg_next -= a.tiles_per_row; ++row_next; }
            }
            base_next = tile_base(row_next, seg_next);
            in_run = 0;
        }
        const bool last_of_run = jump || t + 1 >= a.n_tiles;
        int valid_next = 0;
        if (t_next < a.n_tiles) {
            valid_next = (int)min((int64_t)DBP_TILE, a.cols - seg_next * DBP_TILE);
            if (COLWALK && row_next >= a.rows) valid_next = 0;
            load_tile(a.delta, base_next, valid_next, x_next);
            if (masked) load_tile(a.act, base_next, valid_next, m_next);
        }
        if (masked) {
            // derivative of the rectifier: 1 where the activation is positive (-0.0 and NaN count as not positive)
#pragma unroll
            for (int j = 0; j < 4; ++j) x[j] = m[j] > 0.0f ? x[j] : 0.0f;
        }

        // ---- dither: elements share hash words pairwise by the parity of the GLOBAL index
        const uint64_t g_tile = a.idx_base + (uint64_t)base;          // wave-uniform
        float u[4];
        const uint64_t c_tile = g_tile >> 1;
        const bool paired = VEC && !(g_tile & 1) && (uint32_t)c_tile < 0xFFFFFF00u;    // wave-uniform
        if constexpr (TOPK) {
            const uint32_t thr = a.topk_thr[a.topk_vec_rows == 1 ? row : row / a.topk_vec_rows];   // wave-uniform
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x[j] = magnitude_key(x[j]) >= thr ? x[j] : 0.0f;
                u[j] = 0.5f;
            }
        } else if (paired) {
            const uint32_t k1c = a.k1 + (uint32_t)(c_tile >> 32) * kC;                 // scalar
#ifdef DBP_NSD_DITHER23
            // MEASUREMENT BUILD ONLY (never the product: these codes are not the oracle's): one hash word per ELEMENT and a
            // 23-bit dither u = (2m+1) * 2^-24, to price the choice of one word per element pair and 16 bits.
            const uint32_t c0 = (uint32_t)g_tile + 4u * (uint32_t)lane;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                u[j] = __uint_as_float(0x3F800000u | (hash_word(c0 + (uint32_t)j, a.k0, k1c) >> 9)) - 0x1.fffffep-1f;
#else
            const uint32_t c0 = (uint32_t)c_tile + 2u * (uint32_t)lane;
            const uint32_t hA = hash_word(c0, a.k0, k1c);
            const uint32_t hB = hash_word(c0 + 1u, a.k0, k1c);
            u[0] = dither_from_m16(hA & 0xFFFFu); u[1] = dither_from_m16(hA >> 16);
            u[2] = dither_from_m16(hB & 0xFFFFu); u[3] = dither_from_m16(hB >> 16);
#endif
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) u[j] = dither_u(g_tile + (uint64_t)(c_in + j), a.k0, a.k1);
        }

        // ---- quantise: k = floor(fma(x, 1/Delta, u)) clamped to [-127,127]
        float kf[4], kc[4];
        int k[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            kf[j] = __builtin_floorf(__builtin_fmaf(x[j], inv, u[j]));
            kc[j] = __builtin_amdgcn_fmed3f(kf[j], -127.0f, 127.0f); // NaN -> unspecified here, repaired below
            k[j] = (int)kc[j];
        }
        // Clamping changed the value (saturation, +-Inf input) or the value is NaN (NaN != anything):
        // rare, decided per wavefront.  Finite inputs with |floor| <= 127 never take this branch.
        const bool odd = (kf[0] != kc[0]) | (kf[1] != kc[1]) | (kf[2] != kc[2]) | (kf[3] != kc[3]);
        if (__builtin_amdgcn_ballot_w64(odd)) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // a NaN t (NaN input, or +-Inf input times the 1/Delta = 0 of a degenerate layer) gives code 0
                const bool nan = kf[j] != kf[j];
                const bool bad = (x[j] != x[j]) | (fabsf(x[j]) == __builtin_inff());
                if (nan) { k[j] = 0; kc[j] = 0.f; }
                ws.nonfinite += __builtin_popcountll(__builtin_amdgcn_ballot_w64(bad));
                ws.sat += __builtin_popcountll(__builtin_amdgcn_ballot_w64(!nan && fabsf(kf[j]) > 127.0f));
            }
        }
        ws.maxabs = fmaxf(fmaxf(ws.maxabs, fmaxf(fabsf(kc[0]), fabsf(kc[1]))), fmaxf(fabsf(kc[2]), fabsf(kc[3])));

        // ---- codes
        int8_t *dst = a.codes + base;
        if (VEC) {
            if (c_in < valid) __builtin_nontemporal_store(pack_low_bytes(k[0], k[1], k[2], k[3]), (uint32_t *)(dst + c_in));
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (c_in + j < valid) dst[c_in + j] = (int8_t)k[j];
        }

        // ---- bias gradient: integer sums of the codes (exact, order-free: atomics are deterministic here)
        if (EX && a.bias_sums) {
            if (a.bias_mode == 0) {
                // per column; columns past the row's end hold x = 0 -> code 0 and add nothing
                int64_t *col = a.bias_sums + seg * DBP_TILE + c_in;
                if constexpr (COLWALK) {
                    // at most 16384 rows of |code| <= 127 per run: the 32-bit sums cannot overflow
#pragma unroll
                    for (int j = 0; j < 4; ++j) bias_acc[j] += k[j];
                    if (last_of_run) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (bias_acc[j] != 0) atomicAdd((unsigned long long *)(col + j), (unsigned long long)(long long)bias_acc[j]);
                            bias_acc[j] = 0;
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (k[j] != 0) atomicAdd((unsigned long long *)(col + j), (unsigned long long)(long long)k[j]);
                }
            } else {
                int sum = (k[0] + k[1]) + (k[2] + k[3]);
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
                if (lane == 0 && sum != 0)
                    atomicAdd((unsigned long long *)(a.bias_sums + row % a.bias_len), (unsigned long long)(long long)sum);
            }
        }

        // ---- tile-sparse format
        const uint64_t b0 = __builtin_amdgcn_ballot_w64(k[0] != 0);
        const uint64_t b1 = __builtin_amdgcn_ballot_w64(k[1] != 0);
        const uint64_t b2 = __builtin_amdgcn_ballot_w64(k[2] != 0);
        const uint64_t b3 = __builtin_amdgcn_ballot_w64(k[3] != 0);
        const uint32_t cnt = __builtin_popcountll(b0) + __builtin_popcountll(b1) +
                             __builtin_popcountll(b2) + __builtin_popcountll(b3);
        ws.nnz += cnt;
        if (FORMAT) {
            uint32_t pre = 0;                                          // nonzeros in lower lanes
            pre = __builtin_amdgcn_mbcnt_hi((uint32_t)(b0 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b0, pre));
            pre = __builtin_amdgcn_mbcnt_hi((uint32_t)(b1 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b1, pre));
            pre = __builtin_amdgcn_mbcnt_hi((uint32_t)(b2 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b2, pre));
            pre = __builtin_amdgcn_mbcnt_hi((uint32_t)(b3 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b3, pre));
            uint16_t *ent = a.entries + t * DBP_TILE;                  // scalar base, 32-bit lane offsets
            // Compact through LDS so that the tile's entries leave as ONE contiguous store (lanes 0..cnt/4,
            // four entries each) instead of four sparse 2-byte stores.  A wavefront's LDS operations
            // execute in order, so the read below sees the writes above without a barrier.
            uint16_t *se = s_ent[wave_in_block];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool nz = k[j] != 0;
                if (nz) se[pre] = (uint16_t)(((uint32_t)k[j] & 0xFFu) | (uint32_t)((c_in + j) << 8));
                pre += nz;
            }
            typedef uint64_t __attribute__((may_alias)) u64_alias;     // the 16-bit writes above feed this 64-bit read
            if (4 * lane < (int)cnt) ((u64_alias *)ent)[lane] = ((const u64_alias *)se)[lane];   // up to 256 entries
            // bitmap word j is the ballot of sub-column j: bit l <=> in-tile column 4l+j.  (Re-ordering the
            // bits into plain column order costs ~80 scalar instructions per tile, and the scalar unit is
            // shared by the whole CU: that alone made the pass scalar-bound.)
            // The words and the count of the run's i-th tile are parked in lanes 4i..4i+3 resp. lane i and
            // written once per run: one 512-byte and one 32-byte store instead of 32 small ones.
            const uint64_t mine = (lane & 3) == 0 ? b0 : (lane & 3) == 1 ? b1 : (lane & 3) == 2 ? b2 : b3;
            if ((lane >> 2) == run_pos) run_words = mine;
            if (lane == run_pos) run_cnt = cnt;
            if (last_of_run) {
                const int64_t t0 = t - run_pos;                        // first tile of the run
                if (lane < 4 * (run_pos + 1)) a.bitmap[t0 * 4 + lane] = run_words;
                if (lane <= run_pos) a.tile_nnz[t0 + lane] = (uint16_t)run_cnt;
            }
        }

        t = t_next; row = row_next; seg = seg_next; base = base_next; valid = valid_next;
#pragma unroll
        for (int j = 0; j < 4; ++j) { x[j] = x_next[j]; m[j] = m_next[j]; }
    }

    if (a.stats) {
        // wave-level maxima and sums (sums are already wave-uniform), then one partial per workgroup
        float mx = ws.maxabs;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        __shared__ uint32_t s_nnz[4], s_sat[4], s_nf[4];
        __shared__ int s_mx[4];
        if (lane == 0) { s_nnz[wave_in_block] = ws.nnz; s_sat[wave_in_block] = ws.sat;
                         s_nf[wave_in_block] = ws.nonfinite; s_mx[wave_in_block] = (int)mx; }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint64_t nnz = (uint64_t)s_nnz[0] + s_nnz[1] + s_nnz[2] + s_nnz[3];
            uint64_t sat = (uint64_t)s_sat[0] + s_sat[1] + s_sat[2] + s_sat[3];
            uint64_t nf  = (uint64_t)s_nf[0] + s_nf[1] + s_nf[2] + s_nf[3];
            int m = max(max(s_mx[0], s_mx[1]), max(s_mx[2], s_mx[3]));
            if (a.partials) {
                // same-address device atomics serialise at roughly 12 ns each: keep them off the fast path
                a.partials[block_id] = u32x4{(uint32_t)nnz, (uint32_t)sat, (uint32_t)nf, (uint32_t)m};
            } else {
                if (nnz) atomicAdd((unsigned long long *)&a.stats->nnz, (unsigned long long)nnz);
                if (sat) atomicAdd((unsigned long long *)&a.stats->n_saturated, (unsigned long long)sat);
                if (nf)  atomicAdd((unsigned long long *)&a.stats->n_nonfinite, (unsigned long long)nf);
                if (m)   atomicMax(&a.stats->max_abs_code, m);
            }
        }
    }
}

// Sum the per-workgroup statistics in a fixed order (one workgroup; deterministic, no atomics).
__global__ __launch_bounds__(1024) void finalize_stats_kernel(const u32x4 *partials, int n, dbp_stats *out, StatsJob job)
{
    __shared__ uint64_t s_nnz[1024], s_sat[1024], s_nf[1024];
    __shared__ int s_mx[1024];
    uint64_t nnz = 0, sat = 0, nf = 0; int mx = 0;
    static_assert(kNsdMaxBlocks <= 16 * 1024, "finalize reads at most 16 records per thread");
    u32x4 q[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {                       // all loads in flight at once
        const int i = threadIdx.x + r * 1024;
        q[r] = i < n ? partials[i] : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) { nnz += q[r].x; sat += q[r].y; nf += q[r].z; mx = max(mx, (int)q[r].w); }
    s_nnz[threadIdx.x] = nnz; s_sat[threadIdx.x] = sat; s_nf[threadIdx.x] = nf; s_mx[threadIdx.x] = mx;
    __syncthreads();
    for (int off = 512; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) {
            s_nnz[threadIdx.x] += s_nnz[threadIdx.x + off]; s_sat[threadIdx.x] += s_sat[threadIdx.x + off];
            s_nf[threadIdx.x] += s_nf[threadIdx.x + off]; s_mx[threadIdx.x] = max(s_mx[threadIdx.x], s_mx[threadIdx.x + off]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (out) { out->nnz = s_nnz[0]; out->n_saturated = s_sat[0]; out->n_nonfinite = s_nf[0]; out->max_abs_code = s_mx[0]; out->reserved = 0; }
        write_density_flags(job, s_nnz[0]);
    }
}

__global__ void zero_stats_kernel(dbp_stats *s)
{
    if (threadIdx.x == 0) { s->nnz = 0; s->n_saturated = 0; s->n_nonfinite = 0; s->max_abs_code = 0; s->reserved = 0; }
}

__global__ void zero_i64_kernel(int64_t *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// delta_b = Delta * (sum of codes): one fp64 product rounded to fp32 per bias element.
__global__ void bias_grad_kernel(const int64_t *sums, int64_t n, float step, const float *step_dev, float *grad)
{
    const double d = step_dev ? (double)step_dev[0] : (double)step;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        grad[i] = (float)(d * (double)sums[i]);
}

// ---- step size of Algorithm 1: sigma = std(delta_z), Delta = s * sigma --------------------------------------
// Population standard deviation from S1 = sum x and S2 = sum x*x in fp64 (x*x is exact there).  Delta decides
// integer codes, so the ORDER of the sums is fixed: a radix-16 tree -- groups of 16 consecutive values are
// summed left to right, the group sums again in groups of 16, and so on.  The first kernel does three levels
// (a thread sums its 16 consecutive elements; lane 16g adds the 16 thread sums of its lane group in order; one
// thread adds the workgroup's 16 lane-group sums in order), the second kernel finishes the tree with one
// workgroup and writes {Delta, 1/Delta}.
__global__ __launch_bounds__(256) void std_tree_kernel(const float *delta, const float *act, int64_t n, double *out1, double *out2,
                                                       int64_t *zero, int64_t zero_len)
{
    const int tid = threadIdx.x, lane = tid & 63;
    // by the way: clear the bias code sums that the quantiser (the next kernel of the stream) adds into
    for (int64_t i = (int64_t)blockIdx.x * 256 + tid; i < zero_len; i += (int64_t)gridDim.x * 256) zero[i] = 0;
    const int64_t first = ((int64_t)blockIdx.x * 256 + tid) * 16;     // this thread's 16 consecutive elements
    const int have = (int)max((int64_t)0, min((int64_t)16, n - first));
    float v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = 0.f;
    if (have == 16 && (((uintptr_t)(delta + first)) & 15) == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 t = *(const f32x4 *)(delta + first + 4 * q);
            v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) if (j < have) v[j] = delta[first + j];
    }
    if (act) {                                                         // delta_z = delta_a where the activation is positive
#pragma unroll
        for (int j = 0; j < 16; ++j) if (j < have) v[j] = act[first + j] > 0.0f ? v[j] : 0.0f;
    }
    // level 0 (elements past the end do not exist; adding their +0.0 squares or values changes nothing)
    double s1 = (double)v[0], s2 = (double)v[0] * (double)v[0];
#pragma unroll
    for (int j = 1; j < 16; ++j) {
        const double x = (double)v[j];
        if (j < have) { s1 += x; s2 = __builtin_fma(x, x, s2); }       // x*x is exact: fma == multiply, then add
    }
    // level 1: lane 16g collects lanes 16g+1 .. 16g+15 in order (a thread without elements holds no value)
    const int64_t n0 = (n + 15) / 16;                                  // values at level 0
    const int64_t i0 = (int64_t)blockIdx.x * 256 + tid;
    double a1 = s1, a2 = s2;
#pragma unroll
    for (int i = 1; i < 16; ++i) {
        const double o1 = __shfl(s1, (lane & 48) + i), o2 = __shfl(s2, (lane & 48) + i);
        if ((lane & 15) == 0 && i0 + i < n0) { a1 += o1; a2 += o2; }
    }
    // level 2: the workgroup's 16 lane groups in order
    __shared__ double l1[2][16];
    if ((lane & 15) == 0) { l1[0][tid >> 4] = a1; l1[1][tid >> 4] = a2; }
    __syncthreads();
    if (tid == 0) {
        const int64_t n1 = (n0 + 15) / 16, i1 = (int64_t)blockIdx.x * 16;
        double t1 = l1[0][0], t2 = l1[1][0];
        for (int i = 1; i < 16; ++i)
            if (i1 + i < n1) { t1 += l1[0][i]; t2 += l1[1][i]; }
        out1[blockIdx.x] = t1; out2[blockIdx.x] = t2;
    }
}

__global__ __launch_bounds__(256) void std_finish_kernel(double *a1, double *a2, double *b1, double *b2, int64_t count,
                                                         int64_t n, float s, float *step_out)
{
    // remaining levels of the tree, ping-pong between the two scratch halves
    double *src1 = a1, *src2 = a2, *dst1 = b1, *dst2 = b2;
    while (count > 1) {
        const int64_t groups = (count + 15) / 16;
        for (int64_t g = threadIdx.x; g < groups; g += 256) {
            const int64_t lo = g * 16, hi = min(count, lo + 16);
            double t1 = src1[lo], t2 = src2[lo];
            for (int64_t i = lo + 1; i < hi; ++i) { t1 += src1[i]; t2 += src2[i]; }
            dst1[g] = t1; dst2[g] = t2;
        }
        __syncthreads();
        double *t;
        t = src1; src1 = dst1; dst1 = t;
        t = src2; src2 = dst2; dst2 = t;
        count = groups;
    }
    if (threadIdx.x == 0) {
        float step, inv;
        step_pair_from_sums(n > 0 ? src1[0] : 0.0, n > 0 ? src2[0] : 0.0, n, s, step, inv);
        step_out[0] = step;
        step_out[1] = inv;
    }
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// Symmetric int8 quantiser of weights and activations (Sec. "Quantizing forward pass": the forward pass
// computes with 8-bit weights and activations; the paper takes the quantiser from the work it cites
// and does not print it, so the plainest one is used).  One scale per tensor:
//   amax = max |x_i| over the finite x_i;   scale = amax / 127;   inv = 127 / amax   (fp32 divisions)
//   q_i  = clamp(round-half-even(x_i * inv), -127, 127)   (one fp32 multiplication)
// NaN -> 0, +-Inf -> +-127; amax == 0 (or nothing finite): scale = inv = 0 and every finite q_i is 0.
// ------------------------------------------------------------------------------------------------
constexpr int kQuantBlocks = 2048;

__global__ __launch_bounds__(256) void absmax_kernel(const float *x, int64_t n, uint32_t *partial)
{
    // magnitudes of finite floats order like their bit patterns
    uint32_t m = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const uint32_t b = __float_as_uint(x[i]) & 0x7fffffffu;
        if (b < 0x7f800000u) m = b > m ? b : m;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { const uint32_t o = __shfl_xor(m, off); m = o > m ? o : m; }
    __shared__ uint32_t wm[4];
    if ((threadIdx.x & 63) == 0) wm[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) m = wm[w] > m ? wm[w] : m;
        partial[blockIdx.x] = m;
    }
}

__global__ __launch_bounds__(256) void absmax_finish_kernel(const uint32_t *partial, int blocks, float *scale_out)
{
    uint32_t m = 0;
    for (int i = threadIdx.x; i < blocks; i += 256) m = partial[i] > m ? partial[i] : m;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { const uint32_t o = __shfl_xor(m, off); m = o > m ? o : m; }
    __shared__ uint32_t wm[4];
    if ((threadIdx.x & 63) == 0) wm[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) m = wm[w] > m ? wm[w] : m;
        const float amax = __uint_as_float(m);
        scale_out[0] = amax > 0.0f ? __fdiv_rn(amax, 127.0f) : 0.0f;
        scale_out[1] = amax > 0.0f ? __fdiv_rn(127.0f, amax) : 0.0f;
    }
}

__device__ __forceinline__ int quantize_one(float x, float inv)
{
    const uint32_t b = __float_as_uint(x) & 0x7fffffffu;
    if (b > 0x7f800000u) return 0;                                         // NaN
    if (b == 0x7f800000u) return x > 0.0f ? 127 : -127;                    // +-Inf
    const float t = __builtin_rintf(__fmul_rn(x, inv));                    // ties to even
    return (int)fminf(fmaxf(t, -127.0f), 127.0f);
}

__global__ __launch_bounds__(256) void quantize_int8_kernel(const float *x, int64_t n, const float *scale, int8_t *q)
{
    const float inv = scale[1];
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        q[i] = (int8_t)quantize_one(x[i], inv);
}

size_t quantize_scratch_bytes(int64_t) { return align_up((size_t)kQuantBlocks * sizeof(uint32_t), 256); }

hipError_t launch_quantize_int8(const float *x, int64_t n, int8_t *q, float *scale_out, void *scratch, hipStream_t st)
{
    int64_t blocks = (n + 1023) / 1024;                                    // four elements per thread at least
    blocks = blocks < 1 ? 1 : blocks > kQuantBlocks ? kQuantBlocks : blocks;
    hipLaunchKernelGGL(absmax_kernel, dim3((unsigned)blocks), dim3(256), 0, st, x, n, (uint32_t *)scratch);
    hipLaunchKernelGGL(absmax_finish_kernel, dim3(1), dim3(256), 0, st, (const uint32_t *)scratch, (int)blocks, scale_out);
    hipLaunchKernelGGL(quantize_int8_kernel, dim3((unsigned)blocks), dim3(256), 0, st, x, n, (const float *)scale_out, q);
    return hipGetLastError();
}

size_t step_size_scratch_bytes(int64_t n)
{
    const int64_t wgs = (n + 4095) / 4096 > 0 ? (n + 4095) / 4096 : 1;
    const int64_t second = (wgs + 15) / 16;                            // the finishing kernel's other half
    return align_up((size_t)(2 * wgs + 2 * second) * sizeof(double), 256);
}

hipError_t launch_step_size(const float *delta, const float *act, int64_t n, float s, float *step_out, void *scratch, hipStream_t st,
                            int64_t *zero, int64_t zero_len, StepTree *defer)
{
    const int64_t wgs = (n + 4095) / 4096 > 0 ? (n + 4095) / 4096 : 1;
    const int64_t second = (wgs + 15) / 16;
    double *a1 = (double *)scratch, *a2 = a1 + wgs, *b1 = a2 + wgs, *b2 = b1 + second;
    hipLaunchKernelGGL(std_tree_kernel, dim3((unsigned)wgs), dim3(256), 0, st, delta, act, n, a1, a2, zero, zero_len);
    if (defer) *defer = StepTree{nullptr, nullptr, 0, 0, 0.0f, nullptr};
    if (defer && wgs <= 256) {
        // two levels are left: the quantiser's workgroups add them on their way in (a launch less)
        *defer = StepTree{a1, a2, (int)wgs, n, s, step_out};
        return hipGetLastError();
    }
    hipLaunchKernelGGL(std_finish_kernel, dim3(1), dim3(256), 0, st, a1, a2, b1, b2, wgs, n, s, step_out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Top-k sparsifier, selection: the k-th largest magnitude of every vector, found by a binary search over the 31 bits of
// the magnitude keys, most significant first: the threshold is the largest T with at least k keys >= T.  WAVES
// wavefronts share a vector (one: four vectors per workgroup, no barrier; sixteen: one vector per workgroup, one barrier
// per bit); each lane keeps E keys in registers, or (MEM) re-reads the vector at every bit.
template <int WAVES, int E, bool MEM>
__global__ __launch_bounds__(WAVES == 1 ? 256 : 64 * WAVES) void topk_threshold_kernel(const float *delta, int64_t n_vec, int64_t len,
                                                                                      int64_t k, uint32_t *thr)
{
    constexpr int GROUP = 64 * WAVES;                                  // threads per vector
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t v = WAVES == 1 ? (int64_t)blockIdx.x * 4 + wave : (int64_t)blockIdx.x;
    if (v >= n_vec) return;                                            // whole wavefronts (WAVES == 1) or never (grid = n_vec)
    const int t = WAVES == 1 ? lane : (int)threadIdx.x;
    const float *src = delta + v * len;
    __shared__ uint32_t s_cnt[2][16];
    uint32_t key[E];
    if constexpr (!MEM) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int64_t idx = (int64_t)e * GROUP + t;
            key[e] = idx < len ? magnitude_key(src[idx]) : 0u;        // a candidate is never 0: padding is never counted
        }
    }
    uint32_t prefix = 0;
    for (int b = 30; b >= 0; --b) {
        const uint32_t cand = prefix | (1u << b);
        uint32_t c = 0;
        if constexpr (!MEM) {
#pragma unroll
            for (int e = 0; e < E; ++e) c += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(key[e] >= cand));
        } else {
            for (int64_t base = 0; base < len; base += GROUP) {        // the same trips for every lane
                const int64_t idx = base + t;
                const uint32_t kk = idx < len ? magnitude_key(src[idx]) : 0u;
                c += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(kk >= cand));
            }
        }
        if constexpr (WAVES > 1) {
            // buffer b & 1 is written again two bits later, after the barrier of the bit in between: every read is over by then
            if (lane == 0) s_cnt[b & 1][wave] = c;
            __syncthreads();
            c = 0;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) c += s_cnt[b & 1][w];
        }
        if ((int64_t)c >= k) prefix = cand;
    }
    // k <= 0: a threshold above the key of +-Inf, nothing survives; fewer than k keys >= 1: prefix stays 0, everything does
    if (t == 0) thr[v] = k <= 0 ? 0x7f800001u : prefix;
}

hipError_t launch_topk_threshold(const float *delta, int64_t n_vec, int64_t len, int64_t k, uint32_t *thr, hipStream_t s)
{
    // one wavefront per vector only when there are enough vectors to fill the chip with them (1024 SIMDs); few long-ish
    // vectors get sixteen wavefronts each
    if (len <= 256 || (len <= 4096 && n_vec >= 2048)) {
        const dim3 grid((unsigned)((n_vec + 3) / 4)), block(256);
        if (len <= 256)       hipLaunchKernelGGL((topk_threshold_kernel<1, 4, false>), grid, block, 0, s, delta, n_vec, len, k, thr);
        else if (len <= 1024) hipLaunchKernelGGL((topk_threshold_kernel<1, 16, false>), grid, block, 0, s, delta, n_vec, len, k, thr);
        else                  hipLaunchKernelGGL((topk_threshold_kernel<1, 64, false>), grid, block, 0, s, delta, n_vec, len, k, thr);
    } else {
        const dim3 grid((unsigned)n_vec), block(1024);
        if (len <= 4096)       hipLaunchKernelGGL((topk_threshold_kernel<16, 4, false>), grid, block, 0, s, delta, n_vec, len, k, thr);
        else if (len <= 16384) hipLaunchKernelGGL((topk_threshold_kernel<16, 16, false>), grid, block, 0, s, delta, n_vec, len, k, thr);
        else if (len <= 65536) hipLaunchKernelGGL((topk_threshold_kernel<16, 64, false>), grid, block, 0, s, delta, n_vec, len, k, thr);
        else                   hipLaunchKernelGGL((topk_threshold_kernel<16, 1, true>), grid, block, 0, s, delta, n_vec, len, k, thr);
    }
    return hipGetLastError();
}

DitherKeys make_dither_keys(uint64_t seed)
{
    DitherKeys k;
    k.k0 = mix32((uint32_t)seed ^ kG);
    k.k1 = mix32((uint32_t)(seed >> 32) + k.k0 + kA);
    return k;
}

hipError_t launch_stats_job(const StatsJob &j, hipStream_t s)
{
    if (j.n > 0) hipLaunchKernelGGL(finalize_stats_kernel, dim3(1), dim3(1024), 0, s, j.partials, j.n, j.out, j);
    if (j.bias_len > 0) {
        const int64_t zb = (j.bias_len + 255) / 256;
        hipLaunchKernelGGL(bias_grad_kernel, dim3((unsigned)(zb < 1024 ? zb : 1024)), dim3(256), 0, s, j.bias_sums, j.bias_len,
                           j.step, j.step_dev, j.bias_grad);
    }
    return hipGetLastError();
}

hipError_t launch_nsd(const NsdArgs &a_in, hipStream_t s, StatsJob *defer)
{
    if (defer) *defer = StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr};
    NsdArgs a = a_in;
    if (!a.stats) a.partials = nullptr;
    const bool use_atomics = a.stats && !a.partials;
    if (use_atomics) hipLaunchKernelGGL(zero_stats_kernel, dim3(1), dim3(64), 0, s, a.stats);
    // per-wave element counts are 32-bit: one wave sees at most n_tiles/(4*blocks) tiles of 256 elements
    // One run of consecutive tiles per wavefront: as long as it takes to keep 8192 wavefronts (full
    // occupancy of 256 CUs) busy, at most kMaxRun; beyond kNsdMaxBlocks workgroups the runs are grid-strided.
    int64_t run = a.n_tiles / 8192;
    run = run < 1 ? 1 : run > kMaxRun ? kMaxRun : run;
    // Per-column bias sums without the format: runs go down the rows of one 256-column segment (sums in registers, see
    // nsd_kernel), as many rows as leave 16384 runs for the chip, at most 64; a.n_tiles then counts the row blocks' tiles,
    // the empty ones past the last row included.
    bool colwalk = false;
    if (a.bias_sums && a.bias_mode == 0 && !a.bitmap) {
        int64_t rb = a.n_tiles / 16384;
        rb = rb > 64 ? 64 : rb;
        if (rb >= 2) {
            colwalk = true;
            run = rb;
            a.n_tiles = a.tiles_per_row * ((a.rows + rb - 1) / rb) * rb;
        }
    }
    a.run = (int)run;
    int64_t blocks = (a.n_tiles + 4 * run - 1) / (4 * run);
    const int64_t max_blocks = use_atomics ? 256 : kNsdMaxBlocks;
    if (blocks > max_blocks) blocks = max_blocks;
    if (blocks < 1) blocks = 1;
    const bool vec_d = (a.cols % 4 == 0) && ((uintptr_t)a.delta % 16 == 0) && ((uintptr_t)a.codes % 4 == 0);
    const int64_t jump = (blocks * 4 - 1) * run + 1;        // tiles from the last tile of a run to the next run
    a.wave_stride_rows = jump / a.tiles_per_row;
    a.wave_stride_segs = jump % a.tiles_per_row;
    const dim3 grid((unsigned)blocks), block(256);
    const bool ex = a.act || a.step_dev || a.bias_sums;
    if (a.bias_sums && !a.bias_zeroed) {
        const int64_t zb = (a.bias_len + 255) / 256;
        hipLaunchKernelGGL(zero_i64_kernel, dim3((unsigned)(zb < 1024 ? zb : 1024)), dim3(256), 0, s, a.bias_sums, a.bias_len);
    }
    const bool vec = vec_d && (!a.act || ((uintptr_t)a.act % 16 == 0));
    if (a.topk_thr) {
        if (vec && a.bitmap)       hipLaunchKernelGGL((nsd_kernel<true, true, false, true>), grid, block, 0, s, a);
        else if (vec)              hipLaunchKernelGGL((nsd_kernel<true, false, false, true>), grid, block, 0, s, a);
        else if (a.bitmap)         hipLaunchKernelGGL((nsd_kernel<false, true, false, true>), grid, block, 0, s, a);
        else                       hipLaunchKernelGGL((nsd_kernel<false, false, false, true>), grid, block, 0, s, a);
    } else if (!ex) {
        if (vec && a.bitmap)       hipLaunchKernelGGL((nsd_kernel<true, true, false>), grid, block, 0, s, a);
        else if (vec)              hipLaunchKernelGGL((nsd_kernel<true, false, false>), grid, block, 0, s, a);
        else if (a.bitmap)         hipLaunchKernelGGL((nsd_kernel<false, true, false>), grid, block, 0, s, a);
        else                       hipLaunchKernelGGL((nsd_kernel<false, false, false>), grid, block, 0, s, a);
    } else if (colwalk) {
        if (vec)                   hipLaunchKernelGGL((nsd_kernel<true, false, true, false, true>), grid, block, 0, s, a);
        else                       hipLaunchKernelGGL((nsd_kernel<false, false, true, false, true>), grid, block, 0, s, a);
    } else {
        if (vec && a.bitmap)       hipLaunchKernelGGL((nsd_kernel<true, true, true>), grid, block, 0, s, a);
        else if (vec)              hipLaunchKernelGGL((nsd_kernel<true, false, true>), grid, block, 0, s, a);
        else if (a.bitmap)         hipLaunchKernelGGL((nsd_kernel<false, true, true>), grid, block, 0, s, a);
        else                       hipLaunchKernelGGL((nsd_kernel<false, false, true>), grid, block, 0, s, a);
    }
    StatsJob later{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr};
    if (a.bias_sums && a.bias_grad) {
        later.bias_sums = a.bias_sums; later.bias_len = a.bias_len; later.bias_grad = a.bias_grad;
        later.step = a.step; later.step_dev = a.step_dev;
    }
    if (a.partials) { later.partials = (const u32x4 *)a.partials; later.n = (int)blocks; later.out = a.stats; }
    if (defer) *defer = later;
    else return launch_stats_job(later, s);
    return hipGetLastError();
}

}  // namespace dbp
