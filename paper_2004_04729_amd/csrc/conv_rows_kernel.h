// Gather kernels of the convolutional backward products, Sec. "Computational complexity": work in proportion to the nonzero
// codes, on the vector ALUs (internal header of gather.hip).
//
// Both kernels read the code PLANE (one byte per element), not the compacted entries: a wavefront loads a stretch of a plane,
// the lanes' `v_cmp` results are the nonzero mask, and a scalar loop visits the set bits -- the nonzero's position, its code
// and everything derived from them are wave-uniform (SGPRs), the 64 lanes are 64 channels c.
//
//   conv_dw_rows_kernel   dW[k,c,r,s] = Delta * sum_{n, nonzero (p,q) of plane (n,k)} code * X[n,c,p*st+r-pad,q*st+s-pad]
//     A workgroup owns 64 channels x 64 code planes (16 wavefronts x 4 planes) and walks a share of the (image, row band)
//     units.  Per unit it stages the band of X, with its zero halo, in LDS as cells [pixel][64 channels] (one cell = the
//     64 lanes' operands of one tap: a conflict-free LDS read); per nonzero a lane reads its channel's R*S activations and
//     adds code * x into the R*S accumulators of that plane -- REGISTERS, because the tap index is static and the plane is
//     the wavefront's own.  Shares of the units are summed by conv_dw_rows_reduce_kernel in a fixed order.
//   conv_dx_rows_kernel   dX[n,c,h,w] = Delta * sum_{k,r,s} code[n,k,p,q] * W[k,c,r,s],  h = p+r-pad, w = q+s-pad  (stride 1)
//     A workgroup owns an image's band of output rows x 64 channels, a wavefront one output row.  The row's accumulators
//     [pixel][64 channels] live in LDS (the pixel a nonzero lands on is data).  Weights (prepared once per call as
//     [k][tap][c]) and code rows come through LDS in chunks of 8 planes, shared by the workgroup's wavefronts; a wavefront scans
//     the R code rows that reach its output row and, per nonzero, read-multiply-add-writes S neighbouring cells.  Each cell
//     belongs to one wavefront, so the order of the additions is the program's: the result is deterministic.
#pragma once
#include <type_traits>
#include "common.h"

namespace dbp {

constexpr int CGR_WAVES = 16;                      // dW: wavefronts per workgroup (one workgroup per CU; 8 with two per CU staged X twice as often: 3-20 % slower)
constexpr int CGR_PPW = 4;                         // dW: code planes per wavefront
constexpr int CGR_KB = CGR_WAVES * CGR_PPW;        // dW: code planes per workgroup
constexpr int CGR_MAX_CHUNKS = 20;                 // dW: 64-cell chunks of the X tile, at most (1280 cells)
constexpr int CGR_MAX_LOADS = 4;                   // dW: dwords of a band's codes per lane and plane, at most (1 KiB of codes)
constexpr int CGR_DX_MAX_ROWS = 16;                // dX: output rows (= wavefronts) per workgroup, at most

struct ConvDwRowsArgs {
    const int8_t *codes;              // plane (n, k) at codes + (n*Kt + k) * P*Q; 4-byte aligned, P*Q a multiple of 4
    const void   *X;                  // [N][Ct][H][Wd], fp32 or int8
    void         *out;                // n_split == 1: dW [K][C][R*S] (fp32: scaled); else partial sums [split][K][C][R*S]
    int N, C, K, H, Wd, P, Q, pad, st, Ct, Kt;
    int TH, THx, Wp, bands;           // code rows per band; rows and columns of the X tile; bands per image
    int cells, n_chunks;              // THx*Wp; ceil(cells / 64)
    int units, units_per_split, n_split;
    uint32_t q_magic, wp_magic;       // floor(2^32 / Q) + 1, floor(2^32 / Wp) + 1: x / Q == mulhi(x, q_magic) for x < 2^16
    Scale scale;
    Gate gate;
};

template <class XT, int R, int S>
__global__ __launch_bounds__(CGR_WAVES * 64, 4) void conv_dw_rows_kernel(ConvDwRowsArgs a)
{
    constexpr bool F32 = sizeof(XT) == 4;
    using AccT = typename std::conditional<F32, float, int32_t>::type;
    constexpr int CSB = F32 ? 65 * 4 : 68;                          // bytes per cell: 64 channels + padding against bank conflicts of the staging writes
    constexpr int RS = R * S;
    extern __shared__ uint4 cgr_lds[];
    if (a.gate.closed()) return;
    char *tile = (char *)cgr_lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cblocks = (a.C + 63) >> 6, kblocks = (a.K + CGR_KB - 1) / CGR_KB;
    int b = (int)blockIdx.x;
    const int cb = b % cblocks; b /= cblocks;
    const int kb = b % kblocks, split = b / kblocks;
    const int c0 = cb * 64, k0 = kb * CGR_KB + wave * CGR_PPW;
    const int u_a = split * a.units_per_split, u_b = min(u_a + a.units_per_split, a.units);
    const int PQ = a.P * a.Q, HW = a.H * a.Wd;

    const XT *Xb = (const XT *)a.X;

    AccT acc[CGR_PPW][RS];
#pragma unroll
    for (int pi = 0; pi < CGR_PPW; ++pi)
#pragma unroll
        for (int t = 0; t < RS; ++t) acc[pi][t] = 0;

    const uint32_t row_bytes = (uint32_t)(a.Wp * CSB);              // one tile row further
    const uint32_t lane_off = (uint32_t)(lane * (int)sizeof(XT));

    // A unit = (image, band of code rows).  Three steps per unit: its code dwords into registers, its band of X into the LDS
    // tile, the walk.  (Two tiles of half the size, the next unit staged by each wavefront as soon as its own walk is done, were
    // measured: equal where a whole image fits either way, 10 % slower where the band has to shrink.)
    uint32_t dw[CGR_PPW][CGR_MAX_LOADS];
    auto load_codes = [&](int u) {
        const int n = u / a.bands, band = u - n * a.bands;
        const int p0 = band * a.TH, p1 = min(a.P, p0 + a.TH);
        const int first = p0 * a.Q, start4 = first & ~3, lo = first - start4;      // bytes [lo, endb) of the loaded stretch are the band's
        const int endb = p1 * a.Q - start4, n_dw = (endb + 3) >> 2;
        (void)lo; (void)endb;
#pragma unroll
        for (int pi = 0; pi < CGR_PPW; ++pi) {
            const int k = min(k0 + pi, a.K - 1);                     // planes past the tensor repeat the last one; never walked
            const uint32_t *src = (const uint32_t *)(a.codes + ((int64_t)n * a.Kt + k) * PQ + start4);
#pragma unroll
            for (int j = 0; j < CGR_MAX_LOADS; ++j) dw[pi][j] = src[min(lane + 64 * j, n_dw - 1)];
        }
    };
    auto stage = [&](int u, char *tile) {
        const int n = u / a.bands, band = u - n * a.bands;
        const int h0 = band * a.TH * a.st - a.pad;                  // X row of tile row 0; tile column 0 is X column -pad
        // ---- stage: wavefront w brings channels 4w .. 4w+3, a lane the same cells of each: four 64-cell chunks x 4 channels =
        //      16 loads in flight (the loop is bound by their latency), the cells' geometry computed once per chunk ----
        constexpr int CPW = 64 / CGR_WAVES, IB = 4;
        const int ch0 = wave * CPW;
        const XT *xw = Xb + ((int64_t)n * a.Ct + min(c0 + ch0, a.C - 1)) * HW;           // uniform; channel j of the wavefront: + j*HW (clamped below)
        for (int i0 = 0; i0 < a.n_chunks; i0 += IB) {
            XT v[IB][CPW];
            uint32_t dst[IB];
            bool okc[IB];
#pragma unroll
            for (int ii = 0; ii < IB; ++ii) {
                const uint32_t t = (uint32_t)(lane + 64 * min(i0 + ii, a.n_chunks - 1));   // the tail repeats the last chunk
                const uint32_t tr = __umulhi(t, a.wp_magic), tc = t - tr * (uint32_t)a.Wp;
                const int h = h0 + (int)tr, w = (int)tc - a.pad;
                const bool in = t < (uint32_t)a.cells;
                okc[ii] = in && h >= 0 && h < a.H && w >= 0 && w < a.Wd;
                const int off = okc[ii] ? h * a.Wd + w : 0;
                dst[ii] = in ? t * (uint32_t)CSB + (uint32_t)(ch0 * (int)sizeof(XT)) : 0xFFFFFFFFu;
#pragma unroll
                for (int j = 0; j < CPW; ++j) v[ii][j] = xw[(int64_t)min(j, a.C - 1 - min(c0 + ch0, a.C - 1)) * HW + off];   // unconditional
            }
#pragma unroll
            for (int ii = 0; ii < IB; ++ii) {
                if (dst[ii] == 0xFFFFFFFFu) continue;
#pragma unroll
                for (int j = 0; j < CPW; ++j) {
                    const bool ok = okc[ii] && c0 + ch0 + j < a.C;
                    *(XT *)(tile + dst[ii] + j * (int)sizeof(XT)) = ok ? v[ii][j] : (XT)0;
                }
            }
        }
    };
    auto walk = [&](int u, const char *tile) {
        const int n = u / a.bands, band = u - n * a.bands;
        const int p0 = band * a.TH, p1 = min(a.P, p0 + a.TH);
        const int first = p0 * a.Q, start4 = first & ~3, lo = first - start4;      // bytes [lo, endb) of the loaded stretch are the band's
        const int endb = p1 * a.Q - start4, n_dw = (endb + 3) >> 2;
        (void)n;
        // ---- the wavefront's planes: nonzeros of the band's code rows p0 .. p1-1 ----
#pragma unroll
        for (int pi = 0; pi < CGR_PPW; ++pi) {
            const int k = k0 + pi;
            if (k >= a.K) break;                                     // uniform
#pragma unroll
            for (int j = 0; j < CGR_MAX_LOADS; ++j) {
                const int d = lane + 64 * j;
                uint32_t m = d < n_dw ? 0xFFFFFFFFu : 0u;            // stretches past the band are masked
                if (4 * d < lo) m &= 0xFFFFFFFFu << (8 * (lo - 4 * d));          // lo - 4d in 1..3 (d == 0 only)
                if (4 * d + 4 > endb && d < n_dw) m &= 0xFFFFFFFFu >> (8 * (4 * d + 4 - endb));
                dw[pi][j] &= m;
            }
#pragma unroll
            for (int j = 0; j < CGR_MAX_LOADS; ++j) {
                if (64 * j >= n_dw) break;                           // uniform
                uint64_t mask = __builtin_amdgcn_ballot_w64(dw[pi][j] != 0u);
                while (mask) {
                    const int l = __builtin_ctzll(mask);
                    mask &= mask - 1;
                    const uint32_t word = (uint32_t)__builtin_amdgcn_readlane((int)dw[pi][j], l);
                    const int pos0 = 4 * (l + 64 * j) - lo;          // the word's first byte, counted from the band's first code
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int code = (int)(int8_t)(word >> (8 * e));
                        if (code == 0) continue;                     // uniform
                        const uint32_t flat = (uint32_t)(pos0 + e);
                        const uint32_t pp = __umulhi(flat, a.q_magic), q = flat - pp * (uint32_t)a.Q;
                        const uint32_t cell = (pp * (uint32_t)a.st) * (uint32_t)a.Wp + q * (uint32_t)a.st;
                        const char *x0 = tile + cell * (uint32_t)CSB + lane_off;
                        if constexpr (F32) {
                            const float kf = (float)code;
#pragma unroll
                            for (int r = 0; r < R; ++r) {
                                const char *xr = x0 + r * row_bytes;
#pragma unroll
                                for (int s = 0; s < S; ++s) acc[pi][r * S + s] = fmaf(kf, *(const float *)(xr + s * CSB), acc[pi][r * S + s]);
                            }
                        } else {
#pragma unroll
                            for (int r = 0; r < R; ++r) {
                                const char *xr = x0 + r * row_bytes;
#pragma unroll
                                for (int s = 0; s < S; ++s) acc[pi][r * S + s] += code * (int)*(const int8_t *)(xr + s * CSB);
                            }
                        }
                    }
                }
            }
        }
    };
    for (int u = u_a; u < u_b; ++u) {
        load_codes(u);                                               // in flight while the tile is staged
        __syncthreads();                                             // the tile of the unit before has been read
        stage(u, tile);
        __syncthreads();
        walk(u, tile);
    }

    // ---- out: lane = channel c0 + lane of planes k0 .. k0+PPW-1 ----
    const int c = c0 + lane;
    if (c < a.C) {
        const float sc = a.n_split == 1 && F32 ? a.scale.get() : 1.0f;
        AccT *out = (AccT *)a.out + (int64_t)split * a.K * a.C * RS;
#pragma unroll
        for (int pi = 0; pi < CGR_PPW; ++pi) {
            const int k = k0 + pi;
            if (k >= a.K) break;
            AccT *o = out + ((int64_t)k * a.C + c) * RS;
#pragma unroll
            for (int t = 0; t < RS; ++t) {
                if constexpr (F32) o[t] = a.n_split == 1 ? acc[pi][t] * sc : acc[pi][t]; else o[t] = acc[pi][t];
            }
        }
    }
}

// dW = scale * sum of the shares (fp32: in a fixed order; int32: exact).  `zg` (a power of two, at most 16) threads share an
// element: thread group g adds the shares g, g + zg, ... in that order, eight loads in flight, and group 0 adds the groups'
// sums in group order -- with hundreds of shares of a small dW one thread per element would be a chain of dependent loads.
template <class AccT>
__global__ __launch_bounds__(256) void conv_dw_rows_reduce_kernel(const AccT *partial, AccT *dW, int64_t n, int n_split, int zg, Scale scale, Gate gate)
{
    if (gate.closed()) return;
    __shared__ AccT part[256];
    const int epb = 256 / zg, e = (int)threadIdx.x & (epb - 1), g = (int)threadIdx.x / epb;
    for (int64_t base = (int64_t)blockIdx.x * epb; base < n; base += (int64_t)gridDim.x * epb) {     // uniform trip count: barriers inside
        const int64_t i = base + e;
        AccT s = 0;
        if (i < n) {
            int z = g;
            for (; z + 7 * zg < n_split; z += 8 * zg) {
                AccT v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = partial[(int64_t)(z + j * zg) * n + i];
#pragma unroll
                for (int j = 0; j < 8; ++j) s += v[j];
            }
            for (; z < n_split; z += zg) s += partial[(int64_t)z * n + i];
        }
        if (zg > 1) {
            part[threadIdx.x] = s;
            __syncthreads();
            if (g == 0)
                for (int j = 1; j < zg; ++j) s += part[j * epb + e];
            __syncthreads();                                          // the next round overwrites part
        }
        if (g == 0 && i < n) {
            if constexpr (std::is_same<AccT, float>::value) dW[i] = s * scale.get(); else dW[i] = s;
        }
    }
}

// ---- dX ------------------------------------------------------------------------------------------------------------------
constexpr int CGR_KC = 8;                          // dX: code planes per chunk
constexpr int CGR_DX_CPT = 4;                      // dX: code dwords a thread stages per chunk, at most

struct ConvDxRowsArgs {
    const int8_t *codes;              // plane (n, k) at codes + (n*Kt + k) * P*Q; 4-byte aligned, P*Q a multiple of 4
    const float  *Wt;                 // prepared weights [Kp][R*S][Cp]: K rounded up to a chunk of planes, C to 64, zero padded
    float        *dX;                 // [N][Ct][H][Wd]
    int N, C, K, H, Wd, P, Q, pad, Ct, Kt, Cp;
    int TH, bands, Wp;                // output rows per workgroup; bands per image; cells per row = Q + S - 1 (cell t = w + pad)
    int cb_words;                     // dwords of one plane's stretch in LDS (the code rows that reach the band, rounded)
    uint32_t cbw_magic, wd_magic, q_magic;   // floor(2^32 / x) + 1 for x = cb_words, Wd, Q: y / x == mulhi(y, magic) for y < 2^16
    Scale scale;
    Gate gate;
};

// W [K][C][R*S] -> [Kp][R*S][Cp]
__global__ __launch_bounds__(256) void conv_dx_rows_prep_kernel(const float *W, float *Wt, int K, int Kp, int C, int RS, int Cp, Gate gate)
{
    if (gate.closed()) return;
    const int64_t total = (int64_t)Kp * RS * Cp;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int c = (int)(i % Cp);
        const int64_t t = i / Cp;
        const int rs = (int)(t % RS), k = (int)(t / RS);
        Wt[i] = c < C && k < K ? W[((int64_t)k * C + c) * RS + rs] : 0.0f;
    }
}

// The reduction runs over chunks of CGR_KC code planes.  All threads bring a chunk's weights [plane][tap][64 channels] and its
// code stretches into LDS (loads of chunk i+1 are issued before chunk i is walked and written to the other buffer after it: one
// barrier per chunk); a wavefront then reads, per plane, the R code rows that reach its output row (lane l: dword l of the
// row), and only for rows with a nonzero its channel's S weights.  Per nonzero and tap: read the cell, multiply-add, write it
// back -- LDS operations of one wavefront execute in order and a cell belongs to one wavefront, so no atomics (LDS float
// atomics were measured at 170 cycles per instruction).
// NT threads (256, 512 or 1024 >= 64 * TH): wavefronts beyond the band's rows only help to stage.
template <int R, int S, int NT>
__global__ __launch_bounds__(NT) void conv_dx_rows_kernel(ConvDxRowsArgs a)
{
    constexpr int RS = R * S, CSW = 65;                              // words per cell
    constexpr int WCH = CGR_KC * RS * 64;                            // floats of a chunk's weights
    constexpr int WPT = (WCH + NT - 1) / NT;
    constexpr int CGR_DX_RING = 3;                                   // chunks in flight from global memory
    constexpr int nthreads = NT;
    extern __shared__ uint4 cgr_lds[];
    if (a.gate.closed()) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cblocks = a.Cp >> 6;
    int b = (int)blockIdx.x;
    const int cb = b % cblocks; b /= cblocks;
    const int band = b % a.bands, n = b / a.bands;
    const int c0 = cb * 64, h_first = band * a.TH, rows = min(a.TH, a.H - h_first);
    const int PQ = a.P * a.Q, HW = a.H * a.Wd;
    const int row_words = a.Wp * CSW, acc_words = a.TH * row_words;
    const int cwords = CGR_KC * a.cb_words;                          // dwords of a chunk's codes
    float *accs = (float *)cgr_lds;                                  // [TH rows][Wp cells][65]
    float *wbuf = accs + acc_words;                                  // [2][WCH]
    uint32_t *cbuf = (uint32_t *)(wbuf + 2 * WCH);                   // [2][cwords]

    for (int i = tid; i < acc_words; i += nthreads) accs[i] = 0.0f;

    // the code rows that reach the band: p = h + pad - r
    const int pa = max(h_first + a.pad - (R - 1), 0), pb = min(h_first + rows - 1 + a.pad, a.P - 1);
    const int start4 = (pa * a.Q) & ~3;
    const int n_dw = pb >= pa ? ((pb + 1) * a.Q - start4 + 3) >> 2 : 0;              // <= cb_words (host)
    const int8_t *img = a.codes + (int64_t)n * a.Kt * PQ + start4;
    const int n_chunks = (a.K + CGR_KC - 1) / CGR_KC;

    // chunks on their way: a ring of CGR_DX_RING register sets (chunk j in set j % RING until it is written to LDS)
    // (nothing touches a loaded value before it is written to LDS: an instruction on it would make the wavefront wait for the
    // load right away; which code dwords are real is kept as a bit mask beside them).  A thread's places in a chunk are the
    // same for every chunk: offsets from the chunk's (uniform) first weight row and first code plane, computed once.
    uint32_t woff[WPT], coff[CGR_DX_CPT], ckk[CGR_DX_CPT];
    uint32_t cval = 0;                                               // bit j: code dword j of this thread lies inside the stretch
#pragma unroll
    for (int j = 0; j < WPT; ++j) {
        const int i = min(tid + nthreads * j, WCH - 1);
        woff[j] = (uint32_t)((i >> 6) * a.Cp + (i & 63));            // (the prepared weights are padded to whole chunks of planes)
    }
#pragma unroll
    for (int j = 0; j < CGR_DX_CPT; ++j) {
        const uint32_t i = (uint32_t)min(tid + nthreads * j, cwords - 1);
        const uint32_t kk = __umulhi(i, a.cbw_magic), d = i - kk * (uint32_t)a.cb_words;
        const bool in = (int)d < n_dw;
        ckk[j] = kk; coff[j] = in ? kk * (uint32_t)PQ + 4 * d : 0u;
        cval |= in ? 1u << j : 0u;
    }
    float wreg[CGR_DX_RING][WPT];
    uint32_t creg[CGR_DX_RING][CGR_DX_CPT], cok[CGR_DX_RING];
    auto fetch = [&](int chunk_in, float (&wr)[WPT], uint32_t (&cr)[CGR_DX_CPT], uint32_t &okm) {
        const int kbase = min(chunk_in, n_chunks - 1) * CGR_KC;      // past the end: the last chunk again, never used
        const float *wsrc = a.Wt + c0 + (int64_t)kbase * RS * a.Cp;  // uniform
        const int8_t *csrc = img + (int64_t)kbase * PQ;              // uniform
        const uint32_t k_left = (uint32_t)(a.K - kbase);             // planes of the chunk inside the tensor
#pragma unroll
        for (int j = 0; j < WPT; ++j) wr[j] = wsrc[woff[j]];
        okm = 0u;
#pragma unroll
        for (int j = 0; j < CGR_DX_CPT; ++j) {
            const bool ok = ((cval >> j) & 1u) && ckk[j] < k_left;
            cr[j] = *(const uint32_t *)(csrc + (ok ? coff[j] : 0u));
            okm |= ok ? 1u << j : 0u;
        }
    };
    auto commit = [&](int buf, const float (&wr)[WPT], const uint32_t (&cr)[CGR_DX_CPT], uint32_t okm) {
        float *wd = wbuf + buf * WCH;
        uint32_t *cd = cbuf + buf * cwords;
#pragma unroll
        for (int j = 0; j < WPT; ++j)
            if (tid + nthreads * j < WCH) wd[tid + nthreads * j] = wr[j];
#pragma unroll
        for (int j = 0; j < CGR_DX_CPT; ++j)
            if (tid + nthreads * j < cwords) cd[tid + nthreads * j] = (okm >> j) & 1u ? cr[j] : 0u;
    };

    // This wavefront's output row h and the code rows that reach it, p = h + pad - r: consecutive rows, i.e. one run of bytes of
    // the plane's stretch.  Lane l looks at dword d_lo + l (+ 64 per further pass) of it; bytes of other rows are masked (fixed
    // for the kernel).
    constexpr int NRD = (R * 253 + 6 + 255) / 256;                   // passes of 64 dwords over R rows of at most 253 codes
    const bool active = wave < rows;
    const int h = h_first + min(wave, rows - 1);
    float *mine = accs + min(wave, a.TH - 1) * row_words + lane;     // cell t of this row and lane: mine[t * 65]
    const int p_top = max(h + a.pad - (R - 1), pa), p_bot = min(h + a.pad, pb);
    const bool any_rows = active && p_bot >= p_top;
    const int b_lo = (any_rows ? p_top * a.Q : pa * a.Q) - start4, b_hi = (any_rows ? (p_bot + 1) * a.Q : pa * a.Q) - start4;
    const int d_lo = b_lo >> 2, nd = any_rows ? ((b_hi + 3) >> 2) - d_lo : 0;
    const int passes = (nd + 63) >> 6;
    const int rel0 = start4 - pa * a.Q;                              // byte f of the stretch is code rel0 + f, counted from row pa (rel0 in -3..0)
    uint32_t bmask[NRD];
#pragma unroll
    for (int it = 0; it < NRD; ++it) {
        const int d = d_lo + lane + 64 * it;
        uint32_t m = lane + 64 * it < nd ? 0xFFFFFFFFu : 0u;
        if (4 * d < b_lo) m &= 0xFFFFFFFFu << (8 * min(b_lo - 4 * d, 3));
        if (4 * d + 4 > b_hi && lane + 64 * it < nd) m &= 0xFFFFFFFFu >> (8 * min(4 * d + 4 - b_hi, 3));
        bmask[it] = m;
    }

#pragma unroll
    for (int sl = 0; sl < CGR_DX_RING; ++sl) fetch(sl, wreg[sl], creg[sl], cok[sl]);
    commit(0, wreg[0], creg[0], cok[0]);
    __syncthreads();
    for (int chunk0 = 0; chunk0 < n_chunks; chunk0 += CGR_DX_RING) {
#pragma unroll
        for (int sl = 0; sl < CGR_DX_RING; ++sl) {
            const int chunk = chunk0 + sl;
            if (chunk >= n_chunks) break;                            // uniform
            const int buf = chunk & 1;
            // this chunk is in LDS, its register set takes chunk + RING
            fetch(chunk + CGR_DX_RING, wreg[sl], creg[sl], cok[sl]);
            if (any_rows) {
                const float *wc = wbuf + buf * WCH + lane;
                const uint32_t *cc = cbuf + buf * cwords + d_lo;
                // the chunk's planes pass by pass: all eight reads first (the walk's LDS writes would keep a later read behind them)
#pragma unroll
                for (int it = 0; it < NRD; ++it) {
                    if (it >= passes) break;                         // uniform
                    uint32_t cws[CGR_KC];
#pragma unroll
                    for (int kk = 0; kk < CGR_KC; ++kk) cws[kk] = cc[kk * a.cb_words + min(lane + 64 * it, nd - 1)] & bmask[it];
#pragma unroll
                    for (int kk = 0; kk < CGR_KC; ++kk) {
                        const uint32_t cw = cws[kk];
                        uint64_t mask = __builtin_amdgcn_ballot_w64(cw != 0u);
                        while (mask) {
                            const int l = __builtin_ctzll(mask);
                            mask &= mask - 1;
                            const uint32_t word = (uint32_t)__builtin_amdgcn_readlane((int)cw, l);
                            const uint32_t f0 = (uint32_t)(rel0 + 4 * (d_lo + l + 64 * it));   // the word's first byte, counted from row pa's first code
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const int code = (int)(int8_t)(word >> (8 * e));
                                if (code == 0) continue;             // uniform
                                const uint32_t f = f0 + (uint32_t)e;                 // (a masked byte is zero: f is a real code's place)
                                const uint32_t pr = __umulhi(f, a.q_magic), q = f - pr * (uint32_t)a.Q;
                                const int r = h + a.pad - (pa + (int)pr);            // 0 .. R-1
                                const float kf = (float)code;
                                const float *wk = wc + (kk * RS + r * S) * 64;
                                float *cell = mine + q * CSW;        // w + pad = q + s: cells q .. q+S-1
                                float w[S], cur[S];
#pragma unroll
                                for (int s2 = 0; s2 < S; ++s2) { w[s2] = wk[s2 * 64]; cur[s2] = cell[s2 * CSW]; }
#pragma unroll
                                for (int s2 = 0; s2 < S; ++s2) cell[s2 * CSW] = fmaf(kf, w[s2], cur[s2]);
                            }
                        }
                    }
                }
            }
            // chunk + 1 (loaded RING - 1 iterations ago) goes to the other buffer
            const int nx = (sl + 1) % CGR_DX_RING;
            if (chunk + 1 < n_chunks) commit(buf ^ 1, wreg[nx], creg[nx], cok[nx]);
            __syncthreads();
        }
    }

    // ---- out: a channel's rows of the band are contiguous in dX: lanes along them, channels dealt to the wavefronts ----
    const float sc = a.scale.get();
    const int nw = nthreads >> 6, nc = min(64, a.C - c0), band_px = rows * a.Wd;
    float *out = a.dX + ((int64_t)n * a.Ct + c0) * HW + h_first * a.Wd;
    for (int ch = wave; ch < nc; ch += nw) {
        float *dst = out + (int64_t)ch * HW;
        for (int i = lane; i < band_px; i += 64) {
            const uint32_t row = __umulhi((uint32_t)i, a.wd_magic), w = (uint32_t)i - row * (uint32_t)a.Wd;
            dst[i] = sc * accs[(row * (uint32_t)a.Wp + w + (uint32_t)a.pad) * CSW + ch];
        }
    }
}

}  // namespace dbp
