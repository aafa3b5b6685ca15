// Weight-gradient product of a 3x3, stride-1, padding-1 convolution in the 8-bit mode (int8 codes x int8
// activations, exact int32), the convolutional analogue of Eq. (qdw):
//   dW[k,c,r,s] = sum_{n,h,w} code[n,k,h-r+1,w-s+1] * X[n,c,h,w]
// Same organisation as conv_dw_kernel.h (pitched pixel coordinates, one accumulator per tap, units of whole
// image rows, four multiplying and four staging wavefronts, double-buffered LDS, split over units with a
// deterministic reduction), with a data layout made for what limits the int8 kernel there: vector-ALU work
// of a multiplying wavefront is not hidden behind its own matrix-core instructions, and a one-pixel shift of a
// 16-byte fragment cost four byte-align instructions per tap.
//
//   * A 16-byte LDS cell holds 16 consecutive pixels of a pitched row (pitch PW, a multiple of 16, at least
//     Wd + 1 so that zero columns separate the rows) in TRANSPOSED order: dword d = pixels d, d+4, d+8, d+12.
//     Both operands use it, so the products pair up as before.  A fragment moved by one pixel is then the same
//     cell with its dwords rotated and ONE dword replaced by a byte-align of two dwords:
//       +1 pixel:  {y, z, w, align(next.x, x, 1)}        -1 pixel:  {align(w, prev.w, 3), x, y, z}
//     and since the order of the 16 reduction slots is free as long as both operands agree, the rotation is
//     applied to the activation fragment instead (once per step, for all rows of taps): a tap costs one
//     byte-align in place and, for one of the two shifted taps, a saved and restored dword.
//   * The stagers load 16 pixels with one 16-byte load (dword aligned: Wd % 4 == 0), transpose them with eight
//     byte-permutes and write one cell: 16 loads per thread and unit instead of 48 four-byte ones (a wavefront's
//     load instruction costs the address unit 16 cycles whether it moves 256 bytes or a kilobyte).  A row's last
//     cell that is only partly inside the row is loaded from 16 bytes that end at the row's end and moved into
//     place (the bytes behind the row are zero columns).
#pragma once
#include "conv_dw_kernel.h"
#include "fc2_i8_kernel.h"

namespace dbp {

struct ConvDwI8Args {
    const int8_t *codes;       // [N][K][H][Wd]   (P = H, Q = Wd)
    const int8_t *X;           // [N][C][H][Wd]
    int32_t      *dW;          // [K][C][3][3]
    int32_t      *partial;     // [tile][split][tap][v/4][thread][v%4] (n_split > 1), as conv_dw_reduce_kernel reads it
    int N, C, H, Wd, K;
    int Ct, Kt;                // channels of the tensors that hold X and the codes (C, K unless this is one group's block)
    int PW, CPR, DC;           // row pitch (pixels), cells per pitched row, cells of a row that hold pixels
    int RU, chunks;            // image rows per unit; units per image
    int units, units_per_split, n_split, tiles_k, tiles_c;
    int xcells, ccells;        // LDS cells per channel: activations (RU*CPR, odd), codes ((RU+2)*CPR + 2, odd)
    int n_steps;               // RU*CPR/2 matrix-core steps of 32 pixels per unit
    int xpairs, cpairs;        // (row, cell) pairs a unit loads per channel: RU*DC, (RU+2)*DC
    int lds_cells;
    Gate gate;
};

__global__ __launch_bounds__(512, 1) void conv_dw_i8_kernel(ConvDwI8Args a)
{
    constexpr int TK = 64, TC = 64, RS = 9;
    extern __shared__ uint4 cdw_lds[];
    if (a.gate.closed()) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool stager = wave >= 4;
    const int tid = threadIdx.x & 255;
    const int lcol = lane & 31, lhalf = lane >> 5;
    const int wr = (wave & 3) >> 1, wcl = wave & 1;
    const int tiles = a.tiles_k * a.tiles_c;
    // Workgroup w runs on XCD w % 8, and each XCD has an L2 of its own: renumber so that the tiles of one split (which
    // read the same images at about the same time, each operand tile shared by a row or column of tiles) sit on one XCD.
    const int wg = (gridDim.x & 7) == 0 ? (int)((blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) : (int)blockIdx.x;
    const int tile = wg % tiles, split = wg / tiles;
    const int k0 = (tile % a.tiles_k) * TK, c0 = (tile / a.tiles_k) * TC;
    const int unit_a = split * a.units_per_split, unit_b = min(unit_a + a.units_per_split, a.units);
    const int n_units = unit_b - unit_a;
    const int PI = a.H * a.Wd;
    const uint32_t x_cells_buf = (uint32_t)(TC * a.xcells), buf_cells = x_cells_buf + (uint32_t)(TK * a.ccells);

    for (int i = threadIdx.x; i < a.lds_cells; i += 512) cdw_lds[i] = uint4{0u, 0u, 0u, 0u};

    if (stager) {
        // ---- fixed for the kernel: this thread's (row, cell) pair of each operand, its LDS cell, its offset inside the
        // rows of a tile's first channel, and how a partly filled cell is moved into place.  Passes walk the channels.
        const uint32_t dump = (2u * buf_cells + (uint32_t)tid) * 16u;        // a cell of its own for writes that have no place
        const int xch = tid / a.xpairs, xpr = tid - xch * a.xpairs, XCH = 256 / a.xpairs;
        const bool x_own = xch < XCH;
        const int xrow = xpr / a.DC, xcell = xpr - xrow * a.DC;
        const int xsh = (16 - min(16, a.Wd - 16 * xcell)) >> 2;              // dwords by which the cell's load starts early
        const int x_row0 = xrow * a.Wd + 16 * xcell - 4 * xsh;
        const int x_passes = (TC + XCH - 1) / XCH;
        const uint32_t x_l0 = x_own ? (uint32_t)(xch * a.xcells + xrow * a.CPR + xcell) * 16u : dump;
        const uint32_t x_ls = x_own ? (uint32_t)(XCH * a.xcells) * 16u : 0u;
        const uint32_t x_llast = x_own && xch + XCH * (x_passes - 1) < TC ? x_l0 + (uint32_t)(x_passes - 1) * x_ls : dump;
        const uint32_t xm1 = xsh & 1 ? 0xFFFFFFFFu : 0u, xm2 = xsh & 2 ? 0xFFFFFFFFu : 0u;
        const int x_chmax = min(a.C - c0, TC) - 1;                           // channels past it: the loads repeat it, the results are never stored

        const int cch = tid / a.cpairs, cpr = tid - cch * a.cpairs, CCH = 256 / a.cpairs;
        const bool c_own = cch < CCH;
        const int crow = cpr / a.DC, ccell = cpr - crow * a.DC;
        const int csh = (16 - min(16, a.Wd - 16 * ccell)) >> 2;
        const int c_row0 = crow * a.Wd + 16 * ccell - 4 * csh;               // from the patch's first row, the one above the unit's rows
        const int c_passes = (TK + CCH - 1) / CCH;
        const uint32_t c_l0 = c_own ? (x_cells_buf + (uint32_t)(cch * a.ccells + 1 + crow * a.CPR + ccell)) * 16u : dump;
        const uint32_t c_ls = c_own ? (uint32_t)(CCH * a.ccells) * 16u : 0u;
        const uint32_t c_llast = c_own && cch + CCH * (c_passes - 1) < TK ? c_l0 + (uint32_t)(c_passes - 1) * c_ls : dump;
        const uint32_t cm1 = csh & 1 ? 0xFFFFFFFFu : 0u, cm2 = csh & 2 ? 0xFFFFFFFFu : 0u;
        const int c_chmax = min(a.K - k0, TK) - 1;

        constexpr int XI = 16, CI = 16;                                      // most passes (the host keeps to them)
        u32x4 xr[XI], cr[CI];

        auto issue = [&](int unit) {
            const int n = unit / a.chunks, h_a = (unit - n * a.chunks) * a.RU;
            const int8_t *xb = a.X + ((int64_t)n * a.Ct + c0) * PI + (int64_t)h_a * a.Wd;             // uniform
            // the patch starts a row above the unit's rows: offsets from there are never negative (the address itself may
            // lie in front of the tensor for the first unit, whose row above is not read)
            const int8_t *cb = a.codes + ((int64_t)n * a.Kt + k0) * PI + ((int64_t)h_a - 1) * a.Wd;   // uniform
            // rows outside the image read the first 16 bytes of the unit's first row in the tile's first channel and are
            // cleared when staged
            const bool x_ld = x_own && h_a + xrow < a.H;
            const bool c_ld = c_own && h_a - 1 + crow >= 0 && h_a - 1 + crow < a.H;
            uint32_t xo = x_ld ? (uint32_t)(xch * PI + x_row0) : 0u, co = c_ld ? (uint32_t)(cch * PI + c_row0) : (uint32_t)a.Wd;
            const uint32_t xs = x_ld ? (uint32_t)(XCH * PI) : 0u, cs = c_ld ? (uint32_t)(CCH * PI) : 0u;
            const uint32_t xcap = x_ld ? (uint32_t)(x_chmax * PI + x_row0) : 0u, ccap = c_ld ? (uint32_t)(c_chmax * PI + c_row0) : (uint32_t)a.Wd;
#pragma unroll
            for (int j = 0; j < CI; ++j) {
                if (j >= c_passes) break;
                cr[j] = *(const u32x4_dw *)(cb + min(co, ccap));
                co += cs;
            }
#pragma unroll
            for (int j = 0; j < XI; ++j) {
                if (j >= x_passes) break;
                xr[j] = *(const u32x4_dw *)(xb + min(xo, xcap));
                xo += xs;
            }
        };

        // 16 loaded bytes -> one cell: a partly filled cell's load started sh dwords early (pixel dword d is loaded dword
        // d + sh, dwords past the row are zero); rows outside the image are cleared; then "dword d = pixels d, d+4, d+8, d+12"
        // (rows that fill whole cells have sh = 0, m1 = take2 = 0, take0 = the row's validity mask: the same arithmetic gives v & that mask.  A run-time
        // test for them inside the loop over the passes was two taken branches per cell.)
        auto make_cell = [&](const u32x4 &v, uint32_t m1, uint32_t take2, uint32_t take0) {
            const uint32_t u0 = (v.y & m1) | (v.x & ~m1), u1 = (v.z & m1) | (v.y & ~m1), u2 = (v.w & m1) | (v.z & ~m1), u3 = v.w & ~m1;
            const uint32_t w0 = (u2 & take2) | (u0 & take0), w1 = (u3 & take2) | (u1 & take0), w2 = u2 & take0, w3 = u3 & take0;
            uint32_t o[4];
            fc2i_transpose(w0, w1, w2, w3, o);
            return uint4{o[0], o[1], o[2], o[3]};
        };

        auto stage = [&](int unit, uint32_t buf) {
            const int n = unit / a.chunks, h_a = (unit - n * a.chunks) * a.RU;
            char *lds = (char *)cdw_lds + buf * buf_cells * 16u;
            const uint32_t xok = h_a + xrow < a.H ? 0xFFFFFFFFu : 0u;
            const uint32_t cok = (h_a - 1 + crow >= 0 && h_a - 1 + crow < a.H) ? 0xFFFFFFFFu : 0u;
            const uint32_t xt2 = xm2 & xok, xt0 = ~xm2 & xok, ct2 = cm2 & cok, ct0 = ~cm2 & cok;
            uint32_t cell = x_l0;
#pragma unroll
            for (int j = 0; j < XI; ++j) {
                if (j >= x_passes) break;
                *(uint4 *)(lds + (j == x_passes - 1 ? x_llast : cell)) = make_cell(xr[j], xm1, xt2, xt0);
                cell += x_ls;
            }
            cell = c_l0;
#pragma unroll
            for (int j = 0; j < CI; ++j) {
                if (j >= c_passes) break;
                *(uint4 *)(lds + (j == c_passes - 1 ? c_llast : cell)) = make_cell(cr[j], cm1, ct2, ct0);
                cell += c_ls;
            }
        };

        // Barriers: one after the clearing of LDS, one after the first unit is staged, one per unit (the multipliers
        // execute the same number).
        if (n_units > 0) issue(unit_a);
        __syncthreads();
        if (n_units > 0) stage(unit_a, 0u);
        if (n_units > 1) issue(unit_a + 1);
        __syncthreads();
        for (int i = 0; i < n_units; ++i) {
            if (i + 1 < n_units) {
                stage(unit_a + i + 1, (uint32_t)((i + 1) & 1));
                if (i + 2 < n_units) issue(unit_a + i + 2);
            }
            __syncthreads();
        }
        return;
    }

    // ================================ multipliers ================================
    i32x16 acc[RS];
#pragma unroll
    for (int t = 0; t < RS; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0;

    // per-lane cells of step 0: activations of channel c0 + 32*wcl + lcol, codes of channel k0 + 32*wr + lcol (tap row
    // r reads (2 - r) pitched rows further on; +1 for the margin cell in front of the patch)
    const uint32_t x_lane = (uint32_t)((wcl * 32 + lcol) * a.xcells + lhalf);
    const uint32_t c_lane = x_cells_buf + (uint32_t)((wr * 32 + lcol) * a.ccells + 1 + lhalf);
    // A lane walks a stream of cells: step j uses cell 2j + lhalf ("cur") and, for the shifted taps, one dword of each
    // neighbour.  The cell after cur is the cell before cur of the next step, so it is read once: its first dword now,
    // its last dword carried to the next step.
    struct Frags { uint4 x; uint4 cur[3], next[3]; };
    uint32_t before_w[3];                                                            // last dword of the cell in front of cur
    auto load_frags = [&](uint32_t buf, int step, Frags &f) {
        const uint4 *b = cdw_lds + buf * buf_cells + 2 * step;
        f.x = b[x_lane];
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const uint4 *p = b + c_lane + (2 - r) * a.CPR;
            f.cur[r] = p[0]; f.next[r] = p[1];
        }
    };
    auto multiply = [&](Frags &f) {
        const u32x4 xb = u32x4{f.x.x, f.x.y, f.x.z, f.x.w};
        const u32x4 xr1 = u32x4{f.x.w, f.x.x, f.x.y, f.x.z};      // pairs with {align(next.x, x, 1), y, z, w}: codes moved by +1 pixel
        const u32x4 xr2 = u32x4{f.x.y, f.x.z, f.x.w, f.x.x};      // pairs with {x, y, z, align(w, before.w, 3)}: codes moved by -1 pixel
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            // the whole neighbour cell counts as used: two of its dwords read separately would be LDS reads of one dword
            // with lanes a whole number of cells apart, which collide four at a time in the banks
            asm volatile("" : "+v"(f.next[r].x), "+v"(f.next[r].y), "+v"(f.next[r].z), "+v"(f.next[r].w));
            u32x4 c = u32x4{f.cur[r].x, f.cur[r].y, f.cur[r].z, f.cur[r].w};
            Mma<MODE_I8>::run(c, xb, acc[r * 3 + 1]);                                   // s = 1: code column q = w
            const uint32_t keep = c.x;
            c.x = __builtin_amdgcn_alignbyte(f.next[r].x, keep, 1);
            Mma<MODE_I8>::run(c, xr1, acc[r * 3 + 0]);                                  // s = 0: q = w + 1
            c.x = keep;
            c.w = __builtin_amdgcn_alignbyte(c.w, before_w[r], 3);
            Mma<MODE_I8>::run(c, xr2, acc[r * 3 + 2]);                                  // s = 2: q = w - 1
            before_w[r] = f.next[r].w;
        }
    };

    __syncthreads();
    __syncthreads();
    for (int i = 0; i < n_units; ++i) {
        const uint32_t cur = (uint32_t)(i & 1);
        Frags fa, fb;
        load_frags(cur, 0, fa);
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            uint4 b = cdw_lds[cur * buf_cells + c_lane + (2 - r) * a.CPR - 1];
            asm volatile("" : "+v"(b.x), "+v"(b.y), "+v"(b.z), "+v"(b.w));          // read as one cell (see multiply)
            asm volatile("" : "+v"(fa.cur[r].x), "+v"(fa.cur[r].y), "+v"(fa.cur[r].z), "+v"(fa.cur[r].w));
            before_w[r] = b.w;
        }
        // the loads of the loop body are unconditional (the last one repeats the last step): with a load on only some
        // paths the compiler waits for all LDS loads in flight where it has to wait for one
        int step = 0;
        for (; step + 2 <= a.n_steps; step += 2) {
            load_frags(cur, step + 1, fb);
            multiply(fa);
            load_frags(cur, min(step + 2, a.n_steps - 1), fa);
            multiply(fb);
        }
        if (step < a.n_steps) multiply(fa);
        __syncthreads();
    }

    // ---- results: lane holds column c = lcol, rows k = 8*(v/4) + 4*lhalf + v%4 of its 32x32 block ----
    const int mtid = threadIdx.x;                                                      // 0..255
    if (a.n_split > 1) {
        typedef int32_t I4 __attribute__((ext_vector_type(4)));
        I4 *dst = (I4 *)a.partial + ((int64_t)tile * a.n_split + split) * (RS * 4) * 256 + mtid;
#pragma unroll
        for (int t = 0; t < RS; ++t)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq)
                dst[(t * 4 + vq) * 256] = I4{acc[t][4 * vq], acc[t][4 * vq + 1], acc[t][4 * vq + 2], acc[t][4 * vq + 3]};
    } else {
        const int c = c0 + wcl * 32 + lcol;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = k0 + wr * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
            if (k < a.K && c < a.C) {
#pragma unroll
                for (int t = 0; t < RS; ++t) a.dW[((int64_t)k * a.C + c) * RS + t] = acc[t][v];
            }
        }
    }
}

}  // namespace dbp
