// Weight-gradient product of a stride-1 convolution from int8 codes, the convolutional analogue of Eq. (qdw):
//   dW[k,c,r,s] = Delta * sum_{n,h,w} code[n,k,h-r+pad,w-s+pad] * X[n,c,h,w]
// (the sum written over input pixels).  fp32 X runs on bf16 matrix cores with the bf16x3 split; int8 X
// (8-bit mode) on int8 matrix cores with an exact int32 result.
//
// The reduction runs over pixels, which are contiguous in memory for both operands, so a lane's fragment
// is a run of 8 (bf16) or 16 (int8) consecutive pixels.  The activation fragment of a run is loaded once
// and multiplied with R*S code fragments, one per tap; each tap has its own accumulator, so a wavefront
// produces dW[32 k][32 c][all taps] and never re-reads X for another tap.
//
//   * "Pitched" pixel coordinates: image rows are laid out with pitch PW (a multiple of 8, wide enough
//     that the zero columns between two rows serve as the padding of both).  In these coordinates the code
//     a tap needs for pixel u sits at u + T(r,s) with a constant T, so a tap's fragment is the same run of
//     the code patch moved by T pixels.  T is not a multiple of the fragment length: the fragment is
//     cut out of two aligned 16-byte LDS cells with byte-align instructions.
//   * A workgroup (2x2 wavefronts, one per CU: the accumulators of nine taps leave no room for two) owns
//     a (64*MB) k x 64 c tile of dW for all taps and walks "units" = (image, RU whole image rows).  Per
//     unit it stages the X rows (split into bf16 planes once, for all four wavefronts) and the code patch (the rows plus the taps' reach) in LDS.  Global loads are aligned
//     16-byte / 4-byte pieces of the contiguous row range, scattered into pitched positions; positions no
//     pixel maps to (the zero columns) are cleared once and never written.  The padding is a template parameter: the
//     byte offset of every tap inside its LDS cell is then a constant and the phase is straight-line code.
//   * The reduction is split over units across workgroups; partial sums are written in thread order and
//     added in split order by conv_dw_reduce_kernel (deterministic), which also scatters into [K][C][R][S].
#pragma once
#include <type_traits>
#include "gemm_core.h"

namespace dbp {

constexpr int CDW_M8 = 8;              // pixels of margin in front of the code patch (reach of the widest tap)
constexpr int CDW_MAX_LDS = 144 * 1024; // one workgroup per CU; leaves room for the runtime's own use
constexpr int CDW_OFFR = 8;            // rows added before a division so that it never sees a negative number

struct ConvDwArgs {
    const int8_t *codes;       // [N][K][P][Q]
    const void   *X;           // [N][C][H][Wd] fp32 or int8
    void         *dW;          // [K][C][R][S] fp32 or int32
    void         *partial;     // [tile][split][element][256] (n_split > 1)
    int N, C, H, Wd, K, P, Q, pad;
    int Ct, Kt;                // channels of the tensors that hold X and the codes (C, K unless this is one group's block)
    int PW;                    // row pitch in pitched coordinates
    int RU, TPc, chunks;       // image rows per unit; RU*PW; units per image
    int units, units_per_split, n_split;
    int tiles_k, tiles_c;
    int pitchX, pitchC, lenC;  // LDS row pitches (elements) and code patch length (elements, multiple of 4)
    int NR;                    // code rows that a unit's patch overlaps
    int nqx, nqc;              // aligned 4-element pieces per channel that a unit loads (X, codes; c8: pieces of 8 codes)
    int c8;                    // bf16 modes, code rows of whole 8-code pieces (Q % 8 == 0): the whole-piece path loads the codes 8 bytes at a time
    int xshift, cshift;        // stagers: 2^shift threads along the pieces (>= nq), 256 >> shift channels at a time
    int row4x, row4c;          // Wd % 4 == 0 / Q % 4 == 0: a piece never straddles rows -> one wide LDS write
    int row2x, row2c;          // Wd, Q even: at least its halves never do
    int lds_cells;             // 16-byte cells of LDS in use
    Scale scale;
    Gate gate;
};

template <int I, int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) { f(std::integral_constant<int, I>{}); static_for<I + 1, N>(f); }
}

template <int MODE> struct CdwTraits;
template <> struct CdwTraits<MODE_BF16> { using XT = float;  using XRaw = uint4;    using Acc = f32x16; using AccT = float;   static constexpr int PLANES = 3, ESZ = 2, FRAG = 8; };
template <> struct CdwTraits<MODE_BF16X2> { using XT = float; using XRaw = uint4;   using Acc = f32x16; using AccT = float;   static constexpr int PLANES = 2, ESZ = 2, FRAG = 8; };
template <> struct CdwTraits<MODE_I8>   { using XT = int8_t; using XRaw = uint32_t; using Acc = i32x16; using AccT = int32_t; static constexpr int PLANES = 1, ESZ = 1, FRAG = 16; };

// The bf16 planes of two fp32 values, least significant plane first, packed (`a` in the low half of each word): three exact
// planes, or two rounded to nearest.
template <int PL> __device__ __forceinline__ void cdw_planes(float a, float b, uint32_t (&p)[PL])
{
    if constexpr (PL == 3) {
        uint32_t ha, ma, la, hb, mb, lb;
        split3(a, ha, ma, la); split3(b, hb, mb, lb);
        p[0] = (la >> 16) | lb; p[1] = (ma >> 16) | mb; p[2] = (ha >> 16) | hb;
    } else {
        split2_pk(a, b, p[1], p[0]);
    }
}

// The 16 bytes that start SB bytes into the 32 bytes {lo, hi}.
template <int SB>
__device__ __forceinline__ u32x4 cdw_funnel(const uint4 &lo, const uint4 &hi)
{
    const uint32_t d[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    constexpr int q = SB >> 2, b = SB & 3;
    if constexpr (b == 0) return u32x4{d[q], d[q + 1], d[q + 2], d[q + 3]};
    else return u32x4{__builtin_amdgcn_alignbyte(d[q + 1], d[q], b), __builtin_amdgcn_alignbyte(d[q + 2], d[q + 1], b),
                      __builtin_amdgcn_alignbyte(d[q + 3], d[q + 2], b), __builtin_amdgcn_alignbyte(d[q + 4], d[q + 3], b)};
}

// ROWS: 0 rows of any length; 1 image rows and code rows of whole 4-element pieces; 2 the same with code rows of whole 8-code pieces
template <int MODE, int R, int S, int PAD, int MB, int ROWS>
__global__ __launch_bounds__(512, 1) void conv_dw_kernel(ConvDwArgs a)
{
    constexpr bool ROW4 = ROWS != 0, C8 = ROWS == 2;
    if (a.gate.closed()) return;
    using TR = CdwTraits<MODE>;
    using XT = typename TR::XT;
    using XRaw = typename TR::XRaw;
    using Acc = typename TR::Acc;
    using AccT = typename TR::AccT;
    constexpr int PL = TR::PLANES, ESZ = TR::ESZ, FRAG = TR::FRAG, KSTEP = 2 * FRAG;
    constexpr int TK = 64 * MB, TC = 64, RS = R * S;
    constexpr int CI = TK / 2, XI = TC / 4;                          // most pieces a stager thread handles (128 / 64 along)
    extern __shared__ uint4 cdw_lds[];
    // two buffers of { X [PL][TC][pitchX], codes [TK][pitchC] } elements
    const size_t x_plane = (size_t)TC * a.pitchX * ESZ, x_bytes = PL * x_plane;
    const size_t buf_bytes = x_bytes + (size_t)TK * a.pitchC * ESZ;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool stager = wave >= 4;                                   // uniform per wavefront
    const int tid = threadIdx.x & 255;                               // index inside the role
    const int lcol = lane & 31, lhalf = lane >> 5;
    const int wr = (wave & 3) >> 1, wcl = wave & 1;                  // multiplier's place in the 2x2 arrangement
    const int tiles = a.tiles_k * a.tiles_c;
    // Workgroup w runs on XCD w % 8, and each XCD has an L2 of its own: renumber so that the tiles of one split (which
    // read the same images at about the same time, each operand tile shared by a row or column of tiles) sit on one XCD.
    const int wg = (gridDim.x & 7) == 0 ? (int)((blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) : (int)blockIdx.x;
    const int tile = wg % tiles, split = wg / tiles;
    const int k0 = (tile % a.tiles_k) * TK, c0 = (tile / a.tiles_k) * TC;
    const int unit_a = split * a.units_per_split, unit_b = min(unit_a + a.units_per_split, a.units);
    const int PI = a.H * a.Wd, PQ = a.P * a.Q;

    for (int i = threadIdx.x; i < a.lds_cells; i += 512) cdw_lds[i] = uint4{0u, 0u, 0u, 0u};

    Acc acc[RS][MB];                                                 // multipliers only
    const int xq = tid & ((1 << a.xshift) - 1), xch = tid >> a.xshift, XCH = 256 >> a.xshift, xi_n = TC >> (8 - a.xshift);
    const int cq = tid & ((1 << a.cshift) - 1), cch = tid >> a.cshift, CCH = 256 >> a.cshift, ci_n = TK >> (8 - a.cshift);

    XRaw xr[XI];                                                     // raw loads of the unit being staged next
    uint32_t cr[CI];
    // Pieces of 8 codes where rows allow (a wavefront's load costs the CU's address unit the same 16 cycles whether it
    // moves 256 B or 512 B, and the stagers' loads are what they wait for): half as many code loads.
    typedef uint32_t u32x2_a4 __attribute__((ext_vector_type(2), aligned(4)));
    u32x2_a4 cr8[C8 ? CI / 2 : 1];

    // Aligned loads of a unit's rows.  Pieces outside the tensor or the channel range read offset 0 of the
    // (uniform) base and are replaced by zero when staged, so the loads are straight-line code.
    auto issue_loads = [&](int unit) {
        const int n = unit / a.chunks, h_a = (unit - n * a.chunks) * a.RU;
        const int fe0 = ((h_a * a.Wd) & ~3) + 4 * xq;
        const bool x_ld = xq < a.nqx && fe0 < PI;
        const char *xb0 = (const char *)((const XT *)a.X + ((int64_t)n * a.Ct + c0) * PI);         // uniform
        const int p_lo = h_a - 1 - (R - 1) + a.pad;
        const int fc0 = ((p_lo * a.Q) & ~3) + 4 * cq;
        const bool c_ld = cq < a.nqc && fc0 >= 0 && fc0 < PQ;
        const char *cb0 = (const char *)(a.codes + ((int64_t)n * a.Kt + k0) * PQ);                  // uniform
#pragma unroll
        for (int j = 0; j < CI; ++j) {
            if (j >= ci_n) break;
            const int kl = cch + CCH * j;
            const bool ok = c_ld && k0 + kl < a.K;
            cr[j] = *(const uint32_t *)(cb0 + (ok ? (uint32_t)(kl * PQ + fc0) : 0u));
        }
#pragma unroll
        for (int j = 0; j < XI; ++j) {
            if (j >= xi_n) break;
            const int cl = xch + XCH * j;
            const bool ok = x_ld && c0 + cl < a.C;
            xr[j] = *(const XRaw *)(xb0 + (ok ? (uint32_t)(cl * PI + fe0) * (uint32_t)sizeof(XT) : 0u));
        }
    };

    // ---- ROW4: image rows and code rows are whole numbers of aligned 4-element pieces (Wd % 4 == 0, Q % 4 == 0).
    // A piece then never straddles rows and its place inside a unit is the same for every unit: its LDS address
    // and its lane offset in global memory are computed once; a unit only moves the bases (the same for all
    // lanes) and the limits at the image's top and bottom.  The stagers are single wavefronts per SIMD and are
    // bound by the number of instructions they issue: per piece this path issues an addition, a comparison
    // and a select on either side of the load, where the general path below recomputes positions (two
    // integer divisions per unit), multiplies addresses per piece and branches around every write.
    const int xrel = 4 * xq, crel = (C8 ? 8 : 4) * cq;
    bool x_own = false, c_own = false;
    uint32_t x_lds0 = 0, c_lds0 = 0, x_g0 = 0;
    int c_g0 = 0;
    if constexpr (ROW4) {
        const int xrow = xrel / a.Wd, xw = xrel - xrow * a.Wd;
        x_own = stager && xq < a.nqx && xrow < a.RU;
        x_lds0 = (uint32_t)((xch * a.pitchX + xrow * a.PW + xw) * ESZ);
        x_g0 = (uint32_t)(xch * PI + xrel) * (uint32_t)sizeof(XT);
        const int crow = crel / a.Q, cqq = crel - crow * a.Q;
        const int cps = (crow - 1) * a.PW + cqq + CDW_M8;          // pitched coordinate inside the patch
        c_own = stager && cq < a.nqc && crow < a.NR && cps >= 0 && cps < a.lenC;
        c_lds0 = (uint32_t)(x_bytes + (size_t)(cch * a.pitchC + (c_own ? cps : 0)) * ESZ);
        c_g0 = cch * PQ + crel;
    }
    const uint32_t x_gstep = (uint32_t)(XCH * PI) * (uint32_t)sizeof(XT), x_lstep = (uint32_t)(XCH * a.pitchX * ESZ);
    const int c_gstep = CCH * PQ;
    const uint32_t c_lstep = (uint32_t)(CCH * a.pitchC * ESZ);

    // A tile that has all its 64*MB output channels and 64 input channels needs no test per piece: validity is then
    // one mask per lane and unit (all ones or zero) that is and-ed into the lane offset before the load (an
    // invalid piece reads offset 0) and into the value before the LDS write; no comparison, no select through
    // scalar registers, no branch per piece.
    const bool whole_tile = k0 + TK <= a.K && c0 + TC <= a.C;            // uniform

    auto issue_fast = [&](int unit) {
        const int n = unit / a.chunks, h_a = (unit - n * a.chunks) * a.RU;
        const char *xb = (const char *)((const XT *)a.X + ((int64_t)n * a.Ct + c0) * PI + h_a * a.Wd);      // uniform
        const bool x_ld = x_own && xrel < PI - h_a * a.Wd;               // below the image's last row: nothing to load
        const int c_shift = (h_a - 1 - (R - 1) + a.pad) * a.Q;           // first code element of the patch rows (may be < 0)
        const char *cb = (const char *)(a.codes + ((int64_t)n * a.Kt + k0) * PQ);                         // uniform
        const bool c_ld = c_own && crel + c_shift >= 0 && crel + c_shift < PQ;
        if (whole_tile) {
            const uint32_t cm = c_ld ? 0xFFFFFFFFu : 0u, xm = x_ld ? 0xFFFFFFFFu : 0u;
            uint32_t co = (uint32_t)(c_g0 + c_shift) & cm, xo = x_g0 & xm;
            const uint32_t cs = (uint32_t)c_gstep & cm, xs = x_gstep & xm;
            if constexpr (C8) {
#pragma unroll
                for (int j = 0; j < CI / 2; ++j) {
                    if (j >= ci_n) break;
                    cr8[j] = *(const u32x2_a4 *)(cb + co);
                    co += cs;
                }
            } else {
#pragma unroll
                for (int j = 0; j < CI; ++j) {
                    if (j >= ci_n) break;
                    cr[j] = *(const uint32_t *)(cb + co);
                    co += cs;
                }
            }
#pragma unroll
            for (int j = 0; j < XI; ++j) {
                if (j >= xi_n) break;
                xr[j] = *(const XRaw *)(xb + xo);
                xo += xs;
            }
        } else {
            if constexpr (C8) {
#pragma unroll
                for (int j = 0; j < CI / 2; ++j) {
                    if (j >= ci_n) break;
                    const bool ok = c_ld && k0 + cch + CCH * j < a.K;
                    cr8[j] = *(const u32x2_a4 *)(cb + (ok ? (uint32_t)(c_g0 + c_shift + j * c_gstep) : 0u));
                }
            } else {
#pragma unroll
                for (int j = 0; j < CI; ++j) {
                    if (j >= ci_n) break;
                    const bool ok = c_ld && k0 + cch + CCH * j < a.K;
                    cr[j] = *(const uint32_t *)(cb + (ok ? (uint32_t)(c_g0 + c_shift + j * c_gstep) : 0u));
                }
            }
#pragma unroll
            for (int j = 0; j < XI; ++j) {
                if (j >= xi_n) break;
                const bool ok = x_ld && c0 + xch + XCH * j < a.C;
                xr[j] = *(const XRaw *)(xb + (ok ? x_g0 + (uint32_t)j * x_gstep : 0u));
            }
        }
    };

    // One piece into LDS; `m` is the piece's validity mask (all ones or zero).
    auto put_x = [&](uint32_t addr, const XRaw &raw, uint32_t m) {
        char *d = (char *)cdw_lds + addr;
        if constexpr (MODE != MODE_I8) {
            const uint32_t rw[4] = {raw.x & m, raw.y & m, raw.z & m, raw.w & m};
            uint32_t p01[PL], p23[PL];
            cdw_planes<PL>(__uint_as_float(rw[0]), __uint_as_float(rw[1]), p01);
            cdw_planes<PL>(__uint_as_float(rw[2]), __uint_as_float(rw[3]), p23);
#pragma unroll
            for (int pl = 0; pl < PL; ++pl) *(uint2 *)(d + pl * x_plane) = uint2{p01[pl], p23[pl]};
        } else {
            *(uint32_t *)d = raw & m;
        }
    };
    auto put_c = [&](uint32_t addr, uint32_t t) {
        char *d = (char *)cdw_lds + addr;
        if constexpr (MODE != MODE_I8)
            *(uint2 *)d = uint2{bf16_pair_from_i8((int8_t)t, (int8_t)(t >> 8)), bf16_pair_from_i8((int8_t)(t >> 16), (int8_t)(t >> 24))};
        else
            *(uint32_t *)d = t;
    };

    auto put_c8 = [&](uint32_t addr, uint32_t t0, uint32_t t1) {          // eight codes -> one 16-byte cell of bf16 (bf16 modes only)
        *(uint4 *)((char *)cdw_lds + addr) =
            uint4{bf16_pair_from_i8((int8_t)t0, (int8_t)(t0 >> 8)), bf16_pair_from_i8((int8_t)(t0 >> 16), (int8_t)(t0 >> 24)),
                  bf16_pair_from_i8((int8_t)t1, (int8_t)(t1 >> 8)), bf16_pair_from_i8((int8_t)(t1 >> 16), (int8_t)(t1 >> 24))};
    };

    auto stage_fast = [&](int unit, uint32_t buf_off) {
        const int n = unit / a.chunks, h_a = (unit - n * a.chunks) * a.RU;
        if (x_own) {
            const bool x_ld = xrel < PI - h_a * a.Wd;
            const uint32_t xm = x_ld ? 0xFFFFFFFFu : 0u;
            uint32_t addr = buf_off + x_lds0;                              // 32-bit LDS byte address of the piece
            if (whole_tile) {
#pragma unroll
                for (int j = 0; j < XI; ++j) {
                    if (j >= xi_n) break;
                    put_x(addr, xr[j], xm);
                    addr += x_lstep;
                }
            } else {
#pragma unroll
                for (int j = 0; j < XI; ++j) {
                    if (j >= xi_n) break;
                    put_x(addr, xr[j], c0 + xch + XCH * j < a.C ? xm : 0u);
                    addr += x_lstep;
                }
            }
        }
        if (c_own) {
            const int c_shift = (h_a - 1 - (R - 1) + a.pad) * a.Q;
            const bool c_ld = crel + c_shift >= 0 && crel + c_shift < PQ;
            const uint32_t cm = c_ld ? 0xFFFFFFFFu : 0u;
            uint32_t addr = buf_off + c_lds0;
            if constexpr (C8) {
#pragma unroll
                for (int j = 0; j < CI / 2; ++j) {
                    if (j >= ci_n) break;
                    const uint32_t m = whole_tile || k0 + cch + CCH * j < a.K ? cm : 0u;
                    put_c8(addr, cr8[j].x & m, cr8[j].y & m);
                    addr += c_lstep;
                }
            } else if (whole_tile) {
#pragma unroll
                for (int j = 0; j < CI; ++j) {
                    if (j >= ci_n) break;
                    put_c(addr, cr[j] & cm);
                    addr += c_lstep;
                }
            } else {
#pragma unroll
                for (int j = 0; j < CI; ++j) {
                    if (j >= ci_n) break;
                    put_c(addr, k0 + cch + CCH * j < a.K ? cr[j] & cm : 0u);
                    addr += c_lstep;
                }
            }
        }
    };

    // Convert the raw loads and scatter them to their pitched positions in LDS (rows of any length).
    auto stage = [&](int unit, char *lds_x, char *lds_c) {
        const int n = unit / a.chunks, h_a = (unit - n * a.chunks) * a.RU;
        if (xq < a.nqx) {
            const int fe0 = ((h_a * a.Wd) & ~3) + 4 * xq;
            const bool x_ld = fe0 < PI;
            int h = fe0 / a.Wd, w = fe0 - h * a.Wd;
            int pos[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pos[e] = (h >= h_a && h < h_a + a.RU) ? (h - h_a) * a.PW + w : -1;
                if (++w == a.Wd) { w = 0; ++h; }
            }
            bool done = false;
            if (a.row2x && !a.row4x) {
                // Rows of an even length that is not a multiple of 4 (14x14 planes ...): a piece may straddle two rows, its
                // halves never do, and their places are the same for all channels.  A half with no place in this unit is
                // written as zeros into the zero columns behind the unit's first row (PW - Wd >= 2 for such widths), so
                // the loop over the channels has no branch: a mask on the value, two fixed offsets.
                const uint32_t mA = x_ld && pos[0] >= 0 ? 0xFFFFFFFFu : 0u, mB = x_ld && pos[2] >= 0 ? 0xFFFFFFFFu : 0u;
                const uint32_t oA = (uint32_t)((pos[0] >= 0 ? pos[0] : a.Wd) * ESZ), oB = (uint32_t)((pos[2] >= 0 ? pos[2] : a.Wd) * ESZ);
                char *row = lds_x + (size_t)xch * a.pitchX * ESZ;
                const size_t rstep = (size_t)XCH * a.pitchX * ESZ;
#pragma unroll
                for (int j = 0; j < XI; ++j) {
                    if (j >= xi_n) break;
                    const uint32_t okm = (whole_tile || c0 + xch + XCH * j < a.C) ? 0xFFFFFFFFu : 0u;
                    const uint32_t ma = mA & okm, mb = mB & okm;
                    if constexpr (MODE != MODE_I8) {
                        uint32_t pa[PL], pb[PL];
                        cdw_planes<PL>(__uint_as_float(xr[j].x & ma), __uint_as_float(xr[j].y & ma), pa);
                        cdw_planes<PL>(__uint_as_float(xr[j].z & mb), __uint_as_float(xr[j].w & mb), pb);
#pragma unroll
                        for (int pl = 0; pl < PL; ++pl) {
                            *(uint32_t *)(row + oA + pl * x_plane) = pa[pl];
                            *(uint32_t *)(row + oB + pl * x_plane) = pb[pl];
                        }
                    } else {
                        *(uint16_t *)(row + oA) = (uint16_t)(xr[j] & ma);
                        *(uint16_t *)(row + oB) = (uint16_t)((xr[j] >> 16) & mb);
                    }
                    row += rstep;
                }
                done = true;
            }
#pragma unroll
            for (int j = 0; j < XI; ++j) {
                if (done || j >= xi_n) break;
                const int cl = xch + XCH * j;
                const bool ok = x_ld && c0 + cl < a.C;
                char *row = lds_x + (size_t)cl * a.pitchX * ESZ;
                if constexpr (MODE != MODE_I8) {
                    const uint32_t rw[4] = {xr[j].x, xr[j].y, xr[j].z, xr[j].w};
                    uint32_t pp[2][PL];                                  // elements (0, 1) and (2, 3)
                    cdw_planes<PL>(ok ? __uint_as_float(rw[0]) : 0.0f, ok ? __uint_as_float(rw[1]) : 0.0f, pp[0]);
                    cdw_planes<PL>(ok ? __uint_as_float(rw[2]) : 0.0f, ok ? __uint_as_float(rw[3]) : 0.0f, pp[1]);
                    if (a.row4x) {
                        if (pos[0] >= 0) {
                            char *d = row + pos[0] * ESZ;
#pragma unroll
                            for (int pl = 0; pl < PL; ++pl) *(uint2 *)(d + pl * x_plane) = uint2{pp[0][pl], pp[1][pl]};
                        }
                    } else if (a.row2x) {
#pragma unroll
                        for (int e = 0; e < 4; e += 2)
                            if (pos[e] >= 0) {
                                char *d = row + pos[e] * ESZ;
#pragma unroll
                                for (int pl = 0; pl < PL; ++pl) *(uint32_t *)(d + pl * x_plane) = pp[e >> 1][pl];
                            }
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (pos[e] >= 0) {
                                char *d = row + pos[e] * ESZ;
#pragma unroll
                                for (int pl = 0; pl < PL; ++pl) *(uint16_t *)(d + pl * x_plane) = (uint16_t)(pp[e >> 1][pl] >> (16 * (e & 1)));
                            }
                    }
                } else {
                    const uint32_t t = ok ? xr[j] : 0u;
                    if (a.row4x) {
                        if (pos[0] >= 0) *(uint32_t *)(row + pos[0]) = t;
                    } else if (a.row2x) {
                        if (pos[0] >= 0) *(uint16_t *)(row + pos[0]) = (uint16_t)t;
                        if (pos[2] >= 0) *(uint16_t *)(row + pos[2]) = (uint16_t)(t >> 16);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (pos[e] >= 0) *(uint8_t *)(row + pos[e]) = (uint8_t)(t >> (8 * e));
                    }
                }
            }
        }
        if (cq < a.nqc) {
            const int p_lo = h_a - 1 - (R - 1) + a.pad;
            const int fc0 = ((p_lo * a.Q) & ~3) + 4 * cq;
            const bool c_ld = fc0 >= 0 && fc0 < PQ;
            int p = (fc0 + CDW_OFFR * a.Q) / a.Q - CDW_OFFR, q = fc0 - p * a.Q;
            int pos[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // code (p,q) lives at pitched coordinate (p + R-1 - pad)*PW + q + M8; the patch starts at h_a*PW
                const int ps = (p + (R - 1) - a.pad - h_a) * a.PW + q + CDW_M8;
                pos[e] = (p >= p_lo && p < p_lo + a.NR && ps >= 0 && ps < a.lenC) ? ps : -1;
                if (++q == a.Q) { q = 0; ++p; }
            }
            bool done = false;
            if (a.row2c && !a.row4c) {
                // the same for the codes: a half with no place goes, as zeros, to the zero columns behind the patch's second row
                const uint32_t mA = c_ld && pos[0] >= 0 ? 0xFFFFFFFFu : 0u, mB = c_ld && pos[2] >= 0 ? 0xFFFFFFFFu : 0u;
                const int spare = a.PW + a.Q + CDW_M8;
                const uint32_t oA = (uint32_t)((pos[0] >= 0 ? pos[0] : spare) * ESZ), oB = (uint32_t)((pos[2] >= 0 ? pos[2] : spare) * ESZ);
                char *row = lds_c + (size_t)cch * a.pitchC * ESZ;
                const size_t rstep = (size_t)CCH * a.pitchC * ESZ;
#pragma unroll
                for (int j = 0; j < CI; ++j) {
                    if (j >= ci_n) break;
                    const uint32_t okm = (whole_tile || k0 + cch + CCH * j < a.K) ? 0xFFFFFFFFu : 0u;
                    const uint32_t t = cr[j];
                    if constexpr (MODE != MODE_I8) {
                        *(uint32_t *)(row + oA) = bf16_pair_from_i8((int8_t)t, (int8_t)(t >> 8)) & mA & okm;
                        *(uint32_t *)(row + oB) = bf16_pair_from_i8((int8_t)(t >> 16), (int8_t)(t >> 24)) & mB & okm;
                    } else {
                        *(uint16_t *)(row + oA) = (uint16_t)(t & mA & okm);
                        *(uint16_t *)(row + oB) = (uint16_t)((t >> 16) & mB & okm);
                    }
                    row += rstep;
                }
                done = true;
            }
#pragma unroll
            for (int j = 0; j < CI; ++j) {
                if (done || j >= ci_n) break;
                const int kl = cch + CCH * j;
                const uint32_t t = (c_ld && k0 + kl < a.K) ? cr[j] : 0u;
                char *row = lds_c + (size_t)kl * a.pitchC * ESZ;
                if constexpr (MODE != MODE_I8) {
                    const uint32_t b01 = bf16_pair_from_i8((int8_t)t, (int8_t)(t >> 8));
                    const uint32_t b23 = bf16_pair_from_i8((int8_t)(t >> 16), (int8_t)(t >> 24));
                    if (a.row4c) {
                        if (pos[0] >= 0) *(uint2 *)(row + pos[0] * ESZ) = uint2{b01, b23};
                    } else if (a.row2c) {
                        if (pos[0] >= 0) *(uint32_t *)(row + pos[0] * ESZ) = b01;
                        if (pos[2] >= 0) *(uint32_t *)(row + pos[2] * ESZ) = b23;
                    } else {
                        if (pos[0] >= 0) *(uint16_t *)(row + pos[0] * ESZ) = (uint16_t)b01;
                        if (pos[1] >= 0) *(uint16_t *)(row + pos[1] * ESZ) = (uint16_t)(b01 >> 16);
                        if (pos[2] >= 0) *(uint16_t *)(row + pos[2] * ESZ) = (uint16_t)b23;
                        if (pos[3] >= 0) *(uint16_t *)(row + pos[3] * ESZ) = (uint16_t)(b23 >> 16);
                    }
                } else {
                    if (a.row4c) {
                        if (pos[0] >= 0) *(uint32_t *)(row + pos[0]) = t;
                    } else if (a.row2c) {
                        if (pos[0] >= 0) *(uint16_t *)(row + pos[0]) = (uint16_t)t;
                        if (pos[2] >= 0) *(uint16_t *)(row + pos[2]) = (uint16_t)(t >> 16);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (pos[e] >= 0) *(uint8_t *)(row + pos[e]) = (uint8_t)(t >> (8 * e));
                    }
                }
            }
        }
    };

    // One matrix-core step: the X fragment of this lane's run, and per kernel row r the window of code cells
    // that holds the runs of all S column shifts (byte offsets (M8 + PAD - s) * ESZ from the row's base).
    constexpr int CB_MIN = (CDW_M8 + PAD - (S - 1)) * ESZ, CB_MAX = (CDW_M8 + PAD) * ESZ;
    constexpr int LO_CELL = CB_MIN / 16, NCELL = (CB_MAX + 16 + 15) / 16 - LO_CELL;
    struct StepFrags { uint4 x[PL]; uint4 w[R][MB][NCELL]; };
    // per-lane LDS byte offsets of step 0 (buffer 0), computed once
    const uint32_t frag_x0 = (uint32_t)(((wcl * 32 + lcol) * a.pitchX + FRAG * lhalf) * ESZ);
    uint32_t frag_c0[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
        frag_c0[mb] = (uint32_t)(x_bytes + (((wr * MB + mb) * 32 + lcol) * a.pitchC + FRAG * lhalf) * ESZ + LO_CELL * 16);
    const uint32_t row_bytes = (uint32_t)(a.PW * ESZ);               // one kernel row further: a whole number of cells
    auto load_frags = [&](uint32_t buf_off, int step, StepFrags &f) {
        const char *base = (const char *)cdw_lds + buf_off + (uint32_t)(step * KSTEP * ESZ);
#pragma unroll
        for (int pl = 0; pl < PL; ++pl) f.x[pl] = *(const uint4 *)(base + frag_x0 + pl * (uint32_t)x_plane);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int c = 0; c < NCELL; ++c)
                    f.w[r][mb][c] = *(const uint4 *)(base + frag_c0[mb] + (uint32_t)(R - 1 - r) * row_bytes + 16 * c);
    };
    auto multiply = [&](const StepFrags &f) {
        u32x4 xb[PL];
#pragma unroll
        for (int pl = 0; pl < PL; ++pl) xb[pl] = u32x4{f.x[pl].x, f.x[pl].y, f.x[pl].z, f.x[pl].w};
        // per kernel row: the S shifted code fragments first, then planes outermost, so that consecutive
        // matrix-core instructions never accumulate into the same registers
        static_for<0, R>([&](auto rr) {
            constexpr int r = decltype(rr)::value;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                // Every dword of the cells counts as used: a tap needs only five of a window's eight, and the
                // compiler would then read the window as single dwords, which for lanes one LDS row apart is a
                // four-way bank conflict; whole 16-byte cells are conflict-free.
                uint4 w[NCELL];
#pragma unroll
                for (int c = 0; c < NCELL; ++c) {
                    w[c] = f.w[r][mb][c];
                    if constexpr (MODE == MODE_I8) asm volatile("" : "+v"(w[c].x), "+v"(w[c].y), "+v"(w[c].z), "+v"(w[c].w));
                }
                u32x4 af[S];
                static_for<0, S>([&](auto ss) {
                    constexpr int sx = decltype(ss)::value;
                    constexpr int cb = (CDW_M8 + PAD - sx) * ESZ, ci = cb / 16 - LO_CELL, sb = cb & 15;
                    if constexpr (sb == 0) af[sx] = u32x4{w[ci].x, w[ci].y, w[ci].z, w[ci].w};
                    else af[sx] = cdw_funnel<sb>(w[ci], w[ci + 1]);
                });
#pragma unroll
                for (int pl = 0; pl < PL; ++pl)
#pragma unroll
                    for (int sx = 0; sx < S; ++sx) Mma<MODE>::run(af[sx], xb[pl], acc[r * S + sx][mb]);
            }
        });
    };

    // Barriers: one after the clearing of LDS, one after the first unit is staged, one per unit.  Both roles
    // execute exactly these (their loops have the same trip count), in code of their own so that neither
    // keeps the other's registers alive.
    char *const lds0 = (char *)cdw_lds;
    const int n_units = unit_b - unit_a;
    if (stager) {
        // (the calls are written out: wrapping them in further lambdas keeps the raw-load arrays out of registers)
        if (n_units > 0) { if constexpr (ROW4) issue_fast(unit_a); else issue_loads(unit_a); }
        __syncthreads();
        if (n_units > 0) { if constexpr (ROW4) stage_fast(unit_a, 0u); else stage(unit_a, lds0, lds0 + x_bytes); }
        if (n_units > 1) { if constexpr (ROW4) issue_fast(unit_a + 1); else issue_loads(unit_a + 1); }
        __syncthreads();
        for (int i = 0; i < n_units; ++i) {
            if (i + 1 < n_units) {
                const uint32_t nb_off = (uint32_t)(((i + 1) & 1) * buf_bytes);
                if constexpr (ROW4) stage_fast(unit_a + i + 1, nb_off);
                else stage(unit_a + i + 1, lds0 + nb_off, lds0 + nb_off + x_bytes);
                if (i + 2 < n_units) { if constexpr (ROW4) issue_fast(unit_a + i + 2); else issue_loads(unit_a + i + 2); }
            }
            __syncthreads();
        }
        return;
    }

#pragma unroll
    for (int t = 0; t < RS; ++t)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][mb][v] = 0;
    __syncthreads();
    __syncthreads();
    for (int i = 0; i < n_units; ++i) {
        const uint32_t cur = (uint32_t)((i & 1) * buf_bytes);
        // Fragments are fetched one step ahead of the matrix cores that consume them (ping-pong A/B).
        const int n_steps = a.TPc / KSTEP;
        StepFrags fa, fb;
        load_frags(cur, 0, fa);
        // The scheduling barriers keep the LDS reads of the next step in front of this step's matrix-core
        // instructions (left alone, the compiler sinks them behind and their latency is exposed).  The loads of the
        // loop body are unconditional (the last one repeats the last step): with a load on only some paths the
        // compiler waits for ALL LDS loads in flight where it has to wait for one step's.
        int step = 0;
        for (; step + 2 <= n_steps; step += 2) {
            load_frags(cur, step + 1, fb);
            __builtin_amdgcn_sched_barrier(0);
            multiply(fa);
            __builtin_amdgcn_sched_barrier(0);
            load_frags(cur, min(step + 2, n_steps - 1), fa);
            __builtin_amdgcn_sched_barrier(0);
            multiply(fb);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (step < n_steps) multiply(fa);
        __syncthreads();
    }

    // ---- results: lane holds column c = lcol, rows k = 8*(v/4) + 4*lhalf + v%4 of each block ---------
    if (a.n_split > 1) {
        // [tile][split][tap][block][v / 4][thread][v % 4]: 16-byte stores, 1 KiB contiguous per wavefront
        typedef AccT Acc4 __attribute__((ext_vector_type(4)));
        Acc4 *dst = (Acc4 *)a.partial + ((int64_t)tile * a.n_split + split) * (RS * MB * 4) * 256 + tid;
#pragma unroll
        for (int t = 0; t < RS; ++t)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq)
                    dst[((t * MB + mb) * 4 + vq) * 256] = Acc4{acc[t][mb][4 * vq], acc[t][mb][4 * vq + 1], acc[t][mb][4 * vq + 2], acc[t][mb][4 * vq + 3]};
    } else {
        AccT *out = (AccT *)a.dW;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int c = c0 + wcl * 32 + lcol;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = k0 + (wr * MB + mb) * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
                if (k < a.K && c < a.C) {
#pragma unroll
                    for (int t = 0; t < RS; ++t) {
                        if constexpr (MODE != MODE_I8) out[((int64_t)k * a.C + c) * RS + t] = acc[t][mb][v] * a.scale.get();
                        else out[((int64_t)k * a.C + c) * RS + t] = acc[t][mb][v];
                    }
                }
            }
        }
    }
}

// Sum of the split partials: a workgroup owns 16 thread slots of four accumulator elements (one 16-byte
// group) of a tile; its 16 phases add every 16th split each (in split order) and the 16 sums are added in
// phase order: deterministic, and enough workgroups to fill the chip even when dW is a single tile.
template <int MODE, int R, int S, int MB>
__global__ __launch_bounds__(256) void conv_dw_reduce_kernel(ConvDwArgs a)
{
    if (a.gate.closed()) return;
    using AccT = typename CdwTraits<MODE>::AccT;
    typedef AccT Acc4 __attribute__((ext_vector_type(4)));
    constexpr int RS = R * S, NG = RS * MB * 4;
    __shared__ Acc4 part[16][16];
    const int sixteenth = blockIdx.x & 15, g = (blockIdx.x >> 4) % NG, tile = (blockIdx.x >> 4) / NG;
    const int sl = threadIdx.x & 15, ph = threadIdx.x >> 4, slot = sixteenth * 16 + sl;
    const Acc4 *src = (const Acc4 *)a.partial + ((int64_t)tile * a.n_split * NG + g) * 256 + slot;
    Acc4 sum = Acc4{0, 0, 0, 0};
    for (int q = ph; q < a.n_split; q += 16) sum += src[(int64_t)q * NG * 256];
    part[ph][sl] = sum;
    __syncthreads();
    if (ph != 0) return;
#pragma unroll
    for (int i = 1; i < 16; ++i) sum += part[i][sl];
    const int vq = g & 3, mb = (g >> 2) % MB, t = (g >> 2) / MB;
    const int lane = slot & 63, wave = slot >> 6, lcol = lane & 31, lhalf = lane >> 5, wr = wave >> 1, wcl = wave & 1;
    const int kb = (tile % a.tiles_k) * (64 * MB) + (wr * MB + mb) * 32 + 8 * vq + 4 * lhalf;
    const int c = (tile / a.tiles_k) * 64 + wcl * 32 + lcol;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int k = kb + j;
        if (k < a.K && c < a.C) {
            AccT *out = (AccT *)a.dW + ((int64_t)k * a.C + c) * RS + t;
            if constexpr (MODE != MODE_I8) *out = sum[j] * a.scale.get(); else *out = sum[j];
        }
    }
}

}  // namespace dbp
