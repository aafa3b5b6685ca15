// Host-side launchers of the matrix-core products: fully connected and implicit-im2col convolution,
// dithered (bf16x3 / int8) and dense (fp32) variants, with deterministic split-K.
#include <vector>
#include "conv_loaders.h"
#include "fc_kernel.h"
#include "fc2_kernel.h"
#include "fc2_i8_kernel.h"
#include "conv_dx_kernel.h"
#include "conv_dw_kernel.h"
#include "conv_dw_i8_kernel.h"
#include "conv_lower.h"

namespace dbp {

namespace {

constexpr int kTargetWorkgroups = 512;          // two resident workgroups on each of the 256 CUs

struct Split { int n; int k_per; };

// Split the reduction so that tiles*n reaches kTargetWorkgroups, each part at least 4 K steps long
// and a multiple of `granule` (the K step, or one padded image for conv dW).
Split choose_split(int64_t tiles, int64_t K, int granule)
{
    int64_t want = (kTargetWorkgroups + tiles - 1) / tiles;
    int64_t units = (K + granule - 1) / granule;
    int64_t max_n = units / 4 > 0 ? units / 4 : 1;
    if (want > max_n) want = max_n;
    if (want < 1) want = 1;
    int64_t per = (units + want - 1) / want * granule;
    int64_t n = (K + per - 1) / per;
    return Split{(int)n, (int)per};
}

template <int MODE> constexpr int k_step() { return NCHUNK * ModeTraits<MODE>::KCH; }

template <int MODE, class AL, class BL, class OM>
hipError_t run_gemm(const AL &al, const BL &bl, const OM &om, int M, int N, int K, int granule, Scale scale,
                    typename ModeTraits<MODE>::Acc *out, void *scratch, size_t scratch_bytes, hipStream_t s)
{
    using Acc = typename ModeTraits<MODE>::Acc;
    GemmShape sh;
    sh.M = M; sh.N = N; sh.K = K;
    sh.tiles_m = (M + TM - 1) / TM;
    sh.tiles_n = (N + TN - 1) / TN;
    const int64_t tiles = (int64_t)sh.tiles_m * sh.tiles_n;
    Split sp = choose_split(tiles, K, granule);
    while (sp.n > 1 && (size_t)sp.n * M * N * sizeof(Acc) > scratch_bytes) {      // never exceed the workspace
        int64_t units = (K + granule - 1) / granule;
        int64_t n = sp.n - 1;
        sp.k_per = (int)((units + n - 1) / n * granule);
        sp.n = (int)((K + sp.k_per - 1) / sp.k_per);
    }
    sh.k_per_split = sp.n == 1 ? (K + granule - 1) / granule * granule : sp.k_per;
    dim3 grid((unsigned)tiles, 1, (unsigned)sp.n);
    hipLaunchKernelGGL((gemm_kernel<MODE, AL, BL, OM>), grid, dim3(256), 0, s, al, bl, om, sh, scale, out, (Acc *)scratch);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (sp.n > 1) {
        int64_t total = (int64_t)M * N;
        int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
        hipLaunchKernelGGL((reduce_kernel<Acc, OM>), dim3(blocks), dim3(256), 0, s, (const Acc *)scratch, out, om, M, N, sp.n, scale);
        e = hipGetLastError();
    }
    return e;
}

// Weights re-laid for the dX product of a convolution: Wt[(r*S+s)*Kp + k][c] = W[k][c][r][s], zero for k >= K.
template <class T>
__global__ __launch_bounds__(256) void conv_weight_relayout_kernel(const T *W, T *Wt, ConvGeom g)
{
    const int64_t total = (int64_t)g.R * g.S * g.Kp * g.C;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int c = (int)(i % g.C);
        const int64_t kk = i / g.C;
        const int k = (int)(kk % g.Kp), rs = (int)(kk / g.Kp);
        Wt[i] = k < g.K ? W[((int64_t)k * g.C + c) * g.R * g.S + rs] : (T)0;
    }
}

ConvGeom make_geom(const ConvArgs &a, int kch, int kstep)
{
    ConvGeom g;
    g.N = (int)a.N; g.C = (int)a.C; g.H = (int)a.H; g.Wd = (int)a.Wd; g.K = (int)a.K; g.R = (int)a.R; g.S = (int)a.S;
    g.pad = (int)a.pad; g.st = (int)a.stride;
    g.P = (g.H + 2 * g.pad - g.R) / g.st + 1;
    g.Q = (g.Wd + 2 * g.pad - g.S) / g.st + 1;
    g.Kp = (g.K + kch - 1) / kch * kch;
    g.PQp = (g.P * g.Q + kstep - 1) / kstep * kstep;
    g.Ct = (int)a.ct(); g.Kt = (int)a.kt();
    return g;
}

size_t relayout_bytes(int64_t K, int64_t C, int64_t R, int64_t S)
{
    int64_t Kp = (K + 7) / 8 * 8;                       // multiple of every chunk length in use (4, 8)
    const size_t generic = (size_t)(R * S * Kp * C) * sizeof(float);
    // fast dX kernel: three bf16 planes, channels rounded to 32 on both sides
    const size_t fast = (size_t)(R * S) * ((K + 31) / 32 * 32) * ((C + 31) / 32 * 32) * 6;
    return align_up(generic > fast ? generic : fast, 256);
}

// Geometry of the fast dX kernel for one stride-1 problem (a whole layer, or one class of a strided layer), or
// ok == false when the generic kernel has to serve.  `k` arrives with the problem (N, C, H, Wd, K, R, S, pad, pad_w, P, Q
// and the output mapping) filled in; force_nb != 0 asks for that pixel-block count only.
struct ConvDxPlan { bool ok; int nb; ConvDxArgs args; size_t lds_bytes; int grid; };

static void conv_dx_plan_core(ConvDxPlan &pl, bool i8, int force_nb)
{
    ConvDxArgs &k = pl.args;
    pl.ok = false;
    k.PI = k.H * k.Wd; k.PQ = (k.P * k.Q + 3) / 4 * 4;           // the patch fill reads aligned dwords of a code plane: see conv_dx_codes
    if ((int64_t)(k.C + 32) * k.oPI >= ((int64_t)1 << 31)) return;   // 32-bit offsets inside one image
    k.Cp = (k.C + 31) / 32 * 32;
    const int chunk_k = CDX_KGC * (i8 ? 16 : 8);                 // reduction channels per chunk
    k.KG = (k.K + chunk_k - 1) / chunk_k * CDX_KGC;
    k.n_chunks = k.KG / CDX_KGC;
    const int ncb = k.Cp / 32;
    k.wc = ncb >= 3 ? 4 : ncb;
    k.wpx = 4 / k.wc;
    k.cgroups = (ncb + k.wc - 1) / k.wc;
    k.pw = k.Wd + k.S - 1;
    double best = -1.0;
    const int cand[3] = {7, 4, 2};
    for (int ci = 0; ci < 3; ++ci) {
        const int nb = cand[ci], tile_px = k.wpx * 32 * nb;
        if (force_nb && nb != force_nb) continue;
        const int tiles = (k.PI + tile_px - 1) / tile_px;
        int prow = 0, n_dw = 0;
        for (int t = 0; t < tiles; ++t) {
            const int j0 = t * tile_px, j_end = j0 + tile_px < k.PI ? j0 + tile_px : k.PI;
            const int h_first = j0 / k.Wd, h_last = (j_end - 1) / k.Wd;
            const int p_lo = h_first + k.pad - (k.R - 1);
            const int p_a = p_lo > 0 ? p_lo : 0, p_b = h_last + k.pad < k.P - 1 ? h_last + k.pad : k.P - 1;
            if (h_last - h_first + k.R > prow) prow = h_last - h_first + k.R;
            if (p_b >= p_a) {
                const int f_a = (p_a * k.Q) & ~3, d = ((p_b + 1) * k.Q - f_a + 3) >> 2;
                if (d > n_dw) n_dw = d;
            }
        }
        const int64_t cells = (int64_t)prow * k.pw;
        const size_t lds = (size_t)2 * CDX_KGC * cells * 16;
        // cell indices travel as 16-bit numbers, 0xFFFF meaning "no cell"
        if (lds > (size_t)CDX_MAX_LDS || (int64_t)n_dw * CDX_KGC > 256 * CDX_ITMAX || CDX_KGC * cells >= 0xFFFF) continue;
        // time ~ rounds of workgroups over the chip (two resident per CU) x work per workgroup
        const int64_t grid = (int64_t)k.N * tiles * k.cgroups;
        const double cost = (double)nb * (double)((grid + 511) / 512);
        if (best < 0.0 || cost < best) {
            best = cost; pl.ok = true; pl.nb = nb; pl.lds_bytes = lds;
            k.tiles = tiles; k.prow = prow; k.patch_cells = (int)cells;
        }
    }
    if (!pl.ok) return;
    const int64_t grid = (int64_t)k.N * k.tiles * k.cgroups;
    if (grid > 0x7FFFFFFF) { pl.ok = false; return; }
    pl.grid = (int)grid;
}

ConvDxPlan conv_dx_plan(const ConvArgs &a, bool i8 = false)
{
    ConvDxPlan pl;
    pl.ok = false;
    ConvDxArgs &k = pl.args;
    if (a.stride != 1) return pl;                                // strided layers: conv_dx_strided_plan
    k.N = (int)a.N; k.C = (int)a.C; k.H = (int)a.H; k.Wd = (int)a.Wd; k.K = (int)a.K; k.R = (int)a.R; k.S = (int)a.S;
    k.pad = (int)a.pad; k.pad_w = (int)a.pad;
    k.P = k.H + 2 * k.pad - k.R + 1; k.Q = k.Wd + 2 * k.pad - k.S + 1;
    k.oW = k.Wd; k.oPI = k.H * k.Wd; k.ost = 1; k.oh0 = 0; k.ow0 = 0;
    conv_dx_plan_core(pl, i8, 0);
    return pl;
}

// A strided layer as st*st stride-1 problems, one per class of output pixels (h mod st, w mod st): class (ph, pw) has
// the taps r = r0 + st*t, r0 = (ph + pad) mod st, and reads code row i + (ph + pad - r0)/st - t for its output row i.
// Classes without taps (a 1x1 kernel with stride 2 has three) are all zero: `zero_fill` asks for dX to be cleared first.
struct ConvDxStridedPlan { bool ok, zero_fill; int nb; ConvDxMulti multi; CdxTapMap map; int taps, tap_base[CDX_MAX_CLASSES]; size_t lds_bytes; int grid; };

ConvDxStridedPlan conv_dx_strided_plan(const ConvArgs &a, bool i8)
{
    ConvDxStridedPlan sp;
    sp.ok = false; sp.zero_fill = false; sp.taps = 0; sp.lds_bytes = 0; sp.grid = 0;
    const int st = (int)a.stride, R = (int)a.R, S = (int)a.S, pad = (int)a.pad, H = (int)a.H, Wd = (int)a.Wd;
    if (st < 2 || st * st > CDX_MAX_CLASSES || R * S > 64) return sp;
    const int P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
    // one pixel-block count for all classes (one launch): the one with the least rounds x work per workgroup
    ConvDxStridedPlan best;
    double best_cost = -1.0;
    const int cand[3] = {7, 4, 2};
    for (int attempt = 0; attempt < 3; ++attempt) {
        const int nb = cand[attempt];
        sp.ok = false;
        bool all = true;
        sp.multi.n = 0; sp.taps = 0; sp.zero_fill = false; sp.lds_bytes = 0;
        int64_t grid = 0;
        for (int ph = 0; ph < st && all; ++ph) {
            for (int pw = 0; pw < st && all; ++pw) {
                const int Hv = ph < H ? (H - ph + st - 1) / st : 0, Wv = pw < Wd ? (Wd - pw + st - 1) / st : 0;
                if (Hv == 0 || Wv == 0) continue;                // no such pixels
                const int r0 = (ph + pad) % st, s0 = (pw + pad) % st;
                const int Rv = r0 < R ? (R - r0 + st - 1) / st : 0, Sv = s0 < S ? (S - s0 + st - 1) / st : 0;
                if (Rv == 0 || Sv == 0) { sp.zero_fill = true; continue; }
                ConvDxPlan pl;
                ConvDxArgs &k = pl.args;
                k.N = (int)a.N; k.C = (int)a.C; k.H = Hv; k.Wd = Wv; k.K = (int)a.K; k.R = Rv; k.S = Sv;
                k.pad = (ph + pad - r0) / st; k.pad_w = (pw + pad - s0) / st;
                k.P = P; k.Q = Q;
                k.oW = Wd; k.oPI = H * Wd; k.ost = st; k.oh0 = ph; k.ow0 = pw;
                conv_dx_plan_core(pl, i8, nb);
                if (!pl.ok) { all = false; break; }
                // this class's prepared taps follow the earlier classes'
                for (int t = 0; t < Rv; ++t)
                    for (int u = 0; u < Sv; ++u) sp.map.real[sp.taps + t * Sv + u] = (uint8_t)((r0 + st * t) * S + (s0 + st * u));
                k.codes = nullptr; k.wp = nullptr; k.dX = nullptr; k.scale = Scale{1.0f, nullptr};   // set at the launch
                sp.multi.cls[sp.multi.n] = k;
                sp.multi.first[sp.multi.n] = (int)grid;
                sp.tap_base[sp.multi.n] = sp.taps;
                sp.taps += Rv * Sv;
                grid += pl.grid;
                if (pl.lds_bytes > sp.lds_bytes) sp.lds_bytes = pl.lds_bytes;
                ++sp.multi.n;
            }
        }
        if (!all || grid > 0x7FFFFFFF) continue;
        sp.multi.first[sp.multi.n] = (int)grid;
        sp.ok = true; sp.nb = nb; sp.grid = (int)grid;
        const double cost = (double)nb * (double)((grid + 511) / 512);
        if (best_cost < 0.0 || cost < best_cost) { best_cost = cost; best = sp; }
    }
    if (best_cost < 0.0) { sp.ok = false; return sp; }
    sp = best;
    for (int t = sp.taps; t < 64; ++t) sp.map.real[t] = 0;
    return sp;
}


// Geometry of the fast dW kernel (conv_dw_kernel.h), or ok == false when the generic kernel has to serve.
struct ConvDwPlan { bool ok; int mb; ConvDwArgs args; size_t lds_bytes, partial_bytes; int grid, reduce_grid; };

ConvDwPlan conv_dw_plan(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t pad, bool i8)
{
    ConvDwPlan pl;
    pl.ok = false; pl.partial_bytes = 0; pl.lds_bytes = 0;
    ConvDwArgs &k = pl.args;
    // one accumulator per tap: compiled tap counts only.  (A 1x1 instantiation was measured: a single tap
    // leaves the stagers far behind the matrix cores, and the generic kernel is faster there.)
    if (!(R == 3 && S == 3)) return pl;
    if (pad > 1) return pl;                                          // compiled paddings: 0 and 1
    const int64_t P = H + 2 * pad - R + 1, Q = Wd + 2 * pad - S + 1;
    if ((H * Wd) % 4 || (P * Q) % 4) return pl;                     // rows are fetched as aligned 4-element pieces
    if (C * H * Wd >= ((int64_t)1 << 29) || K * P * Q >= ((int64_t)1 << 29) || K * C * R * S >= ((int64_t)1 << 31)) return pl;
    k.N = (int)N; k.C = (int)C; k.H = (int)H; k.Wd = (int)Wd; k.K = (int)K; k.P = (int)P; k.Q = (int)Q; k.pad = (int)pad;
    k.Ct = k.C; k.Kt = k.K;                                          // one group of a grouped layer: set at the launch
    const int FRAG = i8 ? 16 : 8, KSTEP = 2 * FRAG, ESZ = i8 ? 1 : 2, PL = i8 ? 1 : 3, CQL = 128, XQL = 64;
    int64_t pw = Wd + pad;
    const int64_t over = S - 1 - pad > 0 ? S - 1 - pad : 0;
    if (Q + over > pw) pw = Q + over;
    pw = (pw + FRAG - 1) / FRAG * FRAG;
    if (pw > 256) return pl;
    k.PW = (int)pw;
    const int t_max = CDW_M8 + (int)((R - 1) * pw + pad);
    double best = -1.0;
    for (int mb = 1; mb >= 1 && !pl.ok; --mb) {
        const int TK = 64 * mb, TC = 64;
        for (int ru = 1; ru <= H && ru * Wd <= 4 * XQL - 9 && ru * pw <= 320; ++ru) {
            const int tpc = (int)(ru * pw);
            if (tpc % KSTEP) continue;
            const int len = (tpc + t_max + FRAG + 3) / 4 * 4;
            const int nr = (int)((len - CDW_M8 - 1) / pw) + 2;
            const int nqc = (int)((nr * Q + 9) / 4), nqx = (int)((ru * Wd + 9) / 4);
            if (nqc > CQL || nqx > XQL) continue;
            int xc = tpc / FRAG; if (xc % 2 == 0) ++xc;              // odd cell counts spread a fragment read over the banks
            int cc = (len + FRAG - 1) / FRAG; if (cc % 2 == 0) ++cc;
            const size_t lds = 2 * ((size_t)PL * TC * xc * FRAG * ESZ + (size_t)TK * cc * FRAG * ESZ);   // double buffered
            if (lds > (size_t)CDW_MAX_LDS) continue;
            const int chunks = (int)((H + ru - 1) / ru);
            const double cost = (double)chunks * (tpc + 64.0);      // matrix-core steps plus a fixed cost per unit
            if (best < 0.0 || cost < best) {
                best = cost; pl.ok = true; pl.mb = mb; pl.lds_bytes = lds;
                k.RU = ru; k.TPc = tpc; k.chunks = chunks; k.lenC = len; k.pitchX = xc * FRAG; k.pitchC = cc * FRAG;
                k.NR = nr; k.nqx = nqx; k.nqc = nqc; k.lds_cells = (int)(lds / 16);
            }
        }
    }
    if (!pl.ok) return pl;
    k.row4x = Wd % 4 == 0; k.row4c = Q % 4 == 0;
    k.row2x = Wd % 2 == 0; k.row2c = Q % 2 == 0;
    // code rows of whole 8-code pieces under the whole-piece staging path (bf16 modes): half as many, twice as wide code loads
    k.c8 = !i8 && k.row4x && k.row4c && Q % 8 == 0;
    if (k.c8) k.nqc = (k.nqc + 1) / 2;
    k.xshift = k.nqx <= 16 ? 4 : k.nqx <= 32 ? 5 : 6;
    k.cshift = k.nqc <= 32 ? 5 : k.nqc <= 64 ? 6 : 7;
    const int TK = 64 * pl.mb;
    k.tiles_k = (int)((K + TK - 1) / TK); k.tiles_c = (int)((C + 63) / 64);
    const int64_t tiles = (int64_t)k.tiles_k * k.tiles_c;
    const int64_t units = N * k.chunks;
    if (units >= ((int64_t)1 << 31) || tiles > 65535) { pl.ok = false; return pl; }
    k.units = (int)units;
    int64_t want = tiles >= 256 ? 1 : 256 / tiles;                   // one workgroup per CU
    if (want > units) want = units;
    k.units_per_split = (int)((units + want - 1) / want);
    k.n_split = (int)((units + k.units_per_split - 1) / k.units_per_split);
    const int64_t ne = R * S * pl.mb * 16;
    pl.partial_bytes = k.n_split > 1 ? (size_t)tiles * k.n_split * ne * 256 * 4 : 0;
    pl.grid = (int)(tiles * k.n_split);
    pl.reduce_grid = (int)(tiles * (ne / 4) * 16);                  // (tile, group of 4 elements, 16 of the 256 slots)
    return pl;
}

// Geometry of the int8 3x3 dW kernel with transposed cells (conv_dw_i8_kernel.h); ok == false when it does not apply.
struct ConvDwI8Plan { bool ok; ConvDwI8Args args; size_t lds_bytes, partial_bytes; int grid, reduce_grid; };

ConvDwI8Plan conv_dw_i8_plan(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t pad)
{
    ConvDwI8Plan pl;
    pl.ok = false; pl.partial_bytes = 0; pl.lds_bytes = 0;
    ConvDwI8Args &k = pl.args;
    if (!(R == 3 && S == 3 && pad == 1)) return pl;
    if (Wd % 4 || Wd < 16 || Wd > 224 || H < 1) return pl;           // 16-byte loads at dword-aligned addresses inside a row
    if (H * Wd >= ((int64_t)1 << 24) || K * C * 9 >= ((int64_t)1 << 31)) return pl;   // 64 channels of a tile: 32-bit offsets
    const int pw = (int)((Wd + 1 + 15) / 16 * 16), cpr = pw / 16, dc = (int)((Wd + 15) / 16);
    double best = -1.0;
    for (int ru = 1; ru <= H; ++ru) {
        const int xpairs = ru * dc, cpairs = (ru + 2) * dc;
        if (cpairs > 64) break;                                      // 256 stager threads cover >= 4 channels a pass, 16 passes at most
        const int n_steps = (ru * cpr + 1) / 2;
        const int xcells = (2 * n_steps) | 1;                        // odd: a fragment read spreads over the banks
        int ccells = (ru + 2) * cpr + 2;                             // the patch and a zero cell at either end
        if (ccells < 2 * n_steps + 2 * cpr + 2) ccells = 2 * n_steps + 2 * cpr + 2;   // the last step's reach
        ccells |= 1;
        const size_t lds = 2 * (size_t)64 * (xcells + ccells) * 16 + 256 * 16;   // two buffers and a spare cell per stager thread
        if (lds > (size_t)CDW_MAX_LDS) break;
        const int chunks = (int)((H + ru - 1) / ru);
        const double cost = (double)chunks * (n_steps + 1.5);       // matrix-core steps plus a fixed cost per unit
        if (best < 0.0 || cost < best) {
            best = cost; pl.ok = true; pl.lds_bytes = lds;
            k.RU = ru; k.chunks = chunks; k.n_steps = n_steps; k.xcells = xcells; k.ccells = ccells;
            k.xpairs = xpairs; k.cpairs = cpairs; k.lds_cells = (int)(lds / 16) - 256;
        }
    }
    if (!pl.ok) return pl;
    k.N = (int)N; k.C = (int)C; k.H = (int)H; k.Wd = (int)Wd; k.K = (int)K; k.PW = pw; k.CPR = cpr; k.DC = dc;
    k.Ct = k.C; k.Kt = k.K;
    k.tiles_k = (int)((K + 63) / 64); k.tiles_c = (int)((C + 63) / 64);
    const int64_t tiles = (int64_t)k.tiles_k * k.tiles_c, units = N * k.chunks;
    if (units >= ((int64_t)1 << 31) || tiles > 65535) { pl.ok = false; return pl; }
    k.units = (int)units;
    int64_t want = tiles >= 256 ? 1 : 256 / tiles;                   // one workgroup per CU
    if (want > units) want = units;
    k.units_per_split = (int)((units + want - 1) / want);
    k.n_split = (int)((units + k.units_per_split - 1) / k.units_per_split);
    pl.partial_bytes = k.n_split > 1 ? (size_t)tiles * k.n_split * 144 * 256 * 4 : 0;
    pl.grid = (int)(tiles * k.n_split);
    pl.reduce_grid = (int)(tiles * 36 * 16);                         // (tile, group of 4 accumulator elements, 16 of the 256 slots)
    return pl;
}

hipError_t launch_conv_dw_i8(const ConvDwI8Plan &pl, hipStream_t s)
{
    static bool raised = false;                                      // more than 64 KiB of dynamic LDS: allowed per kernel, once
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_dw_i8_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, CDW_MAX_LDS);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL(conv_dw_i8_kernel, dim3(pl.grid), dim3(512), pl.lds_bytes, s, pl.args);
    if (pl.args.n_split > 1) {
        ConvDwArgs r{};                                              // the reduction reads the partial layout of both dW kernels
        r.partial = pl.args.partial; r.dW = pl.args.dW; r.n_split = pl.args.n_split; r.tiles_k = pl.args.tiles_k;
        r.K = pl.args.K; r.C = pl.args.C; r.scale = Scale{1.0f, nullptr}; r.gate = pl.args.gate;
        hipLaunchKernelGGL((conv_dw_reduce_kernel<MODE_I8, 3, 3, 1>), dim3(pl.reduce_grid), dim3(256), 0, s, r);
    }
    return hipGetLastError();
}

template <int MODE, int R, int S, int PAD, int MB, int ROWS>
hipError_t launch_conv_dw_fast_as(const ConvDwPlan &pl, hipStream_t s)
{
    // more than 64 KiB of dynamic LDS has to be allowed per kernel, once
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_dw_kernel<MODE, R, S, PAD, MB, ROWS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, CDW_MAX_LDS);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((conv_dw_kernel<MODE, R, S, PAD, MB, ROWS>), dim3(pl.grid), dim3(512), pl.lds_bytes, s, pl.args);
    if (pl.args.n_split > 1)
        hipLaunchKernelGGL((conv_dw_reduce_kernel<MODE, R, S, MB>), dim3(pl.reduce_grid), dim3(256), 0, s, pl.args);
    return hipGetLastError();
}

template <int MODE, int R, int S, int PAD, int MB>
hipError_t launch_conv_dw_fast(const ConvDwPlan &pl, hipStream_t s)
{
    // rows that are whole numbers of aligned 4-element pieces have a staging path of their own
    // (and code rows of whole 8-code pieces, bf16 modes, one that loads the codes 8 bytes at a time)
    if constexpr (MODE != MODE_I8) {
        if (pl.args.c8) return launch_conv_dw_fast_as<MODE, R, S, PAD, MB, 2>(pl, s);
    }
    return pl.args.row4x && pl.args.row4c ? launch_conv_dw_fast_as<MODE, R, S, PAD, MB, 1>(pl, s)
                                          : launch_conv_dw_fast_as<MODE, R, S, PAD, MB, 0>(pl, s);
}

// ---- fast fully connected path (fc_kernel.h) -------------------------------------------------------
struct FcPlan { int tiles_m, tiles_n, n_split, k_per_split; int64_t tiles; size_t partial_bytes; };

// Split the reduction of a product with few tiles into about two items per CU, never below 8 K steps per
// item (the length of a dW item at batch 256, so the persistent workgroups stay balanced).  Every split
// costs a partial write + read.
FcPlan fc_plan(int64_t M, int64_t N, int64_t K, int tm = FC_TM, int tn = FC_TN)
{
    FcPlan pl;
    pl.tiles_m = (int)((M + tm - 1) / tm);
    pl.tiles_n = (int)((N + tn - 1) / tn);
    pl.tiles = (int64_t)pl.tiles_m * pl.tiles_n;
    const int64_t steps = (K + FC_KT - 1) / FC_KT;
    int64_t want = (512 + pl.tiles - 1) / pl.tiles;
    const int64_t max_n = steps / 8 > 0 ? steps / 8 : 1;
    if (want > max_n) want = max_n;
    if (want < 1) want = 1;
    const int64_t per = (steps + want - 1) / want;
    pl.k_per_split = (int)(per * FC_KT);
    pl.n_split = (int)((steps + per - 1) / per);
    pl.partial_bytes = pl.n_split > 1 ? (size_t)pl.tiles * pl.n_split * tm * tn * sizeof(float) : 0;
    return pl;
}

// Plans of the two products for the kernel with staging and multiplying wavefronts: reductions are split
// into items of about half a workgroup's share of all K steps (one workgroup per CU), at least 8 steps.
void fc2_plans(int64_t B, int64_t in, int64_t out, bool want_dx, bool want_dw, FcPlan &dx, FcPlan &dw, int kt = FC2_KT)
{
    auto base = [kt](int64_t M, int64_t N, int64_t K, FcPlan &pl) {
        pl.tiles_m = (int)((M + FC2_TM - 1) / FC2_TM);
        pl.tiles_n = (int)((N + FC2_TN - 1) / FC2_TN);
        pl.tiles = (int64_t)pl.tiles_m * pl.tiles_n;
        return (K + kt - 1) / kt;
    };
    const int64_t sx = base(B, in, out, dx), sw = base(out, in, B, dw);
    const int64_t all = (want_dx ? dx.tiles * sx : 0) + (want_dw ? dw.tiles * sw : 0);
    // two items per workgroup when both products share the launch (a dX item and dW tiles interleave well), one when a
    // product runs alone (half the split-K partials: measured 37 instead of 47 us for dX of the 4096x4096 layer)
    int64_t len = all / (want_dx && want_dw ? 512 : 256);
    if (len < 8) len = 8;
    const bool alone = want_dx != want_dw;
    auto split = [len, kt, alone](int64_t steps, FcPlan &pl) {
        int64_t n = (steps + len / 2) / len;
        // a product that runs alone: at most one item per workgroup (256 of them), so that no workgroup takes a second
        // item while the others idle (8 tiles x 33 splits = 264 items ran as two rounds)
        if (alone && pl.tiles <= 256 && n * pl.tiles > 256) n = 256 / pl.tiles;
        if (n < 1) n = 1;
        const int64_t per = (steps + n - 1) / n;
        pl.k_per_split = (int)(per * kt);
        pl.n_split = (int)((steps + per - 1) / per);
        pl.partial_bytes = pl.n_split > 1 ? (size_t)pl.tiles * pl.n_split * FC2_TM * FC2_TN * sizeof(float) : 0;
    };
    split(sx, dx); split(sw, dw);
}

// The two products on two groups of workgroups (FcPairArgs::gx) where that needs fewer split-K partials than the common
// list for the same longest workgroup: group sizes in proportion to the products' K steps (multiples of 8: every XCD
// gets its share of both), a split product cut into about one item per workgroup of its group.  Returns gx, or 0 to keep
// the common list; dx and dw are replaced by the group plan when it is taken.
int fc2_group_plan(int64_t B, int64_t in, int64_t out, FcPlan &dx, FcPlan &dw, int kt = FC2_KT)
{
    const int G = 256;
    const int64_t sx = (out + kt - 1) / kt, sw = (B + kt - 1) / kt;
    const int64_t all_x = dx.tiles * sx, all_w = dw.tiles * sw;
    if (dx.tiles * dx.n_split + dw.tiles * dw.n_split < G) return 0;
    int gx = (int)((G * all_x + (all_x + all_w) / 2) / (all_x + all_w) + 4) / 8 * 8;
    gx = gx < 8 ? 8 : gx > G - 8 ? G - 8 : gx;
    auto cut = [kt](int64_t steps, FcPlan pl, int g) {
        int64_t n = pl.tiles >= g ? 1 : g / pl.tiles;
        const int64_t most = steps / 8 > 0 ? steps / 8 : 1;            // at least eight K steps per item
        if (n > most) n = most;
        const int64_t per = (steps + n - 1) / n;
        pl.k_per_split = (int)(per * kt);
        pl.n_split = (int)((steps + per - 1) / per);
        pl.partial_bytes = pl.n_split > 1 ? (size_t)pl.tiles * pl.n_split * FC2_TM * FC2_TN * sizeof(float) : 0;
        return pl;
    };
    const FcPlan gdx = cut(sx, dx, gx), gdw = cut(sw, dw, G - gx);
    auto rounds = [](const FcPlan &pl, int g) { return (pl.tiles * pl.n_split + g - 1) / g * (int64_t)(pl.k_per_split); };
    const int64_t longest_groups = rounds(gdx, gx) > rounds(gdw, G - gx) ? rounds(gdx, gx) : rounds(gdw, G - gx);
    // the common list: workgroup w takes items p*G + (w or G-1-w) of the concatenated lists
    const int64_t n0 = dx.tiles * dx.n_split, total = n0 + dw.tiles * dw.n_split;
    int64_t longest_common = 0;
    for (int w = 0; w < G; ++w) {
        int64_t len = 0;
        for (int64_t ps = 0; ps * G < total; ++ps) {
            const int64_t t = ps * G + ((ps & 1) ? G - 1 - w : w);
            if (t < total) len += t < n0 ? dx.k_per_split : dw.k_per_split;
        }
        if (len > longest_common) longest_common = len;
    }
    if (longest_groups > longest_common || gdx.partial_bytes + gdw.partial_bytes >= dx.partial_bytes + dw.partial_bytes) return 0;
    if ((gdx.tiles * gdx.n_split + gx - 1) / gx > FC2_MAX_ITEMS || (gdw.tiles * gdw.n_split + G - gx - 1) / (G - gx) > FC2_MAX_ITEMS) return 0;
    dx = gdx; dw = gdw;
    return gx;
}

bool fc_fast_ok(bool a_kfast, const int8_t *A, int64_t lda, const float *B, int64_t ldb, int64_t M, int64_t N, const float *out)
{
    if (N < 4 || N % 4 || ldb % 4 || ((uintptr_t)B % 16) || ((uintptr_t)out % 8)) return false;
    if (lda % 4 || ((uintptr_t)A % 4)) return false;
    if (!a_kfast && (M < 4 || M % 4)) return false;
    return true;
}

FcProblem fc_problem(bool a_kfast, const int8_t *A, int64_t lda, const float *B, int64_t ldb, int M, int N, int K,
                     Scale scale, float *out, const FcPlan &pl, char *&scratch)
{
    FcProblem p;
    p.A = A; p.lda = lda; p.B = B; p.ldb = ldb; p.out = out; p.ldc = N;
    p.M = M; p.N = N; p.K = K; p.scale = scale; p.a_kfast = a_kfast ? 1 : 0;
    p.tiles_m = pl.tiles_m; p.n_split = pl.n_split; p.k_per_split = pl.k_per_split;
    p.n_items = (int)(pl.tiles * pl.n_split);
    p.partial = (float *)scratch;
    p.nt_pq = 0; p.nt_spi = 1; p.nt_a_img = 0; p.nt_b_img = 0;
    scratch += align_up(pl.partial_bytes, 256);
    return p;
}

}  // namespace

size_t linear_scratch_bytes(int64_t B, int64_t in, int64_t out)
{
    // generic kernel: split-K partials of the larger of the two products, at the split the launcher would choose
    auto part = [](int64_t M, int64_t N, int64_t K) {
        int64_t tiles = ((M + TM - 1) / TM) * ((N + TN - 1) / TN);
        Split sp = choose_split(tiles, K, 16);          // smallest K step (fp32 mode) gives the largest split
        return sp.n > 1 ? (size_t)sp.n * M * N * 4 : (size_t)0;
    };
    size_t a = part(B, in, out), b = part(out, in, B);
    const size_t generic = align_up(a > b ? a : b, 256);
    // fast path: both products in one launch, each with its own partials
    const FcPlan dx = fc_plan(B, in, out), dw = fc_plan(out, in, B);
    size_t fast = align_up(dx.partial_bytes, 256) + align_up(dw.partial_bytes, 256);
    for (int m = 1; m < 4; ++m) {                               // every combination of products a call can ask for
        FcPlan dx2, dw2;
        for (int kt = FC2_KT; kt <= FC2I_KT; kt *= 2) {              // the bf16 kernel's K step and the int8 kernel's
            fc2_plans(B, in, out, (m & 1) != 0, (m & 2) != 0, dx2, dw2, kt);
            const size_t fast2 = ((m & 1) ? align_up(dx2.partial_bytes, 256) : 0) + ((m & 2) ? align_up(dw2.partial_bytes, 256) : 0);
            if (fast2 > fast) fast = fast2;
        }
    }
    const size_t gather = align_up(linear_gather_scratch_bytes(B, in, out), 256);      // split partials of the gather dX kernel
    const size_t mfma = generic > fast ? generic : fast;
    return (mfma > gather ? mfma : gather) + 256;
}

// dW of a 1x1, stride-1, unpadded convolution: dW[k][c] = sum_n sum_p code[n][k][p] X[n][c][p] is the batched,
// reduction-contiguous form of the FC kernels (fc2_kernel.h / fc2_i8_kernel.h, NT) straight on the NCHW tensors: no copy
// pass.  kt = reduction indices per K step of the kernel (32 with fp32 activations, 64 with int8 activations).
struct Conv1x1Plan { bool ok; int n_split, imgs_per_split, spi, tiles_m, tiles_n, kt; size_t partial_bytes; };

Conv1x1Plan conv1x1_dw_plan(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t pad, int64_t stride,
                            int kt = FC2_KT)
{
    Conv1x1Plan pl;
    pl.ok = false; pl.partial_bytes = 0;
    const int64_t PQ = H * Wd;
    if (!(R == 1 && S == 1 && pad == 0 && stride == 1)) return pl;
    pl.kt = kt;
    if (K < FC2_TM / 4 || C < 4 || C % 4 || PQ % 4 || PQ < kt) return pl;           // row tiles at least a quarter full (lowering costs more than the idle rows); 16-byte loads and stores
    if (C * PQ >= ((int64_t)1 << 29) || K * PQ >= ((int64_t)1 << 31) || K * C >= ((int64_t)1 << 30)) return pl;   // 32-bit lane offsets
    pl.spi = (int)((PQ + kt - 1) / kt);
    if (N * pl.spi >= ((int64_t)1 << 25)) return pl;                              // the reduction axis counts windows of kt
    pl.tiles_m = (int)((K + FC2_TM - 1) / FC2_TM); pl.tiles_n = (int)((C + FC2_TN - 1) / FC2_TN);
    const int64_t tiles = (int64_t)pl.tiles_m * pl.tiles_n;
    int64_t n = tiles >= 256 ? 1 : 256 / tiles;                                   // at most one item per workgroup
    if (n > N) n = N;
    while (n > 1 && ((N + n - 1) / n) * pl.spi < 8) --n;                          // at least eight steps per item
    pl.imgs_per_split = (int)((N + n - 1) / n);
    pl.n_split = (int)((N + pl.imgs_per_split - 1) / pl.imgs_per_split);
    if (tiles * pl.n_split > (int64_t)FC2_MAX_ITEMS * 256) return pl;
    pl.partial_bytes = pl.n_split > 1 ? (size_t)tiles * pl.n_split * FC2_TM * FC2_TN * sizeof(float) : 0;
    pl.ok = true;
    return pl;
}

template <bool I8>
hipError_t launch_conv1x1_dw(const ConvArgs &a, const Conv1x1Plan &pl, const int8_t *codes, Scale scale, char *scratch, hipStream_t s)
{
    static bool raised = false;
    if (!raised) {
        hipError_t e = I8 ? hipFuncSetAttribute(reinterpret_cast<const void *>(&fc2_i8_pair_kernel<true>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, FC2I_LDS_BYTES)
                          : hipFuncSetAttribute(reinterpret_cast<const void *>(&fc2_pair_kernel<true, 3>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, FC2_LDS_BYTES);
        if (e != hipSuccess) return e;
        if (!I8) e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fc2_pair_kernel<true, 2>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, FC2_LDS_BYTES);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int64_t PQ = a.H * a.Wd;
    FcPairArgs pa;
    FcProblem &p = pa.prob[0];
    p.A = codes; p.lda = PQ; p.B = (const float *)a.X; p.ldb = PQ; p.out = (float *)a.dW; p.ldc = a.C;
    p.partial = (float *)scratch;
    p.M = (int)a.K; p.N = (int)a.C; p.K = (int)(a.N * pl.spi * pl.kt);
    p.k_per_split = pl.imgs_per_split * pl.spi * pl.kt; p.n_split = pl.n_split; p.tiles_m = pl.tiles_m;
    p.n_items = pl.tiles_m * pl.tiles_n * pl.n_split;
    p.scale = scale; p.a_kfast = 1;
    p.nt_pq = (int)PQ; p.nt_spi = pl.spi; p.nt_a_img = a.kt() * PQ; p.nt_b_img = a.ct() * PQ;
    pa.prob[1] = p;
    pa.prob[1].n_items = 0;
    pa.stats = StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr};
    pa.gate = a.gate;
    const int grid = p.n_items < 256 ? p.n_items : 256;
    if constexpr (I8) hipLaunchKernelGGL(fc2_i8_pair_kernel<true>, dim3(grid), dim3(512), FC2I_LDS_BYTES, s, pa);
    else if (a.two_planes) hipLaunchKernelGGL((fc2_pair_kernel<true, 2>), dim3(grid), dim3(512), FC2_LDS_BYTES, s, pa);
    else              hipLaunchKernelGGL((fc2_pair_kernel<true, 3>), dim3(grid), dim3(512), FC2_LDS_BYTES, s, pa);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (pl.n_split > 1) {
        const int tiles = pl.tiles_m * pl.tiles_n;
        if constexpr (I8) hipLaunchKernelGGL(fc2_i8_reduce_kernel, dim3(32 * tiles), dim3(256), 0, s, pa, tiles);
        else              hipLaunchKernelGGL(fc2_reduce_kernel, dim3(32 * tiles), dim3(256), 0, s, pa, tiles);
        e = hipGetLastError();
    }
    return e;
}

// dW lowered to the fully connected kernels (conv_lower.h): taken for shapes the convolution dW kernels decline when the
// column matrix is small enough to sit in the workspace.  esz = bytes per activation (4, or 1 in the 8-bit modes).
struct ConvLowerPlan { bool ok, vec4; int64_t NPQ, CRS; size_t codes_bytes, col_bytes, fc_bytes, bytes; Im2colArgs im; size_t lds_bytes; };

ConvLowerPlan conv_dw_lower_plan(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t pad, int64_t stride, int esz)
{
    ConvLowerPlan lp;
    lp.ok = false; lp.bytes = 0;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    lp.NPQ = N * P * Q; lp.CRS = C * R * S;
    // the product kernels want: reduction rows of the codes a multiple of 4 bytes, columns a multiple of 4 (fp32) or 8
    // (int8) elements; below that, or when the products are tiny, the generic kernel serves
    if (lp.NPQ % 4 || lp.NPQ < 64 || lp.CRS % (esz == 4 ? 4 : 8) || K < 16) return lp;
    if (lp.NPQ * lp.CRS >= ((int64_t)1 << 30) || K * lp.NPQ >= ((int64_t)1 << 30) || K * lp.CRS >= ((int64_t)1 << 30)) return lp;
    if ((double)lp.NPQ * lp.CRS * K < 2e8) return lp;              // launch-bound sizes: three more launches do not pay (measured)
    lp.col_bytes = align_up((size_t)(lp.NPQ * lp.CRS) * esz, 256);
    if (lp.col_bytes > ((size_t)256 << 20)) return lp;              // keep the workspace modest
    lp.codes_bytes = align_up((size_t)(K * lp.NPQ), 256);
    lp.fc_bytes = linear_scratch_bytes(K, lp.CRS, lp.NPQ);
    lp.bytes = lp.codes_bytes + lp.col_bytes + lp.fc_bytes;
    Im2colArgs &m = lp.im;
    m.N = (int)N; m.C = (int)C; m.H = (int)H; m.Wd = (int)Wd; m.R = (int)R; m.S = (int)S; m.pad = (int)pad; m.st = (int)stride;
    m.P = (int)P; m.Q = (int)Q;
    // channels per workgroup: enough for 256 consecutive entries per output pixel; output rows per workgroup: what fits
    const int64_t RS = R * S;
    int64_t ct = (256 + RS - 1) / RS;
    if (ct < 32) ct = 32;
    ct = (ct + 3) / 4 * 4;
    if (ct > C) ct = C;
    lp.vec4 = RS % 4 == 0 || (C % 4 == 0 && ct % 4 == 0);             // every tile's entries and every matrix row: multiples of 4
    if (ct * RS >= (1 << 16) || R > 63 || S > 63) return lp;          // the entry table packs r and s into 6 bits each
    const size_t budget = 40 * 1024;
    int64_t pb = 0;
    for (int64_t t = 1; t <= P; ++t) {
        const int64_t hb = (t - 1) * stride + R < H ? (t - 1) * stride + R : H;
        if ((size_t)(ct * (hb * Wd + 1)) * esz > budget) break;
        pb = t;
    }
    if (pb == 0) return lp;
    const int64_t ctiles = (C + ct - 1) / ct;
    while (pb > 1 && N * ((P + pb - 1) / pb) * ctiles < 1024) --pb;   // enough workgroups to fill the chip
    const int64_t hb = (pb - 1) * stride + R < H ? (pb - 1) * stride + R : H;
    int64_t pitch = hb * Wd;
    if (pitch % 2 == 0) ++pitch;                                      // odd: the channels of a pixel's entries spread over the banks
    if (ct * pitch >= (1 << 20)) return lp;
    m.CT = (int)ct; m.ctiles = (int)((C + ct - 1) / ct);
    m.PB = (int)pb; m.bands = (int)((P + pb - 1) / pb);
    m.pitch = (int)pitch;
    lp.lds_bytes = (size_t)((ct * RS * 4 + 15) & ~15) + (size_t)(ct * pitch) * esz;
    if (N * m.bands * m.ctiles > 0x7FFFFFFF) return lp;
    lp.ok = true;
    return lp;
}

size_t conv_scratch_bytes(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t pad, int64_t stride)
{
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    auto part = [](int64_t M, int64_t Nn, int64_t Kr, int64_t gran) {
        int64_t tiles = ((M + TM - 1) / TM) * ((Nn + TN - 1) / TN);
        Split sp = choose_split(tiles, Kr, (int)gran);
        return sp.n > 1 ? (size_t)sp.n * M * Nn * 4 : (size_t)0;
    };
    size_t dx = part(N * H * Wd, C, R * S * ((K + 7) / 8 * 8), 16);
    const int64_t PQp16 = (P * Q + 15) / 16 * 16;
    size_t dw = part(K, C * R * S, N * PQp16, 16);
    size_t big = dx > dw ? dx : dw;
    bool fast[2] = {false, false};                                   // a convolution dW kernel serves fp32 / int8 activations
    for (int i8 = 0; i8 < 2; ++i8) {
        const ConvDwPlan pl = conv_dw_plan(N, C, H, Wd, K, R, S, pad, i8 != 0);
        if (pl.ok && stride == 1) fast[i8] = true;
        if (pl.ok && pl.partial_bytes > big) big = pl.partial_bytes;
    }
    const ConvDwI8Plan p8 = conv_dw_i8_plan(N, C, H, Wd, K, R, S, pad);
    if (p8.ok && stride == 1) fast[1] = true;
    if (p8.ok && p8.partial_bytes > big) big = p8.partial_bytes;
    for (int i8 = 0; i8 < 2; ++i8) {
        const Conv1x1Plan p1 = conv1x1_dw_plan(N, C, H, Wd, K, R, S, pad, stride, i8 ? FC2I_KT : FC2_KT);
        if (p1.ok && p1.partial_bytes > big) big = p1.partial_bytes;
    }
    const size_t padded = (size_t)(N * K * ((P * Q + 3) / 4 * 4));    // dX: the codes in planes that start on 4-byte boundaries
    if (padded > big) big = padded;
    // dW lowered to the FC kernels: room for the column matrix only where no convolution dW kernel serves the shape (a
    // call whose pointers those kernels cannot take then runs on the generic kernel, which needs less)
    for (int i8 = 0; i8 < 2; ++i8) {
        if (fast[i8]) continue;
        const ConvLowerPlan lp = conv_dw_lower_plan(N, C, H, Wd, K, R, S, pad, stride, i8 ? 1 : 4);
        if (lp.ok && lp.bytes > big) big = lp.bytes;
    }
    return relayout_bytes(K, C, R, S) + align_up(big, 256) + 256;
}

// ------------------------------------------------------------------------------------------------
// Fully connected layer.  dX = q.W : rows b, cols i, reduction o.   dW = q^T.X : rows o, cols i, reduction b.
// ------------------------------------------------------------------------------------------------
hipError_t launch_linear_mfma(const LinearArgs &a, hipStream_t s)
{
    const int B = (int)a.B, in = (int)a.in, out = (int)a.out;
    hipError_t e = hipSuccess;
    RowMajorOut om{a.in};
    StatsJob pending = a.stats_job;
    if (a.plan_only && (!a.codes || a.W8)) { *a.plan_only = 1; return hipSuccess; }
    if (a.codes && a.W8) {
        // full 8-bit mode: both products on int8 matrix cores, exact int32 results
        auto i8_ok = [&](bool a_kfast, const void *Bop, const void *outp, int64_t M) {
            if (in < 8 || in % 8 || ((uintptr_t)Bop % 8) || ((uintptr_t)outp % 16)) return false;     // 8-byte loads, 16-byte stores
            if (out % 4 || ((uintptr_t)a.codes % 4)) return false;
            if (!a_kfast && (M < 16 || M % 4)) return false;
            return true;
        };
        bool dx_fast = a.dX && i8_ok(true, a.W8, a.dX, B) && out >= FC2I_KT && B > FC2_TM / 2;
        bool dw_fast = a.dW && i8_ok(false, a.X, a.dW, out) && B >= FC2I_KT && out > FC2_TM / 2;
        if ((int64_t)B * in >= (1ll << 30) || (int64_t)out * in >= (1ll << 30) || (int64_t)B * out >= (1ll << 30)) dx_fast = dw_fast = false;
        FcPlan pdx, pdw;
        if (dx_fast || dw_fast) {
            fc2_plans(B, in, out, dx_fast, dw_fast, pdx, pdw, FC2I_KT);
            const int64_t items = (dx_fast ? pdx.tiles * pdx.n_split : 0) + (dw_fast ? pdw.tiles * pdw.n_split : 0);
            if (items > (int64_t)FC2_MAX_ITEMS * 256) dx_fast = dw_fast = false;
        }
        int gx = 0;
        if (dx_fast && dw_fast) gx = fc2_group_plan(B, in, out, pdx, pdw, FC2I_KT);
        if (dx_fast || dw_fast) {
            static bool raised = false;
            if (!raised) {
                e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fc2_i8_pair_kernel<false>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, FC2I_LDS_BYTES);
                if (e != hipSuccess) return e;
                raised = true;
            }
            char *scratch = (char *)a.scratch;
            FcPairArgs pa;
            if (!dx_fast) { pdx.n_split = 1; pdx.partial_bytes = 0; }
            if (!dw_fast) { pdw.n_split = 1; pdw.partial_bytes = 0; }
            pa.prob[0] = fc_problem(true, a.codes, a.out, (const float *)a.W8, a.in, B, in, out, Scale{1.0f, nullptr}, a.dX, pdx, scratch);
            pa.prob[1] = fc_problem(false, a.codes, a.out, (const float *)a.X, a.in, out, in, B, Scale{1.0f, nullptr}, (float *)a.dW, pdw, scratch);
            if (!dx_fast) pa.prob[0].n_items = 0;
            if (!dw_fast) pa.prob[1].n_items = 0;
            if ((size_t)(scratch - (char *)a.scratch) > a.scratch_bytes) return hipErrorInvalidValue;
            pa.stats = pending;
            pending.n = 0; pending.bias_len = 0;
            pa.gx = gx; pa.gate = a.gate;
            const int total = pa.prob[0].n_items + pa.prob[1].n_items;
            const int grid = total < 256 ? total : 256;
            hipLaunchKernelGGL(fc2_i8_pair_kernel<false>, dim3(grid), dim3(512), FC2I_LDS_BYTES, s, pa);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            const bool r0 = dx_fast && pdx.n_split > 1, r1 = dw_fast && pdw.n_split > 1;
            if (r0 || r1) {
                const int tiles0 = r0 ? (int)pdx.tiles : 0, tiles1 = r1 ? (int)pdw.tiles : 0;
                hipLaunchKernelGGL(fc2_i8_reduce_kernel, dim3(32 * (tiles0 + tiles1)), dim3(256), 0, s, pa, tiles0);
                e = hipGetLastError();
                if (e != hipSuccess) return e;
            }
        }
        if (pending.n || pending.bias_len) { e = launch_stats_job(pending, s); if (e != hipSuccess) return e; }
        if (a.dX && !dx_fast) {
            MatrixLoader<MODE_I8, true, true>   al{a.codes, a.out, B, out};
            MatrixLoader<MODE_I8, false, false> bl{a.W8, a.in, in, out};
            e = run_gemm<MODE_I8>(al, bl, om, B, in, out, k_step<MODE_I8>(), Scale{1.0f, nullptr}, (int32_t *)a.dX, a.scratch, a.scratch_bytes, s);
            if (e != hipSuccess) return e;
        }
        if (a.dW && !dw_fast) {
            MatrixLoader<MODE_I8, true, false>  al{a.codes, a.out, out, B};
            MatrixLoader<MODE_I8, false, false> bl{(const int8_t *)a.X, a.in, in, B};
            e = run_gemm<MODE_I8>(al, bl, om, out, in, B, k_step<MODE_I8>(), Scale{1.0f, nullptr}, (int32_t *)a.dW, a.scratch, a.scratch_bytes, s);
        }
        return e;
    }
    if (a.codes) {
        // fast path: one launch for every product whose layout allows it
        const bool dx_fast = a.dX && fc_fast_ok(true, a.codes, a.out, a.W, a.in, B, in, a.dX);
        const bool dw_fast = a.dW && a.x_dtype == DBP_F32 &&
                             fc_fast_ok(false, a.codes, a.out, (const float *)a.X, a.in, out, in, (const float *)a.dW);
        // Large products: the kernel with separate staging and multiplying wavefronts (256x128 tiles, one
        // workgroup per CU); small ones (less than half such a tile of rows): the 128x128 kernel.
        const bool big = (!dx_fast || B > FC2_TM / 2) && (!dw_fast || out > FC2_TM / 2) &&
                         (!dx_fast || out >= 32) && (!dw_fast || (B >= 32 && out >= 16)) &&         // a full window of 32 reduction indices; 16-row runs
                         (int64_t)B * in < (1ll << 30) && (int64_t)out * in < (1ll << 30) && (int64_t)B * out < (1ll << 30);                // 32-bit lane offsets
        FcPlan pdx, pdw;
        bool use_fc2 = (dx_fast || dw_fast) && big;
        if (use_fc2) {
            fc2_plans(B, in, out, dx_fast, dw_fast, pdx, pdw);
            const int64_t items = (dx_fast ? pdx.tiles * pdx.n_split : 0) + (dw_fast ? pdw.tiles * pdw.n_split : 0);
            if (items > (int64_t)FC2_MAX_ITEMS * 256) use_fc2 = false;     // the per-workgroup item table is fixed
        }
        int gx = 0;
        if (use_fc2 && dx_fast && dw_fast) gx = fc2_group_plan(B, in, out, pdx, pdw);
        if (a.plan_only) {
            // gated: both requested products on one of the pair kernels (the generic kernel takes no gate)
            const bool int8_dw = a.dW && a.x_dtype != DBP_F32;
            if ((a.dX && !dx_fast) || (a.dW && !dw_fast) || int8_dw) *a.plan_only = 1;
            return hipSuccess;
        }
        if (use_fc2) {
            static bool raised = false;
            if (!raised) {
                e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fc2_pair_kernel<false, 3>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, FC2_LDS_BYTES);
                if (e != hipSuccess) return e;
                e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fc2_pair_kernel<false, 2>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, FC2_LDS_BYTES);
                if (e != hipSuccess) return e;
                raised = true;
            }
            char *scratch = (char *)a.scratch;
            FcPairArgs pa;
            if (!dx_fast) { pdx.n_split = 1; pdx.partial_bytes = 0; }
            if (!dw_fast) { pdw.n_split = 1; pdw.partial_bytes = 0; }
            pa.prob[0] = fc_problem(true, a.codes, a.out, a.W, a.in, B, in, out, Scale{a.step, a.step_dev}, a.dX, pdx, scratch);
            pa.prob[1] = fc_problem(false, a.codes, a.out, (const float *)a.X, a.in, out, in, B, Scale{a.step, a.step_dev}, (float *)a.dW, pdw, scratch);
            if (!dx_fast) pa.prob[0].n_items = 0;
            if (!dw_fast) pa.prob[1].n_items = 0;
            if ((size_t)(scratch - (char *)a.scratch) > a.scratch_bytes) return hipErrorInvalidValue;
            pa.stats = pending;                            // finished by a stager wavefront of the last workgroup
            pending.n = 0; pending.bias_len = 0;
            pa.gx = gx; pa.gate = a.gate;
            const int total = pa.prob[0].n_items + pa.prob[1].n_items;
            const int grid = total < 256 ? total : 256;    // persistent: one workgroup per CU (256 whenever gx > 0)
            if (a.two_planes) hipLaunchKernelGGL((fc2_pair_kernel<false, 2>), dim3(grid), dim3(512), FC2_LDS_BYTES, s, pa);
            else              hipLaunchKernelGGL((fc2_pair_kernel<false, 3>), dim3(grid), dim3(512), FC2_LDS_BYTES, s, pa);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            const bool r0 = dx_fast && pdx.n_split > 1, r1 = dw_fast && pdw.n_split > 1;
            if (r0 || r1) {
                const int tiles0 = r0 ? (int)pdx.tiles : 0, tiles1 = r1 ? (int)pdw.tiles : 0;
                hipLaunchKernelGGL(fc2_reduce_kernel, dim3(32 * (tiles0 + tiles1)), dim3(256), 0, s, pa, tiles0);
                e = hipGetLastError();
                if (e != hipSuccess) return e;
            }
        } else if (dx_fast || dw_fast) {
            char *scratch = (char *)a.scratch;
            FcPairArgs pa;
            const FcPlan none = {0, 0, 1, FC_KT, 0, 0};
            const FcPlan pdx = dx_fast ? fc_plan(B, in, out) : none, pdw = dw_fast ? fc_plan(out, in, B) : none;
            pa.prob[0] = fc_problem(true, a.codes, a.out, a.W, a.in, B, in, out, Scale{a.step, a.step_dev}, a.dX, pdx, scratch);
            pa.prob[1] = fc_problem(false, a.codes, a.out, (const float *)a.X, a.in, out, in, B, Scale{a.step, a.step_dev}, (float *)a.dW, pdw, scratch);
            if (!dx_fast) pa.prob[0].n_items = 0;
            if (!dw_fast) pa.prob[1].n_items = 0;
            if (pending.bias_len) {                        // this kernel folds the statistics only
                StatsJob bias = pending;
                bias.n = 0;
                e = launch_stats_job(bias, s);
                if (e != hipSuccess) return e;
                pending.bias_len = 0;
            }
            pa.stats = pending;                            // summed by the last workgroup of the launch
            pending.n = 0;
            pa.gate = a.gate;
            if ((size_t)(scratch - (char *)a.scratch) > a.scratch_bytes) return hipErrorInvalidValue;
            const int total = pa.prob[0].n_items + pa.prob[1].n_items;
            // odd grid: a persistent workgroup then alternates between the two products
            int grid = total < 767 ? total : 767;          // 3 resident workgroups on each of 256 CUs
            hipLaunchKernelGGL(fc_pair_kernel, dim3(grid), dim3(256), 0, s, pa);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            // split-K: one reduction launch for both products (a problem without splits gets no workgroups)
            const bool r0 = dx_fast && pdx.n_split > 1, r1 = dw_fast && pdw.n_split > 1;
            if (r0 || r1) {
                FcPairArgs ra = pa;
                int tiles0 = r0 ? (int)pdx.tiles : 0, tiles1 = r1 ? (int)pdw.tiles : 0;
                hipLaunchKernelGGL(fc_reduce_kernel, dim3(32 * (tiles0 + tiles1)), dim3(256), 0, s, ra, tiles0);
                e = hipGetLastError();
                if (e != hipSuccess) return e;
            }
        }
        if (pending.n || pending.bias_len) { e = launch_stats_job(pending, s); if (e != hipSuccess) return e; }
        if (a.dX && !dx_fast) {
            MatrixLoader<MODE_BF16, true, true>   al{a.codes, a.out, B, out};
            MatrixLoader<MODE_BF16, false, false> bl{a.W, a.in, in, out};
            e = run_gemm<MODE_BF16>(al, bl, om, B, in, out, k_step<MODE_BF16>(), Scale{a.step, a.step_dev}, a.dX, a.scratch, a.scratch_bytes, s);
            if (e != hipSuccess) return e;
        }
        if (a.dW && a.x_dtype == DBP_F32 && !dw_fast) {
            MatrixLoader<MODE_BF16, true, false>  al{a.codes, a.out, out, B};
            MatrixLoader<MODE_BF16, false, false> bl{(const float *)a.X, a.in, in, B};
            e = run_gemm<MODE_BF16>(al, bl, om, out, in, B, k_step<MODE_BF16>(), Scale{a.step, a.step_dev}, (float *)a.dW, a.scratch, a.scratch_bytes, s);
        } else if (a.dW && a.x_dtype != DBP_F32) {
            MatrixLoader<MODE_I8, true, false>  al{a.codes, a.out, out, B};
            MatrixLoader<MODE_I8, false, false> bl{(const int8_t *)a.X, a.in, in, B};
            e = run_gemm<MODE_I8>(al, bl, om, out, in, B, k_step<MODE_I8>(), Scale{1.0f, nullptr}, (int32_t *)a.dW, a.scratch, a.scratch_bytes, s);
        }
        return e;
    }
    // dense baseline
    if (pending.n || pending.bias_len) { e = launch_stats_job(pending, s); if (e != hipSuccess) return e; }
    if (a.dX) {
        MatrixLoader<MODE_F32, false, true>  al{(const float *)a.dense, a.out, B, out};
        MatrixLoader<MODE_F32, false, false> bl{a.W, a.in, in, out};
        e = run_gemm<MODE_F32>(al, bl, om, B, in, out, k_step<MODE_F32>(), Scale{1.0f, nullptr}, a.dX, a.scratch, a.scratch_bytes, s);
        if (e != hipSuccess) return e;
    }
    if (a.dW && a.x_dtype == DBP_F32) {
        MatrixLoader<MODE_F32, false, false> al{(const float *)a.dense, a.out, out, B};
        MatrixLoader<MODE_F32, false, false> bl{(const float *)a.X, a.in, in, B};
        e = run_gemm<MODE_F32>(al, bl, om, out, in, B, k_step<MODE_F32>(), Scale{1.0f, nullptr}, (float *)a.dW, a.scratch, a.scratch_bytes, s);
    } else if (a.dW) {
        MatrixLoader<MODE_I8, false, false> al{(const int8_t *)a.dense, a.out, out, B};
        MatrixLoader<MODE_I8, false, false> bl{(const int8_t *)a.X, a.in, in, B};
        e = run_gemm<MODE_I8>(al, bl, om, out, in, B, k_step<MODE_I8>(), Scale{1.0f, nullptr}, (int32_t *)a.dW, a.scratch, a.scratch_bytes, s);
    }
    return e;
}

// Clears n 4-byte words (the output pixels of a strided layer that no tap reaches).
__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0u;
}

// Grouped convolution with few channels per group, run as ONE ungrouped layer: the weights [K][Cg][RS] are expanded into
// the block-diagonal [K][C][RS] (zero outside a channel's own group: those products add exact zeros), and the diagonal
// blocks of the ungrouped dW are copied back.  4-byte elements either way (fp32 weights; fp32 or int32 dW).
__global__ __launch_bounds__(256) void group_weights_expand_kernel(const uint32_t *W, uint32_t *full, int K, int C, int Cg, int Kg, int RS)
{
    const int64_t total = (int64_t)K * C * RS;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int rs = (int)(i % RS);
        const int64_t kc = i / RS;
        const int c = (int)(kc % C), k = (int)(kc / C);
        const bool own = c / Cg == k / Kg;
        full[i] = own ? W[((int64_t)k * Cg + c % Cg) * RS + rs] : 0u;
    }
}

__global__ __launch_bounds__(256) void group_dw_extract_kernel(const uint32_t *full, uint32_t *dW, int K, int C, int Cg, int Kg, int RS)
{
    const int64_t total = (int64_t)K * Cg * RS;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int rs = (int)(i % RS);
        const int64_t kc = i / RS;
        const int cl = (int)(kc % Cg), k = (int)(kc / Cg);
        dW[i] = full[((int64_t)k * C + (k / Kg) * Cg + cl) * RS + rs];
    }
}

hipError_t launch_group_weights_expand(const float *W, float *full, int64_t K, int64_t C, int64_t groups, int64_t RS, hipStream_t s)
{
    const int64_t total = K * C * RS;
    const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(group_weights_expand_kernel, dim3(blocks), dim3(256), 0, s, (const uint32_t *)W, (uint32_t *)full, (int)K, (int)C,
                       (int)(C / groups), (int)(K / groups), (int)RS);
    return hipGetLastError();
}

hipError_t launch_group_dw_extract(const void *full, void *dW, int64_t K, int64_t C, int64_t groups, int64_t RS, hipStream_t s)
{
    const int64_t total = K * (C / groups) * RS;
    const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(group_dw_extract_kernel, dim3(blocks), dim3(256), 0, s, (const uint32_t *)full, (uint32_t *)dW, (int)K, (int)C,
                       (int)(C / groups), (int)(K / groups), (int)RS);
    return hipGetLastError();
}

hipError_t launch_zero_words(void *p, int64_t n_words, hipStream_t s)
{
    const int fb = (int)((n_words + 255) / 256 < 8192 ? (n_words + 255) / 256 : 8192);
    hipLaunchKernelGGL(zero_words_kernel, dim3(fb < 1 ? 1 : fb), dim3(256), 0, s, (uint32_t *)p, n_words);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Convolution (fast dX kernel: any stride; fast dW kernels: stride 1; the generic kernel serves the rest).
// ------------------------------------------------------------------------------------------------
template <int MODE_G, int MODE_K>
static hipError_t conv_dx_run(const ConvArgs &a, const void *grad, Scale scale, hipStream_t s)
{
    // MODE_G: MODE_BF16 (codes, fp32 weights), MODE_I8 (codes, int8 weights) or MODE_F32 (dense).  MODE_K: the fast kernels'
    // mode, MODE_G itself or MODE_BF16X2 (fp32 weights in two planes).
    if constexpr (MODE_G != MODE_F32) {
        constexpr bool I8 = MODE_G == MODE_I8;
        constexpr int PL = CdxTraits<MODE_K>::PL;
        auto prepare = [&](int taps, int KG, int Cp, const CdxTapMap *map) {
            const int64_t cells = (int64_t)taps * KG * Cp;
            int pb = (int)((cells + 255) / 256 < 4096 ? (cells + 255) / 256 : 4096);
            const int rs = (int)(a.R * a.S);
            // the quantiser's pending statistics sum / bias gradient ride along in one more workgroup
            StatsJob job{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr};
            if (a.pending && (a.pending->n > 0 || a.pending->bias_len > 0)) { job = *a.pending; a.pending->n = 0; a.pending->bias_len = 0; ++pb; }
            if constexpr (I8) {
                if (map) hipLaunchKernelGGL(conv_dx_weight_prep_i8_kernel<true>, dim3(pb), dim3(256), 0, s, a.W8, (uint4 *)a.scratch, (int)a.K, (int)a.C, taps, KG, Cp, rs, *map, job);
                else     hipLaunchKernelGGL(conv_dx_weight_prep_i8_kernel<false>, dim3(pb), dim3(256), 0, s, a.W8, (uint4 *)a.scratch, (int)a.K, (int)a.C, taps, KG, Cp, rs, CdxTapMap{}, job);
            } else {
                if (map) hipLaunchKernelGGL((conv_dx_weight_prep_kernel<true, PL>), dim3(pb), dim3(256), 0, s, a.W, (uint4 *)a.scratch, (int)a.K, (int)a.C, taps, KG, Cp, rs, *map, job);
                else     hipLaunchKernelGGL((conv_dx_weight_prep_kernel<false, PL>), dim3(pb), dim3(256), 0, s, a.W, (uint4 *)a.scratch, (int)a.K, (int)a.C, taps, KG, Cp, rs, CdxTapMap{}, job);
            }
        };
        // The codes as the kernel wants them: planes that start on 4-byte boundaries.  Planes of a size that is not a
        // multiple of 4 (7x7 outputs ...) or a misaligned tensor are copied into padded planes behind the prepared weights.
        const size_t rbw = relayout_bytes(a.K, a.C, a.R, a.S);
        const int64_t PQ = ((a.H + 2 * a.pad - a.R) / a.stride + 1) * ((a.Wd + 2 * a.pad - a.S) / a.stride + 1);
        const int64_t plane = (PQ + 3) / 4 * 4;
        const bool pad_codes = PQ % 4 != 0 || (uintptr_t)grad % 4 != 0;
        const bool codes_ok = !pad_codes || (rbw + (size_t)(a.N * a.K * plane) <= a.scratch_bytes && plane < (1 << 24));
        auto kernel_codes = [&]() -> const int8_t * {
            if (!pad_codes) return (const int8_t *)grad;
            uint32_t *dst = (uint32_t *)((char *)a.scratch + rbw);
            const int64_t dwords = a.N * a.K * (plane / 4);
            const int pbk = (int)((dwords + 255) / 256 < 4096 ? (dwords + 255) / 256 : 4096);
            hipLaunchKernelGGL(conv_dx_pad_codes_kernel, dim3(pbk), dim3(256), 0, s, (const int8_t *)grad, dst, a.N * a.K, (int)PQ, (int)plane,
                               (int)a.K, (int)a.kt());
            return (const int8_t *)dst;
        };
        if (a.stride != 1 && codes_ok) {
            ConvDxStridedPlan sp = conv_dx_strided_plan(a, I8);
            if (sp.ok && a.plan_only) return hipSuccess;
            if (sp.ok) {
                if (sp.zero_fill && !a.dx_zeroed) {
                    // (one group of a grouped layer never comes here: its dX is not contiguous and the caller has cleared it)
                    const int64_t n = a.N * a.C * a.H * a.Wd;                 // fp32 and int32 zeros are the same bytes
                    const int fb = (int)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
                    hipLaunchKernelGGL(zero_words_kernel, dim3(fb), dim3(256), 0, s, (uint32_t *)a.dX, n);
                }
                if (sp.multi.n > 0) {
                    const int KG = sp.multi.cls[0].KG, Cp = sp.multi.cls[0].Cp;
                    prepare(sp.taps, KG, Cp, &sp.map);
                    const int8_t *kc = kernel_codes();
                    for (int i = 0; i < sp.multi.n; ++i) {
                        ConvDxArgs &k = sp.multi.cls[i];
                        k.codes = kc; k.dX = a.dX; k.scale = scale; k.gate = a.gate;
                        k.code_img = (pad_codes ? a.K : a.kt()) * k.PQ; k.dx_img = a.ct() * k.oPI;
                        k.wp = (const uint4 *)a.scratch + (int64_t)sp.tap_base[i] * KG * PL * Cp;
                    }
                    if (sp.nb == 7)      hipLaunchKernelGGL((conv_dx_multi_kernel<7, MODE_K>), dim3(sp.grid), dim3(256), sp.lds_bytes, s, sp.multi);
                    else if (sp.nb == 4) hipLaunchKernelGGL((conv_dx_multi_kernel<4, MODE_K>), dim3(sp.grid), dim3(256), sp.lds_bytes, s, sp.multi);
                    else                 hipLaunchKernelGGL((conv_dx_multi_kernel<2, MODE_K>), dim3(sp.grid), dim3(256), sp.lds_bytes, s, sp.multi);
                }
                return hipGetLastError();
            }
        }
        ConvDxPlan pl = conv_dx_plan(a, I8);
        if (pl.ok && codes_ok && a.plan_only) return hipSuccess;
        if (pl.ok && codes_ok) {
            ConvDxArgs &k = pl.args;
            k.codes = kernel_codes(); k.wp = (const uint4 *)a.scratch; k.dX = a.dX; k.scale = scale; k.gate = a.gate;
            k.code_img = (pad_codes ? a.K : a.kt()) * k.PQ; k.dx_img = a.ct() * k.PI;
            prepare(k.R * k.S, k.KG, k.Cp, nullptr);
            // tap counts that are a multiple of 3 (3x3 above all) take the form with three weight fragment sets in flight
            const bool ring3 = (k.R * k.S) % 3 == 0;
            const dim3 grid(pl.grid), block(256);
            if (ring3) {
                if (pl.nb == 7)      hipLaunchKernelGGL((conv_dx_kernel<7, MODE_K, true>), grid, block, pl.lds_bytes, s, k);
                else if (pl.nb == 4) hipLaunchKernelGGL((conv_dx_kernel<4, MODE_K, true>), grid, block, pl.lds_bytes, s, k);
                else                 hipLaunchKernelGGL((conv_dx_kernel<2, MODE_K, true>), grid, block, pl.lds_bytes, s, k);
            } else {
                if (pl.nb == 7)      hipLaunchKernelGGL((conv_dx_kernel<7, MODE_K, false>), grid, block, pl.lds_bytes, s, k);
                else if (pl.nb == 4) hipLaunchKernelGGL((conv_dx_kernel<4, MODE_K, false>), grid, block, pl.lds_bytes, s, k);
                else                 hipLaunchKernelGGL((conv_dx_kernel<2, MODE_K, false>), grid, block, pl.lds_bytes, s, k);
            }
            return hipGetLastError();
        }
    }
    if (a.plan_only) { *a.plan_only = 1; return hipSuccess; }         // the generic kernel takes no gate
    ConvGeom g = make_geom(a, ModeTraits<MODE_G>::KCH, k_step<MODE_G>());
    using WT = typename std::conditional<MODE_G == MODE_I8, int8_t, float>::type;      // int8 weights in the full 8-bit mode
    using Acc = typename ModeTraits<MODE_G>::Acc;
    WT *Wt = (WT *)a.scratch;
    const WT *Wsrc = MODE_G == MODE_I8 ? (const WT *)a.W8 : (const WT *)a.W;
    const size_t rb = relayout_bytes(a.K, a.C, a.R, a.S);
    const int64_t total = (int64_t)g.R * g.S * g.Kp * g.C;
    int blocks = (int)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(conv_weight_relayout_kernel<WT>, dim3(blocks), dim3(256), 0, s, Wsrc, Wt, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int M = g.N * g.H * g.Wd, Kred = g.R * g.S * g.Kp;
    ConvDxGradLoader<MODE_G> al{(const typename GradElem<MODE_G>::T *)grad, g};
    MatrixLoader<MODE_G, false, false> bl{Wt, g.C, g.C, Kred};
    ConvDxOut om{g.Ct, g.H * g.Wd};
    return run_gemm<MODE_G>(al, bl, om, M, g.C, Kred, k_step<MODE_G>(), scale, (Acc *)a.dX,
                            (char *)a.scratch + rb, a.scratch_bytes - rb, s);
}

template <int MODE_G>
static hipError_t conv_dx(const ConvArgs &a, const void *grad, Scale scale, hipStream_t s)
{
    if constexpr (MODE_G == MODE_BF16) {
        if (a.two_planes) return conv_dx_run<MODE_G, MODE_BF16X2>(a, grad, scale, s);
    }
    return conv_dx_run<MODE_G, MODE_G>(a, grad, scale, s);
}

template <int MODE>
static hipError_t conv_dw(const ConvArgs &a, const void *grad, Scale scale, hipStream_t s)
{
    using Acc = typename ModeTraits<MODE>::Acc;
    const size_t rb = relayout_bytes(a.K, a.C, a.R, a.S);
    if constexpr (MODE == MODE_I8) {
        ConvDwI8Plan p8 = conv_dw_i8_plan(a.N, a.C, a.H, a.Wd, a.K, a.R, a.S, a.pad);
        if (p8.ok && a.stride == 1 && rb + p8.partial_bytes <= a.scratch_bytes && (uintptr_t)a.X % 4 == 0 && (uintptr_t)grad % 4 == 0) {
            if (a.plan_only) return hipSuccess;
            ConvDwI8Args &k = p8.args;
            k.codes = (const int8_t *)grad; k.X = (const int8_t *)a.X; k.dW = (int32_t *)a.dW; k.partial = (int32_t *)((char *)a.scratch + rb);
            k.gate = a.gate; k.Ct = (int)a.ct(); k.Kt = (int)a.kt();
            return launch_conv_dw_i8(p8, s);
        }
    }
    if constexpr (MODE != MODE_F32) {
        ConvDwPlan pl = conv_dw_plan(a.N, a.C, a.H, a.Wd, a.K, a.R, a.S, a.pad, MODE == MODE_I8);
        if (a.stride != 1) pl.ok = false;                            // the fast kernel is a stride-1 kernel
        const size_t xal = MODE == MODE_I8 ? 4 : 16;                 // aligned 4-element loads of both operands
        if (pl.ok && rb + pl.partial_bytes <= a.scratch_bytes && (uintptr_t)a.X % xal == 0 && (uintptr_t)grad % 4 == 0) {
            if (a.plan_only) return hipSuccess;
            ConvDwArgs &k = pl.args;
            k.codes = (const int8_t *)grad; k.X = a.X; k.dW = a.dW; k.partial = (char *)a.scratch + rb; k.scale = scale; k.gate = a.gate;
            k.Ct = (int)a.ct(); k.Kt = (int)a.kt();
            if constexpr (MODE == MODE_BF16) {
                if (a.two_planes)
                    return a.pad == 1 ? launch_conv_dw_fast<MODE_BF16X2, 3, 3, 1, 1>(pl, s) : launch_conv_dw_fast<MODE_BF16X2, 3, 3, 0, 1>(pl, s);
            }
            return a.pad == 1 ? launch_conv_dw_fast<MODE, 3, 3, 1, 1>(pl, s) : launch_conv_dw_fast<MODE, 3, 3, 0, 1>(pl, s);
        }
    }
    if constexpr (MODE != MODE_F32) {
        constexpr bool I8 = MODE == MODE_I8;
        const Conv1x1Plan p1 = conv1x1_dw_plan(a.N, a.C, a.H, a.Wd, a.K, a.R, a.S, a.pad, a.stride, I8 ? FC2I_KT : FC2_KT);
        if (p1.ok && rb + p1.partial_bytes <= a.scratch_bytes && (uintptr_t)grad % 4 == 0 && (uintptr_t)a.X % (I8 ? 4 : 16) == 0 &&
            (uintptr_t)a.dW % 16 == 0)
            return a.plan_only ? hipSuccess : launch_conv1x1_dw<I8>(a, p1, (const int8_t *)grad, scale, (char *)a.scratch + rb, s);
    }
    if (a.plan_only) { *a.plan_only = 1; return hipSuccess; }         // the lowered and the generic forms are not gated
    if constexpr (MODE != MODE_F32) {
        // neither convolution kernel took it: expand the activations into the column matrix, re-lay the codes, and let the
        // fully connected kernels do dW[k][(c,r,s)] = sum_(n,p,q) code[k][(n,p,q)] col[(n,p,q)][(c,r,s)]
        constexpr int ESZ = MODE == MODE_I8 ? 1 : 4;
        const ConvLowerPlan lp = conv_dw_lower_plan(a.N, a.C, a.H, a.Wd, a.K, a.R, a.S, a.pad, a.stride, ESZ);
        if (lp.ok && (MODE == MODE_BF16 || lp.vec4) &&      // int8 entries written one byte at a time: measured slower than generic
            rb + lp.bytes <= a.scratch_bytes && (uintptr_t)grad % 4 == 0 && (uintptr_t)a.X % 4 == 0 && (uintptr_t)a.dW % 16 == 0) {
            int8_t *ck = (int8_t *)a.scratch + rb;
            char *col = (char *)ck + lp.codes_bytes;
            const int PQ = lp.im.P * lp.im.Q;
            const int64_t groups = (int64_t)a.K * lp.NPQ / (PQ % 4 == 0 ? 4 : 1);
            const int cb = (int)((groups + 255) / 256 < 8192 ? (groups + 255) / 256 : 8192);
            if (PQ % 4 == 0) hipLaunchKernelGGL(conv_codes_kmajor_kernel<4>, dim3(cb), dim3(256), 0, s, (const int8_t *)grad, ck, (int)a.N, (int)a.K, PQ, (int)a.kt());
            else             hipLaunchKernelGGL(conv_codes_kmajor_kernel<1>, dim3(cb), dim3(256), 0, s, (const int8_t *)grad, ck, (int)a.N, (int)a.K, PQ, (int)a.kt());
            Im2colArgs im = lp.im;
            im.X = a.X; im.col = col; im.Ct = (int)a.ct();
            const int grid = (int)(a.N * im.bands * im.ctiles);
            using XT = typename std::conditional<MODE == MODE_I8, int8_t, float>::type;
            if (lp.vec4) hipLaunchKernelGGL((conv_im2col_kernel<XT, 4>), dim3(grid), dim3(256), lp.lds_bytes, s, im);
            else         hipLaunchKernelGGL((conv_im2col_kernel<XT, 1>), dim3(grid), dim3(256), lp.lds_bytes, s, im);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            LinearArgs la{};
            la.codes = ck; la.dense = nullptr; la.step = scale.host; la.step_dev = scale.dev;
            la.W = MODE == MODE_I8 ? nullptr : (const float *)col;
            la.W8 = MODE == MODE_I8 ? (const int8_t *)col : nullptr;
            la.X = nullptr; la.x_dtype = MODE == MODE_I8 ? DBP_I8 : DBP_F32;
            la.B = a.K; la.in = lp.CRS; la.out = lp.NPQ;
            la.dX = (float *)a.dW; la.dW = nullptr;
            la.scratch = col + lp.col_bytes; la.scratch_bytes = lp.fc_bytes;
            la.stats_job = StatsJob{}; la.two_planes = a.two_planes;
            return launch_linear_mfma(la, s);
        }
    }
    ConvGeom g = make_geom(a, ModeTraits<MODE>::KCH, k_step<MODE>());
    const int CRS = g.C * g.R * g.S, Kred = g.N * g.PQp;
    ConvDwGradLoader<MODE> al{(const typename GradElem<MODE>::T *)grad, g};
    ConvDwActLoader<MODE>  bl{(const decltype(ConvDwActLoader<MODE>::base))a.X, g};
    RowMajorOut om{CRS};
    return run_gemm<MODE>(al, bl, om, g.K, CRS, Kred, k_step<MODE>(), scale, (Acc *)a.dW,
                          (char *)a.scratch + rb, a.scratch_bytes - rb, s);
}

static hipError_t conv_products(const ConvArgs &a_in, hipStream_t s)
{
    hipError_t e = hipSuccess;
    const ConvArgs &a = a_in;
    ConvArgs aw = a_in;                                                // what the dW kernels see: their own gate where one is given
    if (a_in.gate_dw.flag) aw.gate = a_in.gate_dw;
    if (a.codes && a.W8) {
        // full 8-bit mode: int8 weights and activations, exact int32 results
        if (a.dX) { e = conv_dx<MODE_I8>(a, a.codes, Scale{1.0f, nullptr}, s); if (e != hipSuccess) return e; }
        if (a.dW) e = conv_dw<MODE_I8>(aw, a.codes, Scale{1.0f, nullptr}, s);
        return e;
    }
    if (a.codes) {
        if (a.dX) { e = conv_dx<MODE_BF16>(a, a.codes, Scale{a.step, a.step_dev}, s); if (e != hipSuccess) return e; }
        if (a.dW) e = a.x_dtype == DBP_F32 ? conv_dw<MODE_BF16>(aw, a.codes, Scale{a.step, a.step_dev}, s) : conv_dw<MODE_I8>(aw, a.codes, Scale{1.0f, nullptr}, s);
        return e;
    }
    if (a.dX) { e = conv_dx<MODE_F32>(a, a.dense, Scale{1.0f, nullptr}, s); if (e != hipSuccess) return e; }
    if (a.dW) e = a.x_dtype == DBP_F32 ? conv_dw<MODE_F32>(aw, a.dense, Scale{1.0f, nullptr}, s) : conv_dw<MODE_I8>(aw, a.dense, Scale{1.0f, nullptr}, s);
    return e;
}

// The quantiser's pending statistics sum and bias gradient go with the first kernel that can take them along (the weight
// preparation of the dX kernels); what nobody took is launched on its own afterwards.
hipError_t launch_conv_mfma(const ConvArgs &a_in, hipStream_t s)
{
    ConvArgs a = a_in;
    StatsJob pending = a_in.stats_job;
    a.pending = &pending;
    hipError_t e = conv_products(a, s);
    if (e == hipSuccess && (pending.n > 0 || pending.bias_len > 0)) e = launch_stats_job(pending, s);
    return e;
}

// ------------------------------------------------------------------------------------------------
// Host-side self-check of the launch plans (no GPU): the planning arithmetic above decides every kernel's indexing, so
// a mistake in it is where an out-of-bounds access would come from.  The checks walk the same functions the launchers
// and the kernels use.  0 = consistent (or the shape takes no planned kernel), otherwise the number of the first
// violated invariant.
// ------------------------------------------------------------------------------------------------
static int check_fc2_pair(int64_t B, int64_t in, int64_t out, bool want_dx, bool want_dw, int kt)
{
    FcPlan pdx, pdw;
    fc2_plans(B, in, out, want_dx, want_dw, pdx, pdw, kt);
    const int64_t items = (want_dx ? pdx.tiles * pdx.n_split : 0) + (want_dw ? pdw.tiles * pdw.n_split : 0);
    if (items > (int64_t)FC2_MAX_ITEMS * 256 || items <= 0) return 0;         // the launcher takes another kernel
    int gx = 0;
    if (want_dx && want_dw) gx = fc2_group_plan(B, in, out, pdx, pdw, kt);
    if (!want_dx) { pdx.n_split = 1; pdx.partial_bytes = 0; }
    if (!want_dw) { pdw.n_split = 1; pdw.partial_bytes = 0; }
    char *scratch = nullptr;
    FcPairArgs pa;
    pa.prob[0] = fc_problem(true, nullptr, out, nullptr, in, (int)B, (int)in, (int)out, Scale{1.0f, nullptr}, nullptr, pdx, scratch);
    pa.prob[1] = fc_problem(false, nullptr, out, nullptr, in, (int)out, (int)in, (int)B, Scale{1.0f, nullptr}, nullptr, pdw, scratch);
    if (!want_dx) pa.prob[0].n_items = 0;
    if (!want_dw) pa.prob[1].n_items = 0;
    pa.gx = gx;
    if ((size_t)(scratch - (char *)nullptr) > linear_scratch_bytes(B, in, out)) return 1;      // partial sums beyond the workspace
    const int total = pa.prob[0].n_items + pa.prob[1].n_items;
    const int G = total < 256 ? total : 256;
    if (gx > 0 && gx >= G) return 2;                                            // the second group would have no workgroup
    std::vector<unsigned char> seen[2];
    seen[0].assign((size_t)pa.prob[0].n_items, 0); seen[1].assign((size_t)pa.prob[1].n_items, 0);
    for (int w = 0; w < G; ++w) {
        const int mine = fc2_items_of_workgroup(pa, G, w);
        if (mine < 0 || mine > FC2_MAX_ITEMS) return 3;
        for (int i = 0; i < mine; ++i) {
            const Fc2Item it = fc2_decode(pa, i, mine, G, w);
            if (it.which < 0 || it.which > 1) return 4;
            const FcProblem &p = pa.prob[it.which];
            if (p.n_items <= 0) return 5;
            const int tiles = p.n_items / p.n_split;
            if (it.tile < 0 || it.tile >= tiles || it.z < 0 || it.z >= p.n_split) return 6;
            if (it.tile_m < 0 || it.tile_m >= p.M || it.tile_n < 0 || it.tile_n >= p.N) return 7;
            if (it.k0 < 0 || it.k0 >= it.k_end || it.k_end > p.K) return 8;
            unsigned char &flag = seen[it.which][(size_t)it.tile * p.n_split + it.z];
            if (flag) return 9;                                                     // an item handed out twice
            flag = 1;
        }
    }
    for (int q = 0; q < 2; ++q)
        for (unsigned char f : seen[q]) if (!f) return 10;                          // an item nobody takes
    return 0;
}

static int check_conv_plans(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad)
{
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    const size_t total = conv_scratch_bytes(N, C, H, Wd, K, R, S, pad, stride), rb = relayout_bytes(K, C, R, S);
    if (rb > total) return 20;
    ConvArgs a{};
    a.N = N; a.C = C; a.H = H; a.Wd = Wd; a.K = K; a.R = R; a.S = S; a.pad = pad; a.stride = stride;
    for (int i8 = 0; i8 < 2; ++i8) {
        // dX: the stride-1 kernel or the classes of a strided layer
        auto check_dx = [&](const ConvDxArgs &k, int nb, size_t lds, int64_t grid) {
            const int tile_px = k.wpx * 32 * nb;
            if (lds > (size_t)CDX_MAX_LDS || lds < (size_t)2 * CDX_KGC * k.patch_cells * 16) return 21;
            if ((int64_t)k.tiles * tile_px < k.PI || (int64_t)(k.tiles - 1) * tile_px >= k.PI) return 22;      // tiles cover the pixels, none is empty
            if (grid != (int64_t)k.N * k.tiles * k.cgroups || grid <= 0) return 23;
            if (k.wc * k.wpx != 4 || (int64_t)k.cgroups * k.wc * 32 < k.Cp || k.Cp < k.C) return 24;
            if (k.KG % CDX_KGC || (int64_t)k.KG * (i8 ? 16 : 8) < k.K || k.n_chunks * CDX_KGC != k.KG) return 25;
            if ((int64_t)k.prow * k.pw != k.patch_cells || CDX_KGC * (int64_t)k.patch_cells >= 0xFFFF) return 26;
            return 0;
        };
        if (stride == 1) {
            const ConvDxPlan pl = conv_dx_plan(a, i8 != 0);
            if (pl.ok) { const int e = check_dx(pl.args, pl.nb, pl.lds_bytes, pl.grid); if (e) return e; }
        } else {
            const ConvDxStridedPlan sp = conv_dx_strided_plan(a, i8 != 0);
            if (sp.ok) {
                if (sp.multi.n < 0 || sp.multi.n > CDX_MAX_CLASSES || sp.taps > 64) return 27;
                for (int i = 0; i < sp.multi.n; ++i) {
                    const int e = check_dx(sp.multi.cls[i], sp.nb, sp.lds_bytes, (int64_t)sp.multi.first[i + 1] - sp.multi.first[i]);
                    if (e) return e;
                    if (sp.tap_base[i] + sp.multi.cls[i].R * sp.multi.cls[i].S > sp.taps) return 28;
                }
                if (sp.multi.first[sp.multi.n] != sp.grid) return 29;
                for (int t = 0; t < sp.taps; ++t) if (sp.map.real[t] >= R * S) return 30;
            }
        }
        const size_t padded = (size_t)(N * K * ((P * Q + 3) / 4 * 4));
        if (rb + padded > total) return 31;                                       // the padded copy of the codes
        // dW
        const ConvDwPlan pw = conv_dw_plan(N, C, H, Wd, K, R, S, pad, i8 != 0);
        if (pw.ok && stride == 1) {
            const ConvDwArgs &k = pw.args;
            if (pw.lds_bytes > (size_t)CDW_MAX_LDS || rb + pw.partial_bytes > total) return 32;
            if ((int64_t)k.n_split * k.units_per_split < k.units || (int64_t)(k.n_split - 1) * k.units_per_split >= k.units) return 33;
            if ((int64_t)k.chunks * k.RU < k.H || (int64_t)(k.chunks - 1) * k.RU >= k.H || k.units != N * k.chunks) return 34;
            if ((int64_t)k.tiles_k * 64 * pw.mb < K || (int64_t)k.tiles_c * 64 < C || pw.grid != k.tiles_k * k.tiles_c * k.n_split) return 35;
        }
        if (i8) {
            const ConvDwI8Plan p8 = conv_dw_i8_plan(N, C, H, Wd, K, R, S, pad);
            if (p8.ok && stride == 1) {
                const ConvDwI8Args &k = p8.args;
                if (p8.lds_bytes > (size_t)CDW_MAX_LDS || rb + p8.partial_bytes > total) return 36;
                if ((int64_t)k.n_split * k.units_per_split < k.units || (int64_t)(k.n_split - 1) * k.units_per_split >= k.units) return 37;
                if ((int64_t)k.chunks * k.RU < k.H || k.units != N * k.chunks || k.PW < k.Wd + 1 || k.PW % 16) return 38;
            }
        }
        const Conv1x1Plan p1 = conv1x1_dw_plan(N, C, H, Wd, K, R, S, pad, stride, i8 ? FC2I_KT : FC2_KT);
        if (p1.ok) {
            if (rb + p1.partial_bytes > total) return 39;
            if ((int64_t)p1.n_split * p1.imgs_per_split < N || (int64_t)(p1.n_split - 1) * p1.imgs_per_split >= N) return 40;
            if ((int64_t)p1.spi * p1.kt < H * Wd) return 41;
        }
        const ConvLowerPlan lp = conv_dw_lower_plan(N, C, H, Wd, K, R, S, pad, stride, i8 ? 1 : 4);
        const bool fast_dw = stride == 1 && (pw.ok || (i8 && conv_dw_i8_plan(N, C, H, Wd, K, R, S, pad).ok));
        if (lp.ok && !fast_dw) {
            if (rb + lp.bytes > total) return 42;
            if (lp.lds_bytes > (size_t)64 * 1024) return 43;
            if ((int64_t)lp.im.bands * lp.im.PB < lp.im.P || (int64_t)lp.im.ctiles * lp.im.CT < C) return 44;
            // the product on the lowered operands is a fully connected dX: its own plan must be consistent too
            const int e = check_fc2_pair(K, lp.CRS, lp.NPQ, true, false, i8 ? FC2I_KT : FC2_KT);
            if (e) return 50 + e;
        }
    }
    return 0;
}

}  // namespace dbp

extern "C" int dbp_plan_check_linear(int64_t B, int64_t in, int64_t out)
{
    if (B <= 0 || in <= 0 || out <= 0 || B > (1 << 24) || in > (1 << 24) || out > (1 << 24)) return -1;
    for (int kt = dbp::FC2_KT; kt <= dbp::FC2I_KT; kt *= 2)
        for (int m = 1; m < 4; ++m) {
            const int e = dbp::check_fc2_pair(B, in, out, (m & 1) != 0, (m & 2) != 0, kt);
            if (e) return e;
        }
    return 0;
}

extern "C" int dbp_plan_check_conv2d(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad)
{
    if (N <= 0 || C <= 0 || H <= 0 || Wd <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0 || H + 2 * pad < R || Wd + 2 * pad < S) return -1;
    if (N > 65535 || C > 65535 || K > 65535 || H > 65535 || Wd > 65535 || R > 255 || S > 255 || pad > 255 || stride > 255) return -1;
    return dbp::check_conv_plans(N, C, H, Wd, K, R, S, stride, pad);
}
