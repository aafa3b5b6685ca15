// Input-gradient product of a stride-1 convolution from int8 codes, the convolutional analogue of Eq. (qda):
//   dX[n,c,h,w] = Delta * sum_{k,r,s} code[n,k,h+pad-r,w+pad-s] * W[k,c,r,s]
// on bf16 matrix cores with the bf16x3 weight split (exact codes x three-plane weights, fp32 accumulate),
// or, in the full 8-bit mode (int8 weights), on int8 matrix cores with an exact int32 result: the same
// kernel with 16 reduction channels per cell instead of 8, one weight plane instead of three, and a byte
// transposition of the codes in place of their conversion.
//
// Orientation: D[c][pixel] = sum_kk Wp[c][kk] * code[kk][pixel], kk = (tap, k).  Output pixels are the
// matrix-core columns, so every store instruction writes runs of 32 consecutive pixels of one channel.
//
//   * A workgroup owns a run of consecutive output pixels of ONE image and up to four 32-channel blocks.
//     Its code patch (the pixels' rows plus the kernel halo, zero outside the image) lives in LDS as bf16
//     cells [k-group][patch pixel][8 k]: one 16-byte cell is exactly the matrix-core fragment of a lane.
//     All R*S taps read the same patch at a per-tap cell offset, so codes are fetched, transposed and
//     converted once per 32 reduction channels instead of once per tap.
//   * Weights are split into bf16 planes and re-laid once per call (conv_dx_weight_prep_kernel) into
//     fragment order [tap][k-group][plane][c][8 k]; a lane then loads its weight fragment with one
//     16-byte global load (L2-resident: every workgroup streams the same few MB in the same order).
//   * The patch is double buffered over 32-channel reduction chunks: one barrier per chunk; the next
//     chunk's codes are in flight as global loads during the current chunk's matrix-core phase.
//   * The whole reduction stays inside the workgroup: no split-K, no second launch.
//
// Stride st > 1: dX[n,c,h,w] only receives the taps r with (h + pad - r) divisible by st (likewise s), so the output
// pixels fall into st*st classes by (h mod st, w mod st), and each class is a stride-1 problem of its own on the same
// code image: output i = (h - ph)/st, taps r = r0 + st*t with r0 = (ph + pad) mod st, code row i + (ph + pad - r0)/st - t.
// The kernel therefore takes a row and a column padding, a tap count per direction and an output mapping
// (virtual pixel (i, j) -> real pixel (st*i + ph, st*j + pw)); conv_dx_multi_kernel runs all classes in one launch.
#pragma once
#include <type_traits>
#include "gemm_core.h"

namespace dbp {

constexpr int CDX_KGC = 4;            // k-groups (of 8 channels, 16 in the int8 mode) per reduction chunk
constexpr int CDX_ITMAX = 2;          // patch-fill items per thread and chunk, at most
constexpr int CDX_MAX_LDS = 64 * 1024;   // dynamic LDS a launch may ask for without raising the function attribute

struct ConvDxArgs {
    const int8_t *codes;      // [N][K][P][Q], planes PQ bytes apart and 4-byte aligned
    const uint4  *wp;         // prepared weights, cell ((tap*KG + kg)*planes + plane)*Cp + c
    void         *dX;         // [N][C][H][Wd] fp32, or int32 in the int8 mode
    int N, C, H, Wd, K, R, S, pad, P, Q;   // H, Wd, R, S, pad: of the (virtual) stride-1 problem; pad = row padding
    int pad_w;                // column padding
    int PI, PQ;               // H*Wd; bytes from one code plane to the next (P*Q, or P*Q rounded up to 4 in a padded copy)
    int64_t code_img, dx_img; // bytes from one image's codes to the next (planes of the tensor x PQ); elements from one image of dX to the next
    int oW, oPI, ost, oh0, ow0;   // output: row length and pixels per channel of the real dX, pixel (i, j) -> (ost*i + oh0, ost*j + ow0)
    int Cp, KG, n_chunks;     // C rounded to 32; k-groups in total (K rounded to a chunk); chunks of CDX_KGC k-groups
    int wc, wpx;              // waves along channels x waves along pixels (wc * wpx == 4)
    int cgroups;              // ceil(C / (32*wc))
    int tiles;                // pixel tiles per image
    int prow, pw, patch_cells;// patch rows (maximum over tiles), patch width Wd+S-1 ... cells per k-group
    Scale scale;
    Gate gate;
};

// fp32 weights [K][C][R][S] -> bf16 planes in fragment order (three planes: 0 = lo, 1 = mid, 2 = hi, their sum the weight exactly;
// two planes: 0 = lo, 1 = hi, rounded to nearest, 16 significant bits), zero padded.
// Prepared tap t holds real tap real[t] (the identity for stride 1; the classes' taps one after the other otherwise).
struct CdxTapMap { uint8_t real[64]; };

// The map is copied to LDS with compile-time indices (a run-time index into a kernel argument would send the whole
// argument through private memory); MAPPED = false: the identity, no map.
template <bool MAPPED>
__device__ __forceinline__ void cdx_stage_map(uint8_t (&lm)[64], const CdxTapMap &map)
{
    if constexpr (MAPPED) {
        if (threadIdx.x == 0) {
#pragma unroll
            for (int t = 0; t < 64; ++t) lm[t] = map.real[t];
        }
        __syncthreads();
    }
}

// The quantiser's pending statistics sum and bias gradient, taken along by the weight preparation (the first kernel after
// the quantiser on the stream): the launch has one workgroup more, and that one does nothing else.  All of its loads are
// in flight at once (the sum is of integers: any order gives the same result).  `workers` = workgroups that prepare weights.
__device__ __forceinline__ bool cdx_side_jobs(const StatsJob &job, int &workers)
{
    workers = (int)gridDim.x;
    if (job.n <= 0 && job.bias_len <= 0) return false;
    workers = (int)gridDim.x - 1;
    if ((int)blockIdx.x != workers) return false;
    if (job.n > 0) {
        __shared__ uint64_t s_sum[3][4];
        __shared__ uint32_t s_max[4];
        uint64_t nnz = 0, sat = 0, nf = 0; uint32_t mx = 0;
        for (int base = 0; base < job.n; base += 256 * 8) {
            u32x4 q[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int i = base + (int)threadIdx.x + 256 * r;
                q[r] = i < job.n ? job.partials[i] : u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int r = 0; r < 8; ++r) { nnz += q[r].x; sat += q[r].y; nf += q[r].z; mx = max(mx, q[r].w); }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            nnz += __shfl_xor((unsigned long long)nnz, off); sat += __shfl_xor((unsigned long long)sat, off);
            nf += __shfl_xor((unsigned long long)nf, off); mx = max(mx, (uint32_t)__shfl_xor((int)mx, off));
        }
        const int w = threadIdx.x >> 6;
        if ((threadIdx.x & 63) == 0) { s_sum[0][w] = nnz; s_sum[1][w] = sat; s_sum[2][w] = nf; s_max[w] = mx; }
        __syncthreads();
        if (threadIdx.x == 0) {
            job.out->nnz = s_sum[0][0] + s_sum[0][1] + s_sum[0][2] + s_sum[0][3];
            job.out->n_saturated = s_sum[1][0] + s_sum[1][1] + s_sum[1][2] + s_sum[1][3];
            job.out->n_nonfinite = s_sum[2][0] + s_sum[2][1] + s_sum[2][2] + s_sum[2][3];
            job.out->max_abs_code = (int32_t)max(max(s_max[0], s_max[1]), max(s_max[2], s_max[3]));
            job.out->reserved = 0;
            write_density_flags(job, s_sum[0][0] + s_sum[0][1] + s_sum[0][2] + s_sum[0][3]);
        }
    }
    if (job.bias_len > 0) {
        const double d = job.step_dev ? (double)job.step_dev[0] : (double)job.step;
        for (int64_t i = threadIdx.x; i < job.bias_len; i += 256) job.bias_grad[i] = (float)(d * (double)job.bias_sums[i]);
    }
    return true;
}

template <bool MAPPED, int PL>
__global__ __launch_bounds__(256) void conv_dx_weight_prep_kernel(const float *W, uint4 *wp, int K, int C, int RS, int KG, int Cp, int RS_real, CdxTapMap map,
                                                                  StatsJob job)
{
    __shared__ uint8_t lm[64];
    int workers;
    if (cdx_side_jobs(job, workers)) return;
    cdx_stage_map<MAPPED>(lm, map);
    const int64_t total = (int64_t)RS * KG * Cp;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)workers * 256) {
        const int c = (int)(i % Cp);
        const int64_t t = i / Cp;
        const int kg = (int)(t % KG), tap = (int)(t / KG);
        const int rtap = MAPPED ? (int)lm[tap] : tap;
        float w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int k = kg * 8 + j;
            w[j] = (k < K && c < C) ? W[((int64_t)k * C + c) * RS_real + rtap] : 0.0f;
        }
        uint4 *dst = wp + ((int64_t)tap * KG + kg) * PL * Cp + c;
        if constexpr (PL == 3) {
            uint32_t h[8], m[8], l[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) split3(w[j], h[j], m[j], l[j]);
            dst[0]      = uint4{(l[0] >> 16) | l[1], (l[2] >> 16) | l[3], (l[4] >> 16) | l[5], (l[6] >> 16) | l[7]};
            dst[Cp]     = uint4{(m[0] >> 16) | m[1], (m[2] >> 16) | m[3], (m[4] >> 16) | m[5], (m[6] >> 16) | m[7]};
            dst[2 * Cp] = uint4{(h[0] >> 16) | h[1], (h[2] >> 16) | h[3], (h[4] >> 16) | h[5], (h[6] >> 16) | h[7]};
        } else {
            uint32_t h[4], l[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) split2_pk(w[2 * j], w[2 * j + 1], h[j], l[j]);
            dst[0]  = uint4{l[0], l[1], l[2], l[3]};
            dst[Cp] = uint4{h[0], h[1], h[2], h[3]};
        }
    }
}

// int8 weights [K][C][R][S] -> cells of 16 reduction channels in fragment order [tap][k-group][c], zero padded.
template <bool MAPPED>
__global__ __launch_bounds__(256) void conv_dx_weight_prep_i8_kernel(const int8_t *W, uint4 *wp, int K, int C, int RS, int KG, int Cp, int RS_real, CdxTapMap map,
                                                                     StatsJob job)
{
    __shared__ uint8_t lm[64];
    int workers;
    if (cdx_side_jobs(job, workers)) return;
    cdx_stage_map<MAPPED>(lm, map);
    const int64_t total = (int64_t)RS * KG * Cp;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)workers * 256) {
        const int c = (int)(i % Cp);
        const int64_t t = i / Cp;
        const int kg = (int)(t % KG), tap = (int)(t / KG);
        const int rtap = MAPPED ? (int)lm[tap] : tap;
        uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int k = kg * 16 + j;
            const uint32_t w = (k < K && c < C) ? (uint32_t)(uint8_t)W[((int64_t)k * C + c) * RS_real + rtap] : 0u;
            d[j >> 2] |= w << (8 * (j & 3));
        }
        wp[i] = uint4{d[0], d[1], d[2], d[3]};
    }
}

// Code planes of P*Q bytes -> planes of `plane` bytes (a multiple of 4, zero filled): the patch fill reads aligned dwords.
// Plane pl = (n, k) of the copy is plane n*Kt + k of the source tensor (Kt = K unless the K planes are one group's block).
__global__ __launch_bounds__(256) void conv_dx_pad_codes_kernel(const int8_t *src, uint32_t *dst, int64_t planes, int pq, int plane, int K, int Kt)
{
    const int dpp = plane >> 2;                                  // dwords per padded plane
    const int64_t total = planes * dpp;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t pl = i / dpp;
        const int j0 = 4 * (int)(i - pl * dpp);
        const int8_t *s = src + (pl / K * Kt + pl % K) * pq + j0;
        uint32_t v = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j0 + e < pq) v |= (uint32_t)(uint8_t)s[e] << (8 * e);
        dst[i] = v;
    }
}

template <int MODE> struct CdxTraits;
template <> struct CdxTraits<MODE_BF16> { static constexpr int G = 8,  PL = 3; using Acc = f32x16; using Out = float; };
template <> struct CdxTraits<MODE_BF16X2> { static constexpr int G = 8, PL = 2; using Acc = f32x16; using Out = float; };
template <> struct CdxTraits<MODE_I8>   { static constexpr int G = 16, PL = 1; using Acc = i32x16; using Out = int32_t; };

__device__ __forceinline__ uint32_t cdx_bf16_pair(uint32_t wa, uint32_t wb, int e)
{
    // bytes e of words wa, wb as signed codes -> two bf16 (exact), wa's in the low half
    const float fa = (float)((int)(wa << (24 - 8 * e)) >> 24), fb = (float)((int)(wb << (24 - 8 * e)) >> 24);
    return __builtin_amdgcn_perm(__float_as_uint(fb), __float_as_uint(fa), 0x07060302u);
}

extern __shared__ uint4 cdx_lds[];                           // [2][CDX_KGC][patch_cells]

// STRIDED = false: the column padding is the row padding and a pixel's flat index is its place in dX (compile-time
// facts of the stride-1 launch).
// RING3: the weight fragments go through three register sets instead of two (tap counts that are a multiple of 3 only; see the
// loop itself).
template <int NB, int MODE, bool STRIDED, bool RING3>
__device__ __forceinline__ void conv_dx_body(const ConvDxArgs &a, int b)
{
    using TR = CdxTraits<MODE>;
    constexpr int G = TR::G, PL = TR::PL;                       // reduction channels per cell; weight planes
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lcol = lane & 31, lhalf = lane >> 5;

    // ---- which tile ------------------------------------------------------------------------------
    const int cg = b % a.cgroups; b /= a.cgroups;
    const int tile = b % a.tiles, n = b / a.tiles;
    const int wave_c = wave % a.wc, wave_p = wave / a.wc;
    const int cb = cg * a.wc + wave_c;                       // 32-channel block of this wave
    const int tile_px = a.wpx * 32 * NB;
    const int j0 = tile * tile_px;                           // first flat pixel of the workgroup
    const int j_end = min(j0 + tile_px, a.PI);               // one past its last pixel
    const int jw0 = j0 + wave_p * 32 * NB;                   // first pixel of this wave

    // patch geometry: code rows p_lo..p_hi, columns q_lo..q_lo+pw-1
    const int h_first = j0 / a.Wd, h_last = (j_end - 1) / a.Wd;
    const int p_lo = h_first + a.pad - (a.R - 1), q_lo = (STRIDED ? a.pad_w : a.pad) - (a.S - 1);
    const int p_a = max(p_lo, 0), p_b = min(h_last + a.pad, a.P - 1);   // rows that exist in the code image
    const int buf_cells = CDX_KGC * a.patch_cells;

    // ---- zero both buffers (halo and out-of-image cells stay zero for good) -----------------------
    for (int i = tid; i < 2 * buf_cells; i += 256) cdx_lds[i] = uint4{0u, 0u, 0u, 0u};

    // ---- patch-fill items of this thread: (k-group, aligned dword of the rows' flat byte range) ----
    const int f_a = (p_a * a.Q) & ~3;
    const int n_dw = p_b >= p_a ? ((p_b + 1) * a.Q - f_a + 3) >> 2 : 0;
    const int n_items = n_dw * CDX_KGC;
    int      item_goff[CDX_ITMAX];                           // byte offset inside the chunk's first code plane
    int      item_k[CDX_ITMAX];                              // first channel of the item's k-group inside the chunk
    uint32_t item_cell[CDX_ITMAX][2];                        // four 16-bit cell indices (0xFFFF = skip)
#pragma unroll
    for (int i = 0; i < CDX_ITMAX; ++i) {
        const int it = tid + 256 * i;
        item_goff[i] = -1; item_k[i] = 0;
        item_cell[i][0] = item_cell[i][1] = 0xFFFFFFFFu;
        if (it < n_items) {
            const int kgl = it / n_dw, f = it - kgl * n_dw;
            const int pix0 = f_a + 4 * f;
            item_goff[i] = kgl * G * a.PQ + pix0; item_k[i] = kgl * G;
            uint32_t cells[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int pix = pix0 + e, p = pix / a.Q, q = pix - p * a.Q;
                const bool need = p >= p_a && p <= p_b && q >= q_lo && q - q_lo < a.pw;
                cells[e] = need ? (uint32_t)(kgl * a.patch_cells + (p - p_lo) * a.pw + (q - q_lo)) : 0xFFFFu;
            }
            item_cell[i][0] = cells[0] | (cells[1] << 16);
            item_cell[i][1] = cells[2] | (cells[3] << 16);
        }
    }
    uint32_t raw[CDX_ITMAX][G];
    const int8_t *img = a.codes + (int64_t)n * a.code_img;
    auto fetch_chunk = [&](int chunk) {
#pragma unroll
        for (int i = 0; i < CDX_ITMAX; ++i) {
#pragma unroll
            for (int kq = 0; kq < G; ++kq) raw[i][kq] = 0u;
            if (item_goff[i] >= 0) {
                const int k0 = chunk * (G * CDX_KGC) + item_k[i];
                const int8_t *src = img + (int64_t)chunk * (G * CDX_KGC) * a.PQ + item_goff[i];
#pragma unroll
                for (int kq = 0; kq < G; ++kq)
                    if (k0 + kq < a.K) raw[i][kq] = *(const uint32_t *)(src + (int64_t)kq * a.PQ);
            }
        }
    };
    auto store_chunk = [&](int buf) {
        uint4 *dst = cdx_lds + buf * buf_cells;
#pragma unroll
        for (int i = 0; i < CDX_ITMAX; ++i) {
            if (item_goff[i] < 0) continue;
            if constexpr (MODE == MODE_I8) {
                // byte e of the 16 channel words -> the 16 bytes of pixel e's cell: four 4x4 byte transpositions
                uint32_t t[4][4];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint32_t r0 = raw[i][4 * g], r1 = raw[i][4 * g + 1], r2 = raw[i][4 * g + 2], r3 = raw[i][4 * g + 3];
                    const uint32_t x0 = __builtin_amdgcn_perm(r1, r0, 0x05010400u), x1 = __builtin_amdgcn_perm(r3, r2, 0x05010400u);
                    const uint32_t y0 = __builtin_amdgcn_perm(r1, r0, 0x07030602u), y1 = __builtin_amdgcn_perm(r3, r2, 0x07030602u);
                    t[g][0] = __builtin_amdgcn_perm(x1, x0, 0x05040100u); t[g][1] = __builtin_amdgcn_perm(x1, x0, 0x07060302u);
                    t[g][2] = __builtin_amdgcn_perm(y1, y0, 0x05040100u); t[g][3] = __builtin_amdgcn_perm(y1, y0, 0x07060302u);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t cell = (item_cell[i][e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                    if (cell == 0xFFFFu) continue;
                    dst[cell] = uint4{t[0][e], t[1][e], t[2][e], t[3][e]};
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t cell = (item_cell[i][e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                    if (cell == 0xFFFFu) continue;
                    dst[cell] = uint4{cdx_bf16_pair(raw[i][0], raw[i][1], e), cdx_bf16_pair(raw[i][2], raw[i][3], e),
                                      cdx_bf16_pair(raw[i][4], raw[i][5], e), cdx_bf16_pair(raw[i][6], raw[i][7], e)};
                }
            }
        }
    };

    // ---- per-lane patch cell of each owned pixel (tap (0,0) position; a tap subtracts r*pw + s) ----
    int lane_cell[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int j = jw0 + 32 * nb + lcol;
        j = min(j, a.PI - 1);                                 // tail lanes compute a valid pixel again; not stored
        const int h = j / a.Wd, w = j - h * a.Wd;
        lane_cell[nb] = (h - h_first + a.R - 1) * a.pw + (w + a.S - 1) + lhalf * a.patch_cells;
    }

    typename TR::Acc acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0;

    const bool wave_active = cb * 32 < a.C && jw0 < j_end;   // uniform per wave
    const int RS = a.R * a.S;
    const int64_t kg_stride = (int64_t)PL * a.Cp;            // cells per k-group
    // Weight fragments: a step is (tap, half of the chunk's k-groups); its row of the prepared weights is a uniform pointer
    // and the lane's place in the row a 32-bit index (one address register per plane).  A cursor walks the steps in the
    // order in which they are multiplied and stays on the last one when it gets there: the loads are the same on every
    // path (a load on only some paths makes the compiler wait for ALL loads in flight at every step).
    const uint32_t wl = (uint32_t)(lhalf * PL * a.Cp + cb * 32 + lcol);
    int l_chunk = 0, l_tap = 0, l_kk = 0;                     // uniform: the step the next load fetches
    auto next_load = [&](u32x4 (&dst)[PL]) {
        const uint4 *row = a.wp + ((int64_t)l_tap * a.KG + l_chunk * CDX_KGC + 2 * l_kk) * kg_stride;
#pragma unroll
        for (int pl = 0; pl < PL; ++pl) { const uint4 t = row[wl + (uint32_t)(pl * a.Cp)]; dst[pl] = u32x4{t.x, t.y, t.z, t.w}; }
        if (l_kk == 0) l_kk = 1;
        else { l_kk = 0; if (++l_tap == RS) { l_tap = 0; ++l_chunk; } }
        if (l_chunk == a.n_chunks) { l_chunk = a.n_chunks - 1; l_tap = RS - 1; l_kk = 1; }
    };

    // ---- the multiply phase ------------------------------------------------------------------------------------------
    // A STEP is (tap, half of the chunk's k-groups): one weight fragment set (PL planes) against the code fragments of the
    // wavefront's NB pixel blocks, PL*NB matrix instructions.  One wavefront per SIMD and workgroup: nothing but the
    // wavefront's own instruction order hides the latency of its operands (in-kernel cycle stamps on the 56x56 layer: a step
    // took 1420 cycles for 672 cycles of matrix instructions, whether the wavefront had its SIMD to itself or not).  Hence:
    //   * weight fragments (from L2, several hundred cycles away) are requested one or two steps ahead (RING3: three register
    //     sets instead of two; tap counts that are a multiple of 3, where six steps bring the ring back to its start and the sets
    //     keep compile-time names);
    //   * code fragments (from LDS) are software-pipelined against the matrix instructions.  Seven pixel blocks: two groups
    //     (blocks 0-3, 4-6); while a step's first group is multiplied its second group is on its way, and while the second
    //     is multiplied the NEXT step's first group is; a group's registers are reused as soon as the instructions that read
    //     them have been issued.  Up to four blocks: one group in two register sets that alternate between the steps;
    //   * every step issues the same loads.  At a chunk's last step the next fragments are not there yet (other buffer,
    //     behind a barrier): that step reads its own again, and the chunk's first fragments are read after the barrier.
    constexpr int NB0 = NB > 4 ? 4 : NB, NB1 = NB > 4 ? NB - 4 : NB;   // seven blocks: the two groups; else: the two sets
    u32x4 bA[NB0], bB[NB1];
    const uint4 *pb = cdx_lds;
    const int hi = 2 * a.patch_cells;                         // the second half of the chunk's k-groups
    int m_r = 0, m_s = 0, m_kk = 0;                           // the step whose patch offset next_off() returns next
    auto next_off = [&]() {
        const int o = (m_kk ? hi : 0) - (m_r * a.pw + m_s);
        if (m_kk == 0) m_kk = 1;
        else { m_kk = 0; if (++m_s == a.S) { m_s = 0; ++m_r; } }
        return o;
    };
    auto read_a = [&](int off) {                              // blocks 0 .. NB0-1 -> bA
#pragma unroll
        for (int nb = 0; nb < NB0; ++nb) { const uint4 t = pb[lane_cell[nb] + off]; bA[nb] = u32x4{t.x, t.y, t.z, t.w}; }
    };
    auto read_b = [&](int off) {                              // seven blocks: blocks 4-6; else blocks 0 .. NB-1 -> bB
        constexpr int first = NB > 4 ? NB0 : 0;
#pragma unroll
        for (int nb = 0; nb < NB1; ++nb) { const uint4 t = pb[lane_cell[first + nb] + off]; bB[nb] = u32x4{t.x, t.y, t.z, t.w}; }
    };
    auto mma_a = [&](const u32x4 (&af)[PL]) {
#pragma unroll
        for (int pl = 0; pl < PL; ++pl)
#pragma unroll
            for (int nb = 0; nb < NB0; ++nb) Mma<MODE>::run(af[pl], bA[nb], acc[nb]);
    };
    auto mma_b = [&](const u32x4 (&af)[PL]) {
        constexpr int first = NB > 4 ? NB0 : 0;
#pragma unroll
        for (int pl = 0; pl < PL; ++pl)
#pragma unroll
            for (int nb = 0; nb < NB1; ++nb) Mma<MODE>::run(af[pl], bB[nb], acc[first + nb]);
    };
    int off = 0;
    // one step with weight set `cur`, the load of the step one or two ahead into `nxt_w`; `again`: the chunk's last step.
    // Seven blocks: both groups belong to this step.  Else: EVEN steps multiply bA and read the next step into bB, odd ones
    // the other way round.
    auto step = [&](u32x4 (&nxt_w)[PL], const u32x4 (&cur)[PL], bool again, auto even) {
        const int nxt = again ? off : next_off();
        next_load(nxt_w);
        if constexpr (NB > 4) { read_b(off); mma_a(cur); read_a(nxt); mma_b(cur); }
        else if constexpr (decltype(even)::value) { read_b(nxt); mma_a(cur); }
        else { read_a(nxt); mma_b(cur); }
        off = nxt;
    };
    constexpr std::true_type EVEN{};
    constexpr std::false_type ODD{};
    auto begin_chunk = [&](int chunk) {                       // all wavefronts: stage the chunk, fetch the next one's codes
        const int buf = chunk & 1;
        store_chunk(buf);
        __syncthreads();
        fetch_chunk(min(chunk + 1, a.n_chunks - 1));          // in flight during the matrix-core phase (the last chunk once more, unused)
        pb = cdx_lds + buf * buf_cells;
        m_r = m_s = m_kk = 0;
    };

    fetch_chunk(0);
    if constexpr (RING3) {
        u32x4 f0[PL], f1[PL], f2[PL];
        if (wave_active) { next_load(f0); next_load(f1); }
        __syncthreads();                                      // zero fill done before the first patch writes
        for (int chunk = 0; chunk < a.n_chunks; ++chunk) {
            begin_chunk(chunk);
            if (wave_active) {
                off = next_off();
                read_a(off);
                for (int tap = 0; tap < RS; tap += 3) {
                    step(f2, f0, false, EVEN); step(f0, f1, false, ODD); step(f1, f2, false, EVEN);
                    step(f2, f0, false, ODD);  step(f0, f1, false, EVEN); step(f1, f2, tap + 3 >= RS, ODD);
                }
            }
        }
    } else {
        u32x4 a0[PL], a1[PL];                                 // weight fragments of the two halves of a chunk's k-groups, one step ahead
        if (wave_active) next_load(a0);
        __syncthreads();                                      // zero fill done before the first patch writes
        for (int chunk = 0; chunk < a.n_chunks; ++chunk) {
            begin_chunk(chunk);
            if (wave_active) {
                off = next_off();
                read_a(off);
                for (int tap = 0; tap < RS; ++tap) {
                    step(a1, a0, false, EVEN);
                    step(a0, a1, tap + 1 >= RS, ODD);
                }
            }
        }
    }

    // ---- store: lane holds pixel column lcol, channel rows 8*(v/4) + 4*lhalf + v%4 of its block ----
    if (wave_active) {
        typename TR::Out *out = (typename TR::Out *)a.dX + (int64_t)n * a.dx_img;  // offsets inside one image fit 31 bits (host check)
        const float sc = MODE == MODE_I8 ? 1.0f : a.scale.get();
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int j = jw0 + 32 * nb + lcol;
            if (j >= j_end) continue;
            const int c0 = cb * 32 + 4 * lhalf;
            int px = j;                                           // where the pixel sits in the real dX plane
            if constexpr (STRIDED) { const int h = j / a.Wd, w = j - h * a.Wd; px = (a.ost * h + a.oh0) * a.oW + a.ost * w + a.ow0; }
            const int opi = STRIDED ? a.oPI : a.PI;
            int off = c0 * opi + px;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int c = c0 + 8 * (v >> 2) + (v & 3);
                if (c < a.C) {
                    if constexpr (MODE == MODE_I8) out[off] = acc[nb][v]; else out[off] = acc[nb][v] * sc;
                }
                off += (v & 3) == 3 ? 5 * opi : opi;
            }
        }
    }
}

template <int NB, int MODE, bool RING3>
__global__ __launch_bounds__(256, 2) void conv_dx_kernel(ConvDxArgs a)
{
    if (a.gate.closed()) return;
    conv_dx_body<NB, MODE, false, RING3>(a, (int)blockIdx.x);
}

// The classes of a strided problem in one launch: workgroups [first[i], first[i + 1]) run class i.
constexpr int CDX_MAX_CLASSES = 9;
struct ConvDxMulti { ConvDxArgs cls[CDX_MAX_CLASSES]; int first[CDX_MAX_CLASSES + 1]; int n; };

template <int NB, int MODE>
__global__ __launch_bounds__(256, 2) void conv_dx_multi_kernel(ConvDxMulti m)
{
    if (m.cls[0].gate.closed()) return;
    int ci = 0;
    for (int i = 1; i < m.n; ++i) if ((int)blockIdx.x >= m.first[i]) ci = i;
    const ConvDxArgs a = m.cls[ci];
    conv_dx_body<NB, MODE, true, false>(a, (int)blockIdx.x - m.first[ci]);
}

}  // namespace dbp
