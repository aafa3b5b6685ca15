// Weight-gradient product of a convolution, Eq. (qdw) "analogously for convolutional layers", lowered to the fully
// connected product kernels for the shapes the specialised convolution kernels decline (1x1 kernels, strides, other
// kernel sizes, rows that are not a multiple of 4 pixels):
//   dW[k][(c,r,s)] = sum_{(n,p,q)} code[k][(n,p,q)] * col[(n,p,q)][(c,r,s)],   col = X[n][c][p*st+r-pad][q*st+s-pad]
// which is the dX form of a fully connected layer (rows k, reduction (n,p,q), columns (c,r,s)) once
//   * the codes [N][K][P*Q] are re-laid reduction-contiguous per channel, [K][N*P*Q]   (conv_codes_kmajor_kernel), and
//   * the activations are expanded into the column matrix, row-major                  (conv_im2col_kernel).
// Both passes are plain copies at memory speed; the product then runs on the kernels of fc2_kernel.h / fc2_i8_kernel.h.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace dbp {

// codes [N][K][PQ] -> [K][N*PQ].  One thread per group of 4 bytes when PQ is a multiple of 4 (VEC = 4), else per byte.
template <int VEC>
__global__ __launch_bounds__(256) void conv_codes_kmajor_kernel(const int8_t *src, int8_t *dst, int N, int K, int PQ, int Kt)
{
    const int64_t row = (int64_t)N * PQ, total = (int64_t)K * row / VEC;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t e = i * VEC;                               // first output byte of the group
        const int k = (int)(e / row);
        const int64_t np = e - (int64_t)k * row;
        const int n = (int)(np / PQ), pq = (int)(np - (int64_t)n * PQ);
        const int8_t *s = src + ((int64_t)n * Kt + k) * PQ + pq;          // Kt: planes per image of the source tensor
        if constexpr (VEC == 4) *(uint32_t *)(dst + e) = *(const uint32_t *)s;
        else dst[e] = *s;
    }
}

struct Im2colArgs {
    const void *X;             // [N][C][H][Wd]
    void       *col;           // [N*P*Q][C*R*S]
    int N, C, H, Wd, R, S, pad, st, P, Q;
    int Ct;                    // channels of the tensor that holds X (C unless this is one group's block)
    int CT, ctiles;            // channels per workgroup; ceil(C / CT)
    int PB, bands;             // output rows per workgroup; ceil(P / PB)
    int pitch;                 // LDS elements per channel (the band's input rows, plus one when that makes it odd)
};

// One workgroup per (image, band of PB output rows, tile of CT channels).  The input rows the band needs go to LDS as
// [channel][row][w] with loads that run along the rows; then the threads walk the band's output, (pixel, entry) with
// the entry (c,r,s) fastest, so that stores run along the rows of the column matrix.  Indices advance by additions
// (thread i handles elements i, i + 256, ...: both coordinates move by constants with a carry); the only divisions
// are in the table that maps an entry to its LDS offset and taps, built once per workgroup.  VEC = 4: a thread writes four
// consecutive entries with one store (every tile's entry count and every row of the column matrix a multiple of 4).
template <class T, int VEC>
__global__ __launch_bounds__(256) void conv_im2col_kernel(Im2colArgs a)
{
    extern __shared__ unsigned char im2col_lds[];
    int b = blockIdx.x;
    const int ct = b % a.ctiles; b /= a.ctiles;
    const int band = b % a.bands, n = b / a.bands;
    const int c0 = ct * a.CT, nc = min(a.CT, a.C - c0);
    const int p0 = band * a.PB, np = min(a.PB, a.P - p0);
    const int RS = a.R * a.S, run = nc * RS;                    // consecutive entries of one output pixel
    const int h_lo = max(p0 * a.st - a.pad, 0), h_hi = min((p0 + np - 1) * a.st - a.pad + a.R - 1, a.H - 1);
    const int rows_n = max(h_hi - h_lo + 1, 0), per_c = rows_n * a.Wd;   // elements of one channel in LDS
    uint32_t *tab = (uint32_t *)im2col_lds;                     // entry -> c*pitch | r << 20 | s << 26
    T *rows = (T *)(im2col_lds + ((run * 4 + 15) & ~15));

    for (int e = threadIdx.x; e < run; e += 256) {
        const int c = e / RS, t = e - c * RS, r = t / a.S, s = t - r * a.S;
        tab[e] = (uint32_t)(c * a.pitch) | ((uint32_t)r << 20) | ((uint32_t)s << 26);
    }
    // ---- load: element i = (c, j), j along the band's rows (contiguous in memory) ----
    if (per_c > 0) {
        const T *X = (const T *)a.X + (((int64_t)n * a.Ct + c0) * a.H + h_lo) * a.Wd;
        const int HW = a.H * a.Wd, dc = 256 / per_c, dj = 256 - dc * per_c;
        int c = threadIdx.x / per_c, j = threadIdx.x - c * per_c;
        while (c < nc) {
            rows[c * a.pitch + j] = X[(int64_t)c * HW + j];
            c += dc; j += dj;
            if (j >= per_c) { j -= per_c; ++c; }
        }
    }
    __syncthreads();
    // ---- store: element i = (pixel, group of VEC entries), pixel = (p - p0) * Q + q ----
    const int64_t CRS = (int64_t)a.C * RS;
    T *col = (T *)a.col + ((int64_t)n * a.P + p0) * a.Q * CRS + (int64_t)c0 * RS;
    const int n_px = np * a.Q, groups = run / VEC;
    const int dpx = 256 / groups, dg = 256 - dpx * groups;      // per step of 256 elements
    const int dp = dpx / a.Q, dq = dpx - dp * a.Q;
    int px = threadIdx.x / groups, g = threadIdx.x - px * groups;
    int pl = px / a.Q, q = px - pl * a.Q;                       // row of the band, column
    struct alignas(sizeof(T) * VEC) Pack { T v[VEC]; };
    while (px < n_px) {
        Pack out;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            const uint32_t t = tab[g * VEC + i];
            const int r = (t >> 20) & 63, s = t >> 26;
            const int h = (p0 + pl) * a.st + r - a.pad, w = q * a.st + s - a.pad;
            out.v[i] = (h >= h_lo && h <= h_hi && w >= 0 && w < a.Wd) ? rows[(t & 0xFFFFFu) + (h - h_lo) * a.Wd + w] : (T)0;
        }
        *(Pack *)(col + (int64_t)px * CRS + g * VEC) = out;
        px += dpx; g += dg; pl += dp; q += dq;
        if (g >= groups) { g -= groups; ++px; ++q; }
        if (q >= a.Q) { q -= a.Q; ++pl; }
        if (q >= a.Q) { q -= a.Q; ++pl; }
    }
}

}  // namespace dbp
