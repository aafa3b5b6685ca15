// Gather path of the fully connected products: walk only the nonzero codes (Sec. "Computational
// complexity": O(p_nz * m*k*n) multiply-adds instead of O(m*k*n)).  Plain fp32 FMA on the vector ALUs,
// one output row slab per workgroup, operands streamed through L2.  Pays off only at very high
// sparsity; the matrix-core path is faster below the measured threshold.
#include "common.h"

namespace dbp {

namespace {

constexpr int kSlab = 1024;     // output columns per workgroup: 256 threads x 4

// dX[b, i] = step * sum over nonzero (o, k) of row b:  k * W[o, i]
template <bool VEC>
__global__ __launch_bounds__(256) void linear_dx_gather_kernel(FormatView f, const float *W, float *dX,
                                                                int in, int out, Scale step_arg)
{
    const int b = blockIdx.y;
    const int i0 = blockIdx.x * kSlab + 4 * threadIdx.x;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const int tpr = (int)f.tiles_per_row;
    for (int seg = 0; seg < tpr; ++seg) {
        const int64_t t = (int64_t)b * tpr + seg;
        const int cnt = f.tile_nnz[t];
        const uint16_t *ent = f.entries + t * DBP_TILE;
        for (int e0 = 0; e0 < cnt; e0 += 4) {
            int o[4]; float k[4]; bool ok[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                ok[u] = e0 + u < cnt;                                  // workgroup-uniform
                const uint32_t en = ok[u] ? ent[e0 + u] : 0u;
                o[u] = seg * DBP_TILE + (int)(en >> 8);
                k[u] = (float)(int8_t)(en & 0xFF);
            }
            if (VEC) {
                if (i0 < in) {
                    f32x4 w[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (ok[u]) w[u] = *(const f32x4 *)(W + (int64_t)o[u] * in + i0);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        if (!ok[u]) continue;
                        acc[0] = __builtin_fmaf(k[u], w[u].x, acc[0]); acc[1] = __builtin_fmaf(k[u], w[u].y, acc[1]);
                        acc[2] = __builtin_fmaf(k[u], w[u].z, acc[2]); acc[3] = __builtin_fmaf(k[u], w[u].w, acc[3]);
                    }
                }
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (ok[u] && i0 + j < in) acc[j] = __builtin_fmaf(k[u], W[(int64_t)o[u] * in + i0 + j], acc[j]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (i0 + j < in) dX[(int64_t)b * in + i0 + j] = step_arg.get() * acc[j];
}

// dW[o, i] = step * sum over batch rows b with code[b,o] != 0:  k * X[b, i]   (int32 sum for int8 X)
template <class XT, class AccT, bool VEC>
__global__ __launch_bounds__(256) void linear_dw_gather_kernel(const int8_t *codes, const XT *X, AccT *dW,
                                                                int B, int in, int out, Scale step_arg)
{
    __shared__ uint32_t s_list[4096];       // (b << 8) | code, batch order; B <= 4096 per pass
    __shared__ int s_cnt[4];
    const int o = blockIdx.y;
    const int i0 = blockIdx.x * kSlab + 4 * threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    AccT acc[4] = {0, 0, 0, 0};

    for (int b_base = 0; b_base < B; b_base += 4096) {
        // deterministic compaction of the nonzero batch indices of column o
        int n_list = 0;
        const int b_lim = min(B, b_base + 4096);
        for (int c0 = b_base; c0 < b_lim; c0 += 256) {
            const int b = c0 + threadIdx.x;
            const int k = b < b_lim ? (int)codes[(int64_t)b * out + o] : 0;
            const uint64_t m = __builtin_amdgcn_ballot_w64(k != 0);
            if (lane == 0) s_cnt[wave] = __builtin_popcountll(m);
            __syncthreads();
            int off = n_list;
            for (int w = 0; w < wave; ++w) off += s_cnt[w];
            const int total = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
            if (k != 0) {
                const int pre = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                s_list[off + pre] = ((uint32_t)b << 8) | (uint32_t)(k & 0xFF);
            }
            n_list += total;
            __syncthreads();
        }
        for (int e0 = 0; e0 < n_list; e0 += 4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (e0 + u >= n_list) break;
                const uint32_t en = s_list[e0 + u];
                const int b = (int)(en >> 8);
                const AccT k = (AccT)(int8_t)(en & 0xFF);
                const XT *xr = X + (int64_t)b * in + i0;
                if (VEC) {
                    if (i0 < in) {
                        if (sizeof(XT) == 4) {
                            const f32x4 x = *(const f32x4 *)xr;
                            acc[0] += k * (AccT)x.x; acc[1] += k * (AccT)x.y; acc[2] += k * (AccT)x.z; acc[3] += k * (AccT)x.w;
                        } else {
                            const uint32_t x = *(const uint32_t *)xr;
                            acc[0] += k * (AccT)(int8_t)x; acc[1] += k * (AccT)(int8_t)(x >> 8);
                            acc[2] += k * (AccT)(int8_t)(x >> 16); acc[3] += k * (AccT)(int8_t)(x >> 24);
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (i0 + j < in) acc[j] += k * (AccT)xr[j];
                }
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (i0 + j < in) {
            if (sizeof(XT) == 4) dW[(int64_t)o * in + i0 + j] = (AccT)(step_arg.get() * (float)acc[j]);
            else dW[(int64_t)o * in + i0 + j] = acc[j];
        }
}

// ---- convolution -------------------------------------------------------------------------------
// The format's rows are the code planes (n, k) of P*Q pixels.  Both kernels give every lane ONE (channel, tap) pair
// and walk the nonzero codes of the planes they need in a fixed order (deterministic sums): 64 / (R*S) channels per
// wavefront, four wavefronts per workgroup.  The walk goes over the tiles of the workgroup's planes in chunks of up to 256
// tiles: their entry counts are scanned, and the entries of as many tiles as fit are copied into LDS as (p, q, code,
// plane) records -- at high sparsity most tiles are empty and one chunk (three barriers) covers hundreds of planes.
struct ConvGatherGeom { int N, C, H, Wd, K, R, S, pad, st, P, Q, cpw; };   // cpw: channels per wavefront

constexpr int kChunkCap = 1024;                           // entry records per chunk (a tile has at most 256)

struct GatherChunk {
    uint32_t ent[kChunkCap];                              // p | q << 12 | code << 24
    uint16_t plane[kChunkCap];                            // index of the plane in the walk
    int wave_sum[4];
    int n_tiles, n_ent;
};

// Tiles i0 .. of the walk (tile i = segment i % tpr of plane i / tpr; plane j is format row row0 + j * row_stride):
// as many as fit, at most 256.  Returns after a barrier; ch.n_tiles >= 1 whenever i0 < n_walk.
__device__ __forceinline__ void conv_gather_chunk(const FormatView &f, int64_t row0, int64_t row_stride, int tpr, int i0, int n_walk,
                                                  int Q, GatherChunk &ch)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = i0 + tid;
    const bool valid = i < n_walk;
    const int j = valid ? i / tpr : 0, seg = valid ? i - j * tpr : 0;
    const int64_t t = (row0 + (int64_t)j * row_stride) * tpr + seg;
    const int cnt = valid ? (int)f.tile_nnz[t] : 0;
    int incl = cnt;                                        // inclusive scan over the workgroup
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    __syncthreads();                                       // the chunk before has been consumed
    if (lane == 63) ch.wave_sum[wave] = incl;
    if (tid == 0) { ch.n_tiles = 0; ch.n_ent = 0; }
    __syncthreads();
    for (int w = 0; w < wave; ++w) incl += ch.wave_sum[w];
    const bool fits = valid && incl <= kChunkCap;          // a prefix of the threads (counts are non-negative)
    const uint64_t m = __builtin_amdgcn_ballot_w64(fits);
    if (lane == 0 && m) { atomicAdd(&ch.n_tiles, __builtin_popcountll(m)); }
    if (fits) atomicMax(&ch.n_ent, incl);
    if (fits) {
        const uint16_t *src = f.entries + t * DBP_TILE;
        const int at = incl - cnt;
        for (int e = 0; e < cnt; ++e) {
            const uint32_t en = src[e];
            const int pix = seg * DBP_TILE + (int)(en >> 8), p = pix / Q, q = pix - p * Q;
            ch.ent[at + e] = (uint32_t)p | ((uint32_t)q << 12) | ((en & 0xFFu) << 24);
            ch.plane[at + e] = (uint16_t)j;
        }
    }
    __syncthreads();
}

// dW[k,c,r,s] = step * sum_n sum_{nonzero (p,q) of plane (n,k)} code * X[n,c,p*st+r-pad,q*st+s-pad]
// Workgroup (channel tile, k); a lane owns one element of dW.  fp32 X accumulates in fp64 (the products are exact
// there), int8 X in int32 (exact).
template <class XT, class AccT, class OutT>
__global__ __launch_bounds__(256) void conv_dw_gather_kernel(FormatView f, const XT *X, OutT *dW, ConvGatherGeom g, Scale step_arg)
{
    __shared__ GatherChunk ch;
    const int k = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int RS = g.R * g.S, cl = lane / RS, tap = lane - cl * RS;
    const int c = ((int)blockIdx.x * 4 + wave) * g.cpw + cl;
    const bool own = cl < g.cpw && c < g.C;
    const int r = tap / g.S, s = tap - r * g.S, tpr = (int)f.tiles_per_row, HW = g.H * g.Wd;
    const int n_walk = g.N * tpr, img = g.C * HW;          // elements of X per image (the host keeps N*C*H*Wd below 2^31)
    const XT *xc = X + (own ? c : 0) * HW;
    AccT acc = 0;
    for (int i0 = 0; i0 < n_walk;) {
        conv_gather_chunk(f, k, g.K, tpr, i0, n_walk, g.Q, ch);     // plane j of the walk = image j: row j*K + k
        const int n_ent = ch.n_ent;
        i0 += ch.n_tiles;
        // eight unconditional loads at a time (pixels outside the image read element 0 and add nothing): the loop is
        // bound by their latency
        for (int e0 = 0; e0 < n_ent; e0 += 8) {
            XT x[8];
            AccT kq[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = min(e0 + u, n_ent - 1);
                const uint32_t v = ch.ent[e];
                const int n = ch.plane[e];
                const int h = (int)(v & 0xFFFu) * g.st + r - g.pad, w = (int)((v >> 12) & 0xFFFu) * g.st + s - g.pad;
                const bool in = own && e0 + u < n_ent && h >= 0 && h < g.H && w >= 0 && w < g.Wd;
                x[u] = xc[in ? n * img + h * g.Wd + w : 0];
                kq[u] = in ? (AccT)(int8_t)(v >> 24) : (AccT)0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += kq[u] * (AccT)x[u];
        }
    }
    if (own) {
        OutT *o = dW + (((int64_t)k * g.C + c) * g.R + r) * g.S + s;
        if constexpr (sizeof(XT) == 4) *o = (OutT)((double)step_arg.get() * acc); else *o = (OutT)acc;
    }
}

// dX[n,c,h,w] = step * sum_k sum_{nonzero (p,q) of plane (n,k)} code * W[k,c,r,s],  h = p*st+r-pad, w = q*st+s-pad
// Workgroup (channel tile, n): the dX planes of its channels accumulate in LDS.  For one nonzero the lanes of a channel
// hit different pixels (one per tap) and different channels different planes, so the read-add-write needs no atomics.
__global__ __launch_bounds__(256) void conv_dx_gather_kernel(FormatView f, const float *W, float *dX, ConvGatherGeom g, Scale step_arg)
{
    extern __shared__ float cg_planes[];                 // [4 * cpw channels][H*Wd], then the chunk
    const int n = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int RS = g.R * g.S, cl = lane / RS, tap = lane - cl * RS;
    const int c_first = (int)blockIdx.x * 4 * g.cpw, c = c_first + wave * g.cpw + cl;
    const bool own = cl < g.cpw && c < g.C;
    const int r = tap / g.S, s = tap - r * g.S, tpr = (int)f.tiles_per_row, HW = g.H * g.Wd;
    const int n_planes = 4 * g.cpw, n_walk = g.K * tpr;
    GatherChunk &ch = *(GatherChunk *)(cg_planes + (size_t)n_planes * HW);
    for (int i = threadIdx.x; i < n_planes * HW; i += 256) cg_planes[i] = 0.f;   // (ordered by the first chunk's barriers)
    float *mine = cg_planes + (size_t)(wave * g.cpw + (own ? cl : 0)) * HW;
    const float *wl = W + ((int64_t)(own ? c : 0) * g.R + r) * g.S + s;          // + k * C*R*S
    const int CRS = g.C * RS;
    for (int i0 = 0; i0 < n_walk;) {
        conv_gather_chunk(f, (int64_t)n * g.K, 1, tpr, i0, n_walk, g.Q, ch);     // plane j of the walk = channel k = j
        const int n_ent = ch.n_ent;
        i0 += ch.n_tiles;
        // Four entries at a time: their weights are loaded together (at high sparsity every entry is another plane k, and
        // one dependent load per entry was the bound).  The read-add-write of the entries stays in order: the taps of two
        // nearby entries reach the same pixels through different lanes.
        for (int e0 = 0; e0 < n_ent; e0 += 4) {
            uint32_t v[4];
            float wv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = min(e0 + u, n_ent - 1);
                v[u] = ch.ent[e];
                wv[u] = own ? wl[(int64_t)ch.plane[e] * CRS] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int h = (int)(v[u] & 0xFFFu) * g.st + r - g.pad, w = (int)((v[u] >> 12) & 0xFFFu) * g.st + s - g.pad;
                if (own && e0 + u < n_ent && h >= 0 && h < g.H && w >= 0 && w < g.Wd)
                    mine[h * g.Wd + w] += (float)(int8_t)(v[u] >> 24) * wv[u];
            }
        }
    }
    __syncthreads();
    const float step = step_arg.get();
    const int nc = min(n_planes, g.C - c_first);
    // plane j of the tile is channel c_first + j (wavefront j / cpw, channel j % cpw of its group)
    float *out = dX + ((int64_t)n * g.C + c_first) * HW;
    for (int i = threadIdx.x; i < nc * HW; i += 256) out[i] = step * cg_planes[i];
}

}  // namespace

// LDS of the dX kernel beside its planes: the chunk of entry records.
constexpr size_t kConvGatherFixedLds = sizeof(GatherChunk) + 16;

bool conv_gather_supported(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t P, int64_t Q, bool want_dx)
{
    if (R * S > 64 || P >= 4096 || Q >= 4096) return false;                      // a lane per tap; 12-bit coordinates
    if (N >= 65536 || K >= 65536 || N * C * H * Wd >= ((int64_t)1 << 31)) return false;   // 16-bit plane numbers, 32-bit offsets into X
    if (want_dx && (size_t)(4 * H * Wd * 4) + kConvGatherFixedLds > (size_t)150 * 1024) return false;   // a plane per wavefront at least
    return true;
}

hipError_t launch_conv_gather(const ConvArgs &a, const FormatView &f, hipStream_t s)
{
    ConvGatherGeom g;
    g.N = (int)a.N; g.C = (int)a.C; g.H = (int)a.H; g.Wd = (int)a.Wd; g.K = (int)a.K; g.R = (int)a.R; g.S = (int)a.S;
    g.pad = (int)a.pad; g.st = (int)a.stride;
    g.P = (int)((a.H + 2 * a.pad - a.R) / a.stride + 1); g.Q = (int)((a.Wd + 2 * a.pad - a.S) / a.stride + 1);
    const int RS = g.R * g.S, cpw_max = 64 / RS;
    const Scale step{a.step, a.step_dev};
    if (a.dX) {
        const size_t HW4 = (size_t)g.H * g.Wd * 4, budget = (size_t)150 * 1024 - kConvGatherFixedLds;
        int cpw = cpw_max;
        while (cpw > 1 && (size_t)4 * cpw * HW4 > budget) --cpw;
        g.cpw = cpw;
        const size_t lds = (((size_t)4 * cpw * HW4 + 15) & ~(size_t)15) + kConvGatherFixedLds;
        static size_t raised = 0;
        if (lds > 64 * 1024 && lds > raised) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_dx_gather_kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
            if (e != hipSuccess) return e;
            raised = 150 * 1024;
        }
        const dim3 grid((unsigned)((g.C + 4 * cpw - 1) / (4 * cpw)), (unsigned)g.N);
        hipLaunchKernelGGL(conv_dx_gather_kernel, grid, dim3(256), lds, s, f, a.W, a.dX, g, step);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (a.dW) {
        g.cpw = cpw_max;
        const dim3 grid((unsigned)((g.C + 4 * g.cpw - 1) / (4 * g.cpw)), (unsigned)g.K);
        if (a.x_dtype == DBP_F32)
            hipLaunchKernelGGL((conv_dw_gather_kernel<float, double, float>), grid, dim3(256), 0, s, f, (const float *)a.X, (float *)a.dW, g, step);
        else
            hipLaunchKernelGGL((conv_dw_gather_kernel<int8_t, int32_t, int32_t>), grid, dim3(256), 0, s, f, (const int8_t *)a.X, (int32_t *)a.dW, g, step);
        return hipGetLastError();
    }
    return hipSuccess;
}

hipError_t launch_linear_gather(const LinearArgs &a, const FormatView &f, hipStream_t s)
{
    const int B = (int)a.B, in = (int)a.in, out = (int)a.out;
    const dim3 block(256);
    const unsigned slabs = (unsigned)((in + kSlab - 1) / kSlab);
    if (a.dX) {
        const bool vec = in % 4 == 0 && ((uintptr_t)a.W % 16) == 0;
        if (vec) hipLaunchKernelGGL(linear_dx_gather_kernel<true>, dim3(slabs, B), block, 0, s, f, a.W, a.dX, in, out, Scale{a.step, a.step_dev});
        else     hipLaunchKernelGGL(linear_dx_gather_kernel<false>, dim3(slabs, B), block, 0, s, f, a.W, a.dX, in, out, Scale{a.step, a.step_dev});
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (a.dW) {
        if (a.x_dtype == DBP_F32) {
            const bool vec = in % 4 == 0 && ((uintptr_t)a.X % 16) == 0;
            if (vec) hipLaunchKernelGGL((linear_dw_gather_kernel<float, float, true>), dim3(slabs, out), block, 0, s,
                                        a.codes, (const float *)a.X, (float *)a.dW, B, in, out, Scale{a.step, a.step_dev});
            else     hipLaunchKernelGGL((linear_dw_gather_kernel<float, float, false>), dim3(slabs, out), block, 0, s,
                                        a.codes, (const float *)a.X, (float *)a.dW, B, in, out, Scale{a.step, a.step_dev});
        } else {
            const bool vec = in % 4 == 0 && ((uintptr_t)a.X % 4) == 0;
            if (vec) hipLaunchKernelGGL((linear_dw_gather_kernel<int8_t, int32_t, true>), dim3(slabs, out), block, 0, s,
                                        a.codes, (const int8_t *)a.X, (int32_t *)a.dW, B, in, out, Scale{a.step, a.step_dev});
            else     hipLaunchKernelGGL((linear_dw_gather_kernel<int8_t, int32_t, false>), dim3(slabs, out), block, 0, s,
                                        a.codes, (const int8_t *)a.X, (int32_t *)a.dW, B, in, out, Scale{a.step, a.step_dev});
        }
        return hipGetLastError();
    }
    return hipSuccess;
}

}  // namespace dbp
