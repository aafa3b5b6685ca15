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
// wavefront, four wavefronts per workgroup.  A tile's entries are decoded once per workgroup (pixel -> (p, q)) into LDS.
struct ConvGatherGeom { int N, C, H, Wd, K, R, S, pad, st, P, Q, cpw; };   // cpw: channels per wavefront

__device__ __forceinline__ void conv_gather_decode(const FormatView &f, int64_t t, int seg, int cnt, int Q, uint32_t *s_ent)
{
    __syncthreads();                                     // the tile before has been consumed
    if ((int)threadIdx.x < cnt) {
        const uint32_t en = f.entries[t * DBP_TILE + threadIdx.x];
        const int pix = seg * DBP_TILE + (int)(en >> 8), p = pix / Q, q = pix - p * Q;
        s_ent[threadIdx.x] = (uint32_t)p | ((uint32_t)q << 12) | ((en & 0xFFu) << 24);
    }
    __syncthreads();
}

// dW[k,c,r,s] = step * sum_n sum_{nonzero (p,q) of plane (n,k)} code * X[n,c,p*st+r-pad,q*st+s-pad]
// Workgroup (channel tile, k); a lane owns one element of dW.  fp32 X accumulates in fp64 (the products are exact
// there), int8 X in int32 (exact).
template <class XT, class AccT, class OutT>
__global__ __launch_bounds__(256) void conv_dw_gather_kernel(FormatView f, const XT *X, OutT *dW, ConvGatherGeom g, Scale step_arg)
{
    __shared__ uint32_t s_ent[DBP_TILE];
    const int k = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int RS = g.R * g.S, cl = lane / RS, tap = lane - cl * RS;
    const int c = ((int)blockIdx.x * 4 + wave) * g.cpw + cl;
    const bool own = cl < g.cpw && c < g.C;
    const int r = tap / g.S, s = tap - r * g.S, tpr = (int)f.tiles_per_row, HW = g.H * g.Wd;
    AccT acc = 0;
    for (int n = 0; n < g.N; ++n) {
        const XT *xc = X + ((int64_t)n * g.C + (own ? c : 0)) * HW;
        for (int seg = 0; seg < tpr; ++seg) {
            const int64_t t = ((int64_t)n * g.K + k) * tpr + seg;
            const int cnt = f.tile_nnz[t];                // the same for the whole workgroup
            if (cnt == 0) continue;
            conv_gather_decode(f, t, seg, cnt, g.Q, s_ent);
#pragma unroll 4
            for (int e = 0; e < cnt; ++e) {
                const uint32_t v = s_ent[e];
                const int h = (int)(v & 0xFFFu) * g.st + r - g.pad, w = (int)((v >> 12) & 0xFFFu) * g.st + s - g.pad;
                if (own && h >= 0 && h < g.H && w >= 0 && w < g.Wd) acc += (AccT)(int8_t)(v >> 24) * (AccT)xc[h * g.Wd + w];
            }
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
    extern __shared__ float cg_planes[];                 // [4 * cpw channels][H*Wd], then the decoded entries
    const int n = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int RS = g.R * g.S, cl = lane / RS, tap = lane - cl * RS;
    const int c_first = (int)blockIdx.x * 4 * g.cpw, c = c_first + wave * g.cpw + cl;
    const bool own = cl < g.cpw && c < g.C;
    const int r = tap / g.S, s = tap - r * g.S, tpr = (int)f.tiles_per_row, HW = g.H * g.Wd;
    const int n_planes = 4 * g.cpw;
    uint32_t *s_ent = (uint32_t *)(cg_planes + (size_t)n_planes * HW);
    for (int i = threadIdx.x; i < n_planes * HW; i += 256) cg_planes[i] = 0.f;
    float *mine = cg_planes + (size_t)(wave * g.cpw + (own ? cl : 0)) * HW;
    for (int k = 0; k < g.K; ++k) {
        const float wv = own ? W[(((int64_t)k * g.C + c) * g.R + r) * g.S + s] : 0.f;
        for (int seg = 0; seg < tpr; ++seg) {
            const int64_t t = ((int64_t)n * g.K + k) * tpr + seg;
            const int cnt = f.tile_nnz[t];
            if (cnt == 0) continue;
            conv_gather_decode(f, t, seg, cnt, g.Q, s_ent);   // (its first barrier also orders the clearing above)
            for (int e = 0; e < cnt; ++e) {
                const uint32_t v = s_ent[e];
                const int h = (int)(v & 0xFFFu) * g.st + r - g.pad, w = (int)((v >> 12) & 0xFFFu) * g.st + s - g.pad;
                if (own && h >= 0 && h < g.H && w >= 0 && w < g.Wd) mine[h * g.Wd + w] += (float)(int8_t)(v >> 24) * wv;
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

bool conv_gather_supported(int64_t H, int64_t Wd, int64_t R, int64_t S, int64_t P, int64_t Q, bool want_dx)
{
    if (R * S > 64 || P >= 4096 || Q >= 4096) return false;
    if (want_dx && (size_t)(4 * H * Wd * 4 + DBP_TILE * 4) > (size_t)150 * 1024) return false;   // a plane per wavefront at least
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
        const size_t HW4 = (size_t)g.H * g.Wd * 4, budget = (size_t)150 * 1024 - DBP_TILE * 4;
        int cpw = cpw_max;
        while (cpw > 1 && (size_t)4 * cpw * HW4 > budget) --cpw;
        g.cpw = cpw;
        const size_t lds = (size_t)4 * cpw * HW4 + DBP_TILE * 4;
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
