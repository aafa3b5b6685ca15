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

}  // namespace

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
