// Host-side launchers of the matrix-core products: fully connected and implicit-im2col convolution,
// dithered (bf16x3 / int8) and dense (fp32) variants, with deterministic split-K.
#include "conv_loaders.h"
#include "fc_kernel.h"

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
hipError_t run_gemm(const AL &al, const BL &bl, const OM &om, int M, int N, int K, int granule, float scale,
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
__global__ __launch_bounds__(256) void conv_weight_relayout_kernel(const float *W, float *Wt, ConvGeom g)
{
    const int64_t total = (int64_t)g.R * g.S * g.Kp * g.C;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int c = (int)(i % g.C);
        const int64_t kk = i / g.C;
        const int k = (int)(kk % g.Kp), rs = (int)(kk / g.Kp);
        Wt[i] = k < g.K ? W[((int64_t)k * g.C + c) * g.R * g.S + rs] : 0.0f;
    }
}

ConvGeom make_geom(const ConvArgs &a, int kch, int kstep)
{
    ConvGeom g;
    g.N = (int)a.N; g.C = (int)a.C; g.H = (int)a.H; g.Wd = (int)a.Wd; g.K = (int)a.K; g.R = (int)a.R; g.S = (int)a.S;
    g.pad = (int)a.pad;
    g.P = g.H + 2 * g.pad - g.R + 1;
    g.Q = g.Wd + 2 * g.pad - g.S + 1;
    g.Kp = (g.K + kch - 1) / kch * kch;
    g.PQp = (g.P * g.Q + kstep - 1) / kstep * kstep;
    return g;
}

size_t relayout_bytes(int64_t K, int64_t C, int64_t R, int64_t S)
{
    int64_t Kp = (K + 7) / 8 * 8;                       // multiple of every chunk length in use (4, 8)
    return align_up((size_t)(R * S * Kp * C) * sizeof(float), 256);
}

// Fast fully connected kernel (fc_kernel.h) when the layout allows 16-byte column loads; returns false
// when the shape needs the generic kernel instead.
template <bool A_KFAST>
bool run_fc_fast(const int8_t *A, int64_t lda, const float *B, int64_t ldb, int M, int N, int K, float scale,
                 float *out, void *scratch, size_t scratch_bytes, hipStream_t s, hipError_t *err)
{
    if (N < 4 || N % 4 || ldb % 4 || ((uintptr_t)B % 16) || ((uintptr_t)out % 16)) return false;
    int avec = 0;
    if (A_KFAST) {
        avec = (lda % 16 == 0 && (uintptr_t)A % 16 == 0) ? 16 : (lda % 8 == 0 && (uintptr_t)A % 8 == 0) ? 8 :
               (lda % 4 == 0 && (uintptr_t)A % 4 == 0) ? 4 : 0;
        if (!avec) return false;
    } else {
        if (M < 4 || M % 4 || lda % 4 || ((uintptr_t)A % 4)) return false;
    }
    FcArgs p;
    p.A = A; p.lda = lda; p.B = B; p.ldb = ldb; p.out = out; p.ldc = N; p.partial = (float *)scratch;
    p.M = M; p.N = N; p.K = K; p.scale = scale;
    p.tiles_m = (M + TM - 1) / TM;
    const int tiles_n = (N + TN - 1) / TN;
    const int64_t tiles = (int64_t)p.tiles_m * tiles_n;
    Split sp = choose_split(tiles, K, 32);
    while (sp.n > 1 && (size_t)sp.n * M * N * sizeof(float) > scratch_bytes) {
        int64_t units = (K + 31) / 32, n = sp.n - 1;
        sp.k_per = (int)((units + n - 1) / n * 32);
        sp.n = (int)((K + sp.k_per - 1) / sp.k_per);
    }
    p.k_per_split = sp.n == 1 ? (K + 31) / 32 * 32 : sp.k_per;
    const dim3 grid((unsigned)tiles, 1, (unsigned)sp.n), block(256);
    if (!A_KFAST)         hipLaunchKernelGGL((fc_bf16_kernel<false, 4>), grid, block, 0, s, p);
    else if (avec == 16)  hipLaunchKernelGGL((fc_bf16_kernel<true, 16>), grid, block, 0, s, p);
    else if (avec == 8)   hipLaunchKernelGGL((fc_bf16_kernel<true, 8>), grid, block, 0, s, p);
    else                  hipLaunchKernelGGL((fc_bf16_kernel<true, 4>), grid, block, 0, s, p);
    *err = hipGetLastError();
    if (*err == hipSuccess && sp.n > 1) {
        const int64_t total4 = (int64_t)M * (N / 4);
        const int blocks = (int)((total4 + 255) / 256 < 2048 ? (total4 + 255) / 256 : 2048);
        hipLaunchKernelGGL(reduce4_kernel, dim3(blocks), dim3(256), 0, s, (const f32x4 *)scratch, out, (int64_t)N, M, N / 4, sp.n, scale);
        *err = hipGetLastError();
    }
    return true;
}

}  // namespace

size_t linear_scratch_bytes(int64_t B, int64_t in, int64_t out)
{
    // split-K partials of the larger of the two products, at the split the launcher would choose
    auto part = [](int64_t M, int64_t N, int64_t K) {
        int64_t tiles = ((M + TM - 1) / TM) * ((N + TN - 1) / TN);
        Split sp = choose_split(tiles, K, 16);          // smallest K step (fp32 mode) gives the largest split
        return sp.n > 1 ? (size_t)sp.n * M * N * 4 : (size_t)0;
    };
    size_t a = part(B, in, out), b = part(out, in, B);
    return align_up(a > b ? a : b, 256) + 256;
}

size_t conv_scratch_bytes(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t pad)
{
    const int64_t P = H + 2 * pad - R + 1, Q = Wd + 2 * pad - S + 1;
    auto part = [](int64_t M, int64_t Nn, int64_t Kr, int64_t gran) {
        int64_t tiles = ((M + TM - 1) / TM) * ((Nn + TN - 1) / TN);
        Split sp = choose_split(tiles, Kr, (int)gran);
        return sp.n > 1 ? (size_t)sp.n * M * Nn * 4 : (size_t)0;
    };
    size_t dx = part(N * H * Wd, C, R * S * ((K + 7) / 8 * 8), 16);
    const int64_t PQp16 = (P * Q + 15) / 16 * 16;
    size_t dw = part(K, C * R * S, N * PQp16, 16);
    return relayout_bytes(K, C, R, S) + align_up(dx > dw ? dx : dw, 256) + 256;
}

// ------------------------------------------------------------------------------------------------
// Fully connected layer.  dX = q.W : rows b, cols i, reduction o.   dW = q^T.X : rows o, cols i, reduction b.
// ------------------------------------------------------------------------------------------------
hipError_t launch_linear_mfma(const LinearArgs &a, hipStream_t s)
{
    const int B = (int)a.B, in = (int)a.in, out = (int)a.out;
    hipError_t e = hipSuccess;
    RowMajorOut om{a.in};
    if (a.codes) {
        if (a.dX && run_fc_fast<true>(a.codes, a.out, a.W, a.in, B, in, out, a.step, a.dX, a.scratch, a.scratch_bytes, s, &e)) {
            if (e != hipSuccess) return e;
        } else if (a.dX) {
            MatrixLoader<MODE_BF16, true, true>   al{a.codes, a.out, B, out};
            MatrixLoader<MODE_BF16, false, false> bl{a.W, a.in, in, out};
            e = run_gemm<MODE_BF16>(al, bl, om, B, in, out, k_step<MODE_BF16>(), a.step, a.dX, a.scratch, a.scratch_bytes, s);
            if (e != hipSuccess) return e;
        }
        if (a.dW && a.x_dtype == DBP_F32 &&
            run_fc_fast<false>(a.codes, a.out, (const float *)a.X, a.in, out, in, B, a.step, (float *)a.dW, a.scratch, a.scratch_bytes, s, &e)) {
            return e;
        }
        if (a.dW && a.x_dtype == DBP_F32) {
            MatrixLoader<MODE_BF16, true, false>  al{a.codes, a.out, out, B};
            MatrixLoader<MODE_BF16, false, false> bl{(const float *)a.X, a.in, in, B};
            e = run_gemm<MODE_BF16>(al, bl, om, out, in, B, k_step<MODE_BF16>(), a.step, (float *)a.dW, a.scratch, a.scratch_bytes, s);
        } else if (a.dW) {
            MatrixLoader<MODE_I8, true, false>  al{a.codes, a.out, out, B};
            MatrixLoader<MODE_I8, false, false> bl{(const int8_t *)a.X, a.in, in, B};
            e = run_gemm<MODE_I8>(al, bl, om, out, in, B, k_step<MODE_I8>(), 1.0f, (int32_t *)a.dW, a.scratch, a.scratch_bytes, s);
        }
        return e;
    }
    // dense baseline
    if (a.dX) {
        MatrixLoader<MODE_F32, false, true>  al{(const float *)a.dense, a.out, B, out};
        MatrixLoader<MODE_F32, false, false> bl{a.W, a.in, in, out};
        e = run_gemm<MODE_F32>(al, bl, om, B, in, out, k_step<MODE_F32>(), 1.0f, a.dX, a.scratch, a.scratch_bytes, s);
        if (e != hipSuccess) return e;
    }
    if (a.dW && a.x_dtype == DBP_F32) {
        MatrixLoader<MODE_F32, false, false> al{(const float *)a.dense, a.out, out, B};
        MatrixLoader<MODE_F32, false, false> bl{(const float *)a.X, a.in, in, B};
        e = run_gemm<MODE_F32>(al, bl, om, out, in, B, k_step<MODE_F32>(), 1.0f, (float *)a.dW, a.scratch, a.scratch_bytes, s);
    } else if (a.dW) {
        MatrixLoader<MODE_I8, false, false> al{(const int8_t *)a.dense, a.out, out, B};
        MatrixLoader<MODE_I8, false, false> bl{(const int8_t *)a.X, a.in, in, B};
        e = run_gemm<MODE_I8>(al, bl, om, out, in, B, k_step<MODE_I8>(), 1.0f, (int32_t *)a.dW, a.scratch, a.scratch_bytes, s);
    }
    return e;
}

// ------------------------------------------------------------------------------------------------
// Convolution (stride 1).
// ------------------------------------------------------------------------------------------------
template <int MODE_G>
static hipError_t conv_dx(const ConvArgs &a, const void *grad, float scale, hipStream_t s)
{
    // MODE_G: MODE_BF16 (codes) or MODE_F32 (dense).  Weights are fp32 in every mode.
    ConvGeom g = make_geom(a, ModeTraits<MODE_G>::KCH, k_step<MODE_G>());
    float *Wt = (float *)a.scratch;
    const size_t rb = relayout_bytes(a.K, a.C, a.R, a.S);
    const int64_t total = (int64_t)g.R * g.S * g.Kp * g.C;
    int blocks = (int)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(conv_weight_relayout_kernel, dim3(blocks), dim3(256), 0, s, a.W, Wt, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int M = g.N * g.H * g.Wd, Kred = g.R * g.S * g.Kp;
    ConvDxGradLoader<MODE_G> al{(const typename GradElem<MODE_G>::T *)grad, g};
    MatrixLoader<MODE_G, false, false> bl{Wt, g.C, g.C, Kred};
    ConvDxOut om{g.C, g.H * g.Wd};
    return run_gemm<MODE_G>(al, bl, om, M, g.C, Kred, k_step<MODE_G>(), scale, a.dX,
                            (char *)a.scratch + rb, a.scratch_bytes - rb, s);
}

template <int MODE>
static hipError_t conv_dw(const ConvArgs &a, const void *grad, float scale, hipStream_t s)
{
    using Acc = typename ModeTraits<MODE>::Acc;
    ConvGeom g = make_geom(a, ModeTraits<MODE>::KCH, k_step<MODE>());
    const size_t rb = relayout_bytes(a.K, a.C, a.R, a.S);
    const int CRS = g.C * g.R * g.S, Kred = g.N * g.PQp;
    ConvDwGradLoader<MODE> al{(const typename GradElem<MODE>::T *)grad, g};
    ConvDwActLoader<MODE>  bl{(const decltype(ConvDwActLoader<MODE>::base))a.X, g};
    RowMajorOut om{CRS};
    return run_gemm<MODE>(al, bl, om, g.K, CRS, Kred, k_step<MODE>(), scale, (Acc *)a.dW,
                          (char *)a.scratch + rb, a.scratch_bytes - rb, s);
}

hipError_t launch_conv_mfma(const ConvArgs &a, hipStream_t s)
{
    hipError_t e = hipSuccess;
    if (a.codes) {
        if (a.dX) { e = conv_dx<MODE_BF16>(a, a.codes, a.step, s); if (e != hipSuccess) return e; }
        if (a.dW) e = a.x_dtype == DBP_F32 ? conv_dw<MODE_BF16>(a, a.codes, a.step, s) : conv_dw<MODE_I8>(a, a.codes, 1.0f, s);
        return e;
    }
    if (a.dX) { e = conv_dx<MODE_F32>(a, a.dense, 1.0f, s); if (e != hipSuccess) return e; }
    if (a.dW) e = a.x_dtype == DBP_F32 ? conv_dw<MODE_F32>(a, a.dense, 1.0f, s) : conv_dw<MODE_I8>(a, a.dense, 1.0f, s);
    return e;
}

}  // namespace dbp
