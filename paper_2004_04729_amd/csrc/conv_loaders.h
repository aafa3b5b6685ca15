// Implicit-im2col loaders: the convolutional analogues of Eqs. (qda)/(qdw) as GEMMs whose operands
// are never materialised.  Any stride, zero padding, NCHW / KCRS storage.
//
//   dX:  rows m = (n,h,w) output pixels, cols c, reduction kk = (r,s,k) with k fastest (k padded to Kp)
//          A(m,kk) = code[n,k,(h+pad-r)/st,(w+pad-s)/st] where both divisions are exact, else 0
//                                                   B(c,kk) = Wt[kk][c]  (weights re-laid by prep kernel)
//   dW:  rows k output channels, cols j = (c,r,s), reduction kk = (n,pq) with pq fastest (pq padded to PQp)
//          A(k,kk) = code[n,k,pq]                   B(j,kk) = X[n,c,p*st+r-pad,q*st+s-pad]
#pragma once
#include "gemm_core.h"

namespace dbp {

struct ConvGeom {
    int N, C, H, Wd, K, R, S, pad, P, Q;
    int st;      // stride
    int Kp;      // K rounded up to the chunk length (dX reduction padding)
    int PQp;     // P*Q rounded up to the K step (dW reduction padding)
    int Ct, Kt;  // channels of the tensors that hold X/dX and the gradient (C, K unless this is one group's block)
};

template <int MODE> struct GradElem;      // element type of the gradient operand per mode
template <> struct GradElem<MODE_BF16> { using T = int8_t; using Raw = RawCodes8; static constexpr bool SPARSE = true; };
template <> struct GradElem<MODE_I8>   { using T = int8_t; using Raw = RawI8x16;  static constexpr bool SPARSE = true; };
template <> struct GradElem<MODE_F32>  { using T = float;  using Raw = RawF32x4;  static constexpr bool SPARSE = false; };

template <int KCH, class Raw, class T> struct RunLoad;
template <> struct RunLoad<8, RawCodes8, int8_t> {
    static __device__ __forceinline__ RawCodes8 strided(const int8_t *p, int64_t st, int nv) { return load_i8_strided8(p, st, nv); }
    static __device__ __forceinline__ RawCodes8 run(const int8_t *p, int nv) { return load_i8_run8(p, nv); }
};
template <> struct RunLoad<16, RawI8x16, int8_t> {
    static __device__ __forceinline__ RawI8x16 strided(const int8_t *p, int64_t st, int nv) { return load_i8_strided16(p, st, nv); }
    static __device__ __forceinline__ RawI8x16 run(const int8_t *p, int nv) { return load_i8_run16(p, nv); }
};
template <> struct RunLoad<4, RawF32x4, float> {
    static __device__ __forceinline__ RawF32x4 strided(const float *p, int64_t st, int nv) { return load_f32_strided4(p, st, nv); }
    static __device__ __forceinline__ RawF32x4 run(const float *p, int nv) { return load_f32_run4(p, nv); }
};

// ---- dX, gradient side: rows are output pixels -------------------------------------------------
template <int MODE> struct ConvDxGradLoader {
    using T = typename GradElem<MODE>::T;
    using Raw = typename GradElem<MODE>::Raw;
    static constexpr int PLANES = 1;
    static constexpr bool SPARSE = GradElem<MODE>::SPARSE;
    static constexpr int KCH = ModeTraits<MODE>::KCH;
    const T *base; ConvGeom g;
    struct Row { int64_t img; int h, w; bool ok; };
    __device__ Row row(int m) const
    {
        const int hw = g.H * g.Wd;
        const int n = m / hw, rem = m - n * hw;
        const int h = rem / g.Wd;
        return Row{(int64_t)n * g.Kt * g.P * g.Q, h, rem - h * g.Wd, m < g.N * hw};
    }
    __device__ Raw fetch(const Row &rw, int kk0) const
    {
        const int rs = kk0 / g.Kp, k0 = kk0 - rs * g.Kp;
        const int r = rs / g.S, s = rs - r * g.S;
        int p = rw.h + g.pad - r, q = rw.w + g.pad - s;
        const int nv = g.K - k0;
        if (!rw.ok || rs >= g.R * g.S || nv <= 0 || p < 0 || q < 0) return raw_zero<Raw>();
        if (g.st != 1) {
            // an input pixel receives from output pixel p only if p*st + r - pad == h exactly
            const int pd = p / g.st, qd = q / g.st;
            if (pd * g.st != p || qd * g.st != q) return raw_zero<Raw>();
            p = pd; q = qd;
        }
        if (p >= g.P || q >= g.Q) return raw_zero<Raw>();
        const int64_t pq = (int64_t)g.P * g.Q;
        return RunLoad<KCH, Raw, T>::strided(base + rw.img + (int64_t)k0 * pq + (int64_t)p * g.Q + q, pq, nv);
    }
};

// ---- dW, gradient side: rows are output channels ------------------------------------------------
template <int MODE> struct ConvDwGradLoader {
    using T = typename GradElem<MODE>::T;
    using Raw = typename GradElem<MODE>::Raw;
    static constexpr int PLANES = 1;
    static constexpr bool SPARSE = GradElem<MODE>::SPARSE;
    static constexpr int KCH = ModeTraits<MODE>::KCH;
    const T *base; ConvGeom g;
    struct Row { int k; bool ok; };
    __device__ Row row(int k) const { return Row{k, k < g.K}; }
    __device__ Raw fetch(const Row &rw, int kk0) const
    {
        const int n = kk0 / g.PQp, pq0 = kk0 - n * g.PQp;
        const int pq = g.P * g.Q, nv = pq - pq0;
        if (!rw.ok || n >= g.N || nv <= 0) return raw_zero<Raw>();
        return RunLoad<KCH, Raw, T>::run(base + ((int64_t)n * g.Kt + rw.k) * pq + pq0, nv);
    }
};

// ---- dW, activation side: rows are (c,r,s), reduction walks the output pixels of image n ---------
template <int MODE> struct ConvDwActLoader;

template <class T> __device__ __forceinline__ void conv_act_walk(const T *X, const ConvGeom &g, int c, int r, int s,
                                                                  int kk0, int kch, T *vals)
{
    const int n = kk0 / g.PQp, pq0 = kk0 - n * g.PQp;
    int p = pq0 / g.Q, q = pq0 - p * g.Q;
    const T *img = X + ((int64_t)n * g.Ct + c) * g.H * g.Wd;
    const bool n_ok = n < g.N;
    for (int j = 0; j < kch; ++j) {
        const int h = p * g.st + r - g.pad, w = q * g.st + s - g.pad;
        T v = 0;
        if (n_ok && p < g.P && h >= 0 && h < g.H && w >= 0 && w < g.Wd) v = img[(int64_t)h * g.Wd + w];
        vals[j] = v;
        if (++q == g.Q) { q = 0; ++p; }
    }
}

struct ConvActRow { int c, r, s; bool ok; };
__device__ __forceinline__ ConvActRow conv_act_row(const ConvGeom &g, int j)
{
    const int rs = g.R * g.S;
    const int c = j / rs, rem = j - c * rs;
    const int r = rem / g.S;
    return ConvActRow{c, r, rem - r * g.S, j < g.C * rs};
}

template <> struct ConvDwActLoader<MODE_BF16> {
    using Raw = RawF32x8;
    static constexpr int PLANES = 3;
    static constexpr bool SPARSE = false;
    const float *base; ConvGeom g;
    using Row = ConvActRow;
    __device__ Row row(int j) const { return conv_act_row(g, j); }
    __device__ Raw fetch(const Row &rw, int kk0) const
    {
        Raw out = raw_zero<Raw>();
        if (rw.ok) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = 0.f;
            conv_act_walk<float>(base, g, rw.c, rw.r, rw.s, kk0, 8, v);
#pragma unroll
            for (int j = 0; j < 8; ++j) out.v[j] = v[j];
        }
        return out;
    }
};
template <> struct ConvDwActLoader<MODE_F32> {
    using Raw = RawF32x4;
    static constexpr int PLANES = 1;
    static constexpr bool SPARSE = false;
    const float *base; ConvGeom g;
    using Row = ConvActRow;
    __device__ Row row(int j) const { return conv_act_row(g, j); }
    __device__ Raw fetch(const Row &rw, int kk0) const
    {
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (rw.ok) conv_act_walk<float>(base, g, rw.c, rw.r, rw.s, kk0, 4, v);
        Raw out; out.v = f32x4{v[0], v[1], v[2], v[3]};
        return out;
    }
};
template <> struct ConvDwActLoader<MODE_I8> {
    using Raw = RawI8x16;
    static constexpr int PLANES = 1;
    static constexpr bool SPARSE = false;
    const int8_t *base; ConvGeom g;
    using Row = ConvActRow;
    __device__ Row row(int j) const { return conv_act_row(g, j); }
    __device__ Raw fetch(const Row &rw, int kk0) const
    {
        int8_t v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = 0;
        if (rw.ok) conv_act_walk<int8_t>(base, g, rw.c, rw.r, rw.s, kk0, 16, v);
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 16; ++j) w[j >> 2] |= (uint32_t)(uint8_t)v[j] << (8 * (j & 3));
        Raw out; out.w = u32x4{w[0], w[1], w[2], w[3]};
        return out;
    }
};

// dX output: row m = (n,hw), col c  ->  dX[n][c][hw]
struct ConvDxOut {
    int Ct, HW;                 // channels of the tensor that holds dX
    __device__ int64_t operator()(int row, int col) const
    {
        const int n = row / HW, hw = row - n * HW;
        return ((int64_t)n * Ct + col) * HW + hw;
    }
};

}  // namespace dbp
