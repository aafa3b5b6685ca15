/*
 * dbp_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, obviously-correct CPU oracle for the dithered-backprop hot path
 * (Wiedemann et al., "Dithered backprop", arXiv 2004.04729).  It exists so that the
 * HIP kernels can be checked element by element.  Only the tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it; it shares no code, header, table or
 * helper with the GPU library and neither includes the other.
 *
 * What it computes, and where the paper defines it:
 *   - NSD quantiser  q = Delta * floor((x + nu)/Delta + 1/2),  nu ~ U(-Delta/2, Delta/2)
 *     on the open interval                                  (Sec. "Non-subtractive dithered
 *     quantization", Eq. (nsd); applied to delta_z in Eq. (qdz)).
 *   - the two backward products that consume q              (Eqs. (qda), (qdw)):
 *         delta_a = W^T . q          delta_W = q . a^T
 *     for fully connected layers, and their convolutional analogues ("analogous for
 *     convolutional layers", Sec. "Dithered backpropagation").
 *   - 8-bit mode: integer codes times int8 activations, exact int32 weight gradient
 *     (Sec. "Quantizing forward pass": everything but the weight update in 8 bit).
 *   - around the quantiser: the layer's step size Delta = s*std(delta_z) (Algorithm 1),
 *     delta_z = delta_a (.) f'(z) in front of it and the bias gradient behind it.
 *
 * The paper fixes no random generator, no code width, no storage layout and no sparse
 * format.  Those readings are stated where they are used below; they are spec decisions
 * of this repository ("parity unpinned" against the paper: the hash constants, the
 * 16-bit dither resolution, the multiply-by-reciprocal, the +-127 saturation and the
 * tile layout are pinned only by frozen test vectors and by the statistical laws the
 * paper does state).
 *
 * Precision: the quantiser's decision is taken in fp32 exactly as specified (one fused
 * multiply-add, one floor) because it decides an integer; every product is accumulated
 * in fp64 in natural index order; integer mode accumulates in int64 and checks int32.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -fPIC -shared.  The OpenMP pragmas
 * only distribute independent output rows over threads; no sum is reordered.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------
 * Dither generator (spec decision; the paper only hints at a cheap congruential-style
 * generator in Sec. "Computational complexity", item 2).
 *
 * Counter based: the dither of element g of a tensor depends only on (seed, g), so any
 * traversal order, any sharding and any hardware give the same draw.
 *
 *   mix(x):   x ^= x>>16; x *= A; x ^= x>>15; x *= C; x ^= x>>16
 *   k0 = mix(lo32(seed) ^ G);  k1 = mix(hi32(seed) + k0 + A)
 *   H(seed,c): h = (lo32(c) ^ k0) * G;  h ^= h>>16;
 *              h = (h + k1 + hi32(c)*C) * A;  h ^= h>>15;  h *= C;  h ^= h>>16
 *   G = floor(2^32/phi), A = frac(sqrt 2)*2^32, C = frac(sqrt 3)*2^32  (all odd)
 *
 * One hash word serves two neighbouring elements: element g uses word H(seed, g>>1),
 * the low 16 bits when g is even and the high 16 bits when g is odd.  With m those 16
 * bits, u = (2m+1) * 2^-17 lies in [2^-17, 1-2^-17], is symmetric about 1/2 and never
 * touches 0 or 1: u - 1/2 is nu/Delta on the OPEN interval (-1/2, 1/2) of Eq. (nsd).
 * ---------------------------------------------------------------------------------- */
#define DBP_G 0x9E3779B9u
#define DBP_A 0x6A09E667u
#define DBP_C 0xBB67AE85u

static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= DBP_A; x ^= x >> 15; x *= DBP_C; x ^= x >> 16;
    return x;
}

uint32_t dbp_oracle_hash(uint64_t seed, uint64_t counter)
{
    uint32_t k0 = mix32((uint32_t)seed ^ DBP_G);
    uint32_t k1 = mix32((uint32_t)(seed >> 32) + k0 + DBP_A);
    uint32_t h = ((uint32_t)counter ^ k0) * DBP_G;
    h ^= h >> 16;
    h = (h + k1 + (uint32_t)(counter >> 32) * DBP_C) * DBP_A;
    h ^= h >> 15;
    h *= DBP_C;
    h ^= h >> 16;
    return h;
}

void dbp_oracle_keys(uint64_t seed, uint32_t *k0, uint32_t *k1)
{
    *k0 = mix32((uint32_t)seed ^ DBP_G);
    *k1 = mix32((uint32_t)(seed >> 32) + *k0 + DBP_A);
}

/* u = nu/Delta + 1/2 for global element index g. */
float dbp_oracle_dither_u(uint64_t seed, uint64_t g)
{
    uint32_t h = dbp_oracle_hash(seed, g >> 1);
    uint32_t m = (g & 1u) ? (h >> 16) : (h & 0xFFFFu);
    return (float)(2u * m + 1u) * 0x1p-17f;      /* exact: a 17-bit odd integer scaled */
}

/* ------------------------------------------------------------------------------------
 * NSD quantiser, Eq. (nsd) / Eq. (qdz).
 *
 *   floor((x + nu)/Delta + 1/2) = floor(x/Delta + u),   u = nu/Delta + 1/2.
 *
 * Readings (the paper is silent): x/Delta is x * inv with inv = 1.0f/Delta rounded once;
 * t = fma(x, inv, u) is ONE fp32 operation (single rounding), k = floor(t); k saturates
 * to [-127, 127] (the paper reports <= 8 bit codes in all experiments, Sec. "Accuracy &
 * Induced Sparsity"); a NaN t gives code 0.  q = k * Delta is never materialised.
 * Algorithm 1 prints Q(delta_z) without the dither; Eq. (qdz) has it, and is followed.
 * ---------------------------------------------------------------------------------- */
typedef struct {
    uint64_t nnz;            /* codes != 0                                   */
    uint64_t n_saturated;    /* |floor(t)| > 127 before clamping (incl. Inf) */
    uint64_t n_nonfinite;    /* inputs that are NaN or +-Inf                 */
    int32_t  max_abs_code;   /* max |k| after clamping                       */
    int32_t  pad_;
} dbp_oracle_stats;

void dbp_oracle_nsd(const float *delta, int64_t n, float step, uint64_t seed,
                    uint64_t idx_base, int8_t *codes, dbp_oracle_stats *st)
{
    const float inv = 1.0f / step;
    dbp_oracle_stats s;
    memset(&s, 0, sizeof s);
    for (int64_t j = 0; j < n; ++j) {
        float x = delta[j];
        float u = dbp_oracle_dither_u(seed, idx_base + (uint64_t)j);
        float t = fmaf(x, inv, u);
        float kf = floorf(t);
        int k;
        if (!isfinite(x)) s.n_nonfinite++;
        if (isnan(t)) {
            k = 0;
        } else if (kf > 127.0f) {
            k = 127;  s.n_saturated++;
        } else if (kf < -127.0f) {
            k = -127; s.n_saturated++;
        } else {
            k = (int)kf;
        }
        if (k != 0) s.nnz++;
        int a = k < 0 ? -k : k;
        if (a > s.max_abs_code) s.max_abs_code = a;
        codes[j] = (int8_t)k;
    }
    if (st) *st = s;
}

/* ------------------------------------------------------------------------------------
 * Top-k sparsifier (the comparison method of Sec. "Comparison to meProp", recalled in
 * Sec. "Related work": keep the k elements of largest magnitude of each gradient vector,
 * drop the rest) emitting the same int8 codes as the dithered quantiser, so that both
 * sparsifiers can feed the same product kernels.
 *
 * Readings (the paper describes the selection in one clause and no code format for it):
 *   - the tensor is cut into n_vec consecutive vectors of `len` elements (one example's
 *     gradient for a fully connected layer); the selection is per vector;
 *   - an element is kept iff fewer than k elements of its vector have a STRICTLY larger
 *     magnitude, i.e. iff |x| >= the k-th largest magnitude of the vector.  Without ties
 *     at the threshold that is exactly the k largest; with ties all of the tied elements
 *     are kept (a unique result that does not depend on any traversal order);
 *     k <= 0 keeps nothing, k >= len keeps everything.  The magnitude of a NaN counts as 0;
 *   - kept elements are quantised with the paper's uniform quantiser of Eq. (nsd) WITHOUT
 *     the dither (nu = 0, so u = 1/2): code = floor(fma(x, 1/Delta, 0.5f)) in fp32,
 *     saturating to [-127, 127], NaN -> 0: deterministic rounding to the nearest level
 *     (this is the "deterministic quantisation function" the paper contrasts with NSD);
 *     dropped elements get code 0.  The statistics are those of the quantiser applied to
 *     the tensor with the dropped elements replaced by +0.
 * ---------------------------------------------------------------------------------- */
static float magnitude_of(float x) { return isnan(x) ? 0.0f : fabsf(x); }

static int descending_float(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x < y) - (x > y);
}

/* thr[v] = k-th largest magnitude of vector v (k clipped to len); +Inf's successor does not
 * exist in fp32, so "keep nothing" (k <= 0) is reported as NaN, which no magnitude reaches. */
void dbp_oracle_topk_threshold(const float *delta, int64_t n_vec, int64_t len, int64_t k, float *thr)
{
    float *mag = (float *)malloc((size_t)(len > 0 ? len : 1) * sizeof(float));
    for (int64_t v = 0; v < n_vec; ++v) {
        if (k <= 0) { thr[v] = NAN; continue; }
        for (int64_t j = 0; j < len; ++j) mag[j] = magnitude_of(delta[v * len + j]);
        qsort(mag, (size_t)len, sizeof(float), descending_float);
        thr[v] = mag[(k < len ? k : len) - 1];
    }
    free(mag);
}

void dbp_oracle_topk_quantize(const float *delta, int64_t n_vec, int64_t len, int64_t k, float step,
                              int8_t *codes, dbp_oracle_stats *st)
{
    const float inv = 1.0f / step;
    float *thr = (float *)malloc((size_t)(n_vec > 0 ? n_vec : 1) * sizeof(float));
    dbp_oracle_topk_threshold(delta, n_vec, len, k, thr);
    dbp_oracle_stats s;
    memset(&s, 0, sizeof s);
    for (int64_t v = 0; v < n_vec; ++v)
        for (int64_t j = 0; j < len; ++j) {
            const float raw = delta[v * len + j];
            const float x = magnitude_of(raw) >= thr[v] ? raw : 0.0f;      /* NaN threshold: never true */
            const float t = fmaf(x, inv, 0.5f);
            const float kf = floorf(t);
            int c;
            if (!isfinite(x)) s.n_nonfinite++;
            if (isnan(t)) c = 0;
            else if (kf > 127.0f) { c = 127; s.n_saturated++; }
            else if (kf < -127.0f) { c = -127; s.n_saturated++; }
            else c = (int)kf;
            if (c != 0) s.nnz++;
            const int a = c < 0 ? -c : c;
            if (a > s.max_abs_code) s.max_abs_code = a;
            codes[v * len + j] = (int8_t)c;
        }
    free(thr);
    if (st) *st = s;
}

/* ------------------------------------------------------------------------------------
 * Step size of a layer (Algorithm 1, the two assignments before the quantiser):  sigma = std(delta_z),
 * Delta = s * sigma.
 *
 * Readings (the paper says only "std"): the population standard deviation (divide by n)
 * of all elements of the tensor,
 *      sigma = sqrt( (S2 - S1*S1/n) / n ),    S1 = sum x,   S2 = sum x*x,
 * evaluated in fp64 (x*x of an fp32 value is exact in fp64), a negative radicand (rounding)
 * counting as 0; Delta = s * sigma rounded once to fp32.  Non-finite inputs make sigma
 * non-finite: the caller's problem, as for any std.
 * Because Delta decides integer codes, the ORDER of the two sums is part of the
 * definition, so that every implementation obtains the same bits:
 *      a radix-16 summation tree -- the values are summed in groups of 16 consecutive
 *      elements, left to right inside a group; the group sums (in order) are summed the
 *      same way; and so on until one value is left.  A short last group is summed as is.
 * ---------------------------------------------------------------------------------- */
static double tree16_sum(double *v, int64_t n)
{
    if (n == 0) return 0.0;
    while (n > 1) {
        int64_t m = (n + 15) / 16;
        for (int64_t b = 0; b < m; ++b) {
            int64_t end = (b + 1) * 16 < n ? (b + 1) * 16 : n;
            double acc = v[b * 16];
            for (int64_t i = b * 16 + 1; i < end; ++i) acc += v[i];
            v[b] = acc;                    /* b <= b*16: never overwrites an unread value */
        }
        n = m;
    }
    return v[0];
}

float dbp_oracle_step_size(const float *delta, int64_t n, float s, double *sigma_out)
{
    double *v = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    for (int64_t j = 0; j < n; ++j) v[j] = (double)delta[j];
    const double s1 = tree16_sum(v, n);
    for (int64_t j = 0; j < n; ++j) v[j] = (double)delta[j] * (double)delta[j];
    const double s2 = tree16_sum(v, n);
    free(v);
    double var = n > 0 ? (s2 - s1 * s1 / (double)n) / (double)n : 0.0;
    if (var < 0.0) var = 0.0;
    const double sigma = sqrt(var);
    if (sigma_out) *sigma_out = sigma;
    return (float)((double)s * sigma);
}

/* ------------------------------------------------------------------------------------
 * The step before the quantiser and its by-product (backward pass as printed before
 * Eq. (da); bias of Eq. (z)).
 *
 *   delta_z = delta_a (.) f'(z).  For the rectifier f(z) = max(0, z) the derivative is 1
 *   for z > 0 and 0 otherwise (the value at 0 is taken as 0, the usual convention; the
 *   paper does not say).  `act` may be z or a = f(z): only "act > 0" is used, so -0.0
 *   and NaN mask the element.  The result is delta_a or +0.0f, exactly.
 *
 *   The bias enters Eq. (z) additively, so its gradient is the sum of the (quantised)
 *   preactivation gradient over everything that shares the bias: delta_b = sum q =
 *   Delta * sum k.  The integer sums are exact (int64); the float gradient is the ONE
 *   product Delta * sum evaluated in fp64 and rounded to fp32 (reading: the paper prints
 *   no formula for delta_b).
 *     mode 0: codes [rows x cols], bias per column:      sums[c] = sum_r k[r][c]   (FC)
 *     mode 1: codes [rows x cols], rows = (n, ch) with ch = r % len fastest:
 *             sums[ch] = sum over rows r with r % len == ch and all columns      (conv)
 * ---------------------------------------------------------------------------------- */
void dbp_oracle_relu_backward(const float *delta_a, const float *act, int64_t n, float *delta_z)
{
    for (int64_t j = 0; j < n; ++j) delta_z[j] = act[j] > 0.0f ? delta_a[j] : 0.0f;
}

void dbp_oracle_bias_grad(const int8_t *codes, int64_t rows, int64_t cols, int mode, int64_t len,
                          float step, int64_t *sums, float *grad)
{
    for (int64_t i = 0; i < len; ++i) sums[i] = 0;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c)
            sums[mode == 0 ? c : r % len] += codes[r * cols + c];
    if (grad)
        for (int64_t i = 0; i < len; ++i) grad[i] = (float)((double)step * (double)sums[i]);
}

/* ------------------------------------------------------------------------------------
 * Tile-sparse format (this repository's design; the paper only says "sparse tensors
 * with low precision non-zero values").  The code plane [rows x cols] is cut, row by
 * row, into tiles of 256 consecutive columns (the last tile of a row may be short);
 * tiles_per_row = ceil(cols/256), tile t = row*tiles_per_row + col/256.  Per tile:
 *   bitmap[4t + j]   bit l set  <=>  code at in-tile column 4l+j is nonzero (j = 0..3)
 *   tile_nnz[t]      number of nonzero codes in the tile
 *   entries[256t+i]  i < tile_nnz[t]: (in-tile column << 8) | (code & 0xFF), columns
 *                    ascending.  Slots at and beyond tile_nnz[t] are left untouched here
 *                    (their contents are unspecified in the format).
 * ---------------------------------------------------------------------------------- */
void dbp_oracle_tile_format(const int8_t *codes, int64_t rows, int64_t cols,
                            uint64_t *bitmap, uint16_t *tile_nnz, uint16_t *entries)
{
    int64_t tpr = (cols + 255) / 256;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t s = 0; s < tpr; ++s) {
            int64_t t = r * tpr + s;
            uint64_t w[4] = {0, 0, 0, 0};
            int cnt = 0;
            for (int c = 0; c < 256; ++c) {
                int64_t col = s * 256 + c;
                if (col >= cols) break;
                int8_t k = codes[r * cols + col];
                if (k != 0) {
                    w[c & 3] |= (uint64_t)1 << (c >> 2);
                    entries[t * 256 + cnt] = (uint16_t)((c << 8) | (uint8_t)k);
                    cnt++;
                }
            }
            for (int i = 0; i < 4; ++i) bitmap[t * 4 + i] = w[i];
            tile_nnz[t] = (uint16_t)cnt;
        }
}

/* Value of the quantised gradient element j: k*Delta from the codes, or (for the dense,
 * undithered comparison of Eqs. (da),(dw)) the raw fp32 gradient. */
static inline double qval(const int8_t *codes, const float *dense, double step, int64_t j)
{
    return codes ? (double)codes[j] * step : (double)dense[j];
}

/* ------------------------------------------------------------------------------------
 * Fully connected layer, Eqs. (qda), (qdw).  Storage is batch-row-major:
 *   Q [B x out],  W [out x in],  X [B x in]   (the paper's column-vector z = W a).
 *   dX[b,i] = sum_o Q[b,o] W[o,i]          (delta_a = W^T . q)
 *   dW[o,i] = sum_b Q[b,o] X[b,i]          (delta_W = q . a^T ; no 1/B factor)
 * Zero q terms are skipped (they add exactly 0).  Either output may be NULL.
 * Pass codes (+step) for the dithered path or dense for the plain backward pass.
 * macs (nullable) returns the number of multiply-adds performed, the p_nz*m*k*n of
 * Sec. "Computational complexity".
 * ---------------------------------------------------------------------------------- */
void dbp_oracle_linear_backward(const int8_t *codes, const float *dense, double step,
                                const float *W, const float *X,
                                int64_t B, int64_t in, int64_t out,
                                double *dX, double *dW, int threads, uint64_t *macs)
{
    uint64_t n_mac = 0;
    if (threads < 1) threads = 1;
    if (dX) {
        #pragma omp parallel for num_threads(threads) schedule(static) reduction(+:n_mac)
        for (int64_t b = 0; b < B; ++b) {
            double *row = dX + b * in;
            for (int64_t i = 0; i < in; ++i) row[i] = 0.0;
            for (int64_t o = 0; o < out; ++o) {
                double q = qval(codes, dense, step, b * out + o);
                if (q == 0.0) continue;
                const float *w = W + o * in;
                for (int64_t i = 0; i < in; ++i) row[i] += q * (double)w[i];
                n_mac += (uint64_t)in;
            }
        }
    }
    if (dW) {
        #pragma omp parallel for num_threads(threads) schedule(static) reduction(+:n_mac)
        for (int64_t o = 0; o < out; ++o) {
            double *row = dW + o * in;
            for (int64_t i = 0; i < in; ++i) row[i] = 0.0;
            for (int64_t b = 0; b < B; ++b) {
                double q = qval(codes, dense, step, b * out + o);
                if (q == 0.0) continue;
                const float *x = X + b * in;
                for (int64_t i = 0; i < in; ++i) row[i] += q * (double)x[i];
                n_mac += (uint64_t)in;
            }
        }
    }
    if (macs) *macs = n_mac;
}

/* 8-bit mode weight gradient: dW32[o,i] = sum_b k[b,o] * x8[b,i], exact.  Returns the
 * number of outputs that do not fit int32 (they are stored wrapped; callers treat a
 * non-zero return as an error). */
int64_t dbp_oracle_linear_dw_i8(const int8_t *codes, const int8_t *X8,
                                int64_t B, int64_t in, int64_t out, int32_t *dW32, int threads)
{
    int64_t bad = 0;
    if (threads < 1) threads = 1;
    #pragma omp parallel for num_threads(threads) schedule(static) reduction(+:bad)
    for (int64_t o = 0; o < out; ++o) {
        int64_t *acc = (int64_t *)calloc((size_t)in, sizeof(int64_t));
        for (int64_t b = 0; b < B; ++b) {
            int64_t k = codes[b * out + o];
            if (k == 0) continue;
            const int8_t *x = X8 + b * in;
            for (int64_t i = 0; i < in; ++i) acc[i] += k * (int64_t)x[i];
        }
        for (int64_t i = 0; i < in; ++i) {
            if (acc[i] > INT32_MAX || acc[i] < INT32_MIN) bad++;
            dW32[o * in + i] = (int32_t)acc[i];
        }
        free(acc);
    }
    return bad;
}

/* ------------------------------------------------------------------------------------
 * 2-D convolution.  The paper gives no formula ("analogous"); this is the standard
 * cross-correlation layer with zero padding:
 *   Y[n,k,p,q] = sum_{c,r,s} W[k,c,r,s] * X[n,c, p*st + r - pad, q*st + s - pad]
 * X [N,C,H,Wd], W [K,C,R,S], Y and its gradient Q [N,K,P,Q'],  P = (H+2pad-R)/st + 1.
 * The backward products are the adjoints of that map (Eqs. (qda),(qdw) carried over):
 *   dX[n,c,h,w]   = sum_{k,r,s} Q[n,k,p,q] W[k,c,r,s]   with h = p*st+r-pad, w = q*st+s-pad
 *   dW[k,c,r,s]   = sum_{n,p,q} Q[n,k,p,q] X[n,c,p*st+r-pad,q*st+s-pad]   (zero outside)
 * ---------------------------------------------------------------------------------- */
void dbp_oracle_conv2d_forward(const float *X, const float *W, int64_t N, int64_t C,
                               int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                               int64_t st, int64_t pad, double *Y)
{
    int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
    for (int64_t n = 0; n < N; ++n)
      for (int64_t k = 0; k < K; ++k)
        for (int64_t p = 0; p < P; ++p)
          for (int64_t q = 0; q < Q; ++q) {
              double acc = 0.0;
              for (int64_t c = 0; c < C; ++c)
                for (int64_t r = 0; r < R; ++r)
                  for (int64_t s = 0; s < S; ++s) {
                      int64_t h = p * st + r - pad, w = q * st + s - pad;
                      if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                      acc += (double)W[((k * C + c) * R + r) * S + s] *
                             (double)X[((n * C + c) * H + h) * Wd + w];
                  }
              Y[((n * K + k) * P + p) * Q + q] = acc;
          }
}

void dbp_oracle_conv2d_backward(const int8_t *codes, const float *dense, double step,
                                const float *W, const float *X,
                                int64_t N, int64_t C, int64_t H, int64_t Wd,
                                int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad,
                                double *dX, double *dW, int threads, uint64_t *macs)
{
    int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
    uint64_t n_mac = 0;
    if (threads < 1) threads = 1;
    if (dX) {
        #pragma omp parallel for num_threads(threads) schedule(dynamic, 1) reduction(+:n_mac)
        for (int64_t n = 0; n < N; ++n) {
            double *img = dX + n * C * H * Wd;
            for (int64_t i = 0; i < C * H * Wd; ++i) img[i] = 0.0;
            for (int64_t k = 0; k < K; ++k)
              for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q) {
                    double g = qval(codes, dense, step, ((n * K + k) * P + p) * Q + q);
                    if (g == 0.0) continue;
                    for (int64_t c = 0; c < C; ++c)
                      for (int64_t r = 0; r < R; ++r)
                        for (int64_t s = 0; s < S; ++s) {
                            int64_t h = p * st + r - pad, w = q * st + s - pad;
                            if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                            img[(c * H + h) * Wd + w] +=
                                g * (double)W[((k * C + c) * R + r) * S + s];
                        }
                    n_mac += (uint64_t)(C * R * S);
                }
        }
    }
    if (dW) {
        #pragma omp parallel for num_threads(threads) schedule(dynamic, 1) reduction(+:n_mac)
        for (int64_t k = 0; k < K; ++k) {
            double *flt = dW + k * C * R * S;
            for (int64_t i = 0; i < C * R * S; ++i) flt[i] = 0.0;
            for (int64_t n = 0; n < N; ++n)
              for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q) {
                    double g = qval(codes, dense, step, ((n * K + k) * P + p) * Q + q);
                    if (g == 0.0) continue;
                    for (int64_t c = 0; c < C; ++c)
                      for (int64_t r = 0; r < R; ++r)
                        for (int64_t s = 0; s < S; ++s) {
                            int64_t h = p * st + r - pad, w = q * st + s - pad;
                            if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                            flt[(c * R + r) * S + s] +=
                                g * (double)X[((n * C + c) * H + h) * Wd + w];
                        }
                    n_mac += (uint64_t)(C * R * S);
                }
        }
    }
    if (macs) *macs = n_mac;
}

/* ------------------------------------------------------------------------------------
 * Grouped convolution (the layer type of the two-tower AlexNet and of later CNNs of the kind
 * Sec. "Experiments" trains; the paper gives no formula, this is the standard definition):
 * input and output channels are cut into `groups` equal consecutive blocks, Cg = C/groups and
 * Kg = K/groups, and output channel k sees only the input channels of its own block
 * g(k) = k / Kg.  W is [K, Cg, R, S].
 *   forward   Y[n,k,p,q]   = sum_{c'<Cg, r, s} W[k,c',r,s] X[n, g(k)*Cg + c', p*st+r-pad, q*st+s-pad]
 *   Eq. (qda) dX[n,c,h,w]  = Delta * sum over k with g(k) == c / Cg, and (r,s) with h = p*st+r-pad, w = q*st+s-pad
 *                            of code[n,k,p,q] W[k, c % Cg, r, s]
 *   Eq. (qdw) dW[k,c',r,s] = Delta * sum_{n,p,q} code[n,k,p,q] X[n, g(k)*Cg + c', p*st+r-pad, q*st+s-pad]
 * groups == 1 is dbp_oracle_conv2d_forward / _backward.
 * ---------------------------------------------------------------------------------- */
void dbp_oracle_conv2d_forward_grouped(const float *X, const float *W, int64_t N, int64_t C, int64_t H, int64_t Wd,
                                       int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad, int64_t groups, double *Y)
{
    const int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
    const int64_t Cg = C / groups, Kg = K / groups;
    for (int64_t n = 0; n < N; ++n)
      for (int64_t k = 0; k < K; ++k)
        for (int64_t p = 0; p < P; ++p)
          for (int64_t q = 0; q < Q; ++q) {
              double acc = 0.0;
              for (int64_t cl = 0; cl < Cg; ++cl)
                for (int64_t r = 0; r < R; ++r)
                  for (int64_t s = 0; s < S; ++s) {
                      const int64_t h = p * st + r - pad, w = q * st + s - pad, c = (k / Kg) * Cg + cl;
                      if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                      acc += (double)W[((k * Cg + cl) * R + r) * S + s] * (double)X[((n * C + c) * H + h) * Wd + w];
                  }
              Y[((n * K + k) * P + p) * Q + q] = acc;
          }
}

void dbp_oracle_conv2d_backward_grouped(const int8_t *codes, const float *dense, double step, const float *W, const float *X,
                                        int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                        int64_t st, int64_t pad, int64_t groups, double *dX, double *dW, int threads)
{
    const int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
    const int64_t Cg = C / groups, Kg = K / groups;
    if (threads < 1) threads = 1;
    if (dX) {
        #pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
        for (int64_t n = 0; n < N; ++n) {
            double *img = dX + n * C * H * Wd;
            for (int64_t i = 0; i < C * H * Wd; ++i) img[i] = 0.0;
            for (int64_t k = 0; k < K; ++k)
              for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q) {
                    const double g = qval(codes, dense, step, ((n * K + k) * P + p) * Q + q);
                    if (g == 0.0) continue;
                    for (int64_t cl = 0; cl < Cg; ++cl)
                      for (int64_t r = 0; r < R; ++r)
                        for (int64_t s = 0; s < S; ++s) {
                            const int64_t h = p * st + r - pad, w = q * st + s - pad, c = (k / Kg) * Cg + cl;
                            if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                            img[(c * H + h) * Wd + w] += g * (double)W[((k * Cg + cl) * R + r) * S + s];
                        }
                }
        }
    }
    if (dW) {
        #pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
        for (int64_t k = 0; k < K; ++k) {
            double *flt = dW + k * Cg * R * S;
            for (int64_t i = 0; i < Cg * R * S; ++i) flt[i] = 0.0;
            for (int64_t n = 0; n < N; ++n)
              for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q) {
                    const double g = qval(codes, dense, step, ((n * K + k) * P + p) * Q + q);
                    if (g == 0.0) continue;
                    for (int64_t cl = 0; cl < Cg; ++cl)
                      for (int64_t r = 0; r < R; ++r)
                        for (int64_t s = 0; s < S; ++s) {
                            const int64_t h = p * st + r - pad, w = q * st + s - pad, c = (k / Kg) * Cg + cl;
                            if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                            flt[(cl * R + r) * S + s] += g * (double)X[((n * C + c) * H + h) * Wd + w];
                        }
                }
        }
    }
}

/* 8-bit mode conv weight gradient, exact; same contract as dbp_oracle_linear_dw_i8. */
int64_t dbp_oracle_conv2d_dw_i8(const int8_t *codes, const int8_t *X8,
                                int64_t N, int64_t C, int64_t H, int64_t Wd,
                                int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad,
                                int32_t *dW32, int threads)
{
    int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
    int64_t bad = 0;
    if (threads < 1) threads = 1;
    #pragma omp parallel for num_threads(threads) schedule(dynamic, 1) reduction(+:bad)
    for (int64_t k = 0; k < K; ++k) {
        int64_t *acc = (int64_t *)calloc((size_t)(C * R * S), sizeof(int64_t));
        for (int64_t n = 0; n < N; ++n)
          for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q) {
                int64_t g = codes[((n * K + k) * P + p) * Q + q];
                if (g == 0) continue;
                for (int64_t c = 0; c < C; ++c)
                  for (int64_t r = 0; r < R; ++r)
                    for (int64_t s = 0; s < S; ++s) {
                        int64_t h = p * st + r - pad, w = q * st + s - pad;
                        if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                        acc[(c * R + r) * S + s] +=
                            g * (int64_t)X8[((n * C + c) * H + h) * Wd + w];
                    }
            }
        for (int64_t i = 0; i < C * R * S; ++i) {
            if (acc[i] > INT32_MAX || acc[i] < INT32_MIN) bad++;
            dW32[k * C * R * S + i] = (int32_t)acc[i];
        }
        free(acc);
    }
    return bad;
}

/* ------------------------------------------------------------------------------------
 * Single-output versions, for checking sampled outputs of problems too large to run in
 * full.  Each is the defining sum of one output element, written in gather form
 * (independently of the scatter loops above, which the tests compare them with).
 * idx holds flat output indices; X8 non-NULL selects the integer weight gradient.
 * ---------------------------------------------------------------------------------- */
void dbp_oracle_linear_dx_at(const int8_t *codes, const float *dense, double step,
                             const float *W, int64_t B, int64_t in, int64_t out,
                             const int64_t *idx, int64_t n_idx, double *val)
{
    (void)B;
    for (int64_t t = 0; t < n_idx; ++t) {
        int64_t b = idx[t] / in, i = idx[t] % in;
        double acc = 0.0;
        for (int64_t o = 0; o < out; ++o)
            acc += qval(codes, dense, step, b * out + o) * (double)W[o * in + i];
        val[t] = acc;
    }
}

void dbp_oracle_linear_dw_at(const int8_t *codes, const float *dense, double step,
                             const float *X, const int8_t *X8, int64_t B, int64_t in, int64_t out,
                             const int64_t *idx, int64_t n_idx, double *val)
{
    for (int64_t t = 0; t < n_idx; ++t) {
        int64_t o = idx[t] / in, i = idx[t] % in;
        double acc = 0.0;
        for (int64_t b = 0; b < B; ++b) {
            double x = X8 ? (double)X8[b * in + i] : (double)X[b * in + i];
            double q = X8 ? (double)codes[b * out + o] : qval(codes, dense, step, b * out + o);
            acc += q * x;
        }
        val[t] = acc;
    }
}

void dbp_oracle_conv2d_dx_at(const int8_t *codes, const float *dense, double step,
                             const float *W, int64_t N, int64_t C, int64_t H, int64_t Wd,
                             int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad,
                             const int64_t *idx, int64_t n_idx, double *val)
{
    (void)N;
    int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
    for (int64_t t = 0; t < n_idx; ++t) {
        int64_t f = idx[t];
        int64_t w = f % Wd; f /= Wd;
        int64_t h = f % H;  f /= H;
        int64_t c = f % C;  int64_t n = f / C;
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
          for (int64_t r = 0; r < R; ++r)
            for (int64_t s = 0; s < S; ++s) {
                int64_t hp = h + pad - r, wq = w + pad - s;
                if (hp < 0 || wq < 0 || hp % st || wq % st) continue;
                int64_t p = hp / st, q = wq / st;
                if (p >= P || q >= Q) continue;
                acc += qval(codes, dense, step, ((n * K + k) * P + p) * Q + q) *
                       (double)W[((k * C + c) * R + r) * S + s];
            }
        val[t] = acc;
    }
}

void dbp_oracle_conv2d_dw_at(const int8_t *codes, const float *dense, double step,
                             const float *X, const int8_t *X8,
                             int64_t N, int64_t C, int64_t H, int64_t Wd,
                             int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad,
                             const int64_t *idx, int64_t n_idx, double *val)
{
    int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
    for (int64_t t = 0; t < n_idx; ++t) {
        int64_t f = idx[t];
        int64_t s = f % S; f /= S;
        int64_t r = f % R; f /= R;
        int64_t c = f % C; int64_t k = f / C;
        double acc = 0.0;
        for (int64_t n = 0; n < N; ++n)
          for (int64_t p = 0; p < P; ++p) {
              int64_t h = p * st + r - pad;
              if (h < 0 || h >= H) continue;
              for (int64_t q = 0; q < Q; ++q) {
                  int64_t w = q * st + s - pad;
                  if (w < 0 || w >= Wd) continue;
                  int64_t j = ((n * K + k) * P + p) * Q + q;
                  int64_t xi = ((n * C + c) * H + h) * Wd + w;
                  double x = X8 ? (double)X8[xi] : (double)X[xi];
                  double g = X8 ? (double)codes[j] : qval(codes, dense, step, j);
                  acc += g * x;
              }
          }
        val[t] = acc;
    }
}

/* ------------------------------------------------------------------------------------
 * Forward-pass quantiser of the 8-bit mode (Sec. "Quantizing forward pass": weights and
 * activations are 8-bit in the forward pass; the paper takes the quantiser from the work
 * it cites and prints no formula).  Reading taken: symmetric, one scale per tensor,
 *      amax  = max |x_i| over the finite x_i
 *      scale = amax / 127,  inv = 127 / amax              (fp32 divisions)
 *      q_i   = clamp(round-half-even(x_i * inv), -127, 127)   (ONE fp32 product)
 * NaN -> 0, +-Inf -> +-127; amax == 0 (or nothing finite): scale = inv = 0, every finite
 * q_i = 0.  Parity unpinned against the cited work; pinned by hand-computed values.
 * ---------------------------------------------------------------------------------- */
void dbp_oracle_quantize_int8(const float *x, int64_t n, int8_t *q, float *scale_out, float *inv_out)
{
    float amax = 0.0f;
    for (int64_t i = 0; i < n; ++i)
        if (isfinite(x[i]) && fabsf(x[i]) > amax) amax = fabsf(x[i]);
    const float scale = amax > 0.0f ? amax / 127.0f : 0.0f;
    const float inv = amax > 0.0f ? 127.0f / amax : 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float v;
        if (isnan(x[i])) v = 0.0f;
        else if (isinf(x[i])) v = x[i] > 0.0f ? 127.0f : -127.0f;
        else {
            volatile float prod = x[i] * inv;          /* one fp32 product, rounded to fp32 before the rounding to integer */
            v = nearbyintf(prod);                      /* default rounding mode: ties to even */
            if (v > 127.0f) v = 127.0f;
            if (v < -127.0f) v = -127.0f;
        }
        q[i] = (int8_t)v;
    }
    *scale_out = scale;
    *inv_out = inv;
}

int dbp_oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
