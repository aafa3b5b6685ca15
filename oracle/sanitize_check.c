/*
 * Sanitizer run of the CPU oracle -- TEST INFRASTRUCTURE.  Built together with dbp_oracle.c under
 * -fsanitize=address,undefined and executed by tests/test_oracle_sanitize.py: every oracle function is called on small,
 * ragged shapes (sizes that are not multiples of any tile, paddings wider than the kernel, strides, empty reductions,
 * saturating and non-finite values), so that an out-of-bounds index, a signed overflow or a misaligned access in the
 * oracle's loops aborts the run.  It checks memory safety only; the values are pinned by the tests in tests/.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { uint64_t nnz, n_saturated, n_nonfinite; int32_t max_abs_code, pad_; } stats_t;
uint32_t dbp_oracle_hash(uint64_t, uint64_t);
void dbp_oracle_keys(uint64_t, uint32_t *, uint32_t *);
float dbp_oracle_dither_u(uint64_t, uint64_t);
void dbp_oracle_nsd(const float *, int64_t, float, uint64_t, uint64_t, int8_t *, stats_t *);
float dbp_oracle_step_size(const float *, int64_t, float, double *);
void dbp_oracle_relu_backward(const float *, const float *, int64_t, float *);
void dbp_oracle_bias_grad(const int8_t *, int64_t, int64_t, int, int64_t, float, int64_t *, float *);
void dbp_oracle_tile_format(const int8_t *, int64_t, int64_t, uint64_t *, uint16_t *, uint16_t *);
void dbp_oracle_linear_backward(const int8_t *, const float *, double, const float *, const float *, int64_t, int64_t, int64_t,
                                double *, double *, int, uint64_t *);
int64_t dbp_oracle_linear_dw_i8(const int8_t *, const int8_t *, int64_t, int64_t, int64_t, int32_t *, int);
void dbp_oracle_conv2d_forward(const float *, const float *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                               int64_t, double *);
void dbp_oracle_conv2d_backward(const int8_t *, const float *, double, const float *, const float *, int64_t, int64_t, int64_t,
                                int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, double *, double *, int, uint64_t *);
int64_t dbp_oracle_conv2d_dw_i8(const int8_t *, const int8_t *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                                int64_t, int64_t, int32_t *, int);
void dbp_oracle_linear_dx_at(const int8_t *, const float *, double, const float *, int64_t, int64_t, int64_t, const int64_t *,
                             int64_t, double *);
void dbp_oracle_linear_dw_at(const int8_t *, const float *, double, const float *, const int8_t *, int64_t, int64_t, int64_t,
                             const int64_t *, int64_t, double *);
void dbp_oracle_conv2d_dx_at(const int8_t *, const float *, double, const float *, int64_t, int64_t, int64_t, int64_t, int64_t,
                             int64_t, int64_t, int64_t, int64_t, const int64_t *, int64_t, double *);
void dbp_oracle_conv2d_dw_at(const int8_t *, const float *, double, const float *, const int8_t *, int64_t, int64_t, int64_t,
                             int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, const int64_t *, int64_t, double *);
void dbp_oracle_quantize_int8(const float *, int64_t, int8_t *, float *, float *);
void dbp_oracle_conv2d_forward_grouped(const float *, const float *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                                       int64_t, int64_t, double *);
void dbp_oracle_conv2d_backward_grouped(const int8_t *, const float *, double, const float *, const float *, int64_t, int64_t, int64_t,
                                        int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, double *, double *, int);
void dbp_oracle_topk_threshold(const float *, int64_t, int64_t, int64_t, float *);
void dbp_oracle_topk_quantize(const float *, int64_t, int64_t, int64_t, float, int8_t *, stats_t *);

static uint64_t lcg = 88172645463325252ull;
static double rnd(void) { lcg ^= lcg << 13; lcg ^= lcg >> 7; lcg ^= lcg << 17; return (double)(lcg >> 11) / 9007199254740992.0 - 0.5; }

/* exact-size heap blocks: the sanitizer sees the first byte past the end */
static float *falloc(int64_t n, double scale) { float *p = malloc((size_t)(n > 0 ? n : 1) * sizeof(float)); for (int64_t i = 0; i < n; ++i) p[i] = (float)(rnd() * scale); return p; }

int main(void)
{
    uint32_t k0, k1;
    dbp_oracle_keys(0xFFFFFFFFFFFFFFFFull, &k0, &k1);
    (void)dbp_oracle_hash(12345678901234ull, 0xFFFFFFFFFFFFFFFFull);
    (void)dbp_oracle_dither_u(1, 0xFFFFFFFFFFFFFFFEull);

    /* quantiser, statistics, format: ragged sizes, saturating and non-finite values */
    const int64_t rows = 3, cols = 517, n = rows * cols;
    float *d = falloc(n, 8e-3);
    d[5] = NAN; d[77] = INFINITY; d[78] = -INFINITY; d[100] = 10.0f; d[n - 1] = -10.0f;
    int8_t *codes = malloc((size_t)n);
    stats_t st;
    dbp_oracle_nsd(d, n, 4e-3f, 1, 0xFFFFFFFFFFFFFF00ull, codes, &st);
    dbp_oracle_nsd(d, 0, 4e-3f, 1, 0, codes, NULL);
    double sigma;
    (void)dbp_oracle_step_size(d, n, 4.0f, &sigma);
    (void)dbp_oracle_step_size(d, 1, 4.0f, &sigma);
    (void)dbp_oracle_step_size(d, n - 1, 4.0f, &sigma);
    float *act = falloc(n, 2.0), *dz = malloc((size_t)n * sizeof(float));
    dbp_oracle_relu_backward(d, act, n, dz);
    int64_t tpr = (cols + 255) / 256, tiles = rows * tpr;
    uint64_t *bitmap = malloc((size_t)tiles * 4 * sizeof(uint64_t));
    uint16_t *tnz = malloc((size_t)tiles * sizeof(uint16_t)), *ent = malloc((size_t)tiles * 256 * sizeof(uint16_t));
    dbp_oracle_tile_format(codes, rows, cols, bitmap, tnz, ent);
    int64_t *sums = malloc((size_t)cols * sizeof(int64_t));
    float *grad = malloc((size_t)cols * sizeof(float));
    dbp_oracle_bias_grad(codes, rows, cols, 0, cols, 4e-3f, sums, grad);
    dbp_oracle_bias_grad(codes, rows, cols, 1, 3, 4e-3f, sums, grad);
    int8_t *q8 = malloc((size_t)n);
    float sc, inv;
    dbp_oracle_quantize_int8(d, n, q8, &sc, &inv);
    float *thr = malloc((size_t)rows * sizeof(float));
    dbp_oracle_topk_threshold(d, rows, cols, 7, thr);
    dbp_oracle_topk_threshold(d, rows, cols, cols + 5, thr);
    dbp_oracle_topk_threshold(d, rows, cols, 0, thr);
    dbp_oracle_topk_quantize(d, rows, cols, 7, 4e-3f, codes, &st);
    dbp_oracle_topk_quantize(d, 1, n, n, 4e-3f, codes, NULL);

    /* fully connected products: B x out codes (the first B*out of `codes`), W [out x in], X [B x in] */
    const int64_t B = 5, in = 13, out = 7;
    dbp_oracle_nsd(d, B * out, 4e-3f, 3, 0, codes, &st);
    float *W = falloc(out * in, 1.0), *X = falloc(B * in, 1.0);
    double *dX = malloc((size_t)(B * in) * sizeof(double)), *dW = malloc((size_t)(out * in) * sizeof(double));
    uint64_t macs;
    dbp_oracle_linear_backward(codes, NULL, 4e-3, W, X, B, in, out, dX, dW, 3, &macs);
    dbp_oracle_linear_backward(NULL, d, 0.0, W, X, B, in, out, dX, NULL, 1, NULL);
    int8_t *X8 = malloc((size_t)(B * in));
    for (int64_t i = 0; i < B * in; ++i) X8[i] = (int8_t)(rnd() * 254.0);
    int32_t *dW32 = malloc((size_t)(out * in) * sizeof(int32_t));
    (void)dbp_oracle_linear_dw_i8(codes, X8, B, in, out, dW32, 2);
    int64_t idx[4] = {0, B * in - 1, 17, 3};
    double val[4];
    dbp_oracle_linear_dx_at(codes, NULL, 4e-3, W, B, in, out, idx, 4, val);
    int64_t idw[4] = {0, out * in - 1, 17, 3};
    dbp_oracle_linear_dw_at(codes, NULL, 4e-3, X, NULL, B, in, out, idw, 4, val);
    dbp_oracle_linear_dw_at(codes, NULL, 1.0, NULL, X8, B, in, out, idw, 4, val);

    /* convolutions: odd sizes, stride 2 and 3, padding wider than the kernel reach */
    const int64_t geo[4][9] = {/* N, C, H, Wd, K, R, S, stride, pad */ {2, 4, 7, 5, 6, 3, 3, 1, 1}, {1, 2, 9, 8, 3, 5, 3, 2, 2},
                               {2, 1, 6, 6, 2, 3, 3, 3, 3}, {1, 4, 4, 4, 4, 1, 1, 1, 0}};
    for (int g = 0; g < 4; ++g) {
        const int64_t N = geo[g][0], C = geo[g][1], H = geo[g][2], Wd = geo[g][3], K = geo[g][4], R = geo[g][5], S = geo[g][6],
                      stv = geo[g][7], pad = geo[g][8];
        const int64_t P = (H + 2 * pad - R) / stv + 1, Q = (Wd + 2 * pad - S) / stv + 1;
        float *cx = falloc(N * C * H * Wd, 1.0), *cw = falloc(K * C * R * S, 1.0), *cd = falloc(N * K * P * Q, 8e-3);
        int8_t *ck = malloc((size_t)(N * K * P * Q));
        dbp_oracle_nsd(cd, N * K * P * Q, 4e-3f, 9, 0, ck, &st);
        double *y = malloc((size_t)(N * K * P * Q) * sizeof(double));
        dbp_oracle_conv2d_forward(cx, cw, N, C, H, Wd, K, R, S, stv, pad, y);
        double *cdx = malloc((size_t)(N * C * H * Wd) * sizeof(double)), *cdw = malloc((size_t)(K * C * R * S) * sizeof(double));
        dbp_oracle_conv2d_backward(ck, NULL, 4e-3, cw, cx, N, C, H, Wd, K, R, S, stv, pad, cdx, cdw, 2, &macs);
        dbp_oracle_conv2d_backward(NULL, cd, 0.0, cw, cx, N, C, H, Wd, K, R, S, stv, pad, NULL, cdw, 1, NULL);
        int8_t *cx8 = malloc((size_t)(N * C * H * Wd));
        for (int64_t i = 0; i < N * C * H * Wd; ++i) cx8[i] = (int8_t)(rnd() * 254.0);
        int32_t *cdw32 = malloc((size_t)(K * C * R * S) * sizeof(int32_t));
        (void)dbp_oracle_conv2d_dw_i8(ck, cx8, N, C, H, Wd, K, R, S, stv, pad, cdw32, 2);
        int64_t ix[3] = {0, N * C * H * Wd - 1, (N * C * H * Wd) / 2}, iw[3] = {0, K * C * R * S - 1, (K * C * R * S) / 2};
        dbp_oracle_conv2d_dx_at(ck, NULL, 4e-3, cw, N, C, H, Wd, K, R, S, stv, pad, ix, 3, val);
        dbp_oracle_conv2d_dw_at(ck, NULL, 4e-3, cx, NULL, N, C, H, Wd, K, R, S, stv, pad, iw, 3, val);
        dbp_oracle_conv2d_dw_at(ck, NULL, 1.0, NULL, cx8, N, C, H, Wd, K, R, S, stv, pad, iw, 3, val);
        for (int64_t grp = 2; grp <= 4; grp += 2)
            if (C % grp == 0 && K % grp == 0) {
                float *gw = falloc(K * (C / grp) * R * S, 1.0);
                double *gdw = malloc((size_t)(K * (C / grp) * R * S) * sizeof(double));
                dbp_oracle_conv2d_forward_grouped(cx, gw, N, C, H, Wd, K, R, S, stv, pad, grp, y);
                dbp_oracle_conv2d_backward_grouped(ck, NULL, 4e-3, gw, cx, N, C, H, Wd, K, R, S, stv, pad, grp, cdx, gdw, 2);
                free(gw); free(gdw);
            }
        free(cx); free(cw); free(cd); free(ck); free(y); free(cdx); free(cdw); free(cx8); free(cdw32);
    }
    free(d); free(codes); free(act); free(dz); free(bitmap); free(tnz); free(ent); free(sums); free(grad); free(q8); free(thr);
    free(W); free(X); free(dX); free(dW); free(X8); free(dW32);
    puts("oracle sanitizer run: ok");
    return 0;
}
