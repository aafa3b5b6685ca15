// C ABI of the library (include/dbp.h): argument validation on the host, workspace carving, launches.
// Every check happens before the first HIP call so that all statuses but DBP_ERR_DEVICE are
// reachable on a machine without a GPU.
#include <cmath>
#include <cstring>
#include <mutex>
#include "common.h"

using namespace dbp;

// Scratch of nsd_quantize_static (the per-workgroup statistics records of the quantiser): device memory that lives in the
// library's code object, one copy per GPU, until the process ends.  In host code `scratch` is only a handle of the symbol:
// its device address comes from hipGetSymbolAddress, once per device (static_scratch below).
static __device__ __align__(256) unsigned char scratch[dbp::kNsdScratchBytes];

namespace {

// `path` = a kernel family, optionally with DBP_PATH_TWO_PLANES.
inline dbp_path path_family(dbp_path p) { return (dbp_path)((int)p & ~(int)DBP_PATH_TWO_PLANES); }
inline bool     path_two_planes(dbp_path p) { return ((int)p & (int)DBP_PATH_TWO_PLANES) != 0; }
inline bool     path_ok(dbp_path p)
{
    const dbp_path f = path_family(p);
    return f == DBP_PATH_AUTO || f == DBP_PATH_MFMA || f == DBP_PATH_GATHER;
}
inline dbp_path path_with_flags(dbp_path family, dbp_path from) { return (dbp_path)((int)family | ((int)from & (int)DBP_PATH_TWO_PLANES)); }


constexpr int64_t kMaxElems = (int64_t)1 << 40;
constexpr int64_t kMaxDim = (int64_t)1 << 30;          // GEMM indices are 32-bit

bool step_ok(float step)
{
    if (!(step > 0.0f) || !std::isfinite(step)) return false;
    const float inv = 1.0f / step;
    return std::isfinite(inv) && inv >= 1.17549435e-38f && step >= 1.17549435e-38f;
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

dbp_status format_layout(int64_t rows, int64_t cols, dbp_format_layout *L)
{
    if (!L) return DBP_ERR_NULL;
    if (rows <= 0 || cols <= 0 || rows > kMaxElems / cols) return DBP_ERR_SHAPE;
    const int64_t tpr = (cols + DBP_TILE - 1) / DBP_TILE;
    const int64_t nt = rows * tpr;
    L->tiles_per_row = tpr;
    L->n_tiles = nt;
    L->bitmap_offset = 0;
    L->tile_nnz_offset = align_up((size_t)nt * 4 * sizeof(uint64_t), 256);
    L->entries_offset = L->tile_nnz_offset + align_up((size_t)nt * sizeof(uint16_t), 256);
    L->scratch_offset = L->entries_offset + align_up((size_t)nt * DBP_TILE * sizeof(uint16_t), 256);
    L->total_bytes = L->scratch_offset + kNsdScratchBytes;
    return DBP_OK;
}

struct Carve {                      // pieces of a backward workspace
    dbp_format_layout fmt;
    size_t codes_offset, scratch_offset, total;
};

Carve carve(int64_t rows, int64_t cols, size_t scratch_bytes)
{
    Carve c;
    format_layout(rows, cols, &c.fmt);
    c.codes_offset = c.fmt.total_bytes;
    c.scratch_offset = c.codes_offset + align_up((size_t)(rows * cols), 256);
    c.total = c.scratch_offset + scratch_bytes;
    return c;
}

// `fmt_base` is a buffer with layout *L; the tile-sparse arrays are written only if `want_format`
// (its statistics records are used either way).
dbp_status run_nsd(const float *delta, int64_t rows, int64_t cols, float step, uint64_t seed, uint64_t idx_base,
                   int8_t *codes, char *fmt_base, const dbp_format_layout *L, dbp_stats *stats, hipStream_t s,
                   bool want_format = true, StatsJob *defer = nullptr, const dbp_nsd_extras *ex = nullptr, bool bias_zeroed = false,
                   const StepTree *tree = nullptr, const uint32_t *topk_thr = nullptr, int64_t topk_vec_rows = 1)
{
    NsdArgs a;
    a.topk_thr = topk_thr; a.topk_vec_rows = topk_vec_rows;
    a.delta = delta; a.codes = codes; a.stats = stats;
    const bool fmt = fmt_base && want_format;
    a.bitmap = fmt ? (uint64_t *)(fmt_base + L->bitmap_offset) : nullptr;
    a.tile_nnz = fmt ? (uint16_t *)(fmt_base + L->tile_nnz_offset) : nullptr;
    a.entries = fmt ? (uint16_t *)(fmt_base + L->entries_offset) : nullptr;
    a.partials = fmt_base ? (u32x4 *)(fmt_base + L->scratch_offset) : nullptr;
    a.rows = rows; a.cols = cols; a.tiles_per_row = L->tiles_per_row; a.n_tiles = L->n_tiles;
    a.inv_step = 1.0f / step;
    a.act = nullptr; a.step_dev = nullptr; a.bias_sums = nullptr; a.bias_grad = nullptr; a.bias_mode = 0; a.bias_len = 0; a.step = step;
    a.bias_zeroed = bias_zeroed ? 1 : 0;
    a.tree = tree ? *tree : StepTree{nullptr, nullptr, 0, 0, 0.0f, nullptr};
    if (ex) {
        a.act = ex->act; a.step_dev = ex->step_dev; a.bias_sums = ex->bias_sums; a.bias_grad = ex->bias_grad;
        a.bias_mode = ex->bias_mode; a.bias_len = ex->bias_len;
    }
    const DitherKeys k = make_dither_keys(seed);
    a.k0 = k.k0; a.k1 = k.k1; a.idx_base = idx_base;
    return launch_nsd(a, s, defer) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
}

dbp_status check_linear_dims(int64_t B, int64_t in, int64_t out)
{
    if (B <= 0 || in <= 0 || out <= 0 || B > kMaxDim || in > kMaxDim || out > kMaxDim) return DBP_ERR_SHAPE;
    if (B > kMaxElems / out || B > kMaxElems / in || out > kMaxElems / in) return DBP_ERR_SHAPE;
    return DBP_OK;
}

dbp_status check_conv_dims(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                           int64_t stride, int64_t pad, int64_t *P, int64_t *Q)
{
    if (N <= 0 || C <= 0 || H <= 0 || Wd <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return DBP_ERR_SHAPE;
    if (N > 65535 || C > 65535 || K > 65535 || H > 65535 || Wd > 65535 || R > 255 || S > 255 || pad > 255 || stride > 255) return DBP_ERR_SHAPE;
    if (H + 2 * pad < R || Wd + 2 * pad < S) return DBP_ERR_SHAPE;
    *P = (H + 2 * pad - R) / stride + 1;
    *Q = (Wd + 2 * pad - S) / stride + 1;
    // every GEMM index (rows, cols, padded reductions) must fit 31 bits
    const int64_t lim = ((int64_t)1 << 31) - 4096;
    if (N * H * Wd >= lim || N * (*P * *Q + 64) >= lim || C * R * S >= lim || R * S * (K + 16) >= lim) return DBP_ERR_SHAPE;
    if (N * K * *P * *Q >= kMaxElems || N * C * H * Wd >= kMaxElems) return DBP_ERR_SHAPE;
    return DBP_OK;
}

dbp_status check_extras(const dbp_nsd_extras *ex, int64_t rows, int64_t cols)
{
    if (!ex) return DBP_OK;
    if (ex->act && !aligned(ex->act, 4)) return DBP_ERR_SHAPE;
    if (ex->step_dev && !aligned(ex->step_dev, 4)) return DBP_ERR_SHAPE;
    if (ex->bias_grad && !ex->bias_sums) return DBP_ERR_NULL;
    if (ex->bias_sums) {
        if (!aligned(ex->bias_sums, 8)) return DBP_ERR_SHAPE;
        if (ex->bias_mode == DBP_BIAS_PER_COLUMN) { if (ex->bias_len != cols) return DBP_ERR_SHAPE; }
        else if (ex->bias_mode == DBP_BIAS_PER_ROW_GROUP) { if (ex->bias_len <= 0 || rows % ex->bias_len) return DBP_ERR_SHAPE; }
        else return DBP_ERR_UNSUPPORTED;
    }
    return DBP_OK;
}

// Workspace of the whole-layer entry points: the backward workspace, then the step-size scratch, the
// {Delta, 1/Delta} pair and the bias code sums.
struct LayerCarve { size_t step_scratch, step_pair, bias_sums, total; };
LayerCarve layer_carve(size_t backward_total, int64_t n, int64_t bias_len)
{
    LayerCarve c;
    c.step_scratch = align_up(backward_total, 256);
    c.step_pair = c.step_scratch + step_size_scratch_bytes(n);
    c.bias_sums = c.step_pair + 256;
    c.total = c.bias_sums + align_up((size_t)bias_len * sizeof(int64_t), 256);
    return c;
}

// ---- density dispatch of DBP_PATH_AUTO ----------------------------------------------------------------------
// The matrix-core kernels do the dense work whatever the codes are; the gather kernels do work in proportion to the
// nonzero codes plus a fixed cost (streaming the dense operand, writing the outputs).  Only the device knows the nonzero
// count when the products are launched, so where the gather family can win at all, BOTH families are launched behind a
// gate: the kernel that sums the quantiser's statistics also writes a flag (1 when fewer than `gather_below` codes are
// nonzero) and each family's kernels return at once unless the flag names them.  No host round trip, no allocation; the
// losing family costs its empty launches, which is why shapes where the gather kernels' fixed cost alone is close to the
// matrix-core time are not dispatched at all.  The estimates below are linear models with constants measured on MI355X
// (microseconds; flop per microsecond; bytes per microsecond).
struct AutoPlan {
    bool dual; uint64_t gather_below;
    // convolution dW alone on the plane-scanning gather kernel below this many nonzeros (0: never), dX staying on matrix cores
    uint64_t dw_rows_below = 0;
    bool gated() const { return dual || dw_rows_below > 0; }
};

AutoPlan linear_auto_plan(const LinearArgs &call, bool launchable)
{
    AutoPlan ap{false, 0};
    if (!launchable) return ap;
    LinearArgs probe = call;
    if (!linear_gather_gated_ok(probe)) return ap;
    int ungated = 0;
    probe.plan_only = &ungated;
    (void)launch_linear_mfma(probe, nullptr);                    // plan only: launches nothing
    if (ungated) return ap;
    const double B = (double)call.B, in = (double)call.in, out = (double)call.out;
    const int products = (call.dX ? 1 : 0) + (call.dW ? 1 : 0);
    const double mfma_us = products * 2.0 * B * in * out * (call.two_planes ? 2.0 : 3.0) / 0.95e9;   // the bf16 planes at 0.95 PFLOP/s
    // gather kernels: a step (one 64-index chunk of one row block: tile through LDS, barrier) costs about 2.2 us however
    // few nonzeros it holds; the nonzeros themselves run at about 32 TFLOP/s per product when all CUs have a workgroup
    GatherShape gs[2];
    linear_gather_shape(call.B, call.in, call.out, gs);
    double fixed_us = 0.0, per_nnz_us = 0.0;
    for (int i = 0; i < 2; ++i) {
        if (!(i == 0 ? call.dX != nullptr : call.dW != nullptr)) continue;
        const double waves = (double)((gs[i].workgroups + 255) / 256);
        fixed_us += waves * gs[i].steps * 2.2 + (gs[i].partial_bytes ? 6.0 + 2.0 * gs[i].partial_bytes / 5.0e6 : 0.0);
        if (i == 1) fixed_us += out * in * 4.0 / 5.0e6;                                // dW is written once
        const double util = gs[i].workgroups >= 256 ? 1.0 : gs[i].workgroups / 256.0;
        per_nnz_us += 2.0 * in / (32e6 * util);
    }
    if (fixed_us > 0.9 * mfma_us) return ap;
    const double thr = (mfma_us - fixed_us) / per_nnz_us;
    ap.dual = true;
    ap.gather_below = thr >= B * out ? (uint64_t)(B * out) + 1 : (uint64_t)thr;
    return ap;
}

AutoPlan conv_auto_plan(const ConvArgs &call, int64_t P, int64_t Q)
{
    AutoPlan ap{false, 0};
    if (!conv_gather_supported(call.N, call.C, call.H, call.Wd, call.K, call.R, call.S, P, Q, false)) return ap;
    ConvArgs probe = call;
    int ungated = 0;
    StatsJob none{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr};
    probe.plan_only = &ungated; probe.stats_job = none;
    (void)launch_conv_mfma(probe, nullptr);                      // plan only: launches nothing
    if (ungated) return ap;
    const double crs = (double)(call.C * call.R * call.S), n_codes = (double)(call.N * call.K * P * Q);
    const double flops = 2.0 * n_codes * crs;                                        // one dense product
    const double planes = call.two_planes ? 2.0 : 3.0;
    // dW alone on the kernel that scans the code planes (fp32 activations: the int8 matrix-core kernel is out of its reach).
    // Matrix-core dW measured on 13 layer shapes: 25 us + the bf16 planes at 0.95 PFLOP/s, within 22 %.  The gather kernel must
    // be modelled 15 % faster to be chosen, and the switch must lie above 0.5 % nonzeros to be worth its two empty launches.
    if (call.dW && call.x_dtype == DBP_F32) {
        double fixed_us = 0.0, per_nnz_us = 0.0;
        if (conv_dw_rows_cost(call, P, Q, call.scratch_bytes, &fixed_us, &per_nnz_us)) {
            const double mfma_dw_us = 25.0 + flops * planes / 0.95e9;
            const double thr = (0.85 * mfma_dw_us - fixed_us) / per_nnz_us;
            // every gated launch that returns at once still costs 2.5-4.5 us: the two launches of this state must have at
            // least 25 us to win at the sparse end, and then stand in for the whole-family state below (whose four launches,
            // format and separate flag kernel cost 10-14 us at every density, to win only beyond ~99.8 % zeros)
            if (thr >= 0.005 * n_codes && mfma_dw_us - fixed_us >= 25.0) {
                ap.dw_rows_below = thr >= n_codes ? (uint64_t)n_codes + 1 : (uint64_t)thr;
                return ap;
            }
        }
    }
    // Both products on the gather family.  The kernels that walk the format's entries give every workgroup a few channels and
    // let it walk ALL entries of its image (dX) or of its output channel (dW): with large planes few channels fit a workgroup
    // (their dX planes accumulate in LDS) and the walk is repeated by many workgroups -- measured on 56x56 planes: 1.0 ms at
    // 99.9 % zeros against 0.41 ms on matrix cores.  This side of the gate is only worth its empty launches on small planes
    // (14x14: 0.065 against 0.155 ms at 99.9 %).
    if (call.H * call.Wd > 1024 || P * Q > 1024) return ap;
    if (call.dX && !conv_gather_supported(call.N, call.C, call.H, call.Wd, call.K, call.R, call.S, P, Q, true)) return ap;
    double mfma_us = 0.0;
    if (call.dX) mfma_us += flops * planes / 0.9e9;
    if (call.dW) mfma_us += call.x_dtype == DBP_I8 ? flops / 1.4e9 : flops * planes / 0.6e9;
    const double x_elems = (double)(call.N * call.C * call.H * call.Wd);
    const double fixed_us = 15.0 + (call.dX ? x_elems * 4.0 : 0.0) / 2.0e6 + (call.dW ? x_elems * (call.x_dtype == DBP_I8 ? 1.0 : 4.0) : 0.0) / 2.0e6;
    if (fixed_us > 0.5 * mfma_us) return ap;
    const int products = (call.dX ? 1 : 0) + (call.dW ? 1 : 0);
    const double per_nnz_us = products * 2.0 * crs / 1.4e6;                          // 1.4 TFLOP/s on nonzeros (LDS read-modify-write bound)
    const double thr = (mfma_us - fixed_us) / per_nnz_us;
    ap.dual = true;
    ap.gather_below = thr >= n_codes ? (uint64_t)n_codes + 1 : (uint64_t)thr;
    return ap;
}

dbp_status linear_products(const int8_t *codes, const void *format, float step, const float *W, const void *X,
                           dbp_dtype x_dtype, int64_t B, int64_t in, int64_t out, float *dX, void *dW,
                           void *workspace, size_t workspace_bytes, dbp_path path, void *stream, StatsJob job,
                           const float *step_dev = nullptr, Gate gate = Gate{})
{
    if (!codes || !W || (!dX && !dW) || (dW && !X)) return DBP_ERR_NULL;
    dbp_status st = check_linear_dims(B, in, out);
    if (st != DBP_OK) return st;
    if (!step_dev && !step_ok(step)) return DBP_ERR_STEP;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return DBP_ERR_DTYPE;
    if (!path_ok(path)) return DBP_ERR_UNSUPPORTED;
    if (x_dtype == DBP_I8 && dW && B * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    if (path_family(path) == DBP_PATH_GATHER && !linear_gather_supported(B, in, out)) return DBP_ERR_UNSUPPORTED;
    LinearArgs a;
    a.codes = codes; a.dense = nullptr; a.step = step; a.step_dev = step_dev; a.W = W; a.W8 = nullptr; a.X = X; a.x_dtype = x_dtype;
    a.B = B; a.in = in; a.out = out; a.dX = dX; a.dW = dW; a.stats_job = job; a.gate = gate;
    a.two_planes = path_two_planes(path);
    if (path_family(path) == DBP_PATH_GATHER) {
        if (!format) return DBP_ERR_NULL;
        if (!aligned(format, 256)) return DBP_ERR_WORKSPACE;
        dbp_format_layout L;
        format_layout(B, out, &L);
        const char *fb = (const char *)format;
        FormatView f{(const uint64_t *)(fb + L.bitmap_offset), (const uint16_t *)(fb + L.tile_nnz_offset),
                     (const uint16_t *)(fb + L.entries_offset), L.tiles_per_row};
        // split partials of the dX kernel live in the workspace; without one the kernel runs unsplit
        const bool ws_ok = workspace && aligned(workspace, 256);
        a.scratch = ws_ok ? workspace : nullptr; a.scratch_bytes = ws_ok ? workspace_bytes : 0;
        if (launch_stats_job(job, (hipStream_t)stream) != hipSuccess) return DBP_ERR_DEVICE;
        return launch_linear_gather(a, f, (hipStream_t)stream) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
    }
    const size_t need = linear_scratch_bytes(B, in, out);
    if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    a.scratch = workspace; a.scratch_bytes = workspace_bytes;
    return launch_linear_mfma(a, (hipStream_t)stream) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
}

dbp_status conv2d_products(const int8_t *codes, const void *format, float step, const float *W, const void *X,
                               dbp_dtype x_dtype, int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K,
                               int64_t R, int64_t S, int64_t stride, int64_t pad, float *dX, void *dW,
                               void *workspace, size_t workspace_bytes, dbp_path path, void *stream, const float *step_dev = nullptr,
                               StatsJob job = StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr}, Gate gate = Gate{},
                               Gate gate_dw = Gate{}, bool rows_gated = false)
{
    if (!codes || !W || (!dX && !dW) || (dW && !X)) return DBP_ERR_NULL;
    int64_t P, Q;
    dbp_status st = check_conv_dims(N, C, H, Wd, K, R, S, stride, pad, &P, &Q);
    if (st != DBP_OK) return st;
    if (!step_dev && !step_ok(step)) return DBP_ERR_STEP;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return DBP_ERR_DTYPE;
    if (!path_ok(path)) return DBP_ERR_UNSUPPORTED;
    if (path_family(path) == DBP_PATH_GATHER && !conv_gather_supported(N, C, H, Wd, K, R, S, P, Q, dX != nullptr)) return DBP_ERR_UNSUPPORTED;
    if (x_dtype == DBP_I8 && dW && N * P * Q * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    if (path_family(path) == DBP_PATH_GATHER) {
        if (!format) return DBP_ERR_NULL;
        if (!aligned(format, 256)) return DBP_ERR_WORKSPACE;
        dbp_format_layout L;
        format_layout(N * K, P * Q, &L);
        const char *fb = (const char *)format;
        FormatView f{(const uint64_t *)(fb + L.bitmap_offset), (const uint16_t *)(fb + L.tile_nnz_offset),
                     (const uint16_t *)(fb + L.entries_offset), L.tiles_per_row};
        ConvArgs g;
        g.codes = codes; g.dense = nullptr; g.step = step; g.step_dev = step_dev; g.W = W; g.W8 = nullptr; g.X = X; g.x_dtype = x_dtype;
        g.N = N; g.C = C; g.H = H; g.Wd = Wd; g.K = K; g.R = R; g.S = S; g.pad = pad; g.stride = stride;
        // the kernels that read the code plane keep prepared weights and partial sums in the workspace; without one the kernels
        // that walk the format's entries serve
        const bool ws_ok = workspace && aligned(workspace, 256);
        g.dX = dX; g.dW = dW; g.scratch = ws_ok ? workspace : nullptr; g.scratch_bytes = ws_ok ? workspace_bytes : 0;
        g.stats_job = StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr}; g.pending = nullptr; g.gate = gate; g.rows_gated = rows_gated;
        if (launch_stats_job(job, (hipStream_t)stream) != hipSuccess) return DBP_ERR_DEVICE;
        return launch_conv_gather(g, f, (hipStream_t)stream) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
    }
    const size_t need = conv_scratch_bytes(N, C, H, Wd, K, R, S, pad, stride);
    if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    ConvArgs a;
    a.codes = codes; a.dense = nullptr; a.step = step; a.step_dev = step_dev; a.W = W; a.W8 = nullptr; a.X = X; a.x_dtype = x_dtype;
    a.N = N; a.C = C; a.H = H; a.Wd = Wd; a.K = K; a.R = R; a.S = S; a.pad = pad; a.stride = stride;
    a.dX = dX; a.dW = dW; a.scratch = workspace; a.scratch_bytes = workspace_bytes;
    a.stats_job = job; a.pending = nullptr; a.gate = gate; a.gate_dw = gate_dw;
    a.two_planes = path_two_planes(path);
    return launch_conv_mfma(a, (hipStream_t)stream) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
}

// The products of a dithered_* call after its quantiser: one family, or (DBP_PATH_AUTO on a shape where the gather
// kernels can win) both behind the density gate.  `ws` is the call's workspace (format region first), `job` the
// quantiser's pending statistics sum.
dbp_status linear_products_dispatch(const AutoPlan &ap, const int8_t *k, char *ws, const Carve &c, size_t scratch_bytes, float step,
                                    const float *W, const void *X, dbp_dtype x_dtype, int64_t B, int64_t in, int64_t out, float *dX,
                                    void *dW, dbp_path path, void *stream, StatsJob job, const float *step_dev)
{
    if (!ap.gated())
        return linear_products(k, ws, step, W, X, x_dtype, B, in, out, dX, dW, ws + c.scratch_offset, scratch_bytes, path, stream, job, step_dev);
    int *flag = (int *)(ws + c.fmt.scratch_offset + kNsdFlagOffset);
    job.flag = flag; job.gather_below = ap.gather_below;
    if (launch_stats_job(job, (hipStream_t)stream) != hipSuccess) return DBP_ERR_DEVICE;
    const StatsJob none{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr};
    dbp_status st = linear_products(k, ws, step, W, X, x_dtype, B, in, out, dX, dW, ws + c.scratch_offset, scratch_bytes, path_with_flags(DBP_PATH_MFMA, path),
                                    stream, none, step_dev, Gate{flag, 0});
    if (st != DBP_OK) return st;
    return linear_products(k, ws, step, W, X, x_dtype, B, in, out, dX, dW, ws + c.scratch_offset, scratch_bytes, DBP_PATH_GATHER,
                           stream, none, step_dev, Gate{flag, 1});
}

dbp_status conv2d_products_dispatch(const AutoPlan &ap, const int8_t *k, char *ws, const Carve &c, size_t scratch_bytes, float step,
                                    const float *W, const void *X, dbp_dtype x_dtype, int64_t N, int64_t C, int64_t H, int64_t Wd,
                                    int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad, float *dX, void *dW, dbp_path path,
                                    void *stream, StatsJob job, const float *step_dev)
{
    if (!ap.gated())
        return conv2d_products(k, ws, step, W, X, x_dtype, N, C, H, Wd, K, R, S, stride, pad, dX, dW, ws + c.scratch_offset, scratch_bytes,
                               path, stream, step_dev, job);
    // Three states, one flag each (write_density_flags): everything on matrix cores; dX on matrix cores and dW on the gather
    // kernel that scans the code planes; everything on the gather kernels that walk the format's entries.
    int *flag = (int *)(ws + c.fmt.scratch_offset + kNsdFlagOffset);
    job.flag = flag; job.gather_below = ap.dual ? ap.gather_below : 0; job.dw_rows_below = dW ? ap.dw_rows_below : 0;
    const bool rows = job.dw_rows_below > 0;
    const StatsJob none{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr};
    // The flags must be there before the first gated kernel: the sum that writes them rides in the weight preparation of the
    // dX kernel as usual (small preparation kernels are not gated), or, without dX, is launched on its own.
    if (!dX) {
        if (launch_stats_job(job, (hipStream_t)stream) != hipSuccess) return DBP_ERR_DEVICE;
        job = none;
    }
    dbp_status st = conv2d_products(k, ws, step, W, X, x_dtype, N, C, H, Wd, K, R, S, stride, pad, dX, dW, ws + c.scratch_offset,
                                    scratch_bytes, path_with_flags(DBP_PATH_MFMA, path), stream, step_dev, job,
                                    ap.dual ? Gate{flag, 0} : Gate{}, rows ? Gate{flag + 2, 1} : Gate{});
    if (st != DBP_OK) return st;
    if (ap.dual) {
        st = conv2d_products(k, ws, step, W, X, x_dtype, N, C, H, Wd, K, R, S, stride, pad, dX, dW, ws + c.scratch_offset,
                             scratch_bytes, DBP_PATH_GATHER, stream, step_dev, none, Gate{flag, 1});
        if (st != DBP_OK) return st;
    }
    if (rows)
        st = conv2d_products(k, ws, step, W, X, x_dtype, N, C, H, Wd, K, R, S, stride, pad, nullptr, dW, ws + c.scratch_offset,
                             scratch_bytes, DBP_PATH_GATHER, stream, step_dev, none, Gate{flag + 1, 1}, Gate{}, true);
    return st;
}

LinearArgs linear_call(const float *W, const void *X, dbp_dtype x_dtype, int64_t B, int64_t in, int64_t out, float *dX, void *dW,
                       const int8_t *codes, char *scratch, size_t scratch_bytes, bool two_planes)
{
    LinearArgs a;
    a.two_planes = two_planes;
    a.codes = codes; a.dense = nullptr; a.step = 1.0f; a.step_dev = nullptr; a.W = W; a.W8 = nullptr; a.X = X; a.x_dtype = x_dtype;
    a.B = B; a.in = in; a.out = out; a.dX = dX; a.dW = dW; a.scratch = scratch; a.scratch_bytes = scratch_bytes;
    a.stats_job = StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr};
    return a;
}

ConvArgs conv_call(const float *W, const void *X, dbp_dtype x_dtype, int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R,
                   int64_t S, int64_t stride, int64_t pad, float *dX, void *dW, const int8_t *codes, char *scratch, size_t scratch_bytes,
                   bool two_planes)
{
    ConvArgs a;
    a.two_planes = two_planes;
    a.codes = codes; a.dense = nullptr; a.step = 1.0f; a.step_dev = nullptr; a.W = W; a.W8 = nullptr; a.X = X; a.x_dtype = x_dtype;
    a.N = N; a.C = C; a.H = H; a.Wd = Wd; a.K = K; a.R = R; a.S = S; a.pad = pad; a.stride = stride;
    a.dX = dX; a.dW = dW; a.scratch = scratch; a.scratch_bytes = scratch_bytes;
    a.stats_job = StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr}; a.pending = nullptr;
    return a;
}

}  // namespace

extern "C" {

uint32_t dbp_abi_version(void) { return DBP_ABI_VERSION; }

const char *dbp_status_string(dbp_status s)
{
    switch (s) {
    case DBP_OK: return "ok";
    case DBP_ERR_NULL: return "required pointer is NULL";
    case DBP_ERR_SHAPE: return "invalid or unsupported shape";
    case DBP_ERR_STEP: return "step size must be positive, finite and invertible in fp32";
    case DBP_ERR_DTYPE: return "unknown dtype";
    case DBP_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
    case DBP_ERR_UNSUPPORTED: return "not implemented in this build";
    case DBP_ERR_OVERFLOW: return "int32 weight gradient could overflow";
    case DBP_ERR_DEVICE: return "HIP error";
    }
    return "unknown status";
}

dbp_status dbp_format_layout_of(int64_t rows, int64_t cols, dbp_format_layout *layout)
{
    return format_layout(rows, cols, layout);
}

size_t dbp_linear_workspace_bytes(int64_t B, int64_t in, int64_t out, dbp_dtype x_dtype)
{
    if (check_linear_dims(B, in, out) != DBP_OK || (x_dtype != DBP_F32 && x_dtype != DBP_I8)) return 0;
    return carve(B, out, linear_scratch_bytes(B, in, out)).total;
}

size_t dbp_conv2d_workspace_bytes(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                  int64_t stride, int64_t pad, dbp_dtype x_dtype)
{
    int64_t P, Q;
    if (check_conv_dims(N, C, H, Wd, K, R, S, stride, pad, &P, &Q) != DBP_OK) return 0;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return 0;
    return carve(N * K, P * Q, conv_scratch_bytes(N, C, H, Wd, K, R, S, pad, stride)).total;
}

dbp_status nsd_quantize(const float *delta, int64_t rows, int64_t cols, float step, uint64_t seed, uint64_t idx_base,
                        int8_t *codes, void *format, size_t format_bytes, dbp_stats *stats, void *stream)
{
    if (!delta || !codes) return DBP_ERR_NULL;
    dbp_format_layout L;
    dbp_status st = format_layout(rows, cols, &L);
    if (st != DBP_OK) return st;
    if (!step_ok(step)) return DBP_ERR_STEP;
    if (format && (format_bytes < L.total_bytes || !aligned(format, 256))) return DBP_ERR_WORKSPACE;
    if (!aligned(delta, 4)) return DBP_ERR_SHAPE;
    return run_nsd(delta, rows, cols, step, seed, idx_base, codes, (char *)format, &L, stats, (hipStream_t)stream);
}

size_t dbp_topk_workspace_bytes(int64_t rows, int64_t vec_rows)
{
    if (rows <= 0 || vec_rows <= 0 || rows % vec_rows != 0) return 0;
    return align_up((size_t)(rows / vec_rows) * sizeof(uint32_t), 256);
}

dbp_status topk_quantize(const float *delta, int64_t rows, int64_t cols, int64_t vec_rows, int64_t k, float step, int8_t *codes,
                         void *format, size_t format_bytes, void *workspace, size_t workspace_bytes, dbp_stats *stats, void *stream)
{
    if (!delta || !codes) return DBP_ERR_NULL;
    dbp_format_layout L;
    dbp_status st = format_layout(rows, cols, &L);
    if (st != DBP_OK) return st;
    if (vec_rows <= 0 || rows % vec_rows != 0) return DBP_ERR_SHAPE;
    if (cols > (((int64_t)1 << 31) - 1) / vec_rows) return DBP_ERR_SHAPE;          // per-vector counts are 32-bit
    if (rows / vec_rows >= ((int64_t)1 << 31)) return DBP_ERR_SHAPE;                // one workgroup (or wavefront) per vector
    if (!step_ok(step)) return DBP_ERR_STEP;
    if (format && (format_bytes < L.total_bytes || !aligned(format, 256))) return DBP_ERR_WORKSPACE;
    if (!workspace || workspace_bytes < dbp_topk_workspace_bytes(rows, vec_rows) || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    if (!aligned(delta, 4)) return DBP_ERR_SHAPE;
    uint32_t *thr = (uint32_t *)workspace;
    if (launch_topk_threshold(delta, rows / vec_rows, vec_rows * cols, k, thr, (hipStream_t)stream) != hipSuccess) return DBP_ERR_DEVICE;
    return run_nsd(delta, rows, cols, step, 0, 0, codes, (char *)format, &L, stats, (hipStream_t)stream, true, nullptr, nullptr, false,
                   nullptr, thr, vec_rows);
}

dbp_status dbp_linear_products(const int8_t *codes, const void *format, float step, const float *W, const void *X,
                               dbp_dtype x_dtype, int64_t B, int64_t in, int64_t out, float *dX, void *dW,
                               void *workspace, size_t workspace_bytes, dbp_path path, void *stream)
{
    return linear_products(codes, format, step, W, X, x_dtype, B, in, out, dX, dW, workspace, workspace_bytes, path,
                           stream, StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr});
}

dbp_status dithered_linear_backward(const float *delta, const float *W, const void *X, dbp_dtype x_dtype,
                                    int64_t B, int64_t in, int64_t out, float step, uint64_t seed, uint64_t idx_base,
                                    int8_t *codes, float *dX, void *dW, void *workspace, size_t workspace_bytes,
                                    dbp_stats *stats, dbp_path path, void *stream)
{
    if (!delta || !W || (!dX && !dW) || (dW && !X)) return DBP_ERR_NULL;
    dbp_status st = check_linear_dims(B, in, out);
    if (st != DBP_OK) return st;
    if (!step_ok(step)) return DBP_ERR_STEP;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return DBP_ERR_DTYPE;
    if (!path_ok(path)) return DBP_ERR_UNSUPPORTED;
    if (x_dtype == DBP_I8 && dW && B * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    if (path_family(path) == DBP_PATH_GATHER && !linear_gather_supported(B, in, out)) return DBP_ERR_UNSUPPORTED;
    const Carve c = carve(B, out, linear_scratch_bytes(B, in, out));
    if (!workspace || workspace_bytes < c.total || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    if (!aligned(delta, 4)) return DBP_ERR_SHAPE;
    char *ws = (char *)workspace;
    int8_t *k = codes ? codes : (int8_t *)(ws + c.codes_offset);
    // only the gather kernels that serve odd shapes read the tile-sparse arrays; the statistics are summed by the
    // products' launch, or, with both families behind the density gate, by the kernel that writes the gate's flag
    const AutoPlan ap = path_family(path) == DBP_PATH_AUTO
        ? linear_auto_plan(linear_call(W, X, x_dtype, B, in, out, dX, dW, k, ws + c.scratch_offset, workspace_bytes - c.scratch_offset, path_two_planes(path)), true)
        : AutoPlan{false, 0};
    dbp_stats *st_dev = stats ? stats : ap.gated() ? (dbp_stats *)(ws + c.fmt.scratch_offset + kNsdFlagOffset + 64) : nullptr;
    StatsJob job;
    st = run_nsd(delta, B, out, step, seed, idx_base, k, ws, &c.fmt, st_dev, (hipStream_t)stream,
                 path_family(path) == DBP_PATH_GATHER, &job);
    if (st != DBP_OK) return st;
    return linear_products_dispatch(ap, k, ws, c, workspace_bytes - c.scratch_offset, step, W, X, x_dtype, B, in, out, dX, dW, path,
                                    stream, job, nullptr);
}

dbp_status dbp_conv2d_products(const int8_t *codes, const void *format, float step, const float *W, const void *X,
                               dbp_dtype x_dtype, int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K,
                               int64_t R, int64_t S, int64_t stride, int64_t pad, float *dX, void *dW,
                               void *workspace, size_t workspace_bytes, dbp_path path, void *stream)
{
    return conv2d_products(codes, format, step, W, X, x_dtype, N, C, H, Wd, K, R, S, stride, pad, dX, dW, workspace,
                           workspace_bytes, path, stream);
}

dbp_status dithered_conv2d_backward(const float *delta, const float *W, const void *X, dbp_dtype x_dtype,
                                    int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                    int64_t stride, int64_t pad, float step, uint64_t seed, uint64_t idx_base,
                                    int8_t *codes, float *dX, void *dW, void *workspace, size_t workspace_bytes,
                                    dbp_stats *stats, dbp_path path, void *stream)
{
    if (!delta || !W || (!dX && !dW) || (dW && !X)) return DBP_ERR_NULL;
    int64_t P, Q;
    dbp_status st = check_conv_dims(N, C, H, Wd, K, R, S, stride, pad, &P, &Q);
    if (st != DBP_OK) return st;
    if (!step_ok(step)) return DBP_ERR_STEP;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return DBP_ERR_DTYPE;
    if (!path_ok(path)) return DBP_ERR_UNSUPPORTED;
    if (path_family(path) == DBP_PATH_GATHER && !conv_gather_supported(N, C, H, Wd, K, R, S, P, Q, dX != nullptr)) return DBP_ERR_UNSUPPORTED;
    if (x_dtype == DBP_I8 && dW && N * P * Q * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    const Carve c = carve(N * K, P * Q, conv_scratch_bytes(N, C, H, Wd, K, R, S, pad, stride));
    if (!workspace || workspace_bytes < c.total || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    if (!aligned(delta, 4)) return DBP_ERR_SHAPE;
    char *ws = (char *)workspace;
    int8_t *k = codes ? codes : (int8_t *)(ws + c.codes_offset);
    const AutoPlan ap = path_family(path) == DBP_PATH_AUTO
        ? conv_auto_plan(conv_call(W, X, x_dtype, N, C, H, Wd, K, R, S, stride, pad, dX, dW, k, ws + c.scratch_offset,
                                   workspace_bytes - c.scratch_offset, path_two_planes(path)), P, Q)
        : AutoPlan{false, 0};
    dbp_stats *st_dev = stats ? stats : ap.gated() ? (dbp_stats *)(ws + c.fmt.scratch_offset + kNsdFlagOffset + 64) : nullptr;
    StatsJob job;
    st = run_nsd(delta, N * K, P * Q, step, seed, idx_base, k, ws, &c.fmt, st_dev, (hipStream_t)stream,
                 path_family(path) == DBP_PATH_GATHER || ap.dual, &job);
    if (st != DBP_OK) return st;
    return conv2d_products_dispatch(ap, k, ws, c, workspace_bytes - c.scratch_offset, step, W, X, x_dtype, N, C, H, Wd, K, R, S, stride,
                                    pad, dX, dW, path, stream, job, nullptr);
}

// ---- grouped convolution: the groups are independent layers on channel blocks of the same tensors, launched one after
// the other on the stream with the kernels of the ungrouped layer (which take the tensors' channel counts as strides)
namespace {

dbp_status check_groups(int64_t C, int64_t K, int64_t groups)
{
    if (groups < 1 || C % groups != 0 || K % groups != 0) return DBP_ERR_SHAPE;
    return DBP_OK;
}

// Groups of fewer than 64 input channels fill less than one 64-channel dW tile and half of a workgroup's 128 dX channels
// each, and every group costs its own launches: such layers run as ONE ungrouped layer with block-diagonal weights
// (measured on N=64, 256->256, 28x28, 3x3: 32 groups 1.74 ms group by group, 0.33 ms this way; 4 groups 0.24 ms group by
// group).  Scratch: the expanded weights and the ungrouped dW (K*C*R*S 4-byte elements each) before the layer's own.
bool grouped_as_block_diagonal(int64_t C, int64_t groups) { return groups > 1 && C / groups < 64; }
size_t block_diagonal_bytes(int64_t C, int64_t K, int64_t R, int64_t S) { return align_up((size_t)(K * C * R * S) * 4, 256); }

size_t grouped_scratch_bytes(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad,
                             int64_t groups)
{
    const size_t per_group = conv_scratch_bytes(N, C / groups, H, Wd, K / groups, R, S, pad, stride);
    if (!grouped_as_block_diagonal(C, groups)) return per_group;
    const size_t whole = 2 * block_diagonal_bytes(C, K, R, S) + conv_scratch_bytes(N, C, H, Wd, K, R, S, pad, stride);
    return whole > per_group ? whole : per_group;                  // the gather path and callers' sizing use one figure
}

dbp_status conv2d_products_grouped(const int8_t *codes, const void *format, float step, const float *W, const void *X, dbp_dtype x_dtype,
                                   int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad,
                                   int64_t groups, float *dX, void *dW, void *scratch, size_t scratch_bytes, dbp_path path, hipStream_t s,
                                   StatsJob job)
{
    int64_t P, Q;
    dbp_status st = check_conv_dims(N, C, H, Wd, K, R, S, stride, pad, &P, &Q);
    if (st != DBP_OK) return st;
    if ((st = check_groups(C, K, groups)) != DBP_OK) return st;
    const int64_t Cg = C / groups, Kg = K / groups, HW = H * Wd;
    const size_t xsz = x_dtype == DBP_I8 ? 1 : 4;
    if (launch_stats_job(job, s) != hipSuccess) return DBP_ERR_DEVICE;
    const bool gather = path_family(path) == DBP_PATH_GATHER;
    FormatView f{nullptr, nullptr, nullptr, 0};
    if (gather) {
        dbp_format_layout L;
        format_layout(N * K, P * Q, &L);
        const char *fb = (const char *)format;
        f = FormatView{(const uint64_t *)(fb + L.bitmap_offset), (const uint16_t *)(fb + L.tile_nnz_offset),
                       (const uint16_t *)(fb + L.entries_offset), L.tiles_per_row};
    }
    ConvArgs a;
    a.dense = nullptr; a.step = step; a.step_dev = nullptr; a.W8 = nullptr; a.x_dtype = x_dtype;
    a.N = N; a.C = Cg; a.H = H; a.Wd = Wd; a.K = Kg; a.R = R; a.S = S; a.pad = pad; a.stride = stride;
    a.Ct = C; a.Kt = K;
    const bool gather_ws = gather && scratch && aligned(scratch, 256);
    a.scratch = gather && !gather_ws ? nullptr : scratch; a.scratch_bytes = gather && !gather_ws ? 0 : scratch_bytes;
    a.stats_job = StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr}; a.pending = nullptr; a.gate = Gate{};
    a.two_planes = path_two_planes(path);
    if (!gather && grouped_as_block_diagonal(C, groups)) {
        const size_t bd = block_diagonal_bytes(C, K, R, S);
        float *w_full = (float *)scratch;
        void *dw_full = (char *)scratch + bd;
        if (launch_group_weights_expand(W, w_full, K, C, groups, R * S, s) != hipSuccess) return DBP_ERR_DEVICE;
        a.C = C; a.K = K; a.Ct = 0; a.Kt = 0;
        a.codes = codes; a.W = w_full; a.X = X; a.dX = dX; a.dW = dW ? dw_full : nullptr;
        a.scratch = (char *)scratch + 2 * bd; a.scratch_bytes = scratch_bytes - 2 * bd;
        if (launch_conv_mfma(a, s) != hipSuccess) return DBP_ERR_DEVICE;
        if (dW && launch_group_dw_extract(dw_full, dW, K, C, groups, R * S, s) != hipSuccess) return DBP_ERR_DEVICE;
        return DBP_OK;
    }
    if (!gather && dX && stride != 1 && groups > 1) {
        // output pixels that no tap reaches (a 1x1 kernel with stride 2 ...): the ungrouped launch clears its contiguous dX
        // itself, a group's block of channels is not contiguous, so the whole tensor is cleared once, here
        if (launch_zero_words(dX, N * C * HW, s) != hipSuccess) return DBP_ERR_DEVICE;
        a.dx_zeroed = true;
    }
    for (int64_t j = 0; j < groups; ++j) {
        a.codes = codes + j * Kg * P * Q;
        a.k_first = j * Kg;
        a.W = W + j * Kg * Cg * R * S;
        a.X = X ? (const char *)X + (size_t)(j * Cg * HW) * xsz : nullptr;
        a.dX = dX ? dX + j * Cg * HW : nullptr;
        a.dW = dW ? (char *)dW + (size_t)(j * Kg * Cg * R * S) * 4 : nullptr;           // fp32 and int32 alike
        const hipError_t e = gather ? launch_conv_gather(a, f, s) : launch_conv_mfma(a, s);
        if (e != hipSuccess) return DBP_ERR_DEVICE;
    }
    return DBP_OK;
}

dbp_status check_grouped_call(const void *W, const void *X, const float *dX, const void *dW, dbp_dtype x_dtype, int64_t N, int64_t C,
                              int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad, int64_t groups,
                              dbp_path path, int64_t *P, int64_t *Q)
{
    if (!W || (!dX && !dW) || (dW && !X)) return DBP_ERR_NULL;
    dbp_status st = check_conv_dims(N, C, H, Wd, K, R, S, stride, pad, P, Q);
    if (st != DBP_OK) return st;
    if ((st = check_groups(C, K, groups)) != DBP_OK) return st;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return DBP_ERR_DTYPE;
    if (!path_ok(path)) return DBP_ERR_UNSUPPORTED;
    // the gather kernels' limits, on the whole tensors (32-bit offsets into X, 16-bit plane numbers)
    if (path_family(path) == DBP_PATH_GATHER && !conv_gather_supported(N, C, H, Wd, K, R, S, *P, *Q, dX != nullptr)) return DBP_ERR_UNSUPPORTED;
    if (x_dtype == DBP_I8 && dW && N * *P * *Q * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    return DBP_OK;
}

}  // namespace

size_t dbp_conv2d_grouped_workspace_bytes(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                          int64_t stride, int64_t pad, int64_t groups, dbp_dtype x_dtype)
{
    int64_t P, Q;
    if (check_conv_dims(N, C, H, Wd, K, R, S, stride, pad, &P, &Q) != DBP_OK || check_groups(C, K, groups) != DBP_OK) return 0;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return 0;
    return carve(N * K, P * Q, grouped_scratch_bytes(N, C, H, Wd, K, R, S, stride, pad, groups)).total;
}

dbp_status dbp_conv2d_products_grouped(const int8_t *codes, const void *format, float step, const float *W, const void *X,
                                       dbp_dtype x_dtype, int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                       int64_t stride, int64_t pad, int64_t groups, float *dX, void *dW, void *workspace,
                                       size_t workspace_bytes, dbp_path path, void *stream)
{
    if (!codes) return DBP_ERR_NULL;
    int64_t P, Q;
    dbp_status st = check_grouped_call(W, X, dX, dW, x_dtype, N, C, H, Wd, K, R, S, stride, pad, groups, path, &P, &Q);
    if (st != DBP_OK) return st;
    if (!step_ok(step)) return DBP_ERR_STEP;
    if (path_family(path) == DBP_PATH_GATHER) {
        if (!format) return DBP_ERR_NULL;
        if (!aligned(format, 256)) return DBP_ERR_WORKSPACE;
    } else {
        const size_t need = grouped_scratch_bytes(N, C, H, Wd, K, R, S, stride, pad, groups);
        if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    }
    return conv2d_products_grouped(codes, format, step, W, X, x_dtype, N, C, H, Wd, K, R, S, stride, pad, groups, dX, dW, workspace,
                                   workspace_bytes, path, (hipStream_t)stream, StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr});
}

dbp_status dithered_conv2d_backward_grouped(const float *delta, const float *W, const void *X, dbp_dtype x_dtype, int64_t N, int64_t C,
                                            int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad,
                                            int64_t groups, float step, uint64_t seed, uint64_t idx_base, int8_t *codes, float *dX,
                                            void *dW, void *workspace, size_t workspace_bytes, dbp_stats *stats, dbp_path path,
                                            void *stream)
{
    if (!delta) return DBP_ERR_NULL;
    int64_t P, Q;
    dbp_status st = check_grouped_call(W, X, dX, dW, x_dtype, N, C, H, Wd, K, R, S, stride, pad, groups, path, &P, &Q);
    if (st != DBP_OK) return st;
    if (!step_ok(step)) return DBP_ERR_STEP;
    const Carve c = carve(N * K, P * Q, grouped_scratch_bytes(N, C, H, Wd, K, R, S, stride, pad, groups));
    if (!workspace || workspace_bytes < c.total || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    if (!aligned(delta, 4)) return DBP_ERR_SHAPE;
    char *ws = (char *)workspace;
    int8_t *k = codes ? codes : (int8_t *)(ws + c.codes_offset);
    StatsJob job;
    st = run_nsd(delta, N * K, P * Q, step, seed, idx_base, k, ws, &c.fmt, stats, (hipStream_t)stream, path_family(path) == DBP_PATH_GATHER, &job);
    if (st != DBP_OK) return st;
    return conv2d_products_grouped(k, ws, step, W, X, x_dtype, N, C, H, Wd, K, R, S, stride, pad, groups, dX, dW, ws + c.scratch_offset,
                                   workspace_bytes - c.scratch_offset, path, (hipStream_t)stream, job);
}

dbp_status dense_linear_backward(const void *delta, const float *W, const void *X, dbp_dtype x_dtype,
                                 int64_t B, int64_t in, int64_t out, float *dX, void *dW,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!delta || !W || (!dX && !dW) || (dW && !X)) return DBP_ERR_NULL;
    dbp_status st = check_linear_dims(B, in, out);
    if (st != DBP_OK) return st;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return DBP_ERR_DTYPE;
    if (x_dtype == DBP_I8 && dX) return DBP_ERR_UNSUPPORTED;          // int8 gradient with fp32 weights
    if (x_dtype == DBP_I8 && dW && B * 128 * 128 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    const size_t need = linear_scratch_bytes(B, in, out);
    if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    LinearArgs a;
    a.codes = nullptr; a.dense = delta; a.step = 1.0f; a.step_dev = nullptr; a.W = W; a.W8 = nullptr; a.X = X; a.x_dtype = x_dtype;
    a.B = B; a.in = in; a.out = out; a.dX = dX; a.dW = dW; a.scratch = workspace; a.scratch_bytes = workspace_bytes;
    a.stats_job = StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr};
    return launch_linear_mfma(a, (hipStream_t)stream) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
}

dbp_status dense_conv2d_backward(const void *delta, const float *W, const void *X, dbp_dtype x_dtype,
                                 int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                 int64_t stride, int64_t pad, float *dX, void *dW,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!delta || !W || (!dX && !dW) || (dW && !X)) return DBP_ERR_NULL;
    int64_t P, Q;
    dbp_status st = check_conv_dims(N, C, H, Wd, K, R, S, stride, pad, &P, &Q);
    if (st != DBP_OK) return st;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return DBP_ERR_DTYPE;
    if (x_dtype == DBP_I8 && dX) return DBP_ERR_UNSUPPORTED;
    if (x_dtype == DBP_I8 && dW && N * P * Q * 128 * 128 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    const size_t need = conv_scratch_bytes(N, C, H, Wd, K, R, S, pad, stride);
    if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    ConvArgs a;
    a.codes = nullptr; a.dense = delta; a.step = 1.0f; a.step_dev = nullptr; a.W = W; a.W8 = nullptr; a.X = X; a.x_dtype = x_dtype;
    a.N = N; a.C = C; a.H = H; a.Wd = Wd; a.K = K; a.R = R; a.S = S; a.pad = pad; a.stride = stride;
    a.dX = dX; a.dW = dW; a.scratch = workspace; a.scratch_bytes = workspace_bytes;
    a.stats_job = StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr}; a.pending = nullptr;
    return launch_conv_mfma(a, (hipStream_t)stream) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
}


// ---- Algorithm 1 on the device, and the steps around the quantiser ---------------------------------------

// ---- full 8-bit backward -------------------------------------------------------------------------------
size_t dbp_quantize_int8_workspace_bytes(int64_t n) { return n > 0 ? quantize_scratch_bytes(n) : 0; }

dbp_status dbp_quantize_int8(const float *x, int64_t n, int8_t *q, float *scale_out, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    if (!x || !q || !scale_out) return DBP_ERR_NULL;
    if (n <= 0) return DBP_ERR_SHAPE;
    if (!aligned(x, 4) || !aligned(scale_out, 8)) return DBP_ERR_SHAPE;
    if (!workspace || workspace_bytes < quantize_scratch_bytes(n) || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    return launch_quantize_int8(x, n, q, scale_out, workspace, (hipStream_t)stream) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
}

dbp_status dithered_linear_backward_q8(const float *delta, const int8_t *W8, const int8_t *X8,
                                       int64_t B, int64_t in, int64_t out, float step, uint64_t seed, uint64_t idx_base,
                                       int8_t *codes, int32_t *dX32, int32_t *dW32, void *workspace,
                                       size_t workspace_bytes, dbp_stats *stats, void *stream)
{
    if (!delta || (!dX32 && !dW32) || (dX32 && !W8) || (dW32 && !X8)) return DBP_ERR_NULL;
    dbp_status st = check_linear_dims(B, in, out);
    if (st != DBP_OK) return st;
    if (!step_ok(step)) return DBP_ERR_STEP;
    if (dX32 && out * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    if (dW32 && B * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    const Carve c = carve(B, out, linear_scratch_bytes(B, in, out));
    if (!workspace || workspace_bytes < c.total || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    if (!aligned(delta, 4)) return DBP_ERR_SHAPE;
    char *ws = (char *)workspace;
    int8_t *k = codes ? codes : (int8_t *)(ws + c.codes_offset);
    st = run_nsd(delta, B, out, step, seed, idx_base, k, ws, &c.fmt, stats, (hipStream_t)stream, false);
    if (st != DBP_OK) return st;
    LinearArgs a;
    a.codes = k; a.dense = nullptr; a.step = 1.0f; a.step_dev = nullptr; a.W = nullptr; a.W8 = W8 ? W8 : X8; a.X = X8;
    a.x_dtype = DBP_I8; a.B = B; a.in = in; a.out = out; a.dX = (float *)dX32; a.dW = dW32;
    a.scratch = ws + c.scratch_offset; a.scratch_bytes = workspace_bytes - c.scratch_offset;
    a.stats_job = StatsJob{nullptr, 0, nullptr, nullptr, 0, nullptr, 0.0f, nullptr};
    return launch_linear_mfma(a, (hipStream_t)stream) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
}

dbp_status dithered_conv2d_backward_q8(const float *delta, const int8_t *W8, const int8_t *X8,
                                       int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                       int64_t stride, int64_t pad, float step, uint64_t seed, uint64_t idx_base,
                                       int8_t *codes, int32_t *dX32, int32_t *dW32, void *workspace,
                                       size_t workspace_bytes, dbp_stats *stats, void *stream)
{
    if (!delta || (!dX32 && !dW32) || (dX32 && !W8) || (dW32 && !X8)) return DBP_ERR_NULL;
    int64_t P, Q;
    dbp_status st = check_conv_dims(N, C, H, Wd, K, R, S, stride, pad, &P, &Q);
    if (st != DBP_OK) return st;
    if (!step_ok(step)) return DBP_ERR_STEP;
    if (dX32 && K * R * S * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    if (dW32 && N * P * Q * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    const Carve c = carve(N * K, P * Q, conv_scratch_bytes(N, C, H, Wd, K, R, S, pad, stride));
    if (!workspace || workspace_bytes < c.total || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    if (!aligned(delta, 4)) return DBP_ERR_SHAPE;
    char *ws = (char *)workspace;
    int8_t *k = codes ? codes : (int8_t *)(ws + c.codes_offset);
    StatsJob job;
    st = run_nsd(delta, N * K, P * Q, step, seed, idx_base, k, ws, &c.fmt, stats, (hipStream_t)stream, false, &job);
    if (st != DBP_OK) return st;
    ConvArgs a;
    a.codes = k; a.dense = nullptr; a.step = 1.0f; a.step_dev = nullptr; a.W = nullptr; a.W8 = W8 ? W8 : X8; a.X = X8;
    a.x_dtype = DBP_I8; a.N = N; a.C = C; a.H = H; a.Wd = Wd; a.K = K; a.R = R; a.S = S; a.pad = pad; a.stride = stride;
    a.dX = (float *)dX32; a.dW = dW32; a.scratch = ws + c.scratch_offset; a.scratch_bytes = workspace_bytes - c.scratch_offset;
    a.stats_job = job; a.pending = nullptr;
    return launch_conv_mfma(a, (hipStream_t)stream) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
}

// ---- the entry point that allocates nothing ------------------------------------------------------------------------
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
hipError_t static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

dbp_status nsd_quantize_static(const float *delta, int64_t rows, int64_t cols, float step, uint64_t seed, uint64_t idx_base,
                               int8_t *codes, dbp_stats *stats, void *stream)
{
    if (!delta || !codes || !stats) return DBP_ERR_NULL;
    dbp_format_layout L;
    dbp_status st = format_layout(rows, cols, &L);
    if (st != DBP_OK) return st;
    if (rows * cols > DBP_STATIC_MAX_ELEMENTS) return DBP_ERR_SHAPE;
    if (!step_ok(step)) return DBP_ERR_STEP;
    if (!aligned(delta, 4)) return DBP_ERR_SHAPE;
    void *base = nullptr;
    if (static_scratch(&base) != hipSuccess) return DBP_ERR_DEVICE;
    // the records need no clearing: every workgroup of the quantiser overwrites its own, and the final sum reads exactly
    // those; run_nsd places them at L.scratch_offset of a format buffer, so hand it the address that puts them at `base`
    char *fmt_base = (char *)((uintptr_t)base - (uintptr_t)L.scratch_offset);        // never dereferenced below L.scratch_offset
    return run_nsd(delta, rows, cols, step, seed, idx_base, codes, fmt_base, &L, stats, (hipStream_t)stream, /*want_format=*/false);
}

size_t dbp_step_size_workspace_bytes(int64_t n)
{
    if (n <= 0 || n > kMaxElems) return 0;
    return step_size_scratch_bytes(n);
}

dbp_status dbp_step_size(const float *delta, const float *act, int64_t n, float s, float *step_out,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (!delta || !step_out) return DBP_ERR_NULL;
    if (n <= 0 || n > kMaxElems) return DBP_ERR_SHAPE;
    if (!(s > 0.0f) || !std::isfinite(s)) return DBP_ERR_STEP;
    if (!aligned(delta, 4) || (act && !aligned(act, 4)) || !aligned(step_out, 8)) return DBP_ERR_SHAPE;
    if (!workspace || workspace_bytes < step_size_scratch_bytes(n) || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    return launch_step_size(delta, act, n, s, step_out, workspace, (hipStream_t)stream) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
}

dbp_status nsd_quantize_ex(const float *delta, int64_t rows, int64_t cols, float step, uint64_t seed, uint64_t idx_base,
                           int8_t *codes, void *format, size_t format_bytes, dbp_stats *stats,
                           const dbp_nsd_extras *extras, void *stream)
{
    if (!delta || !codes) return DBP_ERR_NULL;
    dbp_format_layout L;
    dbp_status st = format_layout(rows, cols, &L);
    if (st != DBP_OK) return st;
    if (!(extras && extras->step_dev) && !step_ok(step)) return DBP_ERR_STEP;
    if (format && (format_bytes < L.total_bytes || !aligned(format, 256))) return DBP_ERR_WORKSPACE;
    if (!aligned(delta, 4)) return DBP_ERR_SHAPE;
    st = check_extras(extras, rows, cols);
    if (st != DBP_OK) return st;
    return run_nsd(delta, rows, cols, step, seed, idx_base, codes, (char *)format, &L, stats, (hipStream_t)stream, true,
                   nullptr, extras);
}

size_t dbp_linear_layer_workspace_bytes(int64_t B, int64_t in, int64_t out, dbp_dtype x_dtype)
{
    const size_t b = dbp_linear_workspace_bytes(B, in, out, x_dtype);
    return b ? layer_carve(b, B * out, out).total : 0;
}

size_t dbp_conv2d_layer_workspace_bytes(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                        int64_t stride, int64_t pad, dbp_dtype x_dtype)
{
    const size_t b = dbp_conv2d_workspace_bytes(N, C, H, Wd, K, R, S, stride, pad, x_dtype);
    if (!b) return 0;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    return layer_carve(b, N * K * P * Q, K).total;
}

dbp_status dithered_linear_layer_backward(const float *delta_a, const float *act, const float *W, const void *X,
                                          dbp_dtype x_dtype, int64_t B, int64_t in, int64_t out, float s,
                                          uint64_t seed, uint64_t idx_base, int8_t *codes, float *dX, void *dW,
                                          float *db, float *step_out, void *workspace, size_t workspace_bytes,
                                          dbp_stats *stats, dbp_path path, void *stream)
{
    if (!delta_a || !W || (!dX && !dW && !db) || (dW && !X)) return DBP_ERR_NULL;
    dbp_status st = check_linear_dims(B, in, out);
    if (st != DBP_OK) return st;
    if (!(s > 0.0f) || !std::isfinite(s)) return DBP_ERR_STEP;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return DBP_ERR_DTYPE;
    if (!path_ok(path)) return DBP_ERR_UNSUPPORTED;
    if (x_dtype == DBP_I8 && dW && B * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    if (path_family(path) == DBP_PATH_GATHER && !linear_gather_supported(B, in, out)) return DBP_ERR_UNSUPPORTED;
    const Carve c = carve(B, out, linear_scratch_bytes(B, in, out));
    const LayerCarve lc = layer_carve(c.total, B * out, out);
    if (!workspace || workspace_bytes < lc.total || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    if (!aligned(delta_a, 4) || (act && !aligned(act, 4)) || (step_out && !aligned(step_out, 8))) return DBP_ERR_SHAPE;
    char *ws = (char *)workspace;
    hipStream_t hs = (hipStream_t)stream;
    float *pair = step_out ? step_out : (float *)(ws + lc.step_pair);
    StepTree tree;
    if (launch_step_size(delta_a, act, B * out, s, pair, ws + lc.step_scratch, hs,
                         db ? (int64_t *)(ws + lc.bias_sums) : nullptr, db ? out : 0, &tree) != hipSuccess) return DBP_ERR_DEVICE;
    dbp_nsd_extras ex;
    ex.act = act; ex.step_dev = pair; ex.bias_sums = db ? (int64_t *)(ws + lc.bias_sums) : nullptr; ex.bias_grad = db;
    ex.bias_mode = DBP_BIAS_PER_COLUMN; ex.bias_len = out;
    int8_t *k = codes ? codes : (int8_t *)(ws + c.codes_offset);
    StatsJob job;
    const AutoPlan ap = path_family(path) == DBP_PATH_AUTO && (dX || dW)
        ? linear_auto_plan(linear_call(W, X, x_dtype, B, in, out, dX, dW, k, ws + c.scratch_offset, c.total - c.scratch_offset, path_two_planes(path)), true)
        : AutoPlan{false, 0};
    dbp_stats *st_dev = stats ? stats : ap.gated() ? (dbp_stats *)(ws + c.fmt.scratch_offset + kNsdFlagOffset + 64) : nullptr;
    st = run_nsd(delta_a, B, out, 1.0f, seed, idx_base, k, ws, &c.fmt, st_dev, hs, path_family(path) == DBP_PATH_GATHER, &job, &ex, true, &tree);
    if (st != DBP_OK) return st;
    if (!dX && !dW) return launch_stats_job(job, hs) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
    return linear_products_dispatch(ap, k, ws, c, c.total - c.scratch_offset, 1.0f, W, X, x_dtype, B, in, out, dX, dW, path, stream, job, pair);
}

dbp_status dithered_conv2d_layer_backward(const float *delta_a, const float *act, const float *W, const void *X,
                                          dbp_dtype x_dtype, int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K,
                                          int64_t R, int64_t S, int64_t stride, int64_t pad, float s, uint64_t seed,
                                          uint64_t idx_base, int8_t *codes, float *dX, void *dW, float *db,
                                          float *step_out, void *workspace, size_t workspace_bytes, dbp_stats *stats,
                                          dbp_path path, void *stream)
{
    if (!delta_a || !W || (!dX && !dW && !db) || (dW && !X)) return DBP_ERR_NULL;
    int64_t P, Q;
    dbp_status st = check_conv_dims(N, C, H, Wd, K, R, S, stride, pad, &P, &Q);
    if (st != DBP_OK) return st;
    if (!(s > 0.0f) || !std::isfinite(s)) return DBP_ERR_STEP;
    if (x_dtype != DBP_F32 && x_dtype != DBP_I8) return DBP_ERR_DTYPE;
    if (!path_ok(path)) return DBP_ERR_UNSUPPORTED;
    if (path_family(path) == DBP_PATH_GATHER && !conv_gather_supported(N, C, H, Wd, K, R, S, P, Q, dX != nullptr)) return DBP_ERR_UNSUPPORTED;
    if (x_dtype == DBP_I8 && dW && N * P * Q * 127 * 127 >= ((int64_t)1 << 31)) return DBP_ERR_OVERFLOW;
    const Carve c = carve(N * K, P * Q, conv_scratch_bytes(N, C, H, Wd, K, R, S, pad, stride));
    const LayerCarve lc = layer_carve(c.total, N * K * P * Q, K);
    if (!workspace || workspace_bytes < lc.total || !aligned(workspace, 256)) return DBP_ERR_WORKSPACE;
    if (!aligned(delta_a, 4) || (act && !aligned(act, 4)) || (step_out && !aligned(step_out, 8))) return DBP_ERR_SHAPE;
    char *ws = (char *)workspace;
    hipStream_t hs = (hipStream_t)stream;
    float *pair = step_out ? step_out : (float *)(ws + lc.step_pair);
    StepTree tree;
    if (launch_step_size(delta_a, act, N * K * P * Q, s, pair, ws + lc.step_scratch, hs,
                         db ? (int64_t *)(ws + lc.bias_sums) : nullptr, db ? K : 0, &tree) != hipSuccess) return DBP_ERR_DEVICE;
    dbp_nsd_extras ex;
    ex.act = act; ex.step_dev = pair; ex.bias_sums = db ? (int64_t *)(ws + lc.bias_sums) : nullptr; ex.bias_grad = db;
    ex.bias_mode = DBP_BIAS_PER_ROW_GROUP; ex.bias_len = K;
    int8_t *k = codes ? codes : (int8_t *)(ws + c.codes_offset);
    StatsJob job;
    const AutoPlan ap = path_family(path) == DBP_PATH_AUTO && (dX || dW)
        ? conv_auto_plan(conv_call(W, X, x_dtype, N, C, H, Wd, K, R, S, stride, pad, dX, dW, k, ws + c.scratch_offset,
                                   c.total - c.scratch_offset, path_two_planes(path)), P, Q)
        : AutoPlan{false, 0};
    dbp_stats *st_dev = stats ? stats : ap.gated() ? (dbp_stats *)(ws + c.fmt.scratch_offset + kNsdFlagOffset + 64) : nullptr;
    st = run_nsd(delta_a, N * K, P * Q, 1.0f, seed, idx_base, k, ws, &c.fmt, st_dev, hs, path_family(path) == DBP_PATH_GATHER || ap.dual, &job, &ex,
                 true, &tree);
    if (st != DBP_OK) return st;
    if (!dX && !dW) return launch_stats_job(job, hs) == hipSuccess ? DBP_OK : DBP_ERR_DEVICE;
    return conv2d_products_dispatch(ap, k, ws, c, c.total - c.scratch_offset, 1.0f, W, X, x_dtype, N, C, H, Wd, K, R, S, stride, pad, dX, dW,
                                    path, stream, job, pair);
}

// The density dispatch a DBP_PATH_AUTO convolution call would set up, from the host's cost models alone (no GPU call).
int dbp_plan_auto_conv2d(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad,
                         int int8_x, int want_dx, int want_dw, int two_planes, uint64_t *gather_below, uint64_t *dw_rows_below)
{
    int64_t P, Q;
    if (check_conv_dims(N, C, H, Wd, K, R, S, stride, pad, &P, &Q) != DBP_OK || (!want_dx && !want_dw)) return -1;
    // stand-ins for the tensors: the planners look at alignment and at which outputs are asked for, and touch nothing
    char *fake = (char *)(uintptr_t)4096;
    const ConvArgs call = conv_call((const float *)fake, fake, int8_x ? DBP_I8 : DBP_F32, N, C, H, Wd, K, R, S, stride, pad,
                                    want_dx ? (float *)fake : nullptr, want_dw ? fake : nullptr, (const int8_t *)fake, fake,
                                    conv_scratch_bytes(N, C, H, Wd, K, R, S, pad, stride), two_planes != 0);
    const AutoPlan ap = conv_auto_plan(call, P, Q);
    if (gather_below) *gather_below = ap.dual ? ap.gather_below : 0;
    if (dw_rows_below) *dw_rows_below = ap.dw_rows_below;
    return ap.dual ? 1 : ap.dw_rows_below ? 2 : 0;
}

// The same for dithered_linear_backward: 0 = matrix cores, no gate; 1 = the gather family below *gather_below nonzero codes.
int dbp_plan_auto_linear(int64_t B, int64_t in, int64_t out, int int8_x, int want_dx, int want_dw, int two_planes, uint64_t *gather_below)
{
    if (check_linear_dims(B, in, out) != DBP_OK || (!want_dx && !want_dw)) return -1;
    char *fake = (char *)(uintptr_t)4096;
    const LinearArgs call = linear_call((const float *)fake, fake, int8_x ? DBP_I8 : DBP_F32, B, in, out, want_dx ? (float *)fake : nullptr,
                                        want_dw ? fake : nullptr, (const int8_t *)fake, fake, linear_scratch_bytes(B, in, out), two_planes != 0);
    const AutoPlan ap = linear_auto_plan(call, true);
    if (gather_below) *gather_below = ap.dual ? ap.gather_below : 0;
    return ap.dual ? 1 : 0;
}

}  // extern "C"
