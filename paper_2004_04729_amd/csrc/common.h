// Shared declarations of the gfx950 dithered-backprop library (internal; the public C ABI is include/dbp.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "dbp.h"

namespace dbp {

typedef float    f32x4  __attribute__((ext_vector_type(4)));
typedef float    f32x16 __attribute__((ext_vector_type(16)));
typedef int32_t  i32x4  __attribute__((ext_vector_type(4)));
typedef int32_t  i32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4  __attribute__((ext_vector_type(4)));
typedef __bf16   bf16x8 __attribute__((ext_vector_type(8)));

// A product's output scale: a host value, or (Algorithm 1 on the device) the Delta an earlier kernel of the
// same stream left in device memory.
struct Scale {
    float host; const float *dev;
    __device__ __forceinline__ float get() const { return dev ? dev[0] : host; }
};

// Device-side dispatch between the kernel families (matrix cores / gather): a gated kernel runs only when the flag an
// earlier kernel of the stream wrote equals `want`; flag == nullptr: always.
struct Gate {
    const int *flag = nullptr; int want = 0;
    __device__ __forceinline__ bool closed() const { return flag && flag[0] != want; }
};

constexpr int kWave = 64;
constexpr int kNsdMaxBlocks = 16384;                                 // measured best on 2^28 elements (8 resident per CU)
constexpr size_t kNsdFlagOffset = (size_t)kNsdMaxBlocks * 16;        // the density flag follows the statistics records
constexpr size_t kNsdScratchBytes = kNsdFlagOffset + 256;            // one 16-byte statistics record per workgroup, then the flag

// Dither keys derived from the 64-bit seed on the host (constants: golden ratio, frac sqrt2, frac sqrt3).
struct DitherKeys { uint32_t k0, k1; };
DitherKeys make_dither_keys(uint64_t seed);

// A step-size tree that launch_step_size left unfinished (at most 256 partial sums): the quantiser's workgroups add the
// last levels themselves, in the tree's order, and its first workgroup writes {Delta, 1/Delta}.  count == 0: none.
struct StepTree { const double *s1, *s2; int count; int64_t n; float s; float *step_out; };

struct NsdArgs {
    const float *delta;
    int8_t      *codes;
    uint64_t    *bitmap;      // nullable (codes only)
    uint16_t    *tile_nnz;
    uint16_t    *entries;
    dbp_stats   *stats;       // nullable
    u32x4       *partials;    // per-workgroup {nnz, saturated, nonfinite, max|k|} (kNsdMaxBlocks records) or nullptr -> atomics
    int64_t      rows, cols, tiles_per_row, n_tiles;
    float        inv_step;
    uint32_t     k0, k1;
    uint64_t     idx_base;
    // ---- extensions around the quantiser (nsd_kernel<.., .., true>); all optional
    const float *act;         // delta_z = delta_a where act > 0, else 0 (rectifier derivative), same shape as delta
    const float *step_dev;    // device {Delta, 1/Delta} (from launch_step_size) instead of inv_step
    int64_t     *bias_sums;   // int64 code sums, zeroed by launch_nsd; bias_mode 0: per column, 1: per (row % bias_len)
    float       *bias_grad;   // Delta * sums, fp32 (nullable)
    int          bias_mode;
    int64_t      bias_len;
    float        step;        // host Delta (bias_grad without step_dev)
    int          bias_zeroed; // bias_sums were cleared by an earlier kernel of the stream (launch_step_size)
    StepTree     tree;        // unfinished step size (then step_dev is what the kernel writes, not what it reads)
    int          run;                                  // consecutive tiles per wavefront run (set by launch_nsd)
    // ---- top-k sparsifier (nsd_kernel<.., .., false, true>): no dither, elements below their vector's threshold are dropped
    const uint32_t *topk_thr = nullptr;                // per vector: smallest magnitude bit pattern that survives
    int64_t      topk_vec_rows = 1;                    // a vector = this many consecutive rows
    int64_t      wave_stride_rows, wave_stride_segs;   // grid stride in tiles = rows*tiles_per_row + segs (set by launch_nsd)
};
// Pending reduction of the per-workgroup statistics records into one dbp_stats (n == 0: nothing pending).
struct StatsJob {
    const u32x4 *partials; int n; dbp_stats *out;                  // statistics records -> dbp_stats (n == 0: none)
    const int64_t *bias_sums; int64_t bias_len; float *bias_grad;   // code sums -> fp32 bias gradient (bias_len == 0: none)
    float step; const float *step_dev;
    // density dispatch (write_density_flags): three flags, exactly one of them 1 -- flag[0]: fewer than gather_below codes
    // are nonzero (the gather family runs); flag[1]: not that, but fewer than dw_rows_below (matrix cores for dX, the
    // plane-scanning gather kernel for dW); flag[2]: neither (matrix cores for both)
    int *flag = nullptr; uint64_t gather_below = 0, dw_rows_below = 0;
};
__device__ __forceinline__ void write_density_flags(const StatsJob &j, uint64_t nnz)
{
    if (!j.flag) return;
    const int state = nnz < j.gather_below ? 0 : nnz < j.dw_rows_below ? 1 : 2;
    j.flag[0] = state == 0; j.flag[1] = state == 1; j.flag[2] = state == 2;
}
// Launches the quantiser.  With `defer` non-null and statistics kept in records, the final sum is not
// launched: *defer describes it, and the caller either folds it into a later kernel of the same stream
// or calls launch_stats_job.
hipError_t launch_nsd(const NsdArgs &a, hipStream_t s, StatsJob *defer = nullptr);
hipError_t launch_stats_job(const StatsJob &j, hipStream_t s);
// Top-k sparsifier, first half: thr[v] = bit pattern of the k-th largest magnitude of vector v (n_vec vectors of len
// consecutive elements, len < 2^31); the quantiser (launch_nsd with NsdArgs::topk_thr) keeps what reaches it.
hipError_t launch_topk_threshold(const float *delta, int64_t n_vec, int64_t len, int64_t k, uint32_t *thr, hipStream_t s);

// Step size of Algorithm 1 on the device: step_out = {Delta = s*std(delta_z), 1/Delta}, delta_z = delta masked by act > 0
// when act is given (both 0 if the standard
// deviation is 0 or not finite).  scratch: step_size_scratch_bytes(n).
size_t     step_size_scratch_bytes(int64_t n);
// symmetric int8 quantiser of the forward pass (nsd.hip)
size_t     quantize_scratch_bytes(int64_t n);
hipError_t launch_quantize_int8(const float *x, int64_t n, int8_t *q, float *scale_out, void *scratch, hipStream_t st);
hipError_t launch_step_size(const float *delta, const float *act, int64_t n, float s, float *step_out, void *scratch, hipStream_t st,
                            int64_t *zero = nullptr, int64_t zero_len = 0,    // also clears zero[0..zero_len)
                            StepTree *defer = nullptr);   // non-null: small trees are left to the quantiser (defer->count > 0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace dbp

namespace dbp {

// ---- products (products.hip) -----------------------------------------------------------------
struct LinearArgs {
    const int8_t *codes;       // dithered path: int8 codes [B,out]
    const void   *dense;       // dense baseline: fp32 (or int8 in 8-bit mode) gradient [B,out]
    float         step;        // Delta (dithered); ignored for dense
    const float  *step_dev;    // device {Delta, 1/Delta} instead of `step` (nullable)
    const float  *W;           // [out,in]
    const int8_t *W8;          // full 8-bit mode: int8 weights [out,in] instead of W; dX is then exact int32 (nullable)
    const void   *X;           // [B,in] fp32 or int8
    dbp_dtype     x_dtype;
    int64_t       B, in, out;
    float        *dX;          // nullable
    void         *dW;          // nullable
    void         *scratch;     // split-K partials
    size_t        scratch_bytes;
    StatsJob      stats_job;   // statistics sum still to be done on this stream (n == 0: none)
    Gate          gate;        // device-side dispatch (fast kernels only)
    int          *plan_only = nullptr;   // non-null: launch nothing, set *plan_only = 1 if some product would run on an ungated kernel
    bool          two_planes = false;    // fp32 operands of the matrix-core kernels in two bf16 planes instead of three (DBP_PATH_TWO_PLANES)
};
struct ConvArgs {
    const int8_t *codes;
    const void   *dense;
    float         step;
    const float  *step_dev;
    const float  *W;           // [K,C,R,S]
    const int8_t *W8;          // full 8-bit mode: int8 weights instead of W; dX is then exact int32 (nullable)
    const void   *X;           // [N,C,H,Wd]
    dbp_dtype     x_dtype;
    int64_t       N, C, H, Wd, K, R, S, pad, stride;
    // One group of a grouped convolution: X/dX and the codes are channel blocks of tensors with Ct resp. Kt channels
    // (image n of X starts n*Ct*H*Wd elements in; 0 = C resp. K: an ordinary layer); W and dW are the group's own block.
    int64_t       Ct = 0, Kt = 0;
    int64_t       k_first = 0;         // first code plane of the group inside an image's Kt planes (what the gather kernels' format rows need)
    bool          dx_zeroed = false;   // dX is already cleared (the strided dX kernels then skip their own clearing pass)
    bool          two_planes = false;  // fp32 operands of the matrix-core kernels in two bf16 planes instead of three (DBP_PATH_TWO_PLANES)
    int64_t ct() const { return Ct ? Ct : C; }
    int64_t kt() const { return Kt ? Kt : K; }
    float        *dX;
    void         *dW;
    void         *scratch;
    size_t        scratch_bytes;
    StatsJob      stats_job;   // statistics sum / bias gradient still to be done on this stream (none: n == 0 and bias_len == 0)
    StatsJob     *pending;     // set by launch_conv_mfma: what of stats_job no kernel has taken along yet
    Gate          gate;        // device-side dispatch (the large kernels; the small preparation kernels run regardless)
    Gate          gate_dw;     // matrix-core family: the dW kernels' gate where it differs from the dX kernels' (flag == nullptr: `gate` serves both)
    bool          rows_gated = false;    // gather family: the plane-scanning kernels also behind a gate (else a gated call takes the entry-walking kernels)
    int          *plan_only = nullptr;   // non-null: launch nothing, set *plan_only = 1 if a large kernel would run ungated
};
size_t     linear_scratch_bytes(int64_t B, int64_t in, int64_t out);
size_t     conv_scratch_bytes(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t pad, int64_t stride = 1);
hipError_t launch_linear_mfma(const LinearArgs &a, hipStream_t s);
hipError_t launch_conv_mfma(const ConvArgs &a, hipStream_t s);
hipError_t launch_zero_words(void *p, int64_t n_words, hipStream_t s);      // clears n 4-byte words
// grouped convolution as one ungrouped layer: block-diagonal weights in, diagonal blocks of dW out (products.hip)
hipError_t launch_group_weights_expand(const float *W, float *full, int64_t K, int64_t C, int64_t groups, int64_t RS, hipStream_t s);
hipError_t launch_group_dw_extract(const void *full, void *dW, int64_t K, int64_t C, int64_t groups, int64_t RS, hipStream_t s);

// ---- gather path (gather.hip) ------------------------------------------------------------------
struct FormatView { const uint64_t *bitmap; const uint16_t *tile_nnz; const uint16_t *entries; int64_t tiles_per_row; };
// flag != nullptr: device-side dispatch, the kernels run only when *flag == flag_want (fc_rows_kernel shapes only).
hipError_t launch_linear_gather(const LinearArgs &a, const FormatView &f, hipStream_t s);   // a.gate: fc_rows_kernel shapes only
bool       linear_gather_gated_ok(const LinearArgs &a);     // every requested product runs on the gated fc_rows_kernel
// Launch shape of fc_rows_kernel for dX ([0]) and dW ([1]): what the density dispatch's cost model needs.
struct GatherShape { int64_t workgroups, steps; size_t partial_bytes; };
void       linear_gather_shape(int64_t B, int64_t in, int64_t out, GatherShape (&gs)[2]);
size_t     linear_gather_scratch_bytes(int64_t B, int64_t in, int64_t out);    // split partials of the gather dX kernel
bool       linear_gather_supported(int64_t B, int64_t in, int64_t out);
// Convolution gather kernels: any stride; kernels of at most 64 taps, output planes below 4096 x 4096, and for dX an input
// plane of at most about 37 KiB (four of them accumulate in LDS).
bool       conv_gather_supported(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t P, int64_t Q, bool want_dx);
hipError_t launch_conv_gather(const ConvArgs &a, const FormatView &f, hipStream_t s);     // honours a.gate
// Cost model of conv_dw_rows_kernel on this layer with `avail` bytes of scratch (microseconds; constants measured on MI355X):
// false when the kernel does not take the shape.
bool       conv_dw_rows_cost(const ConvArgs &a, int64_t P, int64_t Q, size_t avail, double *fixed_us, double *per_nnz_us);


}  // namespace dbp
