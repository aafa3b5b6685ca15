/*
 * dbp.h -- C ABI of the MI355X (gfx950) dithered-backprop library.
 *
 * Method: Wiedemann, Mehari, Kepp, Samek, "Dithered backprop: a sparse and quantized
 * backpropagation algorithm for more efficient deep neural network training"
 * (arXiv 2004.04729).  The library implements the per-layer backward hot path:
 *
 *   1. NSD quantisation of the preactivation gradient delta_z        (Eq. (nsd), Eq. (qdz))
 *          k = floor(delta/Delta + u),  u = nu/Delta + 1/2,  nu ~ U(-Delta/2, Delta/2) open
 *          quantised gradient q = k * Delta, kept as int8 codes k plus a tile-sparse format
 *   2. the two backward products that consume q                      (Eqs. (qda), (qdw))
 *          delta_a = W^T . q        delta_W = q . a^T
 *      for fully connected layers and, "analogously" (Sec. "Dithered backpropagation"),
 *      for 2-D convolutions lowered to an implicit-im2col GEMM
 *   3. the 8-bit mode of Sec. "Quantizing forward pass": int8 activations, int8 codes,
 *      weight gradient accumulated exactly in int32.
 *
 * Conventions that hold for EVERY entry point
 *   - All tensor pointers are DEVICE pointers (HBM) unless a comment says "host".
 *     The caller owns every buffer; the library never allocates, frees or synchronises.
 *     Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default stream).
 *   - Tensors are dense, contiguous, row-major: FC  delta/codes [B,out], W [out,in],
 *     X [B,in], dX [B,in], dW [out,in];  conv  delta/codes [N,K,P,Q], W [K,C,R,S],
 *     X [N,C,H,Wd], dX [N,C,H,Wd], dW [K,C,R,S]  (P = (H+2pad-R)/stride+1, likewise Q).
 *     With W stored [out,in] the paper's W^T.q is  dX[b,i] = sum_o q[b,o] W[o,i]  and
 *     q.a^T is  dW[o,i] = sum_b q[b,o] X[b,i]  (no 1/B factor).
 *   - Outputs are overwritten (beta = 0).  fp32 outputs are in real units (Delta applied);
 *     the int32 weight gradient is the raw sum  k * x8  (the caller scales it).
 *   - Arguments are validated on the host BEFORE any HIP call, so every status except
 *     DBP_ERR_DEVICE can be produced on a machine without a GPU.  Nothing aborts or throws.
 *   - `workspace` is device scratch of at least the size the matching *_workspace_bytes
 *     function returns, 256-byte aligned.  Its contents need not be initialised and are
 *     undefined afterwards, except that the dithered_* calls with path == DBP_PATH_GATHER
 *     leave the tile-sparse format (see below) at the start of the workspace.  The matrix-core
 *     kernels and the fully connected gather kernels read the code plane, not that format, and no
 *     bandwidth is spent writing it for them; nsd_quantize produces it on request.
 *   - The dither of element j of delta is a pure function of (seed, idx_base + j), where j is
 *     the row-major flat index; a shard of a larger tensor passes its offset as idx_base and
 *     obtains bit-identical codes.
 */
#ifndef DBP_H_
#define DBP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DBP_ABI_VERSION 1u
#define DBP_TILE 256                     /* columns per tile of the tile-sparse format */

typedef enum {
    DBP_OK = 0,
    DBP_ERR_NULL = 1,          /* a required pointer is NULL                                   */
    DBP_ERR_SHAPE = 2,         /* a dimension is <= 0, too large, or inconsistent              */
    DBP_ERR_STEP = 3,          /* Delta is <= 0, NaN, Inf, or 1/Delta is not finite            */
    DBP_ERR_DTYPE = 4,         /* unknown dbp_dtype                                            */
    DBP_ERR_WORKSPACE = 5,     /* workspace NULL/too small/misaligned                          */
    DBP_ERR_UNSUPPORTED = 6,   /* valid request this build does not implement (e.g. dilation)   */
    DBP_ERR_OVERFLOW = 7,      /* int32 weight gradient could overflow: reduction*127*127>=2^31 */
    DBP_ERR_DEVICE = 8         /* a HIP call failed (launch error, wrong device, ...)          */
} dbp_status;

typedef enum { DBP_F32 = 0, DBP_I8 = 1 } dbp_dtype;

/* Which kernels compute the two products.
 *   MFMA    the codes as exact bf16 (or int8) operands of matrix-core tiles: dense work, the same at any sparsity (only the
 *           generic kernel that serves odd shapes skips all-zero code fragments).
 *   GATHER  kernels that walk the nonzero codes: work in proportion to the nonzeros (Sec. "Computational complexity",
 *           O(p_nz m k n)) plus the fixed cost of streaming the dense operand and writing the outputs.
 *   AUTO    matrix cores, unless the shape is one where gather kernels can win by a wide margin at high sparsity; then
 *           BOTH candidates are launched behind a gate and the device decides: the kernel that sums the quantiser's statistics
 *           compares the nonzero count with a threshold (a linear cost model with constants measured on MI355X) and writes
 *           flags; the kernels the flags do not name return at once.  No host round trip, no allocation.  A layer has at most
 *           one alternative to "everything on matrix cores": 3x3 convolutions with fp32 activations and 128 channels or
 *           more the gather kernel for dW alone (dX stays on matrix cores; it wins from ~97 % zeros); fully connected layers
 *           and other small-plane convolutions the whole gather family (beyond ~98.5-99.8 % zeros).
 *           Results are those of whichever kernels ran (all meet the same tolerance; each is deterministic). */
typedef enum {
    DBP_PATH_AUTO = 0,
    DBP_PATH_MFMA = 1,
    DBP_PATH_GATHER = 2,
    /* A flag, OR-ed onto one of the three above.  The matrix-core kernels multiply the integer codes with the fp32 operand (W for dX,
     * X for dW) cut into bf16 planes.  By default three planes that add up to the operand exactly, so the only rounding is the fp32
     * accumulation.  With this flag the kernels that support it (the rest ignore it) cut the operand into TWO planes, rounded to
     * nearest: the operand then carries 16 significant bits, |w - hi - lo| <= 2^-16 |w|, and an output differs from the three-plane
     * one by at most 2^-16 * sum_r |q_r| |w_r| over its own reduction (1.5e-5, against the 1e-4 this library's results are held to;
     * the dither of Eq. (nsd) itself moves every term by up to Delta) for two thirds of the matrix-core work.  The int8 products
     * (x_dtype == DBP_I8 dW, the *_q8 calls) and the gather kernels have no planes and are unchanged. */
    DBP_PATH_TWO_PLANES = 0x100
} dbp_path;

/* Per-call statistics, device resident (the paper's reported quantities: sparsity and the
 * width of the non-zero codes, Sec. "Accuracy & Induced Sparsity").  Written by the NSD pass. */
typedef struct {
    uint64_t nnz;              /* codes != 0                                                   */
    uint64_t n_saturated;      /* |floor(t)| > 127 before clamping to [-127,127] (incl. +-Inf) */
    uint64_t n_nonfinite;      /* inputs that were NaN or +-Inf (NaN quantises to code 0)      */
    int32_t  max_abs_code;     /* max |k| after clamping                                       */
    int32_t  reserved;
} dbp_stats;

/*
 * Tile-sparse format written by the NSD pass (this library's design; the paper asks only for
 * "sparse tensors with low precision non-zero values").  The code plane [rows x cols] is cut,
 * row by row, into tiles of DBP_TILE consecutive columns (a row's last tile may be short):
 * tiles_per_row = ceil(cols/256), tile t = row*tiles_per_row + col/256.  Per tile
 *   bitmap  [4t + j]     uint64, j = 0..3: bit l set <=> code at in-tile column 4l+j is nonzero
 *                        (column c is bit c/4 of word c%4: the wavefront ballots of the NSD kernel)
 *   tile_nnz[t]          uint16: number of nonzero codes of the tile
 *   entries [256t + i]   uint16, i < tile_nnz[t]: (in-tile column << 8) | (code & 0xFF),
 *                        columns ascending; the contents of later slots are undefined.
 * All three arrays live in one caller-provided buffer at the byte offsets given here.
 */
typedef struct {
    int64_t tiles_per_row;
    int64_t n_tiles;
    size_t  bitmap_offset;     /* uint64[4*n_tiles]  */
    size_t  tile_nnz_offset;   /* uint16[n_tiles]    */
    size_t  entries_offset;    /* uint16[256*n_tiles]*/
    size_t  scratch_offset;    /* 256 KiB used by the NSD pass itself (per-workgroup statistics) */
    size_t  total_bytes;
} dbp_format_layout;

uint32_t    dbp_abi_version(void);
const char *dbp_status_string(dbp_status s);

/* Layout/size of the tile-sparse format for a [rows x cols] code plane (host computation). */
dbp_status  dbp_format_layout_of(int64_t rows, int64_t cols, dbp_format_layout *layout /*host*/);

/* Bytes of workspace the backward entry points need (format + partial sums + staging);
 * 0 on invalid arguments. */
size_t dbp_linear_workspace_bytes(int64_t B, int64_t in, int64_t out, dbp_dtype x_dtype);
size_t dbp_conv2d_workspace_bytes(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K,
                                  int64_t R, int64_t S, int64_t stride, int64_t pad,
                                  dbp_dtype x_dtype);

/*
 * NSD pass, Eq. (nsd) applied elementwise as in Eq. (qdz) (Algorithm 1, step 4, with the
 * dither the algorithm listing omits).  One fused kernel: counter-based dither, quantise,
 * int8 codes, per-tile nonzero counts (wavefront ballot + popcount), bitmap, compaction.
 *   delta   [rows*cols] fp32, in.      rows/cols only shape the tile-sparse format; the
 *                                      codes themselves depend on the flat index alone.
 *   step    Delta > 0 (the caller's s*sigma of Algorithm 1, steps 2-3).
 *   codes   [rows*cols] int8, out.
 *   format  buffer of dbp_format_layout.total_bytes, 256-byte aligned, out; NULL = codes only.
 *   stats   out, nullable.  With a format buffer the statistics are reduced without atomics (per-workgroup
 *           partial sums in the buffer's scratch region, then one small kernel); without one they are
 *           accumulated with device atomics from fewer workgroups, which is slower on large tensors.
 * Errors: NULL delta/codes -> DBP_ERR_NULL; rows/cols <= 0 or rows*cols >= 2^40 -> SHAPE;
 * bad step -> STEP; format too small/misaligned -> WORKSPACE.
 */
dbp_status nsd_quantize(const float *delta, int64_t rows, int64_t cols, float step,
                        uint64_t seed, uint64_t idx_base, int8_t *codes,
                        void *format, size_t format_bytes, dbp_stats *stats, void *stream);

/*
 * nsd_quantize for callers that cannot allocate device memory or bring a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Codes and statistics as nsd_quantize (no tile-sparse format); the
 * quantiser's scratch (its per-workgroup statistics records, 256 KiB) lives in a device array inside the library, one per
 * GPU, held until the process ends.  The call allocates and frees nothing and launches the same kernels as nsd_quantize.
 *   rows*cols <= DBP_STATIC_MAX_ELEMENTS, else DBP_ERR_SHAPE; stats is required; other errors as nsd_quantize;
 *   DBP_ERR_DEVICE if the array's address cannot be obtained.
 * Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two threads) race on it and
 * may report wrong statistics (the codes are not affected); serialise them, or use nsd_quantize with buffers of your own.
 */
#define DBP_STATIC_MAX_ELEMENTS ((int64_t)1 << 32)
dbp_status nsd_quantize_static(const float *delta, int64_t rows, int64_t cols, float step,
                               uint64_t seed, uint64_t idx_base, int8_t *codes,
                               dbp_stats *stats, void *stream);

/*
 * Top-k sparsifier: the comparison method of Sec. "Comparison to meProp" (of every gradient vector the k elements of
 * largest magnitude survive, the rest become zero), emitting the same int8 codes, tile-sparse format and statistics as
 * nsd_quantize, so that the two sparsifiers can be compared on identical product kernels (dbp_*_products).
 *   delta     [rows*cols] fp32, in; rows/cols shape the tile-sparse format as in nsd_quantize.
 *   vec_rows  a vector = vec_rows consecutive rows (vec_rows*cols consecutive elements); rows % vec_rows == 0.
 *             Fully connected layer: 1 (one example's gradient).  Convolution, codes [N*K x P*Q]: K for one vector per
 *             example, 1 for one per feature-map plane.
 *   k         elements kept per vector: those whose magnitude reaches the k-th largest of the vector (ties at that
 *             magnitude all survive); k <= 0 keeps nothing, k >= the vector's length everything.  NaN has magnitude 0.
 *   step      Delta > 0 of the code grid (e.g. max|delta|/127): survivors become floor(fma(x, 1/Delta, 0.5f)) clamped to
 *             [-127,127] -- Eq. (nsd) without the dither, i.e. deterministic rounding to the nearest level.
 *   workspace dbp_topk_workspace_bytes(rows, vec_rows) bytes, 256-byte aligned (the per-vector thresholds).
 *   format, stats as nsd_quantize (the statistics are those of the tensor with the dropped elements set to 0).
 * Two kernels: a per-vector selection (binary search over the magnitude bits; vectors up to 65536 elements are held in
 * registers, longer ones are re-read 31 times and are slow), then the quantiser's kernel.
 * Errors: as nsd_quantize; vec_rows <= 0, rows % vec_rows != 0, vec_rows*cols >= 2^31 -> SHAPE; workspace -> WORKSPACE.
 */
size_t     dbp_topk_workspace_bytes(int64_t rows, int64_t vec_rows);
dbp_status topk_quantize(const float *delta, int64_t rows, int64_t cols, int64_t vec_rows, int64_t k, float step,
                         int8_t *codes, void *format, size_t format_bytes, void *workspace, size_t workspace_bytes,
                         dbp_stats *stats, void *stream);

/*
 * Dithered backward pass of a fully connected layer, Eqs. (qdz), (qda), (qdw):
 * NSD of delta, then dX = q.W and dW = q^T.X  (storage form of W^T.q and q.a^T).
 *   X, dW   fp32 when x_dtype == DBP_F32; int8 X and int32 dW when x_dtype == DBP_I8
 *           (8-bit mode, Sec. "Quantizing forward pass"; dW32 = sum_b k[b,o]*x8[b,i], exact).
 *   codes   out, nullable (then kept inside the workspace).
 *   dX, dW  nullable = skip that product (not both).
 * Errors as nsd_quantize, plus DBP_ERR_DTYPE, DBP_ERR_OVERFLOW (8-bit mode, B*127*127 >= 2^31).
 */
dbp_status dithered_linear_backward(const float *delta, const float *W, const void *X,
                                    dbp_dtype x_dtype, int64_t B, int64_t in, int64_t out,
                                    float step, uint64_t seed, uint64_t idx_base,
                                    int8_t *codes, float *dX, void *dW,
                                    void *workspace, size_t workspace_bytes,
                                    dbp_stats *stats, dbp_path path, void *stream);

/*
 * Dithered backward pass of a 2-D convolution (cross-correlation, zero padding, dilation = 1; grouped layers:
 * dithered_conv2d_backward_grouped), the convolutional analogue of Eqs. (qdz), (qda), (qdw):
 *   dX[n,c,h,w] = Delta * sum_{k,r,s} code[n,k,p,q] W[k,c,r,s],  h = p*stride+r-pad, w = q*stride+s-pad
 *   dW[k,c,r,s] = Delta * sum_{n,p,q} code[n,k,p,q] X[n,c,p*stride+r-pad,q*stride+s-pad]
 * x_dtype as above.  Errors as above; path == DBP_PATH_GATHER (kernels that visit the nonzero codes only; rows of the
 * format = the planes (n,k) of P*Q codes) needs R*S <= 64, P, Q < 4096 and, for dX, H*Wd <= 9536 (DBP_ERR_UNSUPPORTED
 * otherwise).  3x3 and 1x1 layers whose planes are a multiple of 4 bytes run on kernels that scan the code planes (dX: stride
 * 1 only; they keep prepared weights and partial sums in the workspace), every other shape on kernels that walk the format's
 * entries.  On the matrix-core paths stride 1 runs on the specialised kernels; with another stride dX runs on them as stride*stride
 * stride-1 problems (one per class of output pixels modulo the stride) when stride <= 3, dW as a column-matrix
 * product on the fully connected kernels when the layer is large enough, the rest on the generic implicit-im2col kernel.
 */
dbp_status dithered_conv2d_backward(const float *delta, const float *W, const void *X,
                                    dbp_dtype x_dtype, int64_t N, int64_t C, int64_t H,
                                    int64_t Wd, int64_t K, int64_t R, int64_t S,
                                    int64_t stride, int64_t pad,
                                    float step, uint64_t seed, uint64_t idx_base,
                                    int8_t *codes, float *dX, void *dW,
                                    void *workspace, size_t workspace_bytes,
                                    dbp_stats *stats, dbp_path path, void *stream);

/*
 * Grouped convolution (the layer type of the two-tower AlexNet and of later CNNs of the kind Sec. "Experiments" trains): input
 * and output channels are cut into `groups` equal consecutive blocks and output channel k sees only the input channels of
 * block k / (K/groups).  Eqs. (qdz), (qda), (qdw) as in dithered_conv2d_backward, with
 *   W, dW [K, C/groups, R, S];  X, dX [N, C, H, Wd];  delta, codes [N, K, P, Q]   (groups == 1: dithered_conv2d_backward).
 * One quantiser pass over the whole delta.  With at least 64 input channels per group the groups then run one after the
 * other on the stream as independent layers (N, C/groups, H, Wd, K/groups) on channel blocks of the same tensors, on the
 * kernels of the ungrouped layer.  Smaller groups (down to depthwise layers) would fill little of a 64- or 128-channel
 * matrix-core tile each and cost their own launches: they run as ONE ungrouped layer with block-diagonal weights (the
 * products outside a channel's group are exact zeros) at the ungrouped layer's cost, whatever the group count.
 * DBP_PATH_AUTO takes the matrix-core kernels (no density dispatch).  workspace: dbp_conv2d_grouped_workspace_bytes.
 * Errors as dithered_conv2d_backward; groups < 1 or not dividing C and K -> DBP_ERR_SHAPE.
 */
size_t     dbp_conv2d_grouped_workspace_bytes(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                              int64_t stride, int64_t pad, int64_t groups, dbp_dtype x_dtype);
dbp_status dithered_conv2d_backward_grouped(const float *delta, const float *W, const void *X, dbp_dtype x_dtype,
                                            int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                            int64_t stride, int64_t pad, int64_t groups,
                                            float step, uint64_t seed, uint64_t idx_base,
                                            int8_t *codes, float *dX, void *dW,
                                            void *workspace, size_t workspace_bytes,
                                            dbp_stats *stats, dbp_path path, void *stream);
/* The products alone, as dbp_conv2d_products: `format` (rows = N*K, cols = P*Q) is read by DBP_PATH_GATHER only; the other
 * paths need a workspace of conv scratch for one group (dbp_conv2d_grouped_workspace_bytes is enough). */
dbp_status dbp_conv2d_products_grouped(const int8_t *codes, const void *format, float step,
                                       const float *W, const void *X, dbp_dtype x_dtype,
                                       int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K,
                                       int64_t R, int64_t S, int64_t stride, int64_t pad, int64_t groups,
                                       float *dX, void *dW, void *workspace, size_t workspace_bytes,
                                       dbp_path path, void *stream);

/*
 * Same-library dense baselines: the undithered backward pass, Eqs. (da), (dw), on fp32 matrix
 * cores (x_dtype == DBP_F32) -- the line the dithered path is measured against.  In 8-bit
 * mode (DBP_I8) `delta` is instead a dense int8 gradient [..] and dW is int32.
 */
dbp_status dense_linear_backward(const void *delta, const float *W, const void *X,
                                 dbp_dtype x_dtype, int64_t B, int64_t in, int64_t out,
                                 float *dX, void *dW, void *workspace, size_t workspace_bytes,
                                 void *stream);
dbp_status dense_conv2d_backward(const void *delta, const float *W, const void *X,
                                 dbp_dtype x_dtype, int64_t N, int64_t C, int64_t H, int64_t Wd,
                                 int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad,
                                 float *dX, void *dW, void *workspace, size_t workspace_bytes,
                                 void *stream);

/*
 * The products alone, from codes already quantised (e.g. by nsd_quantize): the second half of
 * dithered_*_backward, exposed so that each kernel can be timed and tested on its own.
 * `format` is the buffer nsd_quantize filled for (rows=B, cols=out) resp. (rows=N*K, cols=P*Q);
 * it may be NULL when path == DBP_PATH_MFMA.
 */
dbp_status dbp_linear_products(const int8_t *codes, const void *format, float step,
                               const float *W, const void *X, dbp_dtype x_dtype,
                               int64_t B, int64_t in, int64_t out, float *dX, void *dW,
                               void *workspace, size_t workspace_bytes, dbp_path path, void *stream);
dbp_status dbp_conv2d_products(const int8_t *codes, const void *format, float step,
                               const float *W, const void *X, dbp_dtype x_dtype,
                               int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K,
                               int64_t R, int64_t S, int64_t stride, int64_t pad,
                               float *dX, void *dW, void *workspace, size_t workspace_bytes,
                               dbp_path path, void *stream);


/*
 * ---------------------------------------------------------------------------------------------------------
 * Algorithm 1 on the device, and the two steps that surround the quantiser in a layer's backward pass.
 * ---------------------------------------------------------------------------------------------------------
 * Step size (Algorithm 1, the two assignments before the quantiser):  sigma = std(delta_z),  Delta = s * sigma.
 *   Readings: population standard deviation (divide by n) over ALL elements of the tensor, from
 *   S1 = sum x and S2 = sum x*x accumulated in fp64; because Delta decides integer codes the order of the
 *   sums is part of the definition: a radix-16 tree (groups of 16 consecutive values summed left to right,
 *   the group sums likewise, until one value is left).  sigma = sqrt((S2 - S1*S1/n)/n), Delta = fp32(s*sigma).
 *   With `act` the deviation is that of delta_z = delta_a (.) f'(z) (see below).
 *   step_out  device, out: {Delta, 1/Delta} (8-byte aligned).  A layer whose sigma is 0 or not finite gets
 *             {0, 0}: every code is then 0 and both products are exactly 0.
 *   workspace dbp_step_size_workspace_bytes(n) bytes, 256-byte aligned.
 * Errors: NULL pointers -> NULL; n <= 0 -> SHAPE; s not positive/finite -> STEP; workspace -> WORKSPACE.
 */
size_t     dbp_step_size_workspace_bytes(int64_t n);
dbp_status dbp_step_size(const float *delta /*device*/, const float *act /*device, nullable*/, int64_t n, float s,
                         float *step_out /*device [2]*/, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Options of nsd_quantize_ex (a host struct of device pointers; every member may be NULL / 0):
 *   act        same shape as delta.  delta_z = delta_a (.) f'(z) (the first line of the backward pass) for the
 *              rectifier: the element is quantised where act > 0 and is +0 elsewhere; act may be z or a = f(z)
 *              (-0.0 and NaN count as not positive).
 *   step_dev   {Delta, 1/Delta} in device memory as written by dbp_step_size; replaces the `step` argument.
 *   bias_sums  out, int64 [bias_len]: exact sums of the codes over everything that shares a bias (the bias
 *              enters Eq. (z) additively, so delta_b = sum of the quantised gradient = Delta * sum of codes).
 *              DBP_BIAS_PER_COLUMN: bias_len == cols, sums[c] = sum_r k[r][c]                      (FC, rows = batch)
 *              DBP_BIAS_PER_ROW_GROUP: rows % bias_len == 0, sums[g] = sum over rows r with r % bias_len == g
 *              and all columns                                       (conv: rows = (n,k), columns = pixels)
 *   bias_grad  out, fp32 [bias_len] = fp32( (double)Delta * (double)sums ); needs bias_sums.
 */
typedef enum { DBP_BIAS_PER_COLUMN = 0, DBP_BIAS_PER_ROW_GROUP = 1 } dbp_bias_mode;
typedef struct {
    const float *act;
    const float *step_dev;
    int64_t     *bias_sums;
    float       *bias_grad;
    int32_t      bias_mode;
    int64_t      bias_len;
} dbp_nsd_extras;

/* nsd_quantize with the options above (extras == NULL: identical to nsd_quantize).
 * Errors as nsd_quantize; inconsistent bias_len -> SHAPE; unknown bias_mode -> UNSUPPORTED. */
dbp_status nsd_quantize_ex(const float *delta, int64_t rows, int64_t cols, float step, uint64_t seed,
                           uint64_t idx_base, int8_t *codes, void *format, size_t format_bytes,
                           dbp_stats *stats, const dbp_nsd_extras *extras /*host*/, void *stream);

/*
 * The whole backward pass of a layer as Algorithm 1 states it, in one call:
 *   delta_z = delta_a (.) f'(z)   (act != NULL; rectifier)
 *   Delta   = s * std(delta_z)    (on the device; also returned in step_out when that is not NULL)
 *   q       = NSD(delta_z)        Eq. (qdz)
 *   dX, dW  = Eqs. (qda), (qdw);  db = Delta * sum over the batch (and pixels) of the codes.
 * dX, dW, db are each nullable (not all three).  Workspace: dbp_*_layer_workspace_bytes.
 * Errors as dithered_*_backward, with `s` checked in place of the step.
 */
size_t     dbp_linear_layer_workspace_bytes(int64_t B, int64_t in, int64_t out, dbp_dtype x_dtype);
size_t     dbp_conv2d_layer_workspace_bytes(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R,
                                            int64_t S, int64_t stride, int64_t pad, dbp_dtype x_dtype);
dbp_status dithered_linear_layer_backward(const float *delta_a, const float *act, const float *W, const void *X,
                                          dbp_dtype x_dtype, int64_t B, int64_t in, int64_t out, float s,
                                          uint64_t seed, uint64_t idx_base, int8_t *codes, float *dX, void *dW,
                                          float *db /*device [out]*/, float *step_out /*device [2]*/,
                                          void *workspace, size_t workspace_bytes, dbp_stats *stats,
                                          dbp_path path, void *stream);
dbp_status dithered_conv2d_layer_backward(const float *delta_a, const float *act, const float *W, const void *X,
                                          dbp_dtype x_dtype, int64_t N, int64_t C, int64_t H, int64_t Wd,
                                          int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad, float s,
                                          uint64_t seed, uint64_t idx_base, int8_t *codes, float *dX, void *dW,
                                          float *db /*device [K]*/, float *step_out /*device [2]*/,
                                          void *workspace, size_t workspace_bytes, dbp_stats *stats,
                                          dbp_path path, void *stream);

/*
 * ---------------------------------------------------------------------------------------------------------
 * Full 8-bit backward (Sec. "Quantizing forward pass": weights and activations are 8-bit too, so that every
 * product of the backward pass is an 8-bit computation and only the weight update stays in full precision).
 * ---------------------------------------------------------------------------------------------------------
 * dbp_quantize_int8: the forward pass's quantiser.  The paper takes it from the work it cites and does not
 * print it; reading taken here: symmetric, one scale per tensor,
 *     amax = max |x_i| over the finite x_i,  scale = amax / 127,  inv = 127 / amax          (fp32 divisions)
 *     q_i  = clamp(round-half-even(x_i * inv), -127, 127)                              (one fp32 product)
 *   NaN -> 0, +-Inf -> +-127; amax == 0 or nothing finite: scale = inv = 0 and every finite q_i is 0.
 *   x device [n]; q device, out [n]; scale_out device, out: {scale, inv} (8-byte aligned);
 *   workspace dbp_quantize_int8_workspace_bytes(n), 256-byte aligned.
 *   Errors: NULL -> NULL; n <= 0 or misaligned -> SHAPE; workspace -> WORKSPACE.
 *
 * dithered_*_backward_q8: NSD of delta, then both products on int8 matrix cores with exact int32 sums:
 *     dX32[b,i] = sum_o k[b,o] * W8[o,i]          dW32[o,i] = sum_b k[b,o] * X8[b,i]        (conv: the adjoints of
 *     the cross-correlation, as in dithered_conv2d_backward).
 *   The real gradients are Delta*scale_W*dX32 and Delta*scale_X*dW32; the caller applies the scales (in the weight
 *   update, which stays in full precision).  dX32 / dW32 nullable (not both); W8 needed for dX32, X8 for dW32.
 *   Workspace: dbp_linear_workspace_bytes / dbp_conv2d_workspace_bytes (any path, DBP_I8).
 *   Errors as dithered_*_backward; a reduction long enough to overflow int32 (length*127*127 >= 2^31) -> OVERFLOW.
 */
size_t     dbp_quantize_int8_workspace_bytes(int64_t n);
dbp_status dbp_quantize_int8(const float *x /*device*/, int64_t n, int8_t *q /*device*/, float *scale_out /*device [2]*/,
                             void *workspace, size_t workspace_bytes, void *stream);
dbp_status dithered_linear_backward_q8(const float *delta, const int8_t *W8, const int8_t *X8,
                                       int64_t B, int64_t in, int64_t out, float step, uint64_t seed, uint64_t idx_base,
                                       int8_t *codes, int32_t *dX32, int32_t *dW32, void *workspace,
                                       size_t workspace_bytes, dbp_stats *stats, void *stream);
dbp_status dithered_conv2d_backward_q8(const float *delta, const int8_t *W8, const int8_t *X8,
                                       int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                       int64_t stride, int64_t pad, float step, uint64_t seed, uint64_t idx_base,
                                       int8_t *codes, int32_t *dX32, int32_t *dW32, void *workspace,
                                       size_t workspace_bytes, dbp_stats *stats, void *stream);

/*
 * Host-side self-check of the launch plans (no GPU call): walks, for one layer shape, the planning arithmetic that decides
 * the kernels' work items, split-K partial sums and workspace offsets -- every work item handed out exactly once, every
 * tile / split / class index in range, every buffer inside the size the *_workspace_bytes functions report -- with the
 * same functions the launchers and kernels use.  Returns 0 when consistent (or when the shape takes a kernel without a
 * plan), a positive number naming the first violated invariant, -1 for invalid dimensions.  For tests and diagnostics.
 */
int dbp_plan_check_linear(int64_t B, int64_t in, int64_t out);
int dbp_plan_check_conv2d(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                          int64_t stride, int64_t pad);
/* The same for the plans of the gather kernels that scan the code planes (3x3 and 1x1 layers): bands, tile sizes, LDS, the
 * reciprocals that replace divisions, the share of `scratch_bytes` of workspace they would use.  int8_x: X is DBP_I8. */
int dbp_plan_check_conv2d_gather(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                 int64_t stride, int64_t pad, int int8_x, size_t scratch_bytes);

/* What DBP_PATH_AUTO would set up for dithered_conv2d_backward on this layer, from the host's cost models alone (no GPU
 * call; see dbp_path): 0 = matrix cores, no gate; 1 = the whole gather family behind the gate, taken when fewer than
 * *gather_below codes are nonzero; 2 = the gather kernel for dW alone (dX on matrix cores) when fewer than *dw_rows_below
 * are; -1 for invalid dimensions.  The thresholds not in use are set to 0; either pointer may be NULL.  int8_x: X is
 * DBP_I8; want_dx / want_dw: which products the call asks for; two_planes: DBP_PATH_TWO_PLANES.  The workspace is taken to
 * be the size dbp_conv2d_workspace_bytes reports.  For tests and diagnostics. */
int dbp_plan_auto_conv2d(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                         int64_t stride, int64_t pad, int int8_x, int want_dx, int want_dw, int two_planes,
                         uint64_t *gather_below, uint64_t *dw_rows_below);
/* The same for dithered_linear_backward: 0 = matrix cores, no gate; 1 = both families behind the gate, the gather kernels
 * taken when fewer than *gather_below codes are nonzero (0 otherwise; may be NULL); -1 for invalid dimensions. */
int dbp_plan_auto_linear(int64_t B, int64_t in, int64_t out, int int8_x, int want_dx, int want_dw, int two_planes,
                         uint64_t *gather_below);

#ifdef __cplusplus
}
#endif
#endif /* DBP_H_ */
