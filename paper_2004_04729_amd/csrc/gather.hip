// Gather path of the backward products: walk only the nonzero codes (Sec. "Computational complexity":
// O(p_nz * m*k*n) multiply-adds instead of O(m*k*n)).  Plain fp32 FMA on the vector ALUs.
//
// Fully connected layers: fc_rows_kernel.  A workgroup of 16 wavefronts owns 128 (dX) or 256 (dW) output rows x 256 output
// columns, stages the dense operand (W for dX, X for dW) through LDS in tiles of 64 reduction indices x 256 columns, and
// every wavefront walks the nonzero codes of its 8 or 16 rows against the staged tile: one LDS read of a lane's four
// columns feeds four multiply-adds, so the staged tile is shared by all rows of the block and the dense operand leaves
// HBM / L2 once per workgroup.  The one-row-per-workgroup kernels
// further down serve the shapes it declines (odd strides and alignments, int8 activations).
// Convolutions: conv_dw_rows_kernel / conv_dx_rows_kernel (conv_rows_kernel.h: 3x3 and 1x1 layers whose planes are a multiple of
// 4 bytes; dX: stride 1) read the code plane, lanes = channels; conv_d{x,w}_gather_kernel, which walk the compacted entries of
// the tile-sparse format with a lane per (channel, tap), serve every other shape.
#include "common.h"
#include "conv_rows_kernel.h"

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

// ---- LDS-staged row-list kernel of the fully connected products ------------------------------------
//   out[r][i] = scale * sum over c with A(r,c) != 0 of  A(r,c) * D[c][i]
//   dX (TR = false): r = b, c = o, A(r,c) = codes[r*ldc + c], D = W [out][in]
//   dW (TR = true):  r = o, c = b, A(r,c) = codes[c*ldc + r], D = X [B][in]
// A workgroup of 16 wavefronts owns 256 output rows x 64*CPL output columns and walks the reduction in chunks of 64
// indices; the chunk's tile of D goes through LDS once and serves all 256 rows.  A wavefront's lanes are the chunk's
// reduction indices when it looks at codes (the nonzero mask of a row is one ballot, a code reaches the scalar unit
// through a lane read) and CPL output columns each when it multiplies (one LDS read of 4*CPL bytes feeds CPL
// multiply-adds).  The accumulators of a wavefront's 16 rows are registers with compile-time indices; the walk over a
// row's nonzeros is a scalar loop.  Sums run in a fixed order (chunks in order, nonzeros by lane): deterministic.
// Codes: dX stages the chunk's 256 x 64 code bytes in LDS beside the tile (coalesced 4-byte loads; a row's codes are
// then one byte read per lane); dW loads, per lane (= batch row), the 16 code bytes of the wavefront's 16 output rows.
// dX (DEEP): W comes from HBM and is fetched two tiles ahead (two sets of staging registers); 128-column slabs keep the
// number of reduction parts, hence of partial sums, low.  dW: X is small and sits in L2; one tile ahead, 256-column slabs.
// Every step issues the same loads in the same order on every path (addresses are clamped and values masked rather
// than loads predicated; steps past the end repeat the last one): the compiler's wait counts can then leave exactly the
// younger loads outstanding -- a load that only some paths issue makes it wait for all of them.
constexpr int FR_THREADS = 1024, FR_WAVES = 16, FR_CH = 64;
constexpr int FR_RW_DX = 8, FR_RW_DW = 16;                        // rows per wavefront: 128-row blocks for dX (fewer reduction parts), 256 for dW
constexpr int FR_CPL_DX = 4, FR_CPL_DW = 4;                       // output columns per lane: 256-column slabs
constexpr size_t fr_lds_bytes(int cpl, int rw, bool tr) { return (size_t)2 * FR_CH * 64 * cpl * sizeof(float) + (tr ? 0 : 2 * FR_WAVES * rw * FR_CH); }

struct FcRowsArgs {
    const int8_t *codes; int64_t ldc;
    const float *D; int64_t ldd;
    float *out, *partial;                     // partial [sparts][rows][cols] when sparts > 1
    int rows, red, cols;
    int slabs, row_blocks, n_chunks;
    int rparts, rb_per_part;                  // parts over the row blocks
    int sparts, ch_per_part;                  // parts over the reduction (partial sums when sparts > 1)
    Scale scale;
    Gate gate;
};

template <bool TR, int FR_RW, int FR_CPL, bool DEEP, int ALIGN>
__global__ __launch_bounds__(FR_THREADS) void fc_rows_kernel(FcRowsArgs a)
{
    static_assert(TR ? FR_RW == 16 : (FR_RW == 8 || FR_RW == 16), "dW: 16 code bytes per lane; dX: code tiles of 8 or 16 KiB");
    constexpr int FR_ROWS = FR_WAVES * FR_RW, FR_CODE_TILE = FR_ROWS * FR_CH;
    constexpr int FR_SLAB = 64 * FR_CPL;
    constexpr int FR_TILE = FR_CH * FR_SLAB;                      // floats per staged tile
    constexpr int FR_STAGE = FR_TILE / 4 / FR_THREADS;            // 16-byte pieces per thread and tile
    constexpr int FR_SROWS = FR_THREADS * 4 / FR_SLAB;            // tile rows one pass of the workgroup's 16-byte loads covers
    extern __shared__ __attribute__((aligned(16))) float fr_lds[];
    if (a.gate.closed()) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slab = (int)blockIdx.x % a.slabs, part = (int)blockIdx.x / a.slabs;
    const int rp = part / a.sparts, sp = part - rp * a.sparts;
    const int col0 = slab * FR_SLAB;
    const int rb_lo = rp * a.rb_per_part, rb_hi = min(a.row_blocks, rb_lo + a.rb_per_part);
    const int ch_lo = sp * a.ch_per_part, ch_hi = min(a.n_chunks, ch_lo + a.ch_per_part);
    const int n_ch = ch_hi - ch_lo, n_steps = (rb_hi - rb_lo) * n_ch;
    if (n_steps <= 0) return;
    int8_t *code_lds = (int8_t *)(fr_lds + 2 * FR_TILE);          // dX: two code tiles [256 rows][64 reduction indices]

    constexpr int NCD = FR_RW / 4;                                // dX: code dwords a thread stages per step
    struct Stage { f32x4 d[FR_STAGE]; int c[TR ? 1 : NCD]; };     // what a thread moves per step: tile pieces (+ dX code dwords)
    // ---- staging: consecutive threads move consecutive 16-byte pieces of a tile row (and of a code row)
    const int sr = tid / (FR_SLAB / 4), sc = (tid % (FR_SLAB / 4)) * 4;
    const int scol = min(col0 + sc, a.cols - 4);                 // columns past the end repeat the last ones (never stored)
    const int cr = tid / (16 / NCD), cc = (tid % (16 / NCD)) * 4 * NCD;   // dX codes: row of the block, first of this thread's reduction indices
    auto stage_load = [&](Stage &st, int rb, int ch) {
        if constexpr (!TR) {
            const int8_t *src = a.codes + (int64_t)min(rb * FR_ROWS + cr, a.rows - 1) * a.ldc;
#pragma unroll
            for (int q = 0; q < NCD; ++q) st.c[q] = *(const int *)(src + min(ch * FR_CH + cc + 4 * q, a.red - 4));
        }
#pragma unroll
        for (int i = 0; i < FR_STAGE; ++i) {
            const int r = min(ch * FR_CH + sr + FR_SROWS * i, a.red - 1);   // rows past the end repeat the last one (never read: their codes are 0)
            st.d[i] = *(const f32x4 *)(a.D + (int64_t)r * a.ldd + scol);
        }
    };
    auto stage_store = [&](Stage &st, int buf, int rb, int ch) {
        float *t = fr_lds + buf * FR_TILE;
#pragma unroll
        for (int i = 0; i < FR_STAGE; ++i) *(f32x4 *)(t + (sr + FR_SROWS * i) * FR_SLAB + sc) = st.d[i];
        if constexpr (!TR) {
            // codes outside the matrix become 0 here (bit masks: a select on a wave-uniform condition would be turned into
            // a branch around the load)
            const int row_mask = -(int)(rb * FR_ROWS + cr < a.rows);
            int *dstc = (int *)(code_lds + buf * FR_CODE_TILE + cr * FR_CH + cc);
#pragma unroll
            for (int q = 0; q < NCD; ++q) dstc[q] = st.c[q] & row_mask & -(int)(ch * FR_CH + cc + 4 * q < a.red);
        }
    };

    // ---- dW: the 16 code bytes of batch row c that belong to the wavefront's output rows, in registers
    auto fetch_codes = [&](int (&raw)[4], int rb, int ch) {
        const int row0 = rb * FR_ROWS + wave * FR_RW;
        const int8_t *src = a.codes + (int64_t)min(ch * FR_CH + lane, a.red - 1) * a.ldc;
        if constexpr (ALIGN == 16) {
            const i32x4 v = *(const i32x4 *)(src + min(row0, a.rows - 16));
            raw[0] = v.x; raw[1] = v.y; raw[2] = v.z; raw[3] = v.w;
        } else if constexpr (ALIGN == 4) {
#pragma unroll
            for (int q = 0; q < 4; ++q) raw[q] = *(const int *)(src + min(row0 + 4 * q, a.rows - 4));
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                raw[q] = (int)(uint8_t)src[min(row0 + 4 * q, a.rows - 1)] | (int)(uint8_t)src[min(row0 + 4 * q + 1, a.rows - 1)] << 8 |
                         (int)(uint8_t)src[min(row0 + 4 * q + 2, a.rows - 1)] << 16 | (int)(uint8_t)src[min(row0 + 4 * q + 3, a.rows - 1)] << 24;
        }
    };
    auto mask_codes = [&](int (&raw)[4], int rb, int ch) {
        const int row0 = rb * FR_ROWS + wave * FR_RW;
        const int lane_mask = -(int)(ch * FR_CH + lane < a.red);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // bytes of the rows that exist (ALIGN 16: rows % 16 == 0, a wavefront's rows exist all or not at all)
            const int left = a.rows - (row0 + 4 * q);
            const int row_mask = left >= 4 ? -1 : left <= 0 ? 0 : (1 << (8 * left)) - 1;
            raw[q] &= lane_mask & row_mask;
        }
    };

    float acc[FR_RW][FR_CPL];
#pragma unroll
    for (int r = 0; r < FR_RW; ++r)
#pragma unroll
        for (int j = 0; j < FR_CPL; ++j) acc[r][j] = 0.f;
    int raw[4] = {0, 0, 0, 0}, raw_next[4] = {0, 0, 0, 0};
    // (row block, chunk) of the steps s, s + 1 and s + 2; steps past the end repeat the last one
    struct Pos { int rb, ch; };
    auto next_pos = [&](Pos p) {
        Pos q = p;
        if (++q.ch == ch_hi) { q.ch = ch_lo; ++q.rb; }
        return q.rb < rb_hi ? q : p;
    };
    Pos p0{rb_lo, ch_lo}, p1 = next_pos(p0), p2 = next_pos(p1);
    const bool partial = a.sparts > 1;
    const float sc_out = partial ? 1.0f : a.scale.get();
    float *dst = partial ? a.partial + (int64_t)sp * a.rows * a.cols : a.out;
    Stage stA, stB;                                    // tiles of the odd / even steps on their way to LDS (stA: DEEP only)
    if constexpr (TR) fetch_codes(raw_next, p0.rb, p0.ch);
    stage_load(stB, p0.rb, p0.ch);
    if constexpr (DEEP) stage_load(stA, p1.rb, p1.ch);
    stage_store(stB, 0, p0.rb, p0.ch);
    __syncthreads();

    // One step: multiply against the tile in buffer s & 1 while tile s + 1 (registers `nxt`) and, DEEP, tile s + 2 (fetched
    // into `cur`, whose tile is already in LDS) are on their way.
    auto step = [&](int s, Stage &cur, Stage &nxt) {
        const int rb = p0.rb, ch = p0.ch;
        if constexpr (TR) {
#pragma unroll
            for (int q = 0; q < 4; ++q) raw[q] = raw_next[q];
            mask_codes(raw, rb, ch);
            fetch_codes(raw_next, p1.rb, p1.ch);
        }
        if constexpr (DEEP) stage_load(cur, p2.rb, p2.ch);
        else                stage_load(nxt, p1.rb, p1.ch);
        const float *tile = fr_lds + (s & 1) * FR_TILE + FR_CPL * lane;
        const int8_t *ctile = code_lds + (s & 1) * FR_CODE_TILE + wave * FR_RW * FR_CH + lane;
#pragma unroll
        for (int r = 0; r < FR_RW; ++r) {
            int code;
            if constexpr (TR) code = (int)(int8_t)(raw[r >> 2] >> (8 * (r & 3)));
            else              code = ctile[r * FR_CH];
            const float kf = (float)code;
            uint64_t m = __builtin_amdgcn_ballot_w64(code != 0);
            float av[FR_CPL];
#pragma unroll
            for (int j = 0; j < FR_CPL; ++j) av[j] = acc[r][j];
            while (m) {
                const int l = __builtin_ctzll(m);
                m &= ~(1ull << l);
                const float k = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(kf), l));
                if constexpr (FR_CPL == 4) {
                    const f32x4 x = *(const f32x4 *)(tile + l * FR_SLAB);
                    av[0] = __builtin_fmaf(k, x.x, av[0]); av[1] = __builtin_fmaf(k, x.y, av[1]);
                    av[2] = __builtin_fmaf(k, x.z, av[2]); av[3] = __builtin_fmaf(k, x.w, av[3]);
                } else {
                    const float2 x = *(const float2 *)(tile + l * FR_SLAB);
                    av[0] = __builtin_fmaf(k, x.x, av[0]); av[1] = __builtin_fmaf(k, x.y, av[1]);
                }
            }
#pragma unroll
            for (int j = 0; j < FR_CPL; ++j) acc[r][j] = av[j];
        }
        if (ch == ch_hi - 1) {
            // the row block is complete for this part: store (scaled when these are final values) and start over
            const int row0 = rb * FR_ROWS + wave * FR_RW, col = col0 + FR_CPL * lane;
#pragma unroll
            for (int r = 0; r < FR_RW; ++r) {
                if (row0 + r < a.rows && col < a.cols) {
                    float *o = dst + (int64_t)(row0 + r) * a.cols + col;
                    if constexpr (FR_CPL == 4) *(f32x4 *)o = f32x4{sc_out * acc[r][0], sc_out * acc[r][1], sc_out * acc[r][2], sc_out * acc[r][3]};
                    else                       *(float2 *)o = float2{sc_out * acc[r][0], sc_out * acc[r][1]};
                }
#pragma unroll
                for (int j = 0; j < FR_CPL; ++j) acc[r][j] = 0.f;
            }
            // Stores and loads share one counter and complete out of order: with stores possibly in flight the compiler
            // would wait for everything at every later wait of the loop.  Drain here, once per row block, instead.
            __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0)
        }
        stage_store(nxt, (s + 1) & 1, p1.rb, p1.ch);   // after the last step: into the buffer nobody reads any more
        __syncthreads();
        p0 = p1; p1 = p2; p2 = next_pos(p2);
    };
    if constexpr (DEEP) {
        // both copies of the step run in every trip (the odd last step is peeled): a copy that only some trips run would
        // again leave the wait counts of the next trip unknown
        int s = 0;
        for (; s + 1 < n_steps; s += 2) {
            step(s, stB, stA);
            step(s + 1, stA, stB);
        }
        if (s < n_steps) step(s, stB, stA);
    } else {
        for (int s = 0; s < n_steps; ++s) step(s, stB, stB);      // one set of staging registers, one tile ahead
    }
}

// out = scale * (partial[0] + partial[1] + ...), in split order (deterministic)
__global__ __launch_bounds__(256) void fc_rows_reduce_kernel(const float *partial, float *out, int64_t n4, int n_split, Scale scale, Gate gate)
{
    if (gate.closed()) return;
    const float sc = scale.get();
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
        f32x4 v = ((const f32x4 *)partial)[i];
        for (int z = 1; z < n_split; ++z) {
            const f32x4 w = ((const f32x4 *)partial)[i + (int64_t)z * n4];
            v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
        }
        ((f32x4 *)out)[i] = f32x4{sc * v.x, sc * v.y, sc * v.z, sc * v.w};
    }
}

// ---- convolution -------------------------------------------------------------------------------
// The format's rows are the code planes (n, k) of P*Q pixels.  Both kernels give every lane ONE (channel, tap) pair
// and walk the nonzero codes of the planes they need in a fixed order (deterministic sums): 64 / (R*S) channels per
// wavefront, four wavefronts per workgroup.  The walk goes over the tiles of the workgroup's planes in chunks of up to 256
// tiles: their entry counts are scanned, and the entries of as many tiles as fit are copied into LDS as (p, q, code,
// plane) records -- at high sparsity most tiles are empty and one chunk (three barriers) covers hundreds of planes.
// cpw: channels per wavefront.  Ct, Kt: channels of the tensors that hold X/dX and the codes, k_first: the first code plane
// of this problem inside an image's Kt planes (C, K, 0 unless the problem is one group of a grouped convolution).
struct ConvGatherGeom { int N, C, H, Wd, K, R, S, pad, st, P, Q, cpw; int Ct, Kt, k_first; Gate gate; };

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
    if (g.gate.closed()) return;
    const int k = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int RS = g.R * g.S, cl = lane / RS, tap = lane - cl * RS;
    const int c = ((int)blockIdx.x * 4 + wave) * g.cpw + cl;
    const bool own = cl < g.cpw && c < g.C;
    const int r = tap / g.S, s = tap - r * g.S, tpr = (int)f.tiles_per_row, HW = g.H * g.Wd;
    const int n_walk = g.N * tpr, img = g.Ct * HW;         // elements of X per image (the host keeps N*Ct*H*Wd below 2^31)
    const XT *xc = X + (own ? c : 0) * HW;
    AccT acc = 0;
    for (int i0 = 0; i0 < n_walk;) {
        conv_gather_chunk(f, g.k_first + k, g.Kt, tpr, i0, n_walk, g.Q, ch);     // plane j of the walk = image j: row j*Kt + k_first + k
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
    if (g.gate.closed()) return;
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
        conv_gather_chunk(f, (int64_t)n * g.Kt + g.k_first, 1, tpr, i0, n_walk, g.Q, ch);     // plane j of the walk = channel k = j
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
    float *out = dX + ((int64_t)n * g.Ct + c_first) * HW;
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

// ---- host side of conv_rows_kernel.h ---------------------------------------------------------------------
namespace {

constexpr size_t kRowsLdsOne = 150 * 1024;                            // LDS budget of the dW kernel's workgroup (one per CU)

bool rows_shape_ok(const ConvArgs &a, int64_t P, int64_t Q)
{
    const bool taps = (a.R == 3 && a.S == 3) || (a.R == 1 && a.S == 1);
    return taps && (P * Q) % 4 == 0 && (uintptr_t)a.codes % 4 == 0 && Q >= 2 && Q <= 253 && P < 32768 &&
           a.H * a.Wd < ((int64_t)1 << 24) && a.K * a.C * a.R * a.S < ((int64_t)1 << 31);
}

struct DwRowsPlan { bool ok; ConvDwRowsArgs k; size_t lds, partial_bytes; int grid; };

// `avail`: bytes of scratch the shares' partial sums may use.
DwRowsPlan conv_dw_rows_plan(const ConvArgs &a, int64_t P, int64_t Q, size_t avail)
{
    DwRowsPlan pl{};
    if (!rows_shape_ok(a, P, Q)) return pl;
    const int64_t csb = a.x_dtype == DBP_F32 ? 65 * 4 : 68, st = a.stride;
    const int64_t Wp = (Q - 1) * st + a.S;
    int64_t TH = 0;
    {
        int64_t thx = (int64_t)kRowsLdsOne / (Wp * csb);              // one workgroup per CU: the band may take most of its LDS
        if (thx > 64 * CGR_MAX_CHUNKS / Wp) thx = 64 * CGR_MAX_CHUNKS / Wp;
        if (thx >= a.R) TH = (thx - a.R) / st + 1;
    }
    if (TH > P) TH = P;
    if (TH > (256 * CGR_MAX_LOADS - 4) / Q) TH = (256 * CGR_MAX_LOADS - 4) / Q;
    if (TH < 1) return pl;
    ConvDwRowsArgs &k = pl.k;
    k.N = (int)a.N; k.C = (int)a.C; k.K = (int)a.K; k.H = (int)a.H; k.Wd = (int)a.Wd; k.P = (int)P; k.Q = (int)Q;
    k.pad = (int)a.pad; k.st = (int)st; k.Ct = (int)a.ct(); k.Kt = (int)a.kt();
    k.bands = (int)((P + TH - 1) / TH);
    k.TH = (int)((P + k.bands - 1) / k.bands);                        // bands of equal height
    k.THx = (k.TH - 1) * k.st + (int)a.R; k.Wp = (int)Wp;
    k.cells = k.THx * k.Wp; k.n_chunks = (k.cells + 63) / 64;
    pl.lds = ((size_t)k.cells * csb + 15) & ~(size_t)15;
    const int64_t units = a.N * k.bands;
    if (units >= ((int64_t)1 << 30)) return pl;
    const int64_t columns = ((a.C + 63) / 64) * ((a.K + CGR_KB - 1) / CGR_KB);
    const int64_t slots = 256;                                        // one 16-wavefront workgroup per CU
    int64_t want = slots / columns < 1 ? 1 : slots / columns;
    if (want > units) want = units;
    const size_t dw_bytes = (size_t)(a.K * a.C * a.R * a.S) * 4;
    if (want > 1 && (size_t)want * dw_bytes > avail) want = (int64_t)(avail / dw_bytes);
    if (want < 1) want = 1;
    k.units = (int)units;
    k.units_per_split = (int)((units + want - 1) / want);
    k.n_split = (int)((units + k.units_per_split - 1) / k.units_per_split);
    k.q_magic = (uint32_t)((((uint64_t)1 << 32) / (uint64_t)Q) + 1);
    k.wp_magic = (uint32_t)((((uint64_t)1 << 32) / (uint64_t)Wp) + 1);
    pl.partial_bytes = k.n_split > 1 ? (size_t)k.n_split * dw_bytes : 0;
    if (columns * k.n_split >= ((int64_t)1 << 31)) return pl;
    pl.grid = (int)(columns * k.n_split);
    pl.ok = true;
    return pl;
}

template <class XT, int R, int S>
hipError_t launch_conv_dw_rows_as(const DwRowsPlan &pl, hipStream_t s)
{
    static bool raised = false;                                       // more than 64 KiB of dynamic LDS: allowed per kernel, once
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_dw_rows_kernel<XT, R, S>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRowsLdsOne);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((conv_dw_rows_kernel<XT, R, S>), dim3(pl.grid), dim3(CGR_WAVES * 64), pl.lds, s, pl.k);
    return hipGetLastError();
}

struct DxRowsPlan { bool ok; ConvDxRowsArgs k; size_t lds, prep_bytes; int grid, threads; };

DxRowsPlan conv_dx_rows_plan(const ConvArgs &a, int64_t P, int64_t Q, size_t avail)
{
    DxRowsPlan pl{};
    if (!rows_shape_ok(a, P, Q) || a.stride != 1 || a.Wd < 2) return pl;
    const int64_t Cp = (a.C + 63) / 64 * 64, Wp = Q + a.S - 1, row_bytes = Wp * 65 * 4, RS = a.R * a.S;
    const int64_t Kp = (a.K + CGR_KC - 1) / CGR_KC * CGR_KC;
    pl.prep_bytes = (size_t)(Kp * RS * Cp) * 4;
    if (pl.prep_bytes > avail || Kp * RS * Cp >= ((int64_t)1 << 31) || (CGR_KC + 1) * P * Q >= ((int64_t)1 << 31)) return pl;
    // LDS of a workgroup with TH output rows: the rows' accumulators, two chunks of weights, two chunks of code stretches
    auto threads_of = [](int64_t th) { return th <= 4 ? 256 : th <= 8 ? 512 : 1024; };
    auto cb_words_of = [&](int64_t th) { const int64_t w = ((th + a.R - 1) * Q + 3 + 3) / 4; return w < 2 ? (int64_t)2 : w; };
    auto lds_of = [&](int64_t th) { return th * row_bytes + 2 * (CGR_KC * RS * 64 * 4 + CGR_KC * cb_words_of(th) * 4); };
    auto fits = [&](int64_t th, int64_t budget) { return lds_of(th) <= budget && CGR_KC * cb_words_of(th) <= CGR_DX_CPT * threads_of(th); };
    const int64_t th_cap = a.H < CGR_DX_MAX_ROWS ? a.H : CGR_DX_MAX_ROWS;
    int64_t TH = 0;
    for (int64_t budget : {(int64_t)79 * 1024, (int64_t)158 * 1024}) {           // two workgroups per CU if at least 8 rows (or the image) fit
        int64_t th = th_cap;
        while (th >= 1 && !fits(th, budget)) --th;
        if (th >= 1 && (th >= 8 || th == th_cap || budget > 79 * 1024)) { TH = th; break; }
    }
    if (TH < 1) return pl;
    ConvDxRowsArgs &k = pl.k;
    k.N = (int)a.N; k.C = (int)a.C; k.K = (int)a.K; k.H = (int)a.H; k.Wd = (int)a.Wd; k.P = (int)P; k.Q = (int)Q;
    k.pad = (int)a.pad; k.Ct = (int)a.ct(); k.Kt = (int)a.kt(); k.Cp = (int)Cp;
    k.bands = (int)((a.H + TH - 1) / TH);
    k.TH = (int)((a.H + k.bands - 1) / k.bands);                      // bands of equal height (never more rows than TH: still fits)
    k.Wp = (int)Wp;
    k.cb_words = (int)cb_words_of(k.TH);
    k.cbw_magic = (uint32_t)((((uint64_t)1 << 32) / (uint64_t)k.cb_words) + 1);
    k.wd_magic = (uint32_t)((((uint64_t)1 << 32) / (uint64_t)a.Wd) + 1);
    k.q_magic = (uint32_t)((((uint64_t)1 << 32) / (uint64_t)Q) + 1);
    pl.lds = ((size_t)lds_of(k.TH) + 15) & ~(size_t)15;
    const int64_t grid = a.N * k.bands * (Cp / 64);
    if (grid >= ((int64_t)1 << 31)) return pl;
    pl.grid = (int)grid; pl.threads = (int)threads_of(k.TH);
    pl.ok = true;
    return pl;
}

template <int R, int S, int NT>
hipError_t launch_conv_dx_rows_nt(const DxRowsPlan &pl, hipStream_t s)
{
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_dx_rows_kernel<R, S, NT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((conv_dx_rows_kernel<R, S, NT>), dim3(pl.grid), dim3(NT), pl.lds, s, pl.k);
    return hipGetLastError();
}

template <int R, int S>
hipError_t launch_conv_dx_rows_as(const DxRowsPlan &pl, const float *W, hipStream_t s)
{
    const int Kp = (pl.k.K + CGR_KC - 1) / CGR_KC * CGR_KC;
    const int64_t total = (int64_t)Kp * R * S * pl.k.Cp;
    const int pb = (int)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(conv_dx_rows_prep_kernel, dim3(pb), dim3(256), 0, s, W, (float *)pl.k.Wt, pl.k.K, Kp, pl.k.C, R * S, pl.k.Cp, pl.k.gate);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return pl.threads == 256 ? launch_conv_dx_rows_nt<R, S, 256>(pl, s) : pl.threads == 512 ? launch_conv_dx_rows_nt<R, S, 512>(pl, s)
                                                                                            : launch_conv_dx_rows_nt<R, S, 1024>(pl, s);
}

}  // namespace

// conv_dw_rows_kernel's time as fixed + nonzeros * per_nnz, from its plan.  Fixed: ~8 us of launches, per unit of a
// workgroup's share ~2 us plus the X band at ~30 GB/s per CU, and the partial sums written and read at ~5 TB/s; per
// nonzero 2*64*R*S flop per 64-channel block at ~21 TFLOP/s (3x3; a 1x1 nonzero has one multiply-add per lane to pay for
// its decoding: ~3 TFLOP/s), scaled by the share of the 256 CUs that have a workgroup.  Measured against 13 layer shapes
// (8x8 to 56x56 planes, 64 to 1024 channels): the fixed part within 20 % (1x1: overestimated by up to 45 %).
bool conv_dw_rows_cost(const ConvArgs &a, int64_t P, int64_t Q, size_t avail, double *fixed_us, double *per_nnz_us)
{
    const DwRowsPlan pl = conv_dw_rows_plan(a, P, Q, avail);
    if (!pl.ok) return false;
    const double csb = a.x_dtype == DBP_I8 ? 68.0 : 260.0;
    const double dw_bytes = (double)(a.K * a.C * a.R * a.S) * 4.0;
    *fixed_us = 8.0 + pl.k.units_per_split * (2.0 + pl.k.cells * csb / 30.0e3) + (pl.k.n_split > 1 ? 2.0 * pl.k.n_split * dw_bytes / 5.0e6 : 0.0);
    const double util = pl.grid >= 256 ? 1.0 : pl.grid / 256.0;
    const double rate = (a.R * a.S >= 9 ? 21.0e6 : 3.0e6) * util;                                 // flop per microsecond
    *per_nnz_us = 2.0 * (double)((a.C + 63) / 64 * 64) * (double)(a.R * a.S) / rate;
    return true;
}

// Host-side walk of the plans above for one layer shape (no GPU call): every limit the kernels rely on, re-derived here from
// the plan's numbers.  0: consistent (or the shape takes the other kernels); otherwise the number of the violated invariant.
int check_conv_rows_plans(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad,
                          bool int8_x, size_t scratch_bytes)
{
    ConvArgs a{};
    a.codes = nullptr; a.x_dtype = int8_x ? DBP_I8 : DBP_F32;
    a.N = N; a.C = C; a.H = H; a.Wd = Wd; a.K = K; a.R = R; a.S = S; a.pad = pad; a.stride = stride;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    const DwRowsPlan w = conv_dw_rows_plan(a, P, Q, scratch_bytes);
    if (w.ok) {
        const ConvDwRowsArgs &k = w.k;
        const int64_t csb = int8_x ? 68 : 260;
        if (k.TH < 1 || (int64_t)k.bands * k.TH < P || (int64_t)(k.bands - 1) * k.TH >= P) return 1;     // the bands cover the code rows, none is empty
        if (k.THx != (k.TH - 1) * k.st + R || k.Wp != (Q - 1) * stride + S || k.cells != k.THx * k.Wp) return 2;
        if (k.n_chunks > CGR_MAX_CHUNKS || (int64_t)k.n_chunks * 64 < k.cells) return 3;
        if ((int64_t)k.TH * Q + 3 > 256 * CGR_MAX_LOADS) return 4;                                   // a band's codes fit the lanes' loads
        if ((size_t)k.cells * csb > w.lds || w.lds > kRowsLdsOne) return 5;
        if ((int64_t)k.n_split * k.units_per_split < k.units || (int64_t)(k.n_split - 1) * k.units_per_split >= k.units) return 6;
        if (w.partial_bytes > scratch_bytes) return 7;
        // the last X row and column a tile can ask for lie inside the zero halo the stager fills: tile row (TH-1)*st + R-1, column (Q-1)*st + S-1
        if ((k.TH - 1) * k.st + R - 1 >= k.THx || (Q - 1) * stride + S - 1 >= k.Wp) return 8;
        for (int64_t x = 0; x < (int64_t)k.TH * Q + 4; ++x)                                          // the reciprocal divides exactly over its range
            if ((int64_t)(((uint64_t)x * k.q_magic) >> 32) != x / Q) return 9;
        for (int64_t x = 0; x < (int64_t)k.n_chunks * 64; ++x)
            if ((int64_t)(((uint64_t)x * k.wp_magic) >> 32) != x / k.Wp) return 10;
        if ((int64_t)w.grid != ((C + 63) / 64) * ((K + CGR_KB - 1) / CGR_KB) * k.n_split) return 11;
    }
    const DxRowsPlan d = conv_dx_rows_plan(a, P, Q, scratch_bytes);
    if (d.ok) {
        const ConvDxRowsArgs &k = d.k;
        if (k.TH < 1 || k.TH > CGR_DX_MAX_ROWS || k.TH * 64 > d.threads || (int64_t)k.bands * k.TH < H || (int64_t)(k.bands - 1) * k.TH >= H) return 21;
        if (d.threads != 256 && d.threads != 512 && d.threads != 1024) return 22;
        const int64_t stretch = ((int64_t)k.TH + R - 1) * Q + 3;                                    // bytes of a plane a band can need, with the alignment slack
        if ((int64_t)k.cb_words * 4 < stretch || k.cb_words < 2) return 23;
        if ((int64_t)CGR_KC * k.cb_words > (int64_t)CGR_DX_CPT * d.threads) return 24;               // a chunk's codes fit the threads' loads
        const int64_t lds = (int64_t)k.TH * k.Wp * 65 * 4 + 2 * ((int64_t)CGR_KC * R * S * 64 * 4 + (int64_t)CGR_KC * k.cb_words * 4);
        if ((size_t)lds > d.lds || d.lds > (size_t)160 * 1024) return 25;
        if (k.Wp != Q + S - 1 || Wd - 1 + pad >= k.Wp) return 26;                                     // every pixel of a row has its cell
        if (d.prep_bytes > scratch_bytes || d.prep_bytes < (size_t)((K + CGR_KC - 1) / CGR_KC * CGR_KC * R * S * k.Cp) * 4) return 27;
        for (int64_t x = 0; x < stretch + 4; ++x)
            if ((int64_t)(((uint64_t)x * k.q_magic) >> 32) != x / Q) return 28;
        for (int64_t x = 0; x < (int64_t)CGR_KC * k.cb_words; ++x)
            if ((int64_t)(((uint64_t)x * k.cbw_magic) >> 32) != x / k.cb_words) return 29;
        for (int64_t x = 0; x < (int64_t)k.TH * Wd; ++x)
            if ((int64_t)(((uint64_t)x * k.wd_magic) >> 32) != x / Wd) return 30;
        if ((int64_t)d.grid != N * k.bands * (k.Cp / 64)) return 31;
    }
    return 0;
}

hipError_t launch_conv_gather(const ConvArgs &a, const FormatView &f, hipStream_t s)
{
    const int64_t P_ = (a.H + 2 * a.pad - a.R) / a.stride + 1, Q_ = (a.Wd + 2 * a.pad - a.S) / a.stride + 1;
    const Scale step_{a.step, a.step_dev};
    // scratch (optional): the dX kernel's prepared weights first, then the dW kernel's partial sums
    const bool have = a.scratch && (uintptr_t)a.scratch % 256 == 0;
    size_t used = 0;
    bool dx_done = false, dw_done = false;
    // Behind the density gate (flag set: both families are launched and the device picks one) the whole gather side only
    // runs beyond ~99.8 % zeros, where the kernels that walk the format's compacted entries have the smaller fixed cost (they
    // touch nothing but the entries); the kernels that scan the code planes win from there down to ~95 % zeros and serve the
    // explicit gather path and, with rows_gated, the dW-only middle state of the gate.
    const bool rows_kernels = a.gate.flag == nullptr || a.rows_gated;
    if (a.dX && rows_kernels) {
        DxRowsPlan pl = conv_dx_rows_plan(a, P_, Q_, have ? a.scratch_bytes : 0);
        if (pl.ok) {
            pl.k.codes = a.codes; pl.k.Wt = (const float *)a.scratch; pl.k.dX = a.dX; pl.k.scale = step_; pl.k.gate = a.gate;
            const hipError_t e = a.R == 3 ? launch_conv_dx_rows_as<3, 3>(pl, a.W, s) : launch_conv_dx_rows_as<1, 1>(pl, a.W, s);
            if (e != hipSuccess) return e;
            used = (pl.prep_bytes + 255) & ~(size_t)255;
            dx_done = true;
        }
    }
    if (a.dW && rows_kernels) {
        DwRowsPlan pl = conv_dw_rows_plan(a, P_, Q_, have && a.scratch_bytes > used ? a.scratch_bytes - used : 0);
        if (pl.ok) {
            ConvDwRowsArgs &k = pl.k;
            void *partial = have ? (char *)a.scratch + used : nullptr;
            k.codes = a.codes; k.X = a.X; k.out = k.n_split > 1 ? partial : a.dW; k.scale = step_; k.gate = a.gate;
            hipError_t e;
            if (a.x_dtype == DBP_F32) e = a.R == 3 ? launch_conv_dw_rows_as<float, 3, 3>(pl, s) : launch_conv_dw_rows_as<float, 1, 1>(pl, s);
            else                      e = a.R == 3 ? launch_conv_dw_rows_as<int8_t, 3, 3>(pl, s) : launch_conv_dw_rows_as<int8_t, 1, 1>(pl, s);
            if (e != hipSuccess) return e;
            if (k.n_split > 1) {
                const int64_t n = (int64_t)k.K * k.C * (int)(a.R * a.S);
                int zg = 1;                                           // threads per element: more where dW is small and the shares are many
                while (zg < 16 && k.n_split / (2 * zg) >= 8 && n * zg / 256 < 2048) zg *= 2;
                const int64_t blocks = (n * zg + 255) / 256;
                const int rb = (int)(blocks < 2048 ? blocks : 2048);
                if (a.x_dtype == DBP_F32)
                    hipLaunchKernelGGL(conv_dw_rows_reduce_kernel<float>, dim3(rb), dim3(256), 0, s, (const float *)partial, (float *)a.dW, n, k.n_split, zg, step_, a.gate);
                else
                    hipLaunchKernelGGL(conv_dw_rows_reduce_kernel<int32_t>, dim3(rb), dim3(256), 0, s, (const int32_t *)partial, (int32_t *)a.dW, n, k.n_split, zg, step_, a.gate);
                e = hipGetLastError();
                if (e != hipSuccess) return e;
            }
            dw_done = true;
        }
    }
    if ((dx_done || !a.dX) && (dw_done || !a.dW)) return hipSuccess;
    if (a.rows_gated) return hipErrorInvalidValue;                    // the caller planned on the plane-scanning kernels (no format was written)
    ConvGatherGeom g;
    g.N = (int)a.N; g.C = (int)a.C; g.H = (int)a.H; g.Wd = (int)a.Wd; g.K = (int)a.K; g.R = (int)a.R; g.S = (int)a.S;
    g.pad = (int)a.pad; g.st = (int)a.stride; g.gate = a.gate;
    g.Ct = (int)a.ct(); g.Kt = (int)a.kt(); g.k_first = (int)a.k_first;
    g.P = (int)((a.H + 2 * a.pad - a.R) / a.stride + 1); g.Q = (int)((a.Wd + 2 * a.pad - a.S) / a.stride + 1);
    const int RS = g.R * g.S, cpw_max = 64 / RS;
    const Scale step{a.step, a.step_dev};
    if (a.dX && !dx_done) {
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
    if (a.dW && !dw_done) {
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

// ---- host side of the fully connected gather path ---------------------------------------------------------
namespace {

constexpr int kGatherWorkgroups = 256;                  // one 1024-thread workgroup per CU

// Shapes fc_rows_kernel takes: 16-byte rows of the dense operand, 16-byte stores; dX also reads the codes as dwords.
bool fc_rows_dx_ok(const LinearArgs &a)
{
    return a.in % 4 == 0 && (uintptr_t)a.W % 16 == 0 && (uintptr_t)a.dX % 16 == 0 && a.out % 4 == 0 && (uintptr_t)a.codes % 4 == 0 &&
           a.B < (1ll << 31) - 256 && a.out < (1ll << 31) - 256 && a.in < (1ll << 31) - 256;
}
bool fc_rows_dw_ok(const LinearArgs &a)
{
    return a.x_dtype == DBP_F32 && a.in % 4 == 0 && (uintptr_t)a.X % 16 == 0 && (uintptr_t)a.dW % 16 == 0 &&
           a.B < (1ll << 31) - 256 && a.out < (1ll << 31) - 256 && a.in < (1ll << 31) - 256;
}

// Parts of one product over the chip: first over the row blocks, then (dX only: `blocks` > 0 counts the blocks of 256
// reduction indices) over the reduction, every reduction part writing a partial [rows][cols] that the reduction kernel
// sums.  `room`: bytes available for partials.
struct FcRowsPlan { int slabs, row_blocks, rparts, rb_per_part, sparts, ch_per_part; size_t partial_bytes; };
FcRowsPlan fc_rows_plan(int64_t rows, int64_t cols, int64_t n_chunks, bool may_split, size_t room)
{
    FcRowsPlan pl;
    const int block_rows = FR_WAVES * (may_split ? FR_RW_DX : FR_RW_DW), slab = 64 * (may_split ? FR_CPL_DX : FR_CPL_DW);
    pl.slabs = (int)((cols + slab - 1) / slab);
    pl.row_blocks = (int)((rows + block_rows - 1) / block_rows);
    int64_t want = kGatherWorkgroups / pl.slabs;
    if (want < 1) want = 1;
    int64_t rparts = want < pl.row_blocks ? want : pl.row_blocks;
    pl.rb_per_part = (int)((pl.row_blocks + rparts - 1) / rparts);
    pl.rparts = (pl.row_blocks + pl.rb_per_part - 1) / pl.rb_per_part;
    int64_t sparts = 1;
    if (may_split) {
        const int64_t blocks = n_chunks;
        sparts = want / pl.rparts;
        if (sparts > blocks) sparts = blocks;
        if (sparts < 1) sparts = 1;
        while (sparts > 1 && (size_t)sparts * rows * cols * sizeof(float) > room) --sparts;
        const int64_t bps = (blocks + sparts - 1) / sparts;
        sparts = (blocks + bps - 1) / bps;
        pl.ch_per_part = (int)bps;
    } else {
        pl.ch_per_part = (int)n_chunks;
    }
    pl.sparts = (int)sparts;
    pl.partial_bytes = sparts > 1 ? (size_t)sparts * rows * cols * sizeof(float) : 0;
    return pl;
}

}  // namespace

size_t linear_gather_scratch_bytes(int64_t B, int64_t in, int64_t out)
{
    return fc_rows_plan(B, in, (out + FR_CH - 1) / FR_CH, true, (size_t)-1).partial_bytes;
}

void linear_gather_shape(int64_t B, int64_t in, int64_t out, GatherShape (&gs)[2])
{
    const int64_t cx = (out + FR_CH - 1) / FR_CH, cw = (B + FR_CH - 1) / FR_CH;
    const FcRowsPlan px = fc_rows_plan(B, in, cx, true, (size_t)-1), pw = fc_rows_plan(out, in, cw, false, 0);
    gs[0] = GatherShape{(int64_t)px.slabs * px.rparts * px.sparts, (int64_t)px.rb_per_part * px.ch_per_part, px.partial_bytes};
    gs[1] = GatherShape{(int64_t)pw.slabs * pw.rparts, (int64_t)pw.rb_per_part * cw, 0};
}

bool linear_gather_supported(int64_t B, int64_t in, int64_t out)
{
    (void)in;
    return B <= 65535 && out <= 65535;                    // the one-row-per-workgroup kernels index workgroups by row
}

bool linear_gather_gated_ok(const LinearArgs &a)
{
    return (!a.dX || fc_rows_dx_ok(a)) && (!a.dW || fc_rows_dw_ok(a));
}

hipError_t launch_linear_gather(const LinearArgs &a, const FormatView &f, hipStream_t s)
{
    const int B = (int)a.B, in = (int)a.in, out = (int)a.out;
    static bool raised = false;
    if (!raised) {
        const void *fns[4] = {reinterpret_cast<const void *>(&fc_rows_kernel<false, FR_RW_DX, FR_CPL_DX, true, 4>),
                              reinterpret_cast<const void *>(&fc_rows_kernel<true, FR_RW_DW, FR_CPL_DW, false, 16>),
                              reinterpret_cast<const void *>(&fc_rows_kernel<true, FR_RW_DW, FR_CPL_DW, false, 4>),
                              reinterpret_cast<const void *>(&fc_rows_kernel<true, FR_RW_DW, FR_CPL_DW, false, 1>)};
        for (int i = 0; i < 4; ++i) {
            hipError_t e = hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)fr_lds_bytes(i ? FR_CPL_DW : FR_CPL_DX, i ? FR_RW_DW : FR_RW_DX, i != 0));
            if (e != hipSuccess) return e;
        }
        raised = true;
    }
    const Scale scale{a.step, a.step_dev};
    const dim3 block(256);
    const unsigned slabs = (unsigned)((in + kSlab - 1) / kSlab);
    if (a.dX && fc_rows_dx_ok(a)) {
        const int n_chunks = (int)((a.out + FR_CH - 1) / FR_CH);
        const FcRowsPlan pl = fc_rows_plan(a.B, a.in, n_chunks, true, a.scratch ? a.scratch_bytes : 0);
        FcRowsArgs k;
        k.codes = a.codes; k.ldc = a.out; k.D = a.W; k.ldd = a.in; k.out = a.dX; k.partial = (float *)a.scratch;
        k.rows = B; k.red = out; k.cols = in;
        k.slabs = pl.slabs; k.row_blocks = pl.row_blocks; k.n_chunks = n_chunks;
        k.rparts = pl.rparts; k.rb_per_part = pl.rb_per_part; k.sparts = pl.sparts; k.ch_per_part = pl.ch_per_part;
        k.scale = scale; k.gate = a.gate;
        hipLaunchKernelGGL((fc_rows_kernel<false, FR_RW_DX, FR_CPL_DX, true, 4>), dim3((unsigned)(k.slabs * k.rparts * k.sparts)), dim3(FR_THREADS), fr_lds_bytes(FR_CPL_DX, FR_RW_DX, false), s, k);
        if (pl.sparts > 1) {
            const int64_t n4 = (int64_t)B * in / 4;
            const int rb = (int)((n4 + 255) / 256 < 2048 ? (n4 + 255) / 256 : 2048);
            hipLaunchKernelGGL(fc_rows_reduce_kernel, dim3(rb), dim3(256), 0, s, (const float *)a.scratch, a.dX, n4, pl.sparts, scale, a.gate);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    } else if (a.dX) {
        if (a.gate.flag) return hipErrorInvalidValue;     // the fallback kernels take no gate
        if (B > 65535) return hipErrorInvalidValue;
        const bool vec = in % 4 == 0 && ((uintptr_t)a.W % 16) == 0;
        if (vec) hipLaunchKernelGGL(linear_dx_gather_kernel<true>, dim3(slabs, B), block, 0, s, f, a.W, a.dX, in, out, scale);
        else     hipLaunchKernelGGL(linear_dx_gather_kernel<false>, dim3(slabs, B), block, 0, s, f, a.W, a.dX, in, out, scale);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (a.dW && fc_rows_dw_ok(a)) {
        const int n_chunks = (B + FR_CH - 1) / FR_CH;
        const FcRowsPlan pl = fc_rows_plan(a.out, a.in, n_chunks, false, 0);
        FcRowsArgs k;
        k.codes = a.codes; k.ldc = a.out; k.D = (const float *)a.X; k.ldd = a.in; k.out = (float *)a.dW; k.partial = nullptr;
        k.rows = out; k.red = B; k.cols = in;
        k.slabs = pl.slabs; k.row_blocks = pl.row_blocks; k.n_chunks = n_chunks;
        const int code_align = (a.out % 16 == 0 && (uintptr_t)a.codes % 16 == 0) ? 16 : (a.out % 4 == 0 && (uintptr_t)a.codes % 4 == 0) ? 4 : 1;
        k.rparts = pl.rparts; k.rb_per_part = pl.rb_per_part; k.sparts = 1; k.ch_per_part = n_chunks;
        k.scale = scale; k.gate = a.gate;
        const dim3 grid((unsigned)(k.slabs * k.rparts));
        if (code_align == 16)     hipLaunchKernelGGL((fc_rows_kernel<true, FR_RW_DW, FR_CPL_DW, false, 16>), grid, dim3(FR_THREADS), fr_lds_bytes(FR_CPL_DW, FR_RW_DW, true), s, k);
        else if (code_align == 4) hipLaunchKernelGGL((fc_rows_kernel<true, FR_RW_DW, FR_CPL_DW, false, 4>), grid, dim3(FR_THREADS), fr_lds_bytes(FR_CPL_DW, FR_RW_DW, true), s, k);
        else                      hipLaunchKernelGGL((fc_rows_kernel<true, FR_RW_DW, FR_CPL_DW, false, 1>), grid, dim3(FR_THREADS), fr_lds_bytes(FR_CPL_DW, FR_RW_DW, true), s, k);
        return hipGetLastError();
    }
    if (a.dW) {
        if (a.gate.flag) return hipErrorInvalidValue;
        if (out > 65535) return hipErrorInvalidValue;
        if (a.x_dtype == DBP_F32) {
            const bool vec = in % 4 == 0 && ((uintptr_t)a.X % 16) == 0;
            if (vec) hipLaunchKernelGGL((linear_dw_gather_kernel<float, float, true>), dim3(slabs, out), block, 0, s,
                                        a.codes, (const float *)a.X, (float *)a.dW, B, in, out, scale);
            else     hipLaunchKernelGGL((linear_dw_gather_kernel<float, float, false>), dim3(slabs, out), block, 0, s,
                                        a.codes, (const float *)a.X, (float *)a.dW, B, in, out, scale);
        } else {
            const bool vec = in % 4 == 0 && ((uintptr_t)a.X % 4) == 0;
            if (vec) hipLaunchKernelGGL((linear_dw_gather_kernel<int8_t, int32_t, true>), dim3(slabs, out), block, 0, s,
                                        a.codes, (const int8_t *)a.X, (int32_t *)a.dW, B, in, out, scale);
            else     hipLaunchKernelGGL((linear_dw_gather_kernel<int8_t, int32_t, false>), dim3(slabs, out), block, 0, s,
                                        a.codes, (const int8_t *)a.X, (int32_t *)a.dW, B, in, out, scale);
        }
        return hipGetLastError();
    }
    return hipSuccess;
}

}  // namespace dbp

extern "C" int dbp_plan_check_conv2d_gather(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride,
                                            int64_t pad, int int8_x, size_t scratch_bytes)
{
    if (N <= 0 || C <= 0 || H <= 0 || Wd <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0 || H + 2 * pad < R || Wd + 2 * pad < S) return -1;
    if (N > 65535 || C > 65535 || K > 65535 || H > 65535 || Wd > 65535 || R > 255 || S > 255 || pad > 255 || stride > 255) return -1;
    return dbp::check_conv_rows_plans(N, C, H, Wd, K, R, S, stride, pad, int8_x != 0, scratch_bytes);
}
