// NSD pass: fused dither + quantise + int8 codes + tile-sparse format + statistics.
//
// Eq. (nsd) of the paper, applied elementwise to the preactivation gradient as in Eq. (qdz):
//   k = floor(x/Delta + u),  u = nu/Delta + 1/2 in (0,1)  <=>  q = Delta*floor((x+nu)/Delta + 1/2).
// The kernel is HBM-bound: 4 B read + 1 B code + 1/8 B bitmap + 2 B per nonzero per element.
//
// Work decomposition: one wavefront owns one 256-column tile of one row per loop iteration.
// Lane l holds the 4 consecutive columns 4l..4l+3 (one 16-byte load, one 4-byte code store), so a
// tile is a single fully coalesced 1 KiB read.  The nonzero flags of the four sub-columns are
// wave ballots (free by-products of the compares); their popcounts give the tile count and, via
// mbcnt, each lane's exclusive prefix, so compaction needs neither LDS nor atomics.  The four
// ballots are bit-interleaved into the natural column order of the bitmap on the scalar unit.
#include "common.h"

namespace dbp {

namespace {

constexpr uint32_t kG = 0x9E3779B9u, kA = 0x6A09E667u, kC = 0xBB67AE85u;

__host__ __device__ inline uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= kA; x ^= x >> 15; x *= kC; x ^= x >> 16;
    return x;
}

// One 32-bit hash word per PAIR of elements; `k1c` already contains k1 + hi32(counter)*C.
__device__ __forceinline__ uint32_t hash_word(uint32_t counter_lo, uint32_t k0, uint32_t k1c)
{
    uint32_t h = (counter_lo ^ k0) * kG;
    h ^= h >> 16;
    h = (h + k1c) * kA;
    h ^= h >> 15;
    h *= kC;
    h ^= h >> 16;
    return h;
}

// u = (2m+1) * 2^-17 for a 16-bit m: build 1 + m*2^-16 in the mantissa, subtract (1 - 2^-17). Exact.
__device__ __forceinline__ float dither_from_m16(uint32_t m)
{
    return __uint_as_float(0x3F800000u | (m << 7)) - 0x1.ffffp-1f;
}

__device__ __forceinline__ float dither_u(uint64_t g, uint32_t k0, uint32_t k1)
{
    uint64_t c = g >> 1;
    uint32_t h = hash_word((uint32_t)c, k0, k1 + (uint32_t)(c >> 32) * kC);
    return dither_from_m16((g & 1) ? (h >> 16) : (h & 0xFFFFu));
}

// Scalar-unit bit doubling: each of the low 32 bits of x appears twice in the result.
__device__ __forceinline__ uint64_t bit_double(uint32_t x)
{
    uint64_t r;
    asm("s_bitreplicate_b64_b32 %0, %1" : "=s"(r) : "s"(x));
    return r;
}

// Bitmap word of 64 consecutive in-tile columns from the 16-bit slices of the four sub-column
// ballots: bit 4i+j = bj[i].  Two rounds of pairwise interleaving (a,c then b,d), all on SGPRs.
__device__ __forceinline__ uint64_t interleave4(uint32_t b0, uint32_t b1, uint32_t b2, uint32_t b3)
{
    const uint32_t p = ((uint32_t)bit_double(b0) & 0x55555555u) | ((uint32_t)bit_double(b2) & 0xAAAAAAAAu);
    const uint32_t q = ((uint32_t)bit_double(b1) & 0x55555555u) | ((uint32_t)bit_double(b3) & 0xAAAAAAAAu);
    return (bit_double(p) & 0x5555555555555555ull) | (bit_double(q) & 0xAAAAAAAAAAAAAAAAull);
}

struct WaveStats { uint32_t nnz, sat, nonfinite; float maxabs; };

// Quantise one element given its dither; returns the clamped code.
__device__ __forceinline__ int quantise(float x, float inv, float u, float &kf_out)
{
    float t  = __builtin_fmaf(x, inv, u);
    float kf = __builtin_floorf(t);
    kf_out   = kf;
    float kc = fminf(fmaxf(kf, -127.0f), 127.0f);     // NaN -> -127 here; fixed up by the caller
    return (int)kc;
}

template <bool VEC>
__global__ __launch_bounds__(256) void nsd_kernel(NsdArgs a)
{
    const int lane = threadIdx.x & 63;
    const int wave_in_block = threadIdx.x >> 6;
    const int64_t wave0 = (int64_t)blockIdx.x * 4 + wave_in_block;
    const int64_t n_waves = (int64_t)gridDim.x * 4;
    const float inv = a.inv_step;

    WaveStats ws = {0u, 0u, 0u, 0.0f};

    for (int64_t t = wave0; t < a.n_tiles; t += n_waves) {
        const int64_t row  = t / a.tiles_per_row;
        const int64_t seg  = t - row * a.tiles_per_row;
        const int64_t col0 = seg * DBP_TILE;
        const int valid    = (int)min((int64_t)DBP_TILE, a.cols - col0);
        const int64_t j0   = row * a.cols + col0 + 4 * lane;         // flat index of this lane's first element
        const int c_in     = 4 * lane;                               // in-tile column of that element

        float x[4] = {0.f, 0.f, 0.f, 0.f};
        if (VEC) {
            if (c_in < valid) {
                f32x4 v = __builtin_nontemporal_load((const f32x4 *)(a.delta + j0));
                x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (c_in + j < valid) x[j] = __builtin_nontemporal_load(a.delta + j0 + j);
        }

        // dither: elements share hash words pairwise by the parity of the GLOBAL index
        const uint64_t g0 = a.idx_base + (uint64_t)j0;
        float u[4];
        if (VEC && !(a.idx_base & 1)) {
            const uint64_t c0 = g0 >> 1;                              // g0 is even here
            const uint32_t k1a = a.k1 + (uint32_t)(c0 >> 32) * kC;
            const uint32_t k1b = a.k1 + (uint32_t)((c0 + 1) >> 32) * kC;
            const uint32_t hA = hash_word((uint32_t)c0, a.k0, k1a);
            const uint32_t hB = hash_word((uint32_t)(c0 + 1), a.k0, k1b);
            u[0] = dither_from_m16(hA & 0xFFFFu); u[1] = dither_from_m16(hA >> 16);
            u[2] = dither_from_m16(hB & 0xFFFFu); u[3] = dither_from_m16(hB >> 16);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) u[j] = dither_u(g0 + j, a.k0, a.k1);
        }

        int k[4];
        float kf[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) k[j] = quantise(x[j], inv, u[j], kf[j]);

        // rare cases, decided per wave: non-finite inputs and saturation
        const float m4 = fmaxf(fmaxf(fabsf(kf[0]), fabsf(kf[1])), fmaxf(fabsf(kf[2]), fabsf(kf[3])));
        const bool weird = (x[0] != x[0]) | (x[1] != x[1]) | (x[2] != x[2]) | (x[3] != x[3]) | !(m4 <= 127.0f);
        if (__builtin_amdgcn_ballot_w64(weird)) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool nan = x[j] != x[j];
                const bool inf = fabsf(x[j]) == __builtin_inff();
                if (nan) k[j] = 0;
                ws.nonfinite += __builtin_popcountll(__builtin_amdgcn_ballot_w64(nan | inf));
                ws.sat += __builtin_popcountll(__builtin_amdgcn_ballot_w64(!nan && fabsf(kf[j]) > 127.0f));
            }
        }
        ws.maxabs = fmaxf(ws.maxabs, fminf(m4, 127.0f));             // fmaxf/fminf drop NaN operands

        // codes
        const uint32_t packed = (uint32_t)(k[0] & 0xFF) | ((uint32_t)(k[1] & 0xFF) << 8) |
                                ((uint32_t)(k[2] & 0xFF) << 16) | ((uint32_t)(k[3] & 0xFF) << 24);
        if (VEC) {
            if (c_in < valid) __builtin_nontemporal_store(packed, (uint32_t *)(a.codes + j0));
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (c_in + j < valid) a.codes[j0 + j] = (int8_t)k[j];
        }

        // tile-sparse format
        const uint64_t b0 = __builtin_amdgcn_ballot_w64(k[0] != 0);
        const uint64_t b1 = __builtin_amdgcn_ballot_w64(k[1] != 0);
        const uint64_t b2 = __builtin_amdgcn_ballot_w64(k[2] != 0);
        const uint64_t b3 = __builtin_amdgcn_ballot_w64(k[3] != 0);
        const uint32_t cnt = __builtin_popcountll(b0) + __builtin_popcountll(b1) +
                             __builtin_popcountll(b2) + __builtin_popcountll(b3);
        ws.nnz += cnt;
        if (a.bitmap) {
            uint32_t pre = 0;                                          // nonzeros in lower lanes
            pre = __builtin_amdgcn_mbcnt_hi((uint32_t)(b0 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b0, pre));
            pre = __builtin_amdgcn_mbcnt_hi((uint32_t)(b1 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b1, pre));
            pre = __builtin_amdgcn_mbcnt_hi((uint32_t)(b2 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b2, pre));
            pre = __builtin_amdgcn_mbcnt_hi((uint32_t)(b3 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b3, pre));
            uint16_t *ent = a.entries + t * DBP_TILE;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (k[j] != 0) {
                    ent[pre] = (uint16_t)(((c_in + j) << 8) | (k[j] & 0xFF));
                    ++pre;
                }
            }
            // word w covers in-tile columns 64w..64w+63 = lanes 16w..16w+15, 4 sub-columns each
            uint64_t w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] = interleave4((uint32_t)(b0 >> (16 * i)) & 0xFFFFu, (uint32_t)(b1 >> (16 * i)) & 0xFFFFu,
                                   (uint32_t)(b2 >> (16 * i)) & 0xFFFFu, (uint32_t)(b3 >> (16 * i)) & 0xFFFFu);
            if (lane < 4) a.bitmap[t * 4 + lane] = lane == 0 ? w[0] : lane == 1 ? w[1] : lane == 2 ? w[2] : w[3];
            if (lane == 0) a.tile_nnz[t] = (uint16_t)cnt;
        }
    }

    if (a.stats) {
        // wave-level maxima and sums (sums are already wave-uniform), then one atomic set per block
        float mx = ws.maxabs;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        __shared__ uint32_t s_nnz[4], s_sat[4], s_nf[4];
        __shared__ int s_mx[4];
        if (lane == 0) { s_nnz[wave_in_block] = ws.nnz; s_sat[wave_in_block] = ws.sat;
                         s_nf[wave_in_block] = ws.nonfinite; s_mx[wave_in_block] = (int)mx; }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint64_t nnz = (uint64_t)s_nnz[0] + s_nnz[1] + s_nnz[2] + s_nnz[3];
            uint64_t sat = (uint64_t)s_sat[0] + s_sat[1] + s_sat[2] + s_sat[3];
            uint64_t nf  = (uint64_t)s_nf[0] + s_nf[1] + s_nf[2] + s_nf[3];
            int m = max(max(s_mx[0], s_mx[1]), max(s_mx[2], s_mx[3]));
            if (nnz) atomicAdd((unsigned long long *)&a.stats->nnz, (unsigned long long)nnz);
            if (sat) atomicAdd((unsigned long long *)&a.stats->n_saturated, (unsigned long long)sat);
            if (nf)  atomicAdd((unsigned long long *)&a.stats->n_nonfinite, (unsigned long long)nf);
            if (m)   atomicMax(&a.stats->max_abs_code, m);
        }
    }
}

__global__ void zero_stats_kernel(dbp_stats *s)
{
    if (threadIdx.x == 0) { s->nnz = 0; s->n_saturated = 0; s->n_nonfinite = 0; s->max_abs_code = 0; s->reserved = 0; }
}

}  // namespace

DitherKeys make_dither_keys(uint64_t seed)
{
    DitherKeys k;
    k.k0 = mix32((uint32_t)seed ^ kG);
    k.k1 = mix32((uint32_t)(seed >> 32) + k.k0 + kA);
    return k;
}

hipError_t launch_nsd(const NsdArgs &a, hipStream_t s)
{
    if (a.stats) hipLaunchKernelGGL(zero_stats_kernel, dim3(1), dim3(64), 0, s, a.stats);
    // per-wave element counts are 32-bit: cap the tiles one wave can see well below 2^32/256
    int64_t blocks = (a.n_tiles + 3) / 4;
    const int64_t max_blocks = 256 * 8;                    // 8 resident workgroups per CU
    if (blocks > max_blocks) blocks = max_blocks;
    if (blocks < 1) blocks = 1;
    const bool vec = (a.cols % 4 == 0) && ((uintptr_t)a.delta % 16 == 0) && ((uintptr_t)a.codes % 4 == 0);
    if (vec) hipLaunchKernelGGL(nsd_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    else     hipLaunchKernelGGL(nsd_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace dbp
