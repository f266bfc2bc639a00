// Curvature of float32 activations on the f16 MFMA: x s = a + b / 2^11 with two float16 terms
// (a = f16(x s), b = f16((x s - a) 2^11): 2 x 11 significand bits; s, a power of two, brings the largest
// magnitude of the tensor to [2^14, 2^15), so that both terms are normal float16 numbers for every element
// down to 2^-28 of the largest), and a product of two values as the three f16 products
//     x y s s' ~=  a a' + (a b' + b a') / 2^11,
// what is left out being below 2^-22 |x y| (with random signs from token to token: 5e-8 of the factor after
// 4096 tokens).  The f16 MFMA has the rate of the bf16 one, so this is half the matrix-core work of the
// three-term bfloat16 split of split3_syrk256.h; the price is a pass over x for its largest magnitude.
//
//   split2_amax_kernel    largest |x| of every item (atomic maximum on the bits of |x|)
//   split2_pack_kernel    the two terms as two planes in the k-interleaved layout of the bf16 kernels
//   curvature_syrk_split2_256_kernel
//                         three sweeps of the packed-plane K loop (s3_pass_planes) into the same accumulators:
//                         a b', b a' (the small products first, see split3_syrk256.h), the accumulators
//                         times 2^-11, then a a'; the epilogue applies alpha / s^2.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "split3_syrk256.h"

namespace kfac {

constexpr int S2_PLANES = 2;
constexpr int S2_LOW_SHIFT = 11;  // the second term is stored times 2^11

// s = 2^(14 - floor(log2(amax))) from the bits of amax (>= 0).  Zero and subnormal maxima: s = 1 (the
// tensor is all zeros as far as float16 terms can tell the difference); infinity / NaN: NaN, and so is the factor.
__host__ __device__ inline float split2_scale(unsigned amax_bits)
{
    const int e = (int)(amax_bits >> 23) & 0xff;
    if (e == 0) return 1.f;
    if (e == 0xff) return __builtin_nanf("");
    const int es = 127 + 14 - (e - 127);  // biased exponent of s
    if (es <= 0) return 0x1p-126f;        // amax >= 2^141: out of float32 range anyway
    if (es >= 255) return 0x1p127f;
    unsigned bits = (unsigned)es << 23;
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_bit_cast(float, bits);
#else
    float f;
    __builtin_memcpy(&f, &bits, 4);
    return f;
#endif
}

struct Split2Item {
    const float *x;       // [n, d] float32, ldx
    unsigned short *dst;  // [2][gp][dp][8]
    int n, d, ldx, dp, gp, pad_;
};
struct Split2Launch {
    Split2Item it[PACK_MAX_ITEMS];
    int first_wg[PACK_MAX_ITEMS + 1];  // workgroups of item i: first_wg[i] .. first_wg[i+1]-1
    unsigned *amax;                    // bits of the largest |x| per item
    int count;
};

constexpr int S2P_COLS = 256;        // columns per workgroup: one per thread
constexpr int S2A_GROUPS = 8;        // k-groups (of 8 tokens) per workgroup of the amax kernel

__global__ __launch_bounds__(256) void split2_clear_kernel(unsigned *amax, int count)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < count) amax[i] = 0u;
}

__device__ inline int split2_find_item(const Split2Launch &pl, int wg)
{
    int i = 0, hi = pl.count;
    while (hi - i > 1) {
        const int mid = (i + hi) >> 1;
        if (pl.first_wg[mid] <= wg)
            i = mid;
        else
            hi = mid;
    }
    return i;
}

// first_wg counts (dp / 256) x ceil(gp / S2A_GROUPS) workgroups per item here.  A workgroup scans 256 columns of
// S2A_GROUPS x 8 = 64 tokens: a wave takes 16 token rows, a lane 4 columns of each (16-byte reads, 1 KB per
// wave and row).
__global__ __launch_bounds__(256) void split2_amax_kernel(const Split2Launch pl)
{
    const int i = split2_find_item(pl, blockIdx.x);
    const Split2Item &it = pl.it[i];
    const int w = blockIdx.x - pl.first_wg[i], cb = it.dp / S2P_COLS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int ROWS = S2A_GROUPS * BF_KG / 4;  // per wave
    const int col = (w % cb) * S2P_COLS + 4 * lane, k0 = (w / cb) * S2A_GROUPS * BF_KG + wave * ROWS;
    const bool vec = ((it.ldx & 3) == 0) && ((reinterpret_cast<uintptr_t>(it.x) & 15) == 0);
    unsigned m = 0u;
    if (col < it.d && k0 < it.n) {
        const float *src = it.x + (size_t)k0 * it.ldx + col;
        if (vec && col + 4 <= it.d && k0 + ROWS <= it.n) {
            float4 v[ROWS];
#pragma unroll
            for (int r = 0; r < ROWS; ++r) v[r] = *reinterpret_cast<const float4 *>(src + (size_t)r * it.ldx);
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                m = max(m, __builtin_bit_cast(unsigned, v[r].x) & 0x7fffffffu);
                m = max(m, __builtin_bit_cast(unsigned, v[r].y) & 0x7fffffffu);
                m = max(m, __builtin_bit_cast(unsigned, v[r].z) & 0x7fffffffu);
                m = max(m, __builtin_bit_cast(unsigned, v[r].w) & 0x7fffffffu);
            }
        } else {
            for (int r = 0; r < ROWS && k0 + r < it.n; ++r)
                for (int e = 0; e < 4 && col + e < it.d; ++e)
                    m = max(m, __builtin_bit_cast(unsigned, src[(size_t)r * it.ldx + e]) & 0x7fffffffu);
        }
    }
    // the bits of non-negative floats order like the floats (NaNs above infinity)
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, o));
    // most waves find nothing larger than what is already there: look before taking the atomic (atomics on one
    // address are served one after the other; a stale smaller value only costs an atomic that changes nothing)
    if (lane == 0 && m > __hip_atomic_load(pl.amax + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(pl.amax + i, m);
}

// first_wg counts (dp / 256) x gp workgroups per item here: one thread takes one column of a k-group
__global__ __launch_bounds__(256) void split2_pack_kernel(const Split2Launch pl)
{
    const int i = split2_find_item(pl, blockIdx.x);
    const Split2Item &it = pl.it[i];
    const int w = blockIdx.x - pl.first_wg[i], cb = it.dp / S2P_COLS;
    const int col = (w % cb) * S2P_COLS + threadIdx.x, g0 = w / cb;
    const float s = split2_scale(pl.amax[i]);
    float v[BF_KG];
    const float *src = it.x + (size_t)g0 * BF_KG * it.ldx + col;
    if (col < it.d && (g0 + 1) * BF_KG <= it.n) {
#pragma unroll
        for (int r = 0; r < BF_KG; ++r) v[r] = src[(size_t)r * it.ldx];
    } else {
#pragma unroll
        for (int r = 0; r < BF_KG; ++r) v[r] = (col < it.d && g0 * BF_KG + r < it.n) ? src[(size_t)r * it.ldx] : 0.f;
    }
    unsigned a[BF_KG], b[BF_KG];
#pragma unroll
    for (int r = 0; r < BF_KG; ++r) {
        const float xs = v[r] * s;  // exact
        const _Float16 ha = static_cast<_Float16>(xs);
        const float r1 = xs - static_cast<float>(ha);  // exact
        const _Float16 hb = static_cast<_Float16>(r1 * (float)(1 << S2_LOW_SHIFT));
        a[r] = (unsigned)__builtin_bit_cast(unsigned short, ha);
        b[r] = (unsigned)__builtin_bit_cast(unsigned short, hb);
    }
    const size_t plane = (size_t)it.gp * it.dp * 8;  // elements
    unsigned short *dst = it.dst + ((size_t)g0 * it.dp + col) * 8;
    *reinterpret_cast<uint4 *>(dst) =
        make_uint4(a[0] | (a[1] << 16), a[2] | (a[3] << 16), a[4] | (a[5] << 16), a[6] | (a[7] << 16));
    *reinterpret_cast<uint4 *>(dst + plane) =
        make_uint4(b[0] | (b[1] << 16), b[2] | (b[3] << 16), b[4] | (b[5] << 16), b[6] | (b[7] << 16));
}

// Descriptor as for split3: x = plane a (at the first k-group of this launch's share of the tokens), n = padded
// tokens of the share, ldx = padded columns, pad_ = k-groups of a whole plane.  amax[i] belongs to problem i.
struct Syrk256LaunchScaled {
    Syrk256Launch l;
    const unsigned *amax;
    int amax_index[SYRK_MAX_PROBLEMS];
};

template <int MODE>
__device__ __forceinline__ void s2_mainloop(const SyrkProblem &pr, int m0, int n0, const char *lds_a, const char *lds_b,
                                            floatx16 (&acc)[4][4])
{
    const size_t row_bytes = (size_t)pr.ldx * 16;
    const int groups = pr.n / BF_KG;
    const char *pa = static_cast<const char *>(pr.x);
    const char *pb = pa + (size_t)pr.pad_ * row_bytes;
    s3_pass_planes<MODE, true>(pa, pb, row_bytes, row_bytes, groups, m0, n0, lds_a, lds_b, acc);  // a b'
    __syncthreads();
    s3_pass_planes<MODE, true>(pb, pa, row_bytes, row_bytes, groups, m0, n0, lds_a, lds_b, acc);  // b a'
    if (MODE != S3_WAVE_IDLE) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] *= 1.f / (float)(1 << S2_LOW_SHIFT);
    }
    __syncthreads();
    s3_pass_planes<MODE, true>(pa, pa, row_bytes, row_bytes, groups, m0, n0, lds_a, lds_b, acc);  // a a'
}

__global__ __launch_bounds__(256, 1) void curvature_syrk_split2_256_kernel(const Syrk256LaunchScaled ls)
{
    __shared__ __attribute__((aligned(16))) char lds_a[B2_STAGES * B2_STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char lds_b[B2_STAGES * B2_STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;

    const B2Tile bt = b2_locate(ls.l);
    const SyrkProblem &pr = ls.l.p[bt.pi];
    const int m0 = bt.m0, n0 = bt.n0;

    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    if (bt.diag && wave_s == 1) {
        s2_mainloop<S3_WAVE_IDLE>(pr, m0, n0, lds_a, lds_b, acc);
        return;
    }
    if (bt.diag && wave_s != 2)
        s2_mainloop<S3_WAVE_LOWER>(pr, m0, n0, lds_a, lds_b, acc);
    else
        s2_mainloop<S3_WAVE_FULL>(pr, m0, n0, lds_a, lds_b, acc);
    const float s = split2_scale(ls.amax[ls.amax_index[bt.pi]]);
    const float inv_s2 = (1.f / s) * (1.f / s);  // exact: s is a power of two
    b2_store_batched(acc, pr, ls.l.alpha * inv_s2, ls.l.beta, m0, n0, wm, wn, li, lh, bt.diag);
}

// ---------------------------------------------------------------------------
// General product C = A^T B on operands split the same way (both [K, columns] row-major before the split:
// the layout the precondition's two products have), for kfac_precondition_grouped_f16x2.  256 x 256 tiles of
// the full output, the same three sweeps, C = acc / (s_A s_B).
struct Gemm2Problem {
    const void *xa, *xb;  // plane a of each operand; plane b follows `groups` k-groups later
    float *c;             // [m, n], ldc
    int m, n, groups;     // groups: padded K / 8
    int dpa, dpb;         // padded columns of the operands
    int ldc;
    int tile_begin;
    int amax_a, amax_b;   // index of each operand's largest magnitude
    int pad_;
};
constexpr int GEMM2_MAX_PROBLEMS = 48;
struct Gemm2Launch {
    Gemm2Problem p[GEMM2_MAX_PROBLEMS];
    const unsigned *amax_a, *amax_b;  // the words of the A operands / of the B operands
    int count, total_tiles;
};

// Which tile a workgroup takes: XCD x (workgroups go round the eight XCDs) takes an eighth of the tiles of every
// problem, problem after problem, the eighth rotating from problem to problem.  The problems differ in K (the
// layer's width), so every XCD gets the same mix, and with the problems sorted by decreasing K on the host
// each starts its long tiles first.  -1: surplus workgroup (the grid is 8 x the longest XCD share).
__host__ __device__ inline int gemm2_share(int n, int xcd, int p, int &lo)
{
    const int part = (xcd + p) & 7;
    lo = (int)((long long)n * part / 8);
    return (int)((long long)n * (part + 1) / 8) - lo;
}
__device__ inline int gemm2_tile_of(const Gemm2Launch &lp, int bid)
{
    const int xcd = bid & 7;
    int q = bid >> 3;
    for (int p = 0; p < lp.count; ++p) {
        const int b = lp.p[p].tile_begin;
        const int n = (p + 1 < lp.count ? lp.p[p + 1].tile_begin : lp.total_tiles) - b;
        int lo;
        const int share = gemm2_share(n, xcd, p, lo);
        if (q < share) return b + lo + q;
        q -= share;
    }
    return -1;
}
inline int gemm2_grid(const Gemm2Launch &lp)
{
    int longest = 0;
    for (int x = 0; x < 8; ++x) {
        int have = 0;
        for (int p = 0; p < lp.count; ++p) {
            const int n = (p + 1 < lp.count ? lp.p[p + 1].tile_begin : lp.total_tiles) - lp.p[p].tile_begin;
            int lo;
            have += gemm2_share(n, x, p, lo);
        }
        longest = have > longest ? have : longest;
    }
    return 8 * longest;
}

__host__ __device__ inline int gemm2_tiles(int m, int n) { return ((m + B2_TILE - 1) / B2_TILE) * ((n + B2_TILE - 1) / B2_TILE); }

__global__ __launch_bounds__(256, 1) void gemm_tn_split2_256_kernel(const Gemm2Launch lp)
{
    __shared__ __attribute__((aligned(16))) char lds_a[B2_STAGES * B2_STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char lds_b[B2_STAGES * B2_STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;

    const int t = gemm2_tile_of(lp, blockIdx.x);
    if (t < 0) return;  // the whole workgroup leaves
    int pi = 0, hi = lp.count;
    while (hi - pi > 1) {
        const int mid = (pi + hi) >> 1;
        if (lp.p[mid].tile_begin <= t)
            pi = mid;
        else
            hi = mid;
    }
    const Gemm2Problem &pr = lp.p[pi];
    const int tn = (pr.n + B2_TILE - 1) / B2_TILE;
    const int local = t - pr.tile_begin;
    const int m0 = (local / tn) * B2_TILE, n0 = (local % tn) * B2_TILE;

    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const size_t rba = (size_t)pr.dpa * 16, rbb = (size_t)pr.dpb * 16;
    const char *aa = static_cast<const char *>(pr.xa), *ab = aa + (size_t)pr.groups * rba;
    const char *ba = static_cast<const char *>(pr.xb), *bb = ba + (size_t)pr.groups * rbb;
    s3_pass_planes<S3_WAVE_FULL, true>(aa, bb, rba, rbb, pr.groups, m0, n0, lds_a, lds_b, acc);
    __syncthreads();
    s3_pass_planes<S3_WAVE_FULL, true>(ab, ba, rba, rbb, pr.groups, m0, n0, lds_a, lds_b, acc);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] *= 1.f / (float)(1 << S2_LOW_SHIFT);
    __syncthreads();
    s3_pass_planes<S3_WAVE_FULL, true>(aa, ba, rba, rbb, pr.groups, m0, n0, lds_a, lds_b, acc);

    const float sa = split2_scale(lp.amax_a[pr.amax_a]), sb = split2_scale(lp.amax_b[pr.amax_b]);
    const float inv = (1.f / sa) * (1.f / sb);  // exact: powers of two
    float *__restrict__ C = pr.c;
    const size_t ldc = (size_t)pr.ldc;
    // accumulator register r of lane (li, lh) in block (bi, bj): row 32 bi + 8 (r/4) + 4 lh + r%4, column 32 bj + li
#pragma unroll
    for (int bi = 0; bi < 4; ++bi)
#pragma unroll
        for (int bj = 0; bj < 4; ++bj) {
            const int n = n0 + wn + 32 * bj + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm + 32 * bi + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (m < pr.m && n < pr.n) C[(size_t)m * ldc + n] = inv * acc[bi][bj][r];
            }
        }
}

}  // namespace kfac
