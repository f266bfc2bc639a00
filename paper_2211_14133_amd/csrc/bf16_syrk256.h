// Curvature of bfloat16 activations on the bf16 MFMA with 256 x 256 tiles.
//
// The 128 x 128 kernel of tn_gemm.h is bound by what one CU can keep in flight:
// with bf16 MFMA a 32-token slab is consumed eight times faster than an fp32
// slab of the same bytes, and 160 KB of LDS cannot hold enough slabs to cover
// the memory latency.  Flops per byte double with the tile edge, so this kernel
// gives one workgroup (4 waves, one per SIMD) a 256 x 256 tile, each wave a
// 128 x 128 quarter as 4 x 4 MFMA 32x32x16 blocks (256 accumulator registers).
// Operands come from the packed layout of pack_bf16_kernel
// (P[token / 8][column][token % 8]); a slab of 32 tokens is 16 KB per operand and
// goes straight into a 4-stage LDS ring (128 KB) with global_load_lds_dwordx4.
//   iteration s:  M(s, 1st half) with R(s, 2nd half) and half of D(s+3) between its MFMAs,
//                 M(s, 2nd half) with R(s+1, 1st half) and the rest of D(s+3),  wait D(s+2)  barrier
// Lower-triangular tile set, mirrored stores (bitwise symmetric result), alpha /
// beta as in the engine.  One fp32 accumulation level: the tolerance of the bf16
// variant (2e-2 on the factor) does not need the chunked sum of the fp32 path.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tn_gemm.h"

namespace kfac {

constexpr int B2_TILE = 256;
constexpr int B2_STAGE_BYTES = BF_SLAB_GROUPS * B2_TILE * 16;  // 16 KB per operand per stage
constexpr int B2_STAGES = 4;

// Same descriptor table as the other curvature launches (SyrkProblem: x = packed
// copy, n = padded tokens, ldx = padded columns (a multiple of 256), tile_begin
// in 256-tiles).
struct Syrk256Launch {
    SyrkProblem p[SYRK_MAX_PROBLEMS];
    int count;
    float alpha, beta;
};

__host__ __device__ inline int b2_tiles(int d)
{
    const int nt = (d + B2_TILE - 1) / B2_TILE;
    return nt * (nt + 1) / 2;
}

// Which problem and which 256 x 256 tile of its lower tile set a workgroup owns.
struct B2Tile {
    int pi, m0, n0;
    bool diag;
};

__device__ inline B2Tile b2_locate(const Syrk256Launch &lp)
{
    const int t = tn_logical_tile(blockIdx.x, gridDim.x);
    int pi = 0, hi = lp.count;
    while (hi - pi > 1) {
        const int mid = (pi + hi) >> 1;
        if (lp.p[mid].tile_begin <= t)
            pi = mid;
        else
            hi = mid;
    }
    int ti, tj;
    tn_decode_lower(t - lp.p[pi].tile_begin, (lp.p[pi].d + B2_TILE - 1) / B2_TILE, ti, tj);
    B2Tile r;
    r.pi = pi;
    r.m0 = ti * B2_TILE;
    r.n0 = tj * B2_TILE;
    r.diag = (ti == tj);
    return r;
}

// Epilogue of a wave's 128 x 128 quarter: factor = beta * factor + alpha * acc on the lower tile set,
// mirrored into the upper one (bitwise symmetric result).
__device__ inline void b2_store(const floatx16 (&acc)[4][4], const SyrkProblem &pr, float alpha, float beta,
                                int m0, int n0, int wm, int wn, int li, int lh, bool diag)
{
    const int d = pr.d;
    // accumulator register r of lane (li, lh) in block (bi, bj): row 32 bi + 8 (r/4) + 4 lh + r%4, column 32 bj + li
    float *__restrict__ C = pr.factor;
    const size_t ldf = (size_t)pr.ldf;
    const bool vec_t = ((pr.ldf & 3) == 0) && ((reinterpret_cast<uintptr_t>(C) & 15) == 0);
#pragma unroll
    for (int bi = 0; bi < 4; ++bi)
#pragma unroll
        for (int bj = 0; bj < 4; ++bj) {
            const int n = n0 + wn + 32 * bj + li;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int mq = m0 + wm + 32 * bi + 8 * q + 4 * lh;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int m = mq + e;
                    v[e] = alpha * acc[bi][bj][4 * q + e];
                    if (m < d && n < d && (!diag || n <= m)) {
                        float *dst = C + (size_t)m * ldf + n;
                        if (beta != 0.f) v[e] += beta * (*dst);
                        *dst = v[e];
                    }
                }
                // mirror: four consecutive rows of C are four consecutive columns of the transposed tile
                if (n < d) {
                    if (!diag && mq + 3 < d && vec_t) {
                        *reinterpret_cast<float4 *>(C + (size_t)n * ldf + mq) = make_float4(v[0], v[1], v[2], v[3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int m = mq + e;
                            if (m < d && (!diag || n < m)) C[(size_t)n * ldf + m] = v[e];
                        }
                    }
                }
            }
        }
}

// The same epilogue with the reads batched: when the call accumulates, the old values of eight
// 32 x 32 blocks (128 registers: the operand registers of the K loop are free by now) are all requested
// before the first is used: two memory latencies per tile instead of one per element (the launches that
// accumulate over micro-batches are the common case here).  One instance per block, written out: as loops
// the sixteen blocks exceed what the compiler unrolls, and the accumulators would leave the registers.
struct B2Out {
    float *C;
    size_t ldf;
    int d, mw, nw;  // first row / column of the wave's quarter, plus the lane's share (4 lh, li)
    float alpha, beta;
    bool diag, vec_t;
};

template <int BI, int BJ>
__device__ __forceinline__ void b2_load_block(float (&old)[16], const B2Out &o)
{
    const int n = o.nw + 32 * BJ, mb = o.mw + 32 * BI;
    const bool accumulate = o.beta != 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = mb + 8 * (r >> 2) + (r & 3);
        old[r] = 0.f;
        if (accumulate && m < o.d && n < o.d && (!o.diag || n <= m)) old[r] = o.C[(size_t)m * o.ldf + n];
    }
}

template <int BI, int BJ>
__device__ __forceinline__ void b2_store_block(const floatx16 &acc, const float (&old)[16], const B2Out &o)
{
    const int d = o.d;
    const int n = o.nw + 32 * BJ, mb = o.mw + 32 * BI;
    float *__restrict__ C = o.C;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int mq = mb + 8 * q;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int m = mq + e;
            v[e] = o.alpha * acc[4 * q + e] + o.beta * old[4 * q + e];
            if (m < d && n < d && (!o.diag || n <= m)) C[(size_t)m * o.ldf + n] = v[e];
        }
        // mirror: four consecutive rows of C are four consecutive columns of the transposed tile
        if (n < d) {
            if (!o.diag && mq + 3 < d && o.vec_t) {
                *reinterpret_cast<float4 *>(C + (size_t)n * o.ldf + mq) = make_float4(v[0], v[1], v[2], v[3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int m = mq + e;
                    if (m < d && (!o.diag || n < m)) C[(size_t)n * o.ldf + m] = v[e];
                }
            }
        }
    }
}

template <int B0>
__device__ __forceinline__ void b2_store_half(const floatx16 (&acc)[4][4], const B2Out &o)
{
    float old[8][16];
#define B2_LOAD2(k, bi)                                \
    b2_load_block<bi, 0>(old[4 * (k) + 0], o);         \
    b2_load_block<bi, 1>(old[4 * (k) + 1], o);         \
    b2_load_block<bi, 2>(old[4 * (k) + 2], o);         \
    b2_load_block<bi, 3>(old[4 * (k) + 3], o)
#define B2_STORE2(k, bi)                                           \
    b2_store_block<bi, 0>(acc[bi][0], old[4 * (k) + 0], o);        \
    b2_store_block<bi, 1>(acc[bi][1], old[4 * (k) + 1], o);        \
    b2_store_block<bi, 2>(acc[bi][2], old[4 * (k) + 2], o);        \
    b2_store_block<bi, 3>(acc[bi][3], old[4 * (k) + 3], o)
    B2_LOAD2(0, B0);
    B2_LOAD2(1, B0 + 1);
    B2_STORE2(0, B0);
    B2_STORE2(1, B0 + 1);
#undef B2_LOAD2
#undef B2_STORE2
}

__device__ __forceinline__ void b2_store_batched(const floatx16 (&acc)[4][4], const SyrkProblem &pr, float alpha, float beta,
                                         int m0, int n0, int wm, int wn, int li, int lh, bool diag)
{
    B2Out o;
    o.C = pr.factor;
    o.ldf = (size_t)pr.ldf;
    o.d = pr.d;
    o.mw = m0 + wm + 4 * lh;
    o.nw = n0 + wn + li;
    o.alpha = alpha;
    o.beta = beta;
    o.diag = diag;
    o.vec_t = ((pr.ldf & 3) == 0) && ((reinterpret_cast<uintptr_t>(pr.factor) & 15) == 0);
    b2_store_half<0>(acc, o);
    b2_store_half<2>(acc, o);
}

__global__ __launch_bounds__(256, 1) void curvature_syrk_bf16_256_kernel(const Syrk256Launch lp)
{
    __shared__ __attribute__((aligned(16))) char lds_a[B2_STAGES * B2_STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char lds_b[B2_STAGES * B2_STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;

    const B2Tile bt = b2_locate(lp);
    const SyrkProblem &pr = lp.p[bt.pi];
    const int m0 = bt.m0, n0 = bt.n0;
    const size_t row_bytes = (size_t)pr.ldx * 16;  // one k-group of all columns
    const int groups = pr.n / BF_KG;
    const int niter = groups / BF_SLAB_GROUPS;
    const char *xp = static_cast<const char *>(pr.x);
    // per-lane byte offsets inside a k-group row (32 bits: padded columns * 16 < 2^32 is checked on the host)
    const unsigned va = (unsigned)(((size_t)m0 + lane) * 16);
    const unsigned vb = (unsigned)(((size_t)n0 + lane) * 16);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const unsigned la0 = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(const __attribute__((address_space(3))) char *)lds_a) + wave_s * (B2_TILE * 16);
    const unsigned lb0 = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(const __attribute__((address_space(3))) char *)lds_b) + wave_s * (B2_TILE * 16);

    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 fa[2][4], fb[2][4];  // [k step parity][block]
    int gd = 0;                // first k-group of the next slab to request
    const char *sbase = xp;    // k-group row this wave requests (wave-uniform: scalar registers)

    // Wave w fetches k-group gd + w: the 256 columns of each operand in four 64-column pieces
    // (piece q of A is load 2q, of B load 2q+1).  The address is a scalar base plus a loop-invariant
    // per-lane offset, so that the loop has no vector arithmetic: with an MFMA that occupies the
    // matrix core for only 32 cycles, every other vector instruction costs MFMA issue slots.
#define B2_DBASE()                                                                         \
    do {                                                                                   \
        sbase = xp + (size_t)min(gd + wave_s, groups - 1) * row_bytes;                     \
        gd += BF_SLAB_GROUPS;                                                              \
    } while (0)
#define B2_D1(st, w)                                                                                           \
    do {                                                                                                       \
        if (((w) & 1) == 0)                                                                                    \
            tn_dma16_s(reinterpret_cast<const float *>(sbase + ((w) >> 1) * 1024), va,                         \
                       la0 + (st) * B2_STAGE_BYTES + ((w) >> 1) * 1024);                                       \
        else                                                                                                   \
            tn_dma16_s(reinterpret_cast<const float *>(sbase + ((w) >> 1) * 1024), vb,                         \
                       lb0 + (st) * B2_STAGE_BYTES + ((w) >> 1) * 1024);                                       \
    } while (0)
    // k step t of a slab uses k-groups 2t and 2t+1 (one per half wave); block b of the wave tile is
    // columns 32b .. 32b+31, so a ds_read_b128 touches 32 consecutive 16-byte units (no conflicts)
#define B2_RA(st, t, set)                                                                                     \
    do {                                                                                                      \
        const int u_ = (st) * B2_STAGE_BYTES + ((2 * (t) + lh) * B2_TILE + li) * 16;                          \
        _Pragma("unroll") for (int b = 0; b < 4; ++b)                                                         \
            fa[set][b] = *reinterpret_cast<const uint4 *>(lds_a + u_ + (wm + 32 * b) * 16);                   \
    } while (0)
#define B2_RB(st, t, set)                                                                                     \
    do {                                                                                                      \
        const int u_ = (st) * B2_STAGE_BYTES + ((2 * (t) + lh) * B2_TILE + li) * 16;                          \
        _Pragma("unroll") for (int b = 0; b < 4; ++b)                                                         \
            fb[set][b] = *reinterpret_cast<const uint4 *>(lds_b + u_ + (wn + 32 * b) * 16);                   \
    } while (0)
#define B2_MG(set, bi)                                                                                        \
    do {                                                                                                      \
        _Pragma("unroll") for (int bj = 0; bj < 4; ++bj)                                                      \
            acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                            \
                __builtin_bit_cast(bf16x8, fa[set][bi]), __builtin_bit_cast(bf16x8, fb[set][bj]),             \
                acc[bi][bj], 0, 0, 0);                                                                        \
    } while (0)
#define B2_PIN() __builtin_amdgcn_sched_barrier(0)
    // One slab.  The order is pinned: reads and loads sit in small pieces between groups of four MFMAs,
    // each operand read a whole batch of 16 MFMAs ahead of its use.
#define B2_ITER(st0, st1, st3)                                                             \
    do {                                                                                   \
        B2_DBASE();                                                                        \
        B2_PIN();                                                                          \
        B2_MG(0, 0);                                                                       \
        B2_PIN();                                                                          \
        B2_RA(st0, 1, 1);                                                                  \
        B2_D1(st3, 0);                                                                     \
        B2_PIN();                                                                          \
        B2_MG(0, 1);                                                                       \
        B2_PIN();                                                                          \
        B2_RB(st0, 1, 1);                                                                  \
        B2_D1(st3, 1);                                                                     \
        B2_PIN();                                                                          \
        B2_MG(0, 2);                                                                       \
        B2_PIN();                                                                          \
        B2_D1(st3, 2);                                                                     \
        B2_PIN();                                                                          \
        B2_MG(0, 3);                                                                       \
        B2_PIN();                                                                          \
        B2_D1(st3, 3);                                                                     \
        B2_PIN();                                                                          \
        B2_MG(1, 0);                                                                       \
        B2_PIN();                                                                          \
        B2_RA(st1, 0, 0);                                                                  \
        B2_D1(st3, 4);                                                                     \
        B2_PIN();                                                                          \
        B2_MG(1, 1);                                                                       \
        B2_PIN();                                                                          \
        B2_RB(st1, 0, 0);                                                                  \
        B2_D1(st3, 5);                                                                     \
        B2_PIN();                                                                          \
        B2_MG(1, 2);                                                                       \
        B2_PIN();                                                                          \
        B2_D1(st3, 6);                                                                     \
        B2_D1(st3, 7);                                                                     \
        B2_PIN();                                                                          \
        B2_MG(1, 3);                                                                       \
        B2_PIN();                                                                          \
        __builtin_amdgcn_s_waitcnt(0x0F78); /* vmcnt(8): all but the newest slab landed */ \
        __syncthreads();                                                                   \
        B2_PIN();                                                                          \
    } while (0)

#pragma unroll
    for (int q = 0; q < 3; ++q) {
        B2_DBASE();
#pragma unroll
        for (int w = 0; w < 8; ++w) B2_D1(q, w);
    }
    __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt(8): slabs 0 and 1 have landed
    __syncthreads();
    B2_RA(0, 0, 0);
    B2_RB(0, 0, 0);
    int s = 0;
    for (; s + 4 <= niter; s += 4) {
        B2_ITER(0, 1, 3);
        B2_ITER(1, 2, 0);
        B2_ITER(2, 3, 1);
        B2_ITER(3, 0, 2);
    }
    const int rest = niter - s;  // s is a multiple of four: the stages continue at 0
    if (rest > 0) B2_ITER(0, 1, 3);
    if (rest > 1) B2_ITER(1, 2, 0);
    if (rest > 2) B2_ITER(2, 3, 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing may still be writing LDS
#undef B2_DBASE
#undef B2_D1
#undef B2_RA
#undef B2_RB
#undef B2_MG
#undef B2_PIN
#undef B2_ITER

    if (lp.beta == 0.f)
        b2_store(acc, pr, lp.alpha, 0.f, m0, n0, wm, wn, li, lh, bt.diag);
    else
        b2_store_batched(acc, pr, lp.alpha, lp.beta, m0, n0, wm, wn, li, lh, bt.diag);
}

// ---------------------------------------------------------------------------
// The same tile without the repacking pre-pass, for inputs that need no padding
// (d a multiple of 256, tokens a multiple of 32, rows 16-byte aligned).
//
// Slabs of the row-major input go straight into LDS as they are: one
// global_load_lds_dwordx4 per token row, lanes 0..31 fetching the 256 columns of
// the A panel and lanes 32..63 those of the B panel (the per-lane global address is
// free, the LDS destination is base + 16 * lane), so an LDS row is
// [A: 256 columns | B: 256 columns] of one token.  The k-contiguous operand
// layout of the MFMA is produced on the way out of LDS by ds_read_b64_tr_b16
// (gfx950): in each group of 16 lanes, lane 4s+q supplies the address of 4
// consecutive columns of token row kb+s, and lane i receives tokens kb .. kb+3 of
// column c0 + i (lane layout probed on the hardware).  Two such reads give a lane
// the 8 consecutive tokens of its column that MFMA 32x32x16 wants.  LDS rows are
// padded by 64 bytes: the 4 rows that half a wave reads (64 bytes of each) then fall
// into different banks.
constexpr int B2R_ROW_BYTES = 2 * B2_TILE * 2 + 64;            // 1088
constexpr int B2R_SLAB_ROWS = 32;                             // tokens per slab = two k steps of 16
constexpr int B2R_STAGE_BYTES = B2R_SLAB_ROWS * B2R_ROW_BYTES;  // 34816

typedef short b2_short4 __attribute__((ext_vector_type(4)));
typedef short b2_short8 __attribute__((ext_vector_type(8)));

__device__ inline b2_short4 b2_read_tr(const char *lds_ptr)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) b2_short4 *)lds_ptr);
}

// What a wave computes of its 128 x 128 quarter.  On a diagonal tile the upper right quarter is only stored as
// the mirror of the lower left one: its wave takes part in the loads and barriers and computes nothing; the two
// quarters on the diagonal leave out their six 32 x 32 blocks above the diagonal.  The tile takes as long as
// its full quarter, but the chip is power-limited under the bf16 MFMA kernels: MFMAs that are not issued let
// the others run at a higher clock.
enum B2WaveMode : int { B2_WAVE_FULL = 0, B2_WAVE_IDLE = 1, B2_WAVE_LOWER = 2 };

template <int MODE>
__device__ __forceinline__ void b2r_mainloop(const SyrkProblem &pr, int m0, int n0, const char *lds, floatx16 (&acc)[4][4])
{
    constexpr bool IDLE = MODE == B2_WAVE_IDLE, LOWER = MODE == B2_WAVE_LOWER;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
    const int K = pr.n;
    const int niter = K / B2R_SLAB_ROWS;
    const size_t row_pitch = (size_t)pr.ldx * 2;  // bytes per token row of x
    const char *xp = static_cast<const char *>(pr.x);
    // this lane's 8 columns of a token row: A panel in the lower half of the wave, B panel in the upper
    const unsigned vcol = (unsigned)(((lane < 32) ? (m0 + 8 * lane) : (n0 + 8 * (lane - 32))) * 2);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const unsigned l0 = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(const __attribute__((address_space(3))) char *)lds) +
                        wave_s * (8 * B2R_ROW_BYTES);  // wave w fetches rows 8w .. 8w+7 of a slab

    // transposing reads: group g = lane / 16 covers k half g / 2 and column half g % 2 of a 32-column block
    const int g = lane >> 4, s4 = (lane >> 2) & 3, q4 = lane & 3;
    const int rd = (8 * (g >> 1) + s4) * B2R_ROW_BYTES + (16 * (g & 1) + 4 * q4) * 2;
    // one address register per stage and operand: what is added per read (k step, block, upper four
    // rows) then fits the 16-bit offset field of the LDS instruction, and the loop has no address arithmetic
    const char *ra[B2_STAGES], *rb[B2_STAGES];
#pragma unroll
    for (int st = 0; st < B2_STAGES; ++st) {
        ra[st] = lds + st * B2R_STAGE_BYTES + rd + wm * 2;
        rb[st] = lds + st * B2R_STAGE_BYTES + rd + B2_TILE * 2 + wn * 2;
    }

    b2_short8 fa[2][4], fb[2][4];  // [k step parity][block]
    int kd = 0;                    // first token of the next slab to request
    const char *sbase = xp;

#define R2_DBASE()                                                                         \
    do {                                                                                   \
        sbase = xp + (size_t)(min(kd, K - B2R_SLAB_ROWS) + 8 * wave_s) * row_pitch;        \
        kd += B2R_SLAB_ROWS;                                                               \
    } while (0)
    // row w of this wave's eight rows of the slab
#define R2_D1(st, w)                                                                       \
    tn_dma16_s(reinterpret_cast<const float *>(sbase + (size_t)(w) * row_pitch), vcol,     \
               l0 + (st) * B2R_STAGE_BYTES + (w) * B2R_ROW_BYTES)
#define R2_R(dst, base, st, t, b)                                                                       \
    do {                                                                                                \
        const char *p_ = (base)[st] + (t) * 16 * B2R_ROW_BYTES + (b) * 64;                              \
        const b2_short4 lo_ = b2_read_tr(p_), hi_ = b2_read_tr(p_ + 4 * B2R_ROW_BYTES);                 \
        dst = __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7);                                \
    } while (0)
#define R2_RA(st, t, set)                                                                  \
    do {                                                                                   \
        if (!IDLE) _Pragma("unroll") for (int b = 0; b < 4; ++b) R2_R(fa[set][b], ra, st, t, b); \
    } while (0)
#define R2_RB(st, t, set)                                                                  \
    do {                                                                                   \
        if (!IDLE) _Pragma("unroll") for (int b = 0; b < 4; ++b) R2_R(fb[set][b], rb, st, t, b); \
    } while (0)
#define R2_MG(set, bi)                                                                                        \
    do {                                                                                                      \
        if (!IDLE) _Pragma("unroll") for (int bj = 0; bj < (LOWER ? (bi) + 1 : 4); ++bj)                      \
            acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                            \
                __builtin_bit_cast(bf16x8, fa[set][bi]), __builtin_bit_cast(bf16x8, fb[set][bj]),             \
                acc[bi][bj], 0, 0, 0);                                                                        \
    } while (0)
#define R2_PIN() __builtin_amdgcn_sched_barrier(0)
    // One slab; same order as the packed kernel: reads and loads in pieces between groups of four MFMAs.
#define R2_ITER(st0, st1, st3)                                                             \
    do {                                                                                   \
        R2_DBASE();                                                                        \
        R2_PIN();                                                                          \
        R2_MG(0, 0);                                                                       \
        R2_PIN();                                                                          \
        R2_RA(st0, 1, 1);                                                                  \
        R2_D1(st3, 0);                                                                     \
        R2_PIN();                                                                          \
        R2_MG(0, 1);                                                                       \
        R2_PIN();                                                                          \
        R2_RB(st0, 1, 1);                                                                  \
        R2_D1(st3, 1);                                                                     \
        R2_PIN();                                                                          \
        R2_MG(0, 2);                                                                       \
        R2_PIN();                                                                          \
        R2_D1(st3, 2);                                                                     \
        R2_PIN();                                                                          \
        R2_MG(0, 3);                                                                       \
        R2_PIN();                                                                          \
        R2_D1(st3, 3);                                                                     \
        R2_PIN();                                                                          \
        R2_MG(1, 0);                                                                       \
        R2_PIN();                                                                          \
        R2_RA(st1, 0, 0);                                                                  \
        R2_D1(st3, 4);                                                                     \
        R2_PIN();                                                                          \
        R2_MG(1, 1);                                                                       \
        R2_PIN();                                                                          \
        R2_RB(st1, 0, 0);                                                                  \
        R2_D1(st3, 5);                                                                     \
        R2_PIN();                                                                          \
        R2_MG(1, 2);                                                                       \
        R2_PIN();                                                                          \
        R2_D1(st3, 6);                                                                     \
        R2_D1(st3, 7);                                                                     \
        R2_PIN();                                                                          \
        R2_MG(1, 3);                                                                       \
        R2_PIN();                                                                          \
        __builtin_amdgcn_s_waitcnt(0x0F78); /* vmcnt(8): all but the newest slab landed */ \
        __syncthreads();                                                                   \
        R2_PIN();                                                                          \
    } while (0)

#pragma unroll
    for (int q = 0; q < 3; ++q) {
        R2_DBASE();
#pragma unroll
        for (int w = 0; w < 8; ++w) R2_D1(q, w);
    }
    __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt(8): slabs 0 and 1 have landed
    __syncthreads();
    R2_RA(0, 0, 0);
    R2_RB(0, 0, 0);
    int s = 0;
    for (; s + 4 <= niter; s += 4) {
        R2_ITER(0, 1, 3);
        R2_ITER(1, 2, 0);
        R2_ITER(2, 3, 1);
        R2_ITER(3, 0, 2);
    }
    const int rest = niter - s;  // s is a multiple of four: the stages continue at 0
    if (rest > 0) R2_ITER(0, 1, 3);
    if (rest > 1) R2_ITER(1, 2, 0);
    if (rest > 2) R2_ITER(2, 3, 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing may still be writing LDS
#undef R2_DBASE
#undef R2_D1
#undef R2_R
#undef R2_RA
#undef R2_RB
#undef R2_MG
#undef R2_PIN
#undef R2_ITER

}

__global__ __launch_bounds__(256, 1) void curvature_syrk_bf16_256_rowmajor_kernel(const Syrk256Launch lp)
{
    __shared__ __attribute__((aligned(16))) char lds[B2_STAGES * B2R_STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;

    const B2Tile bt = b2_locate(lp);
    const SyrkProblem &pr = lp.p[bt.pi];
    const int m0 = bt.m0, n0 = bt.n0;
    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int mode_wave = __builtin_amdgcn_readfirstlane(wave);
    if (bt.diag && mode_wave == 1) {
        b2r_mainloop<B2_WAVE_IDLE>(pr, m0, n0, lds, acc);
        return;
    }
    if (bt.diag && mode_wave != 2)
        b2r_mainloop<B2_WAVE_LOWER>(pr, m0, n0, lds, acc);
    else
        b2r_mainloop<B2_WAVE_FULL>(pr, m0, n0, lds, acc);
    if (lp.beta == 0.f)
        b2_store(acc, pr, lp.alpha, 0.f, m0, n0, wm, wn, li, lh, bt.diag);
    else
        b2_store_batched(acc, pr, lp.alpha, lp.beta, m0, n0, wm, wn, li, lh, bt.diag);
}

}  // namespace kfac
