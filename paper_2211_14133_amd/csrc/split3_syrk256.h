// Curvature of float32 activations on the bf16 MFMA: every float32 value is written as the sum of three
// bfloat16 terms, x = h + m + l (h = bf16(x), m = bf16(x - h), l = bf16(x - h - m): 3 x 8 significand bits,
// the 24 bits of a float32), and a product of two values as the six bf16 products that reach 2^-16 of it,
//     x y  ~=  h h' + (h m' + m h') + (m m' + h l' + l h'),
// what is left out (m l', l m', l l') being below 2^-24 |x y|, the rounding of one float32 operation.  All six
// accumulate in float32 in the MFMA accumulators (the five small ones first, see the kernel).  The bf16 MFMA
// has 16 times the rate of the fp32 one, so six of its products cost 3/8 of one fp32 product.
//
// A pre-pass (split3_pack_kernel) writes the three terms as three planes in the k-interleaved layout of the
// bf16 kernels (P[token / 8][column][token % 8], zero-padded to 32 tokens and 256 columns); the MFMA kernel
// is the 256 x 256 tile of bf16_syrk256.h with a stage of 16 tokens x 3 planes (24 KB per operand) in a
// 3-stage LDS ring (144 KB).  A fragment read from LDS serves two or three products, so LDS reads per MFMA
// are a third of the plain bf16 kernel's and the loop is bound by the matrix core.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bf16_syrk256.h"

namespace kfac {

constexpr int S3_PLANES = 3;
constexpr int S3_GROUP_BYTES = B2_TILE * 16;                    // one k-group of one plane of one operand: 4 KB
constexpr int S3_STAGE_BYTES = S3_PLANES * 2 * S3_GROUP_BYTES;  // 16 tokens: 24 KB per operand
constexpr int S3_STAGES = 3;
constexpr int S3_CHUNK_GROUPS = 1024;  // tokens / 8 that one launch of the MFMA kernel accumulates (a multiple of 4)

// ---------------------------------------------------------------------------
// Pre-pass: float32 [n, d] -> three packed bfloat16 planes, dst + plane * gp * dp * 8 elements.
struct Split3Item {
    const float *x;       // [n, d] float32, ldx
    unsigned short *dst;  // [3][gp][dp][8]
    int n, d, ldx, dp, gp, pad_;
};
struct Split3Launch {
    Split3Item it[PACK_MAX_ITEMS];
    int first_wg[PACK_MAX_ITEMS + 1];  // workgroups of item i: first_wg[i] .. first_wg[i+1]-1 (column blocks of 256 x k-groups)
    int count;
};

// One thread takes one column of a k-group (8 tokens): eight 4-byte reads (a wave reads 256-byte runs of a
// token row), the split in registers, and per plane the eight tokens as one 16-byte packed write (a wave
// writes 1 KB runs): no LDS, every request of a thread in flight at once.
constexpr int S3P_COLS = 256;  // columns per workgroup: one per thread
constexpr int S3P_GROUPS = 1;  // k-groups per workgroup (whole launch of the BERT-Large stage with 1 / 2 / 4: 6.45 / 6.62 / 6.71 ms)

__device__ inline unsigned s3_bf16_bits(float v)
{
    return (unsigned)__builtin_bit_cast(unsigned short, static_cast<__bf16>(v));
}
__device__ inline float s3_bf16_value(unsigned b)
{
    return __builtin_bit_cast(float, b << 16);
}

__global__ __launch_bounds__(256) void split3_pack_kernel(const Split3Launch pl)
{
    int i = 0, hi = pl.count;
    while (hi - i > 1) {
        const int mid = (i + hi) >> 1;
        if (pl.first_wg[mid] <= (int)blockIdx.x)
            i = mid;
        else
            hi = mid;
    }
    const Split3Item &it = pl.it[i];
    const int w = blockIdx.x - pl.first_wg[i], cb = it.dp / S3P_COLS;  // column blocks vary fastest
    const int col = (w % cb) * S3P_COLS + threadIdx.x, g0 = (w / cb) * S3P_GROUPS;
    constexpr int ROWS = S3P_GROUPS * BF_KG;
    float v[ROWS];
    const float *src = it.x + (size_t)g0 * BF_KG * it.ldx + col;
    if (col < it.d && (g0 + S3P_GROUPS) * BF_KG <= it.n) {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) v[r] = src[(size_t)r * it.ldx];
    } else {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) v[r] = (col < it.d && g0 * BF_KG + r < it.n) ? src[(size_t)r * it.ldx] : 0.f;
    }
    unsigned h[ROWS], m[ROWS], l[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        h[r] = s3_bf16_bits(v[r]);
        const float r1 = v[r] - s3_bf16_value(h[r]);  // exact
        m[r] = s3_bf16_bits(r1);
        const float r2 = r1 - s3_bf16_value(m[r]);    // exact
        l[r] = s3_bf16_bits(r2);
    }
    const size_t plane = (size_t)it.gp * it.dp * 8;  // elements
#pragma unroll
    for (int gi = 0; gi < S3P_GROUPS; ++gi) {
        unsigned short *dst = it.dst + ((size_t)(g0 + gi) * it.dp + col) * 8;
        const unsigned *hh = h + 8 * gi, *mm = m + 8 * gi, *ll = l + 8 * gi;
        *reinterpret_cast<uint4 *>(dst) =
            make_uint4(hh[0] | (hh[1] << 16), hh[2] | (hh[3] << 16), hh[4] | (hh[5] << 16), hh[6] | (hh[7] << 16));
        *reinterpret_cast<uint4 *>(dst + plane) =
            make_uint4(mm[0] | (mm[1] << 16), mm[2] | (mm[3] << 16), mm[4] | (mm[5] << 16), mm[6] | (mm[7] << 16));
        *reinterpret_cast<uint4 *>(dst + 2 * plane) =
            make_uint4(ll[0] | (ll[1] << 16), ll[2] | (ll[3] << 16), ll[4] | (ll[5] << 16), ll[6] | (ll[7] << 16));
    }
}

// ---------------------------------------------------------------------------
// The MFMA kernel.  Descriptor as for the bf16 kernels: x = the first of the three planes (at the first k-group
// of this launch's share of the tokens), n = padded tokens of the share, ldx = padded columns, pad_ = k-groups
// of a whole plane.
//
// Two passes over K into the same accumulators.  The matrix core behaves as if it added the sixteen products of
// an instruction to the accumulator with the bits below the accumulator's last place cut off rather than rounded; for
// products of the size of the accumulated sum that is harmless, but products 2^-8 and 2^-16 of it, added to
// an accumulator that already holds the large sum, lose a little at every instruction, always downwards
// (measured: a relative bias of -2e-6 on the diagonal after 4096 tokens).  So the small products go first,
// into accumulators that hold nothing else (pass 1: five of the six products, all three planes), and the
// large one, h h', is added on top in a second sweep over the h plane alone (pass 2).  The result then has the
// error of a plain bf16-MFMA sum (3e-7 after 4096 tokens, no bias) at the price of fetching the h plane twice.
//
// Pass 1, per stage (16 tokens) and wave: 16 blocks x 5 products = 80 MFMAs, in five groups of 16,
//     G1 = Ah Bm   G2 = Am Bm   G3 = Am Bh   G4 = Al Bh   G5 = Ah Bl
// (A = row panel, B = column panel; h, m, l = the planes), so that a fragment set is dead as early as
// possible.  The loop body runs between two barriers and is skewed by one group: G5 of stage s, then G1..G4
// of stage s+1, and every fragment set of stage s+1 is read from LDS inside the body, at least one group
// before its first use, into the registers its predecessor has just left (Ah has two sets, alternating).  So
// a body reads only the slot of stage s+1; of the other two slots one receives stage s+2 (requested one body
// earlier) and one, free since the barrier, stage s+3: two bodies of memory latency are covered.
//
// What a wave computes of its 128 x 128 quarter.  On a diagonal tile the upper right quarter is only stored as
// the mirror of the lower left one: its wave takes part in the loads and barriers and computes nothing; the two
// quarters on the diagonal leave out their six 32 x 32 blocks above the diagonal (the chip is power-limited
// under this kernel: MFMAs that are not issued let the others run at a higher clock).
enum S3WaveMode : int { S3_WAVE_FULL = 0, S3_WAVE_IDLE = 1, S3_WAVE_LOWER = 2 };

template <int MODE>
__device__ __forceinline__ void s3_pass_small(const SyrkProblem &pr, int m0, int n0, const char *lds_a, const char *lds_b,
                                              floatx16 (&acc)[4][4])
{
    constexpr bool IDLE = MODE == S3_WAVE_IDLE, LOWER = MODE == S3_WAVE_LOWER;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
    const size_t row_bytes = (size_t)pr.ldx * 16;  // one k-group of all columns of one plane
    const int groups = pr.n / BF_KG;
    const size_t plane_bytes = (size_t)pr.pad_ * row_bytes;  // pad_: k-groups of a whole plane (groups: of this launch's share)
    const int niter = groups / 2;
    const char *xp = static_cast<const char *>(pr.x);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    // wave w requests columns 64 w .. 64 w + 63 of every (plane, k-group) row of both panels
    const unsigned va = (unsigned)(((size_t)m0 + 64 * wave + lane) * 16);
    const unsigned vb = (unsigned)(((size_t)n0 + 64 * wave + lane) * 16);
    const unsigned la0 = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(const __attribute__((address_space(3))) char *)lds_a) + wave_s * 1024;
    const unsigned lb0 = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(const __attribute__((address_space(3))) char *)lds_b) + wave_s * 1024;

    // one address register per stage and operand; plane and block then fit the offset field of the read
    typedef const __attribute__((address_space(3))) char *lds_ptr;
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(3))) u32x4 *lds_ptr16;
    lds_ptr ra[S3_STAGES], rb[S3_STAGES];
#pragma unroll
    for (int st = 0; st < S3_STAGES; ++st) {
        ra[st] = (lds_ptr)lds_a + st * S3_STAGE_BYTES + lh * S3_GROUP_BYTES + (wm + li) * 16;
        rb[st] = (lds_ptr)lds_b + st * S3_STAGE_BYTES + lh * S3_GROUP_BYTES + (wn + li) * 16;
    }

    u32x4 ah[2][4], am[4], al[4], bh[4], bm[4], bl[4];
    int gd = 0;  // first k-group of the next stage to request
    const char *sb0 = xp, *sb1 = xp;

#define S3_DBASE()                                                                         \
    do {                                                                                   \
        sb0 = xp + (size_t)min(gd, groups - 1) * row_bytes;                                \
        sb1 = xp + (size_t)min(gd + 1, groups - 1) * row_bytes;                            \
        gd += 2;                                                                           \
    } while (0)
    // load w of the twelve of a stage: operand w % 2, plane (w / 2) / 2, k-group (w / 2) % 2
#define S3_D1(st, w)                                                                                           \
    do {                                                                                                       \
        const char *b_ = ((((w) >> 1) & 1) ? sb1 : sb0) + (size_t)((w) >> 2) * plane_bytes;                    \
        if (((w) & 1) == 0)                                                                                    \
            tn_dma16_s(reinterpret_cast<const float *>(b_), va, la0 + (st) * S3_STAGE_BYTES + ((w) >> 1) * S3_GROUP_BYTES); \
        else                                                                                                   \
            tn_dma16_s(reinterpret_cast<const float *>(b_), vb, lb0 + (st) * S3_STAGE_BYTES + ((w) >> 1) * S3_GROUP_BYTES); \
    } while (0)
    // plane p of stage slot st: lane (li, lh) takes k-group lh; block b = columns 32 b .. 32 b + 31
#define S3_R(set, base, st, p)                                                                                 \
    do {                                                                                                       \
        if (!IDLE) _Pragma("unroll") for (int b = 0; b < 4; ++b)                                               \
            set[b] = *(lds_ptr16)((base)[st] + (p) * 2 * S3_GROUP_BYTES + b * 512);                            \
    } while (0)
#define S3_M4(fa, fb, bi)                                                                                      \
    do {                                                                                                       \
        if (!IDLE) _Pragma("unroll") for (int bj = 0; bj < (LOWER ? (bi) + 1 : 4); ++bj)                       \
            acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                             \
                __builtin_bit_cast(bf16x8, fa[bi]), __builtin_bit_cast(bf16x8, fb[bj]), acc[bi][bj], 0, 0, 0); \
    } while (0)
#define S3_PIN() __builtin_amdgcn_sched_barrier(0)
    // G1..G4 of the stage whose fragments are (or are being) read, with the loads w0 .. w0+7 in between
#define S3_FIRST_GROUPS(AH, sl, w0, SN, READ_BL)                                           \
    do {                                                                                   \
        S3_M4(AH, bm, 0);                                                                  \
        S3_PIN();                                                                          \
        S3_D1(sl, (w0) + 0);                                                               \
        S3_D1(sl, (w0) + 1);                                                               \
        S3_PIN();                                                                          \
        S3_M4(AH, bm, 1);                                                                  \
        S3_PIN();                                                                          \
        if (READ_BL) S3_R(bl, rb, SN, 2);                                                  \
        S3_PIN();                                                                          \
        S3_M4(AH, bm, 2);                                                                  \
        S3_PIN();                                                                          \
        S3_D1(sl, (w0) + 2);                                                               \
        S3_D1(sl, (w0) + 3);                                                               \
        S3_PIN();                                                                          \
        S3_M4(AH, bm, 3);                                                                  \
        S3_PIN();                                                                          \
        S3_M4(am, bm, 0);                                                                  \
        S3_PIN();                                                                          \
        S3_D1(sl, (w0) + 4);                                                               \
        S3_D1(sl, (w0) + 5);                                                               \
        S3_PIN();                                                                          \
        S3_M4(am, bm, 1);                                                                  \
        S3_PIN();                                                                          \
        S3_D1(sl, (w0) + 6);                                                               \
        S3_D1(sl, (w0) + 7);                                                               \
        S3_PIN();                                                                          \
        S3_M4(am, bm, 2);                                                                  \
        S3_M4(am, bm, 3);                                                                  \
        S3_PIN();                                                                          \
        S3_M4(am, bh, 0);                                                                  \
        S3_M4(am, bh, 1);                                                                  \
        S3_M4(am, bh, 2);                                                                  \
        S3_M4(am, bh, 3);                                                                  \
        S3_PIN();                                                                          \
        S3_M4(al, bh, 0);                                                                  \
        S3_M4(al, bh, 1);                                                                  \
        S3_M4(al, bh, 2);                                                                  \
        S3_M4(al, bh, 3);                                                                  \
        S3_PIN();                                                                          \
        __builtin_amdgcn_s_waitcnt(0x0F7C); /* vmcnt(12): all but the newest stage landed */ \
        __syncthreads();                                                                   \
        S3_PIN();                                                                          \
    } while (0)
    // G5 of the stage in registers (Ah set P), while the sets of the next stage (slot SN) are read
#define S3_LAST_GROUP(P, Q, SN, sl)                                                        \
    do {                                                                                   \
        S3_R(ah[Q], ra, SN, 0);                                                            \
        S3_R(bm, rb, SN, 1);                                                               \
        S3_PIN();                                                                          \
        S3_M4(ah[P], bl, 0);                                                               \
        S3_PIN();                                                                          \
        S3_D1(sl, 0);                                                                      \
        S3_D1(sl, 1);                                                                      \
        S3_R(am, ra, SN, 1);                                                               \
        S3_PIN();                                                                          \
        S3_M4(ah[P], bl, 1);                                                               \
        S3_PIN();                                                                          \
        S3_R(bh, rb, SN, 0);                                                               \
        S3_PIN();                                                                          \
        S3_M4(ah[P], bl, 2);                                                               \
        S3_PIN();                                                                          \
        S3_D1(sl, 2);                                                                      \
        S3_D1(sl, 3);                                                                      \
        S3_R(al, ra, SN, 2);                                                               \
        S3_PIN();                                                                          \
        S3_M4(ah[P], bl, 3);                                                               \
        S3_PIN();                                                                          \
    } while (0)
#define S3_BODY(SN, sl, P, Q)                                                              \
    do {                                                                                   \
        S3_DBASE();                                                                        \
        S3_PIN();                                                                          \
        S3_LAST_GROUP(P, Q, SN, sl);                                                       \
        S3_FIRST_GROUPS(ah[Q], sl, 4, SN, true);                                           \
    } while (0)

    // stages 0 and 1 requested; stage 0 read in full; G1..G4 of stage 0 with the request of stage 2
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        S3_DBASE();
#pragma unroll
        for (int w = 0; w < 12; ++w) S3_D1(q, w);
    }
    __builtin_amdgcn_s_waitcnt(0x0F7C);  // vmcnt(12): stage 0 has landed
    __syncthreads();
    S3_R(ah[0], ra, 0, 0);
    S3_R(bm, rb, 0, 1);
    S3_R(am, ra, 0, 1);
    S3_R(bh, rb, 0, 0);
    S3_R(al, ra, 0, 2);
    S3_R(bl, rb, 0, 2);
    S3_DBASE();
    S3_PIN();
#pragma unroll
    for (int w = 0; w < 4; ++w) S3_D1(2, w);
    S3_PIN();
    S3_FIRST_GROUPS(ah[0], 2, 4, 0, false);

    const int nb = niter - 1;  // bodies: body s ends stage s and begins stage s+1
    int s = 0;
    for (; s + 6 <= nb; s += 6) {
        S3_BODY(1, 0, 0, 1);
        S3_BODY(2, 1, 1, 0);
        S3_BODY(0, 2, 0, 1);
        S3_BODY(1, 0, 1, 0);
        S3_BODY(2, 1, 0, 1);
        S3_BODY(0, 2, 1, 0);
    }
    const int rest = nb - s;  // s is a multiple of six: slots and parity continue at the start of the cycle
    if (rest > 0) S3_BODY(1, 0, 0, 1);
    if (rest > 1) S3_BODY(2, 1, 1, 0);
    if (rest > 2) S3_BODY(0, 2, 0, 1);
    if (rest > 3) S3_BODY(1, 0, 1, 0);
    if (rest > 4) S3_BODY(2, 1, 0, 1);
    // G5 of the last stage (its Ah set is the one of its parity)
    if (!IDLE && (nb & 1)) {
#pragma unroll
        for (int b = 0; b < 4; ++b) ah[0][b] = ah[1][b];
    }
#pragma unroll
    for (int bi = 0; bi < 4; ++bi) S3_M4(ah[0], bl, bi);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing may still be writing LDS
#undef S3_DBASE
#undef S3_D1
#undef S3_R
#undef S3_M4
#undef S3_PIN
#undef S3_FIRST_GROUPS
#undef S3_LAST_GROUP
#undef S3_BODY
}

// Pass 2: acc += h^T h over the h plane, the K loop of curvature_syrk_bf16_256_kernel (slabs of 32 tokens,
// 16 KB per operand, in a 4-stage ring; the caller has made sure nothing of pass 1 is still using LDS), written
// for any pair of planes.
typedef _Float16 s3_halfx8 __attribute__((ext_vector_type(8)));

// xa, xb: the plane the row panel / the column panel is taken from (packed layout, `groups` k-groups of
// `row_bytes_a` / `row_bytes_b`); F16: the planes hold float16 (MFMA 32x32x16 f16) instead of bfloat16.
template <int MODE, bool F16>
__device__ __forceinline__ void s3_pass_planes(const char *xa, const char *xb, size_t row_bytes_a, size_t row_bytes_b, int groups,
                                               int m0, int n0, const char *lds_a, const char *lds_b, floatx16 (&acc)[4][4])
{
    constexpr bool IDLE = MODE == S3_WAVE_IDLE, LOWER = MODE == S3_WAVE_LOWER;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
    const int niter = groups / BF_SLAB_GROUPS;
    const unsigned va = (unsigned)(((size_t)m0 + lane) * 16);
    const unsigned vb = (unsigned)(((size_t)n0 + lane) * 16);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const unsigned la0 = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(const __attribute__((address_space(3))) char *)lds_a) + wave_s * (B2_TILE * 16);
    const unsigned lb0 = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(const __attribute__((address_space(3))) char *)lds_b) + wave_s * (B2_TILE * 16);
    typedef const __attribute__((address_space(3))) char *lds_ptr;
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(3))) u32x4 *lds_ptr16;
    // k step t of a slab uses k-groups 2t and 2t+1 (one per half wave)
    const lds_ptr ra = (lds_ptr)lds_a + (lh * B2_TILE + wm + li) * 16;
    const lds_ptr rb = (lds_ptr)lds_b + (lh * B2_TILE + wn + li) * 16;

    u32x4 fa[2][4], fb[2][4];  // [k step parity][block]
    int gd = 0;
    const char *sbase_a = xa, *sbase_b = xb;
    // wave w fetches k-group gd + w: the 256 columns of each operand in four 64-column pieces
#define H2_DBASE()                                                                         \
    do {                                                                                   \
        const size_t g_ = (size_t)min(gd + wave_s, groups - 1);                            \
        sbase_a = xa + g_ * row_bytes_a;                                                   \
        sbase_b = xb + g_ * row_bytes_b;                                                   \
        gd += BF_SLAB_GROUPS;                                                              \
    } while (0)
#define H2_D1(st, w)                                                                                           \
    do {                                                                                                       \
        if (((w) & 1) == 0)                                                                                    \
            tn_dma16_s(reinterpret_cast<const float *>(sbase_a + ((w) >> 1) * 1024), va,                       \
                       la0 + (st) * B2_STAGE_BYTES + ((w) >> 1) * 1024);                                       \
        else                                                                                                   \
            tn_dma16_s(reinterpret_cast<const float *>(sbase_b + ((w) >> 1) * 1024), vb,                       \
                       lb0 + (st) * B2_STAGE_BYTES + ((w) >> 1) * 1024);                                       \
    } while (0)
#define H2_R(set, base, st, t)                                                                                 \
    do {                                                                                                       \
        if (!IDLE) _Pragma("unroll") for (int b = 0; b < 4; ++b)                                               \
            set[b] = *(lds_ptr16)((base) + (st) * B2_STAGE_BYTES + 2 * (t) * B2_TILE * 16 + b * 512);          \
    } while (0)
#define H2_MG(set, bi)                                                                                         \
    do {                                                                                                       \
        if (!IDLE) _Pragma("unroll") for (int bj = 0; bj < (LOWER ? (bi) + 1 : 4); ++bj) {                     \
            if (F16)                                                                                           \
                acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(                                          \
                    __builtin_bit_cast(s3_halfx8, fa[set][bi]), __builtin_bit_cast(s3_halfx8, fb[set][bj]),    \
                    acc[bi][bj], 0, 0, 0);                                                                     \
            else                                                                                               \
                acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                         \
                    __builtin_bit_cast(bf16x8, fa[set][bi]), __builtin_bit_cast(bf16x8, fb[set][bj]),          \
                    acc[bi][bj], 0, 0, 0);                                                                     \
        }                                                                                                      \
    } while (0)
#define H2_PIN() __builtin_amdgcn_sched_barrier(0)
#define H2_ITER(st0, st1, st3)                                                             \
    do {                                                                                   \
        H2_DBASE();                                                                        \
        H2_PIN();                                                                          \
        H2_MG(0, 0);                                                                       \
        H2_PIN();                                                                          \
        H2_R(fa[1], ra, st0, 1);                                                           \
        H2_D1(st3, 0);                                                                     \
        H2_PIN();                                                                          \
        H2_MG(0, 1);                                                                       \
        H2_PIN();                                                                          \
        H2_R(fb[1], rb, st0, 1);                                                           \
        H2_D1(st3, 1);                                                                     \
        H2_PIN();                                                                          \
        H2_MG(0, 2);                                                                       \
        H2_PIN();                                                                          \
        H2_D1(st3, 2);                                                                     \
        H2_PIN();                                                                          \
        H2_MG(0, 3);                                                                       \
        H2_PIN();                                                                          \
        H2_D1(st3, 3);                                                                     \
        H2_PIN();                                                                          \
        H2_MG(1, 0);                                                                       \
        H2_PIN();                                                                          \
        H2_R(fa[0], ra, st1, 0);                                                           \
        H2_D1(st3, 4);                                                                     \
        H2_PIN();                                                                          \
        H2_MG(1, 1);                                                                       \
        H2_PIN();                                                                          \
        H2_R(fb[0], rb, st1, 0);                                                           \
        H2_D1(st3, 5);                                                                     \
        H2_PIN();                                                                          \
        H2_MG(1, 2);                                                                       \
        H2_PIN();                                                                          \
        H2_D1(st3, 6);                                                                     \
        H2_D1(st3, 7);                                                                     \
        H2_PIN();                                                                          \
        H2_MG(1, 3);                                                                       \
        H2_PIN();                                                                          \
        __builtin_amdgcn_s_waitcnt(0x0F78); /* vmcnt(8): all but the newest slab landed */ \
        __syncthreads();                                                                   \
        H2_PIN();                                                                          \
    } while (0)

#pragma unroll
    for (int q = 0; q < 3; ++q) {
        H2_DBASE();
#pragma unroll
        for (int w = 0; w < 8; ++w) H2_D1(q, w);
    }
    __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt(8): slabs 0 and 1 have landed
    __syncthreads();
    H2_R(fa[0], ra, 0, 0);
    H2_R(fb[0], rb, 0, 0);
    int s = 0;
    for (; s + 4 <= niter; s += 4) {
        H2_ITER(0, 1, 3);
        H2_ITER(1, 2, 0);
        H2_ITER(2, 3, 1);
        H2_ITER(3, 0, 2);
    }
    const int rest = niter - s;  // s is a multiple of four: the stages continue at 0
    if (rest > 0) H2_ITER(0, 1, 3);
    if (rest > 1) H2_ITER(1, 2, 0);
    if (rest > 2) H2_ITER(2, 3, 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing may still be writing LDS
#undef H2_DBASE
#undef H2_D1
#undef H2_R
#undef H2_MG
#undef H2_PIN
#undef H2_ITER
}

template <int MODE>
__device__ __forceinline__ void s3_mainloop(const SyrkProblem &pr, int m0, int n0, const char *lds_a, const char *lds_b,
                                            floatx16 (&acc)[4][4])
{
    s3_pass_small<MODE>(pr, m0, n0, lds_a, lds_b, acc);
    __syncthreads();  // every wave has read its last fragments of pass 1 (and waited for its own loads)
    const char *h = static_cast<const char *>(pr.x);  // plane 0
    s3_pass_planes<MODE, false>(h, h, (size_t)pr.ldx * 16, (size_t)pr.ldx * 16, pr.n / BF_KG, m0, n0, lds_a, lds_b, acc);
}

__global__ __launch_bounds__(256, 1) void curvature_syrk_split3_256_kernel(const Syrk256Launch lp)
{
    static_assert(S3_STAGES * S3_STAGE_BYTES >= B2_STAGES * B2_STAGE_BYTES, "pass 2 reuses the LDS of pass 1");
    __shared__ __attribute__((aligned(16))) char lds_a[S3_STAGES * S3_STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) char lds_b[S3_STAGES * S3_STAGE_BYTES];

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

    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    if (bt.diag && wave_s == 1) {
        s3_mainloop<S3_WAVE_IDLE>(pr, m0, n0, lds_a, lds_b, acc);
        return;
    }
    if (bt.diag && wave_s != 2)
        s3_mainloop<S3_WAVE_LOWER>(pr, m0, n0, lds_a, lds_b, acc);
    else
        s3_mainloop<S3_WAVE_FULL>(pr, m0, n0, lds_a, lds_b, acc);
    b2_store_batched(acc, pr, lp.alpha, lp.beta, m0, n0, wm, wn, li, lh, bt.diag);
}

}  // namespace kfac
