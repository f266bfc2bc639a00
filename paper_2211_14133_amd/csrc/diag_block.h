// Diagonal-block step of the blocked upper Cholesky factorisation M = U^T U and
// the small helper kernels of the inversion.
//
// One workgroup factors one NB x NB diagonal block held in LDS and also inverts
// the triangular factor, because both the panel solve of the factorisation and
// the bottom level of the triangular inverse need U_kk^-1.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tn_gemm.h"

namespace kfac {

constexpr int NB = INV_NB;  // panel width of the blocked factorisation (= tile size of the engine)
static_assert(NB == 128, "the sub-block structure below is written for 128");
constexpr int DIAG_THREADS = TN_THREADS;
constexpr int PREP_MAX_ITEMS = 80;

struct DiagItem {
    float *F;    // top-left of the diagonal block inside the working copy (upper triangle valid)
    float *S;    // same block of the inverse-factor storage
    int *info;   // status word of the matrix
    int n;       // block size (<= NB)
    int ldf;
    int lds;
    int pivot_base;  // index of the block's first row in the whole matrix
};

constexpr int SB = 32;        // sub-block handled by one wave
constexpr int LDT = NB + 4;   // LDS row stride in floats

typedef float diag_floatx16 __attribute__((ext_vector_type(16)));


// One LDS array X (NB x LDT) holds everything: U on and above the diagonal, W^T = U^-T strictly below it
// (X[c][r] = W[r][c] for r < c) and the diagonal of W in a small array of its own.  With a single array
// two workgroups fit on a CU.  The products read their operands through one of these views (absolute
// coordinates: the element in row `kr`, column `cc` of the operand block):
enum DiagView : int {
    DV_DIRECT = 0,   // X[kr][cc]                         (U, or a product kept above the diagonal)
    DV_TRANSPOSED,   // X[cc][kr]                         (U12^T read from the block above the diagonal)
    DV_W,            // W[kr][cc] (upper triangular):  X[cc][kr] for kr < cc, wd[kr] for kr == cc, 0 for kr > cc
    DV_W_T           // W[cc][kr] (its mirror):        X[kr][cc] for kr > cc, wd[kr] for kr == cc, 0 for kr < cc
};

__device__ inline float diag_bcast(float v, int src_lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src_lane));
}

template <int VIEW>
__device__ __forceinline__ float diag_fetch(const float (*X)[LDT], const float *wd, int kr, int cc)
{
    if (VIEW == DV_DIRECT) return X[kr][cc];
    if (VIEW == DV_TRANSPOSED) return X[cc][kr];
    if (VIEW == DV_W) {
        const float v = (kr < cc) ? X[cc][kr] : wd[kr];  // one LDS read either way
        return (kr > cc) ? 0.f : v;
    }
    const float v = (kr > cc) ? X[kr][cc] : wd[kr];
    return (kr < cc) ? 0.f : v;
}

// One wave: acc = A^T B for a 32 x 32 output; A[k][m] is the element (ak0 + k, am0 + m) of view VA,
// B[k][n] the element (bk0 + k, bn0 + n) of view VB, k < K.
template <int VA, int VB>
__device__ inline diag_floatx16 sb_mma(const float (*X)[LDT], const float *wd, int ak0, int am0, int bk0, int bn0, int K, int lane)
{
    const int i = lane & 31, h = lane >> 5;
    diag_floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll 8
    for (int kk = 0; kk < K; kk += 2) {
        const float a = diag_fetch<VA>(X, wd, ak0 + kk + h, am0 + i);
        const float b = diag_fetch<VB>(X, wd, bk0 + kk + h, bn0 + i);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    }
    return acc;
}

// Store a wave's 32 x 32 result (MFMA accumulator layout: element (i, j) of the block) to X[cm0 + i][cn0 + j],
// or transposed to X[cn0 + j][cm0 + i]; with `sub` the value is subtracted from what X holds (trailing update).
template <bool TRANSPOSED>
__device__ inline void sb_store(diag_floatx16 acc, float (*X)[LDT], int cm0, int cn0, float scale, bool sub, int lane)
{
    const int j = lane & 31, h = lane >> 5;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = 8 * (r >> 2) + 4 * h + (r & 3);
        float v = scale * acc[r];
        if (TRANSPOSED) {
            X[cn0 + j][cm0 + i] = v;
        } else {
            if (sub) v += X[cm0 + i][cn0 + j];
            X[cm0 + i][cn0 + j] = v;
        }
    }
}

// One wave factors the 32 x 32 diagonal sub-block at offset o (upper triangle of X) as U^T U and inverts U,
// all in registers.  The symmetric block T and a second matrix V (starting as the identity) are kept in MFMA
// accumulator layout (lane = column, 16 rows per lane).  Step j takes the pivot with one readlane, scales
// row j and applies the elimination of column j to T and V as rank-one updates, one MFMA 32x32x2 each (the
// vector -u feeds the rows, the scaled pivot row the columns; the second K slot is zero).  The same row
// operations that turn T into U turn the identity into U^-T = W^T.  Row j of U and of W^T are final at step j
// and go to LDS then, as ONE row of X: U[j][c] for c >= j, W^T[j][c] = W[c][j] for c < j, and W[j][j] to wd;
// nothing is read back and there is no barrier inside.  Returns the 1-based local index of the first bad
// pivot, or 0.
__device__ inline int sb_factor_invert(float (*X)[LDT], float *wd, int o, int lane)
{
    __shared__ float dump[2 * SB];  // where lanes put the stores that must not land anywhere
    const int c = lane & 31, h = lane >> 5;
    diag_floatx16 T, V;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = 8 * (r >> 2) + 4 * h + (r & 3);
        T[r] = (i <= c) ? X[o + i][o + c] : X[o + c][o + i];
        V[r] = (i == c) ? 1.f : 0.f;
    }
    // Row j lives in the lanes of half hj = (j / 4) % 2.  Everything that depends on "is this my row"
    // is prepared here for both parities, so that a step has little address arithmetic: the row's store
    // address is a base plus an immediate, and the other half's values are multiplied by zero.
    float *rowp[2];
    float keep[2];
#pragma unroll
    for (int hp = 0; hp < 2; ++hp) {
        const bool mine = (h == hp);
        rowp[hp] = mine ? &X[o][o + c] : &X[o][NB];  // + j rows: element (o + j, o + c); the others hit a pad column
        keep[hp] = mine ? 1.f : 0.f;
    }
    // The 32 steps are one dependent chain (MFMA on T -> pivot -> scale -> MFMA on T), so the order
    // is pinned: first what the next MFMA on T needs, then the update of V, which runs in the shadow
    // of the chain.  Pivots are not checked inside the loop; a pivot that is not positive makes its
    // U[j][j] (= sqrt of the pivot) a NaN, and so everything after it, which is tested at the end
    // (the caller discards the result of a failed matrix).
#pragma unroll
    for (int j = 0; j < SB; ++j) {
        const int hj = (j >> 2) & 1, rj = 4 * (j >> 3) + (j & 3);  // row j lives in half hj, register rj
        const float piv = diag_bcast(T[rj], j + 32 * hj);
        const float rinv = __builtin_amdgcn_rsqf(piv) * keep[hj];  // v_rsq_f32 is accurate to one ulp
        const float u = T[rj] * rinv;            // U[j][c] in the lanes of half hj, 0 in the others
        const float au = (c > j) ? -u : 0.f;     // rows below j are eliminated
        __builtin_amdgcn_sched_barrier(0);
        T = __builtin_amdgcn_mfma_f32_32x32x2f32(au, u, T, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        const float vrow = V[rj] * rinv;         // row j of U^-T = column j of W, final (0 for c > j)
        rowp[hj][j * LDT] = (c >= j) ? u : vrow;
        float *dp = (c == j && h == hj) ? &wd[o + j] : &dump[lane];
        *dp = vrow;
        __builtin_amdgcn_sched_barrier(0);
        V = __builtin_amdgcn_mfma_f32_32x32x2f32(au, vrow, V, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        // row j of V stays unscaled in the accumulator; it is never read again
    }
    // first pivot whose square root is not a positive finite number
    const float ujj = X[o + c][o + c];
    const unsigned long long ok = __ballot(ujj > 0.f && ujj <= 3.0e38f);
    const unsigned fail = ~(unsigned)ok;
    const int bad = fail ? __builtin_ctz(fail) + 1 : 0;
    return bad;
}

// In:  F block = current (already updated) diagonal block, upper triangle.
// Out: S block = W = U_kk^-1 (U_kk^T U_kk = block) with zeros below the diagonal;
//      F block = W^T with zeros above the diagonal.
// The block is handled in LDS as 4 x 4 sub-blocks of 32 with the same blocked
// algorithm as the whole matrix: wave-level factorisation of a diagonal
// sub-block, MFMA products for the panel solve, the trailing update and the
// pairwise merges of the triangular inverse.  A block smaller than NB is padded
// with the identity.  A pivot that is not positive (or not finite) is recorded
// in *info as its 1-based index in the whole matrix (first failure wins); what
// follows it in that matrix is not meaningful (NaNs) and the caller discards the
// result.
__device__ __forceinline__ void diag_block_body(const DiagItem &it, float (*X)[LDT], float *wd)
{
    const int n = it.n;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // the working copy's rows are 16-byte aligned (ld multiple of 32, block offsets multiples of 128)
    {
        const int c4 = (tid & 31) << 2, r0 = tid >> 5;
        float4 v[NB / 8];
#pragma unroll
        for (int q = 0; q < NB / 8; ++q) {
            const int r = r0 + 8 * q;
            v[q] = *reinterpret_cast<const float4 *>(&it.F[(size_t)min(r, n - 1) * it.ldf + min(c4, max(n - 4, 0))]);
        }
        const bool whole = (n == NB);
#pragma unroll
        for (int q = 0; q < NB / 8; ++q) {
            const int r = r0 + 8 * q;
            float e[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
            if (!whole) {  // ragged last block: reload element-wise and pad with the identity
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int c = c4 + t;
                    e[t] = (r < n && c < n) ? it.F[(size_t)r * it.ldf + c] : ((r == c) ? 1.f : 0.f);
                }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int c = c4 + t;
                e[t] = (r <= c || r >= n || c >= n) ? e[t] : 0.f;
            }
            // rows of X are 16-byte aligned (LDT * 4 = 528 bytes)
            *reinterpret_cast<float4 *>(&X[r][c4]) = make_float4(e[0], e[1], e[2], e[3]);
        }
    }
    __syncthreads();
    // Phase 1: right-looking factorisation over the four 32-wide panels.
    for (int p = 0; p < NB / SB; ++p) {
        const int o = p * SB;
        if (wave == 0) {
            const int bad = sb_factor_invert(X, wd, o, lane);
            if (bad != 0 && lane == 0 && o + bad <= n) atomicCAS(it.info, 0, it.pivot_base + o + bad);
        }
        __syncthreads();
        // panel solve: U[p][q] = W_pp^T T[p][q]
        for (int q = p + 1 + wave; q < NB / SB; q += 4) {
            const diag_floatx16 acc = sb_mma<DV_W, DV_DIRECT>(X, wd, o, o, o, q * SB, SB, lane);
            sb_store<false>(acc, X, o, q * SB, 1.f, false, lane);
        }
        __syncthreads();
        // trailing update: T[q][r] -= U[p][q]^T U[p][r] for p < q <= r
        int job = 0;
        for (int q = p + 1; q < NB / SB; ++q)
            for (int r = q; r < NB / SB; ++r, ++job) {
                if ((job & 3) != wave) continue;
                const diag_floatx16 acc = sb_mma<DV_DIRECT, DV_DIRECT>(X, wd, o, q * SB, o, r * SB, SB, lane);
                sb_store<false>(acc, X, q * SB, r * SB, -1.f, true, lane);
            }
        __syncthreads();
    }
    // Phase 2: W = U^-1 by pairwise merges, [U11 U12; 0 U22]^-1 = [W11, -W11 U12 W22; 0, W22].  A level has at
    // most four 32 x 32 output blocks per product, one per wave.
    for (int b = SB; b < NB; b *= 2) {
        const int nodes = NB / (2 * b), sub = b / SB;       // sub x sub output sub-blocks per node
        const int jobs = nodes * sub * sub;                  // 2 (b = 32) or 4 (b = 64)
        const int nd = wave / (sub * sub), bi = (wave / sub) % sub, bj = wave % sub;
        const int r0 = nd * 2 * b, c1 = r0 + b;
        const bool busy = wave < jobs;
        // Y = U12 W22, stored where U12 was: every wave reads U12 before anyone overwrites it
        diag_floatx16 acc;
        if (busy) acc = sb_mma<DV_TRANSPOSED, DV_W>(X, wd, c1, r0 + bi * SB, c1, c1 + bj * SB, b, lane);
        __syncthreads();
        if (busy) sb_store<false>(acc, X, r0 + bi * SB, c1 + bj * SB, 1.f, false, lane);
        __syncthreads();
        // W12 = -W11 Y, W11 read through its mirror; kept as its mirror, below the diagonal
        if (busy) {
            acc = sb_mma<DV_W_T, DV_DIRECT>(X, wd, r0, r0 + bi * SB, r0, c1 + bj * SB, b, lane);
            sb_store<true>(acc, X, r0 + bi * SB, c1 + bj * SB, -1.f, false, lane);
        }
        __syncthreads();
    }
    // S block: W (read transposed from below the diagonal of X) with zeros below its diagonal; F block: W^T with
    // zeros above (U_jj, which was there, is not needed again).
    {
        const int c4 = (tid & 31) << 2, r0 = tid >> 5;
#pragma unroll
        for (int q = 0; q < NB / 8; ++q) {
            const int r = r0 + 8 * q;
            float e[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int c = c4 + t;
                e[t] = (r > c) ? X[r][c] : ((r == c) ? wd[r] : X[c][r]);  // W^T where r >= c, W where r <= c
            }
            float w[4], wt[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                w[t] = r > c4 + t ? 0.f : e[t];
                wt[t] = r < c4 + t ? 0.f : e[t];
            }
            if (n == NB) {
                *reinterpret_cast<float4 *>(&it.S[(size_t)r * it.lds + c4]) = make_float4(w[0], w[1], w[2], w[3]);
                *reinterpret_cast<float4 *>(&it.F[(size_t)r * it.ldf + c4]) = make_float4(wt[0], wt[1], wt[2], wt[3]);
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int c = c4 + t;
                    if (r < n && c < n) {
                        it.S[(size_t)r * it.lds + c] = w[t];
                        it.F[(size_t)r * it.ldf + c] = wt[t];
                    }
                }
            }
        }
    }
}

// The launches of the blocked inversion that contain diagonal blocks: a workgroup either factors one
// diagonal block (INV_DIAG node) or computes one tile of a contraction node, exactly as in
// invert_gemm_kernel.  The diagonal-block algorithm works in one 66 KB array of LDS, a little more than the
// engine's slab ring, so two workgroups share a CU as in every other launch; the few workgroups with
// diagonal blocks are on the critical path of the factorisation while the tiles of independent work keep
// the rest of the chip busy.
__global__ __launch_bounds__(TN_THREADS, 2) void invert_diag_gemm_kernel(const InvLaunch lp)
{
    __shared__ __attribute__((aligned(16))) float lds[NB * LDT + NB];
    static_assert(NB * LDT >= TN_LDS_STAGES * BK * (BM + BN), "the engine's slab ring fits into the same LDS");
    const int logical = tn_logical_tile(blockIdx.x, gridDim.x, lp.c);
    if (logical < 0) return;  // whole workgroup
    TnProblem pr;
    TnAttr at;
    TnTile tl = tn_locate(lp, logical, pr, at);
    const InvNode &nd = lp.n[tl.prob];
    const bool is_diag = nd.op == INV_DIAG;
    if (is_diag && nd.c != 0) {
        // the diagonal block first takes the update with the block rows above it (one tile, K = 128 (a - b))
        pr = lp.diag_update(tl.prob);
        at = InvLaunch::op_attr(INV_ROW_UPDATE);
        tl.ti = tl.tj = tl.m0 = tl.n0 = tl.split = tl.kbase = tl.kt0 = 0;
        tl.kt1 = pr.K / BK;
        tl.diag = false;
    }
    if (!is_diag || nd.c != 0)
        tn_tile_work(lp, pr, at, tl, logical,
                     *reinterpret_cast<float (*)[TN_LDS_STAGES][BK][BM]>(lds),
                     *reinterpret_cast<float (*)[TN_LDS_STAGES][BK][BN]>(lds + TN_LDS_STAGES * BK * BM));
    if (is_diag) {
        if (nd.c != 0) __syncthreads();  // the block's stores above are read back below, by other lanes
        const InvMatDesc &mt = lp.m[nd.mat];
        const size_t q0 = (size_t)nd.a * NB, off = q0 * mt.ld + q0;
        DiagItem it;
        it.F = lp.mat_f(nd.mat) + off;
        it.S = lp.mat_s(nd.mat) + off;
        it.info = mt.info;
        it.n = min(NB, (int)mt.d - (int)q0);
        it.ldf = mt.ld;
        it.lds = mt.ld;
        it.pivot_base = (int)q0;
        diag_block_body(it, reinterpret_cast<float (*)[LDT]>(lds), lds + NB * LDT);
    }
}

struct PrepItem {
    const float *src;  // caller's factor
    float *dst;        // working copy
    int *info;
    int d;
    int lds_;          // ld of src
    int ldd;           // ld of dst
};

struct PrepLaunch {
    PrepItem it[PREP_MAX_ITEMS];
    float damping;
};

__global__ void invert_clear_info_kernel(const PrepLaunch pl, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) *pl.it[i].info = 0;
}

// dst = src + damping * I for the upper triangle (column >= row): only that is input, and nothing reads the
// rest of the working copy before the inversion has written it (what a product reads and discards there, the
// lower part of a diagonal block, may hold anything).  A non-finite element of the upper triangle sets info = -1.
__global__ __launch_bounds__(256) void invert_prepare_kernel(const PrepLaunch pl)
{
    const PrepItem &it = pl.it[blockIdx.y];
    const int d = it.d;
    bool bad = false;
    const bool vec = ((it.lds_ & 3) == 0) && ((reinterpret_cast<uintptr_t>(it.src) & 15) == 0);  // dst rows are aligned
    for (int r = blockIdx.x; r < d; r += gridDim.x) {
        const float *src = it.src + (size_t)r * it.lds_;
        float *dst = it.dst + (size_t)r * it.ldd;
        if (vec) {
            for (int c = (r & ~3) + threadIdx.x * 4; c < d; c += blockDim.x * 4) {
                float4 v;
                if (c + 3 < d) {
                    v = *reinterpret_cast<const float4 *>(src + c);
                } else {
                    v.x = src[c];
                    v.y = (c + 1 < d) ? src[c + 1] : 0.f;
                    v.z = (c + 2 < d) ? src[c + 2] : 0.f;
                    v.w = 0.f;
                }
                if ((c + 0 >= r && !(fabsf(v.x) <= 3.0e38f)) || (c + 1 >= r && !(fabsf(v.y) <= 3.0e38f)) ||
                    (c + 2 >= r && !(fabsf(v.z) <= 3.0e38f)) || (c + 3 >= r && !(fabsf(v.w) <= 3.0e38f)))
                    bad = true;
                if (r >= c && r < c + 4) {
                    if (r == c) v.x += pl.damping;
                    if (r == c + 1) v.y += pl.damping;
                    if (r == c + 2) v.z += pl.damping;
                    if (r == c + 3) v.w += pl.damping;
                }
                *reinterpret_cast<float4 *>(dst + c) = v;  // ld of the working copy is a multiple of 32 >= d
            }
        } else {
            for (int c = r + threadIdx.x; c < d; c += blockDim.x) {
                float v = src[c];
                if (c >= r && !(fabsf(v) <= 3.0e38f)) bad = true;
                if (r == c) v += pl.damping;
                dst[c] = v;
            }
        }
    }
    if (bad) atomicCAS(it.info, 0, -1);
}

}  // namespace kfac
