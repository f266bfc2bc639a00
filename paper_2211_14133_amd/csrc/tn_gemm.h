// Grouped fp32 "TN" contraction engine for gfx950:  C = alpha * A^T B + beta * C.
//
// Both operands are row-major with the contraction index as the ROW index
// (A is K x M, B is K x N).  Every contraction of the K-FAC work items has that
// shape once the symmetry of the factors and of their inverses is used:
//   curvature    X^T X                     (tokens are rows of X)
//   precondition G^T B^-1, then T^T A^-1   (B^-1, A^-1 symmetric)
//   inversion    the updates of an upper Cholesky factorisation M = U^T U,
//                the triangular inverse and the product W W^T, with transposed
//                copies kept so that each left operand can be read row-wise.
// so one main loop serves all of them: rows of both operands are contiguous,
// loads are 512-byte coalesced and go to LDS without a transpose.
//
// Tiling: a 256-thread workgroup (4 wave64) owns a 128 x 128 tile of C; each
// wave owns 64 x 64 as 2 x 2 MFMA 32x32x2 blocks (64 accumulator registers).
// K advances in slabs of 16 through a ring of LDS stages: straight from global
// memory into LDS for aligned tiles (tn_mainloop_direct), through staging
// registers with a zero fix-up for ragged ones (tn_mainloop).
// The token sum is folded into a second accumulator every TN_CHUNK_SLABS slabs, so
// the fp32 rounding error grows with the chunk length, not with K.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <functional>
#include <vector>

namespace kfac {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;
constexpr int BN = 128;
constexpr int BK = 16;
constexpr int TN_THREADS = 256;
constexpr int TN_MAX_PROBLEMS = 48;
constexpr int TN_CHUNK_SLABS = 16;  // fold the running sum every 16 * 16 = 256 rows of K (128 rows cost 1.2 % more time)
constexpr int SUPER_ROWS = 8;      // tiles of 8 consecutive tile-rows are scheduled together

enum TileMode : int { TILE_FULL = 0, TILE_LOWER = 1, TILE_UPPER = 2 };
// Triangular operands.  MASK_ZEROS_K_LT / MASK_ZEROS_K_GT: the caller guarantees that the operand holds zeros
// where k < m (k > m) inside the 128 x 128 block on its diagonal; what lies beyond that block on the zero side
// may hold anything and is never read, because the K range of a tile is clipped to start (end) at its own
// diagonal block.  No element is masked: such tiles take the same loops as every other.
enum OperandMask : int { MASK_NONE = 0, MASK_ZEROS_K_LT = 3, MASK_ZEROS_K_GT = 4 };

struct TnProblem {
    const float *A;    // K x M, lda
    const float *B;    // K x N, ldb
    float *C;          // M x N, ldc (read when beta != 0)
    float *Ct;         // optional mirror: Ct[n * ldct + m] = C[m][n]
    const int *guard;  // optional: stores are skipped when *guard != 0
    int M, N, K;
    int lda, ldb, ldc, ldct;
    int tile_begin;    // first logical tile (tile * splits + split) of this problem
};

// What may differ from problem to problem inside one launch.
struct TnAttr {
    int tile_mode;     // TILE_LOWER / TILE_UPPER need M == N
    int mask_a;
    int mask_b;
    int reverse_cols;  // TILE_FULL only: walk the tile columns from the last to the first (set when K grows
                       // with the column, so that the long tiles of a range run first, not last)
    float alpha;
    float beta;
};

struct TnCommon {
    int count;
    int tile_mode;  // the attributes of every problem of a general or curvature launch (see TnAttr)
    int mask_a;
    int mask_b;
    int splits;     // > 1: partial tiles go to `partial`, the reduce kernel finishes
    float alpha;
    float beta;
    float *partial;  // [total logical tiles][BM * BN]
    int slab_align;  // K ranges of split tiles are multiples of this many slabs (0 or 1: any)
    int reverse_cols;
    int xcd_balanced;  // 0: each XCD takes a contiguous eighth of the tiles; 1: the ranges below;
                       // 2: each XCD takes an eighth of every problem (tn_deal_xcds)
    int total_tiles;   // logical tiles of the launch (used when xcd_balanced == 2)
    // XCD x works on logical tiles xcd_begin[x] .. xcd_begin[x+1]-1 and then on xcd_begin2[x] .. xcd_begin2[x+1]-1
    // (two lists of tiles, each dealt to all eight XCDs: work that the next launch waits for, then work that
    // only fills the chip; see tn_balance_xcds)
    int xcd_begin[9];
    int xcd_begin2[9];
    __host__ __device__ TnAttr attr() const
    {
        TnAttr a;
        a.tile_mode = tile_mode; a.mask_a = mask_a; a.mask_b = mask_b; a.reverse_cols = reverse_cols;
        a.alpha = alpha; a.beta = beta;
        return a;
    }
};

// General launch: up to TN_MAX_PROBLEMS arbitrary problems.
struct TnLaunch {
    static constexpr bool kPackedBf16 = false;
    TnProblem p[TN_MAX_PROBLEMS];
    TnCommon c;
    static constexpr bool kHasDiag = false;
    __host__ __device__ int tile_begin(int i) const { return p[i].tile_begin; }
    __host__ __device__ TnProblem problem(int i) const { return p[i]; }
    __host__ __device__ TnAttr attr(int) const { return c.attr(); }
    __host__ __device__ int fixed_cost(int) const { return 0; }
};

// Curvature launch: factor = beta * factor + alpha * x^T x.  Both operands are x
// and the output is mirrored onto itself, so the descriptor is small enough for
// every factor of a pipeline stage to go into one launch.
constexpr int SYRK_MAX_PROBLEMS = 80;

struct SyrkProblem {
    const void *x;   // float32 [n, d] with ldx, or the packed bfloat16 copy (then n, ldx are its padded sizes)
    float *factor;   // d x d, ldf
    int n, d, ldx, ldf;
    int tile_begin;
    int pad_;
};

// PACKED false: float32 x; true: bfloat16 x repacked for the bf16 MFMA (see pack_bf16_kernel)
template <bool PACKED>
struct SyrkLaunchT {
    static constexpr bool kPackedBf16 = PACKED;
    static constexpr bool kHasDiag = false;
    SyrkProblem p[SYRK_MAX_PROBLEMS];
    TnCommon c;
    __host__ __device__ TnAttr attr(int) const { return c.attr(); }
    __host__ __device__ int fixed_cost(int) const { return 0; }
    __host__ __device__ int tile_begin(int i) const { return p[i].tile_begin; }
    __host__ __device__ TnProblem problem(int i) const
    {
        const SyrkProblem &q = p[i];
        TnProblem r;
        r.A = static_cast<const float *>(q.x); r.B = static_cast<const float *>(q.x); r.C = q.factor; r.Ct = q.factor; r.guard = nullptr;
        r.M = q.d; r.N = q.d; r.K = q.n;
        r.lda = q.ldx; r.ldb = q.ldx; r.ldc = q.ldf; r.ldct = q.ldf;
        r.tile_begin = q.tile_begin;
        return r;
    }
};
typedef SyrkLaunchT<false> SyrkLaunch;       // float32 activations / errors
typedef SyrkLaunchT<true> SyrkLaunchPacked;  // bfloat16 in k-interleaved layout, bf16 MFMA

// Inversion launch: every problem of the blocked inversion is a node (operation, matrix, up to three
// block indices, optionally a range of tile rows); pointers and sizes follow from the matrix table, so
// a whole stage's worth of matrices and a couple of hundred nodes fit into the kernel arguments of a
// single launch.  Nodes of different operations can share a launch: the host puts the nodes the next
// launch waits for first and fills the rest of the chip with independent work (see tn_balance_xcds).
constexpr int INV_NB = 128;  // panel width of the blocked factorisation (= BM = BN)
constexpr int INV_MAX_MATS = 72;
constexpr int INV_MAX_NODES = 216;
constexpr int INV_DIAG_COST = 40;  // a diagonal-block node takes about as long as a tile of 36 slabs

// Working storage of matrix `mat`, two d x d arrays.  F = working copy; then, block by block, the factor U in
// the blocks above the diagonal and W^T = U^-T in the diagonal blocks and below (U_jj itself is not needed
// again once W_jj is there).  S = W = U^-1 in the diagonal blocks and above; its blocks below the diagonal
// are scratch of the triangular inverse (Y^T).  Inside the diagonal blocks both arrays hold explicit zeros on
// the other side of the diagonal, so a product that reads a triangular operand from them only clips its K
// range (MASK_ZEROS_*): no element is masked and every aligned tile takes the direct loop.
enum InvOp : int {
    INV_PANEL_SOLVE = 0,  // a = block row j:                  U[j, j+1:] = W_jj^T M[j, j+1:]
    INV_ROW_UPDATE = 1,   // a = s, b = block row j, c = e:    M[j, j:] -= U[s:e, j]^T U[s:e, j:]
                          // (r0 = 1: without the diagonal tile, M[j, j+1:] only)
    // Triangular inverse of the block range [a, a+b+c) from its two inverted parts (b blocks, then c):
    //   [U11 U12; 0 U22]^-1 = [W11, -W11 U12 W22; 0, W22].
    INV_MERGE_YT = 2,     // Y^T = (W11 U12)^T, kept below the diagonal of S
    INV_MERGE_W = 3,      // W12 = -Y W22, written to S and, transposed, to F
    INV_DIAG = 4          // a = block row j: factor the diagonal block and invert its factor (diag_block.h);
                          // c = 1: first bring it up to date, M[j, j] -= U[b:j, j]^T U[b:j, j] (the diagonal tile
                          // that a row update with r0 = 1 leaves out); only in launches of invert_diag_gemm_kernel
};

struct InvMatDesc {
    int *info;            // status word of the matrix
    unsigned f_off;       // F starts this many 256-byte units into the workspace; S follows F
    unsigned short d;
    unsigned short ld;
};

struct InvNode {
    unsigned char mat, a, b, c;
    unsigned char op;
    unsigned char r0, rn;  // merges: tile rows r0 .. r0+rn-1 of the output (rn = 0: all); row update: see there
    unsigned char pad_;
    int tile_begin;
};

struct InvDims {
    int M, N, K;
};

// Rows of the output that a merge node covers: [first, first + count)
__host__ __device__ inline void inv_row_range(int rows, int r0, int rn, int &first, int &count)
{
    first = 0;
    count = rows;
    if (rn != 0) {
        first = min(rows, r0 * INV_NB);
        count = min(rows - first, rn * INV_NB);
    }
}

__host__ __device__ inline InvDims inv_dims(int op, int d, int a, int b, int c, int r0 = 0, int rn = 0)
{
    InvDims r;
    if (op == INV_PANEL_SOLVE) {
        const int q0 = a * INV_NB, n = min(INV_NB, d - q0);
        r.M = n; r.N = d - q0 - n; r.K = n;
    } else if (op == INV_ROW_UPDATE) {
        const int q0 = b * INV_NB, n = min(INV_NB, d - q0);
        r.M = n; r.N = d - q0 - (r0 ? n : 0); r.K = (c - a) * INV_NB;
    } else if (op == INV_DIAG) {
        const int q0 = a * INV_NB, n = min(INV_NB, d - q0);
        r.M = n; r.N = n; r.K = n;
    } else {
        const int b1 = b * INV_NB, c1 = a * INV_NB + b1, b2 = min(c * INV_NB, d - c1);
        int first, count;
        if (op == INV_MERGE_YT) {
            inv_row_range(b2, r0, rn, first, count);
            r.M = count; r.N = b1; r.K = b1;
        } else {
            inv_row_range(b1, r0, rn, first, count);
            r.M = count; r.N = b2; r.K = b2;
        }
    }
    return r;
}

struct InvLaunch {
    static constexpr bool kPackedBf16 = false;
    static constexpr bool kHasDiag = true;
    InvMatDesc m[INV_MAX_MATS];
    InvNode n[INV_MAX_NODES];
    TnCommon c;
    float *ws;  // workspace base
    __host__ __device__ int tile_begin(int i) const { return n[i].tile_begin; }
    __host__ __device__ int fixed_cost(int i) const
    {
        if (n[i].op != INV_DIAG) return 0;
        return INV_DIAG_COST + (n[i].c ? ((int)n[i].a - (int)n[i].b) * (INV_NB / BK) + 4 : 0);
    }
    // the update of a diagonal block that its own workgroup applies before factoring it (INV_DIAG with c = 1)
    __host__ __device__ TnProblem diag_update(int i) const
    {
        const InvNode &nd = n[i];
        const InvMatDesc &mt = m[nd.mat];
        const size_t ld = (size_t)mt.ld, k0 = (size_t)nd.b * INV_NB, q0 = (size_t)nd.a * INV_NB;
        float *F = mat_f(nd.mat);
        TnProblem r;
        r.M = r.N = min(INV_NB, (int)mt.d - (int)q0);
        r.K = ((int)nd.a - (int)nd.b) * INV_NB;
        r.lda = r.ldb = r.ldc = r.ldct = mt.ld;
        r.tile_begin = nd.tile_begin;
        r.guard = nullptr;
        r.Ct = nullptr;
        r.A = F + k0 * ld + q0;
        r.B = F + k0 * ld + q0;
        r.C = F + q0 * ld + q0;
        return r;
    }
    __host__ __device__ float *mat_f(int mat) const { return ws + (size_t)m[mat].f_off * 64; }
    __host__ __device__ float *mat_s(int mat) const
    {
        const size_t bytes = ((size_t)m[mat].d * m[mat].ld * sizeof(float) + 255) / 256 * 256;
        return mat_f(mat) + bytes / sizeof(float);
    }
    __host__ __device__ static TnAttr op_attr(int op)
    {
        TnAttr t;
        t.tile_mode = TILE_FULL;
        t.mask_a = (op == INV_PANEL_SOLVE) ? MASK_ZEROS_K_GT : MASK_NONE;  // W_jj, upper triangular (S)
        t.mask_b = (op == INV_MERGE_YT) ? MASK_ZEROS_K_LT                  // W11^T, lower triangular (F)
                 : (op == INV_MERGE_W) ? MASK_ZEROS_K_GT : MASK_NONE;      // W22, upper triangular (S)
        t.reverse_cols = (op == INV_MERGE_W) ? 1 : 0;                     // K grows with the tile column
        t.alpha = (op == INV_ROW_UPDATE || op == INV_MERGE_W) ? -1.f : 1.f;
        t.beta = (op == INV_ROW_UPDATE) ? 1.f : 0.f;
        return t;
    }
    __host__ __device__ TnAttr attr(int i) const { return op_attr(n[i].op); }
    __host__ __device__ TnProblem problem(int i) const
    {
        const InvNode &nd = n[i];
        const InvMatDesc &mt = m[nd.mat];
        const size_t ld = (size_t)mt.ld;
        float *F = mat_f(nd.mat), *S = mat_s(nd.mat);
        const InvDims dm = inv_dims(nd.op, mt.d, nd.a, nd.b, nd.c, nd.r0, nd.rn);
        TnProblem r;
        r.M = dm.M; r.N = dm.N; r.K = dm.K;
        r.lda = r.ldb = r.ldc = r.ldct = mt.ld;
        r.tile_begin = nd.tile_begin;
        r.guard = nullptr;
        r.Ct = nullptr;
        if (nd.op == INV_PANEL_SOLVE || nd.op == INV_DIAG) {
            const size_t q0 = (size_t)nd.a * INV_NB, nn = (size_t)dm.M;
            r.A = S + q0 * ld + q0;
            r.B = F + q0 * ld + q0 + nn;
            r.C = F + q0 * ld + q0 + nn;
        } else if (nd.op == INV_ROW_UPDATE) {
            const size_t k0 = (size_t)nd.a * INV_NB, q0 = (size_t)nd.b * INV_NB, skip = nd.r0 ? (size_t)dm.M : 0;
            r.A = F + k0 * ld + q0;
            r.B = F + k0 * ld + q0 + skip;
            r.C = F + q0 * ld + q0 + skip;
        } else {
            const size_t q0 = (size_t)nd.a * INV_NB, c1 = q0 + (size_t)nd.b * INV_NB;
            const int b1 = nd.b * INV_NB, b2 = min(nd.c * INV_NB, (int)mt.d - (int)c1);
            int first, count;
            if (nd.op == INV_MERGE_YT) {
                inv_row_range(b2, nd.r0, nd.rn, first, count);
                r.A = F + q0 * ld + c1 + first;          // U12: K = b1 rows, its columns are the rows of Y^T
                r.B = F + q0 * ld + q0;                  // W11^T: element (k, n) = W11[n][k], zero for k < n
                r.C = S + (c1 + first) * ld + q0;        // Y^T, b2 x b1
            } else {
                inv_row_range(b1, nd.r0, nd.rn, first, count);
                r.A = S + c1 * ld + q0 + first;          // Y^T: K = b2 rows, its columns are the rows of W12
                r.B = S + c1 * ld + c1;                  // W22, zero for k > n
                r.C = S + (q0 + first) * ld + c1;        // W12
                r.Ct = F + c1 * ld + q0 + first;         // and its transpose
            }
        }
        return r;
    }
};

// Last phase of the inversion, inv = W W^T for every matrix of the batch in ONE launch: a node is a band
// of SUPER_ROWS tile rows of one matrix's lower tile set (the tiles of a band differ little in length: the
// K range of a tile starts at its row).  The host sorts the nodes by that length, so that the long tiles
// of all matrices start first and the short ones fill up the end of the launch.
constexpr int WWT_MAX_NODES = 160;
struct WwtMat {
    float *inv;      // output, ldi
    const int *info; // stores are skipped when *info != 0
    unsigned f_off;  // as in InvMatDesc
    unsigned short d, ld;
    int ldi;
};
struct WwtNode {
    unsigned short mat, band;
    int tile_begin;
};
// tiles of a d x d lower tile set (nt tile rows) that lie in the bands before `band`
__host__ __device__ inline int wwt_band_first_tile(int band, int nt)
{
    const int r0 = min(band * 8, nt);
    return r0 * (r0 + 1) / 2;
}
struct WwtLaunch {
    static constexpr bool kPackedBf16 = false;
    static constexpr bool kHasDiag = false;
    WwtMat m[INV_MAX_MATS];
    WwtNode n[WWT_MAX_NODES];
    TnCommon c;
    float *ws;
    __host__ __device__ TnAttr attr(int) const { return c.attr(); }
    __host__ __device__ int fixed_cost(int) const { return 0; }
    __host__ __device__ int tile_begin(int i) const { return n[i].tile_begin; }
    __host__ __device__ TnProblem problem(int i) const
    {
        const WwtNode &nd = n[i];
        const WwtMat &mt = m[nd.mat];
        const float *F = ws + (size_t)mt.f_off * 64;  // W^T in its diagonal blocks and below
        TnProblem r;
        r.A = F; r.B = F; r.C = mt.inv; r.Ct = mt.inv; r.guard = mt.info;
        r.M = r.N = r.K = mt.d;
        r.lda = r.ldb = mt.ld; r.ldc = r.ldct = mt.ldi;
        // the node's tiles are the band's part of the matrix's own tile order
        r.tile_begin = nd.tile_begin - wwt_band_first_tile(nd.band, (mt.d + BM - 1) / BM);
        return r;
    }
};
static_assert(SUPER_ROWS == 8, "wwt_band_first_tile counts bands of eight tile rows");

__host__ __device__ inline int tn_tiles(int M, int N, int mode)
{
    const int tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
    return mode == TILE_FULL ? tm * tn : tm * (tm + 1) / 2;
}

// Order of the tiles of one problem: bands of SUPER_ROWS tile-rows, column by
// column inside a band, so that tiles running at the same time share operand
// columns (they hit in the XCD's L2).
__host__ __device__ inline void tn_decode_full(int idx, int tm, int tn, int &ti, int &tj)
{
    const int band = idx / (SUPER_ROWS * tn);
    const int r = idx - band * SUPER_ROWS * tn;
    const int rows = min(SUPER_ROWS, tm - band * SUPER_ROWS);
    tj = r / rows;
    ti = band * SUPER_ROWS + r % rows;
}

__host__ __device__ inline void tn_decode_lower(int idx, int nt, int &ti, int &tj)
{
    int r0 = 0, r1 = 0;
    for (;;) {
        r1 = min(r0 + SUPER_ROWS, nt);
        const int cnt = (r1 * (r1 + 1) - r0 * (r0 + 1)) / 2;
        if (idx < cnt || r1 == nt) break;
        idx -= cnt;
        r0 = r1;
    }
    const int rows = r1 - r0;
    const int rect = r0 * rows;
    if (idx < rect) {
        tj = idx / rows;
        ti = r0 + idx % rows;
        return;
    }
    idx -= rect;
    ti = tj = r1 - 1;
    for (int j = r0; j < r1; ++j) {
        const int c = r1 - j;
        if (idx < c) {
            tj = j;
            ti = j + idx;
            return;
        }
        idx -= c;
    }
}

// blockIdx -> logical tile.  Workgroups are dealt round-robin to the 8 XCDs and
// dispatched in order; each XCD has its own L2.  Every XCD works on one contiguous
// range of logical tiles (neighbouring tiles share operand panels, which then hit
// in that L2).  When all tiles cost the same the ranges are plain eighths.  When
// they do not (triangular operands clip K, problems of mixed size) the host cuts
// the list into eight ranges of equal cost instead (tn_balance_xcds): with plain
// eighths one XCD would hold the long tiles and finish long after the others.
// The grid then has 8 * (longest range) workgroups and the surplus ones of the
// shorter ranges leave at once (return value -1).
__device__ inline int tn_logical_tile(int bid, int nblocks)
{
    const int base = nblocks >> 3, rem = nblocks & 7;
    const int xcd = bid & 7, q = bid >> 3;
    return xcd * base + min(xcd, rem) + q;
}

__device__ inline int tn_logical_tile(int bid, int nblocks, const TnCommon &c)
{
    if (!c.xcd_balanced) return tn_logical_tile(bid, nblocks);
    const int xcd = bid & 7;
    int q = bid >> 3;
    const int n1 = c.xcd_begin[xcd + 1] - c.xcd_begin[xcd];
    if (q < n1) return c.xcd_begin[xcd] + q;
    q -= n1;
    const int t = c.xcd_begin2[xcd] + q;
    return t < c.xcd_begin2[xcd + 1] ? t : -1;
}

// xcd_balanced == 2: XCD x takes the x-th eighth of the tiles of every problem, problem after problem.
// For launches whose tiles cost the same within a problem and differ between problems (the precondition:
// K is the layer's width): every XCD then holds the same mix, and with the problems sorted by decreasing
// tile cost on the host each XCD starts its long tiles first and fills up with the short ones.
template <class L>
__device__ inline int tn_logical_tile_dealt(const L &ll, int bid)
{
    const int xcd = bid & 7;
    int q = bid >> 3;
    const int count = ll.c.count;
    for (int p = 0; p < count; ++p) {
        const int b = ll.tile_begin(p);
        const int n = (p + 1 < count ? ll.tile_begin(p + 1) : ll.c.total_tiles) - b;
        const int part = (xcd + p) & 7;  // rotated from problem to problem: no XCD always gets the same part
        const int lo = (int)((long long)n * part / 8), hi = (int)((long long)n * (part + 1) / 8);
        if (q < hi - lo) return b + lo + q;
        q -= hi - lo;
    }
    return -1;  // surplus workgroup
}

// K range of a tile that can hold non-zeros under the operand masks: first row kb (a multiple
// of BK) and length in slabs of BK.
__host__ __device__ inline void tn_k_range(const TnAttr &lp, int K, int m0, int n0, int &kb, int &nslab)
{
    kb = 0;
    int ke = K;
    if (lp.mask_a == MASK_ZEROS_K_LT) kb = max(kb, m0);
    if (lp.mask_a == MASK_ZEROS_K_GT) ke = min(ke, m0 + BM);
    if (lp.mask_b == MASK_ZEROS_K_LT) kb = max(kb, n0);
    if (lp.mask_b == MASK_ZEROS_K_GT) ke = min(ke, n0 + BN);
    kb = (kb / BK) * BK;
    nslab = ke > kb ? (ke - kb + BK - 1) / BK : 0;
}

struct TnTile {
    int prob, ti, tj, split, m0, n0, kt0, kt1, kbase;
    bool diag;
};

template <class L>
__device__ __forceinline__ TnTile tn_locate(const L &ll, int t, TnProblem &pr, TnAttr &at)
{
    const TnCommon &lp = ll.c;
    TnTile tl;
    int pi = 0, hi = lp.count;  // tile_begin is ascending: last problem with tile_begin <= t
    while (hi - pi > 1) {
        const int mid = (pi + hi) >> 1;
        if (ll.tile_begin(mid) <= t)
            pi = mid;
        else
            hi = mid;
    }
    pr = ll.problem(pi);
    at = ll.attr(pi);
    const int local = t - pr.tile_begin;
    const int tile = local / lp.splits;
    tl.prob = pi;
    tl.split = local - tile * lp.splits;
    const int tm = (pr.M + BM - 1) / BM, tn = (pr.N + BN - 1) / BN;
    if (at.tile_mode == TILE_FULL) {
        tn_decode_full(tile, tm, tn, tl.ti, tl.tj);
        if (at.reverse_cols) tl.tj = tn - 1 - tl.tj;
    } else {
        tn_decode_lower(tile, tm, tl.ti, tl.tj);
        if (at.tile_mode == TILE_UPPER) {
            const int s = tl.ti;
            tl.ti = tl.tj;
            tl.tj = s;
        }
    }
    tl.diag = (at.tile_mode != TILE_FULL) && (tl.ti == tl.tj);
    tl.m0 = tl.ti * BM;
    tl.n0 = tl.tj * BN;
    int kb, nslab;
    tn_k_range(at, pr.K, tl.m0, tl.n0, kb, nslab);
    int per = (nslab + lp.splits - 1) / lp.splits;
    if (lp.slab_align > 1) per = (per + lp.slab_align - 1) / lp.slab_align * lp.slab_align;
    tl.kbase = kb;
    tl.kt0 = min(nslab, tl.split * per);
    tl.kt1 = min(nslab, tl.kt0 + per);
    return tl;
}

// Host side of the blockIdx -> tile mappings.  Cost of a tile = slabs of its K range plus a constant for
// its prologue and epilogue (or the fixed cost of a node that is not a contraction).
constexpr int TN_TILE_OVERHEAD = 4;  // prologue and epilogue of a tile, in slabs

// Cost of every logical tile of a launch.
template <class L>
inline std::vector<int> tn_tile_costs(const L &ll, int total_tiles)
{
    const TnCommon &c = ll.c;
    std::vector<int> cost((size_t)total_tiles, 0);
    for (int pi = 0; pi < c.count; ++pi) {
        const TnProblem pr = ll.problem(pi);
        const TnAttr at = ll.attr(pi);
        const int fixed = ll.fixed_cost(pi);
        const int end = pi + 1 < c.count ? ll.tile_begin(pi + 1) : total_tiles;
        const int tm = (pr.M + BM - 1) / BM, tn = (pr.N + BN - 1) / BN;
        for (int t = ll.tile_begin(pi); t < end; ++t) {
            if (fixed > 0) {
                cost[(size_t)t] = fixed;
                continue;
            }
            const int local = t - pr.tile_begin, tile = local / c.splits, split = local - tile * c.splits;
            int ti, tj;
            if (at.tile_mode == TILE_FULL) {
                tn_decode_full(tile, tm, tn, ti, tj);
                if (at.reverse_cols) tj = tn - 1 - tj;
            } else {
                tn_decode_lower(tile, tm, ti, tj);
                if (at.tile_mode == TILE_UPPER) { const int sw = ti; ti = tj; tj = sw; }
            }
            int kb, nslab;
            tn_k_range(at, pr.K, ti * BM, tj * BN, kb, nslab);
            int per = (nslab + c.splits - 1) / c.splits;
            if (c.slab_align > 1) per = (per + c.slab_align - 1) / c.slab_align * c.slab_align;
            const int kt0 = min(nslab, split * per), kt1 = min(nslab, kt0 + per);
            cost[(size_t)t] = kt1 - kt0 + TN_TILE_OVERHEAD;
        }
    }
    return cost;
}

// Cost-balanced XCD ranges.  The logical tiles
// [0, first_tiles) are cut into eight contiguous ranges of (nearly) equal cost, one per XCD; the tiles
// [first_tiles, total_tiles), if any, are then dealt out so that the eight XCDs end up with equal total
// cost.  Every XCD works through its first range, then through its second: what the next launch waits
// for is spread over the whole chip and starts at once, the rest fills the chip behind it.  Returns the
// number of workgroups to launch.  (costs: tn_tile_costs of the launch, if the caller has them already)
template <class L>
inline int tn_balance_xcds(L &ll, int total_tiles, int first_tiles = -1, const std::vector<int> *costs = nullptr)
{
    TnCommon &c = ll.c;
    if (first_tiles < 0 || first_tiles > total_tiles) first_tiles = total_tiles;
    c.xcd_balanced = 0;
    if (total_tiles < 64) return total_tiles;
    std::vector<int> own;
    if (costs == nullptr) {
        own = tn_tile_costs(ll, total_tiles);
        costs = &own;
    }
    const std::vector<int> &cost = *costs;
    long long total1 = 0, total2 = 0;
    for (int t = 0; t < first_tiles; ++t) total1 += cost[(size_t)t];
    for (int t = first_tiles; t < total_tiles; ++t) total2 += cost[(size_t)t];
    // first list: equal cost per XCD
    long long run = 0, have[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int x = 0;
    c.xcd_begin[0] = 0;
    for (int t = 0; t < first_tiles; ++t) {
        while (x < 7 && run * 8 >= (long long)(x + 1) * total1) c.xcd_begin[++x] = t;
        run += cost[(size_t)t];
        have[x] += cost[(size_t)t];
    }
    while (x < 8) c.xcd_begin[++x] = first_tiles;
    // second list: each XCD is filled up to the common level
    const long long level = (total1 + total2 + 7) / 8;
    long long want[8], want_sum = 0;
    for (int i = 0; i < 8; ++i) {
        want[i] = level > have[i] ? level - have[i] : 0;
        want_sum += want[i];
    }
    x = 0;
    run = 0;
    long long upto = want[0];
    c.xcd_begin2[0] = first_tiles;
    for (int t = first_tiles; t < total_tiles; ++t) {
        while (x < 7 && run * want_sum >= upto * total2) {
            c.xcd_begin2[++x] = t;
            upto += want[x];
        }
        run += cost[(size_t)t];
    }
    while (x < 8) c.xcd_begin2[++x] = total_tiles;
    int longest = 0;
    for (int i = 0; i < 8; ++i)
        longest = max(longest, c.xcd_begin[i + 1] - c.xcd_begin[i] + c.xcd_begin2[i + 1] - c.xcd_begin2[i]);
    c.xcd_balanced = 1;
    return 8 * longest;
}

// Sets up the dealt mapping (xcd_balanced == 2, see tn_logical_tile_dealt) for a launch whose problems are
// already in the order they should run.  Returns the number of workgroups to launch.
template <class L>
inline int tn_deal_xcds(L &ll, int total_tiles)
{
    TnCommon &c = ll.c;
    c.xcd_balanced = 2;
    c.total_tiles = total_tiles;
    int longest = 0;
    for (int x = 0; x < 8; ++x) {
        int have = 0;
        for (int p = 0; p < c.count; ++p) {
            const int b = ll.tile_begin(p);
            const int n = (p + 1 < c.count ? ll.tile_begin(p + 1) : total_tiles) - b;
            const int part = (x + p) & 7;
            have += (int)((long long)n * (part + 1) / 8) - (int)((long long)n * part / 8);
        }
        longest = max(longest, have);
    }
    return 8 * longest;
}

// Length of a launch under the mapping that is set in ll.c, in slab times: every XCD starts its workgroups in
// order on 64 slots (32 CUs x 2), each slot taking the next tile when it is free.  This list-scheduling model
// reproduces the measured launches of the inversion and the precondition at 2.0 us per slab time; the host
// uses it to choose between the mappings.
template <class L>
inline long long tn_predict_launch(const L &ll, int total_tiles, const std::vector<int> &cost)
{
    const TnCommon &c = ll.c;
    constexpr int SLOTS = 64;
    long long worst = 0;
    std::vector<long long> heap;
    for (int x = 0; x < 8; ++x) {
        heap.assign(SLOTS, 0);  // a min-heap of the times at which the slots get free
        auto run = [&](int t) {
            std::pop_heap(heap.begin(), heap.end(), std::greater<long long>());
            heap.back() += cost[(size_t)t];
            std::push_heap(heap.begin(), heap.end(), std::greater<long long>());
        };
        if (c.xcd_balanced == 2) {
            for (int p = 0; p < c.count; ++p) {
                const int b = ll.tile_begin(p);
                const int n = (p + 1 < c.count ? ll.tile_begin(p + 1) : total_tiles) - b;
                const int part = (x + p) & 7;
                for (int t = b + (int)((long long)n * part / 8); t < b + (int)((long long)n * (part + 1) / 8); ++t) run(t);
            }
        } else if (c.xcd_balanced == 1) {
            for (int t = c.xcd_begin[x]; t < c.xcd_begin[x + 1]; ++t) run(t);
            for (int t = c.xcd_begin2[x]; t < c.xcd_begin2[x + 1]; ++t) run(t);
        } else {
            const int base = total_tiles >> 3, rem = total_tiles & 7;
            const int b = x * base + min(x, rem);
            for (int t = b; t < b + base + (x < rem ? 1 : 0); ++t) run(t);
        }
        for (long long v : heap) worst = max(worst, v);
    }
    return worst;
}

// Sets the mapping with the shorter predicted launch: cost-balanced ranges or dealt.  Returns the number of
// workgroups to launch.
template <class L>
inline int tn_map_xcds(L &ll, int total_tiles)
{
    if (total_tiles < 64) return tn_balance_xcds(ll, total_tiles);
    const std::vector<int> cost = tn_tile_costs(ll, total_tiles);
    const int grid_b = tn_balance_xcds(ll, total_tiles, -1, &cost);
    const long long len_b = tn_predict_launch(ll, total_tiles, cost);
    const TnCommon balanced = ll.c;
    const int grid_d = tn_deal_xcds(ll, total_tiles);
    if (tn_predict_launch(ll, total_tiles, cost) < len_b) return grid_d;
    ll.c = balanced;
    return grid_b;
}

// Unconditional load of four consecutive elements of operand row k starting at
// column c.  Out-of-range rows / columns are clamped to the last valid one, so
// the load never depends on a branch; tn_fix4 zeroes what must not count after
// the MFMA work of the current slab has been issued (the load latency is then
// hidden behind it).
template <bool FAST>
__device__ inline float4 tn_load4(const float *P, int k, int c, int ld, int K, int W)
{
    const int kc = min(k, K - 1);
    const float *row = P + (size_t)kc * (size_t)ld;
    if (FAST) return *reinterpret_cast<const float4 *>(row + c);
    float4 v;
    v.x = row[min(c + 0, W - 1)];
    v.y = row[min(c + 1, W - 1)];
    v.z = row[min(c + 2, W - 1)];
    v.w = row[min(c + 3, W - 1)];
    return v;
}

template <bool FAST>
__device__ inline float4 tn_fix4(float4 v, int k, int c, int K, int W)
{
    // branch-free on purpose: the K loop must stay one basic block
    const bool kz = k >= K;
    bool z0 = kz, z1 = kz, z2 = kz, z3 = kz;
    if (!FAST) {
        z0 |= (c + 0 >= W);
        z1 |= (c + 1 >= W);
        z2 |= (c + 2 >= W);
        z3 |= (c + 3 >= W);
    }
    v.x = z0 ? 0.f : v.x;
    v.y = z1 ? 0.f : v.y;
    v.z = z2 ? 0.f : v.z;
    v.w = z3 ? 0.f : v.w;
    return v;
}

// Which elements of a tile are stored directly / mirrored.  On a diagonal tile
// of a triangular launch only one triangle is stored and the other one is its
// mirror, which makes the result bitwise symmetric.
__device__ inline bool tn_keep(bool diag, int mode, int m, int n)
{
    return !diag || (mode == TILE_LOWER ? n <= m : n >= m);
}

constexpr int TN_STAGES = 3;      // LDS ring of the register-staged loop: slab s lives in stage s % 3
constexpr int TN_LDS_STAGES = 4;  // stages allocated (the direct-to-LDS loops use all of them; a fifth did not pay)

// sched_group_barrier masks
#define TN_SGB(m, n) __builtin_amdgcn_sched_group_barrier(m, n, 0)
constexpr int SG_MFMA = 0x008, SG_VMEM_READ = 0x020, SG_DS_READ = 0x100, SG_DS_WRITE = 0x200;

// K loop of one tile.  FAST: both operands can be read with aligned 16-byte
// loads over the whole tile width.
//
// Software pipeline (slab = BK rows of K; G = global load into staging
// registers, W = staging -> LDS, R = LDS -> MFMA operand registers, M = MFMA):
//   iteration s:  W(s+2)  G(s+3)  R(second half of s)  M(first half of s)
//                 R(first half of s+1)  M(second half of s)  barrier
// so every load is issued a full iteration (or half of one) before its use and
// sits in the shadow of the 32 MFMAs of the iteration.  Three LDS stages make
// one barrier per iteration enough: W(s+2) overwrites the stage of slab s-1,
// which every wave finished reading before the previous barrier.  Loads past
// the end of the K range are clamped to valid rows and their data is never
// used, which keeps the loop body free of branches.
template <bool FAST>
__device__ __forceinline__ void tn_mainloop(const TnAttr &lp, const TnProblem &pr, const TnTile &tl,
                                   float (&As)[TN_LDS_STAGES][BK][BM], float (&Bs)[TN_LDS_STAGES][BK][BN],
                                   floatx16 (&sum)[2][2])
{
    const int tid = threadIdx.x;
    const int M = pr.M, N = pr.N, K = pr.K;
    const float *__restrict__ A = pr.A;
    const float *__restrict__ B = pr.B;
    const int lda = pr.lda, ldb = pr.ldb;

    const int lrow = tid >> 5;         // 0..7 (and +8)
    const int lcol = (tid & 31) << 2;  // 0..124
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int li = lane & 31, lh = lane >> 5;
    const int ca = tl.m0 + lcol, cb = tl.n0 + lcol;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nslab = tl.kt1 - tl.kt0;
    if (nslab <= 0) return;

    float4 ra[2][2], rb[2][2];  // two sets of staging registers (slabs alternate)
    float2 fa[2][4], fb[2][4];  // MFMA operands: [half of the slab][k step pair]
    int kw = tl.kbase + tl.kt0 * BK + lrow;  // K row (of this thread) of the next slab to go to LDS

#define TN_G(set, ahead)                                                        \
    do {                                                                        \
        const int kg_ = kw + (ahead) * BK;                                      \
        ra[set][0] = tn_load4<FAST>(A, kg_, ca, lda, K, M);                     \
        ra[set][1] = tn_load4<FAST>(A, kg_ + 8, ca, lda, K, M);                 \
        rb[set][0] = tn_load4<FAST>(B, kg_, cb, ldb, K, N);                     \
        rb[set][1] = tn_load4<FAST>(B, kg_ + 8, cb, ldb, K, N);                 \
    } while (0)
#define TN_W(st, set)                                                                                                  \
    do {                                                                                                               \
        *reinterpret_cast<float4 *>(&As[st][lrow][lcol]) = tn_fix4<FAST>(ra[set][0], kw, ca, K, M);     \
        *reinterpret_cast<float4 *>(&As[st][lrow + 8][lcol]) = tn_fix4<FAST>(ra[set][1], kw + 8, ca, K, M); \
        *reinterpret_cast<float4 *>(&Bs[st][lrow][lcol]) = tn_fix4<FAST>(rb[set][0], kw, cb, K, N);     \
        *reinterpret_cast<float4 *>(&Bs[st][lrow + 8][lcol]) = tn_fix4<FAST>(rb[set][1], kw + 8, cb, K, N); \
        kw += BK;                                                                                                      \
    } while (0)
    // lane (li, lh) feeds rows 2*li, 2*li+1 of the wave tile at k = 2*step + lh
#define TN_R(st, half)                                                                                            \
    do {                                                                                                          \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                           \
            fa[half][q] = *reinterpret_cast<const float2 *>(&As[st][8 * (half) + 2 * q + lh][wm + 2 * li]);       \
            fb[half][q] = *reinterpret_cast<const float2 *>(&Bs[st][8 * (half) + 2 * q + lh][wn + 2 * li]);       \
        }                                                                                                         \
    } while (0)
#define TN_M(half)                                                                                                \
    do {                                                                                                          \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                           \
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[half][q].x, fb[half][q].x, acc[0][0], 0, 0, 0);   \
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[half][q].x, fb[half][q].y, acc[0][1], 0, 0, 0);   \
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[half][q].y, fb[half][q].x, acc[1][0], 0, 0, 0);   \
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[half][q].y, fb[half][q].y, acc[1][1], 0, 0, 0);   \
        }                                                                                                         \
    } while (0)
    // One iteration: slab s is consumed; slab s+2 (loaded two iterations ago into `set`)
    // goes to LDS and slab s+4 is requested into the same registers.  The LDS writes,
    // global loads and operand reads are spread one by one between the MFMAs.
#define TN_ITER(set)                                                                 \
    do {                                                                             \
        TN_W(st2, set);                                                              \
        TN_G(set, 1);                                                                \
        TN_R(st0, 1);                                                                \
        TN_M(0);                                                                     \
        TN_R(st1, 0);                                                                \
        TN_M(1);                                                                     \
        _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                           \
            TN_SGB(SG_MFMA, 1);                     \
            TN_SGB(SG_DS_READ, 1);                  \
        }                                                                            \
        _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                           \
            TN_SGB(SG_MFMA, 1);                     \
            TN_SGB(SG_DS_WRITE, 1);                 \
        }                                                                            \
        _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                           \
            TN_SGB(SG_MFMA, 1);                     \
            TN_SGB(SG_VMEM_READ, FAST ? 1 : 4);     \
        }                                                                            \
        TN_SGB(SG_MFMA, 4);                         \
        _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                           \
            TN_SGB(SG_MFMA, 1);                     \
            TN_SGB(SG_DS_READ, 1);                  \
        }                                                                            \
        TN_SGB(SG_MFMA, 12);                        \
        __syncthreads();                                                             \
        const int t_ = st0;                                                          \
        st0 = st1;                                                                   \
        st1 = st2;                                                                   \
        st2 = t_;                                                                    \
    } while (0)

    // prologue: slabs 0 and 1 in LDS, slabs 2 and 3 in flight, first half of slab 0 in registers
    TN_G(0, 0);
    TN_G(1, 1);
    TN_W(0, 0);
    TN_W(1, 1);
    TN_G(0, 0);
    TN_G(1, 1);
    __syncthreads();
    TN_R(0, 0);

    int st0 = 0, st1 = 1, st2 = 2;  // stages of slabs s, s+1, s+2
    int folded = 0;
    int s = 0;
    for (; s + 1 < nslab; s += 2) {
        TN_ITER(0);
        TN_ITER(1);
        folded += 2;
        if (folded == TN_CHUNK_SLABS) {
            folded = 0;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    sum[i][j] += acc[i][j];
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
                }
        }
    }
    if (s < nslab) TN_ITER(0);
#undef TN_ITER
#undef TN_G
#undef TN_W
#undef TN_R
#undef TN_M
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) sum[i][j] += acc[i][j];
}

// Values that are the same in every lane, moved to scalar registers.  The direct-to-LDS loads below take
// their base address from scalar registers; where the compiler cannot prove that a problem descriptor
// is wave-uniform (it is: it only depends on the workgroup index) this makes it so.
__device__ inline int tn_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline const float *tn_uniform(const float *p)
{
    const unsigned long long v = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return reinterpret_cast<const float *>(((unsigned long long)hi << 32) | lo);
}

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at
// lds_addr + 16 * l (lds_addr, a byte address in LDS, is the same for the whole wave).  The global
// address is a wave-uniform base (scalar registers) plus a 32-bit per-lane byte offset: a K loop
// advances the base with scalar arithmetic and needs no vector instruction per load.
__device__ inline void tn_dma16_s(const float *sbase, unsigned voff, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory", "m0");
}

// K loop for the common case (fp32 operands, aligned full-width tiles, K range
// a multiple of BK): slabs go from global memory straight into
// LDS (global_load_lds_dwordx4: lane l's 16 bytes land at base + 16*l, so one
// wave instruction fills two 512-byte rows), without staging registers, LDS
// stores or fix-up arithmetic.  Four LDS stages:
//   iteration s:  R(second half of s)  M(first half of s) with the four loads D(s+3) between
//                 its MFMAs  R(first half of s+1)  M(second half of s) with "wait D(s+2),
//                 barrier" in its middle
// D(s+3) overwrites the stage of slab s-1, which every wave finished reading
// before the previous barrier.
//
// A wave issues in order and an MFMA 32x32x2 keeps the matrix core busy for 64 cycles, so
// whatever is not an MFMA must be little and sit between MFMAs.  The loop is unrolled over
// the four stages (LDS addresses become immediates), the loads take a scalar base that is
// advanced with scalar arithmetic, and scheduling barriers pin the order written here.
// IDLE: the wave takes part in the loads and barriers of the tile but computes nothing (its quarter of a
// diagonal tile of a triangular launch lies on the side that is only stored as a mirror).
template <bool IDLE>
__device__ __forceinline__ void tn_mainloop_direct(const TnProblem &pr, const TnTile &tl,
                                          float (&As)[TN_LDS_STAGES][BK][BM], float (&Bs)[TN_LDS_STAGES][BK][BN],
                                          floatx16 (&sum)[2][2])
{
    static_assert(TN_LDS_STAGES == 4, "the loop below is unrolled over four stages");
    const int tid = threadIdx.x;
    const int K = tn_uniform(pr.K);
    const float *__restrict__ A = tn_uniform(pr.A);
    const float *__restrict__ B = tn_uniform(pr.B);
    const size_t lda = (size_t)tn_uniform(pr.lda), ldb = (size_t)tn_uniform(pr.ldb);
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int li = lane & 31, lh = lane >> 5;
    const int drow = 2 * wave + lh;  // row of the slab this lane fetches (and drow + 8)

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nslab = tn_uniform(tl.kt1 - tl.kt0);
    if (nslab <= 0) return;
    float2 fa[2][4], fb[2][4];
    int kd = tn_uniform(tl.kbase + tl.kt0 * BK);  // first K row of the next slab to request (wave-uniform)

    // per-lane byte offsets of the four loads of a slab, relative to the slab's first row
    const unsigned va0 = (unsigned)(((size_t)drow * lda + tl.m0 + 4 * li) * sizeof(float));
    const unsigned va1 = va0 + (unsigned)(8 * lda * sizeof(float));
    const unsigned vb0 = (unsigned)(((size_t)drow * ldb + tl.n0 + 4 * li) * sizeof(float));
    const unsigned vb1 = vb0 + (unsigned)(8 * ldb * sizeof(float));
    // LDS byte addresses of this wave's rows in stage 0
    const unsigned la0 = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(const __attribute__((address_space(3))) float *)&As[0][2 * wave][0]);
    const unsigned lb0 = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(const __attribute__((address_space(3))) float *)&Bs[0][2 * wave][0]);
    constexpr unsigned STAGE = BK * BM * sizeof(float), HALF = 8 * BM * sizeof(float);

    // Slabs past the end of the K range are clamped to the last one: that data is never consumed.
    // The load is inline assembly on purpose: issued through the builtin, the compiler drains
    // vmcnt before every later LDS read (it cannot tell the ring stages apart), which would undo
    // the pipeline.  The waits are placed by hand instead (TN_WAIT_ALL_BUT_NEWEST_SLAB).
    const float *sa = A, *sb = B;  // bases of the slab being requested
#define TN_DBASE()                                            \
    do {                                                      \
        const size_t kc_ = (size_t)min(kd, K - BK);           \
        sa = A + kc_ * lda;                                   \
        sb = B + kc_ * ldb;                                   \
        kd += BK;                                             \
    } while (0)
#define TN_D1(st, w)                                                                               \
    do {                                                                                           \
        if ((w) == 0) tn_dma16_s(sa, va0, la0 + (st) * STAGE);                                     \
        if ((w) == 1) tn_dma16_s(sa, va1, la0 + (st) * STAGE + HALF);                              \
        if ((w) == 2) tn_dma16_s(sb, vb0, lb0 + (st) * STAGE);                                     \
        if ((w) == 3) tn_dma16_s(sb, vb1, lb0 + (st) * STAGE + HALF);                              \
    } while (0)
#define TN_R(st, half)                                                                                            \
    do {                                                                                                          \
        if (!IDLE) _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                \
            fa[half][q] = *reinterpret_cast<const float2 *>(&As[st][8 * (half) + 2 * q + lh][wm + 2 * li]);       \
            fb[half][q] = *reinterpret_cast<const float2 *>(&Bs[st][8 * (half) + 2 * q + lh][wn + 2 * li]);       \
        }                                                                                                         \
    } while (0)
#define TN_MQ(half, q)                                                                                        \
    do {                                                                                                      \
        if (!IDLE) {                                                                                          \
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[half][q].x, fb[half][q].x, acc[0][0], 0, 0, 0);   \
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[half][q].x, fb[half][q].y, acc[0][1], 0, 0, 0);   \
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[half][q].y, fb[half][q].x, acc[1][0], 0, 0, 0);   \
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[half][q].y, fb[half][q].y, acc[1][1], 0, 0, 0);   \
        }                                                                                                     \
    } while (0)
#define TN_PIN() __builtin_amdgcn_sched_barrier(0)
    // s_waitcnt vmcnt(4): everything but the four newest loads has landed (gfx9 encoding:
    // vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8; the other counters are left open)
#define TN_WAIT_ALL_BUT_NEWEST_SLAB() __builtin_amdgcn_s_waitcnt(0x0F74)
    // one slab: consumes the slab in stage st0, reads ahead into st1, requests into st3
#define TN_ITER(st0, st1, st3)                                                                     \
    do {                                                                                           \
        TN_R(st0, 1);                                                                              \
        TN_DBASE();                                                                                \
        TN_PIN();                                                                                  \
        TN_MQ(0, 0);                                                                               \
        TN_PIN();                                                                                  \
        TN_D1(st3, 0);                                                                             \
        TN_PIN();                                                                                  \
        TN_MQ(0, 1);                                                                               \
        TN_PIN();                                                                                  \
        TN_D1(st3, 1);                                                                             \
        TN_PIN();                                                                                  \
        TN_MQ(0, 2);                                                                               \
        TN_PIN();                                                                                  \
        TN_D1(st3, 2);                                                                             \
        TN_PIN();                                                                                  \
        TN_MQ(0, 3);                                                                               \
        TN_PIN();                                                                                  \
        TN_D1(st3, 3);                                                                             \
        TN_PIN();                                                                                  \
        TN_R(st1, 0);                                                                              \
        TN_PIN();                                                                                  \
        TN_MQ(1, 0);                                                                               \
        TN_MQ(1, 1);                                                                               \
        TN_PIN();                                                                                  \
        TN_WAIT_ALL_BUT_NEWEST_SLAB();                                                             \
        __syncthreads();                                                                           \
        TN_PIN();                                                                                  \
        TN_MQ(1, 2);                                                                               \
        TN_MQ(1, 3);                                                                               \
        TN_PIN();                                                                                  \
        if (++folded == TN_CHUNK_SLABS) {                                                          \
            folded = 0;                                                                            \
            _Pragma("unroll") for (int i = 0; i < 2; ++i)                                          \
                _Pragma("unroll") for (int j = 0; j < 2; ++j) {                                    \
                    sum[i][j] += acc[i][j];                                                        \
                    _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;             \
                }                                                                                  \
        }                                                                                          \
    } while (0)

    // prologue: request slabs 0 .. 2, wait for the first two
#pragma unroll
    for (int q = 0; q < TN_LDS_STAGES - 1; ++q) {
        TN_DBASE();
        TN_D1(q, 0);
        TN_D1(q, 1);
        TN_D1(q, 2);
        TN_D1(q, 3);
    }
    TN_WAIT_ALL_BUT_NEWEST_SLAB();
    __syncthreads();
    TN_R(0, 0);

    int folded = 0;
    int s = 0;
    for (; s + 4 <= nslab; s += 4) {
        TN_ITER(0, 1, 3);
        TN_ITER(1, 2, 0);
        TN_ITER(2, 3, 1);
        TN_ITER(3, 0, 2);
    }
    const int rest = nslab - s;  // s is a multiple of four here: the stages continue at 0
    if (rest > 0) TN_ITER(0, 1, 3);
    if (rest > 1) TN_ITER(1, 2, 0);
    if (rest > 2) TN_ITER(2, 3, 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no load may still be writing LDS when the tile ends
#undef TN_DBASE
#undef TN_D1
#undef TN_R
#undef TN_MQ
#undef TN_PIN
#undef TN_ITER
#undef TN_WAIT_ALL_BUT_NEWEST_SLAB
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) sum[i][j] += acc[i][j];
}

// ---------------------------------------------------------------------------
// bfloat16 operands on the bf16 MFMA (v_mfma_f32_32x32x16_bf16).
//
// That instruction wants, per lane, eight consecutive K values of one column
// (lane (i, h) holds k = 8h .. 8h+7 of column i).  The activations are stored
// [tokens, d], so those eight values are d elements apart.  A small pre-pass
// (pack_bf16_kernel) rewrites x as P[k / 8][column][k % 8], zero-padded to a
// multiple of 32 tokens and 256 columns: the eight values are then 16 contiguous
// bytes, a wave fetches 64 columns of a k-group with one global_load_lds_dwordx4
// and reads its MFMA operands from LDS with ds_read_b128, all conflict-free and
// without a transpose.  Slab = 32 tokens = 4 k-groups = 8 KB per operand, the
// same LDS footprint as the fp32 loop.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int BF_KG = 8;           // K values per packed group
constexpr int BF_SLAB_GROUPS = 4;  // groups per slab (32 tokens)

struct PackItem {
    const unsigned short *x;  // [n, d] bfloat16, ldx
    unsigned short *dst;      // [gp][dp][8]
    int n, d, ldx, dp, gp, pad_;
};
constexpr int PACK_MAX_ITEMS = 80;
struct PackLaunch {
    PackItem it[PACK_MAX_ITEMS];
};

// One workgroup repacks 32 tokens x 512 columns through LDS, so that both sides move
// 16 bytes per lane in 1 KB runs per wave: row-major reads (eight columns of a token),
// packed writes (eight tokens of a column).
constexpr int PACK_COLS = 512;
constexpr int PACK_ROWS = BF_KG * BF_SLAB_GROUPS;  // 32 tokens
constexpr int PACK_LDS_ROW = PACK_COLS * 2 + 16;   // bytes per token row in LDS

__global__ __launch_bounds__(256) void pack_bf16_kernel(const PackLaunch pl)
{
    __shared__ __attribute__((aligned(16))) unsigned char tile[PACK_ROWS * PACK_LDS_ROW];
    const PackItem &it = pl.it[blockIdx.z];
    const int c0 = blockIdx.x * PACK_COLS, g0 = blockIdx.y * BF_SLAB_GROUPS;
    if (c0 >= it.dp || g0 >= it.gp) return;  // whole workgroup leaves together (gp is a multiple of 4)
    const int t = threadIdx.x;
    const int cu = t & 63, col = c0 + 8 * cu;
    const bool vec = ((it.ldx & 7) == 0) && ((reinterpret_cast<uintptr_t>(it.x) & 15) == 0);
#pragma unroll
    for (int r = 0; r < PACK_ROWS / 4; ++r) {
        const int row = (t >> 6) + 4 * r;
        const int k = g0 * BF_KG + row;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (k < it.n && col < it.d) {
            const unsigned short *src = it.x + (size_t)k * it.ldx + col;
            if (vec && col + 8 <= it.d) {
                v = *reinterpret_cast<const uint4 *>(src);
            } else {
                unsigned h[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) h[e] = (col + e < it.d) ? src[e] : 0u;
                v = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
            }
        }
        *reinterpret_cast<uint4 *>(tile + row * PACK_LDS_ROW + cu * 16) = v;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 2 * BF_SLAB_GROUPS; ++r) {
        const int gi = r >> 1, c = t + 256 * (r & 1);
        if (c0 + c >= it.dp) continue;
        unsigned h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            h[e] = *reinterpret_cast<const unsigned short *>(tile + (BF_KG * gi + e) * PACK_LDS_ROW + 2 * c);
        *reinterpret_cast<uint4 *>(it.dst + ((size_t)(g0 + gi) * it.dp + c0 + c) * 8) =
            make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
}

// K loop on packed bf16 operands.  pr.A = pr.B = packed array, pr.lda = padded
// column count, pr.K = padded token count.  Same pipeline as the direct fp32
// loop with the operand registers double-buffered per slab (a single fp32
// accumulation level: the tolerance of the bfloat16 variant does not need two):
//   iteration s:  M(s) with R(s+1) and D(s+3) between its two k steps  wait D(s+2)  barrier
__device__ inline void tn_mainloop_bf16_packed(const TnProblem &pr, const TnTile &tl,
                                               float (&As)[TN_LDS_STAGES][BK][BM], float (&Bs)[TN_LDS_STAGES][BK][BN],
                                               floatx16 (&sum)[2][2])
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int li = lane & 31, lh = lane >> 5;
    const size_t row_bytes = (size_t)pr.lda * 16;  // one k-group of all columns
    const int groups = pr.K / BF_KG;
    const char *la = reinterpret_cast<const char *>(&As[0][0][0]);
    const char *lb = reinterpret_cast<const char *>(&Bs[0][0][0]);
    constexpr int STAGE_BYTES = BK * BM * 4;  // 8 KB

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int niter = (tl.kt1 - tl.kt0) / 2;  // slabs of 32 tokens (K ranges are multiples of 32)
    if (niter <= 0) return;
    int gd = (tl.kbase + tl.kt0 * BK) / BF_KG;  // first k-group of the next slab to request
    uint4 fa[2][2][2], fb[2][2][2];              // [register set][k step][block]

    // Wave w fetches k-group gd + w: columns 0..63 and 64..127 of the tile, for both operands.  The
    // address is a scalar base (the k-group row) plus a loop-invariant per-lane offset: no vector
    // arithmetic in the loop (see tn_mainloop_direct).
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const char *xa = reinterpret_cast<const char *>(pr.A), *xb = reinterpret_cast<const char *>(pr.B);
    const unsigned va = (unsigned)(((size_t)tl.m0 + lane) * 16), vb = (unsigned)(((size_t)tl.n0 + lane) * 16);
    const unsigned la0 = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(const __attribute__((address_space(3))) char *)la) + wave_s * 2048;
    const unsigned lb0 = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(const __attribute__((address_space(3))) char *)lb) + wave_s * 2048;
    size_t soff = 0;  // byte offset of the k-group row being requested (wave-uniform)
#define BF_DBASE()                                                                                          \
    do {                                                                                                    \
        soff = (size_t)min(gd + wave_s, groups - 1) * row_bytes;                                            \
        gd += BF_SLAB_GROUPS;                                                                               \
    } while (0)
#define BF_D1(st, w)                                                                                                              \
    do {                                                                                                                          \
        if ((w) == 0) tn_dma16_s(reinterpret_cast<const float *>(xa + soff), va, la0 + (st) * STAGE_BYTES);                       \
        if ((w) == 1) tn_dma16_s(reinterpret_cast<const float *>(xa + soff + 1024), va, la0 + (st) * STAGE_BYTES + 1024);         \
        if ((w) == 2) tn_dma16_s(reinterpret_cast<const float *>(xb + soff), vb, lb0 + (st) * STAGE_BYTES);                       \
        if ((w) == 3) tn_dma16_s(reinterpret_cast<const float *>(xb + soff + 1024), vb, lb0 + (st) * STAGE_BYTES + 1024);         \
    } while (0)
    // lane (li, lh) feeds columns 2*li, 2*li+1 of the wave tile with k-group 2t + lh
#define BF_RT(st, set, t)                                                                                   \
    do {                                                                                                    \
        const int u_ = (st) * STAGE_BYTES + ((2 * (t) + lh) * 128 + 2 * li) * 16;                           \
        fa[set][t][0] = *reinterpret_cast<const uint4 *>(la + u_ + wm * 16);                                \
        fa[set][t][1] = *reinterpret_cast<const uint4 *>(la + u_ + wm * 16 + 16);                           \
        fb[set][t][0] = *reinterpret_cast<const uint4 *>(lb + u_ + wn * 16);                                \
        fb[set][t][1] = *reinterpret_cast<const uint4 *>(lb + u_ + wn * 16 + 16);                           \
    } while (0)
#define BF_R(st, set)                                                                                       \
    do {                                                                                                    \
        BF_RT(st, set, 0);                                                                                  \
        BF_RT(st, set, 1);                                                                                  \
    } while (0)
#define BF_MT(set, t)                                                                                       \
    do {                                                                                                    \
        _Pragma("unroll") for (int bi = 0; bi < 2; ++bi)                                                    \
            _Pragma("unroll") for (int bj = 0; bj < 2; ++bj)                                                \
                acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                      \
                    __builtin_bit_cast(bf16x8, fa[set][t][bi]), __builtin_bit_cast(bf16x8, fb[set][t][bj]), \
                    acc[bi][bj], 0, 0, 0);                                                                  \
    } while (0)
#define BF_PIN() __builtin_amdgcn_sched_barrier(0)
    // slab in stage st (register set cur); reads slab st+1 into set nxt, requests into stage st+3
#define BF_ITER(st, cur, nxt)                                                                               \
    do {                                                                                                    \
        BF_DBASE();                                                                                         \
        BF_PIN();                                                                                           \
        BF_MT(cur, 0);                                                                                      \
        BF_PIN();                                                                                           \
        BF_RT(((st) + 1) & 3, nxt, 0);                                                                      \
        BF_D1(((st) + 3) & 3, 0);                                                                           \
        BF_D1(((st) + 3) & 3, 1);                                                                           \
        BF_PIN();                                                                                           \
        BF_MT(cur, 1);                                                                                      \
        BF_PIN();                                                                                           \
        BF_RT(((st) + 1) & 3, nxt, 1);                                                                      \
        BF_D1(((st) + 3) & 3, 2);                                                                           \
        BF_D1(((st) + 3) & 3, 3);                                                                           \
        BF_PIN();                                                                                           \
        __builtin_amdgcn_s_waitcnt(0x0F74); /* vmcnt(4): all but the newest slab has landed */              \
        __syncthreads();                                                                                    \
        BF_PIN();                                                                                           \
    } while (0)

#pragma unroll
    for (int q = 0; q < 3; ++q) {
        BF_DBASE();
        BF_D1(q, 0);
        BF_D1(q, 1);
        BF_D1(q, 2);
        BF_D1(q, 3);
    }
    __builtin_amdgcn_s_waitcnt(0x0F74);
    __syncthreads();
    BF_R(0, 0);
    int s = 0;
    for (; s + 4 <= niter; s += 4) {
        BF_ITER(0, 0, 1);
        BF_ITER(1, 1, 0);
        BF_ITER(2, 0, 1);
        BF_ITER(3, 1, 0);
    }
    const int rest = niter - s;  // s is a multiple of four: stages and register sets continue at 0
    if (rest > 0) BF_ITER(0, 0, 1);
    if (rest > 1) BF_ITER(1, 1, 0);
    if (rest > 2) BF_ITER(2, 0, 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
#undef BF_DBASE
#undef BF_D1
#undef BF_RT
#undef BF_MT
#undef BF_PIN
#undef BF_R
#undef BF_ITER
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) sum[i][j] += acc[i][j];
}

// One output tile (already located: problem pr with attributes at, tile tl, logical index `logical`).
template <class L>
__device__ __forceinline__ void tn_tile_work(const L &ll, const TnProblem &pr, const TnAttr &at, const TnTile &tl, int logical,
                                    float (&As)[TN_LDS_STAGES][BK][BM], float (&Bs)[TN_LDS_STAGES][BK][BN])
{
    const TnCommon &lp = ll.c;
    const int tid = threadIdx.x;
    const int M = pr.M, N = pr.N;

    // vector loads need 16-byte aligned rows
    const bool fast_a = (tl.m0 + BM <= M) && ((pr.lda & 3) == 0) && ((reinterpret_cast<uintptr_t>(pr.A) & 15) == 0);
    const bool fast_b = (tl.n0 + BN <= N) && ((pr.ldb & 3) == 0) && ((reinterpret_cast<uintptr_t>(pr.B) & 15) == 0);

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int li = lane & 31, lh = lane >> 5;

    floatx16 sum[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) sum[i][j][r] = 0.f;

    bool done = false;
    if constexpr (L::kPackedBf16) {
        tn_mainloop_bf16_packed(pr, tl, As, Bs, sum);
        done = true;
    }
    // (the direct loop addresses a slab with 32-bit byte offsets from its first row)
    const bool direct_ok = (pr.K % BK) == 0 && pr.lda < (1 << 25) && pr.ldb < (1 << 25);
    // diagonal tile of a triangular launch: the wave whose 64 x 64 quarter lies wholly on the mirrored side
    // has nothing to compute (none of it is stored); in the direct loop it only helps to move the slabs,
    // which leaves its share of the matrix core to the co-resident workgroup and saves power
    const bool idle_wave = tl.diag && ((at.tile_mode == TILE_LOWER && wn > wm) || (at.tile_mode == TILE_UPPER && wm > wn));
    if (!done && fast_a && fast_b && direct_ok) {
        if (idle_wave)
            tn_mainloop_direct<true>(pr, tl, As, Bs, sum);
        else
            tn_mainloop_direct<false>(pr, tl, As, Bs, sum);
        done = true;
    }
    if (!done) {
        if (fast_a && fast_b)
            tn_mainloop<true>(at, pr, tl, As, Bs, sum);
        else
            tn_mainloop<false>(at, pr, tl, As, Bs, sum);
    }

    // Accumulator layout of MFMA 32x32: register r of lane (li, lh) is row
    // 8*(r/4) + 4*lh + r%4, column li of the block; block (bi, bj) interleaves
    // rows/columns with stride 2 (see the operand feed above).
    if (lp.splits > 1) {
        float *P = lp.partial + (size_t)logical * (BM * BN);
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lm = wm + 2 * (8 * (r >> 2) + 4 * lh + (r & 3)) + bi;
                const int ln = wn + 2 * li;
                *reinterpret_cast<float2 *>(&P[lm * BN + ln]) = make_float2(sum[bi][0][r], sum[bi][1][r]);
            }
        return;
    }

    if (pr.guard != nullptr && *pr.guard != 0) return;

    float *__restrict__ C = pr.C;
    float *__restrict__ Ct = pr.Ct;
    const int ldc = pr.ldc, ldct = pr.ldct;
    const float alpha = at.alpha, beta = at.beta;
    const bool interior = (tl.m0 + BM <= M) && (tl.n0 + BN <= N) && !tl.diag;
    const bool fast_c = interior && ((ldc & 1) == 0) && ((reinterpret_cast<uintptr_t>(C) & 7) == 0);

    if (fast_c) {
        // element (bi, bj, r) of this lane: row 2 (8 (r / 4) + 4 lh + r % 4) + bi, columns 2 li + bj of the quarter
        float2 *row0 = reinterpret_cast<float2 *>(C + (size_t)(tl.m0 + wm + 8 * lh) * ldc + (tl.n0 + wn + 2 * li));
        auto at_row = [&](int bi, int r) { return row0 + (size_t)(2 * (8 * (r >> 2) + (r & 3)) + bi) * (size_t)(ldc >> 1); };
        if (beta != 0.f) {
            // All of the tile's old values are requested before the first one is used: one memory latency for
            // the tile, not one per row (the compiler cannot move a load over the stores of the rows before it).
            float2 old[2][16];
#pragma unroll
            for (int bi = 0; bi < 2; ++bi)
#pragma unroll
                for (int r = 0; r < 16; ++r) old[bi][r] = *at_row(bi, r);
#pragma unroll
            for (int bi = 0; bi < 2; ++bi)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float2 v = make_float2(alpha * sum[bi][0][r], alpha * sum[bi][1][r]);
                    v.x += beta * old[bi][r].x;
                    v.y += beta * old[bi][r].y;
                    sum[bi][0][r] = v.x;
                    sum[bi][1][r] = v.y;
                }
        } else {
#pragma unroll
            for (int bi = 0; bi < 2; ++bi)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    sum[bi][0][r] *= alpha;
                    sum[bi][1][r] *= alpha;
                }
        }
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) *at_row(bi, r) = make_float2(sum[bi][0][r], sum[bi][1][r]);
    } else {
        // edge and diagonal tiles, element by element; as above, every old value is requested before the first is used
        float old[2][2][16];
        if (beta != 0.f) {
#pragma unroll
            for (int bi = 0; bi < 2; ++bi)
#pragma unroll
                for (int bj = 0; bj < 2; ++bj)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = tl.m0 + wm + 2 * (8 * (r >> 2) + 4 * lh + (r & 3)) + bi;
                        const int n = tl.n0 + wn + 2 * li + bj;
                        const bool mine = m < M && n < N && tn_keep(tl.diag, at.tile_mode, m, n);
                        old[bi][bj][r] = mine ? C[(size_t)m * ldc + n] : 0.f;
                    }
        }
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int bj = 0; bj < 2; ++bj)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = tl.m0 + wm + 2 * (8 * (r >> 2) + 4 * lh + (r & 3)) + bi;
                    const int n = tl.n0 + wn + 2 * li + bj;
                    float v = alpha * sum[bi][bj][r];
                    if (m < M && n < N && tn_keep(tl.diag, at.tile_mode, m, n)) {
                        if (beta != 0.f) v += beta * old[bi][bj][r];
                        C[(size_t)m * ldc + n] = v;
                    }
                    sum[bi][bj][r] = v;
                }
    }

    if (Ct != nullptr) {
        const bool fast_t = interior && ((ldct & 3) == 0) && ((reinterpret_cast<uintptr_t>(Ct) & 15) == 0);
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // eight consecutive rows m of C held by this lane for column n
                const int n = tl.n0 + wn + 2 * li + bj;
                const int mq = tl.m0 + wm + 16 * q + 8 * lh;
                if (fast_t) {
                    float4 *dst = reinterpret_cast<float4 *>(Ct + (size_t)n * ldct + mq);
                    dst[0] = make_float4(sum[0][bj][4 * q + 0], sum[1][bj][4 * q + 0], sum[0][bj][4 * q + 1], sum[1][bj][4 * q + 1]);
                    dst[1] = make_float4(sum[0][bj][4 * q + 2], sum[1][bj][4 * q + 2], sum[0][bj][4 * q + 3], sum[1][bj][4 * q + 3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int m = mq + e;
                        const bool strict = !tl.diag || (m != n && tn_keep(true, at.tile_mode, m, n));
                        if (m < M && n < N && strict) Ct[(size_t)n * ldct + m] = sum[e & 1][bj][4 * q + (e >> 1)];
                    }
                }
            }
    }
}

template <class L>
__device__ __forceinline__ void tn_tile_body(const L &ll, float (&As)[TN_LDS_STAGES][BK][BM], float (&Bs)[TN_LDS_STAGES][BK][BN])
{
    const int logical = ll.c.xcd_balanced == 2 ? tn_logical_tile_dealt(ll, blockIdx.x) : tn_logical_tile(blockIdx.x, gridDim.x, ll.c);
    if (logical < 0) return;  // surplus workgroup of a short XCD range (the whole workgroup leaves)
    TnProblem pr;
    TnAttr at;
    const TnTile tl = tn_locate(ll, logical, pr, at);
    tn_tile_work(ll, pr, at, tl, logical, As, Bs);
}

// Second pass of a split-K launch: adds the partial tiles of each output tile in
// split order (fixed order: the result does not depend on scheduling) and
// applies the same epilogue as the main kernel.  One workgroup per output tile.
template <class L>
__device__ inline void tn_reduce_body(const L &ll)
{
    const TnCommon &lp = ll.c;
    const int t0 = blockIdx.x * lp.splits;  // logical index of split 0 of this output tile
    TnProblem pr;
    TnAttr at;
    const TnTile tl = tn_locate(ll, t0, pr, at);
    if (pr.guard != nullptr && *pr.guard != 0) return;
    const float *P = lp.partial + (size_t)t0 * (BM * BN);
    const int tid = threadIdx.x;
    const int M = pr.M, N = pr.N;
    for (int it = 0; it < BM / 8; ++it) {
        const int lm = (tid >> 5) + 8 * it;
        const int ln = (tid & 31) << 2;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int sp = 0; sp < lp.splits; ++sp) {
            const float4 v = *reinterpret_cast<const float4 *>(&P[(size_t)sp * (BM * BN) + lm * BN + ln]);
            s.x += v.x;
            s.y += v.y;
            s.z += v.z;
            s.w += v.w;
        }
        const float vals[4] = {s.x, s.y, s.z, s.w};
        const int m = tl.m0 + lm;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int n = tl.n0 + ln + e;
            if (m < M && n < N && tn_keep(tl.diag, at.tile_mode, m, n)) {
                float v = at.alpha * vals[e];
                float *dst = pr.C + (size_t)m * pr.ldc + n;
                if (at.beta != 0.f) v += at.beta * (*dst);
                *dst = v;
                if (pr.Ct != nullptr && (!tl.diag || m != n)) pr.Ct[(size_t)n * pr.ldct + m] = v;
            }
        }
    }
}

__global__ __launch_bounds__(TN_THREADS, 2) void tn_gemm_kernel(const TnLaunch lp)
{
    __shared__ float As[TN_LDS_STAGES][BK][BM];
    __shared__ float Bs[TN_LDS_STAGES][BK][BN];
    tn_tile_body(lp, As, Bs);
}

__global__ __launch_bounds__(TN_THREADS) void tn_reduce_kernel(const TnLaunch lp) { tn_reduce_body(lp); }

// The curvature work item: the same tile body under its own name, so that its
// launches can be told apart in a kernel trace.
__global__ __launch_bounds__(TN_THREADS, 2) void curvature_syrk_kernel(const SyrkLaunch lp)
{
    __shared__ float As[TN_LDS_STAGES][BK][BM];
    __shared__ float Bs[TN_LDS_STAGES][BK][BN];
    tn_tile_body(lp, As, Bs);
}

__global__ __launch_bounds__(TN_THREADS) void curvature_reduce_kernel(const SyrkLaunch lp) { tn_reduce_body(lp); }

// bfloat16 inputs repacked by pack_bf16_kernel, multiplied by the bf16 MFMA, accumulated in fp32.
__global__ __launch_bounds__(TN_THREADS, 2) void curvature_syrk_bf16mfma_kernel(const SyrkLaunchPacked lp)
{
    __shared__ float As[TN_LDS_STAGES][BK][BM];
    __shared__ float Bs[TN_LDS_STAGES][BK][BN];
    tn_tile_body(lp, As, Bs);
}

__global__ __launch_bounds__(TN_THREADS) void curvature_reduce_packed_kernel(const SyrkLaunchPacked lp) { tn_reduce_body(lp); }

static_assert(sizeof(InvLaunch) <= 4096 && sizeof(TnLaunch) <= 4096 && sizeof(SyrkLaunch) <= 4096 && sizeof(WwtLaunch) <= 4096,
              "launch descriptors travel in the kernel arguments (4 KB)");

// inv = W W^T of a whole batch (see WwtLaunch)
__global__ __launch_bounds__(TN_THREADS, 2) void invert_product_kernel(const WwtLaunch lp)
{
    __shared__ float As[TN_LDS_STAGES][BK][BM];
    __shared__ float Bs[TN_LDS_STAGES][BK][BN];
    tn_tile_body(lp, As, Bs);
}

// The products of the blocked inversion (panel solves, row updates, merges).
__global__ __launch_bounds__(TN_THREADS, 2) void invert_gemm_kernel(const InvLaunch lp)
{
    __shared__ float As[TN_LDS_STAGES][BK][BM];
    __shared__ float Bs[TN_LDS_STAGES][BK][BN];
    tn_tile_body(lp, As, Bs);
}

}  // namespace kfac
