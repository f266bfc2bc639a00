// C ABI of the K-FAC work-item library (see include/kfac.h) and the host-side
// drivers that turn each work item into launches of the TN contraction engine
// and of the diagonal-block kernel.  Everything runs on the caller's stream;
// nothing here allocates, frees or synchronises.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <functional>
#include <new>
#include <vector>

#include "../../include/kfac.h"
#include "bf16_syrk256.h"
#include "mfma_probe.h"
#include "diag_block.h"
#include "tn_gemm.h"

using namespace kfac;

namespace {

constexpr size_t WS_ALIGN = 256;
constexpr int TARGET_TILES = 512;  // 256 CUs x 2 resident workgroups

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline bool fits_int(int64_t v) { return v > 0 && v < (int64_t(1) << 30); }

inline bool ws_ok(const void *ws, size_t have, size_t need)
{
    if (need == 0) return true;
    return ws != nullptr && have >= need && (reinterpret_cast<uintptr_t>(ws) % WS_ALIGN) == 0;
}

// One kernel launch (or a launch with its second pass) of a recorded sequence.
struct PlanStep {
    std::function<void(hipStream_t)> run;
    double flops;  // model cost: multiply-adds x 2 of the launch (0 for copies)
};
typedef std::vector<PlanStep> PlanSteps;

inline double tn_problem_flops(int M, int N, int K, int tile_mode, int mask_a, int mask_b)
{
    double f = 2.0 * M * N * K;
    if (tile_mode != TILE_FULL) f *= 0.5;
    if (mask_a != MASK_NONE || mask_b != MASK_NONE) f *= (mask_a != MASK_NONE && mask_b != MASK_NONE) ? (2.0 / 3.0) : 0.5;
    return f;
}

// Collects problems that share the launch parameters and sends them to the
// engine in chunks of at most TN_MAX_PROBLEMS (or records the launches).
struct TnBatch {
    PlanSteps *rec = nullptr;
    std::vector<TnProblem> probs;
    int tile_mode = TILE_FULL, mask_a = MASK_NONE, mask_b = MASK_NONE, splits = 1;
    float alpha = 1.f, beta = 0.f;
    float *partial = nullptr;

    void add(const float *A, int lda, const float *B, int ldb, float *C, int ldc, int M, int N, int K,
             float *Ct = nullptr, int ldct = 0, const int *guard = nullptr)
    {
        if (M <= 0 || N <= 0) return;
        TnProblem p;
        p.A = A; p.B = B; p.C = C; p.Ct = Ct; p.guard = guard;
        p.M = M; p.N = N; p.K = K;
        p.lda = lda; p.ldb = ldb; p.ldc = ldc; p.ldct = ldct;
        p.tile_begin = 0;
        probs.push_back(p);
    }

    hipError_t launch(hipStream_t stream)
    {
        size_t i = 0;
        while (i < probs.size()) {
            TnLaunch lp;
            std::memset(&lp, 0, sizeof(lp));
            int tiles = 0, cnt = 0;
            while (i < probs.size() && cnt < TN_MAX_PROBLEMS) {
                lp.p[cnt] = probs[i];
                lp.p[cnt].tile_begin = tiles;
                tiles += tn_tiles(probs[i].M, probs[i].N, tile_mode) * splits;
                ++cnt;
                ++i;
            }
            lp.c.count = cnt;
            lp.c.tile_mode = tile_mode;
            lp.c.mask_a = mask_a;
            lp.c.mask_b = mask_b;
            lp.c.splits = splits;
            lp.c.alpha = alpha;
            lp.c.beta = beta;
            lp.c.partial = partial;
            const int grid = tn_balance_xcds(lp, tiles);
            if (rec != nullptr) {
                double fl = 0.0;
                for (int k = 0; k < cnt; ++k) fl += tn_problem_flops(lp.p[k].M, lp.p[k].N, lp.p[k].K, tile_mode, mask_a, mask_b);
                const int sp = splits;
                rec->push_back(PlanStep{[lp, tiles, sp, grid](hipStream_t s) {
                                            hipLaunchKernelGGL(tn_gemm_kernel, dim3(grid), dim3(TN_THREADS), 0, s, lp);
                                            if (sp > 1)
                                                hipLaunchKernelGGL(tn_reduce_kernel, dim3(tiles / sp), dim3(TN_THREADS), 0, s, lp);
                                        },
                                        fl});
                continue;
            }
            hipLaunchKernelGGL(tn_gemm_kernel, dim3(grid), dim3(TN_THREADS), 0, stream, lp);
            if (splits > 1)
                hipLaunchKernelGGL(tn_reduce_kernel, dim3(tiles / splits), dim3(TN_THREADS), 0, stream, lp);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        probs.clear();
        return hipSuccess;
    }
};

// Split-K factor for a launch with `tiles` output tiles and K rows: enough
// splits to give every CU two workgroups, each split at least 256 rows long.
inline int choose_splits(int64_t tiles, int64_t K)
{
    if (tiles >= TARGET_TILES) return 1;
    const int64_t by_tiles = (TARGET_TILES + tiles - 1) / tiles;
    const int64_t by_k = std::max<int64_t>(1, K / 256);
    return (int)std::max<int64_t>(1, std::min<int64_t>(std::min(by_tiles, by_k), 32));
}

// ------------------------------------------------------------------ curvature

struct CurvPlan {
    int splits;
    int64_t tiles;  // output tiles of all items
    size_t pack;    // bytes of the repacked bf16 inputs (bf16 only), in front of the partial tiles
    size_t ws;
};

inline int pack_groups(int64_t n) { return (int)align_up((size_t)((n + 7) / 8), BF_SLAB_GROUPS); }
inline int pack_cols(int64_t d) { return (int)align_up((size_t)d, B2_TILE); }
inline size_t pack_bytes(int64_t n, int64_t d) { return align_up((size_t)pack_groups(n) * pack_cols(d) * 16, WS_ALIGN); }

bool curvature_plan(const kfac_curvature_item *items, int64_t count, kfac_dtype dtype, CurvPlan &pl)
{
    int64_t tiles = 0, kmin = INT64_MAX;
    for (int64_t i = 0; i < count; ++i) {
        if (!fits_int(items[i].d) || !fits_int(items[i].n_tokens)) return false;
        tiles += tn_tiles((int)items[i].d, (int)items[i].d, TILE_LOWER);
        kmin = std::min(kmin, items[i].n_tokens);
    }
    // a launch holds at most TN_MAX_PROBLEMS items; size the split for one launch
    const int64_t launches = (count + SYRK_MAX_PROBLEMS - 1) / SYRK_MAX_PROBLEMS;
    pl.splits = choose_splits(std::max<int64_t>(1, tiles / std::max<int64_t>(1, launches)), kmin);
    pl.tiles = tiles;
    pl.pack = 0;
    if (dtype == KFAC_BF16)
        for (int64_t i = 0; i < count; ++i) pl.pack += pack_bytes(items[i].n_tokens, items[i].d);
    pl.ws = pl.pack + (pl.splits > 1 ? align_up((size_t)tiles * pl.splits * BM * BN * sizeof(float), WS_ALIGN) : 0);
    return true;
}

// ------------------------------------------------------------------ inversion

inline int work_ld(int64_t d) { return (int)align_up((size_t)d, 32); }

inline size_t invert_item_bytes(int64_t d)
{
    return 2 * align_up((size_t)d * work_ld(d) * sizeof(float), WS_ALIGN);
}

struct InvMat {
    float *F, *S;
    int d, ld, nblk;
    float *inv;
    int ldi;
    int *info;
};

struct TriNode {
    int mat, a, b, c;  // matrix, first block, blocks in the first part, blocks in the second part
};

// Balanced splitting of block range [lo, hi): returns the height of the node and
// files it under that height.  Nodes of equal height are independent.
int build_tree(int mat, int lo, int hi, std::vector<std::vector<TriNode>> &levels)
{
    if (hi - lo <= 1) return 0;
    const int mid = lo + (hi - lo + 1) / 2;
    const int hl = build_tree(mat, lo, mid, levels);
    const int hr = build_tree(mat, mid, hi, levels);
    const int h = 1 + std::max(hl, hr);
    if ((int)levels.size() <= h) levels.resize(h + 1);
    levels[h].push_back(TriNode{mat, lo, mid - lo, hi - mid});
    return h;
}

// Sends the nodes of one phase of the inversion to invert_gemm_kernel, as many per
// launch as the kernel arguments hold.
struct InvBatch {
    PlanSteps *rec = nullptr;
    const std::vector<InvMat> &mats;
    std::vector<TriNode> nodes;
    int op = 0, tile_mode = TILE_FULL, mask_a = MASK_NONE, mask_b = MASK_NONE, reverse_cols = 0;
    float alpha = 1.f, beta = 0.f;

    explicit InvBatch(const std::vector<InvMat> &m) : mats(m) {}

    void add(int mat, int a, int b = 0, int c = 0) { nodes.push_back(TriNode{mat, a, b, c}); }

    hipError_t launch(hipStream_t stream)
    {
        size_t i = 0;
        while (i < nodes.size()) {
            InvLaunch lp;
            std::memset(&lp, 0, sizeof(lp));
            for (size_t k = 0; k < mats.size(); ++k) {
                lp.m[k].F = mats[k].F;
                lp.m[k].S = mats[k].S;
                lp.m[k].d = mats[k].d;
                lp.m[k].ld = mats[k].ld;
            }
            int tiles = 0, cnt = 0;
            while (i < nodes.size() && cnt < INV_MAX_NODES) {
                const TriNode &nd = nodes[i++];
                const InvDims dm = inv_dims(op, mats[(size_t)nd.mat].d, nd.a, nd.b, nd.c);
                if (dm.M <= 0 || dm.N <= 0) continue;
                lp.n[cnt].mat = (unsigned char)nd.mat;
                lp.n[cnt].a = (unsigned char)nd.a;
                lp.n[cnt].b = (unsigned char)nd.b;
                lp.n[cnt].c = (unsigned char)nd.c;
                lp.n[cnt].tile_begin = tiles;
                tiles += tn_tiles(dm.M, dm.N, tile_mode);
                ++cnt;
            }
            if (cnt == 0) continue;
            lp.c.count = cnt;
            lp.c.tile_mode = tile_mode;
            lp.c.mask_a = mask_a;
            lp.c.mask_b = mask_b;
            lp.c.splits = 1;
            lp.c.alpha = alpha;
            lp.c.beta = beta;
            lp.c.reverse_cols = reverse_cols;
            lp.op = op;
            const int grid = tn_balance_xcds(lp, tiles);
            if (rec != nullptr) {
                double fl = 0.0;
                for (int k = 0; k < cnt; ++k) {
                    const InvDims dm = inv_dims(op, lp.m[lp.n[k].mat].d, lp.n[k].a, lp.n[k].b, lp.n[k].c);
                    fl += tn_problem_flops(dm.M, dm.N, dm.K, tile_mode, mask_a, mask_b);
                }
                rec->push_back(PlanStep{[lp, grid](hipStream_t s) {
                                            hipLaunchKernelGGL(invert_gemm_kernel, dim3(grid), dim3(TN_THREADS), 0, s, lp);
                                        },
                                        fl});
                continue;
            }
            hipLaunchKernelGGL(invert_gemm_kernel, dim3(grid), dim3(TN_THREADS), 0, stream, lp);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        nodes.clear();
        return hipSuccess;
    }
};

constexpr int SUPER_PANEL = 4;  // block rows factored before one trailing update (K = 512)

}  // namespace

extern "C" {

const char *kfac_status_string(kfac_status s)
{
    switch (s) {
        case KFAC_OK: return "ok";
        case KFAC_ERR_ARG: return "invalid argument";
        case KFAC_ERR_UNSUPPORTED: return "unsupported dtype or option";
        case KFAC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case KFAC_ERR_HIP: return "HIP launch error";
    }
    return "unknown status";
}

kfac_status kfac_mfma_probe(kfac_dtype dtype, int64_t iters, void *sink, double *flops, void *stream)
{
    if (sink == nullptr || flops == nullptr || iters <= 0 || iters > INT32_MAX) return KFAC_ERR_ARG;
    if (dtype != KFAC_F32 && dtype != KFAC_BF16) return KFAC_ERR_ARG;
    constexpr int WORKGROUPS = 256 * 2 * 8;  // eight rounds of two workgroups per CU
    hipStream_t st = static_cast<hipStream_t>(stream);
    const double per_mfma = dtype == KFAC_F32 ? 4096.0 : 32768.0;
    *flops = (double)WORKGROUPS * 4.0 * (double)iters * PROBE_MFMA_PER_ITER * per_mfma;
    if (dtype == KFAC_F32)
        hipLaunchKernelGGL(mfma_probe_f32_kernel, dim3(WORKGROUPS), dim3(256), 0, st, 1.0f, 2.0f, (int)iters,
                           static_cast<float *>(sink));
    else
        hipLaunchKernelGGL(mfma_probe_bf16_kernel, dim3(WORKGROUPS), dim3(256), 0, st, 0x3f803f80u, 0x3f003f00u, (int)iters,
                           static_cast<float *>(sink));
    return hipGetLastError() == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
}

int kfac_version(void) { return 100; }

// ------------------------------------------------------------------ curvature

size_t kfac_curvature_grouped_workspace(const kfac_curvature_item *items, int64_t count, kfac_dtype dtype)
{
    if (items == nullptr || count <= 0) return 0;
    CurvPlan pl;
    if (!curvature_plan(items, count, dtype, pl)) return 0;
    return pl.ws;
}

kfac_status kfac_curvature_grouped(const kfac_curvature_item *items, int64_t count, kfac_dtype dtype,
                                   float alpha, float beta, void *workspace, size_t workspace_bytes, void *stream)
{
    if (count == 0) return KFAC_OK;
    if (items == nullptr || count < 0) return KFAC_ERR_ARG;
    if (dtype != KFAC_F32 && dtype != KFAC_BF16) return KFAC_ERR_ARG;
    for (int64_t i = 0; i < count; ++i) {
        const kfac_curvature_item &it = items[i];
        if (it.x == nullptr || it.factor == nullptr) return KFAC_ERR_ARG;
        if (!fits_int(it.d) || !fits_int(it.n_tokens)) return KFAC_ERR_ARG;
        if (it.ldx < it.d || it.ldf < it.d || !fits_int(it.ldx) || !fits_int(it.ldf)) return KFAC_ERR_ARG;
        if ((reinterpret_cast<uintptr_t>(it.x) & (dtype == KFAC_BF16 ? 1 : 3)) || (reinterpret_cast<uintptr_t>(it.factor) & 3))
            return KFAC_ERR_ARG;
    }
    if (dtype == KFAC_BF16)
        for (int64_t i = 0; i < count; ++i)
            if (items[i].d > (1 << 26)) return KFAC_ERR_UNSUPPORTED;  // packed rows are addressed with 32-bit byte offsets
    CurvPlan pl;
    if (!curvature_plan(items, count, dtype, pl)) return KFAC_ERR_ARG;
    if (!ws_ok(workspace, workspace_bytes, pl.ws)) return KFAC_ERR_WORKSPACE;

    // One launch per SYRK_MAX_PROBLEMS items (a BERT-Large stage has 72 factors:
    // one launch per micro-batch); each launch gets its own slice of the partial buffer.
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *pack = static_cast<char *>(workspace);
    float *part = reinterpret_cast<float *>(static_cast<char *>(workspace) + pl.pack);
    for (int64_t done = 0; done < count;) {
        const int64_t n = std::min<int64_t>(SYRK_MAX_PROBLEMS, count - done);
        SyrkLaunch lp;
        std::memset(&lp, 0, sizeof(lp));
        PackLaunch pk;
        if (dtype == KFAC_BF16) std::memset(&pk, 0, sizeof(pk));
        int tiles = 0, gmax = 0, cmax = 0;
        for (int64_t i = 0; i < n; ++i) {
            const kfac_curvature_item &it = items[done + i];
            SyrkProblem &q = lp.p[i];
            q.x = it.x;
            q.factor = it.factor;
            q.n = (int)it.n_tokens;
            q.d = (int)it.d;
            q.ldx = (int)it.ldx;
            q.ldf = (int)it.ldf;
            if (dtype == KFAC_BF16) {
                // the kernel reads the repacked copy: [groups of 8 tokens][padded columns][8]
                PackItem &pi = pk.it[i];
                pi.x = static_cast<const unsigned short *>(it.x);
                pi.dst = reinterpret_cast<unsigned short *>(pack);
                pi.n = q.n;
                pi.d = q.d;
                pi.ldx = q.ldx;
                pi.dp = pack_cols(it.d);
                pi.gp = pack_groups(it.n_tokens);
                q.x = pack;
                q.n = pi.gp * BF_KG;
                q.ldx = pi.dp;
                pack += pack_bytes(it.n_tokens, it.d);
                gmax = std::max(gmax, pi.gp);
                cmax = std::max(cmax, pi.dp);
            }
            q.tile_begin = tiles;
            tiles += tn_tiles(q.d, q.d, TILE_LOWER) * pl.splits;
        }
        lp.c.count = (int)n;
        lp.c.tile_mode = TILE_LOWER;
        lp.c.mask_a = MASK_NONE;
        lp.c.mask_b = MASK_NONE;
        lp.c.splits = pl.splits;
        lp.c.alpha = alpha;
        lp.c.beta = beta;
        lp.c.partial = part;
        int tiles256 = 0;
        if (dtype == KFAC_BF16)
            for (int64_t i = 0; i < n; ++i) tiles256 += b2_tiles(lp.p[i].d);
        if (dtype == KFAC_BF16 && tiles256 >= 192) {
            // enough 256 x 256 tiles to occupy the chip: twice the flops per byte fetched
            Syrk256Launch l2;
            std::memset(&l2, 0, sizeof(l2));
            int tb = 0;
            for (int64_t i = 0; i < n; ++i) {
                l2.p[i] = lp.p[i];
                l2.p[i].tile_begin = tb;
                tb += b2_tiles(lp.p[i].d);
            }
            l2.count = (int)n;
            l2.alpha = alpha;
            l2.beta = beta;
            // inputs that need no padding are read as they are (transposing LDS reads), without the pre-pass
            bool rowmajor = true;
            for (int64_t i = 0; i < n; ++i) {
                const kfac_curvature_item &it = items[done + i];
                rowmajor = rowmajor && it.d % B2_TILE == 0 && it.n_tokens % B2R_SLAB_ROWS == 0 && it.ldx % 8 == 0 &&
                           (reinterpret_cast<uintptr_t>(it.x) & 15) == 0;
            }
            if (rowmajor) {
                for (int64_t i = 0; i < n; ++i) {
                    const kfac_curvature_item &it = items[done + i];
                    l2.p[i].x = it.x;
                    l2.p[i].n = (int)it.n_tokens;
                    l2.p[i].ldx = (int)it.ldx;
                }
                hipLaunchKernelGGL(curvature_syrk_bf16_256_rowmajor_kernel, dim3(tb), dim3(256), 0, st, l2);
            } else {
                hipLaunchKernelGGL(pack_bf16_kernel, dim3((cmax + PACK_COLS - 1) / PACK_COLS, gmax / BF_SLAB_GROUPS, (unsigned)n), dim3(256), 0, st, pk);
                hipLaunchKernelGGL(curvature_syrk_bf16_256_kernel, dim3(tb), dim3(256), 0, st, l2);
            }
        } else if (dtype == KFAC_BF16) {
            SyrkLaunchPacked lb;
            static_assert(sizeof(lb) == sizeof(lp), "the curvature launch types share one layout");
            lp.c.slab_align = 2;  // slabs of the engine are 16 tokens, the bf16 loop steps by 32
            std::memcpy(&lb, &lp, sizeof(lp));
            hipLaunchKernelGGL(pack_bf16_kernel, dim3((cmax + PACK_COLS - 1) / PACK_COLS, gmax / BF_SLAB_GROUPS, (unsigned)n), dim3(256), 0, st, pk);
            hipLaunchKernelGGL(curvature_syrk_bf16mfma_kernel, dim3(tiles), dim3(TN_THREADS), 0, st, lb);
            if (pl.splits > 1)
                hipLaunchKernelGGL(curvature_reduce_packed_kernel, dim3(tiles / pl.splits), dim3(TN_THREADS), 0, st, lb);
        } else {
            hipLaunchKernelGGL(curvature_syrk_kernel, dim3(tiles), dim3(TN_THREADS), 0, st, lp);
            if (pl.splits > 1)
                hipLaunchKernelGGL(curvature_reduce_kernel, dim3(tiles / pl.splits), dim3(TN_THREADS), 0, st, lp);
        }
        if (pl.splits > 1) part += (size_t)tiles * BM * BN;
        if (hipGetLastError() != hipSuccess) return KFAC_ERR_HIP;
        done += n;
    }
    return KFAC_OK;
}

size_t kfac_curvature_workspace(int64_t n_tokens, int64_t d, kfac_dtype dtype)
{
    kfac_curvature_item it;
    std::memset(&it, 0, sizeof(it));
    it.n_tokens = n_tokens;
    it.d = d;
    return kfac_curvature_grouped_workspace(&it, 1, dtype);
}

kfac_status kfac_curvature(const void *x, kfac_dtype dtype, int64_t n_tokens, int64_t d, int64_t ldx,
                           float alpha, float beta, float *factor, int64_t ldf,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    kfac_curvature_item it;
    it.x = x;
    it.n_tokens = n_tokens;
    it.d = d;
    it.ldx = ldx;
    it.factor = factor;
    it.ldf = ldf;
    return kfac_curvature_grouped(&it, 1, dtype, alpha, beta, workspace, workspace_bytes, stream);
}

// ------------------------------------------------------------------ inversion

size_t kfac_invert_batched_workspace(const kfac_invert_item *items, int64_t count)
{
    if (items == nullptr || count <= 0) return 0;
    size_t total = 0;
    for (int64_t i = 0; i < count; ++i) {
        if (!fits_int(items[i].d)) return 0;
        total += invert_item_bytes(items[i].d);
    }
    return total;
}

size_t kfac_invert_workspace(int64_t d)
{
    return fits_int(d) ? invert_item_bytes(d) : 0;
}

}  // extern "C"

namespace {

// Validates the arguments and records the launch sequence of a batched inversion.
kfac_status invert_record(const kfac_invert_item *items, int64_t count, float damping,
                          void *workspace, size_t workspace_bytes, PlanSteps &steps)
{
    if (count == 0) return KFAC_OK;
    if (items == nullptr || count < 0) return KFAC_ERR_ARG;
    if (!(damping >= 0.f)) return KFAC_ERR_ARG;
    for (int64_t i = 0; i < count; ++i) {
        const kfac_invert_item &it = items[i];
        if (it.factor == nullptr || it.inv == nullptr || it.info_dev == nullptr) return KFAC_ERR_ARG;
        if (!fits_int(it.d) || it.ldf < it.d || it.ldi < it.d || !fits_int(it.ldf) || !fits_int(it.ldi)) return KFAC_ERR_ARG;
        if ((reinterpret_cast<uintptr_t>(it.factor) & 3) || (reinterpret_cast<uintptr_t>(it.inv) & 3) ||
            (reinterpret_cast<uintptr_t>(it.info_dev) & 3))
            return KFAC_ERR_ARG;
        if (static_cast<const void *>(it.factor) == static_cast<const void *>(it.inv)) return KFAC_ERR_ARG;
    }
    for (int64_t i = 0; i < count; ++i)
        if (items[i].d > 255 * NB) return KFAC_ERR_UNSUPPORTED;  // block indices travel as bytes
    const size_t need = kfac_invert_batched_workspace(items, count);
    if (!ws_ok(workspace, workspace_bytes, need)) return KFAC_ERR_WORKSPACE;
    if (count > INV_MAX_MATS) {
        // more matrices than one launch describes: run the batch in slices, one after the other
        char *base = static_cast<char *>(workspace);
        for (int64_t i0 = 0; i0 < count; i0 += INV_MAX_MATS) {
            const int64_t n = std::min<int64_t>(INV_MAX_MATS, count - i0);
            const size_t bytes = kfac_invert_batched_workspace(items + i0, n);
            const kfac_status stt = invert_record(items + i0, n, damping, base, bytes, steps);
            if (stt != KFAC_OK) return stt;
            base += bytes;
        }
        return KFAC_OK;
    }
    hipStream_t st = nullptr;  // launches are recorded, not issued

    std::vector<InvMat> mats((size_t)count);
    char *cur = static_cast<char *>(workspace);
    int max_blk = 0;
    for (int64_t i = 0; i < count; ++i) {
        InvMat &m = mats[(size_t)i];
        m.d = (int)items[i].d;
        m.ld = work_ld(m.d);
        const size_t one = align_up((size_t)m.d * m.ld * sizeof(float), WS_ALIGN);
        m.F = reinterpret_cast<float *>(cur);
        m.S = reinterpret_cast<float *>(cur + one);
        cur += 2 * one;
        m.nblk = (m.d + NB - 1) / NB;
        m.inv = items[i].inv;
        m.ldi = (int)items[i].ldi;
        m.info = items[i].info_dev;
        max_blk = std::max(max_blk, m.nblk);
    }

    // 1. info = 0; working copy F = factor + damping I.
    for (size_t i0 = 0; i0 < mats.size(); i0 += PREP_MAX_ITEMS) {
        const size_t n = std::min<size_t>(PREP_MAX_ITEMS, mats.size() - i0);
        PrepLaunch pl;
        std::memset(&pl, 0, sizeof(pl));
        int dmax = 0;
        for (size_t i = 0; i < n; ++i) {
            const InvMat &m = mats[i0 + i];
            pl.it[i].src = items[i0 + i].factor;
            pl.it[i].dst = m.F;
            pl.it[i].info = m.info;
            pl.it[i].d = m.d;
            pl.it[i].lds_ = (int)items[i0 + i].ldf;
            pl.it[i].ldd = m.ld;
            dmax = std::max(dmax, m.d);
        }
        pl.damping = damping;
        const int nn = (int)n, gx = std::min(dmax, 512);
        steps.push_back(PlanStep{[pl, nn, gx](hipStream_t s) {
                                     hipLaunchKernelGGL(invert_clear_info_kernel, dim3(1), dim3(128), 0, s, pl, nn);
                                     hipLaunchKernelGGL(invert_prepare_kernel, dim3(gx, (unsigned)nn), dim3(256), 0, s, pl);
                                 },
                                 0.0});
    }

    // 2. Blocked upper Cholesky M = U^T U with panel width NB, all matrices advanced together.
    //    Inside a super-panel of SUPER_PANEL block rows the factorisation is left-looking (a block
    //    row is brought up to date just before it is factored); the rest of the matrix is updated
    //    once per super-panel, so that it is read and written SUPER_PANEL times less often.
    InvBatch solve(mats), rowup(mats), trail(mats);
    solve.rec = rowup.rec = trail.rec = &steps;
    solve.op = INV_PANEL_SOLVE;
    solve.mask_a = MASK_KEEP_K_LE;  // U_jj^-1 is upper triangular: rows k <= column
    rowup.op = INV_ROW_UPDATE;
    rowup.alpha = -1.f;
    rowup.beta = 1.f;
    trail.op = INV_TRAIL_UPDATE;
    trail.tile_mode = TILE_UPPER;
    trail.alpha = -1.f;
    trail.beta = 1.f;
    for (int s0 = 0; s0 < max_blk; s0 += SUPER_PANEL) {
        for (int j = s0; j < std::min(s0 + SUPER_PANEL, max_blk); ++j) {
            std::vector<DiagItem> ditems;
            for (size_t mi = 0; mi < mats.size(); ++mi) {
                const InvMat &m = mats[mi];
                if (j >= m.nblk) continue;
                const int r0 = j * NB;
                const int n = std::min(NB, m.d - r0);
                DiagItem di;
                di.F = m.F + (size_t)r0 * m.ld + r0;
                di.S = m.S + (size_t)r0 * m.ld + r0;
                di.info = m.info;
                di.n = n;
                di.ldf = m.ld;
                di.lds = m.ld;
                di.pivot_base = r0;
                ditems.push_back(di);
                if (j > s0) rowup.add((int)mi, s0, j);
                if (m.d - r0 - n > 0) solve.add((int)mi, j);
            }
            if (rowup.launch(st) != hipSuccess) return KFAC_ERR_HIP;
            for (size_t i0 = 0; i0 < ditems.size(); i0 += DIAG_MAX_ITEMS) {
                const size_t n = std::min<size_t>(DIAG_MAX_ITEMS, ditems.size() - i0);
                DiagLaunch dl;
                std::memset(&dl, 0, sizeof(dl));
                for (size_t i = 0; i < n; ++i) dl.it[i] = ditems[i0 + i];
                const unsigned nb = (unsigned)n;
                double fl = 0.0;
                for (size_t i = 0; i < n; ++i) fl += 2.0 / 3.0 * dl.it[i].n * (double)dl.it[i].n * dl.it[i].n;
                steps.push_back(PlanStep{[dl, nb](hipStream_t s) {
                                             hipLaunchKernelGGL(diag_block_kernel, dim3(nb), dim3(DIAG_THREADS), 0, s, dl);
                                         },
                                         fl});
            }
            if (solve.launch(st) != hipSuccess) return KFAC_ERR_HIP;
        }
        for (size_t mi = 0; mi < mats.size(); ++mi) {
            const int e = std::min(s0 + SUPER_PANEL, mats[mi].nblk);
            if (s0 < mats[mi].nblk && e < mats[mi].nblk) trail.add((int)mi, s0, e);
        }
        if (trail.launch(st) != hipSuccess) return KFAC_ERR_HIP;
    }

    // 3. W = U^-1 by pairwise merging of already inverted diagonal ranges:
    //    [U11 U12; 0 U22]^-1 = [W11, -W11 U12 W22; 0, W22].
    //    Y = U12 W22 goes where U12 was (the factor's upper blocks are no longer needed:
    //    later merges read the mirrored copy below the diagonal).
    std::vector<std::vector<TriNode>> levels;
    for (size_t i = 0; i < mats.size(); ++i) build_tree((int)i, 0, mats[i].nblk, levels);
    InvBatch s1(mats), s2(mats);
    s1.rec = s2.rec = &steps;
    s1.op = INV_MERGE_Y;
    s1.mask_b = MASK_KEEP_K_LE;  // W22 upper triangular
    s1.reverse_cols = 1;         // K grows with the tile column: last columns first
    s2.op = INV_MERGE_W;
    s2.mask_a = MASK_KEEP_K_GE;  // W11 read through its mirror below the diagonal
    s2.alpha = -1.f;
    for (size_t h = 1; h < levels.size(); ++h) {
        s1.nodes = levels[h];
        s2.nodes = levels[h];
        if (s1.launch(st) != hipSuccess) return KFAC_ERR_HIP;
        if (s2.launch(st) != hipSuccess) return KFAC_ERR_HIP;
    }

    // 4. inv = W W^T, read through the mirror: inv[i][j] = sum_{k >= max(i,j)} S[k][i] S[k][j].
    TnBatch lu;
    lu.rec = &steps;
    lu.tile_mode = TILE_LOWER;
    lu.mask_a = MASK_KEEP_K_GE;
    lu.mask_b = MASK_KEEP_K_GE;
    for (const InvMat &m : mats) lu.add(m.S, m.ld, m.S, m.ld, m.inv, m.ldi, m.d, m.d, m.d, m.inv, m.ldi, m.info);
    if (lu.launch(st) != hipSuccess) return KFAC_ERR_HIP;
    return KFAC_OK;
}

}  // namespace

// Opaque handle of a recorded inversion (host memory only).
struct kfac_invert_plan {
    PlanSteps steps;
    int64_t next = 0;
};

extern "C" {

kfac_status kfac_invert_batched(const kfac_invert_item *items, int64_t count, float damping,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    PlanSteps steps;
    const kfac_status st = invert_record(items, count, damping, workspace, workspace_bytes, steps);
    if (st != KFAC_OK) return st;
    if (steps.empty()) return KFAC_OK;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    for (PlanStep &p : steps) p.run(hs);
    return hipGetLastError() == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
}

kfac_status kfac_invert_plan_create(const kfac_invert_item *items, int64_t count, float damping,
                                    void *workspace, size_t workspace_bytes, kfac_invert_plan **plan)
{
    if (plan == nullptr) return KFAC_ERR_ARG;
    *plan = nullptr;
    kfac_invert_plan *p = new (std::nothrow) kfac_invert_plan();
    if (p == nullptr) return KFAC_ERR_ARG;
    const kfac_status st = invert_record(items, count, damping, workspace, workspace_bytes, p->steps);
    if (st != KFAC_OK) {
        delete p;
        return st;
    }
    *plan = p;
    return KFAC_OK;
}

int64_t kfac_invert_plan_steps(const kfac_invert_plan *plan) { return plan ? (int64_t)plan->steps.size() : 0; }

int64_t kfac_invert_plan_position(const kfac_invert_plan *plan) { return plan ? plan->next : 0; }

double kfac_invert_plan_step_flops(const kfac_invert_plan *plan, int64_t step)
{
    if (plan == nullptr || step < 0 || step >= (int64_t)plan->steps.size()) return -1.0;
    return plan->steps[(size_t)step].flops;
}

kfac_status kfac_invert_plan_run(kfac_invert_plan *plan, int64_t n_steps, void *stream)
{
    if (plan == nullptr || n_steps < 0) return KFAC_ERR_ARG;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int64_t end = std::min<int64_t>(plan->next + n_steps, (int64_t)plan->steps.size());
    if (end == plan->next) return KFAC_OK;
    for (; plan->next < end; ++plan->next) plan->steps[(size_t)plan->next].run(hs);
    return hipGetLastError() == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
}

kfac_status kfac_invert_plan_reset(kfac_invert_plan *plan)
{
    if (plan == nullptr) return KFAC_ERR_ARG;
    plan->next = 0;
    return KFAC_OK;
}

void kfac_invert_plan_destroy(kfac_invert_plan *plan) { delete plan; }

kfac_status kfac_invert(const float *factor, int64_t d, int64_t ldf, float damping,
                        float *inv, int64_t ldi, int32_t *info_dev,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    kfac_invert_item it;
    it.factor = factor;
    it.d = d;
    it.ldf = ldf;
    it.inv = inv;
    it.ldi = ldi;
    it.info_dev = info_dev;
    return kfac_invert_batched(&it, 1, damping, workspace, workspace_bytes, stream);
}

// --------------------------------------------------------------- precondition

namespace {
struct PrecPlan {
    int splits1, splits2;
    size_t t_bytes, part_bytes, ws;
};

bool precondition_plan(const kfac_precondition_item *items, int64_t count, PrecPlan &pl)
{
    int64_t tiles1 = 0, tiles2 = 0, k1 = INT64_MAX, k2 = INT64_MAX;
    size_t t_bytes = 0;
    for (int64_t i = 0; i < count; ++i) {
        if (!fits_int(items[i].d_out) || !fits_int(items[i].d_in)) return false;
        const int dout = (int)items[i].d_out, din = (int)items[i].d_in;
        tiles1 += tn_tiles(din, dout, TILE_FULL);
        tiles2 += tn_tiles(dout, din, TILE_FULL);
        k1 = std::min<int64_t>(k1, dout);
        k2 = std::min<int64_t>(k2, din);
        t_bytes += align_up((size_t)din * dout * sizeof(float), WS_ALIGN);
    }
    const int64_t launches = (count + TN_MAX_PROBLEMS - 1) / TN_MAX_PROBLEMS;
    pl.splits1 = choose_splits(std::max<int64_t>(1, tiles1 / launches), k1);
    pl.splits2 = choose_splits(std::max<int64_t>(1, tiles2 / launches), k2);
    pl.t_bytes = t_bytes;
    const size_t p1 = pl.splits1 > 1 ? (size_t)tiles1 * pl.splits1 * BM * BN * sizeof(float) : 0;
    const size_t p2 = pl.splits2 > 1 ? (size_t)tiles2 * pl.splits2 * BM * BN * sizeof(float) : 0;
    pl.part_bytes = align_up(std::max(p1, p2), WS_ALIGN);
    pl.ws = pl.t_bytes + pl.part_bytes;
    return true;
}
}  // namespace

size_t kfac_precondition_grouped_workspace(const kfac_precondition_item *items, int64_t count)
{
    if (items == nullptr || count <= 0) return 0;
    PrecPlan pl;
    if (!precondition_plan(items, count, pl)) return 0;
    return pl.ws;
}

size_t kfac_precondition_workspace(int64_t d_out, int64_t d_in)
{
    kfac_precondition_item it;
    std::memset(&it, 0, sizeof(it));
    it.d_out = d_out;
    it.d_in = d_in;
    return kfac_precondition_grouped_workspace(&it, 1);
}

kfac_status kfac_precondition_grouped(const kfac_precondition_item *items, int64_t count,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    if (count == 0) return KFAC_OK;
    if (items == nullptr || count < 0) return KFAC_ERR_ARG;
    for (int64_t i = 0; i < count; ++i) {
        const kfac_precondition_item &it = items[i];
        if (!it.b_inv || !it.a_inv || !it.grad || !it.out) return KFAC_ERR_ARG;
        if (!fits_int(it.d_out) || !fits_int(it.d_in)) return KFAC_ERR_ARG;
        if (it.ldb < it.d_out || it.lda < it.d_in || it.ldg < it.d_in || it.ldo < it.d_in) return KFAC_ERR_ARG;
        if (!fits_int(it.ldb) || !fits_int(it.lda) || !fits_int(it.ldg) || !fits_int(it.ldo)) return KFAC_ERR_ARG;
        if ((reinterpret_cast<uintptr_t>(it.b_inv) & 3) || (reinterpret_cast<uintptr_t>(it.a_inv) & 3) ||
            (reinterpret_cast<uintptr_t>(it.grad) & 3) || (reinterpret_cast<uintptr_t>(it.out) & 3))
            return KFAC_ERR_ARG;
    }
    PrecPlan pl;
    if (!precondition_plan(items, count, pl)) return KFAC_ERR_ARG;
    if (!ws_ok(workspace, workspace_bytes, pl.ws)) return KFAC_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *tbase = static_cast<char *>(workspace);
    float *partial = reinterpret_cast<float *>(tbase + pl.t_bytes);

    // T^T = G^T B^-1   (d_in x d_out), then  out = (T^T)^T A^-1.
    for (int pass = 0; pass < 2; ++pass) {
        size_t done = 0;
        char *tcur = tbase;
        while (done < (size_t)count) {
            const size_t n = std::min<size_t>(TN_MAX_PROBLEMS, (size_t)count - done);
            TnBatch b;
            b.tile_mode = TILE_FULL;
            b.splits = pass == 0 ? pl.splits1 : pl.splits2;
            b.partial = partial;
            for (size_t i = done; i < done + n; ++i) {
                const kfac_precondition_item &it = items[i];
                const int dout = (int)it.d_out, din = (int)it.d_in;
                float *tt = reinterpret_cast<float *>(tcur);
                tcur += align_up((size_t)din * dout * sizeof(float), WS_ALIGN);
                if (pass == 0)
                    b.add(it.grad, (int)it.ldg, it.b_inv, (int)it.ldb, tt, dout, din, dout, dout);
                else
                    b.add(tt, dout, it.a_inv, (int)it.lda, it.out, (int)it.ldo, dout, din, din);
            }
            if (b.launch(st) != hipSuccess) return KFAC_ERR_HIP;
            done += n;
        }
    }
    return KFAC_OK;
}

kfac_status kfac_precondition(const float *b_inv, int64_t d_out, int64_t ldb,
                              const float *a_inv, int64_t d_in, int64_t lda,
                              const float *grad, int64_t ldg, float *out, int64_t ldo,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    kfac_precondition_item it;
    it.b_inv = b_inv;
    it.d_out = d_out;
    it.ldb = ldb;
    it.a_inv = a_inv;
    it.d_in = d_in;
    it.lda = lda;
    it.grad = grad;
    it.ldg = ldg;
    it.out = out;
    it.ldo = ldo;
    return kfac_precondition_grouped(&it, 1, workspace, workspace_bytes, stream);
}

}  // extern "C"
