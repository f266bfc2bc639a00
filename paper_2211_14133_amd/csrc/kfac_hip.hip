// C ABI of the K-FAC work-item library (see include/kfac.h) and the host-side
// drivers that turn each work item into launches of the TN contraction engine
// and of the diagonal-block kernel.  Everything runs on the caller's stream;
// nothing here allocates or frees device memory or synchronises (host-side
// bookkeeping lives on the heap for the length of a call, or of a plan).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/kfac.h"
#include "bf16_syrk256.h"
#include "split3_syrk256.h"
#include "split2_syrk256.h"
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

// Non-zero elements of a triangular operand: K rows, W columns, column c holds the rows k >= c or k <= c.
inline double kept_elements(int mask, double K, double W)
{
    if (mask == MASK_ZEROS_K_GT) return W <= K ? W * (W + 1) / 2 : K * (K + 1) / 2 + (W - K) * K;
    return W <= K ? W * K - W * (W - 1) / 2 : K * (K + 1) / 2;  // MASK_ZEROS_K_LT
}

// Useful multiply-adds x 2 of a problem: a triangular operand only counts with the elements it keeps; two
// of them with a triangular tile set (W W^T) leave a sixth of the full product, d^3 / 3.
inline double tn_problem_flops(int M, int N, int K, int tile_mode, int mask_a, int mask_b)
{
    const bool ma = mask_a != MASK_NONE, mb = mask_b != MASK_NONE;
    double f;
    if (ma && mb)
        f = 2.0 * M * N * K / (tile_mode != TILE_FULL ? 6.0 : 3.0);
    else if (ma)
        f = 2.0 * N * kept_elements(mask_a, K, M);
    else if (mb)
        f = 2.0 * M * kept_elements(mask_b, K, N);
    else
        f = 2.0 * M * N * K;
    if (tile_mode != TILE_FULL && !(ma && mb)) f *= 0.5;
    return f;
}

// Where the launches of a work item go: straight to a stream, or into a recorded plan.
struct Emitter {
    virtual ~Emitter() {}
    const char *label = "";  // what the next launches do (static string; kept with recorded steps)
    virtual void prep(const PrepLaunch &pl, int count, int grid_x) = 0;
    virtual void inv(const InvLaunch &lp, int grid, bool with_diag, double flops) = 0;
    virtual void tn(const TnLaunch &lp, int grid, int tiles, double flops) = 0;
    virtual void wwt(const WwtLaunch &lp, int grid, double flops) = 0;
};

void launch_prep(hipStream_t s, const PrepLaunch &pl, int count, int grid_x)
{
    hipLaunchKernelGGL(invert_clear_info_kernel, dim3(1), dim3(128), 0, s, pl, count);
    hipLaunchKernelGGL(invert_prepare_kernel, dim3(grid_x, (unsigned)count), dim3(256), 0, s, pl);
}

void launch_inv(hipStream_t s, const InvLaunch &lp, int grid, bool with_diag)
{
    if (with_diag)
        hipLaunchKernelGGL(invert_diag_gemm_kernel, dim3(grid), dim3(TN_THREADS), 0, s, lp);
    else
        hipLaunchKernelGGL(invert_gemm_kernel, dim3(grid), dim3(TN_THREADS), 0, s, lp);
}

void launch_wwt(hipStream_t s, const WwtLaunch &lp, int grid)
{
    hipLaunchKernelGGL(invert_product_kernel, dim3(grid), dim3(TN_THREADS), 0, s, lp);
}

void launch_tn(hipStream_t s, const TnLaunch &lp, int grid, int tiles)
{
    hipLaunchKernelGGL(tn_gemm_kernel, dim3(grid), dim3(TN_THREADS), 0, s, lp);
    if (lp.c.splits > 1) hipLaunchKernelGGL(tn_reduce_kernel, dim3(tiles / lp.c.splits), dim3(TN_THREADS), 0, s, lp);
}

struct StreamEmitter : Emitter {
    hipStream_t s;
    explicit StreamEmitter(hipStream_t st) : s(st) {}
    void prep(const PrepLaunch &pl, int count, int grid_x) override { launch_prep(s, pl, count, grid_x); }
    void inv(const InvLaunch &lp, int grid, bool with_diag, double) override { launch_inv(s, lp, grid, with_diag); }
    void tn(const TnLaunch &lp, int grid, int tiles, double) override { launch_tn(s, lp, grid, tiles); }
    void wwt(const WwtLaunch &lp, int grid, double) override { launch_wwt(s, lp, grid); }
};

// One step of a recorded sequence: a kernel launch (with its helper launch, if it has one).
struct PlanStep {
    std::function<void(hipStream_t)> run;
    double flops;  // model cost: multiply-adds x 2 of the launch (0 for copies)
    const char *label;
};
typedef std::vector<PlanStep> PlanSteps;

struct RecordEmitter : Emitter {
    PlanSteps &steps;
    explicit RecordEmitter(PlanSteps &st) : steps(st) {}
    void prep(const PrepLaunch &pl, int count, int grid_x) override
    {
        steps.push_back(PlanStep{[pl, count, grid_x](hipStream_t s) { launch_prep(s, pl, count, grid_x); }, 0.0, label});
    }
    void inv(const InvLaunch &lp, int grid, bool with_diag, double flops) override
    {
        steps.push_back(PlanStep{[lp, grid, with_diag](hipStream_t s) { launch_inv(s, lp, grid, with_diag); }, flops, label});
    }
    void tn(const TnLaunch &lp, int grid, int tiles, double flops) override
    {
        steps.push_back(PlanStep{[lp, grid, tiles](hipStream_t s) { launch_tn(s, lp, grid, tiles); }, flops, label});
    }
    void wwt(const WwtLaunch &lp, int grid, double flops) override
    {
        steps.push_back(PlanStep{[lp, grid](hipStream_t s) { launch_wwt(s, lp, grid); }, flops, label});
    }
};

// Collects problems that share the launch parameters and sends them to the
// engine in chunks of at most TN_MAX_PROBLEMS.
struct TnBatch {
    std::vector<TnProblem> probs;
    int tile_mode = TILE_FULL, mask_a = MASK_NONE, mask_b = MASK_NONE, splits = 1;
    float alpha = 1.f, beta = 0.f;
    float *partial = nullptr;
    bool sort_by_k = false;  // the order of the problems is free: longest tiles first

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

    void launch(Emitter &em)
    {
        if (sort_by_k)
            std::stable_sort(probs.begin(), probs.end(), [](const TnProblem &a, const TnProblem &b) { return a.K > b.K; });
        size_t i = 0;
        while (i < probs.size()) {
            TnLaunch lp;
            std::memset(&lp, 0, sizeof(lp));
            int tiles = 0, cnt = 0;
            double fl = 0.0;
            while (i < probs.size() && cnt < TN_MAX_PROBLEMS) {
                lp.p[cnt] = probs[i];
                lp.p[cnt].tile_begin = tiles;
                tiles += tn_tiles(probs[i].M, probs[i].N, tile_mode) * splits;
                fl += tn_problem_flops(probs[i].M, probs[i].N, probs[i].K, tile_mode, mask_a, mask_b);
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
            const int grid = tn_map_xcds(lp, tiles);
            em.tn(lp, grid, tiles, fl);
        }
        probs.clear();
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
    size_t pack;    // bytes of the repacked bf16 inputs (bf16, and float32 split into bf16 terms), in front of the partial tiles
    size_t ws;
};

inline int pack_groups(int64_t n) { return (int)align_up((size_t)std::max<int64_t>(1, (n + 7) / 8), BF_SLAB_GROUPS); }
inline int pack_cols(int64_t d) { return (int)align_up((size_t)d, B2_TILE); }
inline size_t pack_bytes(int64_t n, int64_t d) { return align_up((size_t)pack_groups(n) * pack_cols(d) * 16, WS_ALIGN); }

// The three launches that turn float32 tensors into their two float16 planes (split2_syrk256.h): sp.it[0 .. count),
// sp.count and sp.amax are filled in by the caller.
kfac_status split2_prepass(hipStream_t st, Split2Launch &sp)
{
    int64_t wg_amax = 0, wg_pack = 0;
    int first_pack[PACK_MAX_ITEMS + 1];
    const int n = sp.count;
    for (int i = 0; i < n; ++i) {
        const Split2Item &si = sp.it[i];
        sp.first_wg[i] = (int)wg_amax;
        first_pack[i] = (int)wg_pack;
        wg_amax += (int64_t)(si.dp / S2P_COLS) * ((si.gp + S2A_GROUPS - 1) / S2A_GROUPS);
        wg_pack += (int64_t)(si.dp / S2P_COLS) * si.gp;
        if (wg_pack > INT32_MAX) return KFAC_ERR_UNSUPPORTED;  // more workgroups than a grid holds
    }
    sp.first_wg[n] = (int)wg_amax;
    first_pack[n] = (int)wg_pack;
    hipLaunchKernelGGL(split2_clear_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, sp.amax, n);
    hipLaunchKernelGGL(split2_amax_kernel, dim3((unsigned)wg_amax), dim3(256), 0, st, sp);
    std::memcpy(sp.first_wg, first_pack, sizeof(int) * (size_t)(n + 1));
    hipLaunchKernelGGL(split2_pack_kernel, dim3((unsigned)wg_pack), dim3(256), 0, st, sp);
    return hipGetLastError() == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
}

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
    if (dtype == KFAC_F32_BF16X3)
        for (int64_t i = 0; i < count; ++i) pl.pack += S3_PLANES * pack_bytes(items[i].n_tokens, items[i].d);
    if (dtype == KFAC_F32_F16X2) {
        pl.pack += align_up((size_t)count * sizeof(unsigned), WS_ALIGN);  // the largest magnitude of every item
        for (int64_t i = 0; i < count; ++i) pl.pack += S2_PLANES * pack_bytes(items[i].n_tokens, items[i].d);
    }
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
    unsigned f_off;  // offset of F in the workspace in 256-byte units
    float *inv;
    int ldi;
    int *info;
};

// A node of the inversion before it has a place in a launch.
struct NodeSpec {
    unsigned char mat, a, b, c, op, r0, rn;
};

constexpr int SUPER_PANEL = 4;  // block rows factored between two updates of the rest of the matrix (K = 512).
                                // Measured with 2, 3, 6, 8: 11.99, 11.37, 11.37, 11.37 ms against 11.21 for the
                                // BERT-Large stage; 16.6, 16.0, 16.8, 17.0 against 15.8 ms for the stress block.

// Builds the launch sequence of a batched inversion.
//
// The factorisation is a chain of short dependent launches (per block row: update the row, factor
// the diagonal block, solve the panel) that occupy a fraction of the chip.  Everything else - the
// update of the part of the matrix that the chain does not need yet, and the products of the
// triangular inverse, which only need block rows that are already final - is cut into tasks.  A task
// belongs to a group; a group may depend on other groups, and a task is placed in a launch only if
// every group it depends on was completed by earlier launches.  Tasks run
//   * in the launches of the chain that factor diagonal blocks (a few dozen workgroups, most of the chip free):
//     short tasks ride along there, as the second list of the engine's tile order;
//   * in launches of their own when a node of the chain needs a group (the rows a super-panel is about
//     to factor need every earlier update) or when the chain has ended: such a launch takes every
//     task that is ready, whatever its operation.
class InvScheduler {
public:
    InvScheduler(const std::vector<InvMat> &mats, float *ws, Emitter &em) : mats_(mats), ws_(ws), em_(em) {}

    int new_group(const std::vector<int> &deps)
    {
        groups_.push_back(Group{0, -1, deps});
        return (int)groups_.size() - 1;
    }

    // urgent: has a deadline inside the factorisation (deferred row updates); otherwise bulk work
    void push(const NodeSpec &n, int group, bool urgent)
    {
        Task t;
        t.n = n;
        t.group = group;
        shape(n, t.tiles, t.cost, t.flops, &t.longest);
        if (t.tiles == 0) return;
        groups_[(size_t)group].pending++;
        (urgent ? urgent_ : bulk_).push_back(t);
    }

    // One launch of the chain: its own nodes `crit` plus tasks that ride along.
    // fill_round: tasks whose tiles are no longer than the launch's own may take the slots that its last
    // round of workgroups leaves free
    bool launch(const std::vector<NodeSpec> &crit, bool with_diag, const char *label, bool fill_round = false)
    {
        label_ = label;
        size_t i = 0;
        do {
            // leave room for some tasks even when a launch has many nodes of its own
            const size_t n = std::min(crit.size() - i, (size_t)INV_MAX_NODES - 32);
            if (!emit(crit.data() + i, n, with_diag, false, fill_round)) return false;
            i += n;
        } while (i < crit.size());
        return true;
    }

    // Runs tasks until the groups are complete (needed when a node of the chain depends on them).
    bool finish_groups(const std::vector<int> &gs)
    {
        for (;;) {
            bool open = false;
            for (int g : gs)
                if (g >= 0 && groups_[(size_t)g].pending > 0) open = true;
            if (!open) return true;
            if (!emit(nullptr, 0, false, true, false)) return false;
        }
    }

    bool finish_all()
    {
        while (head_u_ < urgent_.size() || head_b_ < bulk_.size())
            if (!emit(nullptr, 0, false, true, false)) return false;
        return true;
    }

private:
    struct Task {
        NodeSpec n;
        int group, tiles, cost, longest = 0;  // longest: cost of its longest tile
        double flops;
        bool done = false;
    };
    struct Group {
        int pending, last_launch;
        std::vector<int> deps;
    };

    void shape(const NodeSpec &n, int &tiles, int &cost, double &flops, int *longest = nullptr) const
    {
        if (longest) *longest = 0;
        const InvMat &m = mats_[n.mat];
        const InvDims dm = inv_dims(n.op, m.d, n.a, n.b, n.c, n.r0, n.rn);
        tiles = cost = 0;
        flops = 0.0;
        if (dm.M <= 0 || dm.N <= 0) return;
        if (n.op == INV_DIAG) {
            const int ku = n.c ? ((int)n.a - (int)n.b) * NB : 0;  // rows of the update it applies to itself first
            tiles = 1;
            cost = INV_DIAG_COST + (ku ? ku / BK + 4 : 0);
            flops = 2.0 / 3.0 * dm.M * (double)dm.M * dm.M + (double)dm.M * dm.M * ku;
            return;
        }
        const TnAttr at = InvLaunch::op_attr(n.op);
        const int tm = (dm.M + BM - 1) / BM, tn = (dm.N + BN - 1) / BN;
        for (int ti = 0; ti < tm; ++ti)
            for (int tj = 0; tj < tn; ++tj) {
                int kb, nslab;
                tn_k_range(at, dm.K, ti * BM, tj * BN, kb, nslab);
                cost += nslab + 4;
                if (longest) *longest = std::max(*longest, nslab + 4);
            }
        tiles = tm * tn;
        flops = tn_problem_flops(dm.M, dm.N, dm.K, at.tile_mode, at.mask_a, at.mask_b);
    }

    bool ready(const Task &t) const
    {
        for (int g : groups_[(size_t)t.group].deps) {
            if (g < 0) continue;
            const Group &d = groups_[(size_t)g];
            if (d.pending > 0 || d.last_launch >= launch_idx_) return false;
        }
        return true;
    }

    // Takes ready tasks from a queue, in order, until `budget` tiles are taken or the launch is full.
    void take(std::vector<Task> &q, size_t &head, long long &budget, int longest_allowed, bool whole_tasks_only,
              InvLaunch &lp, int &cnt, int &tiles, double &flops)
    {
        constexpr size_t WINDOW = 2048;  // tasks looked at behind the first one that cannot go yet
        for (size_t i = head; i < q.size() && i < head + WINDOW && cnt < INV_MAX_NODES && budget > 0; ++i) {
            Task &t = q[i];
            if (t.done || t.longest > longest_allowed || (whole_tasks_only && t.tiles > budget) || !ready(t)) continue;
            add_node(lp, cnt, tiles, t.n, t.tiles);
            flops += t.flops;
            budget -= t.tiles;
            t.done = true;
            Group &g = groups_[(size_t)t.group];
            g.pending--;
            g.last_launch = launch_idx_;
        }
        while (head < q.size() && q[head].done) ++head;
    }

    static void add_node(InvLaunch &lp, int &cnt, int &tiles, const NodeSpec &n, int ntiles)
    {
        InvNode &o = lp.n[cnt++];
        o.mat = n.mat; o.a = n.a; o.b = n.b; o.c = n.c; o.op = n.op; o.r0 = n.r0; o.rn = n.rn; o.pad_ = 0;
        o.tile_begin = tiles;
        tiles += ntiles;
    }

    bool emit(const NodeSpec *crit, size_t ncrit, bool with_diag, bool drain, bool fill_round)
    {
        InvLaunch lp;
        std::memset(&lp, 0, sizeof(lp));
        for (size_t k = 0; k < mats_.size(); ++k) {
            lp.m[k].info = mats_[k].info;
            lp.m[k].f_off = mats_[k].f_off;
            lp.m[k].d = (unsigned short)mats_[k].d;
            lp.m[k].ld = (unsigned short)mats_[k].ld;
        }
        lp.ws = ws_;
        int cnt = 0, tiles = 0;
        double flops = 0.0;
        int own_longest = 0;
        for (size_t i = 0; i < ncrit; ++i) {
            int t, c;
            double f;
            shape(crit[i], t, c, f);
            if (t == 0) continue;
            add_node(lp, cnt, tiles, crit[i], t);
            flops += f;
            own_longest = std::max(own_longest, c / t);
        }
        const int first_tiles = tiles;
        // Which tasks ride along.  A launch that only drains the queues takes everything that is ready.  A
        // launch with diagonal blocks keeps a dozen to 72 workgroups busy for about 40 us (longer when they
        // first update their own tile): tiles of up to that length fill the other workgroup slots of the chip
        // (two per CU), less those of the launch's own row-update tiles.  Measured on the BERT-Large stage /
        // the stress block: 192 riders 11.42 / 16.0 ms, 288: 11.53 / 16.2, 384: 11.42 / 15.9, 480: 11.24 /
        // 15.75, 640 to 1024: 11.22 - 11.36 / 16.0; 480 riders of up to 72 slabs: 11.3 / 15.65, of up to 28:
        // 11.6 / 16.7; riders as long as the launch's own diagonal-block nodes (which take 52 to 68 slab times when
        // they first update their tile): +0.05 / -0.28 ms.  The panel solves take nothing along: they are shorter than any task, and measured
        // with riders they lost as much time as the riders would have taken alone.
        constexpr int RIDER_TILES = TARGET_TILES - 32;
        long long budget = drain ? (1 << 20) : (with_diag ? std::max(0, RIDER_TILES - first_tiles) : 0);
        // a launch of equal tiles runs in rounds of TARGET_TILES workgroups: what the last round leaves free
        // (less one tile per XCD: the eight XCDs take their shares separately)
        if (fill_round && first_tiles > 0)
            budget = std::max(0, (first_tiles + TARGET_TILES - 1) / TARGET_TILES * TARGET_TILES - first_tiles - 8);
        const int longest_allowed = drain ? (1 << 30) : (fill_round ? own_longest : INV_DIAG_COST);
        take(urgent_, head_u_, budget, longest_allowed, fill_round, lp, cnt, tiles, flops);
        take(bulk_, head_b_, budget, longest_allowed, fill_round, lp, cnt, tiles, flops);
        if (cnt == 0) return !drain;  // draining with nothing that can run: a dependency cycle (cannot happen)
        lp.c.count = cnt;
        lp.c.splits = 1;
        if (!in_bounds(lp, cnt)) return false;
        const int grid = tn_balance_xcds(lp, tiles, first_tiles);
        em_.label = drain ? "tasks: deferred row updates and products of the triangular inverse"
                          : (tiles > first_tiles && with_diag ? "diagonal blocks + tasks riding along" : label_);
        em_.inv(lp, grid, with_diag, flops);
        ++launch_idx_;
        return true;
    }

    // Every operand of every node must lie inside the working arrays of its matrix: checked on the
    // host, with the same descriptor arithmetic the kernel uses, before anything is launched.
    bool in_bounds(const InvLaunch &lp, int cnt) const
    {
        for (int i = 0; i < cnt; ++i) {
            const InvNode &nd = lp.n[i];
            if (nd.mat >= mats_.size()) return false;
            const InvMat &m = mats_[nd.mat];
            if (lp.mat_f(nd.mat) != m.F || lp.mat_s(nd.mat) != m.S) return false;
            const TnProblem pr = lp.problem(i);
            auto inside = [&](const float *p, int rows, int cols) {
                if (p == nullptr) return true;
                const float *base = p >= m.S ? m.S : m.F;
                if (p < base) return false;
                const size_t off = (size_t)(p - base), r = off / (size_t)m.ld, c = off % (size_t)m.ld;
                return r + (size_t)rows <= (size_t)m.d && c + (size_t)cols <= (size_t)m.d;
            };
            bool ok;
            if (nd.op == INV_DIAG) {
                ok = (int)nd.a < m.nblk && (nd.c == 0 || nd.b < nd.a);
                if (ok && nd.c != 0) {
                    const TnProblem up = lp.diag_update(i);
                    ok = inside(up.A, up.K, up.M) && inside(up.C, up.M, up.N);
                }
            }
            else
                ok = inside(pr.A, pr.K, pr.M) && inside(pr.B, pr.K, pr.N) && inside(pr.C, pr.M, pr.N) && inside(pr.Ct, pr.N, pr.M);
            if (!ok) return false;
        }
        return true;
    }

    const std::vector<InvMat> &mats_;
    float *ws_;
    Emitter &em_;
    const char *label_ = "";
    std::vector<Group> groups_;
    std::vector<Task> urgent_, bulk_;
    size_t head_u_ = 0, head_b_ = 0;
    int launch_idx_ = 0;
};

// Balanced splitting of the block range [lo, hi) for the triangular inverse.
struct TriNode {
    int lo, mid, hi;
    int left, right;   // children (-1: a single block, inverted by the diagonal-block node)
    int g_y = -1, g_w = -1;  // groups of its two products
};

int build_tree(int lo, int hi, std::vector<TriNode> &nodes)
{
    if (hi - lo <= 1) return -1;
    const int mid = lo + (hi - lo + 1) / 2;
    const int l = build_tree(lo, mid, nodes);
    const int r = build_tree(mid, hi, nodes);
    nodes.push_back(TriNode{lo, mid, hi, l, r});
    return (int)nodes.size() - 1;  // children come before their parent
}

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
    return kfac_mfma_probe_data(dtype, 0, iters, sink, flops, stream);
}

kfac_status kfac_mfma_probe_data(kfac_dtype dtype, int random_operands, int64_t iters, void *sink, double *flops, void *stream)
{
    if (sink == nullptr || flops == nullptr || iters <= 0 || iters > INT32_MAX) return KFAC_ERR_ARG;
    if (dtype != KFAC_F32 && dtype != KFAC_BF16) return KFAC_ERR_ARG;
    constexpr int WORKGROUPS = 256 * 2 * 8;  // eight rounds of two workgroups per CU
    hipStream_t st = static_cast<hipStream_t>(stream);
    const double per_mfma = dtype == KFAC_F32 ? 4096.0 : 32768.0;
    if (random_operands) {
        const int outer = (int)((iters + PROBE_SETS - 1) / PROBE_SETS);  // every pass of the loop takes all operand sets
        *flops = (double)WORKGROUPS * 4.0 * (double)outer * PROBE_SETS * PROBE_MFMA_PER_ITER * per_mfma;
        if (dtype == KFAC_F32)
            hipLaunchKernelGGL(mfma_probe_f32_random_kernel, dim3(WORKGROUPS), dim3(256), 0, st, outer, static_cast<float *>(sink));
        else
            hipLaunchKernelGGL(mfma_probe_bf16_random_kernel, dim3(WORKGROUPS), dim3(256), 0, st, outer, static_cast<float *>(sink));
        return hipGetLastError() == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
    }
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
    if (dtype != KFAC_F32 && dtype != KFAC_BF16 && dtype != KFAC_F32_BF16X3 && dtype != KFAC_F32_F16X2) return KFAC_ERR_ARG;
    for (int64_t i = 0; i < count; ++i) {
        const kfac_curvature_item &it = items[i];
        if (it.x == nullptr || it.factor == nullptr) return KFAC_ERR_ARG;
        if (!fits_int(it.d) || !fits_int(it.n_tokens)) return KFAC_ERR_ARG;
        if (it.ldx < it.d || it.ldf < it.d || !fits_int(it.ldx) || !fits_int(it.ldf)) return KFAC_ERR_ARG;
        if ((reinterpret_cast<uintptr_t>(it.x) & (dtype == KFAC_BF16 ? 1 : 3)) || (reinterpret_cast<uintptr_t>(it.factor) & 3))
            return KFAC_ERR_ARG;
    }
    if (dtype != KFAC_F32)
        for (int64_t i = 0; i < count; ++i)
            if (items[i].d > (1 << 26)) return KFAC_ERR_UNSUPPORTED;  // packed rows are addressed with 32-bit byte offsets
    CurvPlan pl;
    if (!curvature_plan(items, count, dtype, pl)) return KFAC_ERR_ARG;
    if (!ws_ok(workspace, workspace_bytes, pl.ws)) return KFAC_ERR_WORKSPACE;

    // One launch per SYRK_MAX_PROBLEMS items (a BERT-Large stage has 72 factors:
    // one launch per micro-batch); each launch gets its own slice of the partial buffer.
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *pack = static_cast<char *>(workspace);
    unsigned *amax = reinterpret_cast<unsigned *>(workspace);  // KFAC_F32_F16X2: one word per item, in front of the planes
    if (dtype == KFAC_F32_F16X2) pack += align_up((size_t)count * sizeof(unsigned), WS_ALIGN);
    float *part = reinterpret_cast<float *>(static_cast<char *>(workspace) + pl.pack);
    for (int64_t done = 0; done < count;) {
        const int64_t n = std::min<int64_t>(SYRK_MAX_PROBLEMS, count - done);
        SyrkLaunch lp;
        std::memset(&lp, 0, sizeof(lp));
        PackLaunch pk;
        if (dtype == KFAC_BF16) std::memset(&pk, 0, sizeof(pk));
        int tiles256_f32 = 0;
        if (dtype == KFAC_F32_BF16X3 || dtype == KFAC_F32_F16X2)
            for (int64_t i = 0; i < n; ++i) tiles256_f32 += b2_tiles((int)items[done + i].d);
        if (dtype == KFAC_F32_F16X2 && tiles256_f32 >= 192) {
            // float32 input as two float16 terms on the f16 MFMA (split2_syrk256.h); launches too small to occupy
            // the chip with 256 x 256 tiles take the fp32 path below
            Split2Launch sp;
            Syrk256LaunchScaled ls;
            std::memset(&sp, 0, sizeof(sp));
            std::memset(&ls, 0, sizeof(ls));
            for (int64_t i = 0; i < n; ++i) {
                const kfac_curvature_item &it = items[done + i];
                Split2Item &si = sp.it[i];
                si.x = static_cast<const float *>(it.x);
                si.dst = reinterpret_cast<unsigned short *>(pack);
                si.n = (int)it.n_tokens;
                si.d = (int)it.d;
                si.ldx = (int)it.ldx;
                si.dp = pack_cols(it.d);
                si.gp = pack_groups(it.n_tokens);
                pack += S2_PLANES * pack_bytes(it.n_tokens, it.d);
            }
            sp.count = (int)n;
            sp.amax = amax + done;
            const kfac_status pre = split2_prepass(st, sp);
            if (pre != KFAC_OK) return pre;
            // chunks of S3_CHUNK_GROUPS k-groups, as for the three-term split below
            int gmax2 = 0;
            for (int64_t i = 0; i < n; ++i) gmax2 = std::max(gmax2, sp.it[i].gp);
            for (int g0 = 0; g0 < gmax2; g0 += S3_CHUNK_GROUPS) {
                int cnt = 0, tb = 0;
                for (int64_t i = 0; i < n; ++i) {
                    const Split2Item &si = sp.it[i];
                    if (si.gp <= g0) continue;  // this item's tokens are used up
                    ls.amax_index[cnt] = (int)i;
                    SyrkProblem &q = ls.l.p[cnt++];
                    q.x = reinterpret_cast<const char *>(si.dst) + (size_t)g0 * si.dp * 16;
                    q.factor = items[done + i].factor;
                    q.n = std::min(S3_CHUNK_GROUPS, si.gp - g0) * BF_KG;
                    q.d = si.d;
                    q.ldx = si.dp;
                    q.ldf = (int)items[done + i].ldf;
                    q.pad_ = si.gp;  // k-groups of a whole plane: the planes are that far apart
                    q.tile_begin = tb;
                    tb += b2_tiles(si.d);
                }
                ls.l.count = cnt;
                ls.l.alpha = alpha;
                ls.l.beta = g0 == 0 ? beta : 1.f;
                ls.amax = sp.amax;
                hipLaunchKernelGGL(curvature_syrk_split2_256_kernel, dim3(tb), dim3(256), 0, st, ls);
            }
            if (hipGetLastError() != hipSuccess) return KFAC_ERR_HIP;
            done += n;
            continue;
        }
        if (dtype == KFAC_F32_BF16X3 && tiles256_f32 >= 192) {
            // float32 input as three bfloat16 terms on the bf16 MFMA (split3_syrk256.h); launches too small to
            // occupy the chip with 256 x 256 tiles take the fp32 path below
            Split3Launch sp;
            Syrk256Launch l2;
            std::memset(&sp, 0, sizeof(sp));
            std::memset(&l2, 0, sizeof(l2));
            int tb = 0;
            int64_t wgs = 0;
            for (int64_t i = 0; i < n; ++i) {
                const kfac_curvature_item &it = items[done + i];
                Split3Item &si = sp.it[i];
                si.x = static_cast<const float *>(it.x);
                si.dst = reinterpret_cast<unsigned short *>(pack);
                si.n = (int)it.n_tokens;
                si.d = (int)it.d;
                si.ldx = (int)it.ldx;
                si.dp = pack_cols(it.d);
                si.gp = pack_groups(it.n_tokens);
                SyrkProblem &q = l2.p[i];
                q.x = pack;
                q.factor = it.factor;
                q.n = si.gp * BF_KG;
                q.d = si.d;
                q.ldx = si.dp;
                q.ldf = (int)it.ldf;
                q.tile_begin = tb;
                tb += b2_tiles(si.d);
                pack += S3_PLANES * pack_bytes(it.n_tokens, it.d);
                sp.first_wg[i] = (int)wgs;
                wgs += (int64_t)(si.dp / S3P_COLS) * (si.gp / S3P_GROUPS);
                if (wgs > INT32_MAX) return KFAC_ERR_UNSUPPORTED;  // more workgroups than a grid holds
            }
            sp.first_wg[n] = (int)wgs;
            sp.count = (int)n;
            hipLaunchKernelGGL(split3_pack_kernel, dim3((unsigned)wgs), dim3(256), 0, st, sp);
            // The MFMA kernel keeps one fp32 accumulation level, whose rounding error grows with the square
            // root of the tokens: long inputs go in chunks of S3_CHUNK_GROUPS k-groups, each chunk added to the
            // factor by its epilogue (the first with the caller's beta, the others with 1).
            int gmax3 = 0;
            for (int64_t i = 0; i < n; ++i) gmax3 = std::max(gmax3, sp.it[i].gp);
            for (int g0 = 0; g0 < gmax3; g0 += S3_CHUNK_GROUPS) {
                Syrk256Launch lc;
                std::memset(&lc, 0, sizeof(lc));
                int cnt = 0;
                tb = 0;
                for (int64_t i = 0; i < n; ++i) {
                    const Split3Item &si = sp.it[i];
                    if (si.gp <= g0) continue;  // this item's tokens are used up
                    SyrkProblem &q = lc.p[cnt++];
                    q = l2.p[i];
                    q.x = static_cast<const char *>(l2.p[i].x) + (size_t)g0 * si.dp * 16;
                    q.n = std::min(S3_CHUNK_GROUPS, si.gp - g0) * BF_KG;
                    q.pad_ = si.gp;  // k-groups of a whole plane: the planes are that far apart
                    q.tile_begin = tb;
                    tb += b2_tiles(si.d);
                }
                lc.count = cnt;
                lc.alpha = alpha;
                lc.beta = g0 == 0 ? beta : 1.f;
                hipLaunchKernelGGL(curvature_syrk_split3_256_kernel, dim3(tb), dim3(256), 0, st, lc);
            }
            if (hipGetLastError() != hipSuccess) return KFAC_ERR_HIP;
            done += n;
            continue;
        }
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

// Validates the arguments and sends the launch sequence of a batched inversion to `em`.
kfac_status invert_emit(const kfac_invert_item *items, int64_t count, float damping,
                        void *workspace, size_t workspace_bytes, Emitter &em)
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
            const kfac_status stt = invert_emit(items + i0, n, damping, base, bytes, em);
            if (stt != KFAC_OK) return stt;
            base += bytes;
        }
        return KFAC_OK;
    }

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
        m.f_off = (unsigned)((size_t)(cur - static_cast<char *>(workspace)) / WS_ALIGN);
        cur += 2 * one;
        m.nblk = (m.d + NB - 1) / NB;
        m.inv = items[i].inv;
        m.ldi = (int)items[i].ldi;
        m.info = items[i].info_dev;
        max_blk = std::max(max_blk, m.nblk);
    }
    if ((size_t)(cur - static_cast<char *>(workspace)) / WS_ALIGN > 0xFFFFFFFFull) return KFAC_ERR_UNSUPPORTED;

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
        em.label = "copy + damping";
        em.prep(pl, (int)n, std::min(dmax, 512));
    }

    // 2. Blocked upper Cholesky M = U^T U with panel width NB, all matrices advanced together, and
    //    W = U^-1 by pairwise merging of inverted diagonal ranges,
    //        [U11 U12; 0 U22]^-1 = [W11, -W11 U12 W22; 0, W22],
    //    interleaved: see InvScheduler.
    //    Chain, per super-panel of SUPER_PANEL block rows [s0, e): for each row j, bring it up to date
    //    with the rows s0..j-1 of the super-panel, factor its diagonal block, solve its panel.  After
    //    the super-panel the next SUPER_PANEL block rows are updated with it at once (they are
    //    factored next); the rows below are updated by tasks that ride along in later launches.
    //    A product of the triangular inverse becomes a task as soon as the block rows it reads are
    //    final: Y^T = (W11 U12)^T when the rows of the first part are, W12 = -Y W22 when all are.
    InvScheduler sch(mats, static_cast<float *>(workspace), em);
    std::vector<std::vector<TriNode>> trees(mats.size());
    for (size_t mi = 0; mi < mats.size(); ++mi) build_tree(0, mats[mi].nblk, trees[mi]);
    // group of the latest deferred update of block row i of matrix mi (-1: none)
    std::vector<std::vector<int>> row_group(mats.size());
    for (size_t mi = 0; mi < mats.size(); ++mi) row_group[mi].assign((size_t)mats[mi].nblk, -1);
    constexpr int MERGE_TASK_TILES = 64;  // a product is cut into tasks of about this many tiles

    auto push_product = [&](size_t mi, TriNode &t, int op) {
        const InvMat &m = mats[mi];
        const int b1 = (t.mid - t.lo) * NB, c1 = t.mid * NB, b2 = std::min((t.hi - t.mid) * NB, m.d - c1);
        std::vector<int> deps;
        int rows, cols;
        if (op == INV_MERGE_YT) {
            deps.push_back(t.left >= 0 ? trees[mi][(size_t)t.left].g_w : -1);
            rows = b2; cols = b1;
        } else {
            deps.push_back(t.g_y);
            deps.push_back(t.right >= 0 ? trees[mi][(size_t)t.right].g_w : -1);
            rows = b1; cols = b2;
        }
        const int g = sch.new_group(deps);
        (op == INV_MERGE_YT ? t.g_y : t.g_w) = g;
        const int tr = (rows + NB - 1) / NB, tc = (cols + NB - 1) / NB;
        const int step = std::max(1, MERGE_TASK_TILES / std::max(1, tc));
        for (int r0 = 0; r0 < tr; r0 += step) {
            NodeSpec n{(unsigned char)mi, (unsigned char)t.lo, (unsigned char)(t.mid - t.lo), (unsigned char)(t.hi - t.mid),
                       (unsigned char)op, (unsigned char)r0, (unsigned char)std::min(step, tr - r0)};
            sch.push(n, g, false);
        }
    };

    std::vector<NodeSpec> crit;
    std::vector<int> wait;
    for (int s0 = 0; s0 < max_blk; s0 += SUPER_PANEL) {
        const int e = std::min(s0 + SUPER_PANEL, max_blk);
        for (int j = s0; j < e; ++j) {
            // One launch brings block row j up to date with the rows s0..j-1 of the super-panel and factors
            // its diagonal block: the workgroup of the diagonal block updates that tile itself and goes
            // straight on, the other tiles of the row are finished next to it (the panel solve, which
            // needs both, is the next launch).
            crit.clear();
            for (size_t mi = 0; mi < mats.size(); ++mi)
                if (j < mats[mi].nblk)
                    crit.push_back(NodeSpec{(unsigned char)mi, (unsigned char)j, (unsigned char)s0, (unsigned char)(j > s0 ? 1 : 0), INV_DIAG, 0, 0});
            if (j > s0)
                for (size_t mi = 0; mi < mats.size(); ++mi)
                    if (j + 1 < mats[mi].nblk)
                        crit.push_back(NodeSpec{(unsigned char)mi, (unsigned char)s0, (unsigned char)j, (unsigned char)j, INV_ROW_UPDATE, 1, 0});
            if (!crit.empty() && !sch.launch(crit, true, j > s0 ? "diagonal blocks with the update of their block row" : "diagonal blocks"))
                return KFAC_ERR_HIP;
            // W_jj is there: second products of the tree nodes that end with block j, smallest first
            for (size_t mi = 0; mi < mats.size(); ++mi)
                for (TriNode &t : trees[mi])
                    if (t.hi - 1 == j) push_product(mi, t, INV_MERGE_W);
            crit.clear();
            for (size_t mi = 0; mi < mats.size(); ++mi)
                if (j + 1 < mats[mi].nblk) crit.push_back(NodeSpec{(unsigned char)mi, (unsigned char)j, 0, 0, INV_PANEL_SOLVE, 0, 0});
            if (!crit.empty() && !sch.launch(crit, false, "panel solve")) return KFAC_ERR_HIP;
            // block row j of U is final: first products of the tree nodes whose first part ends with it
            for (size_t mi = 0; mi < mats.size(); ++mi)
                for (TriNode &t : trees[mi])
                    if (t.mid - 1 == j) push_product(mi, t, INV_MERGE_YT);
        }
        // the rows factored next take the update with this super-panel now ...
        crit.clear();
        wait.clear();
        for (size_t mi = 0; mi < mats.size(); ++mi)
            for (int i = e; i < std::min(e + SUPER_PANEL, mats[mi].nblk); ++i) {
                crit.push_back(NodeSpec{(unsigned char)mi, (unsigned char)s0, (unsigned char)i, (unsigned char)e, INV_ROW_UPDATE, 0, 0});
                wait.push_back(row_group[mi][(size_t)i]);  // after their earlier deferred updates
            }
        if (!sch.finish_groups(wait)) return KFAC_ERR_HIP;
        // ... the rows below as tasks, each after the previous update of the same row; as many of them as
        // the last round of the launch above leaves room for go with it (their tiles are the same)
        for (size_t mi = 0; mi < mats.size(); ++mi)
            for (int i = e + SUPER_PANEL; i < mats[mi].nblk; ++i) {
                const int g = sch.new_group(std::vector<int>{row_group[mi][(size_t)i]});
                sch.push(NodeSpec{(unsigned char)mi, (unsigned char)s0, (unsigned char)i, (unsigned char)e, INV_ROW_UPDATE, 0, 0}, g, true);
                row_group[mi][(size_t)i] = g;
            }
        if (!crit.empty() && !sch.launch(crit, false, "update of the next super-panel's rows", true)) return KFAC_ERR_HIP;
    }
    if (!sch.finish_all()) return KFAC_ERR_HIP;

    // 3. inv = W W^T = (W^T)^T (W^T): inv[i][j] = sum_{k >= max(i,j)} F[k][i] F[k][j], W^T read from the diagonal
    //    blocks of F and below (zeros above the diagonal inside them: the product only clips its K ranges).
    // One launch for the whole batch (more only when it has more than WWT_MAX_NODES bands): a node is a band of
    // eight tile rows of one matrix; the bands go by decreasing length of their tiles (the first band of every
    // large matrix, then the second ones, ..., the small matrices last).
    struct Band {
        unsigned short mat, band;
        int tiles, longest;
        double flops;
    };
    std::vector<Band> bands;
    for (size_t mi = 0; mi < mats.size(); ++mi) {
        const InvMat &m = mats[mi];
        const int nt = (m.d + BM - 1) / BM;
        for (int b = 0; b * SUPER_ROWS < nt; ++b) {
            const int first = wwt_band_first_tile(b, nt), next = wwt_band_first_tile(b + 1, nt);
            const int k0 = b * SUPER_ROWS * BM;  // the K range of the band's tiles starts at their row, at k0 or later
            // useful flops of the band's rows [k0, k1): sum over rows i of 2 (i + 1) (d - i)
            const double r0 = k0, r1 = std::min(m.d, (b + 1) * SUPER_ROWS * BM), dd = m.d;
            const double s1 = ((r1 - 1) * r1 - (r0 - 1) * r0) / 2;                                    // sum of i
            const double s2 = ((r1 - 1) * r1 * (2 * r1 - 1) - (r0 - 1) * r0 * (2 * r0 - 1)) / 6;      // sum of i^2
            const double fl = 2.0 * ((dd - 1) * s1 - s2 + dd * (r1 - r0));
            bands.push_back(Band{(unsigned short)mi, (unsigned short)b, next - first, (m.d - k0 + BK - 1) / BK, fl});
        }
    }
    std::stable_sort(bands.begin(), bands.end(), [](const Band &x, const Band &y) { return x.longest > y.longest; });
    em.label = "inverse = W W^T";
    for (size_t i0 = 0; i0 < bands.size(); i0 += WWT_MAX_NODES) {
        const size_t n = std::min<size_t>(WWT_MAX_NODES, bands.size() - i0);
        WwtLaunch lw;
        std::memset(&lw, 0, sizeof(lw));
        for (size_t mi = 0; mi < mats.size(); ++mi) {
            lw.m[mi].inv = mats[mi].inv;
            lw.m[mi].info = mats[mi].info;
            lw.m[mi].f_off = mats[mi].f_off;
            lw.m[mi].d = (unsigned short)mats[mi].d;
            lw.m[mi].ld = (unsigned short)mats[mi].ld;
            lw.m[mi].ldi = mats[mi].ldi;
        }
        lw.ws = static_cast<float *>(workspace);
        int tiles = 0;
        double fl = 0.0;
        for (size_t i = 0; i < n; ++i) {
            lw.n[i].mat = bands[i0 + i].mat;
            lw.n[i].band = bands[i0 + i].band;
            lw.n[i].tile_begin = tiles;
            tiles += bands[i0 + i].tiles;
            fl += bands[i0 + i].flops;
        }
        lw.c.count = (int)n;
        lw.c.tile_mode = TILE_LOWER;
        lw.c.mask_a = MASK_ZEROS_K_LT;
        lw.c.mask_b = MASK_ZEROS_K_LT;
        lw.c.splits = 1;
        lw.c.alpha = 1.f;
        lw.c.beta = 0.f;
        const int grid = tn_map_xcds(lw, tiles);
        em.wwt(lw, grid, fl);
    }
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
    if (count == 0) return KFAC_OK;
    StreamEmitter em(static_cast<hipStream_t>(stream));
    const kfac_status st = invert_emit(items, count, damping, workspace, workspace_bytes, em);
    if (st != KFAC_OK) return st;
    return hipGetLastError() == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
}

kfac_status kfac_invert_plan_create(const kfac_invert_item *items, int64_t count, float damping,
                                    void *workspace, size_t workspace_bytes, kfac_invert_plan **plan)
{
    if (plan == nullptr) return KFAC_ERR_ARG;
    *plan = nullptr;
    kfac_invert_plan *p = new (std::nothrow) kfac_invert_plan();
    if (p == nullptr) return KFAC_ERR_ARG;
    RecordEmitter em(p->steps);
    const kfac_status st = invert_emit(items, count, damping, workspace, workspace_bytes, em);
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

const char *kfac_invert_plan_step_label(const kfac_invert_plan *plan, int64_t step)
{
    if (plan == nullptr || step < 0 || step >= (int64_t)plan->steps.size()) return nullptr;
    return plan->steps[(size_t)step].label;
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

// ------------------------------------------- inversion without a workspace argument

// Scratch of kfac_invert_noalloc: the two working arrays of one inversion of up to NOALLOC_MAX_D rows.
// The array lives in the code object, so every GPU that loads the library holds its own copy at its
// own address until the process ends.  The name below is only a host-side handle: the device address
// comes from hipGetSymbolAddress, once per device, and only that pointer is handed to kernels.
constexpr int64_t NOALLOC_MAX_D = 2048;
constexpr size_t NOALLOC_SCRATCH_BYTES = 2 * (size_t)NOALLOC_MAX_D * NOALLOC_MAX_D * sizeof(float);  // 32 MiB
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex scratch_mutex;
void *scratch_ptr[NOALLOC_MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up on the first call for that device).
void *scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= NOALLOC_MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        scratch_ptr[dev] = p;
    }
    return scratch_ptr[dev];
}

}  // namespace

int64_t kfac_invert_noalloc_max_d(void) { return NOALLOC_MAX_D; }

kfac_status kfac_invert_noalloc(const float *factor, int64_t d, int64_t ldf, float damping,
                                float *inv, int64_t ldi, int32_t *info_dev, void *stream)
{
    if (d > NOALLOC_MAX_D) return KFAC_ERR_UNSUPPORTED;
    if (d > 0 && invert_item_bytes(d) > NOALLOC_SCRATCH_BYTES) return KFAC_ERR_UNSUPPORTED;
    void *ws = scratch_of_current_device();
    if (ws == nullptr) return KFAC_ERR_HIP;
    // Every kernel of the inversion writes what it later reads (working copy, factor, inverse factor),
    // so nothing of the previous call's contents has to be cleared.
    return kfac_invert(factor, d, ldf, damping, inv, ldi, info_dev, ws, NOALLOC_SCRATCH_BYTES, stream);
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
    StreamEmitter em(static_cast<hipStream_t>(stream));
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
            b.sort_by_k = true;
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
            b.launch(em);
            if (hipGetLastError() != hipSuccess) return KFAC_ERR_HIP;
            done += n;
        }
    }
    return KFAC_OK;
}

// The two-float16-term precondition.  Two memory regions: the *prepared inverses* (one word per inverse for its
// largest magnitude, two per layer, then the float16 planes of B^-1 and A^-1 of every layer) and the *workspace*
// (one word per layer for G and one for T^T, T^T in float32, then the planes of G and T^T).  The inverses only
// change when they are refreshed, so a caller may prepare them once and precondition many gradients with them
// (kfac_precondition_f16x2_prepare / kfac_precondition_grouped_f16x2_prepared); kfac_precondition_grouped_f16x2
// does both in one call, with the prepared region in front of its workspace.
namespace {
struct PrecSplitPlan {
    size_t prep_amax, prep_bytes;        // prepared inverses
    size_t ws_amax, t_bytes, ws_bytes;   // workspace of a run on prepared inverses
};
inline size_t planes2_bytes(int64_t rows, int64_t cols) { return S2_PLANES * pack_bytes(rows, cols); }
constexpr int64_t PREC_SPLIT_GROUP = PACK_MAX_ITEMS / 2;  // layers per group of launches: 80 operands per pre-pass
static_assert(PREC_SPLIT_GROUP <= GEMM2_MAX_PROBLEMS, "a group of layers is one launch of the product kernel");

bool precondition_split_plan(const kfac_precondition_item *items, int64_t count, PrecSplitPlan &pl)
{
    pl.prep_amax = pl.ws_amax = align_up((size_t)count * 2 * sizeof(unsigned), WS_ALIGN);
    pl.t_bytes = 0;
    size_t inv_planes = 0, run_planes = 0;
    for (int64_t i = 0; i < count; ++i) {
        const int64_t dout = items[i].d_out, din = items[i].d_in;
        if (!fits_int(dout) || !fits_int(din) || dout <= 0 || din <= 0) return false;
        pl.t_bytes += align_up((size_t)din * dout * sizeof(float), WS_ALIGN);
        inv_planes += planes2_bytes(dout, dout) + planes2_bytes(din, din);
        run_planes += planes2_bytes(dout, din) + planes2_bytes(din, dout);
    }
    pl.prep_bytes = pl.prep_amax + inv_planes;
    pl.ws_bytes = pl.ws_amax + pl.t_bytes + run_planes;
    return true;
}

kfac_status precondition_split_check(const kfac_precondition_item *items, int64_t count, bool need_grad)
{
    if (items == nullptr || count < 0) return KFAC_ERR_ARG;
    for (int64_t i = 0; i < count; ++i) {
        const kfac_precondition_item &it = items[i];
        if (!it.b_inv || !it.a_inv) return KFAC_ERR_ARG;
        if (need_grad && (!it.grad || !it.out)) return KFAC_ERR_ARG;
        if (!fits_int(it.d_out) || !fits_int(it.d_in) || it.d_out <= 0 || it.d_in <= 0) return KFAC_ERR_ARG;
        if (it.ldb < it.d_out || it.lda < it.d_in || !fits_int(it.ldb) || !fits_int(it.lda)) return KFAC_ERR_ARG;
        if (need_grad && (it.ldg < it.d_in || it.ldo < it.d_in || !fits_int(it.ldg) || !fits_int(it.ldo))) return KFAC_ERR_ARG;
        if ((reinterpret_cast<uintptr_t>(it.b_inv) & 3) || (reinterpret_cast<uintptr_t>(it.a_inv) & 3)) return KFAC_ERR_ARG;
        if (need_grad && ((reinterpret_cast<uintptr_t>(it.grad) & 3) || (reinterpret_cast<uintptr_t>(it.out) & 3)))
            return KFAC_ERR_ARG;
        if (it.d_out > (1 << 26) || it.d_in > (1 << 26)) return KFAC_ERR_UNSUPPORTED;  // 32-bit byte offsets in packed rows
    }
    return KFAC_OK;
}

inline void split2_item(Split2Item &si, const float *x, int64_t rows, int64_t cols, int64_t ld, char *dst)
{
    si.x = x;
    si.dst = reinterpret_cast<unsigned short *>(dst);
    si.n = (int)rows;
    si.d = (int)cols;
    si.ldx = (int)ld;
    si.dp = pack_cols(cols);
    si.gp = pack_groups(rows);
}

// Problems by decreasing K (stable), tile ranges renumbered: see gemm2_tile_of.
void gemm2_order(Gemm2Launch &gl)
{
    std::stable_sort(gl.p, gl.p + gl.count, [](const Gemm2Problem &a, const Gemm2Problem &b) { return a.groups > b.groups; });
    int tiles = 0;
    for (int i = 0; i < gl.count; ++i) {
        gl.p[i].tile_begin = tiles;
        tiles += gemm2_tiles(gl.p[i].m, gl.p[i].n);
    }
    gl.total_tiles = tiles;
}

// Largest magnitudes and planes of B^-1 (word 2 i) and A^-1 (word 2 i + 1) of every layer.
kfac_status precondition_split_prepare(const kfac_precondition_item *items, int64_t count, const PrecSplitPlan &pl,
                                       void *prepared, hipStream_t st)
{
    unsigned *amax = static_cast<unsigned *>(prepared);
    char *pcur = static_cast<char *>(prepared) + pl.prep_amax;
    for (int64_t done = 0; done < count; done += PREC_SPLIT_GROUP) {
        const int n = (int)std::min<int64_t>(PREC_SPLIT_GROUP, count - done);
        Split2Launch sp;
        std::memset(&sp, 0, sizeof(sp));
        for (int i = 0; i < n; ++i) {
            const kfac_precondition_item &it = items[done + i];
            split2_item(sp.it[2 * i], it.b_inv, it.d_out, it.d_out, it.ldb, pcur);
            pcur += planes2_bytes(it.d_out, it.d_out);
            split2_item(sp.it[2 * i + 1], it.a_inv, it.d_in, it.d_in, it.lda, pcur);
            pcur += planes2_bytes(it.d_in, it.d_in);
        }
        sp.count = 2 * n;
        sp.amax = amax + 2 * done;
        const kfac_status pre = split2_prepass(st, sp);
        if (pre != KFAC_OK) return pre;
    }
    return KFAC_OK;
}

kfac_status precondition_split_run(const kfac_precondition_item *items, int64_t count, const PrecSplitPlan &pl,
                                   const void *prepared, void *workspace, hipStream_t st)
{
    const unsigned *amax_inv = static_cast<const unsigned *>(prepared);
    const char *inv_cur = static_cast<const char *>(prepared) + pl.prep_amax;
    unsigned *amax_run = static_cast<unsigned *>(workspace);  // word 2 i: G of layer i, word 2 i + 1: its T^T
    char *tcur = static_cast<char *>(workspace) + pl.ws_amax;
    char *pcur = tcur + pl.t_bytes;
    for (int64_t done = 0; done < count; done += PREC_SPLIT_GROUP) {
        const int n = (int)std::min<int64_t>(PREC_SPLIT_GROUP, count - done);
        float *tt[PREC_SPLIT_GROUP];
        const char *pl_b[PREC_SPLIT_GROUP], *pl_a[PREC_SPLIT_GROUP];
        char *pl_g[PREC_SPLIT_GROUP], *pl_t[PREC_SPLIT_GROUP];
        // T^T = G^T B^-1  (d_in x d_out): contraction over the rows of G and of B^-1
        Split2Launch sp;
        Gemm2Launch gl;
        std::memset(&sp, 0, sizeof(sp));
        std::memset(&gl, 0, sizeof(gl));
        for (int i = 0; i < n; ++i) {
            const kfac_precondition_item &it = items[done + i];
            const int64_t dout = it.d_out, din = it.d_in;
            tt[i] = reinterpret_cast<float *>(tcur);
            tcur += align_up((size_t)din * dout * sizeof(float), WS_ALIGN);
            pl_b[i] = inv_cur; inv_cur += planes2_bytes(dout, dout);
            pl_a[i] = inv_cur; inv_cur += planes2_bytes(din, din);
            pl_g[i] = pcur; pcur += planes2_bytes(dout, din);
            pl_t[i] = pcur; pcur += planes2_bytes(din, dout);
            split2_item(sp.it[i], it.grad, dout, din, it.ldg, pl_g[i]);
            Gemm2Problem &q = gl.p[i];
            q.xa = pl_g[i];
            q.xb = pl_b[i];
            q.c = tt[i];
            q.m = (int)din;
            q.n = (int)dout;
            q.groups = pack_groups(dout);
            q.dpa = pack_cols(din);
            q.dpb = pack_cols(dout);
            q.ldc = (int)dout;
            q.amax_a = i;                           // in this group's words for G
            q.amax_b = (int)(2 * (done + i));       // B^-1 of the layer
        }
        // (the pre-pass numbers its items 0 .. n-1: G's words of this group are amax_run[2 done .. 2 done + n),
        //  T^T's the n words after them)
        sp.count = n;
        sp.amax = amax_run + 2 * done;
        kfac_status pre = split2_prepass(st, sp);
        if (pre != KFAC_OK) return pre;
        gl.count = n;
        gl.amax_a = amax_run + 2 * done;
        gl.amax_b = amax_inv;
        gemm2_order(gl);
        hipLaunchKernelGGL(gemm_tn_split2_256_kernel, dim3(gemm2_grid(gl)), dim3(256), 0, st, gl);
        // out = (T^T)^T A^-1  (d_out x d_in): contraction over the rows of T^T and of A^-1
        std::memset(&sp, 0, sizeof(sp));
        std::memset(&gl, 0, sizeof(gl));
        for (int i = 0; i < n; ++i) {
            const kfac_precondition_item &it = items[done + i];
            const int64_t dout = it.d_out, din = it.d_in;
            split2_item(sp.it[i], tt[i], din, dout, dout, pl_t[i]);
            Gemm2Problem &q = gl.p[i];
            q.xa = pl_t[i];
            q.xb = pl_a[i];
            q.c = it.out;
            q.m = (int)dout;
            q.n = (int)din;
            q.groups = pack_groups(din);
            q.dpa = pack_cols(dout);
            q.dpb = pack_cols(din);
            q.ldc = (int)it.ldo;
            q.amax_a = i;
            q.amax_b = (int)(2 * (done + i) + 1);   // A^-1 of the layer
        }
        sp.count = n;
        sp.amax = amax_run + 2 * done + n;
        pre = split2_prepass(st, sp);
        if (pre != KFAC_OK) return pre;
        gl.count = n;
        gl.amax_a = amax_run + 2 * done + n;
        gl.amax_b = amax_inv;
        gemm2_order(gl);
        hipLaunchKernelGGL(gemm_tn_split2_256_kernel, dim3(gemm2_grid(gl)), dim3(256), 0, st, gl);
        if (hipGetLastError() != hipSuccess) return KFAC_ERR_HIP;
    }
    return KFAC_OK;
}
}  // namespace

size_t kfac_precondition_f16x2_prepared_bytes(const kfac_precondition_item *items, int64_t count)
{
    if (items == nullptr || count <= 0) return 0;
    PrecSplitPlan pl;
    if (!precondition_split_plan(items, count, pl)) return 0;
    return pl.prep_bytes;
}

size_t kfac_precondition_grouped_f16x2_prepared_workspace(const kfac_precondition_item *items, int64_t count)
{
    if (items == nullptr || count <= 0) return 0;
    PrecSplitPlan pl;
    if (!precondition_split_plan(items, count, pl)) return 0;
    return pl.ws_bytes;
}

size_t kfac_precondition_grouped_f16x2_workspace(const kfac_precondition_item *items, int64_t count)
{
    if (items == nullptr || count <= 0) return 0;
    PrecSplitPlan pl;
    if (!precondition_split_plan(items, count, pl)) return 0;
    return align_up(pl.prep_bytes, WS_ALIGN) + pl.ws_bytes;
}

kfac_status kfac_precondition_f16x2_prepare(const kfac_precondition_item *items, int64_t count,
                                            void *prepared, size_t prepared_bytes, void *stream)
{
    if (count == 0) return KFAC_OK;
    const kfac_status chk = precondition_split_check(items, count, false);
    if (chk != KFAC_OK) return chk;
    PrecSplitPlan pl;
    if (!precondition_split_plan(items, count, pl)) return KFAC_ERR_ARG;
    if (!ws_ok(prepared, prepared_bytes, pl.prep_bytes)) return KFAC_ERR_WORKSPACE;
    return precondition_split_prepare(items, count, pl, prepared, static_cast<hipStream_t>(stream));
}

kfac_status kfac_precondition_grouped_f16x2_prepared(const kfac_precondition_item *items, int64_t count,
                                                     const void *prepared, size_t prepared_bytes,
                                                     void *workspace, size_t workspace_bytes, void *stream)
{
    if (count == 0) return KFAC_OK;
    const kfac_status chk = precondition_split_check(items, count, true);
    if (chk != KFAC_OK) return chk;
    PrecSplitPlan pl;
    if (!precondition_split_plan(items, count, pl)) return KFAC_ERR_ARG;
    if (!ws_ok(const_cast<void *>(prepared), prepared_bytes, pl.prep_bytes)) return KFAC_ERR_WORKSPACE;
    if (!ws_ok(workspace, workspace_bytes, pl.ws_bytes)) return KFAC_ERR_WORKSPACE;
    return precondition_split_run(items, count, pl, prepared, workspace, static_cast<hipStream_t>(stream));
}

kfac_status kfac_precondition_grouped_f16x2(const kfac_precondition_item *items, int64_t count,
                                            void *workspace, size_t workspace_bytes, void *stream)
{
    if (count == 0) return KFAC_OK;
    const kfac_status chk = precondition_split_check(items, count, true);
    if (chk != KFAC_OK) return chk;
    PrecSplitPlan pl;
    if (!precondition_split_plan(items, count, pl)) return KFAC_ERR_ARG;
    const size_t prep = align_up(pl.prep_bytes, WS_ALIGN);
    if (!ws_ok(workspace, workspace_bytes, prep + pl.ws_bytes)) return KFAC_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const kfac_status pre = precondition_split_prepare(items, count, pl, workspace, st);
    if (pre != KFAC_OK) return pre;
    return precondition_split_run(items, count, pl, workspace, static_cast<char *>(workspace) + prep, st);
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
