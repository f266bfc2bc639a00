// Host-side pieces around the work items: the greedy assignment of K-FAC work to
// pipeline bubbles (section 3.1 of the paper) and the closed forms of its
// performance model (section 3.3).  No device code here.
#include <cstdint>
#include <cstddef>
#include <limits>
#include <utility>
#include <vector>

#include "../../include/kfac.h"

namespace {
constexpr int64_t MAX_PIPELINE_STEPS = 1 << 20;
}

extern "C" {

kfac_status kfac_assign_work(int64_t n_bubbles, const double *bubble_start, const double *bubble_length,
                             double step_period,
                             int64_t n_works, const int64_t *chunk_count, const double *chunk_time,
                             const double *release, const int64_t *dep_begin, const int64_t *dep_ids,
                             int64_t *out_step, int64_t *out_bubble, double *out_start,
                             int64_t *steps_needed)
{
    if (n_bubbles <= 0 || n_works < 0 || !bubble_start || !bubble_length || !(step_period > 0.0)) return KFAC_ERR_ARG;
    if (n_works > 0 && (!chunk_count || !chunk_time || !release || !dep_begin || !out_step || !out_bubble || !out_start))
        return KFAC_ERR_ARG;
    if (steps_needed == nullptr) return KFAC_ERR_ARG;
    double longest = 0.0, prev_end = 0.0;
    for (int64_t b = 0; b < n_bubbles; ++b) {
        if (!(bubble_length[b] >= 0.0) || bubble_start[b] < prev_end || bubble_start[b] + bubble_length[b] > step_period)
            return KFAC_ERR_ARG;
        prev_end = bubble_start[b] + bubble_length[b];
        if (bubble_length[b] > longest) longest = bubble_length[b];
    }
    // busy[s][b]: the pieces already placed in bubble b of pipeline step s as (start, end) relative to
    // that step's start, sorted by start.  A piece may go behind them or into a hole in front of one
    // that had to wait for its release: a bubble is whatever part of it is still idle.
    typedef std::vector<std::pair<double, double>> Pieces;
    std::vector<std::vector<Pieces>> busy;
    std::vector<double> finish((size_t)n_works, 0.0);  // absolute completion time of each work
    int64_t chunk = 0, last_step = -1;
    for (int64_t w = 0; w < n_works; ++w) {
        if (chunk_count[w] < 0 || dep_begin[w + 1] < dep_begin[w]) return KFAC_ERR_ARG;
        double ready = release[w];
        for (int64_t k = dep_begin[w]; k < dep_begin[w + 1]; ++k) {
            const int64_t dep = dep_ids[k];
            if (dep < 0 || dep >= w) return KFAC_ERR_ARG;
            if (finish[(size_t)dep] > ready) ready = finish[(size_t)dep];
        }
        for (int64_t c = 0; c < chunk_count[w]; ++c, ++chunk) {
            const double dur = chunk_time[chunk];
            if (!(dur >= 0.0)) return KFAC_ERR_ARG;
            if (dur > longest) return KFAC_ERR_UNSUPPORTED;
            bool placed = false;
            int64_t s = (int64_t)(ready / step_period);
            if (s < 0) s = 0;
            for (; s < MAX_PIPELINE_STEPS && !placed; ++s) {
                while ((int64_t)busy.size() <= s) busy.emplace_back((size_t)n_bubbles);
                const double base = (double)s * step_period;
                for (int64_t b = 0; b < n_bubbles && !placed; ++b) {
                    Pieces &pc = busy[(size_t)s][(size_t)b];
                    const double bubble_end = bubble_start[b] + bubble_length[b];
                    // holes in time order: in front of piece 0, between pieces, behind the last one
                    double hole_begin = bubble_start[b];
                    for (size_t h = 0; h <= pc.size(); ++h) {
                        const double hole_end = h < pc.size() ? pc[h].first : bubble_end;
                        double t = hole_begin;
                        if (ready - base > t) t = ready - base;
                        if (t + dur <= hole_end) {
                            pc.insert(pc.begin() + (std::ptrdiff_t)h, std::make_pair(t, t + dur));
                            out_step[chunk] = s;
                            out_bubble[chunk] = b;
                            out_start[chunk] = t;
                            ready = base + t + dur;
                            if (s > last_step) last_step = s;
                            placed = true;
                            break;
                        }
                        if (h < pc.size()) hole_begin = pc[h].second;
                    }
                }
            }
            if (!placed) return KFAC_ERR_UNSUPPORTED;
        }
        finish[(size_t)w] = ready;
    }
    *steps_needed = last_step + 1;
    return KFAC_OK;
}

kfac_status kfac_gpipe_stage(int64_t stage, int64_t depth, int64_t n_micro, double t_f, double t_b,
                             double *forward_end, double *backward_end,
                             double *bubble_start, double *bubble_length, int64_t *n_bubbles, double *t_step)
{
    if (depth <= 0 || stage < 0 || stage >= depth || n_micro <= 0 || !(t_f > 0.0) || !(t_b > 0.0)) return KFAC_ERR_ARG;
    if (!forward_end || !backward_end || !bubble_start || !bubble_length || !n_bubbles || !t_step) return KFAC_ERR_ARG;
    // Forward passes enter stage `stage` after `stage` earlier stages and follow one another; the backward
    // passes start on the last stage once it has seen every micro-batch and travel back stage by stage.
    const double first_forward = (double)stage * t_f;
    const double all_forward_done = (double)(depth - 1 + n_micro) * t_f;  // on the last stage
    const double first_backward = all_forward_done + (double)(depth - 1 - stage) * t_b;
    for (int64_t m = 0; m < n_micro; ++m) {
        forward_end[m] = first_forward + (double)(m + 1) * t_f;
        backward_end[m] = first_backward + (double)(m + 1) * t_b;
    }
    *t_step = (double)(depth - 1 + n_micro) * (t_f + t_b);
    // idle: before the first forward pass, between the last forward and the first backward pass, after the last
    // backward pass until the last stage-0 backward pass ends the step
    const double idle_from[3] = {0.0, forward_end[n_micro - 1], backward_end[n_micro - 1]};
    const double idle_to[3] = {first_forward, first_backward, *t_step};
    int64_t nb = 0;
    for (int k = 0; k < 3; ++k)
        if (idle_to[k] > idle_from[k]) {
            bubble_start[nb] = idle_from[k];
            bubble_length[nb] = idle_to[k] - idle_from[k];
            ++nb;
        }
    *n_bubbles = nb;
    return KFAC_OK;
}

kfac_status kfac_perf_model(double c_f, double c_b, double t_f, double t_b, int64_t n_micro,
                            double t_curv, double t_inv, double t_prec, double *out)
{
    if (out == nullptr || n_micro <= 0 || !(t_f >= 0.0) || !(t_b >= 0.0) || !(c_f >= 0.0) || !(c_b >= 0.0))
        return KFAC_ERR_ARG;
    const double t_pipe = c_f * t_f + c_b * t_b;
    const double t_bubble = t_pipe - (double)n_micro * (t_f + t_b);
    const double fill = (double)n_micro * t_curv + t_inv;
    out[0] = t_pipe;
    out[1] = t_bubble;
    out[2] = fill + t_prec;
    out[3] = t_bubble > 0.0 ? fill / t_bubble : std::numeric_limits<double>::infinity();
    out[4] = t_pipe + t_prec;
    return KFAC_OK;
}

}  // extern "C"
