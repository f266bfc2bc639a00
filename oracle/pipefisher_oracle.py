"""Plain-Python oracle for the host-side pieces: bubble filling and the performance model.

TEST INFRASTRUCTURE ONLY (same rules as kfac_oracle.py: never imported by the product path).

* ``assign_work`` follows section 3.1 of the paper ("Automatic Work Assignments"): K-FAC work is
  taken from a queue, one piece at a time, and put into the first bubble that lies after everything
  the piece has to wait for (rule 1: the forward / backward pass of its micro-batch; rule 2: all
  curvature work of the factor for an inversion) and is long enough; when the bubbles of a pipeline
  step are used up the bubbles of the following steps are taken.  It is written as a walk along the
  time line over the idle intervals of every bubble instance (see the reading stated in its docstring).
* ``perf_model`` is section 3.3: T_pipe = C_f T_f + C_b T_b, T_bubble = T_pipe - N_micro (T_f + T_b),
  T_kfac = N_micro T_curv + T_inv + T_prec, and the (curvature + inversion) / bubble ratio.
* ``gpipe_stage_timeline`` lays out one GPipe step of one stage (all forward passes, then all backward
  passes, section 2.1) to get bubbles and release times for tests.
"""


def assign_work(bubble_start, bubble_length, step_period, chunk_times, release, deps, max_steps=100000):
    """Returns (placements, steps_needed); placements[w] = [(step, bubble, start_in_step), ...].

    Reading of "assign it to a bubble if its duration is shorter than the bubble duration, otherwise
    subsequent bubbles are utilized" (section 3.1; the paper does not say what happens to idle time that
    is left in FRONT of a piece which had to wait for its release): a bubble is whatever part of it
    is still idle.  The time line is walked from the moment the piece may start; the piece goes into the
    first idle interval that can hold it, be it the rest of a bubble behind earlier pieces or a hole an
    earlier, later-released piece left in front of itself.
    """
    idle = {}  # (step, bubble) -> idle intervals [begin, end) of that bubble instance, in time order
    finish = []
    placements = []
    last_step = -1
    for w, chunks in enumerate(chunk_times):
        ready = release[w]
        for d in deps[w]:
            assert 0 <= d < w
            ready = max(ready, finish[d])
        spots = []
        for dur in chunks:
            if all(dur > length for length in bubble_length):
                raise ValueError("chunk longer than every bubble")
            found = None
            step = max(0, int(ready // step_period))
            while found is None:
                if step >= max_steps:
                    raise ValueError("no room")
                base = step * step_period
                for b, (s0, length) in enumerate(zip(bubble_start, bubble_length)):
                    holes = idle.setdefault((step, b), [(s0, s0 + length)])
                    for h, (begin, end) in enumerate(holes):
                        t = max(begin, ready - base)
                        if t + dur <= end:
                            found = (step, b, t)
                            # what stays idle: the part in front of the piece and the part behind it
                            holes[h:h + 1] = [(begin, t), (t + dur, end)]
                            break
                    if found is not None:
                        break
                step += 1
            spots.append(found)
            ready = found[0] * step_period + found[2] + dur
            last_step = max(last_step, found[0])
        placements.append(spots)
        finish.append(ready)
    return placements, last_step + 1


def perf_model(c_f, c_b, t_f, t_b, n_micro, t_curv, t_inv, t_prec):
    t_pipe = c_f * t_f + c_b * t_b
    t_bubble = t_pipe - n_micro * (t_f + t_b)
    fill = n_micro * t_curv + t_inv
    return {
        "t_pipe": t_pipe,
        "t_bubble": t_bubble,
        "t_kfac": fill + t_prec,
        "ratio": fill / t_bubble if t_bubble > 0 else float("inf"),
        "t_step": t_pipe + t_prec,
    }


def gpipe_stage_timeline(stage, depth, n_micro, t_f, t_b):
    """One GPipe step seen from `stage` (0-based): busy intervals, bubbles and the step length.

    Forward of micro-batch m runs at [(stage + m) t_f, (stage + m + 1) t_f); the backward passes start
    on the last stage when its forwards are done and travel back one stage per t_b.
    """
    fwd = [((stage + m) * t_f, (stage + m + 1) * t_f) for m in range(n_micro)]
    t0 = (depth - 1 + n_micro) * t_f
    bwd = [(t0 + (depth - 1 - stage + m) * t_b, t0 + (depth - stage + m) * t_b) for m in range(n_micro)]
    t_step = (depth - 1 + n_micro) * (t_f + t_b)
    busy = sorted(fwd + bwd)
    bubbles, cur = [], 0.0
    for s, e in busy:
        if s > cur + 1e-12:
            bubbles.append((cur, s - cur))
        cur = max(cur, e)
    if t_step > cur + 1e-12:
        bubbles.append((cur, t_step - cur))
    return {"forward": fwd, "backward": bwd, "bubbles": bubbles, "t_step": t_step}
