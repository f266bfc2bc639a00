"""Measured K-FAC work -> bubbles of a pipeline step -> execution in that order (section 3.1 of the paper).

Orchestration only.  Durations come from HIP events around library calls, the timeline of a
GPipe stage from ``kfac_gpipe_stage``, the assignment from ``kfac_assign_work`` (rules 1 and 2 as
release times and dependencies), and every arithmetic step of the method runs in the HIP library
when a chunk is executed.  Nothing here computes a factor, an inverse or a gradient.
"""
import torch

from . import binding


def time_ms(fn, reps=3, warmup=1, stream=None):
    """Median HIP-event duration of ``fn()`` (which enqueues work on ``stream``) in milliseconds."""
    stream = stream or torch.cuda.current_stream()
    for _ in range(warmup):
        fn()
    out = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fn()
        e1.record(stream)
        e1.synchronize()
        out.append(e0.elapsed_time(e1))
    out.sort()
    return out[len(out) // 2]


def measure_plan_steps(plan, reps=3, stream=None):
    """Duration of every step of an inversion plan (median of ``reps`` full runs), in milliseconds.

    The plan is run to its end each time, so its outputs are written as by ``kfac_invert_batched``.
    """
    stream = stream or torch.cuda.current_stream()
    n = plan.steps
    runs = []
    for _ in range(reps + 1):  # the first run warms up
        plan.reset()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        ev[0].record(stream)
        for i in range(n):
            plan.run(1, stream=stream)
            ev[i + 1].record(stream)
        ev[n].synchronize()
        runs.append([ev[i].elapsed_time(ev[i + 1]) for i in range(n)])
    runs = runs[1:]
    return [sorted(r[i] for r in runs)[len(runs) // 2] for i in range(n)]


class Work:
    """One entry of the queue: chunks that run in order, each an indivisible call with a measured duration."""

    def __init__(self, name, chunks, durations_ms, release_ms=0.0, deps=()):
        assert len(chunks) == len(durations_ms)
        self.name, self.chunks, self.durations_ms = name, list(chunks), [float(d) for d in durations_ms]
        self.release_ms, self.deps = float(release_ms), list(deps)


def assign(timeline, step_period_ms, works):
    """Places the queue into the bubbles of the stage; returns (placements, steps_needed).

    ``timeline`` is what ``kfac_gpipe_stage`` returns (times in milliseconds); ``step_period_ms`` is the
    start-to-start time of consecutive pipeline steps (the step plus the precondition work, rule 3).
    """
    return binding.kfac_assign_work([b[0] for b in timeline["bubbles"]], [b[1] for b in timeline["bubbles"]],
                                    step_period_ms, [w.durations_ms for w in works], [w.release_ms for w in works],
                                    [w.deps for w in works])


def run_steps(timeline, t_f_ms, t_b_ms, works, placements, steps_needed, forward, backward, end_of_step):
    """Runs ``steps_needed`` pipeline steps on the current stream in the order of the static schedule.

    Per step: the forward and backward passes of the stage (``forward(m)``, ``backward(m)``) and the chunks
    placed into that step, sorted by start time; then ``end_of_step(step)`` (the precondition work).
    Returns the list of (pipeline step, start time, name) in execution order.
    """
    order = []
    for step in range(steps_needed):
        events = []
        for m, end in enumerate(timeline["forward_end"]):
            events.append((end - t_f_ms, 0, "forward %d" % m, lambda m=m: forward(m)))
        for m, end in enumerate(timeline["backward_end"]):
            events.append((end - t_b_ms, 0, "backward %d" % m, lambda m=m: backward(m)))
        for w, spots in zip(works, placements):
            for ci, (s, _bubble, start) in enumerate(spots):
                if s == step:
                    events.append((start, 1, "%s [%d]" % (w.name, ci), w.chunks[ci]))
        events.sort(key=lambda e: (e[0], e[1]))
        for start, _kind, name, fn in events:
            fn()
            order.append((step, start, name))
        end_of_step(step)
    return order
