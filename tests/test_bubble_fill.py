"""Host-side bubble filling and performance model: pins for the oracle, then product vs oracle.

CPU only (no kernel is launched): the C ABI functions kfac_assign_work / kfac_perf_model are host code.
"""
import numpy as np
import pytest

from oracle import pipefisher_oracle as po
import paper_2211_14133_amd as k


# ------------------------------------------------------------------ oracle pins

def test_perf_model_closed_forms_from_the_paper():
    # section 3.3 / symbol table: N_micro = D: GPipe and 1F1B have C_f = C_b = 2D - 1, Chimera C_f = D, C_b = 2D - 2
    d, tf, tb = 4, 1.0, 2.0
    m = po.perf_model(2 * d - 1, 2 * d - 1, tf, tb, d, 0.25, 3.0, 0.5)
    assert m["t_pipe"] == 7 * 3.0 and m["t_bubble"] == 21.0 - 12.0
    assert m["t_kfac"] == 4 * 0.25 + 3.0 + 0.5 and m["ratio"] == 4.0 / 9.0 and m["t_step"] == 21.5
    c = po.perf_model(d, 2 * d - 2, tf, tb, d, 0.25, 3.0, 0.5)
    assert c["t_pipe"] == 4 * 1.0 + 6 * 2.0 and c["t_bubble"] == 16.0 - 12.0
    # Chimera has fewer bubbles than GPipe for the same work (section 2.1)
    assert c["t_bubble"] < m["t_bubble"]


def test_gpipe_timeline_matches_the_model():
    for depth, n_micro, tf, tb in [(4, 4, 1.0, 2.0), (8, 8, 0.7, 1.3), (4, 8, 1.0, 1.0)]:
        tot = None
        for stage in range(depth):
            tl = po.gpipe_stage_timeline(stage, depth, n_micro, tf, tb)
            bub = sum(length for _, length in tl["bubbles"])
            model = po.perf_model(depth - 1 + n_micro, depth - 1 + n_micro, tf, tb, n_micro, 0, 0, 0)
            assert abs(tl["t_step"] - model["t_pipe"]) < 1e-12
            assert abs(bub - model["t_bubble"]) < 1e-9  # every stage idles for the same total time
            tot = bub if tot is None else tot
            # busy intervals do not overlap and bubbles are their complement
            busy = sorted(tl["forward"] + tl["backward"])
            assert all(busy[i][1] <= busy[i + 1][0] + 1e-12 for i in range(len(busy) - 1))


def test_assign_work_by_hand():
    # two bubbles per step: [1,3) and [5,6); period 10
    placements, steps = po.assign_work([1.0, 5.0], [2.0, 1.0], 10.0, [[0.5], [1.0, 1.0], [0.9]], [0.0, 0.0, 0.0],
                                       [[], [0], [1]])
    assert placements == [[(0, 0, 1.0)], [(0, 0, 1.5), (0, 1, 5.0)], [(1, 0, 1.0)]]
    assert steps == 2
    # release time inside a bubble: the piece starts at its release, not at the bubble start; the idle
    # time it leaves in front of itself is still part of the bubble, and the next piece of the queue
    # (free from the start, too long for the 0.5 behind the first piece) goes there
    placements, steps = po.assign_work([0.0], [4.0], 5.0, [[1.0], [1.0]], [2.5, 0.0], [[], []])
    assert placements == [[(0, 0, 2.5)], [(0, 0, 0.0)]] and steps == 1
    with pytest.raises(ValueError):
        po.assign_work([0.0], [1.0], 5.0, [[2.0]], [0.0], [[]])


def test_assign_work_holes_by_hand():
    """Worked on paper.  One bubble [0, 10) per step, period 12.
    w0: released at 6, 2 long            -> [6, 8)                       idle: [0, 6) [8, 10)
    w1: released at 0, 5 long            -> the hole in front: [0, 5)    idle: [5, 6) [8, 10)
    w2: released at 0, chunks 1.5, 1.5   -> 1.5 does not fit [5, 6): [8, 9.5); the second chunk must follow
                                            the first (>= 9.5) and 0.5 is left in this step -> next step [0, 1.5)
    w3: after w1, 1 long                 -> [5, 6) exactly
    w4: released at 9, 0.5 long          -> [9.5, 10)
    w5: released at 0, 0.25 long         -> step 0 is full -> step 1 behind w2's second chunk: [1.5, 1.75)
    """
    chunk_times = [[2.0], [5.0], [1.5, 1.5], [1.0], [0.5], [0.25]]
    release = [6.0, 0.0, 0.0, 0.0, 9.0, 0.0]
    deps = [[], [], [], [1], [], []]
    want = [[(0, 0, 6.0)], [(0, 0, 0.0)], [(0, 0, 8.0), (1, 0, 0.0)], [(0, 0, 5.0)], [(0, 0, 9.5)], [(1, 0, 1.5)]]
    placements, steps = po.assign_work([0.0], [10.0], 12.0, chunk_times, release, deps)
    assert placements == want and steps == 2
    got, got_steps = k.kfac_assign_work([0.0], [10.0], 12.0, chunk_times, release, deps)
    assert got == want and got_steps == 2
    # two bubbles [0, 2) and [5, 7), period 8.  w0 (released 5.5) -> [5.5, 6.5).  w1 is released at 1.5: it never
    # starts before that, so [1.5, 2) is too short, as are [5, 5.5) and [6.5, 7) -> first bubble of the next step
    placements, steps = po.assign_work([0.0, 5.0], [2.0, 2.0], 8.0, [[1.0], [1.0]], [5.5, 1.5], [[], []])
    assert placements == [[(0, 1, 5.5)], [(1, 0, 0.0)]] and steps == 2


def _kfac_queue(depth, stage, n_micro, t_f, t_b, layers, t_curv_a, t_curv_b, inv_chunks):
    """K-FAC work of one stage in queue order with the paper's rules 1 and 2."""
    tl = po.gpipe_stage_timeline(stage, depth, n_micro, t_f, t_b)
    chunk_times, release, deps, kinds = [], [], [], []
    curv_ids = {}
    for m in range(n_micro):  # rule 1: A after forward(m), B after backward(m)
        for l in range(layers):
            curv_ids.setdefault((l, "A"), []).append(len(chunk_times))
            chunk_times.append([t_curv_a]); release.append(tl["forward"][m][1]); deps.append([]); kinds.append(("curvA", l, m))
    for m in range(n_micro):
        for l in range(layers):
            curv_ids.setdefault((l, "B"), []).append(len(chunk_times))
            chunk_times.append([t_curv_b]); release.append(tl["backward"][m][1]); deps.append([]); kinds.append(("curvB", l, m))
    for l in range(layers):  # rule 2: inversion after all curvature work of the factor
        for f in ("A", "B"):
            chunk_times.append(list(inv_chunks)); release.append(0.0); deps.append(list(curv_ids[(l, f)])); kinds.append(("inv" + f, l, -1))
    return tl, chunk_times, release, deps, kinds


def _check_schedule(tl, period, chunk_times, release, deps, placements):
    bstart = [b[0] for b in tl["bubbles"]]
    blen = [b[1] for b in tl["bubbles"]]
    finish, used = [], {}
    for w, spots in enumerate(placements):
        ready = max([release[w]] + [finish[d] for d in deps[w]])
        for (step, b, t), dur in zip(spots, chunk_times[w]):
            assert t >= bstart[b] - 1e-12 and t + dur <= bstart[b] + blen[b] + 1e-12  # inside a bubble
            assert step * period + t >= ready - 1e-12  # rules 1 and 2
            for (s2, e2) in used.get((step, b), []):
                assert t >= e2 - 1e-12 or t + dur <= s2 + 1e-12  # no two pieces overlap
            used.setdefault((step, b), []).append((t, t + dur))
            ready = step * period + t + dur
        finish.append(ready)


def test_assign_work_invariants_on_a_gpipe_stage():
    for stage in range(4):
        tl, chunk_times, release, deps, kinds = _kfac_queue(4, stage, 4, 1.0, 2.0, 3, 0.3, 0.3, [0.4] * 6)
        period = tl["t_step"] + 0.5  # precondition after the last backward pass (rule 3)
        placements, steps = po.assign_work([b[0] for b in tl["bubbles"]], [b[1] for b in tl["bubbles"]], period,
                                           chunk_times, release, deps)
        _check_schedule(tl, period, chunk_times, release, deps, placements)
        total = sum(sum(c) for c in chunk_times)
        bubble = sum(b[1] for b in tl["bubbles"])
        assert steps >= int(np.ceil(total / bubble - 1e-9))  # cannot be faster than the model's ratio
        assert steps <= int(np.ceil(total / bubble)) + 2


# ------------------------------------------------------------ product vs oracle

def test_product_perf_model_matches_oracle():
    rng = np.random.default_rng(0)
    for _ in range(20):
        a = [float(x) for x in rng.uniform(0.1, 5.0, 7)]
        n_micro = int(rng.integers(1, 16))
        got = k.kfac_perf_model(a[0] + 8, a[1] + 8, a[2], a[3], n_micro, a[4], a[5], a[6])
        want = po.perf_model(a[0] + 8, a[1] + 8, a[2], a[3], n_micro, a[4], a[5], a[6])
        for key in want:
            assert got[key] == pytest.approx(want[key], rel=1e-15, abs=0)


def _holes_used(placements):
    """Chunks that start in front of a chunk placed earlier in the same bubble instance."""
    seen, n = {}, 0
    for spots in placements:
        for (step, b, t) in spots:
            if any(t < t2 for t2 in seen.get((step, b), [])):
                n += 1
            seen.setdefault((step, b), []).append(t)
    return n


def test_product_assign_work_matches_oracle_exactly():
    rng = np.random.default_rng(1)
    holes = 0
    for case in range(30):
        depth = int(rng.integers(2, 9))
        n_micro = int(rng.integers(1, 9))
        stage = int(rng.integers(0, depth))
        layers = int(rng.integers(1, 5))
        t_f, t_b = float(rng.uniform(0.5, 2)), float(rng.uniform(0.5, 3))
        inv_chunks = [float(x) for x in rng.uniform(0.05, 0.5, int(rng.integers(1, 9)))]
        tl, chunk_times, release, deps, kinds = _kfac_queue(depth, stage, n_micro, t_f, t_b, layers,
                                                            float(rng.uniform(0.05, 0.4)), float(rng.uniform(0.05, 0.4)),
                                                            inv_chunks)
        if not tl["bubbles"]:
            continue
        bstart = [b[0] for b in tl["bubbles"]]
        blen = [b[1] for b in tl["bubbles"]]
        period = tl["t_step"] + float(rng.uniform(0, 0.5))
        longest = max(blen)
        if any(c > longest for ch in chunk_times for c in ch):
            with pytest.raises(k.KfacError):
                k.kfac_assign_work(bstart, blen, period, chunk_times, release, deps)
            continue
        want, want_steps = po.assign_work(bstart, blen, period, chunk_times, release, deps)
        got, got_steps = k.kfac_assign_work(bstart, blen, period, chunk_times, release, deps)
        assert got_steps == want_steps
        assert got == want  # same arithmetic on the same doubles: exact
        _check_schedule(tl, period, chunk_times, release, deps, got)
        holes += _holes_used(got)
    assert holes == 0  # in a GPipe step every release time lies at or before the start of the next bubble


def test_product_assign_work_matches_oracle_with_holes():
    """Arbitrary bubbles and release times anywhere in the first steps: pieces that have to wait leave idle
    time in front of themselves, which later pieces of the queue take."""
    rng = np.random.default_rng(5)
    holes = 0
    for case in range(40):
        nb = int(rng.integers(1, 5))
        cuts = np.sort(rng.uniform(0.0, 10.0, 2 * nb))
        bstart = [float(cuts[2 * i]) for i in range(nb)]
        blen = [float(cuts[2 * i + 1] - cuts[2 * i]) for i in range(nb)]
        period = 10.0 + float(rng.uniform(0, 1))
        longest = max(blen)
        n_works = int(rng.integers(10, 40))
        chunk_times = [[float(x) for x in rng.uniform(0.0, 0.3 * longest, int(rng.integers(1, 4)))] for _ in range(n_works)]
        release = [float(rng.uniform(0.0, 1.5 * period)) if rng.random() < 0.6 else 0.0 for _ in range(n_works)]
        deps = [sorted(set(int(x) for x in rng.integers(0, w, int(rng.integers(0, 3))))) if w else [] for w in range(n_works)]
        want, want_steps = po.assign_work(bstart, blen, period, chunk_times, release, deps)
        got, got_steps = k.kfac_assign_work(bstart, blen, period, chunk_times, release, deps)
        assert got == want and got_steps == want_steps
        _check_schedule({"bubbles": list(zip(bstart, blen))}, period, chunk_times, release, deps, got)
        holes += _holes_used(got)
    assert holes >= 30


def test_product_gpipe_stage_matches_oracle_timeline():
    for depth, n_micro, tf, tb in [(4, 4, 1.0, 2.0), (8, 8, 0.7, 1.3), (4, 8, 1.0, 1.0), (1, 3, 0.5, 0.25), (6, 1, 2.0, 3.0)]:
        for stage in range(depth):
            want = po.gpipe_stage_timeline(stage, depth, n_micro, tf, tb)
            got = k.kfac_gpipe_stage(stage, depth, n_micro, tf, tb)
            assert got["t_step"] == pytest.approx(want["t_step"], rel=1e-14)
            assert got["forward_end"] == pytest.approx([e for _, e in want["forward"]], rel=1e-14)
            assert got["backward_end"] == pytest.approx([e for _, e in want["backward"]], rel=1e-14)
            assert len(got["bubbles"]) == len(want["bubbles"])
            for (gs, gl), (ws, wl) in zip(got["bubbles"], want["bubbles"]):
                assert gs == pytest.approx(ws, rel=1e-14, abs=1e-14) and gl == pytest.approx(wl, rel=1e-13)
            # idle time of every stage = the bubble term of section 3.3 with C_f = C_b = n_micro + depth - 1
            c = n_micro + depth - 1
            assert sum(l for _, l in got["bubbles"]) == pytest.approx(k.kfac_perf_model(c, c, tf, tb, n_micro, 0, 0, 0)["t_bubble"], rel=1e-12)
    with pytest.raises(k.KfacError):
        k.kfac_gpipe_stage(4, 4, 2, 1.0, 1.0)


def test_product_assign_work_rejects_bad_input():
    with pytest.raises(k.KfacError):
        k.kfac_assign_work([2.0, 1.0], [1.0, 1.0], 10.0, [[0.1]], [0.0], [[]])  # bubbles not sorted
    with pytest.raises(k.KfacError):
        k.kfac_assign_work([0.0], [1.0], 10.0, [[0.1], [0.1]], [0.0, 0.0], [[1], []])  # dependency on a later work
    with pytest.raises(k.KfacError):
        k.kfac_assign_work([0.0], [1.0], 0.5, [[0.1]], [0.0], [[]])  # bubble longer than the step
