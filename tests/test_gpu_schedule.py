"""Section 3.1 end to end on the GPU: measured durations -> assignment to the bubbles of a GPipe stage ->
execution in schedule order between stand-in forward / backward passes -> results against the oracle.

The stage is a small one (two encoder blocks with d_model 256, d_ff 1024; 4 micro-batches of 1024 tokens)
so that the oracle redoes every layer in seconds; the machinery is the one bench.py uses at full size.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2211_14133_amd import synth  # noqa: E402

pytestmark = pytest.mark.gpu

CFG = 9  # tensor-id namespace of this test's synthetic inputs


def test_measured_work_is_assigned_to_bubbles_and_run_in_that_order(oracle):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_14133_amd as k
    from paper_2211_14133_amd import bubble_schedule as bs

    dev = torch.device("cuda:0")
    tokens, n_micro, blocks, lam = 1024, 4, 2, synth.DAMPING
    layer_defs = synth.block_layers(256, 1024)
    layers, hx, he = [], [], []
    for b in range(blocks):
        for li, (name, d_in, d_out, gelu) in enumerate(layer_defs):
            layers.append((name, d_in, d_out))
            hx.append([synth.activations(CFG, b, li, m, tokens, d_in, gelu=gelu) for m in range(n_micro)])
            he.append([synth.errors(CFG, b, li, m, tokens, d_out, scale=1.0) for m in range(n_micro)])
    hg = [synth.weight_gradient(he[i], hx[i]) for i in range(len(layers))]
    xa = [[torch.from_numpy(hx[i][m]).to(dev) for i in range(len(layers))] for m in range(n_micro)]
    xb = [[torch.from_numpy(he[i][m]).to(dev) for i in range(len(layers))] for m in range(n_micro)]
    grads = [torch.from_numpy(g).to(dev) for g in hg]
    fa = [torch.zeros(di, di, device=dev) for (_, di, do) in layers]
    fb = [torch.zeros(do, do, device=dev) for (_, di, do) in layers]
    # inverses of the previous refresh (here: the identity) are what precondition uses until the new ones are there
    ia = [torch.eye(di, device=dev) for (_, di, do) in layers]
    ib = [torch.eye(do, device=dev) for (_, di, do) in layers]
    outs = [torch.empty_like(g) for g in grads]
    alpha = 1.0 / (tokens * n_micro)

    # ---- stand-ins for the stage's forward and backward pass of one micro-batch (only their duration matters)
    wa = torch.randn(2048, 2048, device=dev)
    wb = torch.randn(2048, 2048, device=dev)

    def forward(m):
        torch.mm(wa, wb)

    def backward(m):
        torch.mm(wa, wb)
        torch.mm(wb, wa)

    t_f, t_b = bs.time_ms(lambda: forward(0), reps=5), bs.time_ms(lambda: backward(0), reps=5)

    # ---- the K-FAC work of the stage with measured durations
    t_curv_a = bs.time_ms(lambda: k.kfac_curvature_grouped(xa[0], fa, alpha, 0.0), reps=5)
    t_curv_b = bs.time_ms(lambda: k.kfac_curvature_grouped(xb[0], fb, alpha, 0.0), reps=5)
    plan = k.InvertPlan(fa + fb, lam, ia + ib)
    step_ms = bs.measure_plan_steps(plan, reps=3)
    assert len(step_ms) == plan.steps and all(t > 0 for t in step_ms)
    labels = [plan.step_label(i) for i in range(plan.steps)]
    assert labels[0] == "copy + damping" and labels[-1] == "inverse = W W^T" and "panel solve" in labels
    assert plan.step_label(plan.steps) is None
    t_prec = bs.time_ms(lambda: k.kfac_precondition_grouped(ib, ia, grads, outs), reps=5)
    # (measuring ran the plan on zero factors + damping: put the "previous" inverses back)
    for t in ia + ib:
        t.copy_(torch.eye(t.shape[0], device=dev))
    torch.cuda.synchronize()

    depth, stage = 4, 1
    tl = k.kfac_gpipe_stage(stage, depth, n_micro, t_f, t_b)
    period = tl["t_step"] + t_prec  # rule 3: precondition after the last backward pass, before the next step
    started = {"A": False, "B": False}

    def curvature(side, m):
        def run():
            xs, fs = (xa, fa) if side == "A" else (xb, fb)
            k.kfac_curvature_grouped(xs[m], fs, alpha, 1.0 if started[side] else 0.0)
            started[side] = True
        return run

    def inversion_chunk(i):
        def run():
            if i == 0:
                plan.reset()
            assert plan.position == i
            plan.run(1)
        return run

    works = []
    for m in range(n_micro):  # rule 1: A after the forward pass of the micro-batch, B after its backward pass
        works.append(bs.Work("curvature A mb%d" % m, [curvature("A", m)], [t_curv_a], release_ms=tl["forward_end"][m]))
    for m in range(n_micro):
        works.append(bs.Work("curvature B mb%d" % m, [curvature("B", m)], [t_curv_b], release_ms=tl["backward_end"][m]))
    curv_ids = list(range(len(works)))
    # rule 2: inversion after the curvature work of all micro-batches; its chunks are the plan's steps
    works.append(bs.Work("inversion", [inversion_chunk(i) for i in range(plan.steps)], step_ms, deps=curv_ids))
    placements, steps_needed = bs.assign(tl, period, works)
    total = sum(sum(w.durations_ms) for w in works)
    bubble = sum(length for _, length in tl["bubbles"])
    print("t_f %.3f t_b %.3f ms; curvature A %.3f B %.3f, inversion %.3f (%d chunks), precondition %.3f ms; "
          "bubbles %.3f ms per step -> %d pipeline steps per refresh (model ratio %.2f)"
          % (t_f, t_b, t_curv_a, t_curv_b, sum(step_ms), len(step_ms), t_prec, bubble, steps_needed, total / bubble), flush=True)
    assert steps_needed >= int(np.ceil(total / bubble - 1e-9))

    # ---- run the static schedule: precondition every step with whatever inverses are there
    stale_used = []

    def end_of_step(step):
        k.kfac_precondition_grouped(ib, ia, grads, outs)
        stale_used.append(plan.position < plan.steps)

    plan.reset()
    order = bs.run_steps(tl, t_f, t_b, works, placements, steps_needed, forward, backward, end_of_step)
    torch.cuda.synchronize()
    assert plan.position == plan.steps and int(plan.infos.abs().max()) == 0
    assert stale_used[-1] is False  # the last step preconditions with the fresh inverses
    # the order respects the rules: curvature after its pass, the inversion after all curvature, chunks in order
    names = [n for _, _, n in order]
    first_inv = names.index("inversion [0]")
    for m in range(n_micro):
        assert names.index("forward %d" % m) < names.index("curvature A mb%d [0]" % m) < first_inv
        assert names.index("backward %d" % m) < names.index("curvature B mb%d [0]" % m) < first_inv
    inv_pos = [names.index("inversion [%d]" % i) for i in range(plan.steps)]
    assert inv_pos == sorted(inv_pos)

    # ---- against the oracle, layer by layer
    for li, (name, d_in, d_out) in enumerate(layers):
        oa, ob, oai, obi, op = oracle.kfac_chain(hx[li], he[li], hg[li], lam)
        errs = [oracle.rel_fro(t.cpu().numpy(), o) for t, o in ((fa[li], oa), (fb[li], ob), (ia[li], oai), (ib[li], obi), (outs[li], op))]
        print("  layer %2d %-5s A %.2e B %.2e A^-1 %.2e B^-1 %.2e P %.2e" % ((li, name) + tuple(errs)), flush=True)
        assert errs[0] <= 1e-4 and errs[1] <= 1e-4 and errs[4] <= 5e-3
    plan.close()


def test_layers_that_share_their_input_share_one_a_factor(oracle):
    """The query, key and value projections of a block read the same activations, so their A factors are one
    matrix.  A caller builds and inverts it once (one curvature item, one inversion item) and hands the same
    inverse to the precondition work of the three layers: 2 of the 6 factor builds and inversions are saved.
    The result is what the three layers get when each computes its own A (the paper counts 2L products,
    section 2.3.1): bit for bit on the GPU, and within the gates against the oracle run layer by layer."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_14133_amd as k

    dev = torch.device("cuda:0")
    n, d, lam = 700, 384, synth.DAMPING
    x = synth.activations(CFG, 5, 0, 0, n, d)
    es = [synth.errors(CFG, 5, l, 0, n, d, scale=1.0) for l in range(3)]
    gs = [synth.weight_gradient([e], [x]) for e in es]
    xd = torch.from_numpy(x).to(dev)
    ed = [torch.from_numpy(e).to(dev) for e in es]
    gd = [torch.from_numpy(g).to(dev) for g in gs]
    # shared: 1 + 3 curvature items, 1 + 3 inversions
    a = torch.empty(d, d, device=dev)
    bsh = [torch.empty(d, d, device=dev) for _ in range(3)]
    k.kfac_curvature_grouped([xd] + ed, [a] + bsh, 1.0 / n, 0.0)
    ai = torch.empty_like(a)
    bi = [torch.empty_like(b) for b in bsh]
    infos = k.kfac_invert_batched([a] + bsh, lam, [ai] + bi)
    p_shared = [torch.empty_like(g) for g in gd]
    k.kfac_precondition_grouped(bi, [ai, ai, ai], gd, p_shared)
    # every layer on its own: 3 + 3 items
    a3 = [torch.empty(d, d, device=dev) for _ in range(3)]
    b3 = [torch.empty(d, d, device=dev) for _ in range(3)]
    k.kfac_curvature_grouped([xd, xd, xd] + ed, a3 + b3, 1.0 / n, 0.0)
    ai3 = [torch.empty_like(t) for t in a3]
    bi3 = [torch.empty_like(t) for t in b3]
    infos3 = k.kfac_invert_batched(a3 + b3, lam, ai3 + bi3)
    p_own = [torch.empty_like(g) for g in gd]
    k.kfac_precondition_grouped(bi3, ai3, gd, p_own)
    torch.cuda.synchronize()
    assert int(infos.abs().max()) == 0 and int(infos3.abs().max()) == 0
    for l in range(3):
        assert torch.equal(a3[l], a) and torch.equal(ai3[l], ai) and torch.equal(p_own[l], p_shared[l])
        oa, ob, oai, obi, op = oracle.kfac_chain([x], [es[l]], gs[l], lam)
        assert oracle.rel_fro(a.cpu().numpy(), oa) <= 1e-4
        assert oracle.rel_fro(p_shared[l].cpu().numpy(), op) <= 5e-3


def test_small_and_large_factors_on_two_streams(oracle):
    """The inversions of a stage split into its small and its large factors on two streams (default
    priority), each with a workspace of its own, and the precondition work of the layers that only need small
    factors right behind the first: the same bits as the one-stream sequence, and the oracle's result."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_14133_amd as k

    dev = torch.device("cuda:0")
    n, lam = 1200, synth.DAMPING
    shapes = [(256, 256)] * 4 + [(256, 1024), (1024, 256)]  # one block: attention linears, then the feed-forward pair
    hx = [synth.activations(CFG, 6, l, 0, n, di, gelu=(l == 5)) for l, (di, do) in enumerate(shapes)]
    he = [synth.errors(CFG, 6, l, 0, n, do, scale=1.0) for l, (di, do) in enumerate(shapes)]
    hg = [synth.weight_gradient([e], [x]) for e, x in zip(he, hx)]
    xs = [torch.from_numpy(t).to(dev) for t in hx]
    es = [torch.from_numpy(t).to(dev) for t in he]
    gs = [torch.from_numpy(t).to(dev) for t in hg]
    fa = [torch.empty(di, di, device=dev) for di, do in shapes]
    fb = [torch.empty(do, do, device=dev) for di, do in shapes]
    k.kfac_curvature_grouped(xs + es, fa + fb, 1.0 / n, 0.0)

    def run(two_streams):
        ia = [torch.full_like(f, 7.0) for f in fa]
        ib = [torch.full_like(f, 7.0) for f in fb]
        outs = [torch.empty_like(g) for g in gs]
        facs, invs = fa + fb, ia + ib
        small = [i for i, f in enumerate(facs) if f.shape[0] <= 256]
        large = [i for i, f in enumerate(facs) if f.shape[0] > 256]
        attn = [l for l, (di, do) in enumerate(shapes) if di <= 256 and do <= 256]
        ffn = [l for l in range(len(shapes)) if l not in attn]
        if not two_streams:
            infos = k.kfac_invert_batched(facs, lam, invs)
            k.kfac_precondition_grouped(ib, ia, gs, outs)
            torch.cuda.synchronize()
            return ia, ib, outs, infos
        main = torch.cuda.current_stream()
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        ready = torch.cuda.Event()
        ready.record(main)
        s1.wait_event(ready)
        s2.wait_event(ready)
        with torch.cuda.stream(s1):
            i1 = k.kfac_invert_batched([facs[i] for i in small], lam, [invs[i] for i in small], stream=s1)
            k.kfac_precondition_grouped([ib[l] for l in attn], [ia[l] for l in attn], [gs[l] for l in attn],
                                        [outs[l] for l in attn], stream=s1)
        with torch.cuda.stream(s2):
            i2 = k.kfac_invert_batched([facs[i] for i in large], lam, [invs[i] for i in large], stream=s2)
        main.wait_stream(s1)
        main.wait_stream(s2)
        k.kfac_precondition_grouped([ib[l] for l in ffn], [ia[l] for l in ffn], [gs[l] for l in ffn], [outs[l] for l in ffn])
        torch.cuda.synchronize()
        return ia, ib, outs, torch.cat([i1, i2])

    one = run(False)
    two = run(True)
    assert int(one[3].abs().max()) == 0 and int(two[3].abs().max()) == 0
    for a, b in zip(one[0] + one[1] + one[2], two[0] + two[1] + two[2]):
        assert torch.equal(a, b)
    for l in (0, 4, 5):
        op = oracle.kfac_chain([hx[l]], [he[l]], hg[l], lam)[4]
        assert oracle.rel_fro(two[2][l].cpu().numpy(), op) <= 5e-3
