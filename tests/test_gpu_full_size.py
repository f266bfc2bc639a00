"""Parity at the benchmark's full size (one BERT-Large pipeline stage, 8 micro-batches),
in the launch configuration bench.py times: grouped curvature (72 factors per launch),
batched inversion (72 matrices), grouped precondition (36 layers).

The check is made of
 * sampled factor entries, each recomputed by the oracle as a plain dot product;
 * every inverse through its residual against the GPU's own factor
   (rows sampled; the fp64 products are formed on the host);
 * every preconditioned gradient through sampled entries of B~ P A~ = G;
 * every one of the 36 layers redone end to end by the oracle (factors from all 8
   micro-batches, both inverses, the preconditioned gradient), compared over whole matrices.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2211_14133_amd import synth  # noqa: E402

pytestmark = pytest.mark.gpu


class Stage:
    """The BERT-Large stage run once on the GPU; the tests below look at its results."""


@pytest.fixture(scope="module")
def stage():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_14133_amd as k

    cfg = synth.CONFIGS[4]
    st = Stage()
    st.tokens, st.n_micro, blocks = cfg["tokens"], cfg["n_micro"], cfg["blocks"]
    st.lam = synth.DAMPING
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.SEED)
    st.layers, st.xs, st.grads = [], [[] for _ in range(st.n_micro)], []
    for b in range(blocks):
        for (name, d_in, d_out, gelu) in cfg["layers"]:
            st.layers.append((name, d_in, d_out))
            g = torch.zeros(d_out, d_in, device=dev, dtype=torch.float64)
            for m in range(st.n_micro):
                x = torch.randn(st.tokens, d_in, device=dev, generator=gen)
                if gelu:
                    x = torch.nn.functional.gelu(x)
                e = torch.randn(st.tokens, d_out, device=dev, generator=gen) * 1e-3
                st.xs[m] += [x, e]
                g += e.double().t() @ x.double()
            st.grads.append((g / (st.tokens * st.n_micro)).float())
    st.facs = [torch.empty(d, d, device=dev) for (_, di, do) in st.layers for d in (di, do)]
    st.invs = [torch.empty_like(f) for f in st.facs]
    st.outs = [torch.empty_like(g) for g in st.grads]
    st.alpha = 1.0 / (st.tokens * st.n_micro)
    print("curvature", flush=True)
    for m in range(st.n_micro):
        k.kfac_curvature_grouped(st.xs[m], st.facs, st.alpha, 0.0 if m == 0 else 1.0)
    print("inversion", flush=True)
    infos = k.kfac_invert_batched(st.facs, st.lam, st.invs)
    print("precondition", flush=True)
    k.kfac_precondition_grouped(st.invs[1::2], st.invs[0::2], st.grads, st.outs)
    torch.cuda.synchronize()
    assert np.all(infos.cpu().numpy() == 0)
    yield st
    del st.xs, st.facs, st.invs, st.outs, st.grads
    torch.cuda.empty_cache()


def test_stage_full_size_identities(stage, oracle):
    st = stage
    dev = torch.device("cuda:0")
    facs, invs, outs, grads, xs, lam = st.facs, st.invs, st.outs, st.grads, st.xs, st.lam
    rng = np.random.default_rng(7)
    # --- sampled factor entries against plain fp64 dot products
    print("sampled factor entries", flush=True)
    worst = 0.0
    for fi in range(0, len(facs), 5):
        d = facs[fi].shape[0]
        scale = float(facs[fi].diagonal().abs().max())
        for _ in range(4):
            i, j = int(rng.integers(d)), int(rng.integers(d))
            want = 0.0
            for m in range(st.n_micro):
                cols = xs[m][fi][:, [i, j]].cpu().numpy()
                want += oracle.curvature_entry(cols, 0, 1, st.alpha)
            got = float(facs[fi][i, j])
            assert got == float(facs[fi][j, i])
            worst = max(worst, abs(got - want) / scale)
    print("  worst |err| / max diag = %.2e" % worst, flush=True)
    assert worst <= 1e-5
    # --- every inverse: residual of sampled rows, products in fp64
    print("inverse residuals", flush=True)
    for fi, (f, v) in enumerate(zip(facs, invs)):
        d = f.shape[0]
        rows = torch.from_numpy(rng.integers(d, size=8)).to(dev)
        ft = f.double() + lam * torch.eye(d, device=dev, dtype=torch.float64)
        res = ft[rows] @ v.double()
        res[torch.arange(8), rows] -= 1.0
        r = float(res.norm() / np.sqrt(8))
        assert r <= 2e-3, (fi, d, r)
        assert torch.equal(v, v.t())
    # --- every preconditioned gradient: sampled entries of (B + lam I) P (A + lam I) = G
    print("precondition identity", flush=True)
    for li, (name, d_in, d_out) in enumerate(st.layers):
        a = facs[2 * li].double() + lam * torch.eye(d_in, device=dev, dtype=torch.float64)
        b = facs[2 * li + 1].double() + lam * torch.eye(d_out, device=dev, dtype=torch.float64)
        rows = torch.from_numpy(rng.integers(d_out, size=4)).to(dev)
        back = b[rows] @ outs[li].double() @ a
        g = grads[li].double()[rows]
        err = float((back - g).norm() / g.norm())
        assert err <= 5e-3, (li, name, err)


@pytest.mark.parametrize("block", range(6))
def test_stage_full_size_against_oracle(stage, oracle, capsys, block):
    """Every layer of the stage (six per encoder block, one block per test case so that a case ends within a
    minute) end to end against the oracle: factors from all 8 micro-batches, both inverses and the
    preconditioned gradient, element by element (relative Frobenius error over the whole matrix)."""
    import time

    st = stage
    t_start = time.perf_counter()
    for li in range(6 * block, 6 * block + 6):
        name, d_in, d_out = st.layers[li]
        hx = [st.xs[m][2 * li].cpu().numpy() for m in range(st.n_micro)]
        he = [st.xs[m][2 * li + 1].cpu().numpy() for m in range(st.n_micro)]
        g = st.grads[li].cpu().numpy()
        oa, ob, oai, obi, op = oracle.kfac_chain(hx, he, g, st.lam)
        errs = {
            "A": oracle.rel_fro(st.facs[2 * li].cpu().numpy(), oa),
            "B": oracle.rel_fro(st.facs[2 * li + 1].cpu().numpy(), ob),
            "Ainv": oracle.rel_fro(st.invs[2 * li].cpu().numpy(), oai),
            "Binv": oracle.rel_fro(st.invs[2 * li + 1].cpu().numpy(), obi),
            "P": oracle.rel_fro(st.outs[li].cpu().numpy(), op),
        }
        with capsys.disabled():  # progress must be visible while the test runs
            print("  layer %2d %-5s %4d -> %4d: A %.2e  B %.2e  A^-1 %.2e  B^-1 %.2e  P %.2e   (%.0f s)"
                  % (li, name, d_in, d_out, errs["A"], errs["B"], errs["Ainv"], errs["Binv"], errs["P"],
                     time.perf_counter() - t_start), flush=True)
        assert errs["A"] <= 1e-4 and errs["B"] <= 1e-4, (li, name, errs)
        assert errs["P"] <= 5e-3, (li, name, errs)
        # the inverses carry the factor error times the condition number (a few for the attention factors
        # at 32768 tokens, more for the GELU-fed 4096-dimensional one)
        assert errs["Ainv"] <= 1e-4 and errs["Binv"] <= 1e-5, (li, name, errs)


@pytest.mark.parametrize("mode", ["bf16x3", "f16x2"])
def test_stage_full_size_on_the_16_bit_matrix_cores(stage, mode):
    """The variants that take the float32 inputs as bfloat16 / float16 terms, at the benchmark's full size and in
    the launch configuration bench.py times them in, against the fp32-MFMA results of the same stage (which the
    tests above and below hold against the oracle): every factor, and with the float16 terms every preconditioned
    gradient (through the variant's own factors and the fp32 inversion)."""
    import paper_2211_14133_amd as k

    st = stage
    facs = [torch.empty_like(f) for f in st.facs]
    for m in range(st.n_micro):
        k.kfac_curvature_grouped(st.xs[m], facs, st.alpha, 0.0 if m == 0 else 1.0, split_bf16=mode)
    torch.cuda.synchronize()
    worst = 0.0
    for f, r in zip(facs, st.facs):
        worst = max(worst, float((f.double() - r.double()).norm() / r.double().norm()))
        assert torch.equal(f, f.t())
    print("%s: factors differ from the fp32 path's by at most %.3g" % (mode, worst), flush=True)
    assert worst <= 6e-7
    if mode != "f16x2":
        return
    invs = [torch.empty_like(f) for f in facs]
    infos = k.kfac_invert_batched(facs, st.lam, invs)
    outs = [torch.empty_like(g) for g in st.grads]
    k.kfac_precondition_grouped(invs[1::2], invs[0::2], st.grads, outs, f16x2=True)
    torch.cuda.synchronize()
    assert int(infos.abs().max()) == 0
    worst = 0.0
    for o, r in zip(outs, st.outs):
        worst = max(worst, float((o.double() - r.double()).norm() / r.double().norm()))
    print("%s: preconditioned gradients differ from the fp32 path's by at most %.3g" % (mode, worst), flush=True)
    assert worst <= 5e-5  # the fp32 path itself is within 7.3e-6 of the oracle on this stage


def test_curvature_long_sequence(oracle):
    """The longest micro-batch of the paper's performance-model table (32 x 2048 = 65,536 tokens) at the
    BERT-Large factor sizes: the whole 1024-dimensional factor against the oracle, sampled entries
    of the 4096-dimensional one, and the split into two halves of the tokens."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_14133_amd as k

    cfg = synth.CONFIGS[7]
    n = cfg["tokens"]
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.SEED + 7)
    xs = [torch.randn(n, 1024, device=dev, generator=gen),
          torch.nn.functional.gelu(torch.randn(n, 4096, device=dev, generator=gen))]
    facs = [torch.empty(1024, 1024, device=dev), torch.empty(4096, 4096, device=dev)]
    k.kfac_curvature_grouped(xs, facs, 1.0 / n, 0.0)
    torch.cuda.synchronize()
    want = oracle.curvature(xs[0].cpu().numpy())
    err = oracle.rel_fro(facs[0].cpu().numpy(), want)
    print("  d=1024, 65536 tokens: %.2e" % err, flush=True)
    assert err <= 1e-6
    rng = np.random.default_rng(11)
    scale = float(facs[1].diagonal().abs().max())
    worst = 0.0
    for _ in range(6):
        i, j = int(rng.integers(4096)), int(rng.integers(4096))
        cols = xs[1][:, [i, j]].cpu().numpy()
        w = oracle.curvature_entry(cols, 0, 1, 1.0 / n)
        got = float(facs[1][i, j])
        assert got == float(facs[1][j, i])
        worst = max(worst, abs(got - w) / scale)
    print("  d=4096 sampled entries: %.2e" % worst, flush=True)
    assert worst <= 1e-5
    # the same factor from two calls on halves of the tokens (a work item cut to a bubble's length)
    f2 = torch.empty_like(facs[0])
    k.kfac_curvature(xs[0][: n // 2], f2, 1.0 / n, 0.0)
    k.kfac_curvature(xs[0][n // 2:], f2, 1.0 / n, 1.0)
    torch.cuda.synchronize()
    assert oracle.rel_fro(f2.cpu().numpy(), want) <= 1e-6


def test_block_diagonal_factor_at_the_size_the_appendix_names(oracle, capsys):
    """Appendix A.2: for d >= 16,384 a factor is replaced by K independent diagonal blocks.  A 16,384-dimensional
    A factor as K = 4 blocks of 4096 (B: 1024-dimensional, whole), every step on the blocks addressed inside the
    big arrays through leading dimensions; against the oracle block by block."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import time

    import paper_2211_14133_amd as k

    dev = torch.device("cuda:0")
    n, d_in, d_out, kb, lam = 4096, 16384, 1024, 4, synth.DAMPING
    blk = d_in // kb
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.SEED + 16384)
    x = torch.randn(n, d_in, device=dev, generator=gen)
    e = torch.randn(n, d_out, device=dev, generator=gen) * 1e-3
    g = ((e.double().t() @ x.double()) / n).float()
    a = torch.zeros(d_in, d_in, device=dev)
    a_inv = torch.zeros(d_in, d_in, device=dev)
    b = torch.empty(d_out, d_out, device=dev)
    b_inv = torch.empty_like(b)
    ablocks = [a[i * blk:(i + 1) * blk, i * blk:(i + 1) * blk] for i in range(kb)]
    iblocks = [a_inv[i * blk:(i + 1) * blk, i * blk:(i + 1) * blk] for i in range(kb)]
    k.kfac_curvature_grouped([x[:, i * blk:(i + 1) * blk] for i in range(kb)] + [e], ablocks + [b], 1.0 / n, 0.0)
    infos = k.kfac_invert_batched(ablocks + [b], lam, iblocks + [b_inv])
    p = torch.empty_like(g)
    k.kfac_precondition_grouped([b_inv] * kb, iblocks, [g[:, i * blk:(i + 1) * blk] for i in range(kb)],
                                [p[:, i * blk:(i + 1) * blk] for i in range(kb)])
    torch.cuda.synchronize()
    assert int(infos.abs().max()) == 0
    # nothing outside the diagonal blocks was touched
    mask = torch.ones(kb, kb, device=dev) - torch.eye(kb, device=dev)
    assert float((a.view(kb, blk, kb, blk).abs().amax(dim=(1, 3)) * mask).max()) == 0.0
    assert float((a_inv.view(kb, blk, kb, blk).abs().amax(dim=(1, 3)) * mask).max()) == 0.0
    he, hg = e.cpu().numpy(), g.cpu().numpy()
    ob = oracle.curvature(he)
    obi, _ = oracle.invert(ob, lam)
    t0 = time.perf_counter()
    for i in range(kb):
        hx = x[:, i * blk:(i + 1) * blk].cpu().numpy()
        oa = oracle.curvature(hx)
        oai, info = oracle.invert(oa, lam)
        assert info == 0
        op = oracle.precondition(obi, hg[:, i * blk:(i + 1) * blk], oai)
        ea = oracle.rel_fro(ablocks[i].cpu().numpy(), oa)
        eai = oracle.rel_fro(iblocks[i].cpu().numpy(), oai)
        ep = oracle.rel_fro(p[:, i * blk:(i + 1) * blk].cpu().numpy(), op)
        with capsys.disabled():
            print("  block %d of %d: A %.2e  A^-1 %.2e  P %.2e   (%.0f s)" % (i, kb, ea, eai, ep, time.perf_counter() - t0), flush=True)
        assert ea <= 1e-4 and ep <= 5e-3


def test_inversion_at_the_largest_size_the_library_takes(capsys):
    """d = 32,640 = 255 panels of 128, the limit stated at the boundary (block indices travel as bytes).  The
    oracle cannot invert a matrix of this size in minutes, so the result is checked through what holds at any
    size: info, bitwise symmetry, and the residual of sampled columns with the fp64 products formed by torch."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_14133_amd as k

    dev = torch.device("cuda:0")
    d, lam = 255 * 128, synth.DAMPING
    n = 2 * d  # eigenvalues of X^T X / n within about [(1 - sqrt(1/2))^2, (1 + sqrt(1/2))^2]: condition number 34
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.SEED + d)
    f = torch.empty(d, d, device=dev)
    half = n // 2
    for i in range(2):  # two halves of the tokens, so that the activations take 4 GiB at a time
        x = torch.randn(half, d, device=dev, generator=gen)
        k.kfac_curvature(x, f, 1.0 / n, 0.0 if i == 0 else 1.0)
        torch.cuda.synchronize()
        del x
    with capsys.disabled():
        print("  factor of %d rows built" % d, flush=True)
    inv = torch.empty_like(f)
    info = k.kfac_invert(f, lam, inv)
    torch.cuda.synchronize()
    assert int(info) == 0
    with capsys.disabled():
        print("  inverted", flush=True)
    # symmetric bit for bit (compared in row chunks, so that no transposed copy of the whole matrix is made)
    for r0 in range(0, d, 4096):
        r1 = min(d, r0 + 4096)
        assert torch.equal(inv[r0:r1, :], inv[:, r0:r1].t())
    cols = sorted({0, 1, 127, 128, 129, 511, 512, 4095, 4096, d // 2, d - 4097, d - 513, d - 129, d - 128, d - 2, d - 1})
    inv_j = inv[:, cols].double()
    res = lam * inv_j
    for r0 in range(0, d, 2048):
        r1 = min(d, r0 + 2048)
        res[r0:r1] += f[r0:r1].double() @ inv_j
    for c, j in enumerate(cols):
        res[j, c] -= 1.0
    worst = float(res.norm(dim=0).max())  # every sampled column of the identity has norm 1
    with capsys.disabled():
        print("  worst column residual %.2e" % worst, flush=True)
    assert worst <= 2e-6 * 34 + 1e-6 * (d / 1024) ** 0.5
