"""Parity of the HIP path against the fp64 oracle, element by element, through the C ABI.

Tolerances (relative Frobenius error over the whole matrix, accumulated in fp64):
factors <= 1e-4 for fp32 inputs, preconditioned gradient <= 5e-3 (the
benchmark definition's gates); inverses are checked against the oracle with
a bound scaled by the condition number, and by their residual.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2211_14133_amd import synth  # noqa: E402

pytestmark = pytest.mark.gpu

FACTOR_TOL = 1e-4
PRECOND_TOL = 5e-3


@pytest.fixture(scope="module")
def k():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_14133_amd as lib

    lib.load()
    return lib


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def gpu_factor(k, x, alpha=None, beta=0.0, factor=None, ld_pad=0):
    n, d = x.shape
    if alpha is None:
        alpha = 1.0 / n
    if factor is None:
        buf = torch.full((d, d + ld_pad), 7.0, dtype=torch.float32, device="cuda")
        factor = buf[:, :d]
    k.kfac_curvature(x, factor, alpha, beta)
    return factor


# ------------------------------------------------------------------ curvature

@pytest.mark.parametrize("n,d", [(256, 64), (300, 200), (1000, 129), (513, 767), (4096, 768), (2048, 1024), (16, 1), (1, 5)])
def test_curvature_parity(k, oracle, n, d):
    print("curvature n=%d d=%d" % (n, d), flush=True)
    x = synth.activations(1, 0, 0, 0, n, d, gelu=(d % 2 == 1))
    f = host(gpu_factor(k, dev(x)))
    want = oracle.curvature(x)
    err = oracle.rel_fro(f, want)
    print("  rel_fro", err, flush=True)
    assert err <= FACTOR_TOL
    assert err <= 5e-7  # chunked fp32 accumulation: a few ulp
    assert np.array_equal(f, f.T)


def test_curvature_strided_input_and_output(k, oracle):
    n, d = 700, 300
    big = synth.activations(1, 0, 1, 0, n, d + 37)
    xb = dev(big)
    x = xb[:, 5:5 + d]  # ldx = d + 37, pointer offset by 5 floats: unaligned rows
    f = gpu_factor(k, x, ld_pad=3)
    want = oracle.curvature(big[:, 5:5 + d])
    assert oracle.rel_fro(host(f), want) <= 5e-7
    # the padding columns of the output buffer are untouched
    assert torch.all(f.as_strided((d, 3), (d + 3, 1), d) == 7.0)


def test_curvature_hadamard_exact(k):
    for n, d in [(256, 256), (1024, 640), (4096, 1024)]:
        x = synth.hadamard_columns(n, d)
        f = host(gpu_factor(k, dev(x)))
        assert np.array_equal(f, np.eye(d, dtype=np.float32)), (n, d)


def test_curvature_small_integers_bitwise(k, oracle):
    rng = np.random.default_rng(5)
    for n, d in [(4096, 384), (1000, 130)]:
        x = rng.integers(-8, 9, size=(n, d)).astype(np.float32)
        f = host(gpu_factor(k, dev(x), alpha=1.0))
        want = oracle.curvature_update(x, 1.0, 0.0)
        assert np.array_equal(f.astype(np.float64), want)


def test_curvature_ones_and_one_hot(k):
    f = host(gpu_factor(k, torch.ones(64, 40, device="cuda")))
    assert np.array_equal(f, np.ones((40, 40), dtype=np.float32))
    idx = torch.arange(512, device="cuda") % 7
    x = torch.zeros(512, 9, device="cuda")
    x[torch.arange(512), idx] = 1.0
    f = host(gpu_factor(k, x, alpha=1.0))
    want = np.diag(np.bincount(host(idx), minlength=9)).astype(np.float32)
    assert np.array_equal(f, want)


def test_curvature_microbatch_accumulation(k, oracle):
    d, n, nm = 320, 512, 4
    xs = [synth.activations(1, 0, 2, m, n, d) for m in range(nm)]
    alpha = 1.0 / (n * nm)
    f = None
    for m, x in enumerate(xs):
        f = gpu_factor(k, dev(x), alpha=alpha, beta=0.0 if m == 0 else 1.0, factor=f)
    want = oracle.curvature(xs)
    assert oracle.rel_fro(host(f), want) <= 5e-7
    assert np.array_equal(host(f), host(f).T)
    # general beta
    x = xs[0]
    f0 = np.asarray(np.random.default_rng(3).standard_normal((d, d)), dtype=np.float32)
    f0 = (f0 + f0.T) / 2
    fd = dev(f0)
    k.kfac_curvature(dev(x), fd, 0.5, 0.25)
    want = oracle.curvature_update(x, 0.5, 0.25, f0)
    assert oracle.rel_fro(host(fd), want) <= 5e-7


def test_curvature_grouped_matches_single_and_oracle(k, oracle):
    shapes = [(512, 64), (512, 300), (384, 1024), (512, 129), (256, 640)]
    xs = [synth.activations(1, 0, 3 + i, 0, n, d) for i, (n, d) in enumerate(shapes)]
    xd = [dev(x) for x in xs]
    fg = [torch.empty(d, d, device="cuda") for _, d in shapes]
    k.kfac_curvature_grouped(xd, fg, 1.0 / 512, 0.0)
    for x, xdv, f in zip(xs, xd, fg):
        want = oracle.curvature_update(x, 1.0 / 512, 0.0)
        assert oracle.rel_fro(host(f), want) <= 5e-7
        assert np.array_equal(host(f), host(f).T)
    # 100 items: more than the 80 problems one launch describes
    many = [dev(synth.activations(1, 1, i, 0, 128, 96)) for i in range(100)]
    fm = [torch.empty(96, 96, device="cuda") for _ in many]
    k.kfac_curvature_grouped(many, fm, 1.0 / 128, 0.0)
    for x, f in zip(many, fm):
        assert oracle.rel_fro(host(f), oracle.curvature(host(x))) <= 5e-7


def test_curvature_is_deterministic(k):
    x = dev(synth.activations(1, 0, 9, 0, 4096, 768))
    a = host(gpu_factor(k, x)).copy()
    for _ in range(2):
        assert np.array_equal(a, host(gpu_factor(k, x)))


# ------------------------------------------------------------------ inversion

def gpu_invert(k, f, lam):
    d = f.shape[0]
    fd = dev(f.astype(np.float32))
    inv = torch.full((d, d), 3.0, device="cuda")
    info = k.kfac_invert(fd, lam, inv)
    return host(inv), int(host(info)[0])


@pytest.mark.parametrize("d", [1, 2, 3, 63, 64, 65, 127, 128, 129, 200, 256, 257, 384, 511, 513, 767, 768, 769, 1024, 1025, 1537, 2049])
def test_invert_parity(k, oracle, d):
    print("invert d=%d" % d, flush=True)
    n = max(2 * d, 64)
    x = synth.activations(2, 0, 0, 0, n, d, gelu=(d % 3 == 0))
    a = oracle.curvature(x).astype(np.float32)
    lam = 1e-3
    inv, info = gpu_invert(k, a, lam)
    assert info == 0
    want, _ = oracle.invert(a.astype(np.float64), lam)
    at = a.astype(np.float64) + lam * np.eye(d)
    cond = np.linalg.cond(at)
    err = oracle.rel_fro(inv, want)
    res = np.linalg.norm(at @ inv.astype(np.float64) - np.eye(d)) / np.sqrt(d)
    print("  cond %.3g rel_fro %.3g residual %.3g" % (cond, err, res), flush=True)
    assert err <= 2e-6 * cond + 1e-6
    assert res <= 2e-6 * cond + 1e-6
    assert np.array_equal(inv, inv.T)


def test_invert_closed_forms(k):
    d = 300
    inv, info = gpu_invert(k, np.zeros((d, d)), 4.0)
    assert info == 0 and np.array_equal(inv, np.eye(d, dtype=np.float32) / 4.0)
    al, be = 0.7, 0.3
    inv, info = gpu_invert(k, be * np.ones((d, d)), al)
    want = (np.eye(d) - be / (al + be * d) * np.ones((d, d))) / al
    assert info == 0 and np.linalg.norm(inv - want) <= 1e-5 * np.linalg.norm(want)
    i = np.arange(1, d + 1)
    t = 2 * np.eye(d) - np.eye(d, k=1) - np.eye(d, k=-1)
    inv, info = gpu_invert(k, t, 0.0)
    want = np.minimum.outer(i, i) * (d + 1 - np.maximum.outer(i, i)) / (d + 1.0)
    assert info == 0 and np.linalg.norm(inv - want) <= 1e-3 * np.linalg.norm(want)  # cond ~ 4e4


def test_invert_only_reads_upper_triangle(k, oracle):
    d = 200
    a = oracle.curvature(synth.activations(2, 0, 1, 0, 400, d)).astype(np.float32)
    junk = a.copy()
    junk[np.tril_indices(d, -1)] = 123.0
    i1, _ = gpu_invert(k, a, 1e-3)
    i2, _ = gpu_invert(k, junk, 1e-3)
    assert np.array_equal(i1, i2)


@pytest.mark.parametrize("d", [5, 200, 300, 1024])
def test_invert_ignores_non_finite_values_below_the_diagonal(k, oracle, d):
    """Only the upper triangle is input: a caller that keeps nothing (or NaN / Inf / uninitialised memory)
    below the diagonal gets info = 0 and the same bits as with the full symmetric matrix."""
    a = oracle.curvature(synth.activations(2, 0, 2, 0, 2 * d + 8, d)).astype(np.float32)
    junk = a.copy()
    low = np.tril_indices(d, -1)
    junk[low] = np.where(np.arange(low[0].size) % 3 == 0, np.nan, np.where(np.arange(low[0].size) % 3 == 1, np.inf, -np.inf))
    i1, info1 = gpu_invert(k, a, 1e-3)
    i2, info2 = gpu_invert(k, junk, 1e-3)
    assert info1 == 0 and info2 == 0
    assert np.array_equal(i1, i2)
    # a non-finite value ON or ABOVE the diagonal is still an error
    junk[d // 2, d - 1] = np.inf
    inv, info = gpu_invert(k, junk, 1e-3)
    assert info == -1 and np.all(inv == 3.0)


def test_invert_failure_reports_pivot_and_keeps_inverse(k):
    d = 300
    m = np.eye(d)
    m[170, 170] = -1.0
    inv, info = gpu_invert(k, m, 0.0)
    assert info == 171
    assert np.all(inv == 3.0)  # untouched
    m = np.eye(d)
    m[5, 9] = np.nan
    inv, info = gpu_invert(k, m, 0.0)
    assert info == -1 and np.all(inv == 3.0)
    # rank-deficient factor without damping fails, with damping succeeds
    x = np.ones((4, 150), dtype=np.float32)
    a = (x.T @ x / 4).astype(np.float32)
    inv, info = gpu_invert(k, a, 0.0)
    assert info > 0
    inv, info = gpu_invert(k, a, 1e-3)
    assert info == 0


def test_invert_batched_mixed_sizes(k, oracle):
    ds = [64, 300, 128, 513, 1, 256, 767]
    fs = [oracle.curvature(synth.activations(2, 1, i, 0, 2 * d + 8, d)).astype(np.float32) for i, d in enumerate(ds)]
    fd = [dev(f) for f in fs]
    invs = [torch.empty(d, d, device="cuda") for d in ds]
    infos = k.kfac_invert_batched(fd, 1e-3, invs)
    assert np.all(host(infos) == 0)
    for f, inv in zip(fs, invs):
        want, _ = oracle.invert(f.astype(np.float64), 1e-3)
        assert oracle.rel_fro(host(inv), want) <= 1e-4
        single, _ = gpu_invert(k, f, 1e-3)
        assert np.array_equal(single, host(inv))


def test_invert_result_does_not_depend_on_what_the_workspace_holds(k, oracle):
    """The working copy is only filled where the algorithm reads it: whatever else the caller's workspace holds
    (zeros, NaNs, infinities, the remains of another call) must not change a single bit of the result."""
    ds = [257, 513, 1024, 96, 640]
    fs = [oracle.curvature(synth.activations(2, 3, i, 0, 2 * d + 8, d)).astype(np.float32) for i, d in enumerate(ds)]
    fd = [dev(f) for f in fs]
    need = k.kfac_invert_batched_workspace(fd, [torch.empty_like(f) for f in fd])
    results = []
    for fill in (0.0, float("nan"), float("inf"), -1.0e30):
        ws = torch.full((need // 4 + 64,), fill, dtype=torch.float32, device="cuda")
        invs = [torch.zeros(d, d, device="cuda") for d in ds]
        infos = k.kfac_invert_batched(fd, 1e-3, invs, workspace=ws)
        torch.cuda.synchronize()
        assert np.all(host(infos) == 0), fill
        results.append([host(i) for i in invs])
    for other in results[1:]:
        for a, b in zip(results[0], other):
            assert np.array_equal(a, b)
    for f, inv in zip(fs, results[0]):
        want, _ = oracle.invert(f.astype(np.float64), 1e-3)
        assert oracle.rel_fro(inv, want) <= 1e-4


def test_invert_batch_larger_than_the_launch_descriptors(k, oracle):
    """90 matrices: more than the 72 one launch describes (the batch is run in slices), and in the first slice more
    row bands than one launch of the final product holds.  Every inverse must equal, bit for bit, what a call with
    that matrix alone gives; two of them are compared with the oracle."""
    ds = [2100] * 60 + [96] * 30
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.SEED + 90)
    fd = []
    for d in ds:
        x = torch.randn(2 * d + 8, d, device="cuda", generator=gen)
        f = torch.empty(d, d, device="cuda")
        k.kfac_curvature(x, f, 1.0 / x.shape[0], 0.0)
        fd.append(f)
    invs = [torch.empty(d, d, device="cuda") for d in ds]
    infos = k.kfac_invert_batched(fd, 1e-3, invs)
    assert np.all(host(infos) == 0)
    for i in (0, 17, 59, 60, 89):
        single = torch.empty_like(fd[i])
        assert int(k.kfac_invert(fd[i], 1e-3, single)) == 0
        assert torch.equal(single, invs[i]), i
    for i in (59, 89):
        want, _ = oracle.invert(host(fd[i]).astype(np.float64), 1e-3)
        assert oracle.rel_fro(host(invs[i]), want) <= 1e-4
    for i in range(len(ds)):  # all of them are inverses: residual of a few columns
        cols = [0, ds[i] // 2, ds[i] - 1]
        res = fd[i].double() @ invs[i][:, cols].double() + 1e-3 * invs[i][:, cols].double()
        for c, j in enumerate(cols):
            res[j, c] -= 1.0
        assert float(res.norm(dim=0).max()) <= 1e-4, i


# --------------------------------------------------------------- precondition

@pytest.mark.parametrize("d_out,d_in", [(64, 64), (2, 3), (5, 7), (130, 257), (768, 300), (256, 1024), (1024, 1024)])
def test_precondition_parity(k, oracle, d_out, d_in):
    print("precondition %dx%d" % (d_out, d_in), flush=True)
    rng = np.random.default_rng(d_out * 7 + d_in)
    b = rng.standard_normal((d_out, d_out)).astype(np.float32)
    b = (b + b.T) / 2
    a = rng.standard_normal((d_in, d_in)).astype(np.float32)
    a = (a + a.T) / 2
    g = rng.standard_normal((d_out, d_in)).astype(np.float32)
    out = torch.empty(d_out, d_in, device="cuda")
    k.kfac_precondition(dev(b), dev(a), dev(g), out)
    want = oracle.precondition(b, g, a)
    err = oracle.rel_fro(host(out), want)
    print("  rel_fro", err, flush=True)
    assert err <= 2e-6


def test_precondition_identity_diagonal_and_alias(k):
    d_out, d_in = 150, 260
    g = dev(np.random.default_rng(1).standard_normal((d_out, d_in)).astype(np.float32))
    out = torch.empty_like(g)
    k.kfac_precondition(torch.eye(d_out, device="cuda"), torch.eye(d_in, device="cuda"), g, out)
    assert torch.equal(out, g)
    bd = torch.rand(d_out, device="cuda") + 1
    ad = torch.rand(d_in, device="cuda") + 1
    k.kfac_precondition(torch.diag(bd), torch.diag(ad), g, out)
    want = g * bd[:, None] * ad[None, :]
    assert torch.allclose(out, want, rtol=1e-6, atol=0)
    g2 = g.clone()
    k.kfac_precondition(torch.diag(bd), torch.diag(ad), g2, g2)  # in place
    assert torch.equal(g2, out)


def test_precondition_grouped(k, oracle):
    shapes = [(64, 64), (300, 128), (128, 300), (1, 9)]
    rng = np.random.default_rng(2)
    bs, as_, gs = [], [], []
    for do, di in shapes:
        b = rng.standard_normal((do, do)).astype(np.float32)
        a = rng.standard_normal((di, di)).astype(np.float32)
        bs.append((b + b.T) / 2)
        as_.append((a + a.T) / 2)
        gs.append(rng.standard_normal((do, di)).astype(np.float32))
    outs = [torch.empty(do, di, device="cuda") for do, di in shapes]
    k.kfac_precondition_grouped([dev(b) for b in bs], [dev(a) for a in as_], [dev(g) for g in gs], outs)
    for b, a, g, o in zip(bs, as_, gs, outs):
        assert oracle.rel_fro(host(o), oracle.precondition(b, g, a)) <= 2e-6


def test_precondition_grouped_many_ragged_problems(k, oracle):
    """More problems than one launch descriptor holds, ragged sizes, layers of different width (the launches are
    dealt over the XCDs problem by problem, with tile counts that do not divide by eight)."""
    shapes = [(1000, 1300), (700, 2100), (384, 520)] + [(130, 257), (65, 129), (257, 130)] * 17
    rng = np.random.default_rng(3)
    bs, as_, gs = [], [], []
    for do, di in shapes:
        b = rng.standard_normal((do, do)).astype(np.float32)
        a = rng.standard_normal((di, di)).astype(np.float32)
        bs.append((b + b.T) / 2)
        as_.append((a + a.T) / 2)
        gs.append(rng.standard_normal((do, di)).astype(np.float32))
    outs = [torch.full((do, di), 7.0, device="cuda") for do, di in shapes]
    k.kfac_precondition_grouped([dev(b) for b in bs], [dev(a) for a in as_], [dev(g) for g in gs], outs)
    worst = 0.0
    for b, a, g, o in zip(bs, as_, gs, outs):
        worst = max(worst, oracle.rel_fro(host(o), oracle.precondition(b, g, a)))
    print("  %d problems, worst rel_fro %.2e" % (len(shapes), worst), flush=True)
    assert worst <= 2e-6


# ---------------------------------------------------------------- whole chain

def run_chain(k, oracle, cfg_id, layers=None):
    c = synth.CONFIGS[cfg_id]
    worst = 0.0
    for li, (name, d_in, d_out, gelu) in enumerate(c["layers"]):
        if layers is not None and name not in layers:
            continue
        n = c["tokens"]
        x = synth.activations(cfg_id, 0, li, 0, n, d_in, gelu=gelu)
        e = synth.errors(cfg_id, 0, li, 0, n, d_out)
        g = synth.weight_gradient([e], [x])
        xd, ed, gd = dev(x), dev(e), dev(g)
        a = torch.empty(d_in, d_in, device="cuda")
        b = torch.empty(d_out, d_out, device="cuda")
        k.kfac_curvature(xd, a, 1.0 / n, 0.0)
        k.kfac_curvature(ed, b, 1.0 / n, 0.0)
        ai, bi = torch.empty_like(a), torch.empty_like(b)
        info_a = k.kfac_invert(a, synth.DAMPING, ai)
        info_b = k.kfac_invert(b, synth.DAMPING, bi)
        p = torch.empty_like(gd)
        k.kfac_precondition(bi, ai, gd, p)
        assert int(info_a[0]) == 0 and int(info_b[0]) == 0
        oa, ob, oai, obi, op = oracle.kfac_chain([x], [e], g, synth.DAMPING)
        ea, eb = oracle.rel_fro(host(a), oa), oracle.rel_fro(host(b), ob)
        eai, ebi = oracle.rel_fro(host(ai), oai), oracle.rel_fro(host(bi), obi)
        ep = oracle.rel_fro(host(p), op)
        print("cfg %d %-5s A %.2e B %.2e A^-1 %.2e B^-1 %.2e P %.2e" % (cfg_id, name, ea, eb, eai, ebi, ep), flush=True)
        assert ea <= FACTOR_TOL and eb <= FACTOR_TOL
        assert ep <= PRECOND_TOL
        worst = max(worst, ep)
    return worst


def test_chain_config1_and_kronecker(k, oracle):
    run_chain(k, oracle, 1)
    # the GPU result against the explicit Kronecker solve
    c = synth.CONFIGS[1]
    x = synth.activations(1, 0, 0, 0, c["tokens"], 64)
    e = synth.errors(1, 0, 0, 0, c["tokens"], 64)
    g = synth.weight_gradient([e], [x])
    a = torch.empty(64, 64, device="cuda")
    b = torch.empty(64, 64, device="cuda")
    k.kfac_curvature(dev(x), a, 1.0 / 256, 0.0)
    k.kfac_curvature(dev(e), b, 1.0 / 256, 0.0)
    ai, bi = torch.empty_like(a), torch.empty_like(b)
    k.kfac_invert(a, synth.DAMPING, ai)
    k.kfac_invert(b, synth.DAMPING, bi)
    p = torch.empty(64, 64, device="cuda")
    k.kfac_precondition(bi, ai, dev(g), p)
    brute = oracle.kron_solve(oracle.curvature(x), oracle.curvature(e), g, synth.DAMPING)
    assert oracle.rel_fro(host(p), brute) <= PRECOND_TOL


def test_chain_config2_bert_base_block(k, oracle):
    run_chain(k, oracle, 2)


def test_chain_config3_bert_large_block(k, oracle):
    # the hard case for conditioning: FFN2's A factor has d = tokens = 4096 (smallest eigenvalue ~ damping)
    run_chain(k, oracle, 3)


# --------------------------------------------------- bf16 activations / errors

BF16_FACTOR_TOL = 2e-2


@pytest.mark.parametrize("n,d", [(256, 64), (1000, 300), (2048, 1024), (517, 129)])
def test_curvature_bf16_inputs(k, oracle, n, d):
    # the oracle sees the same bf16-rounded values, widened exactly; products of bf16 values are exact in fp32
    x = synth.activations(5, 0, 0, 0, n, d, gelu=(d % 2 == 1), bf16=True)
    xd = dev(x).to(torch.bfloat16)
    assert torch.equal(xd.float().cpu(), torch.from_numpy(x))
    f = torch.empty(d, d, device="cuda")
    k.kfac_curvature(xd, f, 1.0 / n, 0.0)
    err = oracle.rel_fro(host(f), oracle.curvature(x))
    print("bf16 curvature n=%d d=%d rel_fro %.3g" % (n, d, err), flush=True)
    assert err <= BF16_FACTOR_TOL and err <= 5e-7
    assert np.array_equal(host(f), host(f).T)
    # against the un-rounded fp32 inputs the error is the input rounding, far inside the gate
    x32 = synth.activations(5, 0, 0, 0, n, d, gelu=(d % 2 == 1), bf16=False)
    assert oracle.rel_fro(host(f), oracle.curvature(x32)) <= BF16_FACTOR_TOL
    # strided bf16 input (odd offset: rows not 8-byte aligned)
    big = dev(synth.activations(5, 0, 1, 0, n, d + 9, bf16=True)).to(torch.bfloat16)
    xs = big[:, 3:3 + d]
    k.kfac_curvature(xs, f, 1.0 / n, 0.0)
    assert oracle.rel_fro(host(f), oracle.curvature(host(xs.float()))) <= 5e-7


def test_curvature_bf16_hadamard_exact(k):
    x = dev(synth.hadamard_columns(1024, 512)).to(torch.bfloat16)
    f = torch.empty(512, 512, device="cuda")
    k.kfac_curvature(x, f, 1.0 / 1024, 0.0)
    assert np.array_equal(host(f), np.eye(512, dtype=np.float32))


def test_chain_config5_bf16_attention_layer(k, oracle):
    # stress workload, one attention linear (2048 x 2048, 8192 tokens, bf16 activations and errors)
    c = synth.CONFIGS[5]
    n, d = c["tokens"], 2048
    x = synth.activations(5, 0, 0, 0, n, d, bf16=True)
    e = synth.errors(5, 0, 0, 0, n, d, bf16=True)
    g = synth.weight_gradient([e], [x])
    a = torch.empty(d, d, device="cuda")
    b = torch.empty(d, d, device="cuda")
    k.kfac_curvature_grouped([dev(x).to(torch.bfloat16), dev(e).to(torch.bfloat16)], [a, b], 1.0 / n, 0.0)
    ai, bi = torch.empty_like(a), torch.empty_like(b)
    infos = k.kfac_invert_batched([a, b], synth.DAMPING, [ai, bi])
    p = torch.empty(d, d, device="cuda")
    k.kfac_precondition(bi, ai, dev(g), p)
    assert host(infos).tolist() == [0, 0]
    oa, ob, oai, obi, op = oracle.kfac_chain([x], [e], g, synth.DAMPING)
    ea, eb, ep = oracle.rel_fro(host(a), oa), oracle.rel_fro(host(b), ob), oracle.rel_fro(host(p), op)
    print("cfg 5 attention layer: A %.2e B %.2e P %.2e" % (ea, eb, ep), flush=True)
    assert ea <= BF16_FACTOR_TOL and eb <= BF16_FACTOR_TOL and ep <= PRECOND_TOL


# ------------------------------------------------ chunked inversion (plan API)

def test_invert_plan_equals_batched_and_can_be_cut_anywhere(k, oracle):
    ds = [64, 300, 513, 1024]
    fs = [oracle.curvature(synth.activations(2, 2, i, 0, 2 * d + 8, d)).astype(np.float32) for i, d in enumerate(ds)]
    fd = [dev(f) for f in fs]
    ref = [torch.empty(d, d, device="cuda") for d in ds]
    infos = k.kfac_invert_batched(fd, 1e-3, ref)
    assert np.all(host(infos) == 0)
    out = [torch.full((d, d), 5.0, device="cuda") for d in ds]
    plan = k.InvertPlan(fd, 1e-3, out)
    n = plan.steps
    assert n > 10 and plan.position == 0
    flops = [plan.step_flops(i) for i in range(n)]
    assert all(f >= 0 for f in flops) and plan.step_flops(n) == -1.0
    # model cost: d^3 per matrix (the LAPACK count of the three phases; triangular work at its useful share)
    assert 0.9 * sum(d ** 3 for d in ds) <= sum(flops) <= 1.3 * sum(d ** 3 for d in ds)
    side = torch.cuda.Stream()
    rng = np.random.default_rng(0)
    while plan.position < n:
        before = plan.position
        # the inverse is not touched before the last launches
        if before < n - 2:
            assert all(bool(torch.all(o == 5.0)) for o in out)
        plan.run(int(rng.integers(1, 7)))
        torch.cuda.synchronize()
        # unrelated work on another stream between the pieces
        with torch.cuda.stream(side):
            torch.zeros(1 << 20, device="cuda").add_(1.0)
        side.synchronize()
        assert plan.position > before
    assert plan.position == n
    for o, r in zip(out, ref):
        assert torch.equal(o, r)  # bitwise: the same launches in the same order
    assert np.all(host(plan.infos) == 0)
    # and what the pieces add up to is the inverse the oracle computes
    for f, o in zip(fs, out):
        want, _ = oracle.invert(f.astype(np.float64), 1e-3)
        cond = np.linalg.cond(f.astype(np.float64) + 1e-3 * np.eye(f.shape[0]))
        err = oracle.rel_fro(host(o), want)
        print("  plan d=%d cond %.3g rel_fro %.3g" % (f.shape[0], cond, err), flush=True)
        assert err <= 2e-6 * cond + 1e-6
    # a plan can be run again after a reset (next refresh)
    for o in out:
        o.fill_(0.0)
    plan.reset()
    plan.run(n)
    torch.cuda.synchronize()
    for o, r in zip(out, ref):
        assert torch.equal(o, r)
    plan.close()


# ----------------------------------------- K-block-diagonal factors (appendix)

def test_block_diagonal_factors(k, oracle):
    # appendix A.2: a factor of size K*d is replaced by K independent blocks of size d; every step of the
    # path then runs on the blocks, addressed inside the big arrays through leading dimensions
    n, d_in, d_out, kb = 600, 384, 256, 2
    x = synth.activations(2, 3, 0, 0, n, d_in)
    e = synth.errors(2, 3, 0, 0, n, d_out, scale=1.0)
    g = synth.weight_gradient([e], [x])
    xd, ed, gd = dev(x), dev(e), dev(g)
    a = torch.zeros(d_in, d_in, device="cuda")
    b = torch.zeros(d_out, d_out, device="cuda")
    bi, bo = d_in // kb, d_out // kb
    xs = [xd[:, i * bi:(i + 1) * bi] for i in range(kb)] + [ed[:, i * bo:(i + 1) * bo] for i in range(kb)]
    fblocks = [a[i * bi:(i + 1) * bi, i * bi:(i + 1) * bi] for i in range(kb)] + \
              [b[i * bo:(i + 1) * bo, i * bo:(i + 1) * bo] for i in range(kb)]
    k.kfac_curvature_grouped(xs, fblocks, 1.0 / n, 0.0)
    ai, binv = torch.zeros_like(a), torch.zeros_like(b)
    iblocks = [ai[i * bi:(i + 1) * bi, i * bi:(i + 1) * bi] for i in range(kb)] + \
              [binv[i * bo:(i + 1) * bo, i * bo:(i + 1) * bo] for i in range(kb)]
    infos = k.kfac_invert_batched(fblocks, 1e-2, iblocks)
    assert np.all(host(infos) == 0)
    p = torch.empty_like(gd)
    items = [(io, ii) for io in range(kb) for ii in range(kb)]
    k.kfac_precondition_grouped([iblocks[kb + io] for io, ii in items], [iblocks[ii] for io, ii in items],
                                [gd[io * bo:(io + 1) * bo, ii * bi:(ii + 1) * bi] for io, ii in items],
                                [p[io * bo:(io + 1) * bo, ii * bi:(ii + 1) * bi] for io, ii in items])
    # oracle: the dense factors with the off-diagonal blocks set to zero
    oa, ob = oracle.curvature(x), oracle.curvature(e)
    ma, mb = np.zeros_like(oa), np.zeros_like(ob)
    for i in range(kb):
        ma[i * bi:(i + 1) * bi, i * bi:(i + 1) * bi] = oa[i * bi:(i + 1) * bi, i * bi:(i + 1) * bi]
        mb[i * bo:(i + 1) * bo, i * bo:(i + 1) * bo] = ob[i * bo:(i + 1) * bo, i * bo:(i + 1) * bo]
    assert oracle.rel_fro(host(a), ma) <= FACTOR_TOL and oracle.rel_fro(host(b), mb) <= FACTOR_TOL
    oai, _ = oracle.invert(ma, 1e-2)
    obi, _ = oracle.invert(mb, 1e-2)
    assert oracle.rel_fro(host(ai), oai) <= 1e-4 and oracle.rel_fro(host(binv), obi) <= 1e-4
    assert oracle.rel_fro(host(p), oracle.precondition(obi, g, oai)) <= PRECOND_TOL


def test_inversion_and_precondition_are_deterministic(k, oracle):
    d = 640
    a = dev(oracle.curvature(synth.activations(2, 4, 0, 0, 1500, d, gelu=True)).astype(np.float32))
    g = dev(np.random.default_rng(3).standard_normal((d, d)).astype(np.float32))
    first_inv = first_p = None
    for _ in range(3):
        inv = torch.empty(d, d, device="cuda")
        k.kfac_invert(a, 1e-3, inv)
        p = torch.empty(d, d, device="cuda")
        k.kfac_precondition(inv, inv, g, p)
        if first_inv is None:
            first_inv, first_p = inv.clone(), p.clone()
        assert torch.equal(inv, first_inv) and torch.equal(p, first_p)


def test_chain_config5_largest_factor(k, oracle):
    # the largest and worst conditioned factor of all workloads: the second feed-forward linear of the stress
    # block, A is 8192 x 8192 from 8192 bf16 GELU tokens (smallest eigenvalue about the damping)
    c = synth.CONFIGS[5]
    n, d_in, d_out = c["tokens"], 8192, 2048
    print("generating", flush=True)
    x = synth.activations(5, 0, 5, 0, n, d_in, gelu=True, bf16=True)
    e = synth.errors(5, 0, 5, 0, n, d_out, bf16=True)
    g = synth.weight_gradient([e], [x])
    a = torch.empty(d_in, d_in, device="cuda")
    b = torch.empty(d_out, d_out, device="cuda")
    k.kfac_curvature_grouped([dev(x).to(torch.bfloat16), dev(e).to(torch.bfloat16)], [a, b], 1.0 / n, 0.0)
    ai, bi = torch.empty_like(a), torch.empty_like(b)
    infos = k.kfac_invert_batched([a, b], synth.DAMPING, [ai, bi])
    p = torch.empty(d_out, d_in, device="cuda")
    k.kfac_precondition(bi, ai, dev(g), p)
    torch.cuda.synchronize()
    assert host(infos).tolist() == [0, 0]
    print("oracle chain (8192-dimensional inverse in fp64)", flush=True)
    oa, ob, oai, obi, op = oracle.kfac_chain([x], [e], g, synth.DAMPING)
    ea, eb = oracle.rel_fro(host(a), oa), oracle.rel_fro(host(b), ob)
    eai, ep = oracle.rel_fro(host(ai), oai), oracle.rel_fro(host(p), op)
    print("cfg 5 ffn2: A %.2e B %.2e A^-1 %.2e P %.2e" % (ea, eb, eai, ep), flush=True)
    assert ea <= BF16_FACTOR_TOL and eb <= BF16_FACTOR_TOL and ep <= PRECOND_TOL


def test_curvature_bf16_large_tiles(k, oracle):
    # enough 256 x 256 tiles for the large-tile bf16 kernel; ragged size, accumulation over two micro-batches
    n, d = 600, 5000
    xs = [synth.activations(5, 1, m, 0, n, d, bf16=True) for m in range(2)]
    f = torch.empty(d, d, device="cuda")
    for m, x in enumerate(xs):
        k.kfac_curvature(dev(x).to(torch.bfloat16), f, 1.0 / (2 * n), 0.0 if m == 0 else 1.0)
    err = oracle.rel_fro(host(f), oracle.curvature(xs))
    print("bf16 large tiles rel_fro %.3g" % err, flush=True)
    assert err <= BF16_FACTOR_TOL and err <= 2e-6
    assert np.array_equal(host(f), host(f).T)


@pytest.mark.parametrize("n", [32, 96, 160, 288])
def test_curvature_bf16_rowmajor_tiles(k, oracle, n):
    """Sizes that need no padding take the kernel that reads the row-major input directly (transposing
    LDS reads): 1, 3, 5 and 9 slabs of 32 tokens, a row pitch larger than d, two micro-batches."""
    d = 5120  # 20 x 21 / 2 = 210 tiles of 256 x 256
    xs = [synth.activations(5, 2, m, 0, n, d, bf16=True) for m in range(2)]
    f = torch.empty(d, d, device="cuda")
    for m, x in enumerate(xs):
        buf = torch.zeros(n, d + 64, device="cuda", dtype=torch.bfloat16)
        buf[:, :d] = dev(x).to(torch.bfloat16)
        k.kfac_curvature(buf[:, :d], f, 1.0 / (2 * n), 0.0 if m == 0 else 1.0)
    err = oracle.rel_fro(host(f), oracle.curvature(xs))
    print("bf16 row-major tiles n=%d rel_fro %.3g" % (n, err), flush=True)
    assert err <= BF16_FACTOR_TOL and err <= 2e-6
    assert np.array_equal(host(f), host(f).T)


def test_chain_with_order_one_errors_and_few_tokens(k, oracle):
    """In the configurations B = E^T E / N is tiny against the damping, so B's inverse is almost I / damping
    and the chain hardly exercises it.  Here the errors are O(1) and there are fewer tokens than output
    features, so B is rank-deficient: its inverse spans six orders of magnitude and carries the result."""
    n, d_in, d_out = 384, 320, 640
    x = synth.activations(3, 7, 0, 0, n, d_in, gelu=True)
    e = synth.errors(3, 7, 0, 0, n, d_out, scale=1.0)
    g = synth.weight_gradient([e], [x])
    a, b = torch.empty(d_in, d_in, device="cuda"), torch.empty(d_out, d_out, device="cuda")
    k.kfac_curvature(dev(x), a, 1.0 / n, 0.0)
    k.kfac_curvature(dev(e), b, 1.0 / n, 0.0)
    ai, bi = torch.empty_like(a), torch.empty_like(b)
    infos = k.kfac_invert_batched([a, b], synth.DAMPING, [ai, bi])
    p = torch.empty(d_out, d_in, device="cuda")
    k.kfac_precondition(bi, ai, dev(g), p)
    assert int(infos.abs().max()) == 0
    oa, ob, oai, obi, op = oracle.kfac_chain([x], [e], g, synth.DAMPING)
    errs = [oracle.rel_fro(host(t), o) for t, o in ((a, oa), (b, ob), (ai, oai), (bi, obi), (p, op))]
    print("O(1) errors: A %.2e B %.2e A^-1 %.2e B^-1 %.2e P %.2e" % tuple(errs), flush=True)
    assert errs[0] <= FACTOR_TOL and errs[1] <= FACTOR_TOL and errs[4] <= PRECOND_TOL
    # the Kronecker identity of section 2.3.1 on the GPU's own result: (B + lam I) P (A + lam I) = G
    at = oa + synth.DAMPING * np.eye(d_in)
    bt = ob + synth.DAMPING * np.eye(d_out)
    back = bt @ host(p).astype(np.float64) @ at
    assert oracle.rel_fro(back, g) <= PRECOND_TOL


def test_more_items_than_one_launch_describes(k, oracle):
    """90 inversions (a launch describes 72 matrices) and 60 preconditions (48 problems per launch):
    the calls cut themselves into several launches; every item still equals its single-item result."""
    ds = [96 + 32 * (i % 5) for i in range(90)]
    fs = [oracle.curvature(synth.activations(2, 5, i, 0, d + 40, d)).astype(np.float32) for i, d in enumerate(ds)]
    fd = [dev(f) for f in fs]
    invs = [torch.empty(d, d, device="cuda") for d in ds]
    infos = k.kfac_invert_batched(fd, 1e-2, invs)
    assert np.all(host(infos) == 0)
    for i in (0, 44, 71, 72, 89):
        want, _ = oracle.invert(fs[i].astype(np.float64), 1e-2)
        assert oracle.rel_fro(host(invs[i]), want) <= 1e-4
        single, _ = gpu_invert(k, fs[i], 1e-2)
        assert np.array_equal(single, host(invs[i]))
    # 60 layers: B^-1 = inverses 0..59 padded to a common pairing with A^-1 = inverses 30..89
    b_invs, a_invs = invs[:60], invs[30:90]
    grads = [dev(synth.errors(2, 6, i, 0, b.shape[0], a.shape[0], scale=1.0)) for i, (b, a) in enumerate(zip(b_invs, a_invs))]
    outs = [torch.empty_like(g) for g in grads]
    k.kfac_precondition_grouped(b_invs, a_invs, grads, outs)
    for i in (0, 47, 48, 59):
        want = oracle.precondition(host(b_invs[i]), host(grads[i]), host(a_invs[i]))
        assert oracle.rel_fro(host(outs[i]), want) <= 2e-6
        one = torch.empty_like(outs[i])
        k.kfac_precondition(b_invs[i], a_invs[i], grads[i], one)
        assert torch.equal(one, outs[i])


def test_work_items_follow_the_callers_stream(k, oracle):
    """Everything is enqueued on the stream the caller names: a chain issued on a side stream (default
    priority), with its inputs produced on that stream just before, equals the default-stream result."""
    n, d_in, d_out = 512, 384, 256
    x = dev(synth.activations(2, 0, 0, 0, n, d_in))
    e = dev(synth.errors(2, 0, 0, 0, n, d_out))
    g = dev(synth.weight_gradient([host(e)], [host(x)]))

    def chain(stream, xin, ein):
        a = torch.empty(d_in, d_in, device="cuda")
        b = torch.empty(d_out, d_out, device="cuda")
        k.kfac_curvature(xin, a, 1.0 / n, 0.0, stream=stream)
        k.kfac_curvature(ein, b, 1.0 / n, 0.0, stream=stream)
        ai, bi = torch.empty_like(a), torch.empty_like(b)
        infos = k.kfac_invert_batched([a, b], synth.DAMPING, [ai, bi], stream=stream)
        p = torch.empty_like(g)
        k.kfac_precondition(bi, ai, g, p, stream=stream)
        return a, b, ai, bi, p, infos

    ref = chain(None, x, e)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        x2 = x * 1.0  # produced on the side stream: only stream order makes it visible to the kernels
        e2 = e * 1.0
        got = chain(side, x2, e2)
    side.synchronize()
    for r, o in zip(ref, got):
        assert torch.equal(r, o)
    assert int(got[5].abs().max()) == 0


def test_chain_can_be_captured_in_a_graph(k, oracle):
    """The library allocates nothing and enqueues only kernels, so a whole chain (two curvature work
    items, the batched inversion with its chain of launches, the precondition) can be captured in a HIP
    graph.  Every replay, with eager work and synchronisation in between and fresh inputs written into
    the captured buffers, must equal the eager result bit for bit."""
    n, d_in, d_out = 512, 640, 384
    x = torch.empty(n, d_in, device="cuda")
    e = torch.empty(n, d_out, device="cuda")
    g = torch.empty(d_out, d_in, device="cuda")
    a, b = torch.empty(d_in, d_in, device="cuda"), torch.empty(d_out, d_out, device="cuda")
    ai, bi, p = torch.empty_like(a), torch.empty_like(b), torch.empty_like(g)
    infos = torch.zeros(2, dtype=torch.int32, device="cuda")
    need = max(k.kfac_curvature_grouped_workspace([x, e], [a, b]), k.kfac_invert_batched_workspace([a, b], [ai, bi]),
               k.kfac_precondition_grouped_workspace([bi], [ai], [g], [p]))
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")

    def chain(stream):
        k.kfac_curvature_grouped([x, e], [a, b], 1.0 / n, 0.0, workspace=ws, stream=stream)
        k.kfac_invert_batched([a, b], synth.DAMPING, [ai, bi], infos=infos, workspace=ws, stream=stream)
        k.kfac_precondition(bi, ai, g, p, workspace=ws, stream=stream)

    def fill(mb):
        hx, he = synth.activations(2, 1, 0, mb, n, d_in), synth.errors(2, 1, 0, mb, n, d_out)
        x.copy_(dev(hx))
        e.copy_(dev(he))
        g.copy_(dev(synth.weight_gradient([he], [hx])))

    fill(0)
    chain(None)  # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain(torch.cuda.current_stream())
    for mb in range(3):
        fill(mb)
        chain(None)
        torch.cuda.synchronize()
        want = [t.clone() for t in (a, b, ai, bi, p)]
        for t in (a, b, ai, bi, p):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for w, t in zip(want, (a, b, ai, bi, p)):
            assert torch.equal(w, t)
        assert int(infos.abs().max()) == 0
    op = oracle.kfac_chain([host(x)], [host(e)], host(g), synth.DAMPING)[4]
    assert oracle.rel_fro(host(p), op) <= PRECOND_TOL


def test_mfma_probe_reports_its_work(k):
    """The measurement aid runs, leaves its sink alone and reports 4096 / 32768 flops per MFMA."""
    sink = torch.zeros(64, device="cuda")
    for code, per_mfma in ((0, 4096.0), (1, 32768.0)):
        flops = k.kfac_mfma_probe(code, 50, sink)
        torch.cuda.synchronize()
        assert flops == 256 * 2 * 8 * 4 * 50 * 8 * per_mfma
        flops = k.kfac_mfma_probe(code, 50, sink, random_operands=True)  # 50 rounded up to 52: 13 passes of 4 operand sets
        torch.cuda.synchronize()
        assert flops == 256 * 2 * 8 * 4 * 52 * 8 * per_mfma
    assert float(sink.abs().max()) == 0.0


def test_stage_wise_errors_at_block_shapes(k, oracle):
    """Each stage of the path fed with the oracle's previous-stage output (rounded once to fp32), so that the error a
    kernel adds is seen apart from what the conditioning of its input amplifies: BERT-Large block shapes, the
    attention linear and the second feed-forward linear (4096-dimensional A, smallest eigenvalue about the damping)."""
    c = synth.CONFIGS[3]
    n = c["tokens"]
    for li in (0, 5):
        name, d_in, d_out, gelu = c["layers"][li]
        x = synth.activations(3, 0, li, 0, n, d_in, gelu=gelu)
        e = synth.errors(3, 0, li, 0, n, d_out)
        g = synth.weight_gradient([e], [x])
        oa32 = oracle.curvature(x).astype(np.float32)
        ob32 = oracle.curvature(e).astype(np.float32)
        # inversion alone: GPU and oracle invert the same fp32 matrix
        ai, bi = torch.empty(d_in, d_in, device="cuda"), torch.empty(d_out, d_out, device="cuda")
        infos = k.kfac_invert_batched([dev(oa32), dev(ob32)], synth.DAMPING, [ai, bi])
        assert host(infos).tolist() == [0, 0]
        oai, _ = oracle.invert(oa32.astype(np.float64), synth.DAMPING)
        obi, _ = oracle.invert(ob32.astype(np.float64), synth.DAMPING)
        e_ai, e_bi = oracle.rel_fro(host(ai), oai), oracle.rel_fro(host(bi), obi)
        # precondition alone: GPU and oracle multiply the same fp32 inverses
        oai32, obi32 = oai.astype(np.float32), obi.astype(np.float32)
        p = torch.empty(d_out, d_in, device="cuda")
        k.kfac_precondition(dev(obi32), dev(oai32), dev(g), p)
        want_p = oracle.precondition(obi32, g, oai32)
        e_p = oracle.rel_fro(host(p), want_p)
        cond = np.linalg.cond(oa32.astype(np.float64) + synth.DAMPING * np.eye(d_in))
        # what rounding may cost a product whose terms cancel: |B^-1| |G| |A^-1| against |B^-1 G A^-1|
        cancel = np.linalg.norm(np.abs(obi32).astype(np.float64) @ np.abs(g).astype(np.float64) @ np.abs(oai32).astype(np.float64)) / np.linalg.norm(want_p)
        print("cfg 3 %-5s stage-wise: A^-1 %.2e (cond %.2e)  B^-1 %.2e  P %.2e (cancellation %.1f)"
              % (name, e_ai, cond, e_bi, e_p, cancel), flush=True)
        assert e_ai <= 2e-6 * cond + 1e-6 and e_bi <= 1e-5
        assert e_p <= 1e-6 * cancel + 1e-6  # two fp32 products with chunked accumulation: a few ulp of the terms


# ------- float32 input as three bfloat16 terms (KFAC_F32_BF16X3) or two float16 terms (KFAC_F32_F16X2)

SPLIT_MODES = ["bf16x3", "f16x2"]

SPLIT_FACTOR_TOL = 6e-7  # measured 3.3e-7 at 4096 tokens; the fp32 path is held to 5e-7


@pytest.mark.parametrize("mode", SPLIT_MODES)
@pytest.mark.parametrize("n,d", [(4096, 4096), (600, 5000), (77, 3600), (1, 3584), (4100, 3585)])
def test_curvature_split_bf16_parity(k, oracle, n, d, mode):
    """Two factors with enough 256 x 256 tiles between them for the bf16-MFMA kernel (d >= 3584: 2 x 105),
    ragged sizes, a row pitch larger than d, GELU inputs for the second."""
    print("split curvature %s n=%d d=%d" % (mode, n, d), flush=True)
    xs = [synth.activations(6, 0, i, 0, n, d, gelu=(i == 1)) for i in range(2)]
    bufs = [torch.zeros(n, d + 12, device="cuda") for _ in xs]
    for b, x in zip(bufs, xs):
        b[:, :d] = dev(x)
    fs = [torch.full((d, d), 7.0, device="cuda") for _ in xs]
    k.kfac_curvature_grouped([b[:, :d] for b in bufs], fs, 1.0 / n, 0.0, split_bf16=mode)
    for x, f in zip(xs, fs):
        err = oracle.rel_fro(host(f), oracle.curvature(x))
        print("  rel_fro %.3g" % err, flush=True)
        assert err <= FACTOR_TOL and err <= SPLIT_FACTOR_TOL
        assert np.array_equal(host(f), host(f).T)


@pytest.mark.parametrize("mode", SPLIT_MODES)
def test_curvature_split_bf16_accumulates_and_has_no_bias(k, oracle, mode):
    """Two micro-batches (beta = 0, then 1) at the BERT-Large sizes; the diagonal (a sum of squares, where a
    matrix core that cuts off low bits would show) must not be systematically low."""
    n, d, cnt = 4096, 1024, 24  # 24 x 10 = 240 tiles
    xs = [[synth.activations(6, 1, i, m, n, d) for i in range(cnt)] for m in range(2)]
    fs = [torch.empty(d, d, device="cuda") for _ in range(cnt)]
    for m in range(2):
        k.kfac_curvature_grouped([dev(x) for x in xs[m]], fs, 1.0 / (2 * n), float(m), split_bf16=mode)
    bias = []
    for i in (0, 7, 23):
        want = oracle.curvature([xs[0][i], xs[1][i]])
        got = host(fs[i])
        err = oracle.rel_fro(got, want)
        bias.append(float(np.mean((np.diag(got).astype(np.float64) - np.diag(want)) / np.diag(want))))
        print("  factor %d rel_fro %.3g diagonal bias %.3g" % (i, err, bias[-1]), flush=True)
        assert err <= SPLIT_FACTOR_TOL
        assert np.array_equal(got, got.T)
    assert max(abs(b) for b in bias) <= 2e-7


@pytest.mark.parametrize("mode", SPLIT_MODES)
def test_curvature_split_bf16_small_launch_takes_the_fp32_path(k, oracle, mode):
    """Launches with too few 256 x 256 tiles are computed exactly as KFAC_F32: same bits."""
    n, d = 300, 200
    x = dev(synth.activations(6, 2, 0, 0, n, d))
    f1, f2 = torch.empty(d, d, device="cuda"), torch.empty(d, d, device="cuda")
    k.kfac_curvature(x, f1, 1.0 / n, 0.0, split_bf16=mode)
    k.kfac_curvature(x, f2, 1.0 / n, 0.0)
    assert torch.equal(f1, f2)
    with pytest.raises(k.KfacError):
        k.kfac_curvature(x.to(torch.bfloat16), f1, 1.0 / n, 0.0, split_bf16=mode)


@pytest.mark.parametrize("mode", SPLIT_MODES)
def test_curvature_split_bf16_exact_cases_and_determinism(k, mode):
    """Values that are exact in bfloat16 give the exact factor (the m and l planes are zero); two runs agree
    bit for bit."""
    n, d = 512, 3840
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    x = torch.randint(-3, 4, (n, d), device="cuda", generator=g).float()
    fs = [torch.empty(d, d, device="cuda") for _ in range(2)]
    k.kfac_curvature_grouped([x, x], fs, 1.0, 0.0, split_bf16=mode)
    want = x.double().t() @ x.double()
    assert torch.equal(fs[0].double(), want) and torch.equal(fs[0], fs[1])
    y = torch.randn(n, d, device="cuda", generator=g)
    f3, f4 = torch.empty(d, d, device="cuda"), torch.empty(d, d, device="cuda")
    k.kfac_curvature_grouped([y, x], [f3, fs[0]], 0.5, 0.0, split_bf16=mode)
    k.kfac_curvature_grouped([y, x], [f4, fs[1]], 0.5, 0.0, split_bf16=mode)
    assert torch.equal(f3, f4)


@pytest.mark.parametrize("mode", SPLIT_MODES)
def test_chain_config3_feed_forward_layers_with_split_bf16_curvature(k, oracle, mode):
    """The worst-conditioned factors of the configurations (FFN2's A: d = tokens = 4096, GELU inputs, smallest
    eigenvalue about the damping) built by the bf16-MFMA path, then inverted and applied: the preconditioned
    gradient stays inside its tolerance."""
    c = synth.CONFIGS[3]
    n = c["tokens"]
    lay = [(li, l) for li, l in enumerate(c["layers"]) if l[0] in ("ffn1", "ffn2")]
    assert len(lay) == 2
    xs, es, gs = [], [], []
    for li, (name, d_in, d_out, gelu) in lay:
        xs.append(synth.activations(3, 0, li, 0, n, d_in, gelu=gelu))
        es.append(synth.errors(3, 0, li, 0, n, d_out))
        gs.append(synth.weight_gradient([es[-1]], [xs[-1]]))
    ins = [dev(x) for x in xs] + [dev(e) for e in es]
    facs = [torch.empty(t.shape[1], t.shape[1], device="cuda") for t in ins]
    k.kfac_curvature_grouped(ins, facs, 1.0 / n, 0.0, split_bf16=mode)
    invs = [torch.empty_like(f) for f in facs]
    infos = k.kfac_invert_batched(facs, synth.DAMPING, invs)
    assert int(infos.abs().max()) == 0
    for i, (li, (name, d_in, d_out, gelu)) in enumerate(lay):
        p = torch.empty(d_out, d_in, device="cuda")
        k.kfac_precondition(invs[2 + i], invs[i], dev(gs[i]), p)
        oa, ob, oai, obi, op = oracle.kfac_chain([xs[i]], [es[i]], gs[i], synth.DAMPING)
        ea, eb = oracle.rel_fro(host(facs[i]), oa), oracle.rel_fro(host(facs[2 + i]), ob)
        eai, ep = oracle.rel_fro(host(invs[i]), oai), oracle.rel_fro(host(p), op)
        print("cfg 3 %-5s split curvature: A %.2e B %.2e A^-1 %.2e P %.2e" % (name, ea, eb, eai, ep), flush=True)
        assert ea <= SPLIT_FACTOR_TOL and eb <= SPLIT_FACTOR_TOL
        assert ep <= PRECOND_TOL


@pytest.mark.parametrize("mode", SPLIT_MODES)
def test_curvature_split_bf16_long_inputs_go_in_chunks(k, oracle, mode):
    """More than 8192 tokens: the bf16-MFMA kernel runs once per chunk of 8192 and adds up through the factor, so
    the error stays that of one chunk; items of different lengths drop out of the later launches."""
    d = 3584
    lens = [20000, 9000]
    xs = [synth.activations(6, 3, i, 0, n, d, gelu=(i == 1)) for i, n in enumerate(lens)]
    fs = [torch.zeros(d, d, device="cuda") for _ in xs]  # beta = 1 on zeros: the first chunk must honour beta too
    want = [oracle.curvature(x) * (x.shape[0] * 1e-4) for x in xs]
    k.kfac_curvature_grouped([dev(x) for x in xs], fs, 1e-4, 1.0, split_bf16=mode)
    for n, f, w in zip(lens, fs, want):
        err = oracle.rel_fro(host(f), w)
        print("  %d tokens rel_fro %.3g" % (n, err), flush=True)
        assert err <= SPLIT_FACTOR_TOL
        assert np.array_equal(host(f), host(f).T)


@pytest.mark.parametrize("mode", SPLIT_MODES)
def test_curvature_split_bf16_more_items_than_one_launch_describes(k, oracle, mode):
    """90 items: the first 80 fill a launch of the bf16-MFMA kernel, the other 10 are too few tiles for it and
    take the fp32 path inside the same call."""
    n, d, cnt = 64, 1024, 90
    xs = [synth.activations(6, 4, i, 0, n, d) for i in range(cnt)]
    fs = [torch.empty(d, d, device="cuda") for _ in xs]
    k.kfac_curvature_grouped([dev(x) for x in xs], fs, 1.0 / n, 0.0, split_bf16=mode)
    worst = max(oracle.rel_fro(host(fs[i]), oracle.curvature(xs[i])) for i in (0, 41, 79, 80, 89))
    print("  worst rel_fro %.3g" % worst, flush=True)
    assert worst <= SPLIT_FACTOR_TOL
    ref = torch.empty(d, d, device="cuda")
    k.kfac_curvature(dev(xs[85]), ref, 1.0 / n, 0.0)
    assert torch.equal(ref, fs[85])  # the fp32 path's bits


def test_curvature_f16x2_dynamic_range_and_scaling(k, oracle):
    """The two-float16-term path scales every tensor by a power of two from its largest magnitude: tensors of
    very different sizes in one call (1e-6 .. 1e6), and a tensor with one outlier 10^4 times its typical value
    (the bulk then sits 13 bits lower in the float16 range), keep the error of the ordinary case."""
    n, d = 512, 3584
    scales = [1e-6, 1.0, 1e6]
    xs = [synth.activations(7, 0, i, 0, n, d) * np.float32(sc) for i, sc in enumerate(scales)]
    out = synth.activations(7, 0, 3, 0, n, d).copy()
    out[17, 1234] = 3.0e4
    xs.append(out)
    fs = [torch.empty(d, d, device="cuda") for _ in xs]
    k.kfac_curvature_grouped([dev(x) for x in xs], fs, 1.0 / n, 0.0, split_bf16="f16x2")
    for i, (x, f) in enumerate(zip(xs, fs)):
        want = oracle.curvature(x)
        got = host(f)
        if i == 3:  # judge the bulk apart from the outlier's row and column, which dominate the norm
            keep = np.ones(d, bool)
            keep[1234] = False
            err_bulk = oracle.rel_fro(got[np.ix_(keep, keep)], want[np.ix_(keep, keep)])
            print("  outlier: bulk rel_fro %.3g" % err_bulk, flush=True)
            assert err_bulk <= 5e-6
        err = oracle.rel_fro(got, want)
        print("  tensor %d rel_fro %.3g" % (i, err), flush=True)
        assert err <= SPLIT_FACTOR_TOL


def test_curvature_split_modes_propagate_non_finite_inputs(k):
    """A NaN or an infinity in the input must not give finite numbers in its row and column of the factor."""
    n, d = 64, 3584
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    for mode in SPLIT_MODES:
        for bad in (float("nan"), float("inf")):
            xs = [torch.randn(n, d, device="cuda", generator=g) for _ in range(2)]
            xs[0][5, 100] = bad
            fs = [torch.zeros(d, d, device="cuda") for _ in xs]
            k.kfac_curvature_grouped(xs, fs, 1.0 / n, 0.0, split_bf16=mode)
            assert not bool(torch.isfinite(fs[0][100, :]).any()) and not bool(torch.isfinite(fs[0][:, 100]).any())
            assert bool(torch.isfinite(fs[1]).all())


# ------------------------------------- precondition with operands as two float16 terms (f16 MFMA)

@pytest.mark.parametrize("d_out,d_in", [(64, 64), (2, 3), (5, 7), (130, 257), (768, 300), (256, 1024), (1024, 1024), (1100, 2300)])
def test_precondition_f16x2_parity(k, oracle, d_out, d_in):
    print("precondition f16x2 %dx%d" % (d_out, d_in), flush=True)
    rng = np.random.default_rng(d_out * 7 + d_in)
    b = rng.standard_normal((d_out, d_out)).astype(np.float32)
    b = (b + b.T) / 2
    a = rng.standard_normal((d_in, d_in)).astype(np.float32)
    a = (a + a.T) / 2
    g = rng.standard_normal((d_out, d_in)).astype(np.float32)
    buf = torch.full((d_out, d_in + 5), 7.0, device="cuda")
    out = buf[:, :d_in]
    k.kfac_precondition_grouped([dev(b)], [dev(a)], [dev(g)], [out], f16x2=True)
    want = oracle.precondition(b, g, a)
    err = oracle.rel_fro(host(out), want)
    print("  rel_fro", err, flush=True)
    assert err <= 2e-6
    assert float(buf[:, d_in:].min()) == 7.0  # nothing written past the row


def test_precondition_f16x2_many_ragged_problems_and_scales(k, oracle):
    """More layers than one group of launches takes (40), ragged sizes, operands of very different magnitude
    (inverses of order 1e3 next to gradients of order 1e-6)."""
    shapes = [(1000, 1300), (700, 2100), (384, 520)] + [(130, 257), (65, 129), (257, 130)] * 14
    rng = np.random.default_rng(4)
    bs, as_, gs = [], [], []
    for i, (do, di) in enumerate(shapes):
        b = rng.standard_normal((do, do)).astype(np.float32)
        a = rng.standard_normal((di, di)).astype(np.float32)
        bs.append(((b + b.T) / 2 * np.float32(1e3)).astype(np.float32))
        as_.append(((a + a.T) / 2 * np.float32(10.0 ** (i % 5 - 2))).astype(np.float32))
        gs.append((rng.standard_normal((do, di)) * 1e-6).astype(np.float32))
    outs = [torch.full((do, di), 7.0, device="cuda") for do, di in shapes]
    k.kfac_precondition_grouped([dev(b) for b in bs], [dev(a) for a in as_], [dev(g) for g in gs], outs, f16x2=True)
    worst = 0.0
    for b, a, g, o in zip(bs, as_, gs, outs):
        worst = max(worst, oracle.rel_fro(host(o), oracle.precondition(b, g, a)))
    print("  %d problems, worst rel_fro %.2e" % (len(shapes), worst), flush=True)
    assert worst <= 2e-6


def test_chain_config3_with_f16x2_curvature_and_precondition(k, oracle):
    """The feed-forward layers of the BERT-Large block through both float16-term paths: factors, fp32 inversion,
    preconditioned gradient against the oracle's chain."""
    c = synth.CONFIGS[3]
    n = c["tokens"]
    lay = [(li, l) for li, l in enumerate(c["layers"]) if l[0] in ("ffn1", "ffn2")]
    xs, es, gs = [], [], []
    for li, (name, d_in, d_out, gelu) in lay:
        xs.append(synth.activations(3, 0, li, 0, n, d_in, gelu=gelu))
        es.append(synth.errors(3, 0, li, 0, n, d_out))
        gs.append(synth.weight_gradient([es[-1]], [xs[-1]]))
    ins = [dev(x) for x in xs] + [dev(e) for e in es]
    facs = [torch.empty(t.shape[1], t.shape[1], device="cuda") for t in ins]
    k.kfac_curvature_grouped(ins, facs, 1.0 / n, 0.0, split_bf16="f16x2")
    invs = [torch.empty_like(f) for f in facs]
    infos = k.kfac_invert_batched(facs, synth.DAMPING, invs)
    assert int(infos.abs().max()) == 0
    ps = [torch.empty(l[1][2], l[1][1], device="cuda") for l in lay]
    k.kfac_precondition_grouped([invs[2], invs[3]], [invs[0], invs[1]], [dev(g) for g in gs], ps, f16x2=True)
    for i, (li, (name, d_in, d_out, gelu)) in enumerate(lay):
        op = oracle.kfac_chain([xs[i]], [es[i]], gs[i], synth.DAMPING)[4]
        ep = oracle.rel_fro(host(ps[i]), op)
        print("cfg 3 %-5s f16x2 curvature and precondition: P %.2e" % (name, ep), flush=True)
        assert ep <= PRECOND_TOL


def test_f16x2_paths_can_be_captured_in_a_graph(k):
    """The float16-term curvature and precondition enqueue only kernels too (the largest magnitudes are cleared
    by a kernel and raised with atomics): captured with the fp32 inversion between them, every replay on fresh
    inputs must equal the eager result bit for bit."""
    n, d = 256, 3584  # two factors of 105 tiles of 256 x 256: the bf16/f16 path, not the fp32 fallback
    x = torch.empty(n, d, device="cuda")
    e = torch.empty(n, d, device="cuda")
    g = torch.empty(d, d, device="cuda")
    a, b = torch.empty(d, d, device="cuda"), torch.empty(d, d, device="cuda")
    ai, bi, p = torch.empty_like(a), torch.empty_like(b), torch.empty_like(g)
    infos = torch.zeros(2, dtype=torch.int32, device="cuda")
    need = max(k.kfac_curvature_grouped_workspace([x, e], [a, b], split_bf16="f16x2"),
               k.kfac_invert_batched_workspace([a, b], [ai, bi]),
               k.kfac_precondition_grouped_workspace([bi], [ai], [g], [p], f16x2=True))
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")

    def chain(stream):
        k.kfac_curvature_grouped([x, e], [a, b], 1.0 / n, 0.0, workspace=ws, stream=stream, split_bf16="f16x2")
        k.kfac_invert_batched([a, b], synth.DAMPING, [ai, bi], infos=infos, workspace=ws, stream=stream)
        k.kfac_precondition_grouped([bi], [ai], [g], [p], workspace=ws, stream=stream, f16x2=True)

    gen = torch.Generator(device="cuda")

    def fill(mb):
        gen.manual_seed(100 + mb)
        # the scale changes from replay to replay (modestly: n < d, so the damping alone bounds the condition number)
        x.copy_(torch.randn(n, d, device="cuda", generator=gen) * (1.0, 2.0, 0.5)[mb])
        e.copy_(torch.randn(n, d, device="cuda", generator=gen) * 1e-3)
        g.copy_((e.t() @ x) / n)

    fill(0)
    chain(None)  # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain(torch.cuda.current_stream())
    for mb in range(3):
        fill(mb)
        chain(None)
        torch.cuda.synchronize()
        want = [t.clone() for t in (a, b, ai, bi, p)]
        for t in (a, b, ai, bi, p):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for w, t in zip(want, (a, b, ai, bi, p)):
            assert torch.equal(w, t)
        assert int(infos.abs().max()) == 0
    # (with fewer tokens than features G lies in A's range while A^-1 is largest on its null space: the product
    # cancels 10^4-fold and no fp32 product is accurate to better than 5e-3 here, on either path; the accuracy
    # of the paths is the business of the tests above, this one is about replays)
    assert bool(torch.isfinite(p).all())


def test_precondition_f16x2_with_prepared_inverses(k, oracle):
    """The inverses' float16 planes made once (kfac_precondition_f16x2_prepare) and applied to two different
    gradients give, bit for bit, what the one-call form gives; 45 layers (more than one group of launches)."""
    shapes = [(1000, 1300), (700, 2100), (384, 520)] + [(130, 257), (65, 129), (257, 130)] * 14
    rng = np.random.default_rng(6)
    bs, as_ = [], []
    for do, di in shapes:
        b = rng.standard_normal((do, do)).astype(np.float32)
        a = rng.standard_normal((di, di)).astype(np.float32)
        bs.append(dev((b + b.T) / 2))
        as_.append(dev((a + a.T) / 2))
    prepared = k.PreparedInverses(bs, as_)
    for trial in range(2):
        gs = [dev(rng.standard_normal((do, di)).astype(np.float32) * np.float32(10.0 ** -trial)) for do, di in shapes]
        o1 = [torch.full((do, di), 7.0, device="cuda") for do, di in shapes]
        o2 = [torch.full((do, di), 8.0, device="cuda") for do, di in shapes]
        prepared.precondition(gs, o1)
        k.kfac_precondition_grouped(bs, as_, gs, o2, f16x2=True)
        for x, y in zip(o1, o2):
            assert torch.equal(x, y)
        worst = max(oracle.rel_fro(host(o), oracle.precondition(host(b), host(g), host(a)))
                    for b, a, g, o in list(zip(bs, as_, gs, o1))[:6])
        print("  prepared inverses, trial %d: worst rel_fro %.2e" % (trial, worst), flush=True)
        assert worst <= 2e-6
