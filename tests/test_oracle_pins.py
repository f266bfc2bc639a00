"""Pins for the fp64 oracle: closed forms, brute force, library cross-checks.

Each test fixes the oracle to something other than itself, so that a dropped
term, a wrong sign or index, or a transposed operand fails at least one.
Citations are to the paper's section 2.3 (definition of the factors and of the
Kronecker product) and 2.3.1 (work items and the two Kronecker identities).
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.linalg

from paper_2211_14133_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _spd(rng, d, cond=50.0):
    q, _ = np.linalg.qr(rng.standard_normal((d, d)))
    ev = np.geomspace(1.0, cond, d)
    return (q * ev) @ q.T


# ----------------------------------------------------------------- curvature

def test_curvature_matches_per_example_outer_products(oracle):
    # section 2.3: A = mean over examples of a a^T, written out as python loops
    rng = np.random.default_rng(1)
    x = rng.standard_normal((7, 5))
    want = np.zeros((5, 5))
    for t in range(7):
        for i in range(5):
            for j in range(5):
                want[i, j] += x[t, i] * x[t, j] / 7.0
    assert np.allclose(oracle.curvature(x), want, rtol=0, atol=1e-15)
    assert np.allclose(oracle.curvature_loops(x), want, rtol=0, atol=1e-15)


def test_curvature_symmetric_psd(oracle):
    x = synth.activations(1, 0, 0, 0, 256, 64)
    a = oracle.curvature(x)
    assert np.array_equal(a, a.T)
    assert np.linalg.eigvalsh(a).min() >= -1e-12 * np.linalg.norm(a)


def test_curvature_hadamard_is_identity(oracle):
    # orthogonal +-1 columns: X^T X / n = I exactly
    for n, d in [(64, 64), (256, 100), (1024, 257)]:
        x = synth.hadamard_columns(n, d)
        assert np.array_equal(oracle.curvature(x), np.eye(d))
        assert np.array_equal(oracle.curvature_loops(x), np.eye(d))


def test_curvature_small_integers_exact(oracle):
    rng = np.random.default_rng(2)
    x = rng.integers(-8, 9, size=(300, 17))
    want = np.array([[sum(int(x[t, i]) * int(x[t, j]) for t in range(300)) for j in range(17)] for i in range(17)])
    got = oracle.curvature_update(x.astype(np.float32), 1.0, 0.0)
    assert np.array_equal(got, want.astype(np.float64))
    assert oracle.curvature_entry(x.astype(np.float32), 3, 11, 1.0) == float(want[3, 11])


def test_curvature_ones_and_one_hot(oracle):
    assert np.array_equal(oracle.curvature(np.ones((16, 6))), np.ones((6, 6)))
    idx = np.array([0, 2, 2, 3, 3, 3, 5, 5])
    x = np.zeros((8, 6))
    x[np.arange(8), idx] = 1.0
    want = np.diag(np.bincount(idx, minlength=6) / 8.0)
    assert np.array_equal(oracle.curvature(x), want)


def test_curvature_not_transposed(oracle):
    # rectangular input: the factor is d x d (features), never tokens x tokens
    x = np.arange(12, dtype=np.float64).reshape(4, 3)
    a = oracle.curvature(x)
    assert a.shape == (3, 3)
    assert a[0, 1] == (0 * 1 + 3 * 4 + 6 * 7 + 9 * 10) / 4.0


def test_curvature_microbatch_accumulation(oracle):
    # section 3.1: one curvature work item per micro-batch; the factor is the mean over the mini-batch
    xs = [synth.activations(1, 0, 0, m, 96, 40) for m in range(4)]
    whole = oracle.curvature(np.concatenate(xs, 0))
    parts = oracle.curvature(xs)
    assert np.allclose(parts, whole, rtol=1e-14, atol=1e-15)
    alpha = 1.0 / (4 * 96)
    f = None
    for m, x in enumerate(xs):
        f = oracle.curvature_update(x, alpha, 0.0 if m == 0 else 1.0, f)
    assert np.allclose(f, whole, rtol=1e-14, atol=1e-15)
    g = None
    for m, x in enumerate(xs):
        g = oracle.curvature_loops(x, alpha, 0.0 if m == 0 else 1.0, g)
    assert np.allclose(g, whole, rtol=1e-14, atol=1e-15)


def test_curvature_alpha_beta(oracle):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((20, 6))
    f0 = rng.standard_normal((6, 6))
    want = 0.25 * f0 + 3.0 * np.einsum("ti,tj->ij", x, x)
    assert np.allclose(oracle.curvature_update(x, 3.0, 0.25, f0), want, rtol=1e-14)
    assert np.allclose(oracle.curvature_loops(x, 3.0, 0.25, f0), want, rtol=1e-14)


# ----------------------------------------------------------------- inversion

def test_invert_by_hand_small(oracle):
    inv, info = oracle.invert(np.array([[3.0]]), 1.0)
    assert info == 0 and inv[0, 0] == 0.25
    inv, info = oracle.invert(np.array([[2.0, 1.0], [1.0, 2.0]]), 0.0)
    assert np.allclose(inv, np.array([[2.0, -1.0], [-1.0, 2.0]]) / 3.0, rtol=1e-15)
    # 3x3: M = [[4,2,0],[2,5,2],[0,2,5]] -> L = [[2,0,0],[1,2,0],[0,1,2]]
    m = np.array([[4.0, 2, 0], [2, 5, 2], [0, 2, 5]])
    l, info = oracle.cholesky(m)
    assert info == 0 and np.array_equal(l, np.array([[2.0, 0, 0], [1, 2, 0], [0, 1, 2]]))
    inv, _ = oracle.invert(m, 0.0)
    want = np.array([[21.0, -10, 4], [-10, 20, -8], [4, -8, 16]]) / 64.0
    assert np.allclose(inv, want, rtol=1e-15)


def test_invert_closed_forms(oracle):
    d = 37
    inv, _ = oracle.invert(np.zeros((d, d)), 4.0)  # damping alone: (cI)^-1 = I/c
    assert np.array_equal(inv, np.eye(d) / 4.0)
    inv, _ = oracle.invert(np.diag(np.arange(1.0, d + 1)), 1.0)
    assert np.allclose(inv, np.diag(1.0 / np.arange(2.0, d + 2)), rtol=1e-15, atol=0)
    # alpha I + beta 11^T (Sherman-Morrison)
    al, be = 0.7, 0.3
    inv, _ = oracle.invert(be * np.ones((d, d)), al)
    want = (np.eye(d) - be / (al + be * d) * np.ones((d, d))) / al
    assert np.allclose(inv, want, rtol=1e-12, atol=1e-14)
    # M_ij = min(i,j): L = ones lower triangle, inverse = second-difference matrix with last entry 1
    i = np.arange(1, d + 1)
    m = np.minimum.outer(i, i).astype(np.float64)
    l, info = oracle.cholesky(m)
    assert info == 0 and np.array_equal(l, np.tril(np.ones((d, d))))
    inv, _ = oracle.invert(m, 0.0)
    want = 2 * np.eye(d) - np.eye(d, k=1) - np.eye(d, k=-1)
    want[-1, -1] = 1.0
    assert np.allclose(inv, want, rtol=0, atol=1e-12)
    # tridiag(-1,2,-1)^-1_ij = min(i,j) (d+1-max(i,j)) / (d+1)
    t = 2 * np.eye(d) - np.eye(d, k=1) - np.eye(d, k=-1)
    inv, _ = oracle.invert(t, 0.0)
    want = np.minimum.outer(i, i) * (d + 1 - np.maximum.outer(i, i)) / (d + 1.0)
    assert np.allclose(inv, want, rtol=1e-12)


@pytest.mark.parametrize("d", [1, 2, 3, 63, 64, 65, 127, 128, 129, 255, 257])
def test_invert_residual_and_library(oracle, d):
    rng = np.random.default_rng(100 + d)
    m = _spd(rng, d, cond=1e3)
    lam = 1e-3
    inv, info = oracle.invert(m, lam)
    assert info == 0
    mt = m + lam * np.eye(d)
    assert np.linalg.norm(mt @ inv - np.eye(d)) / np.sqrt(d) < 1e-11
    assert np.linalg.norm(inv @ mt - np.eye(d)) / np.sqrt(d) < 1e-11
    assert np.linalg.norm(inv - inv.T) <= 1e-12 * np.linalg.norm(inv)
    lib = scipy.linalg.cho_solve(scipy.linalg.cho_factor(mt, lower=True), np.eye(d))
    assert np.linalg.norm(inv - lib) <= 1e-11 * np.linalg.norm(lib)
    assert np.linalg.norm(inv - np.linalg.inv(mt)) <= 1e-11 * np.linalg.norm(lib)


def test_invert_block_edges_768(oracle):
    for d in (767, 768, 769):
        x = synth.activations(2, 0, 0, 0, 1024, d)
        a = oracle.curvature(x)
        inv, info = oracle.invert(a, 1e-3)
        assert info == 0
        at = a + 1e-3 * np.eye(d)
        assert np.linalg.norm(at @ inv - np.eye(d)) / np.sqrt(d) < 1e-10
        assert np.linalg.norm(inv - np.linalg.inv(at)) <= 1e-10 * np.linalg.norm(inv)


def test_cholesky_is_lower_and_reproduces(oracle):
    rng = np.random.default_rng(7)
    m = _spd(rng, 50)
    l, info = oracle.cholesky(m)
    assert info == 0 and np.array_equal(l, np.tril(l))
    assert np.allclose(l @ l.T, m, rtol=1e-13, atol=1e-13)
    assert np.allclose(l, np.linalg.cholesky(m), rtol=1e-12, atol=1e-13)


def test_invert_damping_goes_on_the_diagonal(oracle):
    rng = np.random.default_rng(8)
    m = _spd(rng, 12)
    a, _ = oracle.invert(m, 0.5)
    b, _ = oracle.invert(m + 0.5 * np.eye(12), 0.0)
    assert np.allclose(a, b, rtol=1e-13)


def test_invert_reports_failing_pivot(oracle):
    m = np.eye(6)
    m[3, 3] = -1.0
    inv, info = oracle.invert(m, 0.0)
    assert inv is None and info == 4
    # rank-deficient without damping: x x^T with one example fails at the second pivot
    x = np.array([[1.0, 2.0, 3.0]])
    inv, info = oracle.invert(oracle.curvature(x), 0.0)
    assert info == 2
    inv, info = oracle.invert(oracle.curvature(x), 1e-3)
    assert info == 0


# -------------------------------------------------------------- precondition

def test_precondition_identity_and_diagonal(oracle):
    rng = np.random.default_rng(9)
    g = rng.standard_normal((5, 7))
    assert np.array_equal(oracle.precondition(np.eye(5), g, np.eye(7)), g)
    b = rng.uniform(1, 2, 5)
    a = rng.uniform(1, 2, 7)
    want = g * b[:, None] * a[None, :]
    assert np.allclose(oracle.precondition(np.diag(b), g, np.diag(a)), want, rtol=1e-15)
    assert np.allclose(oracle.precondition_loops(np.diag(b), g, np.diag(a)), want, rtol=1e-15)


def test_precondition_operand_order(oracle):
    # non-commuting, non-symmetric operands: B on the left, A on the right
    b = np.array([[1.0, 2.0], [0.0, 1.0]])
    a = np.array([[1.0, 0.0, 0.0], [3.0, 1.0, 0.0], [0.0, 0.0, 1.0]])
    g = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])
    want = np.zeros((2, 3))
    for i in range(2):
        for j in range(3):
            for k in range(2):
                for l in range(3):
                    want[i, j] += b[i, k] * g[k, l] * a[l, j]
    assert np.array_equal(oracle.precondition(b, g, a), want)
    assert np.array_equal(oracle.precondition_loops(b, g, a), want)


def test_precondition_golden_fractions(oracle):
    rows = []
    with open(os.path.join(GOLDEN, "kron_2x2_exact.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append([float(Fraction(tok)) for tok in line.split()])
    want = np.array(rows)
    a = np.array([[2.0, 1.0], [1.0, 2.0]])
    b = np.array([[3.0, 1.0], [1.0, 2.0]])
    g = np.array([[1.0, 2.0], [3.0, 4.0]])
    a_inv, _ = oracle.invert(a, 0.0)
    b_inv, _ = oracle.invert(b, 0.0)
    assert np.allclose(oracle.precondition(b_inv, g, a_inv), want, rtol=1e-14)
    assert np.allclose(oracle.kron_solve(a, b, g, 0.0), want, rtol=1e-14)


@pytest.mark.parametrize("d_out,d_in", [(2, 3), (3, 2), (5, 7), (1, 4)])
def test_kronecker_identity_rectangular(oracle, d_out, d_in):
    # section 2.3.1: (A (x) B)^-1 vec(G) = vec(B^-1 G A^-1); catches d_in/d_out swaps and vec order
    rng = np.random.default_rng(10 * d_out + d_in)
    a = _spd(rng, d_in)
    b = _spd(rng, d_out)
    g = rng.standard_normal((d_out, d_in))
    lam = 0.05
    a_inv, _ = oracle.invert(a, lam)
    b_inv, _ = oracle.invert(b, lam)
    p = oracle.precondition(b_inv, g, a_inv)
    assert np.allclose(oracle.kron_solve(a, b, g, lam), p, rtol=1e-10, atol=1e-13)
    # library cross-check with numpy's own Kronecker product (block (j,j') = At[j,j'] * Bt)
    k = np.kron(a + lam * np.eye(d_in), b + lam * np.eye(d_out))
    sol = np.linalg.solve(k, g.reshape(-1, order="F")).reshape((d_out, d_in), order="F")
    assert np.allclose(sol, p, rtol=1e-10, atol=1e-13)


def test_kronecker_identity_config1(oracle):
    # the 64 x 64 layer of the smallest workload: explicit 4096 x 4096 Kronecker system
    c = synth.CONFIGS[1]
    x = synth.activations(1, 0, 0, 0, c["tokens"], 64)
    e = synth.errors(1, 0, 0, 0, c["tokens"], 64)
    g = synth.weight_gradient([e], [x])
    a, b, a_inv, b_inv, p = oracle.kfac_chain([x], [e], g, synth.DAMPING)
    brute = oracle.kron_solve(a, b, g, synth.DAMPING)
    assert oracle.rel_fro(p, brute) < 1e-9


def test_precondition_linearity_and_roundtrip(oracle):
    rng = np.random.default_rng(11)
    a, b = _spd(rng, 9), _spd(rng, 6)
    a_inv, _ = oracle.invert(a, 0.0)
    b_inv, _ = oracle.invert(b, 0.0)
    g1, g2 = rng.standard_normal((2, 6, 9))
    p = oracle.precondition(b_inv, 2.0 * g1 - 3.0 * g2, a_inv)
    assert np.allclose(p, 2.0 * oracle.precondition(b_inv, g1, a_inv) - 3.0 * oracle.precondition(b_inv, g2, a_inv), rtol=1e-12)
    h = rng.standard_normal((6, 9))
    assert np.allclose(oracle.precondition(b_inv, b @ h @ a, a_inv), h, rtol=1e-10, atol=1e-12)


def test_precondition_loops_match_matmul(oracle):
    rng = np.random.default_rng(12)
    b = rng.standard_normal((11, 11))
    a = rng.standard_normal((13, 13))
    g = rng.standard_normal((11, 13))
    assert np.allclose(oracle.precondition(b, g, a), oracle.precondition_loops(b, g, a), rtol=1e-13, atol=1e-13)


# ------------------------------------------------------------------- inputs

def test_synthetic_inputs_are_reproducible_and_shaped():
    x1 = synth.activations(3, 0, 5, 0, 128, 32, gelu=True)
    x2 = synth.activations(3, 0, 5, 0, 128, 32, gelu=True)
    assert x1.dtype == np.float32 and np.array_equal(x1, x2)
    assert not np.array_equal(x1, synth.activations(3, 0, 4, 0, 128, 32, gelu=True))
    z = synth.standard_normal(42, 1 << 18)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01
    g = synth.gelu_exact(z)
    assert abs(g.mean() - 0.2819) < 0.01 and abs((g * g).mean() - 0.4251) < 0.01
    e = synth.errors(3, 0, 5, 0, 4096, 16)
    assert abs(e.std() - 1e-3) < 5e-5
    b = synth.round_to_bf16(x1)
    assert np.all((b.view(np.uint32) & 0xFFFF) == 0) and np.max(np.abs(b - x1) / np.maximum(np.abs(x1), 1e-30)) <= 2.0 ** -8
