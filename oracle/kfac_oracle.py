"""fp64 CPU oracle for the K-FAC work that PipeFisher places into pipeline bubbles.

TEST INFRASTRUCTURE ONLY.  The product path (the HIP library and its Python
binding) never imports this module; only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg do.  It shares no code with the HIP path.

Every function is the plain definition from section 2.3 / 2.3.1 of the paper,
evaluated in float64:

* ``curvature``       A = <a a^T>, B = <e e^T> over the examples of the
                      mini-batch (definition of A_l, B_l; A = U_A U_A^T with
                      U_A the concatenated per-example vectors over
                      sqrt(|B|)).  Every token row counts as one example.
                      The matrix product is numpy's float64 matmul.
* ``invert``          (factor + damping I)^-1 by Cholesky decomposition and
                      the inverse from the Cholesky factor (the paper's
                      cholesky / cholesky_inverse pair), textbook loops in C.
                      Damping is not in the paper: it is added to each
                      factor's diagonal (this build's stated reading).
* ``precondition``    B^-1 G A^-1, two float64 matmuls.
* ``kron_solve``      tiny sizes only: the Kronecker product is formed
                      explicitly and the linear system is solved, which checks
                      (A (x) B)^-1 vec(G) = vec(B^-1 G A^-1) with the paper's
                      column-stacking vec.

Pins: see tests/test_oracle_pins.py (closed forms, brute force, library
cross-checks, the explicit Kronecker solve).  No function here is unpinned.
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        i64, f64, p = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_curvature.argtypes = [p, i64, i64, i64, f64, f64, p, i64]
        lib.oracle_curvature.restype = None
        lib.oracle_cholesky.argtypes = [p, i64, i64, p, i64]
        lib.oracle_cholesky.restype = i64
        lib.oracle_cholesky_inverse.argtypes = [p, i64, i64, p, i64]
        lib.oracle_cholesky_inverse.restype = None
        lib.oracle_invert.argtypes = [p, i64, i64, f64, p, i64]
        lib.oracle_invert.restype = i64
        lib.oracle_precondition.argtypes = [p, i64, p, i64, p, p]
        lib.oracle_precondition.restype = None
        lib.oracle_kron_solve.argtypes = [p, i64, p, i64, f64, p, p]
        lib.oracle_kron_solve.restype = i64
        _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads():
    """Threads the C loops use (OpenMP default for this process)."""
    return int(_load().oracle_num_threads())


def curvature(xs, factor=None, n_total=None):
    """Mean of outer products over all rows of all micro-batches in ``xs``.

    ``xs`` is one ``[tokens, d]`` array or a list of them (micro-batches of one
    mini-batch); the result is ``sum_m X_m^T X_m / n_total`` with ``n_total``
    the total number of rows, i.e. <x x^T> over the mini-batch (section 2.3).
    If ``factor`` is given the new term is added to it (accumulation over
    micro-batches, one curvature work item per micro-batch, section 3.1).
    """
    if isinstance(xs, np.ndarray):
        xs = [xs]
    xs = [_f64(x) for x in xs]
    if n_total is None:
        n_total = sum(x.shape[0] for x in xs)
    d = xs[0].shape[1]
    out = np.zeros((d, d)) if factor is None else _f64(factor).copy()
    for x in xs:
        out += (x.T @ x) / float(n_total)
    return out


def curvature_update(x, alpha, beta, factor=None):
    """``beta * factor + alpha * x^T x`` in float64 (one curvature work item)."""
    x = _f64(x)
    upd = alpha * (x.T @ x)
    if factor is None or beta == 0.0:
        return upd
    return beta * _f64(factor) + upd


def curvature_loops(x, alpha=None, beta=0.0, factor=None):
    """Same quantity as ``curvature_update`` by the plain triple loop in C."""
    x = _f64(x)
    n, d = x.shape
    if alpha is None:
        alpha = 1.0 / n
    out = np.zeros((d, d)) if factor is None else _f64(factor).copy()
    _load().oracle_curvature(_ptr(x), n, d, d, float(alpha), float(beta), _ptr(out), d)
    return out


def curvature_entry(x, i, j, alpha):
    """One entry ``alpha * sum_t x[t,i] x[t,j]`` (for sampled full-size checks)."""
    x = np.asarray(x)
    xi = x[:, i].astype(np.float64)
    xj = x[:, j].astype(np.float64)
    return float(alpha) * float(np.dot(xi, xj))


def cholesky(m):
    """Lower Cholesky factor by the textbook column algorithm; returns (L, info)."""
    m = _f64(m)
    d = m.shape[0]
    l = np.empty((d, d))
    info = _load().oracle_cholesky(_ptr(m), d, d, _ptr(l), d)
    return l, int(info)


def invert(factor, damping):
    """``(factor + damping I)^-1`` via Cholesky; returns (inverse, info).

    info = 0 on success, k > 0 if the k-th pivot of the Cholesky decomposition
    is not positive (the inverse is then None).
    """
    factor = _f64(factor)
    d = factor.shape[0]
    assert factor.shape == (d, d)
    inv = np.empty((d, d))
    info = _load().oracle_invert(_ptr(factor), d, d, float(damping), _ptr(inv), d)
    if info != 0:
        return None, int(info)
    return inv, 0


def precondition(b_inv, grad, a_inv):
    """``B^-1 G A^-1`` for a ``d_out x d_in`` gradient (section 2.3.1)."""
    return _f64(b_inv) @ _f64(grad) @ _f64(a_inv)


def precondition_loops(b_inv, grad, a_inv):
    """Same by plain triple loops in C (pins the matmul form)."""
    b_inv, grad, a_inv = _f64(b_inv), _f64(grad), _f64(a_inv)
    d_out, d_in = grad.shape
    out = np.empty((d_out, d_in))
    _load().oracle_precondition(_ptr(b_inv), d_out, _ptr(a_inv), d_in, _ptr(grad), _ptr(out))
    return out


def kron_solve(a, b, grad, damping):
    """Solve ((A + damping I) (x) (B + damping I)) p = vec(G) explicitly (tiny sizes).

    Returns p reshaped to ``d_out x d_in``; vec stacks columns (section 2.3.1).
    """
    a, b, grad = _f64(a), _f64(b), _f64(grad)
    d_out, d_in = grad.shape
    assert a.shape == (d_in, d_in) and b.shape == (d_out, d_out)
    out = np.empty((d_out, d_in))
    info = _load().oracle_kron_solve(_ptr(a), d_in, _ptr(b), d_out, float(damping), _ptr(grad), _ptr(out))
    if info != 0:
        raise np.linalg.LinAlgError("Kronecker system not positive definite at pivot %d" % info)
    return out


def kfac_chain(xs, es, grad, damping):
    """Whole path for one layer: factors, damped inverses, preconditioned gradient."""
    a = curvature(xs)
    b = curvature(es)
    a_inv, ia = invert(a, damping)
    b_inv, ib = invert(b, damping)
    if ia or ib:
        raise np.linalg.LinAlgError("factor not positive definite")
    return a, b, a_inv, b_inv, precondition(b_inv, grad, a_inv)


def rel_fro(got, want):
    """Relative Frobenius error ||got - want||_F / ||want||_F in float64."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.linalg.norm(want)
    num = np.linalg.norm(got - want)
    return num / den if den > 0 else num
