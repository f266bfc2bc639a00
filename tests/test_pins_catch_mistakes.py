"""The pins are only worth something if a plausible mistake in the oracle fails one of them.

Each case below plants one mistake in a copy of the oracle (on the CPU, never in the GPU path) and
checks that at least one pin of tests/test_oracle_pins.py then fails.
"""
import types

import numpy as np
import pytest

from oracle import kfac_oracle as real
import tests.test_oracle_pins as pins

PIN_FUNCS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_") and "synthetic" not in n]


def _mutant(**overrides):
    m = types.SimpleNamespace(**{k: getattr(real, k) for k in dir(real) if not k.startswith("__")})
    for k, v in overrides.items():
        setattr(m, k, v)
    # functions of the oracle that call each other must see the mutated versions
    def kfac_chain(xs, es, grad, damping):
        a, b = m.curvature(xs), m.curvature(es)
        a_inv, _ = m.invert(a, damping)
        b_inv, _ = m.invert(b, damping)
        return a, b, a_inv, b_inv, m.precondition(b_inv, grad, a_inv)
    m.kfac_chain = kfac_chain
    return m


def _some_pin_fails(mutant):
    import inspect

    for f in PIN_FUNCS:
        params = inspect.signature(f).parameters
        if "oracle" not in params:
            continue
        extra = {}
        if "d" in params:
            extra = {"d": 65}
        if "d_out" in params:
            extra = {"d_out": 2, "d_in": 3}
        try:
            f(oracle=mutant, **extra)
        except AssertionError:
            return True
        except Exception:
            return True
    return False


def test_the_unmodified_oracle_passes_this_harness():
    assert not _some_pin_fails(_mutant())


MISTAKES = {
    "tokens x tokens instead of features x features": dict(
        curvature=lambda xs, factor=None, n_total=None: real.curvature([np.asarray(x).T for x in ([xs] if isinstance(xs, np.ndarray) else xs)])),
    "curvature not divided by the number of examples": dict(
        curvature=lambda xs, factor=None, n_total=None: real.curvature(xs, factor, 1)),
    "micro-batches averaged instead of pooled": dict(
        curvature=lambda xs, factor=None, n_total=None: sum(real.curvature(x) for x in ([xs] if isinstance(xs, np.ndarray) else xs))),
    "beta ignored": dict(
        curvature_update=lambda x, alpha, beta, factor=None: real.curvature_update(x, alpha, 0.0)),
    "damping dropped": dict(invert=lambda f, lam: real.invert(f, 0.0)),
    "damping added twice": dict(invert=lambda f, lam: real.invert(f, 2.0 * lam)),
    "inverse of the Cholesky factor instead of the matrix": dict(
        invert=lambda f, lam: (np.linalg.inv(np.linalg.cholesky(np.asarray(f, float) + lam * np.eye(len(f)))), 0)),
    "A and B swapped in precondition": dict(
        precondition=lambda b_inv, g, a_inv: real.precondition(a_inv, np.asarray(g).T, b_inv).T
        if np.shape(b_inv) != np.shape(a_inv) else np.asarray(a_inv) @ np.asarray(g) @ np.asarray(b_inv)),
    "Kronecker factors in the wrong order": dict(
        kron_solve=lambda a, b, g, lam: np.linalg.solve(
            np.kron(np.asarray(b) + lam * np.eye(len(b)), np.asarray(a) + lam * np.eye(len(a))),
            np.asarray(g).reshape(-1, order="F")).reshape(np.shape(g), order="F")),
    "row-stacking vec in the Kronecker solve": dict(
        kron_solve=lambda a, b, g, lam: np.linalg.solve(
            np.kron(np.asarray(a) + lam * np.eye(len(a)), np.asarray(b) + lam * np.eye(len(b))),
            np.asarray(g).reshape(-1)).reshape(np.shape(g))),
    "Cholesky factor returned transposed": dict(cholesky=lambda m: (real.cholesky(m)[0].T, real.cholesky(m)[1])),
    "failing pivot reported 0-based": dict(
        invert=lambda f, lam: (lambda r: (r[0], r[1] - 1 if r[1] > 0 else 0))(real.invert(f, lam))),
}


@pytest.mark.parametrize("name", sorted(MISTAKES))
def test_planted_mistake_is_caught(name):
    assert _some_pin_fails(_mutant(**MISTAKES[name])), name
