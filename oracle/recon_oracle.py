"""CPU oracle of the two iterative solvers built on the projector pair.  Test infrastructure only.

Plain numpy, double precision, written against callables A(x) and AT(y) so that the same code runs on a small dense
matrix (for its pins) and on the projector oracles (for parity with the GPU).

What it follows: "CT Projection Models and Geometries" states the least-squares cost 1/2 ||A x - y||^2 and its
gradient A^T (A x - y); steepest descent with the exact line search is the textbook iteration on that cost
    g = A^T (A x - y),   alpha = <g, g> / <A g, A g>,   x <- x - alpha g.
SIRT is the standard simultaneous iterative reconstruction technique
    x <- x + lambda C A^T ( R (y - A x) ),   R = diag(1 / (A 1)),  C = diag(1 / (A^T 1))   (0 where a sum is 0),
optionally clipped at zero from below after every update.

Pins: tests/test_recon_pins.py (hand-worked 2x2 steps, fixed points against numpy.linalg solutions, monotone cost).
"""
from __future__ import annotations

import numpy as np


def _safe_reciprocal(v):
    out = np.zeros_like(v)
    np.divide(1.0, v, out=out, where=v > 0)
    return out


def sirt(A, AT, y, x0, iterations, relaxation=1.0, nonneg=False):
    """A, AT: callables on float64 arrays; y, x0: arrays of the sinogram / volume shape."""
    y = np.asarray(y, dtype=np.float64)
    x = np.array(x0, dtype=np.float64)
    R = _safe_reciprocal(A(np.ones_like(x)))
    C = _safe_reciprocal(AT(np.ones_like(y)))
    for _ in range(iterations):
        x = x + relaxation * C * AT(R * (y - A(x)))
        if nonneg:
            x = np.maximum(x, 0.0)
    return x


def least_squares_descent(A, AT, y, x0, iterations):
    y = np.asarray(y, dtype=np.float64)
    x = np.array(x0, dtype=np.float64)
    for _ in range(iterations):
        g = AT(A(x) - y)
        q = A(g)
        den = float((q * q).sum())
        alpha = float((g * g).sum()) / den if den > 0 else 0.0
        x = x - alpha * g
    return x
