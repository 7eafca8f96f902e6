"""CPU oracle for the pattern-selection side of the pruning framework (paper, section 5.1): the proximal step of the
ADMM iteration, its multiplier update, and the final projection of the relaxed selection variables onto one pattern.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the bench's cpu_baseline leg; never by the product
path, with which it shares no code.  Plain numpy, float64 arithmetic, one kernel (one selection vector) at a time in
the paper's order; nothing is blocked, fused or reordered.

Notation follows section 5.1: every 3x3 kernel W_i has a selection vector z in R^K over the K patterns of the library,
an auxiliary copy u constrained to the probability simplex (u_j in [0,1], sum_j u_j = 1), a multiplier mu and the
penalty rho > 0.
"""
from __future__ import annotations

import numpy as np


def simplex_project(d) -> np.ndarray:
    """The proximal step's minimiser (section 5.1, problem over u and its analytical solution): the point of the
    probability simplex nearest to d, u = [d - nu 1]_+ with nu the root of 1^T [d - nu 1]_+ = 1.

    g(nu) = sum_j max(d_j - nu, 0) is continuous, piecewise linear and strictly decreasing wherever it is positive; it
    changes slope only at the d_j.  Between two neighbouring breakpoints, with the m largest entries above nu,
    g(nu) = (sum of those m) - m nu, so the root is nu = (sum of the m largest - 1) / m for the m for which that nu
    lies in its own interval.  d: [..., K]; returns the same shape, float64."""
    d = np.asarray(d, dtype=np.float64)
    flat = d.reshape(-1, d.shape[-1])
    out = np.empty_like(flat)
    for r in range(flat.shape[0]):
        v = flat[r]
        s = np.sort(v)[::-1]                       # breakpoints, largest first
        nu = None
        total = 0.0
        for m in range(1, s.size + 1):
            total += s[m - 1]
            cand = (total - 1.0) / m               # root if exactly the m largest entries lie above it
            lower = s[m] if m < s.size else -np.inf
            if cand < s[m - 1] and cand >= lower:
                nu = cand
                break
        if nu is None:                             # (cannot happen for finite input; kept as a loud failure)
            raise ArithmeticError("no root found")
        out[r] = np.maximum(v - nu, 0.0)
    return out.reshape(d.shape)


def proximal_step(z, mu, rho: float):
    """One proximal step and multiplier update of the ADMM iteration (section 5.1): d = z + mu / rho,
    u = argmin_u rho/2 ||u - d||^2 over the simplex, mu_new = mu + rho (z - u).  Returns (u, mu_new), float64."""
    z = np.asarray(z, dtype=np.float64)
    mu = np.asarray(mu, dtype=np.float64)
    if not rho > 0:
        raise ValueError("rho must be positive")
    d = z + mu / rho
    u = simplex_project(d)
    return u, mu + rho * (z - u)


def binarize(z) -> np.ndarray:
    """Projection of the relaxed selection onto one pattern (section 5.1, last problem): z_binary has a single one at
    argmax_j z_j.  Returned as the index of that pattern (the one-hot vector is implied); ties go to the lowest index,
    the rule the pattern assignment of this repository uses everywhere.  z: [..., K] -> int32 [...]."""
    z = np.asarray(z, dtype=np.float64)
    return np.argmax(z, axis=-1).astype(np.int32)
