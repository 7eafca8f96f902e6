"""Pins of oracle/admm_oracle.py to what the paper and the mathematics fix (section 5.1: the proximal problem over u, its
closed-form solution u = [d - nu 1]_+ with 1^T u = 1, the multiplier update, the argmax projection).  None of these
tests re-types the oracle's formula: they check optimality conditions, closed forms of special cases, brute force on
a grid, and invariances that a dropped term, a wrong sign or a wrong index would break."""
import itertools

import numpy as np
import pytest

import oracle
from workloads import rng


def vectors(seed, n, K, scale=1.0):
    return (rng.normal(rng.stream_seed(77, seed, K), n * K).reshape(n, K) * scale)


@pytest.mark.parametrize("K", [1, 2, 3, 4, 8, 12])
def test_result_is_on_the_simplex_and_satisfies_the_optimality_conditions(K):
    d = vectors(1, 200, K, 2.0)
    u = oracle.simplex_project(d)
    assert np.all(u >= 0.0) and np.all(u <= 1.0 + 1e-15)
    np.testing.assert_allclose(u.sum(axis=1), 1.0, atol=1e-12)
    # KKT of min ||u - d||^2 on the simplex: one nu with d_j - u_j = nu where u_j > 0 and d_j <= nu where u_j = 0
    for r in range(d.shape[0]):
        pos = u[r] > 0
        nus = d[r][pos] - u[r][pos]
        assert np.ptp(nus) < 1e-12
        assert np.all(d[r][~pos] <= nus[0] + 1e-12)


def test_a_point_of_the_simplex_is_left_alone():
    p = np.abs(vectors(2, 50, 6))
    p /= p.sum(axis=1, keepdims=True)
    np.testing.assert_allclose(oracle.simplex_project(p), p, atol=1e-15)
    e = np.eye(5)
    np.testing.assert_array_equal(oracle.simplex_project(e), e)


def test_closed_forms():
    # K = 1: the simplex is the point 1
    np.testing.assert_array_equal(oracle.simplex_project(np.array([[3.7], [-2.0]])), [[1.0], [1.0]])
    # equal entries: 1/K each
    for K in (2, 5, 8):
        np.testing.assert_allclose(oracle.simplex_project(np.full((1, K), -4.25)), np.full((1, K), 1.0 / K), atol=1e-15)
    # K = 2: projection onto the segment, u_1 = clip((d_1 - d_2 + 1) / 2, 0, 1)
    d = vectors(3, 300, 2, 1.5)
    u1 = np.clip((d[:, 0] - d[:, 1] + 1.0) / 2.0, 0.0, 1.0)
    np.testing.assert_allclose(oracle.simplex_project(d), np.stack([u1, 1.0 - u1], axis=1), atol=1e-14)
    # one entry far above the rest: that vertex
    np.testing.assert_array_equal(oracle.simplex_project(np.array([[0.1, 9.0, -1.0, 0.3]])), [[0.0, 1.0, 0.0, 0.0]])


def test_shift_invariance_and_permutation_equivariance():
    d = vectors(4, 100, 8)
    u = oracle.simplex_project(d)
    np.testing.assert_allclose(oracle.simplex_project(d + 3.25), u, atol=1e-13)      # the constraint absorbs a shift
    perm = np.array([3, 0, 7, 1, 6, 2, 5, 4])
    np.testing.assert_allclose(oracle.simplex_project(d[:, perm]), u[:, perm], atol=1e-15)


def test_nearest_point_against_brute_force_on_a_grid():
    # K = 3: every point of the simplex with coordinates in steps of 1/200
    n = 200
    grid = np.array([(i, j, n - i - j) for i in range(n + 1) for j in range(n + 1 - i)], dtype=np.float64) / n
    d = vectors(5, 40, 3, 0.8)
    u = oracle.simplex_project(d)
    for r in range(d.shape[0]):
        best = grid[np.argmin(((grid - d[r]) ** 2).sum(axis=1))]
        assert np.abs(best - u[r]).max() <= 1.0 / n + 1e-12
        # and no grid point is nearer than the projection itself
        assert ((u[r] - d[r]) ** 2).sum() <= ((grid - d[r]) ** 2).sum(axis=1).min() + 1e-12


def test_nearer_than_any_other_feasible_point():
    d = vectors(6, 30, 8, 1.5)
    u = oracle.simplex_project(d)
    q = np.abs(vectors(7, 500, 8))
    q /= q.sum(axis=1, keepdims=True)
    for r in range(d.shape[0]):
        assert ((u[r] - d[r]) ** 2).sum() <= (((q - d[r]) ** 2).sum(axis=1)).min() + 1e-12


def test_proximal_step_and_multiplier_update():
    z, mu, rho = vectors(8, 64, 8, 0.5), vectors(9, 64, 8, 0.1), 0.75
    u, mu2 = oracle.proximal_step(z, mu, rho)
    # u is the projection of z + mu / rho (argument checked through the optimality conditions, with the multiplier)
    np.testing.assert_allclose(u.sum(axis=1), 1.0, atol=1e-12)
    assert np.all(u >= 0)
    # multiplier update: mu_new - mu = rho (z - u); summed over j: rho (sum z - 1)
    np.testing.assert_allclose(mu2 - mu, rho * (z - u), atol=1e-15)
    np.testing.assert_allclose((mu2 - mu).sum(axis=1), rho * (z.sum(axis=1) - 1.0), atol=1e-12)
    # where u_j > 0, (d_j - u_j) is one constant nu per kernel, and mu_new_j = rho (d_j - u_j) = rho nu there
    d = z + mu / rho
    for r in range(8):
        pos = u[r] > 0
        np.testing.assert_allclose(mu2[r][pos], rho * (d[r][pos] - u[r][pos]), atol=1e-13)
        assert np.ptp(mu2[r][pos]) < 1e-12
    # a fixed point: z on the simplex and mu = 0 give u = z and mu stays 0
    p = np.abs(z); p /= p.sum(axis=1, keepdims=True)
    u, mu2 = oracle.proximal_step(p, np.zeros_like(p), 2.0)
    np.testing.assert_allclose(u, p, atol=1e-15)
    np.testing.assert_allclose(mu2, 0.0, atol=1e-15)
    with pytest.raises(ValueError):
        oracle.proximal_step(p, p, 0.0)


def test_binarize_is_the_nearest_one_hot_vector_with_ties_to_the_lowest_index():
    z = vectors(10, 200, 6)
    idx = oracle.binarize(z)
    eye = np.eye(6)
    for r in range(z.shape[0]):
        dist = ((eye - z[r]) ** 2).sum(axis=1)           # distance to every feasible binary vector
        assert idx[r] == int(np.argmin(dist))
    assert oracle.binarize(np.array([[0.2, 0.5, 0.5, 0.1]]))[0] == 1
    assert oracle.binarize(np.array([[0.0, 0.0, 0.0]]))[0] == 0
    assert oracle.binarize(z).dtype == np.int32
