"""Pins of the solver oracle (oracle/recon_oracle.py) on small dense systems, against numpy.linalg and hand-worked
steps (no GPU)."""
import numpy as np
import pytest

from oracle import recon_oracle as ro


def ops(M):
    return (lambda x: M @ x), (lambda y: M.T @ y)


def test_r1_one_sirt_step_by_hand():
    """A = [[1,2],[3,4]], y = (1,1), x0 = 0: R = (1/3, 1/7), C = (1/4, 1/6);
    A^T (R y) = (1/3 + 3/7, 2/3 + 4/7) = (16/21, 26/21); x1 = (4/21, 13/63)."""
    M = np.array([[1.0, 2.0], [3.0, 4.0]])
    A, AT = ops(M)
    x1 = ro.sirt(A, AT, np.array([1.0, 1.0]), np.zeros(2), 1)
    np.testing.assert_allclose(x1, [4.0 / 21.0, 13.0 / 63.0], rtol=1e-14)
    # relaxation scales the step; the clip acts after the step
    x1h = ro.sirt(A, AT, np.array([1.0, 1.0]), np.zeros(2), 1, relaxation=0.5)
    np.testing.assert_allclose(x1h, [2.0 / 21.0, 13.0 / 126.0], rtol=1e-14)
    xneg = ro.sirt(A, AT, np.array([-1.0, -1.0]), np.zeros(2), 1, nonneg=True)
    np.testing.assert_array_equal(xneg, [0.0, 0.0])


def test_r2_one_descent_step_by_hand():
    """Same A, y = (1,1), x0 = 0: g = A^T(-y) = (-4,-6), A g = (-16,-36), alpha = 52/1552, x1 = alpha (4, 6)."""
    M = np.array([[1.0, 2.0], [3.0, 4.0]])
    A, AT = ops(M)
    x1 = ro.least_squares_descent(A, AT, np.array([1.0, 1.0]), np.zeros(2), 1)
    np.testing.assert_allclose(x1, np.array([4.0, 6.0]) * 52.0 / 1552.0, rtol=1e-14)


def test_r3_sirt_fixed_point_solves_the_row_weighted_normal_equations():
    rng = np.random.default_rng(3)
    M = rng.random((30, 8)) * (rng.random((30, 8)) < 0.6)
    M[:, 0] += 0.1
    y = rng.random(30)                                  # inconsistent on purpose
    A, AT = ops(M)
    x = ro.sirt(A, AT, y, np.zeros(8), 20000)
    R = np.diag(1.0 / M.sum(axis=1))
    want = np.linalg.solve(M.T @ R @ M, M.T @ R @ y)
    np.testing.assert_allclose(x, want, rtol=1e-8, atol=1e-10)


def test_r4_descent_converges_to_the_least_squares_solution_with_monotone_cost():
    rng = np.random.default_rng(4)
    M = rng.random((40, 6))
    y = rng.random(40)
    A, AT = ops(M)
    costs = [0.5 * np.sum((M @ ro.least_squares_descent(A, AT, y, np.zeros(6), k) - y) ** 2) for k in range(0, 40, 4)]
    assert all(b <= a * (1 + 1e-12) for a, b in zip(costs, costs[1:]))
    x = ro.least_squares_descent(A, AT, y, np.zeros(6), 5000)
    np.testing.assert_allclose(x, np.linalg.lstsq(M, y, rcond=None)[0], rtol=1e-8, atol=1e-10)


def test_r5_rays_and_voxels_nobody_sees_are_left_alone():
    M = np.array([[1.0, 0.0, 2.0], [0.0, 0.0, 0.0], [3.0, 0.0, 1.0]])     # row 1 and column 1 are empty
    A, AT = ops(M)
    x = ro.sirt(A, AT, np.array([3.0, 5.0, 4.0]), np.array([0.0, 7.0, 0.0]), 5000)
    assert x[1] == 7.0
    np.testing.assert_allclose(M @ x, [3.0, 0.0, 4.0], atol=1e-9)


@pytest.mark.parametrize("model", ["sf", "siddon"])
def test_r6_consistent_ct_data_are_reproduced(oracle_mod, model):
    """On the projector oracle itself: data y = A x_true of a tiny scan; the SIRT residual falls monotonically."""
    from synthetic import CTConfig, uniform_volume
    from synthetic.configs import CONE
    cfg = CTConfig("t", CONE, nviews=12, arc_deg=360.0, nrows=10, ncols=12, pixel_v=1.3, pixel_u=1.2, nx=8, ny=8, nz=6,
                   voxel_xy=1.0, voxel_z=1.1, sod=30.0, sdd=47.0, shift_u=0.2)
    orc = oracle_mod if model == "sf" else oracle_mod.siddon
    A = lambda x: orc.project(cfg, x.astype(np.float32))
    AT = lambda y: orc.backproject(cfg, y.astype(np.float32))
    xt = uniform_volume(cfg, 1)[0].astype(np.float64)
    y = A(xt)
    res = [np.linalg.norm(A(ro.sirt(A, AT, y, np.zeros_like(xt), k)) - y) for k in (0, 5, 10, 20, 40)]
    assert all(b < a for a, b in zip(res, res[1:])) and res[-1] < 0.05 * res[0], res
