"""Pins of the Siddon CPU oracle on the modular geometry (every view has its own source position, detector centre and
detector orientation), against things other than itself (no GPU): the flat-panel cone-beam scan written as a modular
one, brute-force numpy chords on independently built rays for tilted and shifted modules and for a source looking down
the z axis, invariance under moving the detector along its own rays, dense transposes."""
import numpy as np
import pytest

import reference_math as rm
from synthetic import CTConfig, modular_from, perturbed_poses, uniform_sinogram, uniform_volume
from synthetic.configs import CONE, MODULAR
from test_siddon_pins import all_rays, voxel_boxes


@pytest.fixture(scope="module")
def sd(oracle_mod):
    return oracle_mod.siddon


def tiny(**kw):
    base = dict(name="tinym", geom=CONE, nviews=7, arc_deg=360.0, nrows=6, ncols=9, pixel_v=1.3, pixel_u=0.9,
                nx=5, ny=4, nz=3, voxel_xy=0.8, voxel_z=1.1, sod=30.0, sdd=47.0, shift_v=0.3, shift_u=-0.7,
                center_x=0.4, center_y=-0.3, center_z=0.25, start_deg=11.0)
    base.update(kw)
    return CTConfig(**base)


def brute(cfg):
    p, d = all_rays(cfg)
    lo, hi = voxel_boxes(cfg)
    return rm.box_chord(p[:, None, :], d[:, None, :], lo[None], hi[None])


def test_m1_a_cone_beam_scan_written_as_modular_is_the_same_matrix(sd):
    cone = tiny()
    np.testing.assert_allclose(sd.dense_matrix(modular_from(cone)), sd.dense_matrix(cone), rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_m2_tilted_and_shifted_modules_match_numpy_chords(sd, seed):
    cfg = perturbed_poses(tiny(), seed, shift_mm=2.0, tilt_rad=0.3)
    A = sd.dense_matrix(cfg)
    assert A.max() > 0.5 * cfg.voxel_xy
    np.testing.assert_allclose(A, brute(cfg), rtol=0, atol=1e-12)


def test_m3_source_above_the_volume(sd):
    """Rays that advance fastest along z: source on the z axis above the volume, detector below, facing up."""
    pose = (0.3, -0.2, 25.0, 0.0, 0.0, -18.0, 1.0, 0.0, 0.0, 0.0, 1.0, 0.0)
    tilt = (4.0, 1.0, 22.0, -1.0, 0.5, -15.0, 0.8, 0.6, 0.0, -0.6, 0.8, 0.0)
    cfg = tiny(nviews=2).replace(geom=MODULAR, poses=(pose, tilt), ncols=7, nrows=7)
    A = sd.dense_matrix(cfg)
    assert (A > 0).sum() > 20
    np.testing.assert_allclose(A, brute(cfg), rtol=0, atol=1e-12)
    x, y = uniform_volume(cfg, 3)[0], uniform_sinogram(cfg, 4)[0]
    np.testing.assert_allclose(sd.project(cfg, x).ravel(), A @ x.astype(np.float64).ravel(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(sd.backproject(cfg, y).ravel(), A.T @ y.astype(np.float64).ravel(), rtol=0, atol=1e-12)


def test_m4_moving_the_detector_along_its_rays_changes_nothing(sd):
    """Detector twice as far from the source, pixels twice as large: the same rays, so the same matrix."""
    cfg = perturbed_poses(tiny(), 5, shift_mm=2.0, tilt_rad=0.2)
    far = []
    for p in cfg.poses:
        p = np.asarray(p)
        far.append(tuple(np.concatenate([p[0:3], p[0:3] + 2.0 * (p[3:6] - p[0:3]), p[6:12]])))
    cfg2 = cfg.replace(poses=tuple(far), pixel_u=2 * cfg.pixel_u, pixel_v=2 * cfg.pixel_v)
    np.testing.assert_allclose(sd.dense_matrix(cfg2), sd.dense_matrix(cfg), rtol=0, atol=1e-11)


def test_m5_dense_matrix_agrees_with_both_loops(sd):
    cfg = perturbed_poses(tiny(), 7, shift_mm=2.0, tilt_rad=0.3)
    A = sd.dense_matrix(cfg)
    x, y = uniform_volume(cfg, 3)[0], uniform_sinogram(cfg, 4)[0]
    ax, aty = A @ x.astype(np.float64).ravel(), A.T @ y.astype(np.float64).ravel()
    np.testing.assert_allclose(sd.project(cfg, x).ravel(), ax, rtol=0, atol=1e-12)
    np.testing.assert_allclose(sd.backproject(cfg, y).ravel(), aty, rtol=0, atol=1e-12)
    rays, vox = np.arange(0, A.shape[0], 3), np.arange(0, A.shape[1], 2)
    np.testing.assert_allclose(sd.project_rays(cfg, x, rays), ax[rays], atol=1e-12)
    np.testing.assert_allclose(sd.backproject_voxels(cfg, y, vox), aty[vox], atol=1e-12)
    assert sd.nnz(cfg) == int((A > 0).sum())
    sub = cfg.with_views([1, 4])
    per = cfg.nrows * cfg.ncols
    np.testing.assert_array_equal(sd.dense_matrix(sub), np.concatenate([A[per:2 * per], A[4 * per:5 * per]]))


def test_m6_exactly_vertical_ray(sd):
    """Detector centre straight below the source, odd pixel counts, no shifts: the central pixel's ray has no in-plane
    component at all.  It crosses the column of voxels under the source, Tz in each."""
    pose = (0.1, 0.2, 25.0, 0.1, 0.2, -18.0, 1.0, 0.0, 0.0, 0.0, 1.0, 0.0)
    cfg = tiny(nviews=1, shift_u=0.0, shift_v=0.0, center_x=0.0, center_y=0.0, center_z=0.0).replace(
        geom=MODULAR, poses=(pose,), ncols=5, nrows=5)
    A = sd.dense_matrix(cfg)
    np.testing.assert_allclose(A, brute(cfg), rtol=0, atol=1e-12)
    central = A[2 * 5 + 2].reshape(cfg.vol_shape)                  # pixel (2, 2)
    i, j = 2, 2                                                    # x = 0.1 in voxel 2 of 5 (0.8 mm), y = 0.2 in voxel 2 of 4
    expect = np.zeros(cfg.vol_shape)
    expect[:, j, i] = cfg.voxel_z
    np.testing.assert_allclose(central, expect, rtol=0, atol=1e-12)
    x = uniform_volume(cfg, 3)[0]
    np.testing.assert_allclose(sd.project(cfg, x).ravel(), A @ x.astype(np.float64).ravel(), rtol=0, atol=1e-12)
