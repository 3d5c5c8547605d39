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


# ---------------------------------------------------------------- footprint model on upright modules

def upright(cfg, seed, shift_mm=2.0, tilt_rad=0.3):
    return perturbed_poses(cfg, seed, shift_mm=shift_mm, tilt_rad=tilt_rad, upright=True)


def test_mf1_a_cone_beam_scan_written_as_modular_is_the_same_footprint_matrix(oracle_mod):
    cone = tiny()
    np.testing.assert_allclose(oracle_mod.dense_matrix(modular_from(cone)), oracle_mod.dense_matrix(cone), rtol=0, atol=1e-12)


def test_mf2_each_view_is_a_circular_cone_beam_view_of_a_shifted_scene(oracle_mod):
    """A module with source (lS, tS, zS) and detector centre (lS - sdd, tC, zC) in its own frame sees the volume as a
    circular scanner with SOD = lS, SDD = sdd at the same angle sees the volume moved by -(tS e_u + zS e_z), with the
    detector shifted by (tC - tS, zC - zS): translate the scene so that the source sits on the frame's axis."""
    base = tiny()
    cfg = upright(base, 4)
    A = oracle_mod.dense_matrix(cfg).reshape(cfg.nviews, -1)
    for a, pose in enumerate(cfg.poses):
        S, C_, eu = np.array(pose[0:3]), np.array(pose[3:6]), np.array(pose[6:9])
        es = np.array([eu[1], -eu[0], 0.0])
        phi = float(np.arctan2(es[1], es[0]))
        lS, tS, zS = float(S @ es), float(S @ eu), float(S[2])
        sdd = lS - float(C_ @ es)
        tC, zC = float(C_ @ eu), float(C_[2])
        moved = np.array([base.center_x, base.center_y, base.center_z]) - tS * eu - np.array([0.0, 0.0, zS])
        one = base.replace(nviews=1, angles_override=(phi,), sod=lS, sdd=sdd, center_x=float(moved[0]),
                           center_y=float(moved[1]), center_z=float(moved[2]),
                           shift_u=base.shift_u + (tC - tS) / base.pixel_u, shift_v=base.shift_v + (zC - zS) / base.pixel_v)
        np.testing.assert_allclose(A[a], oracle_mod.dense_matrix(one).ravel(), rtol=0, atol=1e-11)


def test_mf3_weights_track_the_beam_average_of_true_chords(oracle_mod):
    from test_curved_pins import _beam_average_chord
    from synthetic import config, reduced
    cfg = upright(reduced(config(3), 32).with_views([0, 37, 90, 200, 333, 610]), 9, shift_mm=20.0, tilt_rad=0.2)
    A = oracle_mod.dense_matrix(cfg)
    rng = np.random.default_rng(5)
    nz_pairs = np.argwhere(A > 0)
    pick = nz_pairs[rng.choice(len(nz_pairs), 300, replace=False)]
    devs = []
    for ray, vox in pick:
        a, rem = divmod(ray, cfg.nrows * cfg.ncols)
        r, c = divmod(rem, cfg.ncols)
        k, rem = divmod(vox, cfg.ny * cfg.nx)
        j, i = divmod(rem, cfg.nx)
        devs.append(A[ray, vox] - _beam_average_chord(cfg, a, r, c, i, j, k))
    devs = np.abs(np.array(devs))
    assert devs.max() < 0.06 * A.max() and devs.mean() < 0.012 * A.max(), (devs.max(), devs.mean(), A.max())


def test_mf4_converges_to_analytic_line_integrals(oracle_mod):
    from synthetic.phantoms import Ellipsoid, rasterize
    from test_siddon_pins import _rot
    base = CTConfig("anm", CONE, nviews=5, arc_deg=360.0, nrows=16, ncols=24, pixel_v=6.0, pixel_u=6.0,
                    nx=16, ny=16, nz=12, voxel_xy=4.0, voxel_z=4.0, sod=400.0, sdd=600.0,
                    shift_u=0.35, shift_v=-0.2, center_x=3.0, center_y=-2.0, center_z=1.5, start_deg=17.0)
    ells = [Ellipsoid((8.0, -5.0, 3.0), (20.0, 11.0, 14.0), _rot(0.4, 0.3, -0.5), 1.0),
            Ellipsoid((-9.0, 10.0, -4.0), (9.0, 14.0, 8.0), _rot(-0.8, 0.1, 0.6), 0.6)]
    errs = []
    for f in (1, 2, 4):
        fine = base.replace(nrows=base.nrows * f, ncols=base.ncols * f, pixel_u=base.pixel_u / f, pixel_v=base.pixel_v / f,
                            nx=base.nx * f, ny=base.ny * f, nz=base.nz * f, voxel_xy=base.voxel_xy / f,
                            voxel_z=base.voxel_z / f, shift_u=base.shift_u * f, shift_v=base.shift_v * f)
        cfg = upright(fine, 13, shift_mm=25.0, tilt_rad=0.25)        # the same poses at every refinement (same seed)
        y = oracle_mod.project(cfg, rasterize(cfg, ells))
        ref = rm.analytic_sinogram(cfg, ells)
        errs.append(np.linalg.norm(y - ref) / np.linalg.norm(ref))
    assert errs[2] < 0.06, errs
    assert errs[0] / errs[1] > 1.5 and errs[1] / errs[2] > 1.5, errs


def test_mf5_dense_matrix_agrees_with_both_loops(oracle_mod):
    cfg = upright(tiny(), 7)
    A = oracle_mod.dense_matrix(cfg)
    x, y = uniform_volume(cfg, 3)[0], uniform_sinogram(cfg, 4)[0]
    ax, aty = A @ x.astype(np.float64).ravel(), A.T @ y.astype(np.float64).ravel()
    np.testing.assert_allclose(oracle_mod.project(cfg, x).ravel(), ax, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle_mod.backproject(cfg, y).ravel(), aty, rtol=0, atol=1e-12)
    rays, vox = np.arange(0, A.shape[0], 3), np.arange(0, A.shape[1], 2)
    np.testing.assert_allclose(oracle_mod.project_rays(cfg, x, rays), ax[rays], atol=1e-12)
    np.testing.assert_allclose(oracle_mod.backproject_voxels(cfg, y, vox), aty[vox], atol=1e-12)
    assert oracle_mod.nnz(cfg) == int((A > 0).sum())


def test_mf6_tilted_modules_are_refused(oracle_mod):
    with pytest.raises(AssertionError):
        oracle_mod.dense_matrix(perturbed_poses(tiny(), 1, tilt_rad=0.2))
