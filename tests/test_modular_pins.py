"""Pins of the CPU oracles on the modular geometry (every view has its own source position, detector centre and
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


# ---------------------------------------------------------------- footprint model on tilted modules
# Reading: knots = u of the central projections of the voxel's in-plane corners (at the centre's height) onto the module's
# plane, [v-, v+] = v of the central projections of the lower and upper face centres, amplitude from pixel - source.

def tilted(cfg, seed, shift_mm=2.0, tilt_rad=0.25):
    return perturbed_poses(cfg, seed, shift_mm=shift_mm, tilt_rad=tilt_rad)


def test_mt1_the_tilted_reading_meets_the_upright_one_as_the_tilt_vanishes(oracle_mod):
    """The same upright poses with their axes rotated by 1e-7 rad about the column axis and the normal: these views
    take the tilted construction (every voxel's own corner projections), the unrotated ones the per-view frame."""
    up = upright(tiny(), 4)
    eps = 1e-7
    poses = []
    for p in up.poses:
        p = np.asarray(p)
        eu, ev = p[6:9], p[9:12]
        n = np.cross(eu, ev)
        eu2 = eu + eps * ev
        eu2 /= np.linalg.norm(eu2)
        ev2 = ev + eps * n
        ev2 -= np.dot(eu2, ev2) * eu2
        ev2 /= np.linalg.norm(ev2)
        poses.append(tuple(np.concatenate([p[0:6], eu2, ev2])))
    near = up.replace(poses=tuple(poses))
    A0, A1 = oracle_mod.dense_matrix(up), oracle_mod.dense_matrix(near)
    assert abs(np.asarray(near.poses)[:, 8]).min() > 1e-9               # column axes leave the horizontal: tilted branch
    np.testing.assert_allclose(A1, A0, rtol=0, atol=2e-5 * A0.max())


def test_mt2_a_module_turned_upside_down_is_the_upright_module_read_backwards(oracle_mod):
    """Both axes negated (a half turn about the normal): pixel (r, c) of the turned module is pixel (nrows-1-r,
    ncols-1-c) of the upright one with the detector shifts negated.  The turned module has row axis -z, so it takes the
    tilted construction at full strength; the upright one takes the per-view frame."""
    up = upright(tiny(), 6)
    turned = up.replace(poses=tuple(tuple(np.concatenate([np.asarray(p)[0:6], -np.asarray(p)[6:12]])) for p in up.poses),
                        shift_u=-up.shift_u, shift_v=-up.shift_v)
    A0 = oracle_mod.dense_matrix(up).reshape(up.nviews, up.nrows, up.ncols, -1)
    A1 = oracle_mod.dense_matrix(turned).reshape(up.nviews, up.nrows, up.ncols, -1)
    np.testing.assert_allclose(A1, A0[:, ::-1, ::-1], rtol=0, atol=1e-12)


def test_mt3_pitched_detector_worked_by_hand(oracle_mod):
    """Source on the x axis at x = L, detector centre at x = L - D, column axis +y, row axis (sin b, 0, cos b) (the top
    of the detector leans towards the source).  A point (x, y, z) with a = L - x projects to
        lambda = D / (a + z tan b),   u = lambda y,   v = lambda z / cos b
    (intersect the ray with the plane by eliminating v from its x and z equations).  One voxel's weight on one pixel is
    then trapezoid and rectangle overlaps worked out below with plain interval arithmetic."""
    L, D, b = 40.0, 65.0, 0.35
    pose = (L, 0.0, 0.0, L - D, 0.0, 0.0, 0.0, 1.0, 0.0, np.sin(b), 0.0, np.cos(b))
    cfg = CTConfig("pitch", CONE, nviews=1, arc_deg=360.0, nrows=9, ncols=11, pixel_v=1.7, pixel_u=1.4,
                   nx=4, ny=5, nz=4, voxel_xy=1.5, voxel_z=1.2, sod=L, sdd=D, shift_u=0.2, shift_v=-0.3,
                   center_x=0.5, center_y=-0.4, center_z=0.3).replace(geom=MODULAR, poses=(pose,))
    u_c, v_c = rm.pixel_centres(cfg)

    def proj(x, y, z):
        lam = D / ((L - x) + z * np.tan(b))
        return lam * y, lam * z / np.cos(b)

    def trap_area_between(t, lo, hi):           # integral over [lo, hi] of the unit-height trapezoid with knots t
        g = np.linspace(lo, hi, 20001)
        h = np.interp(g, t, [0.0, 1.0, 1.0, 0.0], left=0.0, right=0.0)
        return float(np.sum(0.5 * (h[1:] + h[:-1]) * np.diff(g)))

    seen = 0
    for (i, j, k) in [(0, 0, 0), (3, 4, 3), (1, 2, 1), (2, 0, 3), (0, 3, 2)]:
        x = cfg.center_x + (i - 1.5) * cfg.voxel_xy
        y = cfg.center_y + (j - 2.0) * cfg.voxel_xy
        z = cfg.center_z + (k - 1.5) * cfg.voxel_z
        h = cfg.voxel_xy / 2
        t = sorted(proj(x + sx * h, y + sy * h, z)[0] for sx in (-1, 1) for sy in (-1, 1))
        va, vb = proj(x, y, z - cfg.voxel_z / 2)[1], proj(x, y, z + cfg.voxel_z / 2)[1]
        assert vb > va
        for r in range(cfg.nrows):
            for c in range(cfg.ncols):
                fu = trap_area_between(t, u_c[c] - cfg.pixel_u / 2, u_c[c] + cfg.pixel_u / 2) / cfg.pixel_u
                fv = max(0.0, min(v_c[r] + cfg.pixel_v / 2, vb) - max(v_c[r] - cfg.pixel_v / 2, va)) / cfg.pixel_v
                d = np.array([L - D + v_c[r] * np.sin(b) - L, u_c[c], v_c[r] * np.cos(b)])
                amp = cfg.voxel_xy * np.linalg.norm(d) / max(abs(d[0]), abs(d[1]))
                w, Fu, Fv, Am = oracle_mod.weight(cfg, 0, r, c, i, j, k)
                assert abs(Fu - fu) < 2e-7 and abs(Fv - fv) < 1e-12 and abs(Am - amp) < 1e-12, (i, j, k, r, c)
                assert abs(w - amp * fu * fv) < 1e-6
                seen += w > 0
    assert seen > 20


def test_mt4_weights_track_the_beam_average_of_true_chords(oracle_mod):
    from test_curved_pins import _beam_average_chord
    from synthetic import config, reduced
    cfg = tilted(reduced(config(3), 32).with_views([0, 37, 90, 200, 333, 610]), 9, shift_mm=20.0, tilt_rad=0.25)
    assert min(abs(np.asarray(cfg.poses)[:, 8])) > 1e-3
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
    # (measured: 3.5 % at most, 0.7 % on average; a rolled detector sees the voxel's outline turned against its
    # axes, which a separable footprint cannot follow)
    assert devs.max() < 0.08 * A.max() and devs.mean() < 0.015 * A.max(), (devs.max(), devs.mean(), A.max())


def test_mt5_converges_to_analytic_line_integrals(oracle_mod):
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
        cfg = tilted(fine, 13, shift_mm=25.0, tilt_rad=0.25)         # the same poses at every refinement (same seed)
        y = oracle_mod.project(cfg, rasterize(cfg, ells))
        ref = rm.analytic_sinogram(cfg, ells)
        errs.append(np.linalg.norm(y - ref) / np.linalg.norm(ref))
    assert errs[2] < 0.06, errs
    assert errs[0] / errs[1] > 1.5 and errs[1] / errs[2] > 1.5, errs


def test_mt6_moving_the_detector_along_its_rays_changes_nothing(oracle_mod):
    """Detector twice as far from the source, pixels twice as large: every central projection doubles, so the same
    footprints in pixel units and the same ray directions."""
    cfg = tilted(tiny(), 5)
    far = []
    for p in cfg.poses:
        p = np.asarray(p)
        far.append(tuple(np.concatenate([p[0:3], p[0:3] + 2.0 * (p[3:6] - p[0:3]), p[6:12]])))
    cfg2 = cfg.replace(poses=tuple(far), pixel_u=2 * cfg.pixel_u, pixel_v=2 * cfg.pixel_v)
    np.testing.assert_allclose(oracle_mod.dense_matrix(cfg2), oracle_mod.dense_matrix(cfg), rtol=0, atol=1e-11)


def test_mt7_dense_matrix_agrees_with_both_loops_and_mixed_scans(oracle_mod):
    """Tilted and upright views in one scan; the matrix from single weights against the scatter and gather loops."""
    t, u = tilted(tiny(), 7), upright(tiny(), 7)
    cfg = t.replace(poses=tuple(t.poses[a] if a % 2 else u.poses[a] for a in range(t.nviews)))
    A = oracle_mod.dense_matrix(cfg)
    per = cfg.nrows * cfg.ncols
    np.testing.assert_array_equal(A[per:2 * per], oracle_mod.dense_matrix(t)[per:2 * per])
    np.testing.assert_array_equal(A[0:per], oracle_mod.dense_matrix(u)[0:per])
    x, y = uniform_volume(cfg, 3)[0], uniform_sinogram(cfg, 4)[0]
    ax, aty = A @ x.astype(np.float64).ravel(), A.T @ y.astype(np.float64).ravel()
    np.testing.assert_allclose(oracle_mod.project(cfg, x).ravel(), ax, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle_mod.backproject(cfg, y).ravel(), aty, rtol=0, atol=1e-12)
    rays, vox = np.arange(0, A.shape[0], 3), np.arange(0, A.shape[1], 2)
    np.testing.assert_allclose(oracle_mod.project_rays(cfg, x, rays), ax[rays], atol=1e-12)
    np.testing.assert_allclose(oracle_mod.backproject_voxels(cfg, y, vox), aty[vox], atol=1e-12)
    assert oracle_mod.nnz(cfg) == int((A > 0).sum())
    assert (A[per:2 * per] > 0).sum() > 50


def test_mt8_scans_without_a_reading_are_refused(oracle_mod):
    """A source inside the volume's slab in front of the module, and a module that a vertical ray from the source
    would hit: neither has a footprint (no central projection; no amplitude)."""
    inside = (0.3, 0.1, 0.0, -20.0, 0.0, 0.0, 0.0, 1.0, 0.0, 0.1, 0.0, np.sqrt(1 - 0.01))
    below = (0.3, -0.2, 25.0, 0.0, 0.0, -18.0, 1.0, 0.0, 0.0, 0.0, 1.0, 0.0)
    for pose in (inside, below):
        cfg = tiny(nviews=1).replace(geom=MODULAR, poses=(pose,))
        with pytest.raises(AssertionError):
            oracle_mod.dense_matrix(cfg)
        with pytest.raises(AssertionError):
            oracle_mod.project(cfg, uniform_volume(cfg, 1)[0])
