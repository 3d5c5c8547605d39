"""Pins of the CPU oracle against things other than itself (no GPU).

The paper prints no worked numbers for its projector, so the oracle's weight model
(oracle/sf_oracle.h) is tied down by: hand-worked values (tests/golden/worked_values.txt),
closed forms (mass conservation, exact beam/voxel intersection volumes by polygon
clipping), brute-force chord quadrature, analytic ellipsoid line integrals, the dense
matrix and its transpose, symmetries, the parallel-beam limit of cone-beam, and unit
scaling ("CT Projection Models and Geometries": quantitative mm / 1/mm units, matched
transpose).
"""
import math
import os

import numpy as np
import pytest

import reference_math as rm
from synthetic import CTConfig, config, reduced, standard_volume, uniform_sinogram, uniform_volume
from synthetic.configs import CONE, FAN, PARALLEL
from synthetic.phantoms import Ellipsoid, draw_ellipsoids_3d, rasterize

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_values.txt")


def golden():
    vals = {}
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    return vals


def tiny(geom, **kw):
    base = dict(name="tiny", geom=geom, nviews=7, arc_deg=360.0, nrows=6, ncols=9, pixel_v=1.3, pixel_u=0.9,
                nx=5, ny=4, nz=3, voxel_xy=0.8, voxel_z=1.1, sod=30.0, sdd=47.0, shift_v=0.3, shift_u=-0.7,
                center_x=0.4, center_y=-0.3, center_z=0.25, start_deg=11.0)
    if geom == FAN:
        base.update(nrows=1, nz=1, shift_v=0.0, center_z=0.0)
    base.update(kw)
    return CTConfig(**base)


# ---------------------------------------------------------------- P1 worked values

def test_p1_parallel_axis_aligned_views(oracle_mod):
    """phi = 0: image row iy falls wholly into bin iy+16 with weight 1; phi = 90 deg: columns, reversed."""
    cfg = config(1).with_views([0, 45])           # 0 and 90 degrees
    x = standard_volume(1, cfg)
    y = oracle_mod.project(cfg, x)
    x64 = x.astype(np.float64)[0]
    np.testing.assert_allclose(y[0, 0, 16:80], x64.sum(axis=1), rtol=0, atol=1e-12)
    assert np.all(y[0, 0, :16] == 0) and np.all(y[0, 0, 80:] == 0)
    np.testing.assert_allclose(y[1, 0, 16:80], x64.sum(axis=0)[::-1], rtol=0, atol=1e-10)
    assert np.abs(y[1, 0, :16]).max() < 1e-12 and np.abs(y[1, 0, 80:]).max() < 1e-12


def test_p1_parallel_45_degrees(oracle_mod):
    g = golden()
    cfg = config(1).with_views([0]).replace(start_deg=45.0, angles_override=(math.pi / 4,))
    # voxel (i,j)=(32,32) has centre (0.5,0.5): triangle footprint on [-sqrt2/2, sqrt2/2]
    tau, mag = oracle_mod.knots(cfg, 0, 32, 32)
    np.testing.assert_allclose(tau, [-math.sqrt(0.5), 0.0, 0.0, math.sqrt(0.5)], atol=1e-12)
    for c in (47, 48):                             # bins [-1,0] and [0,1]
        w, fu, fv, amp = oracle_mod.weight(cfg, 0, 0, c, 32, 32, 0)
        assert abs(fu - g["par45_Fu"]) < 1e-6
        assert abs(amp - g["par45_amp"]) < 1e-6
        assert abs(w - g["par45_w"]) < 1e-9
    assert oracle_mod.weight(cfg, 0, 0, 46, 32, 32, 0)[0] == 0.0
    assert oracle_mod.weight(cfg, 0, 0, 49, 32, 32, 0)[0] == 0.0


def test_p1_cone_single_voxel(oracle_mod):
    g = golden()
    cfg = CTConfig("one", CONE, nviews=1, arc_deg=360.0, nrows=5, ncols=5, pixel_v=1.0, pixel_u=1.0,
                   nx=1, ny=1, nz=1, voxel_xy=1.0, voxel_z=1.0, sod=1000.0, sdd=1500.0)
    tau, mag = oracle_mod.knots(cfg, 0, 0, 0)
    np.testing.assert_allclose(tau, [-g["cone_tau3"], -g["cone_tau2"], g["cone_tau2"], g["cone_tau3"]], atol=5e-8)
    assert abs(mag - 1.5) < 1e-15
    assert abs(oracle_mod.trapezoid_integral(tau, 10.0) - g["cone_Gtot"]) < 5e-8
    w, fu, fv, amp = oracle_mod.weight(cfg, 0, 2, 2, 0, 0, 0)
    assert abs(w - 1.0) < 1e-14 and abs(fu - 1.0) < 1e-14 and fv == 1.0 and amp == 1.0
    w, fu, fv, amp = oracle_mod.weight(cfg, 0, 2, 3, 0, 0, 0)      # u neighbour
    assert abs(fu - g["cone_Fu_neighbour"]) < 5e-8 and fv == 1.0
    assert abs(amp - g["cone_amp_neighbour"]) < 5e-9
    assert abs(w - g["cone_w_u_neighbour"]) < 1e-7
    w, fu, fv, amp = oracle_mod.weight(cfg, 0, 3, 2, 0, 0, 0)      # v neighbour
    assert abs(fv - 0.25) < 1e-14 and abs(fu - 1.0) < 1e-14
    assert abs(amp - g["cone_amp_neighbour"]) < 5e-9
    # symmetric partners
    assert abs(oracle_mod.weight(cfg, 0, 2, 1, 0, 0, 0)[0] - g["cone_w_u_neighbour"]) < 1e-7
    assert abs(oracle_mod.weight(cfg, 0, 1, 2, 0, 0, 0)[2] - 0.25) < 1e-14


def test_trapezoid_integral_is_integral_of_unit_trapezoid(oracle_mod):
    tau = [-1.3, -0.2, 0.5, 2.0]
    us = np.linspace(-2, 3, 20001)
    trap = np.interp(us, tau, [0, 1, 1, 0], left=0, right=0)
    cum = np.concatenate([[0], np.cumsum(0.5 * (trap[1:] + trap[:-1]) * np.diff(us))])
    got = np.array([oracle_mod.trapezoid_integral(tau, u) for u in us[::500]])
    np.testing.assert_allclose(got, cum[::500], atol=1e-7)
    # degenerate ramps (axis-aligned view): a rectangle
    rect = [0.0, 0.0, 1.0, 1.0]
    assert oracle_mod.trapezoid_integral(rect, 0.25) == 0.25
    assert oracle_mod.trapezoid_integral(rect, 0.0) == 0.0
    assert oracle_mod.trapezoid_integral(rect, 1.0) == 1.0
    assert oracle_mod.trapezoid_integral(rect, 7.0) == 1.0


# ---------------------------------------------------------------- P2 / P3 mass

def test_p2_parallel_mass_is_conserved_every_view(oracle_mod):
    cfg = config(1)
    x = standard_volume(1, cfg)
    y = oracle_mod.project(cfg, x)
    mass = x.astype(np.float64).sum() * cfg.voxel_xy ** 2 * cfg.voxel_z
    per_view = y.sum(axis=(1, 2)) * cfg.pixel_u * cfg.pixel_v
    np.testing.assert_allclose(per_view, mass, rtol=1e-13)


def test_p2_parallel_mass_3d_anisotropic(oracle_mod):
    cfg = CTConfig("m", PARALLEL, nviews=11, arc_deg=180.0, nrows=24, ncols=40, pixel_v=0.7, pixel_u=0.6,
                   nx=12, ny=10, nz=9, voxel_xy=1.1, voxel_z=1.3, shift_u=0.4, shift_v=-0.8,
                   center_x=0.5, center_y=-1.0, center_z=0.3, start_deg=3.0)
    x = uniform_volume(cfg, 7)[0]
    y = oracle_mod.project(cfg, x)
    mass = x.astype(np.float64).sum() * cfg.voxel_xy ** 2 * cfg.voxel_z
    np.testing.assert_allclose(y.sum(axis=(1, 2)) * cfg.pixel_u * cfg.pixel_v, mass, rtol=1e-13)


def test_p3_cone_footprint_mass(oracle_mod):
    """Interior voxel: sum over pixels of (w/amp) pu pv = G_tot * M_c * Tz, knots = projected corners."""
    cfg = tiny(CONE, nrows=40, ncols=40, pixel_u=0.5, pixel_v=0.5, shift_u=0.2, shift_v=-0.4)
    for a in range(cfg.nviews):
        phi = cfg.angles()[a]
        for (i, j, k) in [(0, 0, 0), (2, 1, 1), (4, 3, 2)]:
            x = cfg.center_x + (i - (cfg.nx - 1) / 2) * cfg.voxel_xy
            y = cfg.center_y + (j - (cfg.ny - 1) / 2) * cfg.voxel_xy
            us = []
            for dx in (-0.5, 0.5):
                for dy in (-0.5, 0.5):
                    xx, yy = x + dx * cfg.voxel_xy, y + dy * cfg.voxel_xy
                    t = -xx * math.sin(phi) + yy * math.cos(phi)
                    l = xx * math.cos(phi) + yy * math.sin(phi)
                    us.append(cfg.sdd * t / (cfg.sod - l))
            us.sort()
            gtot = 0.5 * ((us[3] - us[0]) + (us[2] - us[1]))
            mc = cfg.sdd / (cfg.sod - (x * math.cos(phi) + y * math.sin(phi)))
            total = 0.0
            for r in range(cfg.nrows):
                for c in range(cfg.ncols):
                    w, fu, fv, amp = oracle_mod.weight(cfg, a, r, c, i, j, k)
                    total += fu * fv
            total *= cfg.pixel_u * cfg.pixel_v
            assert abs(total - gtot * mc * cfg.voxel_z) < 1e-12 * max(1.0, total)


# ---------------------------------------------------------------- P4 exact parallel weights

def test_p4_parallel_weight_is_exact_intersection_volume(oracle_mod):
    cfg = tiny(PARALLEL, nviews=9, arc_deg=180.0)
    A = oracle_mod.dense_matrix(cfg)
    u, v = rm.pixel_centres(cfg)
    n = cfg.nx * cfg.ny * cfg.nz
    worst = 0.0
    for a in range(cfg.nviews):
        phi = cfg.angles()[a]
        for r in range(cfg.nrows):
            for c in range(cfg.ncols):
                row = A[(a * cfg.nrows + r) * cfg.ncols + c].reshape(cfg.vol_shape)
                for k in range(cfg.nz):
                    z = cfg.center_z + (k - (cfg.nz - 1) / 2) * cfg.voxel_z
                    zo = max(0.0, min(v[r] + cfg.pixel_v / 2, z + cfg.voxel_z / 2) - max(v[r] - cfg.pixel_v / 2, z - cfg.voxel_z / 2))
                    for j in range(cfg.ny):
                        for i in range(cfg.nx):
                            x = cfg.center_x + (i - (cfg.nx - 1) / 2) * cfg.voxel_xy
                            y = cfg.center_y + (j - (cfg.ny - 1) / 2) * cfg.voxel_xy
                            area = rm.strip_square_area((x, y), cfg.voxel_xy, phi, u[c] - cfg.pixel_u / 2, u[c] + cfg.pixel_u / 2) if zo > 0 else 0.0
                            expect = area * zo / (cfg.pixel_u * cfg.pixel_v)
                            worst = max(worst, abs(row[k, j, i] - expect))
    assert worst < 1e-12, worst
    assert A.max() > 0.3


# ---------------------------------------------------------------- P5 cone: SF approximates the beam average of chords

def _beam_average_chord(cfg, a, r, c, i, j, k, nsub=24):
    u, v = rm.pixel_centres(cfg)
    s = (np.arange(nsub) + 0.5) / nsub - 0.5
    uu, vv = np.meshgrid(u[c] + s * cfg.pixel_u, v[r] + s * cfg.pixel_v)
    p, d = rm.ray_endpoints(cfg, a, uu, vv)
    ctr = np.array([cfg.center_x + (i - (cfg.nx - 1) / 2) * cfg.voxel_xy,
                    cfg.center_y + (j - (cfg.ny - 1) / 2) * cfg.voxel_xy,
                    cfg.center_z + (k - (cfg.nz - 1) / 2) * cfg.voxel_z])
    h = np.array([cfg.voxel_xy, cfg.voxel_xy, cfg.voxel_z]) / 2
    return rm.box_chord(p, d, ctr - h, ctr + h).mean()


def test_p5_cone_weights_track_true_chord_average(oracle_mod):
    """C3's cone angles on a coarse grid: SF is an approximation, so only a loose bound is asserted."""
    cfg = reduced(config(3), 32).with_views([0, 37, 90, 200, 333, 610])       # 16^3 volume, 16x16 detector
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
    scale = A.max()
    assert devs.max() < 0.05 * scale, (devs.max(), scale)
    assert devs.mean() < 0.01 * scale, (devs.mean(), scale)
    # a pair the model says is disjoint must be (nearly) disjoint for real rays too
    zero_pairs = np.argwhere(A[:, ::7] == 0)
    pick0 = zero_pairs[rng.choice(len(zero_pairs), 200, replace=False)]
    for ray, vq in pick0:
        vox = vq * 7
        a, rem = divmod(ray, cfg.nrows * cfg.ncols)
        r, c = divmod(rem, cfg.ncols)
        k, rem = divmod(vox, cfg.ny * cfg.nx)
        j, i = divmod(rem, cfg.nx)
        assert _beam_average_chord(cfg, a, r, c, i, j, k, nsub=8) < 0.05 * scale


# ---------------------------------------------------------------- P6 analytic ellipsoids

def _analytic_error(oracle_mod, cfg, ells):
    x = rasterize(cfg, ells)
    y = oracle_mod.project(cfg, x)
    ref = rm.analytic_sinogram(cfg, ells)
    return np.linalg.norm(y - ref) / np.linalg.norm(ref)


@pytest.mark.parametrize("geom", [PARALLEL, CONE])
def test_p6_converges_to_analytic_line_integrals(oracle_mod, geom):
    """Oblique, off-centre ellipsoids, shifted detector and volume: the sinogram of the voxelised
    phantom approaches the closed-form chords as grid and detector are refined together."""
    base = CTConfig("an", geom, nviews=5, arc_deg=360.0, nrows=16, ncols=24, pixel_v=4.0, pixel_u=4.0,
                    nx=16, ny=16, nz=12, voxel_xy=4.0, voxel_z=4.0, sod=400.0, sdd=600.0,
                    shift_u=0.35, shift_v=-0.2, center_x=3.0, center_y=-2.0, center_z=1.5, start_deg=17.0)
    if geom == CONE:
        base = base.replace(pixel_u=6.0, pixel_v=6.0)
    ells = [Ellipsoid((8.0, -5.0, 3.0), (20.0, 11.0, 14.0), _rot(0.4, 0.3, -0.5), 1.0),
            Ellipsoid((-9.0, 10.0, -4.0), (9.0, 14.0, 8.0), _rot(-0.8, 0.1, 0.6), 0.6)]
    errs = [_analytic_error(oracle_mod, reduced(base, 1), ells)]
    for f in (2, 4):
        fine = base.replace(nrows=base.nrows * f, ncols=base.ncols * f, pixel_u=base.pixel_u / f, pixel_v=base.pixel_v / f,
                            nx=base.nx * f, ny=base.ny * f, nz=base.nz * f, voxel_xy=base.voxel_xy / f,
                            voxel_z=base.voxel_z / f, shift_u=base.shift_u * f, shift_v=base.shift_v * f)
        errs.append(_analytic_error(oracle_mod, fine, ells))
    assert errs[2] < 0.06, errs
    assert errs[0] / errs[1] > 1.5 and errs[1] / errs[2] > 1.5, errs


def _rot(a, b, c):
    ca, sa, cb, sb, cc, sc = math.cos(a), math.sin(a), math.cos(b), math.sin(b), math.cos(c), math.sin(c)
    rz = np.array([[ca, -sa, 0], [sa, ca, 0], [0, 0, 1]])
    ry = np.array([[cb, 0, sb], [0, 1, 0], [-sb, 0, cb]])
    rx = np.array([[1, 0, 0], [0, cc, -sc], [0, sc, cc]])
    return tuple((rz @ ry @ rx).reshape(-1))


def test_p6_fan_matches_analytic_disc(oracle_mod):
    cfg = CTConfig("fan", FAN, nviews=8, arc_deg=360.0, nrows=1, ncols=160, pixel_v=1.0, pixel_u=0.5,
                   nx=128, ny=128, nz=1, voxel_xy=0.25, voxel_z=1.0, sod=80.0, sdd=130.0, shift_u=1.25,
                   center_x=1.0, center_y=0.5, start_deg=5.0)
    ells = [Ellipsoid((3.0, -2.0, 0.0), (9.0, 5.0, 1e9), _rot(0.5, 0.0, 0.0), 1.0)]
    err = _analytic_error(oracle_mod, cfg, ells)
    assert err < 0.02, err


# ---------------------------------------------------------------- P7 / P8 transpose

@pytest.mark.parametrize("geom", [PARALLEL, FAN, CONE])
def test_p7_dense_matrix_agrees_with_both_loops(oracle_mod, geom):
    cfg = tiny(geom)
    A = oracle_mod.dense_matrix(cfg)
    assert (A >= 0).all() and A.max() > 0
    x = uniform_volume(cfg, 3)[0]
    y = uniform_sinogram(cfg, 4)[0]
    np.testing.assert_allclose(oracle_mod.project(cfg, x).ravel(), A @ x.astype(np.float64).ravel(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle_mod.backproject(cfg, y).ravel(), A.T @ y.astype(np.float64).ravel(), rtol=0, atol=1e-12)
    # sampled entry points and the nonzero count
    rays = np.arange(0, A.shape[0], 3)
    vox = np.arange(0, A.shape[1], 2)
    np.testing.assert_allclose(oracle_mod.project_rays(cfg, x, rays), (A @ x.astype(np.float64).ravel())[rays], atol=1e-12)
    np.testing.assert_allclose(oracle_mod.backproject_voxels(cfg, y, vox), (A.T @ y.astype(np.float64).ravel())[vox], atol=1e-12)
    assert oracle_mod.nnz(cfg) == int((A > 0).sum())
    per = cfg.nrows * cfg.ncols
    assert oracle_mod.nnz(cfg, 2, 5) == int((A[2 * per:5 * per] > 0).sum())


@pytest.mark.parametrize("number,factor,nviews", [(1, 1, 90), (2, 8, 12), (3, 16, 24), (5, 32, 16)])
def test_p8_adjoint_identity(oracle_mod, number, factor, nviews):
    cfg = reduced(config(number), factor, nviews=nviews)
    x = uniform_volume(cfg, 11)[0]
    y = uniform_sinogram(cfg, 12)[0]
    lhs = float((oracle_mod.project(cfg, x) * y).sum())
    rhs = float((oracle_mod.backproject(cfg, y) * x).sum())
    assert abs(lhs - rhs) <= 1e-12 * abs(lhs)


# ---------------------------------------------------------------- P9 symmetries

@pytest.mark.parametrize("geom", [PARALLEL, CONE])
def test_p9_quarter_turn(oracle_mod, geom):
    """Rotating the object by +90 deg about z equals looking from 90 deg less."""
    cfg = tiny(geom, nx=6, ny=6, center_x=0.4, center_y=-0.3)
    x = uniform_volume(cfg, 21)[0]
    y0 = oracle_mod.project(cfg, x)
    # rotate by +90 deg: new(x', y') = old(y', -x')  -> array [z][y][x]: rot90 in the (y,x) plane
    xr = np.ascontiguousarray(np.rot90(x, k=1, axes=(2, 1)))        # new[j', i'] = old[j=nx-1-i' ... ]
    cfg_r = cfg.replace(center_x=-cfg.center_y, center_y=cfg.center_x, start_deg=cfg.start_deg + 90.0)
    y1 = oracle_mod.project(cfg_r, xr)
    np.testing.assert_allclose(y1, y0, rtol=0, atol=1e-12)


@pytest.mark.parametrize("geom", [PARALLEL, CONE])
def test_p9_axial_flip(oracle_mod, geom):
    cfg = tiny(geom)
    x = uniform_volume(cfg, 22)[0]
    y0 = oracle_mod.project(cfg, x)
    cfg_f = cfg.replace(center_z=-cfg.center_z, shift_v=-cfg.shift_v)
    y1 = oracle_mod.project(cfg_f, np.ascontiguousarray(x[::-1]))
    np.testing.assert_allclose(y1[:, ::-1, :], y0, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P10 / P11

def test_p10_far_source_reproduces_parallel(oracle_mod):
    """Deviation from parallel-beam weights shrinks like (detector distance)/SOD as the source recedes."""
    par = tiny(PARALLEL)
    Ap = oracle_mod.dense_matrix(par)
    devs = []
    for far in (1e5, 1e7, 1e9):
        cone = par.replace(geom=CONE, sod=far, sdd=far + 50.0)
        devs.append(np.abs(Ap - oracle_mod.dense_matrix(cone)).max() / Ap.max())
    assert devs[0] < 5e-3 and devs[1] < 5e-5 and devs[2] < 5e-7, devs
    assert devs[0] > 50 * devs[1] > 50 * 50 * devs[2] * 0.5, devs


@pytest.mark.parametrize("geom", [PARALLEL, FAN, CONE])
def test_p11_unit_scaling(oracle_mod, geom):
    """Lengths times s and densities divided by s leave the (dimensionless) sinogram unchanged."""
    cfg = tiny(geom)
    s = 2.5
    big = cfg.replace(pixel_u=cfg.pixel_u * s, pixel_v=cfg.pixel_v * s, voxel_xy=cfg.voxel_xy * s,
                      voxel_z=cfg.voxel_z * s, sod=cfg.sod * s, sdd=cfg.sdd * s,
                      center_x=cfg.center_x * s, center_y=cfg.center_y * s, center_z=cfg.center_z * s)
    A0 = oracle_mod.dense_matrix(cfg)
    A1 = oracle_mod.dense_matrix(big)
    np.testing.assert_allclose(A1, A0 * s, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- geometry conventions

def test_detector_shift_moves_pixel_centres_positive(oracle_mod):
    """A point-like voxel at t>0 lands at higher column index; +shift_u lowers that index by the shift."""
    cfg = CTConfig("s", PARALLEL, nviews=1, arc_deg=180.0, nrows=1, ncols=41, pixel_v=1.0, pixel_u=1.0,
                   nx=1, ny=1, nz=1, voxel_xy=1.0, voxel_z=1.0, center_y=5.0)
    A = oracle_mod.dense_matrix(cfg)[:, 0]
    assert A.argmax() == 25
    A = oracle_mod.dense_matrix(cfg.replace(shift_u=3.0))[:, 0]
    assert A.argmax() == 22


def test_cone_magnification_and_row_order(oracle_mod):
    cfg = CTConfig("m", CONE, nviews=1, arc_deg=360.0, nrows=41, ncols=41, pixel_v=1.0, pixel_u=1.0,
                   nx=1, ny=1, nz=1, voxel_xy=0.2, voxel_z=0.2, sod=100.0, sdd=200.0,
                   center_x=50.0, center_y=2.0, center_z=1.0)
    # voxel half way to the source: magnification 200/(100-50)=4 -> u=8, v=4
    A = oracle_mod.dense_matrix(cfg)[:, 0].reshape(41, 41)
    r, c = np.unravel_index(A.argmax(), A.shape)
    assert (r, c) == (24, 28)
