"""Pins of the Siddon CPU oracle (oracle/siddon_oracle.c) against things other than itself (no GPU).

The Siddon weight has a plain definition (length of the pixel-centre ray inside the voxel box), so the pins are:
a brute-force recomputation of every weight with an independent numpy slab routine on rays built from the coordinate
conventions (tests/reference_math.py), the sum rule (the chords of one ray add up to its chord through the whole
volume box), hand-worked rays, the half-open rule for a ray inside a face plane, analytic ellipsoid line integrals,
the dense matrix and its transpose, symmetries, unit scaling and the parallel-beam limit of cone-beam.
"""
import math

import numpy as np
import pytest

import reference_math as rm
from synthetic import CTConfig, config, reduced, uniform_sinogram, uniform_volume
from synthetic.configs import CONE, FAN, PARALLEL
from synthetic.phantoms import Ellipsoid, rasterize


@pytest.fixture(scope="module")
def sd(oracle_mod):
    return oracle_mod.siddon


def tiny(geom, **kw):
    base = dict(name="tiny", geom=geom, nviews=7, arc_deg=360.0, nrows=6, ncols=9, pixel_v=1.3, pixel_u=0.9,
                nx=5, ny=4, nz=3, voxel_xy=0.8, voxel_z=1.1, sod=30.0, sdd=47.0, shift_v=0.3, shift_u=-0.7,
                center_x=0.4, center_y=-0.3, center_z=0.25, start_deg=11.0)
    if geom == FAN:
        base.update(nrows=1, nz=1, shift_v=0.0, center_z=0.0)
    base.update(kw)
    return CTConfig(**base)


def voxel_boxes(cfg):
    """(lo, hi) corner arrays [nvox][3] in the linear voxel order (k*ny+j)*nx+i."""
    k, j, i = np.meshgrid(np.arange(cfg.nz), np.arange(cfg.ny), np.arange(cfg.nx), indexing="ij")
    cx = cfg.center_x + (i - (cfg.nx - 1) / 2.0) * cfg.voxel_xy
    cy = cfg.center_y + (j - (cfg.ny - 1) / 2.0) * cfg.voxel_xy
    cz = cfg.center_z + (k - (cfg.nz - 1) / 2.0) * cfg.voxel_z
    c = np.stack([cx, cy, cz], axis=-1).reshape(-1, 3)
    h = np.array([cfg.voxel_xy, cfg.voxel_xy, cfg.voxel_z]) / 2.0
    if cfg.geom == FAN:
        h[2] = 1e6                       # in-plane square: the slice is as thick as it likes
    return c - h, c + h


def volume_box(cfg):
    c = np.array([cfg.center_x, cfg.center_y, cfg.center_z])
    h = np.array([cfg.nx * cfg.voxel_xy, cfg.ny * cfg.voxel_xy, cfg.nz * cfg.voxel_z]) / 2.0
    if cfg.geom == FAN:
        h[2] = 1e6
    return c - h, c + h


def all_rays(cfg):
    """(p, d) [nrays][3] in the linear ray order (view*nrows+r)*ncols+c, from reference_math's conventions."""
    u, v = rm.pixel_centres(cfg)
    uu, vv = np.meshgrid(u, v)
    ps, ds = [], []
    for a in range(cfg.nviews):
        p, d = rm.ray_endpoints(cfg, a, uu, vv)
        ps.append(np.broadcast_to(p, d.shape).reshape(-1, 3))
        ds.append(d.reshape(-1, 3))
    return np.concatenate(ps), np.concatenate(ds)


# ---------------------------------------------------------------- S1 brute force

@pytest.mark.parametrize("geom", [PARALLEL, FAN, CONE])
def test_s1_every_weight_equals_numpy_slab_chord(sd, geom):
    cfg = tiny(geom)
    A = sd.dense_matrix(cfg)
    p, d = all_rays(cfg)
    lo, hi = voxel_boxes(cfg)
    ref = rm.box_chord(p[:, None, :], d[:, None, :], lo[None], hi[None])
    assert A.shape == ref.shape and A.max() > 0.5 * cfg.voxel_xy
    np.testing.assert_allclose(A, ref, rtol=0, atol=1e-12)


def test_s1_anisotropic_steep_cone(sd):
    """Thin slices and a wide cone angle: rays cross several slices inside one in-plane voxel."""
    cfg = tiny(CONE, nz=9, voxel_z=0.21, nrows=8, pixel_v=2.9, sod=9.0, sdd=14.0, center_z=-0.1)
    A = sd.dense_matrix(cfg)
    p, d = all_rays(cfg)
    lo, hi = voxel_boxes(cfg)
    np.testing.assert_allclose(A, rm.box_chord(p[:, None, :], d[:, None, :], lo[None], hi[None]), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- S2 sum rule

@pytest.mark.parametrize("number,factor,nviews", [(1, 1, 30), (2, 8, 9), (3, 16, 12), (5, 32, 8)])
def test_s2_chords_add_up_to_the_chord_through_the_volume(sd, number, factor, nviews):
    cfg = reduced(config(number), factor, nviews=nviews)
    y = sd.project(cfg, np.ones(cfg.vol_shape, dtype=np.float32))
    p, d = all_rays(cfg)
    lo, hi = volume_box(cfg)
    ref = rm.box_chord(p, d, lo, hi).reshape(cfg.sino_shape)
    assert ref.max() > 0
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-9 * ref.max())


# ---------------------------------------------------------------- S3 hand-worked rays

def test_s3_parallel_axis_aligned(sd):
    """phi = 0: the ray of column c runs along x at y = u_c, through one image row, T per voxel."""
    cfg = CTConfig("hand", PARALLEL, nviews=1, arc_deg=360.0, nrows=1, ncols=8, pixel_v=1.0, pixel_u=0.5,
                   nx=6, ny=4, nz=1, voxel_xy=1.0, voxel_z=1.0, sod=0.0, sdd=0.0)
    x = uniform_volume(cfg, 5)[0]
    y = sd.project(cfg, x)
    # u_c = (c - 3.5) * 0.5 = -1.75 .. 1.75; row faces at y = -2,-1,0,1,2 -> rows 0,0,1,1,2,2,3,3
    rows = [0, 0, 1, 1, 2, 2, 3, 3]
    for c in range(8):
        assert y[0, 0, c] == pytest.approx(float(x[0, rows[c]].astype(np.float64).sum()), abs=1e-12)


def test_s3_parallel_diagonal(sd):
    """phi = 45 deg, ray through the volume centre: sqrt(2) T in every diagonal voxel, nothing elsewhere;
    its neighbour at distance T/(2 sqrt 2) cuts a corner triangle leg T/2 off... in closed form."""
    T = 0.7
    cfg = CTConfig("diag", PARALLEL, nviews=1, arc_deg=360.0, nrows=1, ncols=3, pixel_v=1.0, pixel_u=T / math.sqrt(8.0),
                   nx=4, ny=4, nz=1, voxel_xy=T, voxel_z=1.0, sod=0.0, sdd=0.0, start_deg=45.0)
    A = sd.dense_matrix(cfg).reshape(3, 4, 4)            # [c][j][i]
    centre = np.zeros((4, 4))
    centre[np.arange(4), np.arange(4)] = math.sqrt(2.0) * T
    np.testing.assert_allclose(A[1], centre, rtol=0, atol=1e-12)
    # offset ray at u = +T/(2 sqrt 2): the line y = x + T/2; it crosses diagonal voxels for half their diagonal
    # and the voxels above the diagonal (j = i + 1) for the other half
    off = np.zeros((4, 4))
    off[np.arange(4), np.arange(4)] = T / math.sqrt(2.0)
    off[np.arange(1, 4), np.arange(3)] = T / math.sqrt(2.0)
    np.testing.assert_allclose(A[2], off, rtol=0, atol=1e-12)


def test_s3_cone_central_and_oblique_ray(sd):
    """One voxel of side 2 at the origin, source at distance 10.  The central ray has chord 2.  The ray to
    (u, v) = (1.5, 0) at SDD 15 has slope 0.1 in the plane: it enters through x = 1 at y = 0.9 and leaves through
    x = -1 at y = 1.1, i.e. it exits through the face y = 1 at x = 0: chord = sqrt(1 + 0.01) * 1."""
    cfg = CTConfig("one", CONE, nviews=1, arc_deg=360.0, nrows=1, ncols=3, pixel_v=1.0, pixel_u=1.5,
                   nx=1, ny=1, nz=1, voxel_xy=2.0, voxel_z=2.0, sod=10.0, sdd=15.0)
    A = sd.dense_matrix(cfg).ravel()
    assert A[1] == pytest.approx(2.0, abs=1e-12)
    assert A[2] == pytest.approx(math.sqrt(1.01), abs=1e-12)
    assert A[0] == pytest.approx(math.sqrt(1.01), abs=1e-12)
    # same voxel, ray tilted axially only: (u, v) = (0, 1.5): leaves through z = 1 at x = 0
    cfg = cfg.replace(nrows=3, ncols=1, pixel_v=1.5, pixel_u=1.0)
    A = sd.dense_matrix(cfg).ravel()
    assert A[1] == pytest.approx(2.0, abs=1e-12)
    assert A[0] == pytest.approx(math.sqrt(1.01), abs=1e-12) and A[2] == pytest.approx(math.sqrt(1.01), abs=1e-12)


def test_s3_fan_ignores_the_slice_thickness(sd):
    cfg = tiny(FAN)
    A0 = sd.dense_matrix(cfg)
    A1 = sd.dense_matrix(cfg.replace(voxel_z=0.01))
    np.testing.assert_array_equal(A0, A1)


# ---------------------------------------------------------------- S4 half-open rule

def test_s4_ray_inside_a_face_plane_belongs_to_the_upper_voxel(sd):
    """phi = 0 exactly (sin 0 = 0): with an odd number of columns and an even number of rows the middle ray runs in
    the plane y = 0, the face between image rows 1 and 2; the half-open box gives it to row 2, once."""
    cfg = CTConfig("face", PARALLEL, nviews=1, arc_deg=360.0, nrows=1, ncols=5, pixel_v=1.0, pixel_u=1.0,
                   nx=3, ny=4, nz=1, voxel_xy=1.0, voxel_z=1.0, sod=0.0, sdd=0.0)
    A = sd.dense_matrix(cfg).reshape(5, 4, 3)
    np.testing.assert_array_equal(A[2, 2], [1.0, 1.0, 1.0])
    assert A[2, 1].max() == 0.0 and A[2, 0].max() == 0.0 and A[2, 3].max() == 0.0
    # the outermost rays run in the planes y = -2 (lower face of row 0: inside) and y = +2 (upper face of row 3: outside)
    np.testing.assert_array_equal(A[0, 0], [1.0, 1.0, 1.0])
    assert A[4].max() == 0.0


# ---------------------------------------------------------------- S5 analytic ellipsoids

def _rot(a, b, c):
    ca, sa, cb, sb, cc, sc = math.cos(a), math.sin(a), math.cos(b), math.sin(b), math.cos(c), math.sin(c)
    rz = np.array([[ca, -sa, 0], [sa, ca, 0], [0, 0, 1]])
    ry = np.array([[cb, 0, sb], [0, 1, 0], [-sb, 0, cb]])
    rx = np.array([[1, 0, 0], [0, cc, -sc], [0, sc, cc]])
    return tuple((rz @ ry @ rx).reshape(-1))


def _analytic_error(sd, cfg, ells):
    y = sd.project(cfg, rasterize(cfg, ells))
    ref = rm.analytic_sinogram(cfg, ells)
    return np.linalg.norm(y - ref) / np.linalg.norm(ref)


@pytest.mark.parametrize("geom", [PARALLEL, CONE])
def test_s5_converges_to_analytic_line_integrals(sd, geom):
    """The detector stays fixed (Siddon rays are lines through pixel centres, exactly what the closed form
    integrates along); only the voxel grid is refined."""
    base = CTConfig("an", geom, nviews=5, arc_deg=360.0, nrows=24, ncols=32, pixel_v=3.0, pixel_u=3.0,
                    nx=16, ny=16, nz=12, voxel_xy=4.0, voxel_z=4.0, sod=400.0, sdd=600.0,
                    shift_u=0.35, shift_v=-0.2, center_x=3.0, center_y=-2.0, center_z=1.5, start_deg=17.0)
    if geom == CONE:
        base = base.replace(pixel_u=4.5, pixel_v=4.5)
    ells = [Ellipsoid((8.0, -5.0, 3.0), (20.0, 11.0, 14.0), _rot(0.4, 0.3, -0.5), 1.0),
            Ellipsoid((-9.0, 10.0, -4.0), (9.0, 14.0, 8.0), _rot(-0.8, 0.1, 0.6), 0.6)]
    errs = []
    for f in (1, 2, 4):
        fine = base.replace(nx=base.nx * f, ny=base.ny * f, nz=base.nz * f, voxel_xy=base.voxel_xy / f,
                            voxel_z=base.voxel_z / f)
        errs.append(_analytic_error(sd, fine, ells))
    assert errs[2] < 0.05, errs
    assert errs[0] / errs[1] > 1.4 and errs[1] / errs[2] > 1.4, errs


def test_s5_fan_matches_analytic_disc(sd):
    cfg = CTConfig("fan", FAN, nviews=8, arc_deg=360.0, nrows=1, ncols=160, pixel_v=1.0, pixel_u=0.5,
                   nx=128, ny=128, nz=1, voxel_xy=0.25, voxel_z=1.0, sod=80.0, sdd=130.0, shift_u=1.25,
                   center_x=1.0, center_y=0.5, start_deg=5.0)
    ells = [Ellipsoid((3.0, -2.0, 0.0), (9.0, 5.0, 1e9), _rot(0.5, 0.0, 0.0), 1.0)]
    assert _analytic_error(sd, cfg, ells) < 0.02


# ---------------------------------------------------------------- S6 transpose

@pytest.mark.parametrize("geom", [PARALLEL, FAN, CONE])
def test_s6_dense_matrix_agrees_with_both_loops(sd, geom):
    cfg = tiny(geom)
    A = sd.dense_matrix(cfg)
    x = uniform_volume(cfg, 3)[0]
    y = uniform_sinogram(cfg, 4)[0]
    ax, aty = A @ x.astype(np.float64).ravel(), A.T @ y.astype(np.float64).ravel()
    np.testing.assert_allclose(sd.project(cfg, x).ravel(), ax, rtol=0, atol=1e-12)
    np.testing.assert_allclose(sd.backproject(cfg, y).ravel(), aty, rtol=0, atol=1e-12)
    rays = np.arange(0, A.shape[0], 3)
    vox = np.arange(0, A.shape[1], 2)
    np.testing.assert_allclose(sd.project_rays(cfg, x, rays), ax[rays], atol=1e-12)
    np.testing.assert_allclose(sd.backproject_voxels(cfg, y, vox), aty[vox], atol=1e-12)
    assert sd.nnz(cfg) == int((A > 0).sum())
    per = cfg.nrows * cfg.ncols
    assert sd.nnz(cfg, 2, 5) == int((A[2 * per:5 * per] > 0).sum())


def test_s6_steep_cone_loops_agree_with_dense(sd):
    cfg = tiny(CONE, nz=9, voxel_z=0.21, nrows=8, pixel_v=2.9, sod=9.0, sdd=14.0, center_z=-0.1)
    A = sd.dense_matrix(cfg)
    x = uniform_volume(cfg, 3)[0]
    y = uniform_sinogram(cfg, 4)[0]
    np.testing.assert_allclose(sd.project(cfg, x).ravel(), A @ x.astype(np.float64).ravel(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(sd.backproject(cfg, y).ravel(), A.T @ y.astype(np.float64).ravel(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("number,factor,nviews", [(1, 1, 45), (2, 8, 12), (3, 16, 24), (5, 32, 16)])
def test_s6_adjoint_identity(sd, number, factor, nviews):
    cfg = reduced(config(number), factor, nviews=nviews)
    x = uniform_volume(cfg, 11)[0]
    y = uniform_sinogram(cfg, 12)[0]
    lhs = float((sd.project(cfg, x) * y).sum())
    rhs = float((sd.backproject(cfg, y) * x).sum())
    assert abs(lhs - rhs) <= 1e-12 * abs(lhs)


# ---------------------------------------------------------------- S7 symmetries

@pytest.mark.parametrize("geom", [PARALLEL, CONE])
def test_s7_quarter_turn(sd, geom):
    cfg = tiny(geom, nx=6, ny=6, center_x=0.4, center_y=-0.3)
    x = uniform_volume(cfg, 21)[0]
    y0 = sd.project(cfg, x)
    xr = np.ascontiguousarray(np.rot90(x, k=1, axes=(2, 1)))
    cfg_r = cfg.replace(center_x=-cfg.center_y, center_y=cfg.center_x, start_deg=cfg.start_deg + 90.0)
    np.testing.assert_allclose(sd.project(cfg_r, xr), y0, rtol=0, atol=1e-12)


@pytest.mark.parametrize("geom", [PARALLEL, CONE])
def test_s7_axial_flip(sd, geom):
    cfg = tiny(geom)
    x = uniform_volume(cfg, 22)[0]
    y0 = sd.project(cfg, x)
    cfg_f = cfg.replace(center_z=-cfg.center_z, shift_v=-cfg.shift_v)
    y1 = sd.project(cfg_f, np.ascontiguousarray(x[::-1]))
    np.testing.assert_allclose(y1[:, ::-1, :], y0, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- S8 / S9

@pytest.mark.parametrize("geom", [PARALLEL, FAN, CONE])
def test_s8_unit_scaling(sd, geom):
    cfg = tiny(geom)
    s = 2.5
    big = cfg.replace(pixel_u=cfg.pixel_u * s, pixel_v=cfg.pixel_v * s, voxel_xy=cfg.voxel_xy * s,
                      voxel_z=cfg.voxel_z * s, sod=cfg.sod * s, sdd=cfg.sdd * s,
                      center_x=cfg.center_x * s, center_y=cfg.center_y * s, center_z=cfg.center_z * s)
    np.testing.assert_allclose(sd.dense_matrix(big), sd.dense_matrix(cfg) * s, rtol=1e-12, atol=1e-13)


def test_s9_far_source_reproduces_parallel(sd):
    """Siddon weights jump when a ray moves across a voxel corner, so compare sums over the volume (which are
    continuous in the ray) rather than single weights: the sinogram of a smooth volume."""
    par = tiny(PARALLEL)
    k, j, i = np.meshgrid(np.arange(par.nz), np.arange(par.ny), np.arange(par.nx), indexing="ij")
    x = (1.0 + 0.1 * i + 0.05 * j + 0.2 * k).astype(np.float32)
    yp = sd.project(par, x)
    devs = []
    for far in (1e4, 1e6, 1e8):
        cone = par.replace(geom=CONE, sod=far, sdd=far + 50.0)
        devs.append(np.abs(sd.project(cone, x) - yp).max() / yp.max())
    assert devs[0] < 2e-2 and devs[1] < 2e-4 and devs[2] < 2e-6, devs
    assert devs[0] > 30 * devs[1] > 30 * 30 * devs[2] * 0.5, devs


# ---------------------------------------------------------------- conventions shared with the other projector

def test_siddon_and_footprint_agree_on_smooth_objects(sd, oracle_mod):
    """Both models discretise the same line integrals: on a smooth ellipsoid phantom sampled finely they agree to a
    few percent; the rest is the jagged edge of the voxelised ellipsoid, which thin rays feel more than footprints do
    (a wrong detector shift, row order, volume offset or unit would show up as tens of percent)."""
    cfg = reduced(config(3), 8, nviews=6).replace(shift_u=1.3, shift_v=-0.8, center_x=3.0, center_z=-2.0)
    ells = [Ellipsoid((20.0, -15.0, 10.0), (60.0, 35.0, 45.0), _rot(0.4, 0.3, -0.5), 1.0)]
    x = rasterize(cfg, ells)
    a, b = sd.project(cfg, x), oracle_mod.project(cfg, x)
    assert np.linalg.norm(a - b) / np.linalg.norm(b) < 0.08
