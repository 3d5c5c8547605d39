"""Parity of the Siddon projector pair of the HIP library (through its C ABI) with the Siddon CPU oracle.

Same bar as the separable-footprint pair: relative L2 error <= 1e-5 per sinogram (A) and per volume (A^T) on the same
float32 inputs, adjoint identity to 1e-5.  A thin ray that runs inside a voxel face plane (the central column of an
odd detector at an axis-aligned view of an even grid) is a discontinuity of the model, and which side it falls on
depends on the last bit of sin(pi): the parity cases keep pixel centres off those planes with a fractional detector
shift, and one test checks what is unique there (the total chord) instead.
"""
import numpy as np
import pytest

from synthetic import (CTConfig, config, modular_from, perturbed_poses, reduced, standard_volume, uniform_sinogram,
                       uniform_volume)
from synthetic.configs import CONE, CONE_CURVED, FAN, PARALLEL

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def run_pair(torch, cfg, x, y):
    from paper_2307_05801_amd import Geometry
    print(f"[gpu] siddon {cfg.name} views={cfg.nviews} vol={cfg.vol_shape} det={cfg.nrows}x{cfg.ncols}", flush=True)
    geo = Geometry(cfg, model="siddon")
    print("[gpu]   " + geo.describe(), flush=True)
    ax = geo.project(torch.from_numpy(np.ascontiguousarray(x)).cuda())
    aty = geo.backproject(torch.from_numpy(np.ascontiguousarray(y)).cuda())
    torch.cuda.synchronize()
    out = ax.cpu().numpy(), aty.cpu().numpy()
    geo.close()
    return out


def off_face(cfg):
    return cfg.replace(shift_u=cfg.shift_u + 0.123)


SMALL_CASES = [
    ("c1_full", 1, lambda: off_face(config(1))),
    ("c2_div4_ragged", 2, lambda: off_face(reduced(config(2), 4, nviews=36)).replace(nx=70, ny=61, nz=53, nrows=59, ncols=75)),
    ("c3_div8_ragged", 3, lambda: off_face(reduced(config(3), 8, nviews=40)).replace(nx=67, ny=70, nz=45, nrows=61, ncols=77)),
    ("c3_div4_offsets", 3, lambda: reduced(config(3), 4, nviews=12).replace(
        shift_u=1.3, shift_v=-2.7, center_x=6.0, center_y=-4.5, center_z=3.25, start_deg=7.0)),
    ("c4_div4", 4, lambda: off_face(reduced(config(4), 4, nviews=15))),
    ("c5_div16_shifted", 5, lambda: off_face(reduced(config(5), 16, nviews=36))),
    ("c5_div8_tall_voxels", 5, lambda: off_face(reduced(config(5), 8, nviews=10)).replace(
        voxel_z=1.7, nz=40, pixel_v=2.1, nrows=70)),
    ("fan", 3, lambda: CTConfig("fan_200", FAN, nviews=50, arc_deg=360.0, nrows=1, ncols=150, pixel_v=1.0,
                                pixel_u=2.0, nx=130, ny=120, nz=1, voxel_xy=1.0, voxel_z=1.0, sod=500.0,
                                sdd=900.0, shift_u=0.8, center_x=2.0)),
    ("fine_detector", 3, lambda: off_face(reduced(config(3), 8, nviews=9)).replace(
        pixel_u=1.7, pixel_v=1.9, nrows=300, ncols=280)),
    ("coarse_detector", 3, lambda: off_face(reduced(config(3), 8, nviews=9)).replace(
        pixel_u=37.0, pixel_v=29.0, nrows=14, ncols=12)),
    ("steep_thin_slices", 3, lambda: CTConfig(
        "steep", CONE, nviews=11, arc_deg=360.0, nrows=40, ncols=36, pixel_v=2.9, pixel_u=1.4, nx=30, ny=28, nz=60,
        voxel_xy=1.0, voxel_z=0.21, sod=40.0, sdd=62.0, shift_u=0.3, shift_v=-0.4, center_x=0.7, center_z=-0.3,
        start_deg=3.0)),
    ("curved_c3_div8_ragged", 3, lambda: reduced(config(3), 8, nviews=40).replace(
        geom=CONE_CURVED, nx=67, ny=70, nz=45, nrows=61, ncols=77, shift_u=0.6, shift_v=-1.2, center_x=3.0)),
    ("curved_wide_fan", 3, lambda: CTConfig("curved_wide", CONE_CURVED, nviews=16, arc_deg=360.0, nrows=48, ncols=120,
                                            pixel_v=2.0, pixel_u=1.6, nx=64, ny=60, nz=40, voxel_xy=1.0, voxel_z=1.2,
                                            sod=110.0, sdd=170.0, shift_u=-0.8, shift_v=0.3, center_y=1.5, start_deg=4.0)),
    ("parallel_3d", 3, lambda: CTConfig(
        "par3", PARALLEL, nviews=13, arc_deg=180.0, nrows=66, ncols=90, pixel_v=0.9, pixel_u=0.8, nx=70, ny=66, nz=51,
        voxel_xy=1.0, voxel_z=1.1, sod=0.0, sdd=0.0, shift_u=0.3, shift_v=-0.4, center_y=0.7, center_z=-0.3,
        start_deg=1.0)),
]


@pytest.mark.parametrize("name,number,make", SMALL_CASES, ids=[c[0] for c in SMALL_CASES])
def test_forward_and_adjoint_match_oracle(torch_mod, oracle_mod, name, number, make):
    cfg = make()
    sd = oracle_mod.siddon
    x = standard_volume(number, cfg) if cfg.nz > 1 or number == 1 else uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 50 + number)[0]
    ax, aty = run_pair(torch_mod, cfg, x, y)
    e_a, e_t = rel_l2(ax, sd.project(cfg, x)), rel_l2(aty, sd.backproject(cfg, y))
    print(f"{name}: A {e_a:.2e}  A^T {e_t:.2e}")
    assert e_a <= TOL and e_t <= TOL
    lhs = float((ax.astype(np.float64) * y).sum())
    rhs = float((aty.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


@pytest.mark.parametrize("geom", [PARALLEL, FAN, CONE])
def test_columns_of_A_match_the_dense_oracle_matrix(torch_mod, oracle_mod, geom):
    """Unit volumes through the GPU give columns of A; unit sinograms give rows.  Compared weight by weight."""
    from paper_2307_05801_amd import Geometry
    torch = torch_mod
    cfg = CTConfig("dense", geom, nviews=5, arc_deg=360.0, nrows=5, ncols=8, pixel_v=1.3, pixel_u=0.9,
                   nx=6, ny=5, nz=4, voxel_xy=0.8, voxel_z=1.1, sod=30.0, sdd=47.0, shift_v=0.3, shift_u=-0.7,
                   center_x=0.4, center_y=-0.3, center_z=0.25, start_deg=11.0)
    if geom == FAN:
        cfg = cfg.replace(nrows=1, nz=1, shift_v=0.0, center_z=0.0)
    A = oracle_mod.siddon.dense_matrix(cfg)
    nvox, nray = A.shape[1], A.shape[0]
    print(f"[gpu] siddon dense geom={geom}", flush=True)
    geo = Geometry(cfg, model="siddon")
    cols = geo.project(torch.eye(nvox, device="cuda").reshape(nvox, *cfg.vol_shape)).reshape(nvox, nray).T.cpu().numpy()
    rows = geo.backproject(torch.eye(nray, device="cuda").reshape(nray, *cfg.sino_shape)).reshape(nray, nvox).cpu().numpy()
    geo.close()
    np.testing.assert_allclose(cols, A, rtol=0, atol=2e-6 * A.max())
    np.testing.assert_allclose(rows, A, rtol=0, atol=2e-6 * A.max())


def test_rays_inside_face_planes_keep_the_total_chord(torch_mod, oracle_mod):
    """Odd detector, even grid, views at exact multiples of 90 degrees: the central column's rays run inside the face
    plane between two voxel columns.  Which of the two they are given to is not unique (it hangs on the last bit of
    sin and cos), but every ray's chords still add up to its chord through the volume box, and every other ray
    matches the oracle."""
    cfg = reduced(config(3), 8, nviews=4).replace(ncols=65, nrows=40, angles_override=tuple(np.deg2rad([0.0, 90.0, 180.0, 270.0])))
    sd = oracle_mod.siddon
    ones = np.ones(cfg.vol_shape, np.float32)
    x = uniform_volume(cfg, 5)[0]
    ax1, _ = run_pair(torch_mod, cfg, ones, uniform_sinogram(cfg, 3)[0])
    assert rel_l2(ax1, sd.project(cfg, ones)) <= TOL
    ax, _ = run_pair(torch_mod, cfg, x, uniform_sinogram(cfg, 3)[0])
    ref = sd.project(cfg, x)
    keep = np.ones(cfg.ncols, bool)
    keep[32] = False
    assert rel_l2(ax[:, :, keep], ref[:, :, keep]) <= TOL


def test_long_batch_is_split_over_several_launches(torch_mod):
    """Up to 16 items of a batch go into one launch of the fast kernels (one scratch copy of the volume each); a batch
    of 19 needs two, and every item must come out as if projected alone."""
    from paper_2307_05801_amd import Geometry
    cfg = off_face(reduced(config(4), 8, nviews=6)).replace(batch=19)
    geo = Geometry(cfg, model="siddon")
    assert "A=columns" in geo.describe() and "AT=tiled" in geo.describe(), geo.describe()
    xs = torch_mod.from_numpy(uniform_volume(cfg, 3, batch=19)).cuda()
    ys = torch_mod.from_numpy(uniform_sinogram(cfg, 4, batch=19)).cuda()
    a_all, at_all = geo.project(xs), geo.backproject(ys)
    for b in (0, 7, 15, 16, 18):
        assert torch_mod.equal(a_all[b], geo.project(xs[b].contiguous())), b
        assert torch_mod.equal(at_all[b], geo.backproject(ys[b].contiguous())), b
    geo.close()


def test_batch_autograd_and_overwrite(torch_mod, oracle_mod):
    from paper_2307_05801_amd import Projector
    torch = torch_mod
    cfg = off_face(reduced(config(3), 8, nviews=7)).replace(batch=3)
    sd = oracle_mod.siddon
    print("[gpu] siddon batch/autograd", flush=True)
    P = Projector(cfg, model="siddon")
    xs = np.stack([standard_volume(3, cfg, item=b) for b in range(3)])
    x = torch.from_numpy(xs).cuda().requires_grad_(True)
    y = torch.from_numpy(uniform_sinogram(cfg, 9, batch=3)).cuda()
    ax = P(x)
    loss = 0.5 * ((ax - y) ** 2).sum()
    loss.backward()
    torch.cuda.synchronize()
    for b in range(3):
        ref = sd.project(cfg, xs[b])
        assert rel_l2(ax[b].detach().cpu().numpy(), ref) <= TOL
        resid = (ax[b].detach().cpu().numpy() - y[b].cpu().numpy()).astype(np.float32)
        assert rel_l2(x.grad[b].cpu().numpy(), sd.backproject(cfg, resid)) <= TOL
    # outputs are overwritten, not accumulated into
    out = torch.full((3, *cfg.sino_shape), 7.0, device="cuda")
    P.geometry.project(x.detach(), out=out)
    torch.cuda.synchronize()
    assert torch.equal(out, ax.detach())
    P.geometry.close()


def test_general_kernels_agree_with_fast_kernels(torch_mod, oracle_mod, monkeypatch):
    """The same geometry through the column-wise / tiled kernels and through the general kernels."""
    from paper_2307_05801_amd import Geometry
    torch = torch_mod
    cfg = off_face(reduced(config(3), 4, nviews=10)).replace(center_x=2.5, shift_v=0.4)
    x = torch.from_numpy(standard_volume(3, cfg)).cuda()
    y = torch.from_numpy(uniform_sinogram(cfg, 8)[0]).cuda()
    print("[gpu] siddon fast vs general", flush=True)
    fast = Geometry(cfg, model="siddon")
    assert "A=columns" in fast.describe() and "AT=tiled" in fast.describe(), fast.describe()
    ax_f, aty_f = fast.project(x), fast.backproject(y)
    fast.close()
    monkeypatch.setenv("LEAP_DEBUG", "general=1")
    gen = Geometry(cfg, model="siddon")
    assert "A=general" in gen.describe() and "AT=general" in gen.describe(), gen.describe()
    ax_g, aty_g = gen.project(x), gen.backproject(y)
    torch.cuda.synchronize()
    gen.close()
    assert rel_l2(ax_f.cpu().numpy(), ax_g.cpu().numpy()) <= 2e-6
    assert rel_l2(aty_f.cpu().numpy(), aty_g.cpu().numpy()) <= 2e-6
    assert rel_l2(ax_f.cpu().numpy(), oracle_mod.siddon.project(cfg, x.cpu().numpy())) <= TOL


@pytest.mark.parametrize("seed,curved", [(s, False) for s in range(12)] + [(s, True) for s in (1, 2, 5, 7, 8, 10)])
def test_random_geometries(torch_mod, oracle_mod, seed, curved):
    from random_geometries import random_config
    cfg = random_config(seed)
    cfg = cfg.replace(shift_u=cfg.shift_u + 0.0617)
    if curved:
        if cfg.geom != CONE:
            pytest.skip("parallel-beam draw")
        cfg = cfg.replace(geom=CONE_CURVED)
    sd = oracle_mod.siddon
    x = uniform_volume(cfg, 100 + seed)[0]
    y = uniform_sinogram(cfg, 200 + seed)[0]
    ax, aty = run_pair(torch_mod, cfg, x, y)
    e_a, e_t = rel_l2(ax, sd.project(cfg, x)), rel_l2(aty, sd.backproject(cfg, y))
    print(f"seed {seed}: A {e_a:.2e}  A^T {e_t:.2e}")
    assert e_a <= TOL and e_t <= TOL


@pytest.fixture(scope="module")
def c3_siddon(oracle_mod):
    import torch
    from paper_2307_05801_amd import Geometry
    cfg = config(3)
    print("[gpu] siddon full-size C3: inputs", flush=True)
    x = standard_volume(3, cfg)
    noise = np.random.default_rng([1003, 2]).random(cfg.sino_shape, dtype=np.float32)
    geo = Geometry(cfg, model="siddon")
    desc = geo.describe()
    print("[gpu] siddon full-size C3: " + desc, flush=True)
    ax = geo.project(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    print("[gpu] siddon full-size C3: backproject", flush=True)
    atn = geo.backproject(torch.from_numpy(noise).cuda())
    torch.cuda.synchronize()
    out = dict(cfg=cfg, x=x, noise=noise, ax=ax.cpu().numpy(), atn=atn.cpu().numpy(), describe=desc)
    geo.close()
    return out


def test_c3_full_size_samples_match_oracle(c3_siddon, oracle_mod):
    """512^3 cone-beam, 720 views, in the launch configuration the benchmark times: two whole views, random rays and
    random voxels recomputed one by one by the oracle; adjoint identity over the full arrays."""
    run, sd = c3_siddon, oracle_mod.siddon
    cfg = run["cfg"]
    assert "A=columns" in run["describe"] and "AT=tiled" in run["describe"], run["describe"]
    views = [89, 404]
    ref = sd.project(cfg.with_views(views), run["x"])
    for n, a in enumerate(views):
        assert rel_l2(run["ax"][a], ref[n]) <= TOL
    rng = np.random.default_rng(46)
    rays = rng.integers(0, cfg.nviews * cfg.nrows * cfg.ncols, 600)
    assert rel_l2(run["ax"].ravel()[rays], sd.project_rays(cfg, run["x"], rays)) <= TOL
    n = cfg.nx * cfg.ny * cfg.nz
    vox = np.unique(np.concatenate([rng.integers(0, n, 8000), np.array([0, cfg.nx - 1, n - 1, n - cfg.nx, n // 2 + 255])]))
    got, want = run["atn"].ravel()[vox], sd.backproject_voxels(cfg, run["noise"], vox)
    assert rel_l2(got, want) <= TOL
    assert np.abs(got - want).max() <= 5e-5 * np.abs(want).max()
    lhs = float((run["ax"].astype(np.float64) * run["noise"]).sum())
    rhs = float((run["atn"].astype(np.float64) * run["x"]).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


def test_c3_tilted_modules_full_size_samples_match_oracle(torch_mod, oracle_mod):
    """The 512^3 x 720 scan with every module moved by up to 5 mm and turned by up to 0.05 rad about each of its axes
    (what `bench.py --tilted-modules 0.05` times), on the per-lane slab kernel and the tiled kernel with per-sample
    slopes: two whole views, random rays and random voxels recomputed by the oracle; adjoint identity."""
    import torch
    from paper_2307_05801_amd import Geometry
    cfg = perturbed_poses(config(3), 3, shift_mm=5.0, tilt_rad=0.05)
    sd = oracle_mod.siddon
    print("[gpu] tilted siddon full-size C3: inputs", flush=True)
    x = standard_volume(3, cfg)
    noise = np.random.default_rng([1003, 7]).random(cfg.sino_shape, dtype=np.float32)
    geo = Geometry(cfg, model="siddon")
    desc = geo.describe()
    print("[gpu] tilted siddon full-size C3: " + desc, flush=True)
    assert "A=columns" in desc and "AT=tiled" in desc and "tilted" in desc, desc
    ax = geo.project(torch.from_numpy(x).cuda()).cpu().numpy()
    print("[gpu] tilted siddon full-size C3: backproject", flush=True)
    atn = geo.backproject(torch.from_numpy(noise).cuda()).cpu().numpy()
    geo.close()
    views = [89, 404]
    ref = sd.project(cfg.with_views(views), x)
    for n, a in enumerate(views):
        assert rel_l2(ax[a], ref[n]) <= TOL
    rng = np.random.default_rng(47)
    rays = rng.integers(0, cfg.nviews * cfg.nrows * cfg.ncols, 600)
    assert rel_l2(ax.ravel()[rays], sd.project_rays(cfg, x, rays)) <= TOL
    n = cfg.nx * cfg.ny * cfg.nz
    vox = np.unique(np.concatenate([rng.integers(0, n, 4000), np.array([0, cfg.nx - 1, n - 1, n - cfg.nx, n // 2 + 255])]))
    got, want = atn.ravel()[vox], sd.backproject_voxels(cfg, noise, vox)
    assert rel_l2(got, want) <= TOL
    assert np.abs(got - want).max() <= 5e-5 * np.abs(want).max()
    lhs = float((ax.astype(np.float64) * noise).sum())
    rhs = float((atn.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


@pytest.mark.parametrize("seed", range(8))
def test_random_tilted_scans(torch_mod, oracle_mod, seed):
    """Random tilts, shifts, voxel aspect ratios and sizes on the per-lane kernels (window shapes from 32 x 21 to 64 x 48)."""
    from paper_2307_05801_amd import Geometry
    from random_geometries import random_tilted_scan
    cfg = random_tilted_scan(seed)
    sd = oracle_mod.siddon
    x, y = uniform_volume(cfg, 5)[0], uniform_sinogram(cfg, 6)[0]
    geo = Geometry(cfg, model="siddon")
    desc = geo.describe()
    print(f"[gpu] random tilted scan {seed}: {desc}", flush=True)
    assert "A=columns" in desc and "AT=tiled" in desc, desc
    ax = geo.project(torch_mod.from_numpy(x).cuda()).cpu().numpy()
    aty = geo.backproject(torch_mod.from_numpy(y).cuda()).cpu().numpy()
    geo.close()
    ref_a, ref_t = sd.project(cfg, x), sd.backproject(cfg, y)
    e_a, e_t = rel_l2(ax, ref_a), rel_l2(aty, ref_t)
    print(f"seed {seed}: A {e_a:.2e}  A^T {e_t:.2e}")
    assert e_a <= TOL and e_t <= TOL
    assert np.abs(ax - ref_a).max() <= 2e-5 * np.abs(ref_a).max() and np.abs(aty - ref_t).max() <= 2e-5 * np.abs(ref_t).max()


MODULAR_CASES = [
    ("cone_as_modular", lambda: modular_from(reduced(config(3), 8, nviews=12).replace(shift_u=0.123))),
    ("tilted_modules", lambda: perturbed_poses(reduced(config(3), 8, nviews=16).replace(nx=67, ny=70, nz=45, nrows=61, ncols=77),
                                               3, shift_mm=20.0, tilt_rad=0.25)),
    ("wobbly_orbit", lambda: perturbed_poses(reduced(config(5), 16, nviews=24), 11, shift_mm=8.0, tilt_rad=0.05)),
    ("looking_down", lambda: CTConfig("down", 4, nviews=2, arc_deg=360.0, nrows=40, ncols=48, pixel_v=1.5, pixel_u=1.4,
                                      nx=36, ny=32, nz=24, voxel_xy=1.0, voxel_z=1.3, shift_u=0.2, shift_v=-0.3,
                                      poses=((0.3, -0.2, 60.0, 0.0, 0.0, -45.0, 1.0, 0.0, 0.0, 0.0, 1.0, 0.0),
                                             (9.0, 3.0, 58.0, -3.0, 1.5, -42.0, 0.8, 0.6, 0.0, -0.6, 0.8, 0.0)))),
]


UPRIGHT_MODULAR_CASES = [
    ("cone_as_modular", lambda: modular_from(reduced(config(3), 8, nviews=12).replace(shift_u=0.123))),
    ("shifted_upright_modules", lambda: perturbed_poses(
        reduced(config(3), 8, nviews=16).replace(nx=67, ny=70, nz=45, nrows=61, ncols=77), 3, shift_mm=25.0, tilt_rad=0.3,
        upright=True)),
    ("wobbly_upright_orbit", lambda: perturbed_poses(reduced(config(5), 16, nviews=24), 11, shift_mm=10.0, tilt_rad=0.1,
                                                     upright=True)),
]


@pytest.mark.parametrize("name,make", UPRIGHT_MODULAR_CASES, ids=[c[0] for c in UPRIGHT_MODULAR_CASES])
def test_upright_modules_take_the_fast_kernels(torch_mod, oracle_mod, monkeypatch, name, make):
    """Upright modules run the column / tiled Siddon kernels on per-view parameter blocks; they must agree with the
    oracle and with the general modular kernels."""
    from paper_2307_05801_amd import Geometry
    cfg = make()
    sd = oracle_mod.siddon
    x = standard_volume(3, cfg)
    y = uniform_sinogram(cfg, 6)[0]
    geo = Geometry(cfg, model="siddon")
    desc = geo.describe()
    print(f"[gpu] {name}: {desc}", flush=True)
    assert "A=columns" in desc and "AT=tiled" in desc and "upright" in desc, desc
    ax = geo.project(torch_mod.from_numpy(x).cuda()).cpu().numpy()
    aty = geo.backproject(torch_mod.from_numpy(y).cuda()).cpu().numpy()
    geo.close()
    monkeypatch.setenv("LEAP_DEBUG", "general=1")
    gen = Geometry(cfg, model="siddon")
    assert "A=general" in gen.describe() and "AT=general" in gen.describe(), gen.describe()
    ax_g = gen.project(torch_mod.from_numpy(x).cuda()).cpu().numpy()
    aty_g = gen.backproject(torch_mod.from_numpy(y).cuda()).cpu().numpy()
    gen.close()
    e_a, e_t = rel_l2(ax, sd.project(cfg, x)), rel_l2(aty, sd.backproject(cfg, y))
    print(f"{name}: A {e_a:.2e}  A^T {e_t:.2e}  vs general {rel_l2(ax, ax_g):.2e} {rel_l2(aty, aty_g):.2e}", flush=True)
    assert e_a <= TOL and e_t <= TOL
    assert rel_l2(ax, ax_g) <= TOL and rel_l2(aty, aty_g) <= TOL
    lhs = float((ax.astype(np.float64) * y).sum())
    rhs = float((aty.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


TILTED_FAST_CASES = [
    ("tilted_modules", MODULAR_CASES[1][1]),
    ("wobbly_orbit", MODULAR_CASES[2][1]),
    ("rolled_modules_tall_voxels", lambda: perturbed_poses(
        reduced(config(3), 8, nviews=14).replace(nx=70, ny=61, nz=40, voxel_z=reduced(config(3), 8).voxel_z * 1.6, nrows=90,
                                                 ncols=83, shift_u=0.4, center_y=7.0), 21, shift_mm=12.0, tilt_rad=0.35)),
]


@pytest.mark.parametrize("name,make", TILTED_FAST_CASES, ids=[c[0] for c in TILTED_FAST_CASES])
def test_tilted_modules_take_the_fast_kernels(torch_mod, oracle_mod, monkeypatch, name, make):
    """Tilted modules whose rays stay flat run the per-lane slab kernel (A) and the tiled kernel with per-pixel slopes
    (A^T); they must agree with the oracle and with the general modular kernels."""
    from paper_2307_05801_amd import Geometry
    cfg = make()
    sd = oracle_mod.siddon
    x = uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 6)[0]
    geo = Geometry(cfg, model="siddon")
    desc = geo.describe()
    print(f"[gpu] {name}: {desc}", flush=True)
    assert "A=columns" in desc and "AT=tiled" in desc and "tilted" in desc, desc
    ax = geo.project(torch_mod.from_numpy(x).cuda()).cpu().numpy()
    aty = geo.backproject(torch_mod.from_numpy(y).cuda()).cpu().numpy()
    aty_again = geo.backproject(torch_mod.from_numpy(y).cuda()).cpu().numpy()
    geo.close()
    monkeypatch.setenv("LEAP_DEBUG", "general=1")
    gen = Geometry(cfg, model="siddon")
    assert "A=general" in gen.describe() and "AT=general" in gen.describe(), gen.describe()
    ax_g = gen.project(torch_mod.from_numpy(x).cuda()).cpu().numpy()
    aty_g = gen.backproject(torch_mod.from_numpy(y).cuda()).cpu().numpy()
    gen.close()
    ref_a, ref_t = sd.project(cfg, x), sd.backproject(cfg, y)
    e_a, e_t = rel_l2(ax, ref_a), rel_l2(aty, ref_t)
    print(f"{name}: A {e_a:.2e}  A^T {e_t:.2e}  vs general {rel_l2(ax, ax_g):.2e} {rel_l2(aty, aty_g):.2e}", flush=True)
    assert e_a <= TOL and e_t <= TOL
    assert np.abs(ax - ref_a).max() <= 2e-5 * np.abs(ref_a).max() and np.abs(aty - ref_t).max() <= 2e-5 * np.abs(ref_t).max()
    assert rel_l2(ax, ax_g) <= TOL and rel_l2(aty, aty_g) <= TOL
    assert np.array_equal(aty, aty_again)                     # no atomics: bitwise reproducible
    lhs = float((ax.astype(np.float64) * y).sum())
    rhs = float((aty.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


@pytest.mark.parametrize("name,make", MODULAR_CASES, ids=[c[0] for c in MODULAR_CASES])
def test_modular_geometry_matches_oracle(torch_mod, oracle_mod, name, make):
    """Per-view source position, detector centre and detector orientation (Siddon model)."""
    cfg = make()
    sd = oracle_mod.siddon
    x = uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 6)[0]
    ax, aty = run_pair(torch_mod, cfg, x, y)
    e_a, e_t = rel_l2(ax, sd.project(cfg, x)), rel_l2(aty, sd.backproject(cfg, y))
    print(f"{name}: A {e_a:.2e}  A^T {e_t:.2e}")
    assert e_a <= TOL and e_t <= TOL
    lhs = float((ax.astype(np.float64) * y).sum())
    rhs = float((aty.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


