"""Parity of the HIP library (through its C ABI) with the CPU oracle on the same seeded inputs.

Tolerance (stated by the build's target): relative L2 error <= 1e-5 per sinogram (A) and per volume (A^T),
per batch item, both sides fed the same float32 arrays and compared in double; the adjoint identity
<Ax,y> = <x,A^T y> to <= 1e-5 relative.  Every case prints its name before it touches the GPU.
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


def gpu_project(torch, cfg, x):
    from paper_2307_05801_amd import Geometry
    print(f"[gpu] project {cfg.name} views={cfg.nviews} vol={cfg.vol_shape} det={cfg.nrows}x{cfg.ncols}", flush=True)
    geo = Geometry(cfg)
    out = geo.project(torch.from_numpy(np.ascontiguousarray(x)).cuda())
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    geo.close()
    return res


def gpu_backproject(torch, cfg, y):
    from paper_2307_05801_amd import Geometry
    print(f"[gpu] backproject {cfg.name} views={cfg.nviews} vol={cfg.vol_shape} det={cfg.nrows}x{cfg.ncols}", flush=True)
    geo = Geometry(cfg)
    out = geo.backproject(torch.from_numpy(np.ascontiguousarray(y)).cuda())
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    geo.close()
    return res


def ragged(cfg, **kw):
    """Sizes that are no multiple of any tile edge."""
    return cfg.replace(**kw)


SMALL_CASES = [
    ("c1_full", 1, lambda: config(1)),
    ("c2_div4_ragged", 2, lambda: ragged(reduced(config(2), 4, nviews=36), nx=70, ny=61, nz=53, nrows=59, ncols=75)),
    ("c3_div8_ragged", 3, lambda: ragged(reduced(config(3), 8, nviews=40), nx=67, ny=70, nz=45, nrows=61, ncols=77)),
    ("c3_div4_offsets", 3, lambda: reduced(config(3), 4, nviews=12).replace(
        shift_u=1.3, shift_v=-2.7, center_x=6.0, center_y=-4.5, center_z=3.25, start_deg=7.0)),
    ("c4_div4", 4, lambda: reduced(config(4), 4, nviews=15)),
    ("c5_div16_shifted", 5, lambda: reduced(config(5), 16, nviews=36)),
    ("c5_div8_tall_voxels", 5, lambda: reduced(config(5), 8, nviews=10).replace(voxel_z=1.7, nz=40, pixel_v=2.1, nrows=70)),
    # voxels 1.6 to 2.4 rows tall: the four-row instance of the tiled back projection (general gather)
    ("c5_div8_taller_voxels", 5, lambda: reduced(config(5), 8, nviews=10).replace(voxel_z=2.6, nz=28, pixel_v=2.1, nrows=70)),
    ("fan", 3, lambda: CTConfig("fan_200", FAN, nviews=50, arc_deg=360.0, nrows=1, ncols=150, pixel_v=1.0,
                                pixel_u=2.0, nx=130, ny=120, nz=1, voxel_xy=1.0, voxel_z=1.0, sod=500.0,
                                sdd=900.0, shift_u=0.8, center_x=2.0)),
    ("fine_detector", 3, lambda: reduced(config(3), 8, nviews=9).replace(pixel_u=1.7, pixel_v=1.9, nrows=300, ncols=280)),
    ("coarse_detector", 3, lambda: reduced(config(3), 8, nviews=9).replace(pixel_u=37.0, pixel_v=29.0, nrows=14, ncols=12)),
    ("curved_c3_div8_ragged", 3, lambda: ragged(reduced(config(3), 8, nviews=40), geom=CONE_CURVED, nx=67, ny=70, nz=45,
                                                nrows=61, ncols=77, shift_u=0.6, shift_v=-1.2, center_x=3.0)),
    ("curved_c3_div4", 3, lambda: reduced(config(3), 4, nviews=12).replace(geom=CONE_CURVED, start_deg=7.0)),
    ("curved_wide_fan", 3, lambda: CTConfig("curved_wide", CONE_CURVED, nviews=16, arc_deg=360.0, nrows=48, ncols=120,
                                            pixel_v=2.0, pixel_u=1.6, nx=64, ny=60, nz=40, voxel_xy=1.0, voxel_z=1.2,
                                            sod=110.0, sdd=170.0, shift_u=-0.8, shift_v=0.3, center_y=1.5, start_deg=4.0)),
    ("curved_close_source", 3, lambda: CTConfig("curved_close", CONE_CURVED, nviews=9, arc_deg=360.0, nrows=40, ncols=200,
                                                pixel_v=2.0, pixel_u=1.0, nx=48, ny=48, nz=24, voxel_xy=1.0, voxel_z=1.5,
                                                sod=45.0, sdd=90.0, shift_u=0.4, shift_v=0.0, start_deg=2.0)),
]


@pytest.mark.parametrize("name,number,make", SMALL_CASES, ids=[c[0] for c in SMALL_CASES])
def test_forward_and_adjoint_match_oracle(torch_mod, oracle_mod, name, number, make):
    cfg = make()
    x = standard_volume(number, cfg) if cfg.nz > 1 or number == 1 else uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 100 + number)[0]
    ax = gpu_project(torch_mod, cfg, x)
    aty = gpu_backproject(torch_mod, cfg, y)
    ax_ref = oracle_mod.project(cfg, x)
    aty_ref = oracle_mod.backproject(cfg, y)
    e_a, e_at = rel_l2(ax, ax_ref), rel_l2(aty, aty_ref)
    print(f"{name}: rel-L2 A {e_a:.2e}  A^T {e_at:.2e}")
    assert e_a <= TOL and e_at <= TOL
    # no single element far off either (rounding errors of float32 sums stay well inside this bound)
    assert np.abs(ax - ax_ref).max() <= 2e-5 * np.abs(ax_ref).max()
    assert np.abs(aty - aty_ref).max() <= 2e-5 * np.abs(aty_ref).max()
    for a in range(cfg.nviews):                       # per view as well: no view may hide behind the others
        assert rel_l2(ax[a], ax_ref[a]) <= TOL
    lhs = float((ax.astype(np.float64) * y).sum())
    rhs = float((aty.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)
    # A^T of the projection itself (the benchmark's second operand)
    if cfg.nviews * cfg.nx * cfg.ny * cfg.nz < 3e7:
        ax32 = ax_ref.astype(np.float32)
        assert rel_l2(gpu_backproject(torch_mod, cfg, ax32), oracle_mod.backproject(cfg, ax32)) <= TOL


def test_voxels_around_one_row_tall_in_64_voxel_chunks(torch_mod, oracle_mod):
    """A scan whose voxels are 0.8 to 1.3 detector rows tall, on a volume tall enough for 64 voxels per thread: the tiled
    back projection takes its three-row instance under the tall window, and the line where a voxel is exactly one row
    tall crosses the tiles, so that lanes of one wavefront run different row schemes in the same view."""
    from paper_2307_05801_amd import Geometry
    cfg = CTConfig("around_one_row", CONE, nviews=12, arc_deg=360.0, nrows=210, ncols=99, pixel_v=1.0, pixel_u=2.0,
                   nx=64, ny=61, nz=160, voxel_xy=1.0, voxel_z=0.65, sod=200.0, sdd=300.0, shift_u=0.4, shift_v=-0.7,
                   center_x=1.5, start_deg=3.0)
    geo = Geometry(cfg)
    desc = geo.describe()
    geo.close()
    print(f"[gpu] {cfg.name}: {desc}", flush=True)
    assert "nv=3,zc=64" in desc, desc
    x = standard_volume(3, cfg)
    y = uniform_sinogram(cfg, 321)[0]
    ax = gpu_project(torch_mod, cfg, x)
    aty = gpu_backproject(torch_mod, cfg, y)
    ax_ref = oracle_mod.project(cfg, x)
    aty_ref = oracle_mod.backproject(cfg, y)
    e_a, e_at = rel_l2(ax, ax_ref), rel_l2(aty, aty_ref)
    print(f"{cfg.name}: rel-L2 A {e_a:.2e}  A^T {e_at:.2e}")
    assert e_a <= TOL and e_at <= TOL
    assert np.abs(aty - aty_ref).max() <= 2e-5 * np.abs(aty_ref).max()
    lhs = float((ax.astype(np.float64) * y).sum())
    rhs = float((aty.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


@pytest.mark.parametrize("cw", ["1", "2", "4"])
@pytest.mark.parametrize("name,number,make", [c for c in SMALL_CASES if c[0] in ("c2_div4_ragged", "c3_div8_ragged")],
                         ids=["c2_div4_ragged", "c3_div8_ragged"])
def test_forward_bundle_widths_on_ragged_detectors(torch_mod, oracle_mod, monkeypatch, name, number, make, cw):
    """Every bundle width of the column-wise forward kernel on detectors whose column count is odd: the last bundle is
    partial and the 8- and 16-byte stores of whole bundles are only 4-byte aligned."""
    from paper_2307_05801_amd import Geometry
    cfg = make()
    assert cfg.ncols % 2 == 1
    x = standard_volume(number, cfg)
    monkeypatch.setenv("LEAP_DEBUG", "cw=" + cw)
    geo = Geometry(cfg)
    desc = geo.describe()
    print(f"[gpu] {name} cw={cw}: {desc}", flush=True)
    assert f"cw={cw}" in desc and "A=columns" in desc, desc
    ax = geo.project(torch_mod.from_numpy(x).cuda()).cpu().numpy()
    geo.close()
    assert rel_l2(ax, oracle_mod.project(cfg, x)) <= TOL


@pytest.mark.parametrize("geom", [PARALLEL, FAN, CONE])
def test_columns_of_A_match_the_dense_oracle_matrix(torch_mod, oracle_mod, geom):
    """Every entry of A and of A^T on a tiny grid with shifts and centre offsets, by unit vectors in a batch."""
    from paper_2307_05801_amd import Geometry
    base = dict(name="tiny", geom=geom, nviews=7, arc_deg=360.0, nrows=6, ncols=9, pixel_v=1.3, pixel_u=0.9,
                nx=5, ny=4, nz=3, voxel_xy=0.8, voxel_z=1.1, sod=30.0, sdd=47.0, shift_v=0.3, shift_u=-0.7,
                center_x=0.4, center_y=-0.3, center_z=0.25, start_deg=11.0)
    if geom == FAN:
        base.update(nrows=1, nz=1, shift_v=0.0, center_z=0.0)
    cfg = CTConfig(**base)
    A = oracle_mod.dense_matrix(cfg)
    m, n = A.shape
    print(f"[gpu] dense columns geom={geom}", flush=True)
    geo = Geometry(cfg)
    eye_v = torch_mod.eye(n, dtype=torch_mod.float32, device="cuda").reshape((n,) + cfg.vol_shape)
    cols = geo.project(eye_v).reshape(n, m).T.cpu().numpy()            # column j = A e_j
    eye_s = torch_mod.eye(m, dtype=torch_mod.float32, device="cuda").reshape((m,) + cfg.sino_shape)
    rows = geo.backproject(eye_s).reshape(m, n).cpu().numpy()          # row i = A^T e_i
    geo.close()
    scale = A.max()
    assert np.abs(cols - A).max() <= 2e-6 * scale
    assert np.abs(rows - A).max() <= 2e-6 * scale
    assert ((cols > 0) == (A > 1e-7 * scale)).mean() > 0.999           # same support up to rounding-size entries


def test_axis_aligned_and_diagonal_views(torch_mod, oracle_mod):
    """Degenerate trapezoids: rectangles at multiples of 90 degrees, triangles at 45."""
    angles = tuple(np.deg2rad([0.0, 45.0, 90.0, 135.0, 180.0, 225.0, 270.0, 315.0, 359.999]))
    for base in (reduced(config(2), 8), reduced(config(3), 8)):
        cfg = base.replace(nviews=len(angles), angles_override=angles, shift_u=0.5)
        x = uniform_volume(cfg, 9)[0]
        y = uniform_sinogram(cfg, 10)[0]
        assert rel_l2(gpu_project(torch_mod, cfg, x), oracle_mod.project(cfg, x)) <= TOL
        assert rel_l2(gpu_backproject(torch_mod, cfg, y), oracle_mod.backproject(cfg, y)) <= TOL


def test_few_noisy_views_backprojection_keeps_tolerance(torch_mod, oracle_mod):
    """One and two views of white noise: nothing averages the coordinate rounding away."""
    for number, factor in ((3, 2), (5, 4)):
        full = reduced(config(number), factor)
        cfg = full.with_views([3]).replace(nz=24, nrows=40)
        y = uniform_sinogram(cfg, 77)[0]
        assert rel_l2(gpu_backproject(torch_mod, cfg, y), oracle_mod.backproject(cfg, y)) <= TOL


def test_truncated_and_missing_detector(torch_mod, oracle_mod):
    base = reduced(config(3), 8, nviews=8)
    small = base.replace(nrows=20, ncols=24)                     # detector smaller than the shadow
    x = uniform_volume(small, 3)[0]
    y = uniform_sinogram(small, 4)[0]
    assert rel_l2(gpu_project(torch_mod, small, x), oracle_mod.project(small, x)) <= TOL
    assert rel_l2(gpu_backproject(torch_mod, small, y), oracle_mod.backproject(small, y)) <= TOL
    away = base.replace(shift_u=500.0)                           # detector beside the shadow: all rays miss
    x = uniform_volume(away, 3)[0]
    y = uniform_sinogram(away, 4)[0]
    assert np.all(gpu_project(torch_mod, away, x) == 0.0)
    assert np.all(gpu_backproject(torch_mod, away, y) == 0.0)
    up = base.replace(shift_v=400.0)
    assert np.all(gpu_project(torch_mod, up, uniform_volume(up, 3)[0]) == 0.0)
    assert np.all(gpu_backproject(torch_mod, up, uniform_sinogram(up, 4)[0]) == 0.0)


def test_single_voxel_single_pixel_single_view(torch_mod, oracle_mod):
    cfg = CTConfig("one", CONE, nviews=1, arc_deg=360.0, nrows=1, ncols=1, pixel_v=1.0, pixel_u=1.0,
                   nx=1, ny=1, nz=1, voxel_xy=1.0, voxel_z=1.0, sod=1000.0, sdd=1500.0)
    x = np.full(cfg.vol_shape, 2.0, dtype=np.float32)
    got = gpu_project(torch_mod, cfg, x)
    assert abs(float(got[0, 0, 0]) - 2.0) <= 2e-6        # hand-worked: centre pixel weight is exactly 1
    y = np.full(cfg.sino_shape, 3.0, dtype=np.float32)
    assert abs(float(gpu_backproject(torch_mod, cfg, y)[0, 0, 0]) - 3.0) <= 3e-6


def test_zero_in_zero_out_and_overwrite(torch_mod):
    from paper_2307_05801_amd import Geometry
    cfg = reduced(config(3), 8, nviews=6)
    geo = Geometry(cfg)
    out = torch_mod.full(cfg.sino_shape, 7.0, dtype=torch_mod.float32, device="cuda")
    geo.project(torch_mod.zeros(cfg.vol_shape, dtype=torch_mod.float32, device="cuda"), out=out)
    assert float(out.abs().max()) == 0.0                     # outputs are overwritten, not accumulated
    outv = torch_mod.full(cfg.vol_shape, 7.0, dtype=torch_mod.float32, device="cuda")
    geo.backproject(torch_mod.zeros(cfg.sino_shape, dtype=torch_mod.float32, device="cuda"), out=outv)
    assert float(outv.abs().max()) == 0.0
    geo.close()


def test_batch_equals_item_by_item_and_is_reproducible(torch_mod):
    from paper_2307_05801_amd import Geometry
    cfg = reduced(config(4), 4, nviews=10, batch=3)
    geo = Geometry(cfg)
    xs = torch_mod.from_numpy(uniform_volume(cfg, 1, batch=3)).cuda()
    ys = torch_mod.from_numpy(uniform_sinogram(cfg, 2, batch=3)).cuda()
    a_all, at_all = geo.project(xs), geo.backproject(ys)
    for b in range(3):
        assert torch_mod.equal(a_all[b], geo.project(xs[b].contiguous()))
        assert torch_mod.equal(at_all[b], geo.backproject(ys[b].contiguous()))
    assert torch_mod.equal(a_all, geo.project(xs)) and torch_mod.equal(at_all, geo.backproject(ys))
    geo.close()


def test_long_batch_is_split_over_several_launches(torch_mod):
    """The fast kernels take up to 16 items of a batch per launch (one scratch copy of the volume each); a batch of 19
    needs two launches, and every item must come out as if projected alone."""
    from paper_2307_05801_amd import Geometry
    cfg = reduced(config(4), 8, nviews=6, batch=19)
    geo = Geometry(cfg)
    assert "A=columns" in geo.describe() and "AT=tiled" in geo.describe(), geo.describe()
    xs = torch_mod.from_numpy(uniform_volume(cfg, 3, batch=19)).cuda()
    ys = torch_mod.from_numpy(uniform_sinogram(cfg, 4, batch=19)).cuda()
    a_all, at_all = geo.project(xs), geo.backproject(ys)
    for b in (0, 7, 15, 16, 18):
        assert torch_mod.equal(a_all[b], geo.project(xs[b].contiguous())), b
        assert torch_mod.equal(at_all[b], geo.backproject(ys[b].contiguous())), b
    geo.close()


def test_autograd_gradient_is_the_matched_transpose(torch_mod, oracle_mod):
    """d/dx 1/2 |Ax - y|^2 = A^T (Ax - y) (the paper's least-squares example), and A^T differentiates to A."""
    from paper_2307_05801_amd import Projector
    cfg = reduced(config(4), 8, nviews=8)
    proj = Projector(cfg)
    x = uniform_volume(cfg, 31, batch=2)
    y = uniform_sinogram(cfg, 32, batch=2)
    xt = torch_mod.from_numpy(x).cuda().requires_grad_(True)
    yt = torch_mod.from_numpy(y).cuda()
    loss = 0.5 * ((proj(xt) - yt) ** 2).sum()
    loss.backward()
    for b in range(2):
        resid = (oracle_mod.project(cfg, x[b]) - y[b]).astype(np.float32)
        assert rel_l2(xt.grad[b].cpu().numpy(), oracle_mod.backproject(cfg, resid)) <= 2 * TOL
    # directional derivative of the loss along a random direction
    d = torch_mod.from_numpy(uniform_volume(cfg, 33, batch=2)).cuda() - 0.5
    eps = 1e-2
    with torch_mod.no_grad():
        lp = 0.5 * ((proj(xt + eps * d) - yt).double() ** 2).sum()
        lm = 0.5 * ((proj(xt - eps * d) - yt).double() ** 2).sum()
    fd = float((lp - lm) / (2 * eps))
    an = float((xt.grad.double() * d.double()).sum())
    assert abs(fd - an) <= 1e-4 * abs(an)
    st = yt.clone().requires_grad_(True)
    (proj.backproject(st) * xt.detach()).sum().backward()
    with torch_mod.no_grad():
        assert rel_l2(st.grad.cpu().numpy(), proj(xt.detach()).cpu().numpy()) <= 1e-6


def test_streams_are_honoured(torch_mod):
    from paper_2307_05801_amd import Geometry
    cfg = reduced(config(3), 8, nviews=12)
    geo = Geometry(cfg)
    x = torch_mod.from_numpy(uniform_volume(cfg, 1)[0]).cuda()
    ref = geo.project(x)
    torch_mod.cuda.synchronize()
    s = torch_mod.cuda.Stream()
    with torch_mod.cuda.stream(s):
        got = geo.project(x)
    s.synchronize()
    assert torch_mod.equal(ref, got)
    geo.close()


def test_two_streams_share_one_handle(torch_mod):
    """Calls on one handle share its forward scratch; the library orders them on the device.  Two streams project two
    different volumes through one handle back to back, without any synchronisation in between, several times over:
    every result equals the one a lone call gives."""
    from paper_2307_05801_amd import Geometry
    torch = torch_mod
    cfg = reduced(config(3), 4, nviews=90)
    geo = Geometry(cfg)
    assert "A=columns" in geo.describe()
    x1 = torch.from_numpy(uniform_volume(cfg, 1)[0]).cuda()
    x2 = torch.from_numpy(uniform_volume(cfg, 2)[0]).cuda()
    ref1, ref2 = geo.project(x1), geo.project(x2)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for _ in range(4):
        with torch.cuda.stream(s1):
            y1 = geo.project(x1)
        with torch.cuda.stream(s2):
            y2 = geo.project(x2)
        outs.append((y1, y2))
    s1.synchronize(); s2.synchronize()
    for y1, y2 in outs:
        assert torch.equal(y1, ref1) and torch.equal(y2, ref2)
    geo.close()


def test_training_step_of_case_4(torch_mod, oracle_mod):
    """Batch of volumes: y = A x, residual against a photon-noise measurement, gradient g = A^T r."""
    from paper_2307_05801_amd import Geometry
    from synthetic import measured_sinogram, perturbed_volume
    cfg = reduced(config(4), 4, nviews=15, batch=3)
    truth = [standard_volume(4, cfg, item=b) for b in range(cfg.batch)]
    x = np.stack([perturbed_volume(t, 1004 + b) for b, t in enumerate(truth)])
    y_meas = np.stack([measured_sinogram(oracle_mod.project(cfg, t), 1004 + b) for b, t in enumerate(truth)])
    print(f"[gpu] training step {cfg.name} batch={cfg.batch}", flush=True)
    geo = Geometry(cfg)
    xt, yt = torch_mod.from_numpy(x).cuda(), torch_mod.from_numpy(y_meas).cuda()
    r = geo.project(xt) - yt
    g = geo.backproject(r)
    torch_mod.cuda.synchronize()
    r_np, g_np = r.cpu().numpy(), g.cpu().numpy()
    geo.close()
    for b in range(cfg.batch):
        ax_ref = oracle_mod.project(cfg, x[b])
        # the residual is a small difference of large numbers: judge A by the projection, A^T by the gradient
        assert rel_l2(r_np[b] + y_meas[b], ax_ref) <= TOL
        assert rel_l2(g_np[b], oracle_mod.backproject(cfg, r_np[b])) <= TOL


def test_general_kernels_agree_with_fast_kernels(torch_mod, oracle_mod, monkeypatch):
    """The fallback loop nests and the tiled kernels evaluate the same weights."""
    from paper_2307_05801_amd import Geometry
    cfg = reduced(config(3), 8, nviews=20)
    x = torch_mod.from_numpy(uniform_volume(cfg, 8)[0]).cuda()
    y = torch_mod.from_numpy(uniform_sinogram(cfg, 9)[0]).cuda()
    fast = Geometry(cfg)
    assert "A=columns" in fast.describe() and "AT=tiled" in fast.describe()
    a_fast, at_fast = fast.project(x).cpu().numpy(), fast.backproject(y).cpu().numpy()
    fast.close()
    monkeypatch.setenv("LEAP_DEBUG", "general=1")
    slow = Geometry(cfg)
    assert "A=general" in slow.describe() and "AT=general" in slow.describe()
    a_slow, at_slow = slow.project(x).cpu().numpy(), slow.backproject(y).cpu().numpy()
    slow.close()
    assert rel_l2(a_fast, a_slow) <= 2e-6 and rel_l2(at_fast, at_slow) <= 2e-6
    assert rel_l2(a_slow, oracle_mod.project(cfg, x.cpu().numpy())) <= TOL


@pytest.mark.parametrize("seed", range(16))
def test_random_geometries(torch_mod, oracle_mod, seed):
    _random_case(torch_mod, oracle_mod, seed, curved=False)


@pytest.mark.parametrize("seed", [1, 2, 5, 7, 8, 10, 11, 13])
def test_random_geometries_curved_detector(torch_mod, oracle_mod, seed):
    _random_case(torch_mod, oracle_mod, seed, curved=True)


def _random_case(torch_mod, oracle_mod, seed, curved):
    """Random scanners (cone and parallel, shifted and truncated detectors, anisotropic voxels, irregular angles)."""
    from random_geometries import random_config
    cfg = random_config(seed)
    if curved:
        if cfg.geom != CONE:
            pytest.skip("parallel-beam draw")
        cfg = cfg.replace(geom=CONE_CURVED)
    x = uniform_volume(cfg, seed)[0]
    y = uniform_sinogram(cfg, seed)[0]
    ax = gpu_project(torch_mod, cfg, x)
    aty = gpu_backproject(torch_mod, cfg, y)
    assert rel_l2(ax, oracle_mod.project(cfg, x)) <= TOL
    assert rel_l2(aty, oracle_mod.backproject(cfg, y)) <= TOL


UPRIGHT_MODULAR_CASES = [
    ("cone_as_modular", lambda: modular_from(reduced(config(3), 8, nviews=12).replace(shift_u=0.3, shift_v=-0.4))),
    ("shifted_upright_modules", lambda: perturbed_poses(
        reduced(config(3), 8, nviews=16).replace(nx=67, ny=70, nz=45, nrows=61, ncols=77), 3, shift_mm=25.0, tilt_rad=0.3,
        upright=True)),
    ("wobbly_orbit", lambda: perturbed_poses(reduced(config(5), 16, nviews=24), 11, shift_mm=10.0, tilt_rad=0.1, upright=True)),
]


@pytest.mark.parametrize("name,make", UPRIGHT_MODULAR_CASES, ids=[c[0] for c in UPRIGHT_MODULAR_CASES])
def test_modular_geometry_with_upright_modules(torch_mod, oracle_mod, name, make):
    """Per-view source and detector positions, detector rotated about the vertical: footprints in each view's frame."""
    cfg = make()
    x = uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 6)[0]
    ax = gpu_project(torch_mod, cfg, x)
    aty = gpu_backproject(torch_mod, cfg, y)
    e_a, e_t = rel_l2(ax, oracle_mod.project(cfg, x)), rel_l2(aty, oracle_mod.backproject(cfg, y))
    print(f"{name}: A {e_a:.2e}  A^T {e_t:.2e}")
    assert e_a <= TOL and e_t <= TOL
    lhs = float((ax.astype(np.float64) * y).sum())
    rhs = float((aty.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


TILTED_MODULAR_CASES = [
    ("tilted_modules", lambda: perturbed_poses(reduced(config(3), 8, nviews=16).replace(nx=67, ny=70, nz=45, nrows=61, ncols=77),
                                               3, shift_mm=20.0, tilt_rad=0.25)),
    ("tilted_tall_voxels", lambda: perturbed_poses(
        reduced(config(3), 8, nviews=12).replace(nx=70, ny=66, nz=21, voxel_z=reduced(config(3), 8).voxel_z * 2.7, nrows=75, ncols=81),
        8, shift_mm=15.0, tilt_rad=0.35)),
    ("wobbly_tilted_orbit", lambda: perturbed_poses(reduced(config(5), 16, nviews=24), 11, shift_mm=10.0, tilt_rad=0.1)),
    ("looking_down_obliquely", lambda: CTConfig(
        "down", 4, nviews=2, arc_deg=360.0, nrows=70, ncols=84, pixel_v=1.5, pixel_u=1.4, nx=68, ny=66, nz=37,
        voxel_xy=1.0, voxel_z=1.3, shift_u=0.2, shift_v=-0.3,
        poses=((120.0, -4.0, 160.0, -88.0, 3.0, -120.0, 0.0, 1.0, 0.0, 0.8, 0.0, -0.6),
               (24.0, 136.0, 152.0, -8.0, -100.0, -112.0, 0.8, 0.6, 0.0, -0.36, 0.48, -0.8)))),
]


@pytest.mark.parametrize("name,make", TILTED_MODULAR_CASES, ids=[c[0] for c in TILTED_MODULAR_CASES])
def test_modular_geometry_with_tilted_modules(torch_mod, oracle_mod, name, make):
    """Footprints on modules with any orthonormal axes: knots and axial interval from central projections onto the
    module's own axes; one thread per ray / per voxel."""
    from paper_2307_05801_amd import Geometry
    cfg = make()
    assert "tilted modules" in Geometry(cfg, model="sf").describe()
    x = uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 6)[0]
    ax = gpu_project(torch_mod, cfg, x)
    aty = gpu_backproject(torch_mod, cfg, y)
    ref_a, ref_t = oracle_mod.project(cfg, x), oracle_mod.backproject(cfg, y)
    e_a, e_t = rel_l2(ax, ref_a), rel_l2(aty, ref_t)
    print(f"{name}: A {e_a:.2e}  A^T {e_t:.2e}")
    assert e_a <= TOL and e_t <= TOL
    assert np.abs(ax - ref_a).max() <= 2e-5 * np.abs(ref_a).max()
    assert np.abs(aty - ref_t).max() <= 2e-5 * np.abs(ref_t).max()
    lhs = float((ax.astype(np.float64) * y).sum())
    rhs = float((aty.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


@pytest.mark.parametrize("seed", range(4))
def test_random_tilted_scans_with_footprints(torch_mod, oracle_mod, seed):
    from random_geometries import random_tilted_scan
    cfg = random_tilted_scan(seed)
    x, y = uniform_volume(cfg, 5)[0], uniform_sinogram(cfg, 6)[0]
    ax = gpu_project(torch_mod, cfg, x)
    aty = gpu_backproject(torch_mod, cfg, y)
    ref_a, ref_t = oracle_mod.project(cfg, x), oracle_mod.backproject(cfg, y)
    e_a, e_t = rel_l2(ax, ref_a), rel_l2(aty, ref_t)
    print(f"seed {seed}: A {e_a:.2e}  A^T {e_t:.2e}")
    assert e_a <= TOL and e_t <= TOL
    assert np.abs(ax - ref_a).max() <= 2e-5 * np.abs(ref_a).max() and np.abs(aty - ref_t).max() <= 2e-5 * np.abs(ref_t).max()


def test_tilted_scan_without_footprints_is_refused(torch_mod):
    from paper_2307_05801_amd import Geometry, binding as B
    below = (0.3, -0.2, 40.0, 0.0, 0.0, -30.0, 0.8, 0.6, 0.0, -0.6, 0.8, 0.0)
    cfg = CTConfig("bad", 4, nviews=1, arc_deg=360.0, nrows=20, ncols=24, pixel_v=1.5, pixel_u=1.4, nx=18, ny=16, nz=12,
                   voxel_xy=1.0, voxel_z=1.3, poses=(below,))
    with pytest.raises(B.LeapError) as err:
        Geometry(cfg, model="sf")
    assert err.value.status == B.LEAP_BAD_GEOMETRY
