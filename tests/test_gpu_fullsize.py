"""Parity at the benchmark's full size (512^3 cone-beam, 720 views), in the launch configuration bench.py
times: the whole operator runs once on the GPU, and the oracle recomputes samples of the output one by one
(whole views of A x for a handful of views, single rays, single voxels of A^T y).  The 1024^3 case checks
the 64-bit offsets on a 16-view subset of its scanner."""
import numpy as np
import pytest

from synthetic import config, standard_volume, uniform_sinogram

pytestmark = pytest.mark.gpu

TOL = 1e-5


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / np.linalg.norm(ref))


@pytest.fixture(scope="module")
def c3_run(oracle_mod):
    import torch
    from paper_2307_05801_amd import Geometry
    cfg = config(3)
    print("[gpu] full-size C3: phantom", flush=True)
    x = standard_volume(3, cfg)
    geo = Geometry(cfg)
    xt = torch.from_numpy(x).cuda()
    print("[gpu] full-size C3: project", flush=True)
    ax = geo.project(xt)
    torch.cuda.synchronize()
    print("[gpu] full-size C3: backproject of the projection", flush=True)
    atax = geo.backproject(ax)
    torch.cuda.synchronize()
    print("[gpu] full-size C3: backproject of noise", flush=True)
    rng = np.random.default_rng([1003, 2])
    noise = torch.from_numpy(rng.random(cfg.sino_shape, dtype=np.float32)).cuda()
    atn = geo.backproject(noise)
    torch.cuda.synchronize()
    out = dict(cfg=cfg, x=x, ax=ax.cpu().numpy(), atax=atax.cpu().numpy(), noise=noise.cpu().numpy(),
               atn=atn.cpu().numpy(), describe=geo.describe())
    geo.close()
    return out


def test_c3_forward_views_match_oracle(c3_run, oracle_mod):
    cfg = c3_run["cfg"]
    views = [0, 89, 181, 270, 404, 555, 633, 719]
    ref = oracle_mod.project(cfg.with_views(views), c3_run["x"])
    for n, a in enumerate(views):
        e = rel_l2(c3_run["ax"][a], ref[n])
        print(f"view {a}: rel-L2 {e:.2e}")
        assert e <= TOL
    assert rel_l2(c3_run["ax"][views], ref) <= TOL


def test_c3_forward_random_rays_match_oracle(c3_run, oracle_mod):
    cfg = c3_run["cfg"]
    rng = np.random.default_rng(42)
    rays = rng.integers(0, cfg.nviews * cfg.nrows * cfg.ncols, 600)
    ref = oracle_mod.project_rays(cfg, c3_run["x"], rays)
    got = c3_run["ax"].ravel()[rays]
    assert rel_l2(got, ref) <= TOL
    assert np.abs(got - ref).max() <= 2e-5 * np.abs(ref).max()


@pytest.mark.parametrize("which", ["atax", "atn"])
def test_c3_backprojection_samples_match_oracle(c3_run, oracle_mod, which):
    cfg = c3_run["cfg"]
    sino = c3_run["ax"] if which == "atax" else c3_run["noise"]
    rng = np.random.default_rng(43)
    n = cfg.nx * cfg.ny * cfg.nz
    vox = np.unique(np.concatenate([
        rng.integers(0, n, 12000),
        np.array([0, cfg.nx - 1, n - 1, n - cfg.nx, (cfg.nz // 2 * cfg.ny + cfg.ny // 2) * cfg.nx + cfg.nx // 2]),
    ]))
    ref = oracle_mod.backproject_voxels(cfg, sino, vox)
    got = c3_run[which].ravel()[vox]
    e = rel_l2(got, ref)
    print(f"{which}: sampled rel-L2 {e:.2e}")
    assert e <= TOL
    assert np.abs(got - ref).max() <= 5e-5 * np.abs(ref).max()


def test_c3_adjoint_identity(c3_run):
    lhs = float((c3_run["ax"].astype(np.float64) * c3_run["noise"]).sum())
    rhs = float((c3_run["atn"].astype(np.float64) * c3_run["x"]).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


def test_c5_subset_of_views_large_offsets(oracle_mod):
    """1024^3 volume (4 GiB: byte offsets beyond 2^32) seen from 16 of the 1440 views."""
    import torch
    from paper_2307_05801_amd import Geometry
    full = config(5)
    views = list(range(7, 1440, 90))
    cfg = full.with_views(views)
    print("[gpu] C5 subset: inputs", flush=True)
    rng = np.random.default_rng([1005, 3])
    x = rng.random(cfg.vol_shape, dtype=np.float32)
    y = uniform_sinogram(cfg, 1005)[0]
    geo = Geometry(cfg)
    print("[gpu] C5 subset: project", flush=True)
    ax = geo.project(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    print("[gpu] C5 subset: backproject", flush=True)
    aty = geo.backproject(torch.from_numpy(y).cuda())
    torch.cuda.synchronize()
    ax, aty = ax.cpu().numpy(), aty.cpu().numpy()
    geo.close()
    rs = np.random.default_rng(44)
    rays = rs.integers(0, cfg.nviews * cfg.nrows * cfg.ncols, 400)
    assert rel_l2(ax.ravel()[rays], oracle_mod.project_rays(cfg, x, rays)) <= TOL
    n = cfg.nx * cfg.ny * cfg.nz
    vox = np.unique(np.concatenate([rs.integers(0, n, 20000), np.array([0, n - 1, n - 1024 * 1024 + 5])]))
    assert rel_l2(aty.ravel()[vox], oracle_mod.backproject_voxels(cfg, y, vox)) <= TOL
    lhs = float((ax.astype(np.float64) * y).sum())
    rhs = float(np.dot(aty.astype(np.float64).ravel(), x.astype(np.float64).ravel()))
    assert abs(lhs - rhs) <= TOL * abs(lhs)


def test_c5_full_size_all_views(oracle_mod):
    """The largest case whole: 1024^3 volume, 1440 views, 1024x1024 detector shifted by 2.5 pixels (4 GiB volume,
    5.6 GiB sinogram).  Inputs are uniform noise (rasterising 50 ellipsoids on 10^9 voxels takes minutes on the CPU);
    outputs are sampled on the GPU and recomputed one by one by the oracle."""
    import torch
    from paper_2307_05801_amd import Geometry
    cfg = config(5)
    print("[gpu] C5 full: inputs", flush=True)
    x = np.random.default_rng([2005, 3]).random(cfg.vol_shape, dtype=np.float32)
    y = np.random.default_rng([2005, 2]).random(cfg.sino_shape, dtype=np.float32)
    geo = Geometry(cfg)
    xt, yt = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    print("[gpu] C5 full: project", flush=True)
    ax = geo.project(xt)
    torch.cuda.synchronize()
    print("[gpu] C5 full: backproject", flush=True)
    aty = geo.backproject(yt)
    torch.cuda.synchronize()
    print("[gpu] C5 full: samples", flush=True)
    rs = np.random.default_rng(45)
    nray, nvox = cfg.nviews * cfg.nrows * cfg.ncols, cfg.nx * cfg.ny * cfg.nz
    rays = np.unique(np.concatenate([rs.integers(0, nray, 300), np.array([0, nray - 1, nray // 2 + 517])]))
    vox = np.unique(np.concatenate([rs.integers(0, nvox, 6000), np.array([0, nvox - 1, nvox // 2 + 1023])]))
    ax_s = ax.view(-1)[torch.from_numpy(rays).cuda()].cpu().numpy()
    aty_s = aty.view(-1)[torch.from_numpy(vox).cuda()].cpu().numpy()

    def dot64(p, q, chunk=1 << 26):
        p, q, total = p.view(-1), q.view(-1), 0.0
        for s in range(0, p.numel(), chunk):
            total += float(torch.dot(p[s:s + chunk].double(), q[s:s + chunk].double()))
        return total

    lhs, rhs = dot64(ax, yt), dot64(aty, xt)
    geo.close()
    del ax, aty, xt, yt
    assert abs(lhs - rhs) <= TOL * abs(lhs)
    assert rel_l2(ax_s, oracle_mod.project_rays(cfg, x, rays)) <= TOL
    assert rel_l2(aty_s, oracle_mod.backproject_voxels(cfg, y, vox)) <= TOL
