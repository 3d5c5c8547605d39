"""The host-memory entry points (leap_project_host, leap_backproject_host) and the parameter-file loader on the GPU:
arrays in pageable and in pinned host memory, batches that exercise the upload / run / download pipeline and its
two-deep buffer rotation, staging buffers far smaller than the arrays, against the device-pointer entry points
(bit-equal: the same kernels on the same data) and against the CPU oracle."""
import numpy as np
import pytest

from synthetic import config, reduced, uniform_sinogram, uniform_volume

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def rel_l2(got, ref):
    return float(np.linalg.norm(np.asarray(got, np.float64) - ref) / np.linalg.norm(ref))


def device_results(torch, geo, x, y):
    """Per-item results of the device-pointer entry points (one call per item, as the host pipeline issues them)."""
    ax = torch.stack([geo.project(torch.from_numpy(x[b]).cuda()) for b in range(x.shape[0])]).cpu().numpy()
    aty = torch.stack([geo.backproject(torch.from_numpy(y[b]).cuda()) for b in range(y.shape[0])]).cpu().numpy()
    return ax, aty


@pytest.mark.parametrize("model", ["sf", "siddon"])
@pytest.mark.parametrize("pinned", [False, True], ids=["pageable", "pinned"])
def test_host_pipeline_matches_the_device_entry_points(torch_mod, oracle_mod, monkeypatch, model, pinned):
    torch = torch_mod
    from paper_2307_05801_amd import Geometry
    monkeypatch.setenv("LEAP_DEBUG", "stage_kib=256")           # arrays of 1.2 and 2.6 MB: several chunks, ragged tail
    # (detector and volume off the symmetric position: no ray of the Siddon model runs inside a voxel face)
    cfg = reduced(config(3), 8, nviews=40).replace(nx=67, ny=70, nz=61, nrows=75, ncols=91, shift_u=0.123, shift_v=-0.231,
                                                   center_x=3.0, center_y=-1.7, center_z=0.9, start_deg=3.0)
    batch = 5
    print(f"[gpu] host pipeline {model} pinned={pinned} batch={batch} {cfg.vol_shape} {cfg.sino_shape}", flush=True)
    x = np.stack([uniform_volume(cfg, 20 + b)[0] for b in range(batch)])
    y = np.stack([uniform_sinogram(cfg, 40 + b)[0] for b in range(batch)])
    geo = Geometry(cfg, model=model)
    ax_ref, aty_ref = device_results(torch, geo, x, y)
    if pinned:
        xin, yin = torch.from_numpy(x).pin_memory(), torch.from_numpy(y).pin_memory()
        ax = torch.full((batch,) + cfg.sino_shape, float("nan")).pin_memory()
        aty = torch.full((batch,) + cfg.vol_shape, float("nan")).pin_memory()
    else:
        xin, yin = x, y
        ax = np.full((batch,) + cfg.sino_shape, np.nan, np.float32)
        aty = np.full((batch,) + cfg.vol_shape, np.nan, np.float32)
    geo.project_host(xin, ax)
    geo.backproject_host(yin, aty)
    one = np.full(cfg.sino_shape, np.nan, np.float32)
    geo.project_host(x[3], one)                                  # batch 1 after a batch: the handle's buffers are reused
    again = np.full((2,) + cfg.vol_shape, np.nan, np.float32)
    geo.backproject_host(y[1:3], again)
    geo.close()
    ax, aty = np.asarray(ax), np.asarray(aty)
    assert np.array_equal(ax, ax_ref) and np.array_equal(aty, aty_ref)
    assert np.array_equal(one, ax_ref[3]) and np.array_equal(again, aty_ref[1:3])
    orc = oracle_mod if model == "sf" else oracle_mod.siddon
    assert rel_l2(ax[4], orc.project(cfg, x[4])) <= TOL
    assert rel_l2(aty[4], orc.backproject(cfg, y[4])) <= TOL


def test_host_arrays_are_checked(torch_mod):
    from paper_2307_05801_amd import Geometry
    cfg = reduced(config(3), 16, nviews=6)
    geo = Geometry(cfg)
    x = np.zeros(cfg.vol_shape, np.float32)
    with pytest.raises(ValueError):
        geo.project_host(x.astype(np.float64), np.zeros(cfg.sino_shape, np.float32))
    with pytest.raises(ValueError):
        geo.project_host(x, np.zeros((2,) + cfg.sino_shape, np.float32))
    with pytest.raises(ValueError):
        geo.project_host(torch_mod.zeros(cfg.vol_shape, device="cuda"), np.zeros(cfg.sino_shape, np.float32))
    geo.close()


def test_geometry_from_a_parameter_file(torch_mod, tmp_path):
    """The scanner written to a parameter file and read back projects exactly as the one built from the configuration."""
    torch = torch_mod
    from paper_2307_05801_amd import Geometry, params as P
    cfg = reduced(config(3), 8, nviews=24)
    path = str(tmp_path / "scan.txt")
    P.save_parameters(path, dict(
        type=cfg.geom, model="sf", nviews=cfg.nviews, nrows=cfg.nrows, ncols=cfg.ncols, nx=cfg.nx, ny=cfg.ny, nz=cfg.nz,
        pixel_v=cfg.pixel_v, pixel_u=cfg.pixel_u, shift_v=cfg.shift_v, shift_u=cfg.shift_u, sod=cfg.sod, sdd=cfg.sdd,
        voxel_xy=cfg.voxel_xy, voxel_z=cfg.voxel_z, center_x=cfg.center_x, center_y=cfg.center_y, center_z=cfg.center_z,
        angles_rad=[float(a) for a in cfg.angles()]))
    x = torch.from_numpy(uniform_volume(cfg, 3)[0]).cuda()
    a, b = Geometry(cfg), P.geometry_from_file(path)
    ya, yb = a.project(x), b.project(x)
    torch.cuda.synchronize()
    assert a.describe() == b.describe()
    assert rel_l2(yb.cpu().numpy(), ya.cpu().numpy().astype(np.float64)) <= 1e-6      # angles go through degrees and text
    a.close(); b.close()
