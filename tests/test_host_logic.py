"""Host logic of the HIP library, exercised on the CPU (no GPU): the real geometry module (validation, table
building, kernel selection and its static limits) linked against stubs of the HIP runtime, the general kernel bodies
stepped thread by thread, the window arithmetic of the tiled back projection, and the arithmetic of the column-wise
forward kernel.  tests/host/host_harness.cpp holds the C++ side."""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

from paper_2307_05801_amd import binding as B
from synthetic import (CTConfig, config, modular_from, perturbed_poses, reduced, standard_volume, uniform_sinogram,
                       uniform_volume)
from synthetic.configs import CONE, CONE_CURVED, FAN, PARALLEL

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "host", "host_harness.cpp")
LIB = os.path.join(HERE, "host", "libhost_harness.so")
TOL = 1e-5


@pytest.fixture(scope="module")
def host():
    deps = [SRC, os.path.join(ROOT, "paper_2307_05801_amd", "csrc")]
    newest = max(os.path.getmtime(os.path.join(d, f)) if os.path.isdir(d) else os.path.getmtime(d)
                 for d in deps for f in (os.listdir(d) if os.path.isdir(d) else [""]))
    import fcntl
    with open(LIB + ".lock", "w") as lock:          # several pytest-xdist workers may arrive here together
        fcntl.flock(lock, fcntl.LOCK_EX)
        if not os.path.exists(LIB) or os.path.getmtime(LIB) < newest:
            tmp = f"{LIB}.{os.getpid()}.tmp"
            cmd = ["g++", "-O2", "-fopenmp", "-std=c++17", "-fPIC", "-shared", "-D__HIP_PLATFORM_AMD__",
                   "-I/opt/rocm/include", "-o", tmp, SRC,
                   os.path.join(ROOT, "paper_2307_05801_amd", "csrc", "leap_geometry.cpp"),
                   os.path.join(ROOT, "paper_2307_05801_amd", "csrc", "leap_host.cpp")]
            subprocess.run(cmd, check=True, capture_output=True)
            os.replace(tmp, LIB)
    lib = C.CDLL(LIB)
    B.declare(lib, solvers=False)
    lib.host_check_backproject_windows.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
    lib.host_project_columns.restype = C.c_long
    lib.host_project_columns.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.host_curved_column_deviation.argtypes = [C.c_void_p, C.POINTER(C.c_double)]
    lib.host_sd_project_columns.restype = C.c_long
    lib.host_sd_project_columns.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.host_md_backproject_tiled.restype = C.c_long
    lib.host_md_backproject_tiled.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int64)]
    lib.host_md_project_columns.restype = C.c_long
    lib.host_md_project_columns.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
    return lib


def rel_l2(got, ref):
    return float(np.linalg.norm(np.asarray(got, np.float64) - ref) / np.linalg.norm(ref))


def handle(lib, cfg, model=B.LEAP_MODEL_SF):
    d, keep = B.desc_from_config(cfg, model)
    return B.leap_geometry_create(d, lib)


CASES = {
    "c1": (1, lambda: config(1)),
    "c2_div8": (2, lambda: reduced(config(2), 8, nviews=20)),
    "c3_div8_ragged": (3, lambda: reduced(config(3), 8, nviews=24).replace(nx=67, ny=70, nz=45, nrows=61, ncols=77)),
    "c3_div8_offsets": (3, lambda: reduced(config(3), 8, nviews=9).replace(
        shift_u=1.3, shift_v=-2.7, center_x=6.0, center_y=-4.5, center_z=3.25, start_deg=7.0)),
    "c4_div4": (4, lambda: reduced(config(4), 4, nviews=10)),
    "c5_div16": (5, lambda: reduced(config(5), 16, nviews=18)),
    "curved_c3_div8": (3, lambda: reduced(config(3), 8, nviews=24).replace(
        geom=CONE_CURVED, nx=67, ny=70, nz=45, nrows=61, ncols=77, shift_u=0.6, shift_v=-1.2, center_x=3.0)),
    "curved_wide_fan": (3, lambda: CTConfig("curved_wide", CONE_CURVED, nviews=16, arc_deg=360.0, nrows=48, ncols=120,
                                            pixel_v=2.0, pixel_u=1.6, nx=64, ny=60, nz=40, voxel_xy=1.0, voxel_z=1.2,
                                            sod=110.0, sdd=170.0, shift_u=-0.8, shift_v=0.3, center_y=1.5, start_deg=4.0)),
    # rows up to 1.9, 2.4 and 2.9 voxels tall: a pair of adjacent rows overlaps up to 5, 6 and 7 voxels
    "tall_rows_5": (3, lambda: reduced(config(3), 8, nviews=12).replace(pixel_v=8.0, nrows=56, voxel_z=3.4, nz=70, shift_v=0.3)),
    "tall_rows_6": (3, lambda: reduced(config(3), 8, nviews=12).replace(pixel_v=10.2, nrows=44, voxel_z=3.4, nz=70, center_z=2.0)),
    "tall_rows_7": (3, lambda: reduced(config(3), 8, nviews=12).replace(pixel_v=12.3, nrows=36, voxel_z=3.4, nz=70, shift_v=-0.4)),
    # rows under half a voxel tall: a pair stays within 2 voxels
    "short_rows_2": (3, lambda: reduced(config(3), 8, nviews=12).replace(pixel_v=2.3, nrows=200, voxel_z=4.0, nz=64)),
    # the source barely clears the volume's bounding circle (27.6 mm) and nx, ny are no multiples of the tile edge: the
    # padding voxels of the edge tiles reach past the source plane, where the window functions must stay defined
    "source_grazing_ragged_volume": (3, lambda: CTConfig("grazing", CONE, nviews=11, arc_deg=360.0, nrows=40, ncols=150,
                                                         pixel_v=1.5, pixel_u=1.5, nx=37, ny=41, nz=12, voxel_xy=1.0,
                                                         voxel_z=1.0, sod=28.5, sdd=60.0, shift_u=0.4, start_deg=2.0)),
    "fan": (3, lambda: CTConfig("fan", FAN, nviews=20, arc_deg=360.0, nrows=1, ncols=90, pixel_v=1.0, pixel_u=2.0,
                                nx=70, ny=64, nz=1, voxel_xy=1.0, voxel_z=1.0, sod=300.0, sdd=500.0, shift_u=0.8)),
}


@pytest.mark.parametrize("name", list(CASES))
def test_general_kernel_bodies_match_oracle_on_cpu(host, oracle_mod, name):
    number, make = CASES[name]
    cfg = make()
    x = standard_volume(number, cfg) if cfg.nz > 1 or number == 1 else uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 50 + number)[0]
    h = handle(host, cfg)
    ax = np.zeros(cfg.sino_shape, np.float32)
    aty = np.zeros(cfg.vol_shape, np.float32)
    B.leap_project(h, x.ctypes.data, ax.ctypes.data, 1, 0, host)
    B.leap_backproject(h, y.ctypes.data, aty.ctypes.data, 1, 0, host)
    B.leap_geometry_destroy(h, host)
    assert rel_l2(ax, oracle_mod.project(cfg, x)) <= TOL
    assert rel_l2(aty, oracle_mod.backproject(cfg, y)) <= TOL
    lhs, rhs = float((ax.astype(np.float64) * y).sum()), float((aty.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


SIDDON_CASES = dict(CASES)
SIDDON_CASES["steep_thin_slices"] = (3, lambda: CTConfig(
    "steep", CONE, nviews=11, arc_deg=360.0, nrows=40, ncols=36, pixel_v=2.9, pixel_u=1.4, nx=30, ny=28, nz=60,
    voxel_xy=1.0, voxel_z=0.21, sod=40.0, sdd=62.0, shift_u=0.3, shift_v=-0.4, center_x=0.7, center_z=-0.3,
    start_deg=3.0))
SIDDON_CASES["parallel_3d"] = (3, lambda: CTConfig(
    "par3", PARALLEL, nviews=13, arc_deg=180.0, nrows=40, ncols=50, pixel_v=0.9, pixel_u=0.8, nx=40, ny=36, nz=21,
    voxel_xy=1.0, voxel_z=1.1, sod=0.0, sdd=0.0, shift_u=0.3, shift_v=-0.4, center_y=0.7, center_z=-0.3,
    start_deg=1.0))


@pytest.mark.parametrize("name", list(SIDDON_CASES))
def test_siddon_kernel_bodies_match_oracle_on_cpu(host, oracle_mod, name):
    number, make = SIDDON_CASES[name]
    cfg = make()
    # A thin ray that runs inside a voxel face plane (central column at an axis-aligned view) is a discontinuity of
    # the Siddon model: which side it falls on depends on the last bit of sin(pi).  Keep the pixel centres off them.
    cfg = cfg.replace(shift_u=cfg.shift_u + 0.123)
    x = standard_volume(number, cfg) if cfg.nz > 1 or number == 1 else uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 50 + number)[0]
    h = handle(host, cfg, B.LEAP_MODEL_SIDDON)
    ax = np.zeros(cfg.sino_shape, np.float32)
    aty = np.zeros(cfg.vol_shape, np.float32)
    B.leap_project(h, x.ctypes.data, ax.ctypes.data, 1, 0, host)
    B.leap_backproject(h, y.ctypes.data, aty.ctypes.data, 1, 0, host)
    fast = np.zeros(cfg.sino_shape, np.float32)
    bad = host.host_sd_project_columns(h, x.ctypes.data, fast.ctypes.data)
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    sd = oracle_mod.siddon
    assert ("A=columns" in desc) == (bad >= 0)
    assert ("A=columns" in desc) == (name not in ("c1", "fan", "steep_thin_slices")), desc
    if bad >= 0:
        assert bad == 0, desc
        assert rel_l2(fast, sd.project(cfg, x)) <= TOL, desc
    assert rel_l2(ax, sd.project(cfg, x)) <= TOL
    assert rel_l2(aty, sd.backproject(cfg, y)) <= TOL
    lhs, rhs = float((ax.astype(np.float64) * y).sum()), float((aty.astype(np.float64) * x).sum())
    assert abs(lhs - rhs) <= TOL * abs(lhs)


@pytest.mark.parametrize("name", ["c2_div8", "c3_div8_ragged", "c3_div8_offsets", "c4_div4", "c5_div16", "curved_c3_div8",
                                  "curved_wide_fan", "tall_rows_5", "tall_rows_6", "tall_rows_7", "short_rows_2"])
def test_column_forward_arithmetic_matches_oracle_on_cpu(host, oracle_mod, name, monkeypatch):
    number, make = CASES[name]
    cfg = make()
    x = standard_volume(number, cfg)
    ref = oracle_mod.project(cfg, x)
    for cw in ("1", "2", "4"):
        monkeypatch.setenv("LEAP_DEBUG", "cw=" + cw)
        h = handle(host, cfg)
        out = np.zeros(cfg.sino_shape, np.float32)
        uncovered = host.host_project_columns(h, x.ctypes.data, out.ctypes.data)
        desc = B.leap_geometry_describe(h, host)
        B.leap_geometry_destroy(h, host)
        assert uncovered == 0, desc
        assert rel_l2(out, ref) <= TOL, desc
        if name.startswith("tall_rows_") or name.startswith("short_rows_"):
            assert "nkp=" + name.rsplit("_", 1)[1] in desc, desc


def scratch_bytes(desc):
    return int(desc.split("scratch=")[1].split()[0])


@pytest.mark.parametrize("number", [2, 3, 4, 5])
@pytest.mark.parametrize("model", [B.LEAP_MODEL_SF, B.LEAP_MODEL_SIDDON])
def test_forward_scratch_is_bounded(host, number, model):
    """The z-fastest copy the fast forward kernels read holds one slab of the volume at a time: an eighth of the volume
    (a quarter with Siddon weights) from 512 MiB volumes on, 128 MiB for smaller ones."""
    cfg = config(number)
    h = handle(host, cfg, model)
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    assert "A=columns" in desc, desc
    volume_bytes = 4 * cfg.nx * cfg.ny * cfg.nz
    if volume_bytes >= 512 << 20:
        bound = volume_bytes // (8 if model == B.LEAP_MODEL_SF else 4)
    else:
        bound = 128 << 20
    assert 0 < scratch_bytes(desc) <= bound, desc


def test_scratch_override_and_general_kernels_need_none(host, monkeypatch):
    cfg = reduced(config(3), 4, nviews=8)
    monkeypatch.setenv("LEAP_DEBUG", "slab=16,scratch_mib=3")
    h = handle(host, cfg)
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    assert "slab=16" in desc and scratch_bytes(desc) == 3 << 20, desc
    monkeypatch.setenv("LEAP_DEBUG", "general=1")
    h = handle(host, cfg)
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    assert "A=general" in desc and scratch_bytes(desc) == 0, desc


@pytest.mark.parametrize("case,model,tokens", [
    (2, B.LEAP_MODEL_SF, ("A=columns(", "cw=4", "AT=tiled(nc=3,nv=2,zc=64")),
    (3, B.LEAP_MODEL_SF, ("A=columns(", "rg=4,cw=4", "AT=tiled(nc=3,nv=2,zc=64")),
    (4, B.LEAP_MODEL_SF, ("A=columns(", "rg=3,cw=4", "AT=tiled(nc=4,nv=3,zc=16")),
    (5, B.LEAP_MODEL_SF, ("A=columns(", "rg=4,cw=4", "AT=tiled(nc=3,nv=3,zc=64")),
    (3, B.LEAP_MODEL_SIDDON, ("A=columns(rg=8", "AT=tiled(nc=2,zc=32")),
])
def test_benchmark_cases_take_the_instances_the_measurements_name(host, case, model, tokens):
    """The kernel instances the measured figures belong to: a change of the selection rules that moves a benchmark case
    to another instance (or to the general kernels) shows up here, on the CPU."""
    h = handle(host, config(case), model)
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    for token in tokens:
        assert token in desc, desc


def test_row_schemes_of_the_tiled_back_projection_follow_the_voxel_height(host):
    """The three-row instance of the tiled back projection runs schemes that need every voxel at most two detector rows
    tall: a bound on the height within a thousandth of two rows takes the four-row instance, and volumes of 128 layers
    and more keep 64 voxels per thread for footprints up to two rows tall when their window fits."""
    base = reduced(config(2), 4, nviews=8)                 # parallel beam: a voxel is voxel_z / pixel_v rows tall
    for voxel_z, nz, token in ((0.99, 40, "nv=2,"), (1.0, 40, "nv=2,"), (1.25, 40, "nv=3,"), (1.99, 40, "nv=3,"),
                               (1.9995, 40, "nv=4,"), (2.4, 40, "nv=4,"),
                               (1.0, 160, "nv=2,zc=64"), (1.2, 160, "nv=3,zc=64"), (1.9, 160, "nv=3,zc=16")):
        cfg = base.replace(voxel_z=voxel_z, pixel_v=1.0, nz=nz, nrows=int(voxel_z * nz) + 12)
        h = handle(host, cfg)
        desc = B.leap_geometry_describe(h, host)
        B.leap_geometry_destroy(h, host)
        assert "AT=tiled" in desc and token in desc, (voxel_z, nz, desc)


def window_report(host, cfg):
    h = handle(host, cfg)
    rep = (C.c_int64 * 8)()
    host.host_check_backproject_windows(h, rep)
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    return list(rep), desc


@pytest.mark.parametrize("name", ["c2_div8", "c3_div8_ragged", "c3_div8_offsets", "c4_div4", "c5_div16", "curved_c3_div8",
                                  "curved_wide_fan"])
def test_tiled_backprojection_reads_stay_inside_the_staged_window(host, name):
    rep, desc = window_report(host, CASES[name][1]())
    assert rep[0] == 1, desc
    assert rep[7] == 0, (rep, desc)


@pytest.mark.parametrize("name", ["curved_c3_div8", "curved_wide_fan"])
def test_curved_tile_relative_columns_agree_with_the_general_function(host, name):
    """The tiled back projection takes a voxel column's fan angle relative to its tile's centre and the corner angles
    from a short series.  Against the general function (double atan2, atanf) the column coordinate may move by the
    float roundings of the small angle (four of them: about 2.4e-7 x angle x pixels per radian, a few 1e-6 pixel on
    these cases), the knot offsets by less."""
    h = handle(host, CASES[name][1]())
    out = (C.c_double * 3)()
    assert host.host_curved_column_deviation(h, out) == 0
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    assert "AT=tiled" in desc, desc
    assert out[0] < 4e-6 and out[1] < 1e-6, list(out)
    assert out[2] < 0.08, list(out)


def test_curved_source_too_close_for_the_series(host):
    """Corner angles above 0.08 rad: the tiled curved kernel is not chosen."""
    cfg = CTConfig("curved_close", CONE_CURVED, nviews=8, arc_deg=360.0, nrows=40, ncols=64, pixel_v=2.5, pixel_u=2.5,
                   nx=16, ny=16, nz=16, voxel_xy=2.0, voxel_z=2.0, sod=28.0, sdd=60.0)
    h = handle(host, cfg)
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    assert "AT=general" in desc, desc


def test_window_limits_at_full_benchmark_sizes(host):
    """Every tile and chunk of a spread of views of the 512^3 and 1024^3 cone-beam cases, and the batch case."""
    for cfg in (config(3).with_views(list(range(0, 720, 45))), config(5).with_views([0, 181, 542, 1260]), config(4)):
        rep, desc = window_report(host, cfg)
        assert rep[0] == 1 and rep[7] == 0, (rep, desc)


def test_kernel_selection(host):
    def desc(cfg):
        h = handle(host, cfg)
        s = B.leap_geometry_describe(h, host)
        B.leap_geometry_destroy(h, host)
        return s
    assert "A=columns" in desc(config(3)) and "AT=tiled" in desc(config(3))
    assert "A=general" in desc(CASES["fan"][1]()) and "AT=general" in desc(CASES["fan"][1]())
    assert "A=general" in desc(config(1))                                  # one detector row: nothing to tile
    coarse = reduced(config(3), 8, nviews=4).replace(pixel_u=37.0, pixel_v=29.0, nrows=14, ncols=12)
    assert "A=general" in desc(coarse)                                     # a row spans six voxels
    fine = reduced(config(3), 8, nviews=4).replace(pixel_u=1.7, pixel_v=1.9, nrows=300, ncols=280)
    assert "AT=general" in desc(fine)                                      # a voxel spans six pixels


@pytest.mark.parametrize("seed", range(24))
def test_random_geometries_on_cpu(host, oracle_mod, seed):
    """Whatever kernels a random scanner selects, their static limits hold and the arithmetic matches the oracle."""
    from random_geometries import random_config
    cfg = random_config(seed)
    x = uniform_volume(cfg, seed)[0]
    y = uniform_sinogram(cfg, seed)[0]
    h = handle(host, cfg)
    desc = B.leap_geometry_describe(h, host)
    rep = (C.c_int64 * 8)()
    host.host_check_backproject_windows(h, rep)
    assert rep[7] == 0, (list(rep), desc)
    ref = oracle_mod.project(cfg, x)
    out = np.zeros(cfg.sino_shape, np.float32)
    uncovered = host.host_project_columns(h, x.ctypes.data, out.ctypes.data)
    if uncovered >= 0:
        assert uncovered == 0, desc
        assert rel_l2(out, ref) <= TOL, desc
    ax = np.zeros(cfg.sino_shape, np.float32)
    aty = np.zeros(cfg.vol_shape, np.float32)
    B.leap_project(h, x.ctypes.data, ax.ctypes.data, 1, 0, host)
    B.leap_backproject(h, y.ctypes.data, aty.ctypes.data, 1, 0, host)
    B.leap_geometry_destroy(h, host)
    assert rel_l2(ax, ref) <= TOL, desc
    assert rel_l2(aty, oracle_mod.backproject(cfg, y)) <= TOL, desc


MODULAR_CASES = {
    "cone_as_modular": lambda: modular_from(reduced(config(3), 16, nviews=10).replace(shift_u=0.123)),
    "tilted_modules": lambda: perturbed_poses(reduced(config(3), 16, nviews=9).replace(nx=29, ny=35, nz=22, nrows=27, ncols=31),
                                              3, shift_mm=20.0, tilt_rad=0.25),
    "looking_down": lambda: CTConfig("down", 4, nviews=2, arc_deg=360.0, nrows=20, ncols=24, pixel_v=1.5, pixel_u=1.4,
                                     nx=18, ny=16, nz=12, voxel_xy=1.0, voxel_z=1.3, shift_u=0.2, shift_v=-0.3,
                                     poses=((0.3, -0.2, 40.0, 0.0, 0.0, -30.0, 1.0, 0.0, 0.0, 0.0, 1.0, 0.0),
                                            (6.0, 2.0, 38.0, -2.0, 1.0, -28.0, 0.8, 0.6, 0.0, -0.6, 0.8, 0.0))),
}


@pytest.mark.parametrize("name", list(MODULAR_CASES))
def test_modular_siddon_bodies_match_oracle_on_cpu(host, oracle_mod, name):
    cfg = MODULAR_CASES[name]()
    x = uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 6)[0]
    h = handle(host, cfg, B.LEAP_MODEL_SIDDON)
    ax = np.zeros(cfg.sino_shape, np.float32)
    aty = np.zeros(cfg.vol_shape, np.float32)
    B.leap_project(h, x.ctypes.data, ax.ctypes.data, 1, 0, host)
    B.leap_backproject(h, y.ctypes.data, aty.ctypes.data, 1, 0, host)
    B.leap_geometry_destroy(h, host)
    sd = oracle_mod.siddon
    assert rel_l2(ax, sd.project(cfg, x)) <= TOL
    assert rel_l2(aty, sd.backproject(cfg, y)) <= TOL
    if name == "cone_as_modular":
        cone = reduced(config(3), 16, nviews=10).replace(shift_u=0.123)
        assert rel_l2(ax, sd.project(cone, x)) <= TOL


TILTED_FOOTPRINT_CASES = {
    "tilted_modules": MODULAR_CASES["tilted_modules"],
    "tilted_tall_voxels": lambda: perturbed_poses(
        reduced(config(3), 16, nviews=7).replace(nx=23, ny=19, nz=9, voxel_z=3.1, nrows=33, ncols=29), 8, shift_mm=15.0,
        tilt_rad=0.35),
    "looking_down_obliquely": lambda: CTConfig(
        "down", 4, nviews=2, arc_deg=360.0, nrows=20, ncols=24, pixel_v=1.5, pixel_u=1.4, nx=18, ny=16, nz=12,
        voxel_xy=1.0, voxel_z=1.3, shift_u=0.2, shift_v=-0.3,
        poses=((30.0, -4.0, 40.0, -22.0, 3.0, -30.0, 0.0, 1.0, 0.0, 0.8, 0.0, -0.6),
               (6.0, 34.0, 38.0, -2.0, -25.0, -28.0, 0.8, 0.6, 0.0, -0.36, 0.48, -0.8))),
    "mixed_upright_and_tilted": lambda: _mixed_scan(),
}


def _mixed_scan():
    base = reduced(config(3), 16, nviews=8).replace(nx=21, ny=26, nz=17, nrows=25, ncols=30)
    t = perturbed_poses(base, 5, shift_mm=10.0, tilt_rad=0.2)
    u = perturbed_poses(base, 5, shift_mm=10.0, tilt_rad=0.2, upright=True)
    return t.replace(poses=tuple(t.poses[a] if a % 2 else u.poses[a] for a in range(t.nviews)))


@pytest.mark.parametrize("name", list(TILTED_FOOTPRINT_CASES))
def test_tilted_footprint_bodies_match_oracle_on_cpu(host, oracle_mod, name):
    """The one-thread-per-ray / per-voxel bodies of the footprint model on tilted modules, stepped on the CPU."""
    cfg = TILTED_FOOTPRINT_CASES[name]()
    x = uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 6)[0]
    h = handle(host, cfg, B.LEAP_MODEL_SF)
    desc = B.leap_geometry_describe(h, host)
    assert "tilted modules" in desc and "A=general" in desc and "AT=general" in desc, desc
    ax = np.zeros(cfg.sino_shape, np.float32)
    aty = np.zeros(cfg.vol_shape, np.float32)
    B.leap_project(h, x.ctypes.data, ax.ctypes.data, 1, 0, host)
    B.leap_backproject(h, y.ctypes.data, aty.ctypes.data, 1, 0, host)
    B.leap_geometry_destroy(h, host)
    ref_a, ref_t = oracle_mod.project(cfg, x), oracle_mod.backproject(cfg, y)
    assert np.abs(ref_a).max() > 0 and np.abs(ref_t).max() > 0
    assert rel_l2(ax, ref_a) <= 1e-6 and rel_l2(aty, ref_t) <= 1e-6
    assert np.abs(ax - ref_a).max() <= 2e-6 * np.abs(ref_a).max()
    assert np.abs(aty - ref_t).max() <= 2e-6 * np.abs(ref_t).max()


def test_tilted_scans_without_footprints_are_refused(host):
    """A source beside the volume with the module on the far side of only part of it, and a module below a source that
    looks straight down: LEAP_BAD_GEOMETRY with a message, as the oracle refuses them."""
    base = dict(nviews=1, arc_deg=360.0, nrows=20, ncols=24, pixel_v=1.5, pixel_u=1.4, nx=18, ny=16, nz=12, voxel_xy=1.0,
                voxel_z=1.3)
    grazing = (10.5, 0.0, 0.0, -30.0, 0.0, 0.0, 0.0, 1.0, 0.0, 0.6, 0.0, 0.8)       # the plane's normal tilts: corners behind
    below = (0.3, -0.2, 40.0, 0.0, 0.0, -30.0, 1.0, 0.0, 0.0, 0.0, 1.0, 0.0)
    for pose in (grazing, below):
        cfg = CTConfig("bad", 4, poses=(pose,), **base)
        with pytest.raises(B.LeapError) as err:
            handle(host, cfg, B.LEAP_MODEL_SF)
        assert err.value.status == B.LEAP_BAD_GEOMETRY and "no footprints" in str(err.value)
    # a source 0.2 mm in front of the volume's face: the nearest voxels' footprints span hundreds of pixels
    roll = np.sqrt(1 - 0.01)
    close = (9.2, 0.0, 0.0, -300.0, 0.0, 0.0, 0.0, roll, -0.1, 0.0, 0.1, roll)        # rolled about its normal (the x axis)
    with pytest.raises(B.LeapError) as err:
        handle(host, CTConfig("close", 4, poses=(close,), **base), B.LEAP_MODEL_SF)
    assert err.value.status == B.LEAP_UNSUPPORTED and "64 pixels" in str(err.value)


UPRIGHT_CASES = {
    "cone_as_modular": lambda: modular_from(reduced(config(3), 16, nviews=10).replace(shift_u=0.3, shift_v=-0.4)),
    "shifted_upright_modules": lambda: perturbed_poses(
        reduced(config(3), 16, nviews=9).replace(nx=29, ny=35, nz=22, nrows=41, ncols=31), 3, shift_mm=25.0, tilt_rad=0.3,
        upright=True),
    "wobbly_orbit": lambda: perturbed_poses(reduced(config(5), 32, nviews=12), 11, shift_mm=10.0, tilt_rad=0.1, upright=True),
}


@pytest.mark.parametrize("name", list(UPRIGHT_CASES))
def test_modular_footprint_bodies_match_oracle_on_cpu(host, oracle_mod, name):
    cfg = UPRIGHT_CASES[name]()
    x = uniform_volume(cfg, 5)[0]
    y = uniform_sinogram(cfg, 6)[0]
    h = handle(host, cfg, B.LEAP_MODEL_SF)
    ax = np.zeros(cfg.sino_shape, np.float32)
    aty = np.zeros(cfg.vol_shape, np.float32)
    B.leap_project(h, x.ctypes.data, ax.ctypes.data, 1, 0, host)
    B.leap_backproject(h, y.ctypes.data, aty.ctypes.data, 1, 0, host)
    # the fast kernels' host-side re-enactments on the per-view parameter blocks
    rep = (C.c_int64 * 8)()
    host.host_check_backproject_windows(h, rep)
    fast = np.zeros(cfg.sino_shape, np.float32)
    uncovered = host.host_project_columns(h, x.ctypes.data, fast.ctypes.data)
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    ref = oracle_mod.project(cfg, x)
    assert rel_l2(ax, ref) <= TOL
    assert rel_l2(aty, oracle_mod.backproject(cfg, y)) <= TOL
    assert "AT=tiled" in desc and rep[0] == 1 and rep[7] == 0, (list(rep), desc)
    if name != "wobbly_orbit":          # that one has 32 detector rows at most: below the column kernel's minimum
        assert "A=columns" in desc, desc
    if uncovered >= 0:
        assert uncovered == 0, desc
        assert rel_l2(fast, ref) <= TOL, desc


@pytest.mark.parametrize("name", list(UPRIGHT_CASES))
def test_upright_modular_siddon_uses_the_ray_table(host, oracle_mod, name):
    """Upright modules get the Siddon model's per-column ray table, built on each view's own parameter block: the
    column kernel's host re-enactment must reproduce the oracle and stay inside the scratch volume."""
    cfg = UPRIGHT_CASES[name]()
    x = standard_volume(3, cfg)
    h = handle(host, cfg, B.LEAP_MODEL_SIDDON)
    fast = np.zeros(cfg.sino_shape, np.float32)
    bad = host.host_sd_project_columns(h, x.ctypes.data, fast.ctypes.data)
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    assert "upright" in desc and "AT=tiled" in desc, desc
    assert "A=columns" in desc and bad == 0, (bad, desc)
    assert rel_l2(fast, oracle_mod.siddon.project(cfg, x)) <= TOL, desc


def test_modular_argument_checks(host):
    cfg = MODULAR_CASES["looking_down"]()
    d, keep = B.desc_from_config(cfg, B.LEAP_MODEL_SF)
    hnd = C.c_void_p()
    assert host.leap_geometry_create(C.byref(d), C.byref(hnd)) == B.LEAP_BAD_GEOMETRY     # a pixel's ray runs along z: no footprint
    d, keep = B.desc_from_config(cfg, B.LEAP_MODEL_SIDDON)
    d.poses = C.POINTER(C.c_double)()
    assert host.leap_geometry_create(C.byref(d), C.byref(hnd)) == B.LEAP_INVALID_ARG
    skew = cfg.replace(poses=((0.3, -0.2, 40.0, 0.0, 0.0, -30.0, 1.0, 0.0, 0.0, 0.1, 1.0, 0.0),) * 2)
    d, keep = B.desc_from_config(skew, B.LEAP_MODEL_SIDDON)
    assert host.leap_geometry_create(C.byref(d), C.byref(hnd)) == B.LEAP_INVALID_ARG
    inside = cfg.replace(poses=((0.3, -0.2, 1.0, 0.0, 0.0, -30.0, 1.0, 0.0, 0.0, 0.0, 1.0, 0.0),) * 2)
    d, keep = B.desc_from_config(inside, B.LEAP_MODEL_SIDDON)
    assert host.leap_geometry_create(C.byref(d), C.byref(hnd)) == B.LEAP_BAD_GEOMETRY


def test_host_memory_pipeline_rotates_buffers_and_chunks_correctly(host, monkeypatch):
    """leap_project_host / leap_backproject_host against the device-pointer calls, with every asynchronous HIP call
    of the pipeline carried out at once (the harness' stubs): 5 items through the two-deep buffer rotation, staging
    buffers of 4 KiB so that every array takes many chunks with a ragged last one, both directions on one handle."""
    monkeypatch.setenv("LEAP_DEBUG", "stage_kib=4")
    cfg = reduced(config(3), 32, nviews=5).replace(nx=19, ny=17, nz=11, nrows=13, ncols=23)
    batch = 5
    x = np.stack([uniform_volume(cfg, 20 + b)[0] for b in range(batch)])
    y = np.stack([uniform_sinogram(cfg, 40 + b)[0] for b in range(batch)])
    h = handle(host, cfg)
    ax_ref = np.zeros((batch,) + cfg.sino_shape, np.float32)
    aty_ref = np.zeros((batch,) + cfg.vol_shape, np.float32)
    B.leap_project(h, x.ctypes.data, ax_ref.ctypes.data, batch, 0, host)
    B.leap_backproject(h, y.ctypes.data, aty_ref.ctypes.data, batch, 0, host)
    ax = np.full_like(ax_ref, np.nan)
    aty = np.full_like(aty_ref, np.nan)
    B.leap_project_host(h, x.ctypes.data, ax.ctypes.data, batch, host)
    B.leap_backproject_host(h, y.ctypes.data, aty.ctypes.data, batch, host)      # arrays of the other sizes on the same handle
    one = np.full(cfg.sino_shape, np.nan, np.float32)
    B.leap_project_host(h, x[3].ctypes.data, one.ctypes.data, 1, host)
    with pytest.raises(B.LeapError):
        B.leap_project_host(h, x.ctypes.data, x.ctypes.data, 1, host)
    with pytest.raises(B.LeapError):
        B.leap_project_host(h, x.ctypes.data, ax.ctypes.data, 0, host)
    B.leap_geometry_destroy(h, host)
    assert np.array_equal(ax, ax_ref) and np.array_equal(aty, aty_ref) and np.array_equal(one, ax_ref[3])


TILTED_SIDDON_FAST_CASES = {
    "tilted_modules": lambda: perturbed_poses(reduced(config(3), 16, nviews=9).replace(nx=29, ny=35, nz=22, nrows=43, ncols=31),
                                              3, shift_mm=20.0, tilt_rad=0.25),
    "wobbly_tilted_orbit": lambda: perturbed_poses(reduced(config(5), 32, nviews=12), 11, shift_mm=10.0, tilt_rad=0.1),
    "tall_voxels": lambda: perturbed_poses(
        reduced(config(3), 16, nviews=7).replace(nx=23, ny=19, nz=9, voxel_z=3.1, nrows=33, ncols=29), 8, shift_mm=15.0,
        tilt_rad=0.35),
}


@pytest.mark.parametrize("name", list(TILTED_SIDDON_FAST_CASES))
@pytest.mark.parametrize("width", [4, 1000])
def test_tilted_siddon_slab_kernel_matches_oracle_on_cpu(host, oracle_mod, name, width):
    """The per-lane slab walk of the tilted-module Siddon forward kernel, re-enacted slab by slab with the kernel's own
    functions (narrow slabs of 4 layers, and the whole volume at once)."""
    cfg = TILTED_SIDDON_FAST_CASES[name]()
    x = uniform_volume(cfg, 5)[0]
    h = handle(host, cfg, B.LEAP_MODEL_SIDDON)
    desc = B.leap_geometry_describe(h, host)
    out = np.zeros(cfg.sino_shape, np.float32)
    bad = host.host_md_project_columns(h, x.ctypes.data, out.ctypes.data, width)
    B.leap_geometry_destroy(h, host)
    assert "A=columns" in desc and "tilted modules" in desc and bad == 0, (bad, desc)
    ref = oracle_mod.siddon.project(cfg, x)
    assert rel_l2(out, ref) <= TOL, desc
    assert np.abs(out - ref).max() <= 2e-5 * np.abs(ref).max()


def test_steep_or_close_tilted_scans_keep_the_general_siddon_kernels(host):
    """Rays that rise by more than a cell per slab (modules seen obliquely from above), and a source within a voxel of the
    volume's box: the per-lane slab kernel is not chosen."""
    for cfg in (TILTED_FOOTPRINT_CASES["looking_down_obliquely"]().replace(nrows=40), MODULAR_CASES["looking_down"]().replace(nrows=40)):
        h = handle(host, cfg, B.LEAP_MODEL_SIDDON)
        desc = B.leap_geometry_describe(h, host)
        B.leap_geometry_destroy(h, host)
        assert "A=general" in desc, desc
    base = reduced(config(3), 16, nviews=4).replace(nx=24, ny=24, nz=16, nrows=40, ncols=30)
    near = perturbed_poses(base, 2, shift_mm=1.0, tilt_rad=0.1)
    half = 0.5 * base.nx * base.voxel_xy
    poses = [list(p) for p in near.poses]
    poses[1][0:3] = [half + 0.5 * base.voxel_xy, 0.0, 0.0]           # half a voxel outside the +x face
    poses[1][3:6] = [-300.0, 0.0, 0.0]
    h = handle(host, near.replace(poses=tuple(tuple(p) for p in poses)), B.LEAP_MODEL_SIDDON)
    desc = B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    assert "A=general" in desc, desc


def far_scanner(**kw):
    """A cone-beam scanner whose source keeps more than a hundred voxels from the volume (what the tiled back projection
    on tilted modules asks for), small enough for the CPU."""
    base = dict(name="far", geom=2, nviews=9, arc_deg=360.0, nrows=48, ncols=56, pixel_v=1.5, pixel_u=1.5, nx=37, ny=41,
                nz=29, voxel_xy=1.0, voxel_z=1.0, sod=160.0, sdd=240.0, shift_u=0.3, shift_v=-0.4, center_x=1.0,
                center_y=-2.0, center_z=0.5, start_deg=3.0)
    base.update(kw)
    return CTConfig(**base)


TILTED_SIDDON_TILED_CASES = {
    "small_tilts": lambda: perturbed_poses(far_scanner(), 3, shift_mm=4.0, tilt_rad=0.05),
    "rolled_modules": lambda: perturbed_poses(far_scanner(nviews=7), 5, shift_mm=6.0, tilt_rad=0.3),
    "tall_voxels": lambda: perturbed_poses(far_scanner(nz=19, voxel_z=1.7, nviews=8), 8, shift_mm=5.0, tilt_rad=0.15),
}


@pytest.mark.parametrize("name", list(TILTED_SIDDON_TILED_CASES))
def test_tilted_siddon_tiled_back_projection_matches_oracle_on_cpu(host, oracle_mod, name):
    """The tiled back projection on tilted modules re-enacted tile by tile with the kernel's own functions: every staged
    window fits, every read stays inside it, every slot inside the sums, and the result is the oracle's."""
    cfg = TILTED_SIDDON_TILED_CASES[name]()
    y = uniform_sinogram(cfg, 6)[0]
    h = handle(host, cfg, B.LEAP_MODEL_SIDDON)
    desc = B.leap_geometry_describe(h, host)
    out = np.full(cfg.vol_shape, np.nan, np.float32)
    rep = (C.c_int64 * 4)()
    bad = host.host_md_backproject_tiled(h, y.ctypes.data, out.ctypes.data, rep)
    B.leap_geometry_destroy(h, host)
    assert "AT=tiled" in desc and bad == 0, (bad, list(rep), desc)
    ref = oracle_mod.siddon.backproject(cfg, y)
    assert rel_l2(out, ref) <= TOL, desc
    assert np.abs(out - ref).max() <= 2e-5 * np.abs(ref).max()


def test_host_memory_pipeline_with_threaded_staging_copies(host, monkeypatch):
    """Staging buffers of 1 MiB: every chunk's copy to or from pinned memory is shared out among the helper threads, and
    arrays of 2.4 and 1.6 MB take a ragged last chunk."""
    monkeypatch.setenv("LEAP_DEBUG", "stage_kib=1024")
    cfg = reduced(config(3), 8, nviews=6).replace(nx=96, ny=96, nz=64, nrows=96, ncols=112)
    batch = 3
    x = np.stack([uniform_volume(cfg, 60 + b)[0] for b in range(batch)])
    h = handle(host, cfg)
    ref = np.zeros((batch,) + cfg.sino_shape, np.float32)
    B.leap_project(h, x.ctypes.data, ref.ctypes.data, batch, 0, host)
    ax = np.full_like(ref, np.nan)
    B.leap_project_host(h, x.ctypes.data, ax.ctypes.data, batch, host)
    back_ref = np.zeros((batch,) + cfg.vol_shape, np.float32)
    B.leap_backproject(h, ref.ctypes.data, back_ref.ctypes.data, batch, 0, host)
    back = np.full_like(back_ref, np.nan)
    B.leap_backproject_host(h, ref.ctypes.data, back.ctypes.data, batch, host)
    B.leap_geometry_destroy(h, host)
    assert np.array_equal(ax, ref) and np.array_equal(back, back_ref)


def test_large_scans_behind_a_source_plane_are_refused_for_the_siddon_model(host):
    """A module turned 60 degrees away from the line source - volume and rolled a little: the plane through the source
    parallel to the module cuts the volume, so the general back projection would test every pixel for the voxels behind
    it.  Tiny scans run that way (the oracle agrees); at 256^3 x 256^2 the handle is refused."""
    c, s_ = np.cos(np.pi / 3), np.sin(np.pi / 3)
    n = np.array([c, s_, 0.0])
    eu = np.array([-s_, c, 0.0]) * np.sqrt(1 - 0.01) + np.array([0.0, 0.0, -0.1])
    ev = np.cross(n, eu)
    S = np.array([200.0, 0.0, 0.0])
    pose = tuple(np.concatenate([S, S - 300.0 * n, eu / np.linalg.norm(eu), ev / np.linalg.norm(ev)]))
    big = CTConfig("cut", 4, nviews=4, arc_deg=360.0, nrows=256, ncols=256, pixel_v=1.0, pixel_u=1.0, nx=256, ny=256, nz=256,
                   voxel_xy=1.0, voxel_z=1.0, poses=(pose,) * 4)
    with pytest.raises(B.LeapError) as err:
        handle(host, big, B.LEAP_MODEL_SIDDON)
    assert err.value.status == B.LEAP_UNSUPPORTED and "behind the source's plane" in str(err.value)
    small = big.replace(nrows=24, ncols=24, nx=20, ny=20, nz=20, voxel_xy=12.8, voxel_z=12.8, pixel_u=10.0, pixel_v=10.0)
    h = handle(host, small, B.LEAP_MODEL_SIDDON)
    assert "AT=general" in B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)


@pytest.mark.parametrize("seed", range(16))
def test_flatness_decision_of_tilted_siddon_scans_matches_brute_force(host, seed):
    """The per-lane slab kernel is chosen iff no ray rises by more than 0.999 axial cells per slab along its faster in-plane
    axis.  The library decides that by clipping the detector's rectangle with four half-planes per view; here every pixel
    (and a 4 x finer grid between the pixel centres) is simply tried."""
    rng = np.random.default_rng([seed, 77])
    base = far_scanner(nviews=6, voxel_z=float(rng.uniform(0.5, 2.0)), nz=int(rng.integers(10, 40)))
    cfg = perturbed_poses(base, seed, shift_mm=float(rng.uniform(0, 30)), tilt_rad=float(rng.uniform(0.05, 1.3)))
    lift = float(rng.uniform(0.0, 260.0))            # sources raised above the volume: their rays dive
    cfg = cfg.replace(poses=tuple(tuple(np.asarray(p) + np.array([0, 0, lift * (a % 2)] + [0] * 9)) for a, p in enumerate(cfg.poses)))
    h = handle(host, cfg, B.LEAP_MODEL_SIDDON)
    fast = "A=columns" in B.leap_geometry_describe(h, host)
    B.leap_geometry_destroy(h, host)
    kappa = cfg.voxel_xy / cfg.voxel_z
    u = (np.linspace(0, cfg.ncols - 1, 4 * cfg.ncols - 3) - (cfg.ncols - 1) / 2 + cfg.shift_u) * cfg.pixel_u
    v = (np.linspace(0, cfg.nrows - 1, 4 * cfg.nrows - 3) - (cfg.nrows - 1) / 2 + cfg.shift_v) * cfg.pixel_v
    uu, vv = np.meshgrid(u, v)
    worst = 0.0
    for p in cfg.poses:
        p = np.asarray(p)
        D = (p[3:6] - p[0:3]) + uu[..., None] * p[6:9] + vv[..., None] * p[9:12]
        with np.errstate(divide="ignore"):
            worst = max(worst, float((kappa * np.abs(D[..., 2]) / np.maximum(np.abs(D[..., 0]), np.abs(D[..., 1]))).max()))
    if worst > 1.0:
        assert not fast, worst
    elif worst < 0.99:
        assert fast, worst          # (these scanners keep every source far more than a voxel from the volume)


@pytest.mark.parametrize("seed", range(8))
def test_tilted_siddon_kernels_on_random_scans_match_oracle_on_cpu(host, oracle_mod, seed):
    """Random tilts (up to 0.5 rad about every axis), shifts, voxel aspect ratios and sizes: wherever the library picks the
    per-lane kernels, their re-enactments stay inside their buffers and agree with the oracle."""
    from random_geometries import random_tilted_scan
    cfg = random_tilted_scan(seed)
    x, y = uniform_volume(cfg, 5)[0], uniform_sinogram(cfg, 6)[0]
    h = handle(host, cfg, B.LEAP_MODEL_SIDDON)
    desc = B.leap_geometry_describe(h, host)
    sd = oracle_mod.siddon
    checked = 0
    if "A=columns" in desc:
        out = np.zeros(cfg.sino_shape, np.float32)
        assert host.host_md_project_columns(h, x.ctypes.data, out.ctypes.data, 8) == 0, desc
        assert rel_l2(out, sd.project(cfg, x)) <= TOL, desc
        checked += 1
    if "AT=tiled" in desc:
        out = np.full(cfg.vol_shape, np.nan, np.float32)
        rep = (C.c_int64 * 4)()
        assert host.host_md_backproject_tiled(h, y.ctypes.data, out.ctypes.data, rep) == 0, (list(rep), desc)
        ref = sd.backproject(cfg, y)
        assert rel_l2(out, ref) <= TOL and np.abs(out - ref).max() <= 2e-5 * np.abs(ref).max(), desc
        checked += 1
    B.leap_geometry_destroy(h, host)
    assert checked >= 1, desc
