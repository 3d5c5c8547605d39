"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared symbol, and
rejects bad arguments with the documented status codes before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2307_05801_amd import binding as B
from synthetic import config, reduced
from synthetic.configs import CONE, FAN, PARALLEL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2307_05801_amd.build import build_library
        build_library()
    return B.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "leap.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(leap_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    for code in (0, -1, -2, -3, -4):
        assert lib.leap_status_string(code).decode()
    assert lib.leap_status_string(-99).decode() == "unknown status"


def _create(lib, cfg, **over):
    d, keep = B.desc_from_config(cfg)
    for k, v in over.items():
        setattr(d, k, v)
    h = C.c_void_p()
    rc = lib.leap_geometry_create(C.byref(d), C.byref(h))
    if rc == 0:
        lib.leap_geometry_destroy(h)
    return rc


def test_invalid_arguments_are_rejected_before_the_device_is_touched(lib):
    cfg = reduced(config(3), 32, nviews=4)
    h = C.c_void_p()
    assert lib.leap_geometry_create(None, C.byref(h)) == B.LEAP_INVALID_ARG
    d, keep = B.desc_from_config(cfg)
    assert lib.leap_geometry_create(C.byref(d), None) == B.LEAP_INVALID_ARG
    for field in ("nviews", "nrows", "ncols", "nx", "ny", "nz"):
        assert _create(lib, cfg, **{field: 0}) == B.LEAP_INVALID_ARG
        assert _create(lib, cfg, **{field: -3}) == B.LEAP_INVALID_ARG
    for field in ("pixel_u", "pixel_v", "voxel_xy", "voxel_z"):
        assert _create(lib, cfg, **{field: 0.0}) == B.LEAP_INVALID_ARG
        assert _create(lib, cfg, **{field: float("nan")}) == B.LEAP_INVALID_ARG
    assert _create(lib, cfg, type=7) == B.LEAP_INVALID_ARG
    assert _create(lib, cfg, shift_u=float("inf")) == B.LEAP_INVALID_ARG
    assert _create(lib, cfg, angles_rad=C.POINTER(C.c_double)()) == B.LEAP_INVALID_ARG
    assert _create(lib, cfg, type=FAN) == B.LEAP_INVALID_ARG          # fan needs one row, one slice
    assert lib.leap_last_error().decode()


def test_source_inside_volume_is_bad_geometry(lib):
    cfg = reduced(config(3), 32, nviews=4)      # field half-diagonal = 128*sqrt(2) = 181 mm
    assert _create(lib, cfg, sod=150.0) == B.LEAP_BAD_GEOMETRY
    assert _create(lib, cfg, sod=181.0) == B.LEAP_BAD_GEOMETRY
    assert _create(lib, cfg, sdd=0.0) == B.LEAP_BAD_GEOMETRY
    assert _create(lib, cfg, center_x=900.0) == B.LEAP_BAD_GEOMETRY
    # parallel-beam ignores sod/sdd
    par = cfg.replace(geom=PARALLEL)
    assert _create(lib, par, sod=0.0, sdd=0.0) in (B.LEAP_OK, B.LEAP_HIP_ERROR)


def test_null_data_pointers_are_rejected(lib):
    fake = C.c_void_p(0x1000)
    assert lib.leap_project(None, fake, fake, 1, None) == B.LEAP_INVALID_ARG
    assert lib.leap_backproject(None, fake, fake, 1, None) == B.LEAP_INVALID_ARG
    buf = C.create_string_buffer(8)
    assert lib.leap_geometry_describe(None, buf, 8) == B.LEAP_INVALID_ARG


def test_python_binding_raises_with_the_library_message(lib):
    cfg = reduced(config(3), 32, nviews=4).replace(sod=10.0)
    d, keep = B.desc_from_config(cfg)
    with pytest.raises(B.LeapError) as err:
        B.leap_geometry_create(d)
    assert err.value.status == B.LEAP_BAD_GEOMETRY and "sod" in str(err.value)


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        B.load_library(str(tmp_path / "nope.so"))


def test_projector_refuses_cpu_devices():
    from paper_2307_05801_amd import Geometry
    with pytest.raises(RuntimeError, match="GPU"):
        Geometry(reduced(config(1), 1), device="cpu")
