"""ctypes binding of the C ABI declared in include/leap.h: argument marshalling only.

Every step of the projector pair runs inside libleap_hip.so; nothing here computes.  PyTorch supplies
device memory (tensor.data_ptr()) and the current HIP stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("LEAP_LIB_PATH") or os.path.join(HERE, "libleap_hip.so")   # override: testing a variant build

LEAP_PARALLEL, LEAP_FAN, LEAP_CONE, LEAP_CONE_CURVED, LEAP_MODULAR = 0, 1, 2, 3, 4
LEAP_MODEL_SF, LEAP_MODEL_SIDDON = 0, 1
MODELS = {"sf": LEAP_MODEL_SF, "siddon": LEAP_MODEL_SIDDON}
LEAP_OK, LEAP_INVALID_ARG, LEAP_BAD_GEOMETRY, LEAP_HIP_ERROR, LEAP_UNSUPPORTED = 0, -1, -2, -3, -4

EXPORTS = ("leap_geometry_create", "leap_geometry_destroy", "leap_project", "leap_backproject", "leap_project_static_scratch",
           "leap_project_host", "leap_backproject_host",
           "leap_status_string", "leap_last_error", "leap_geometry_describe",
           "leap_recon_workspace_floats", "leap_sirt", "leap_least_squares_descent")


class leap_geometry_desc(C.Structure):
    _fields_ = [
        ("type", C.c_int32),
        ("nviews", C.c_int32), ("nrows", C.c_int32), ("ncols", C.c_int32),
        ("nx", C.c_int32), ("ny", C.c_int32), ("nz", C.c_int32),
        ("pixel_v", C.c_double), ("pixel_u", C.c_double),
        ("shift_v", C.c_double), ("shift_u", C.c_double),
        ("sod", C.c_double), ("sdd", C.c_double),
        ("voxel_xy", C.c_double), ("voxel_z", C.c_double),
        ("center_x", C.c_double), ("center_y", C.c_double), ("center_z", C.c_double),
        ("angles_rad", C.POINTER(C.c_double)),
        ("model", C.c_int32),
        ("poses", C.POINTER(C.c_double)),
    ]


class LeapError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"leap status {status}: {message}")
        self.status = status


_lib = None


def declare(lib, solvers: bool = True) -> None:
    """Attach the prototypes of include/leap.h to a loaded library (solvers=False: the entry points of the geometry module
    only, for test builds that link it without the kernel launchers)."""
    lib.leap_geometry_create.restype = C.c_int
    lib.leap_geometry_create.argtypes = [C.POINTER(leap_geometry_desc), C.POINTER(C.c_void_p)]
    lib.leap_geometry_destroy.restype = None
    lib.leap_geometry_destroy.argtypes = [C.c_void_p]
    for fn in (lib.leap_project, lib.leap_backproject) + ((lib.leap_project_static_scratch,) if solvers else ()):
        fn.restype = C.c_int
        fn.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
    for fn in (lib.leap_project_host, lib.leap_backproject_host):
        fn.restype = C.c_int
        fn.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
    if solvers:
        lib.leap_recon_workspace_floats.restype = C.c_int
        lib.leap_recon_workspace_floats.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
        lib.leap_sirt.restype = C.c_int
        lib.leap_sirt.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_int32,
                                  C.c_void_p]
        lib.leap_least_squares_descent.restype = C.c_int
        lib.leap_least_squares_descent.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
    lib.leap_status_string.restype = C.c_char_p
    lib.leap_status_string.argtypes = [C.c_int]
    lib.leap_last_error.restype = C.c_char_p
    lib.leap_last_error.argtypes = []
    lib.leap_geometry_describe.restype = C.c_int
    lib.leap_geometry_describe.argtypes = [C.c_void_p, C.c_char_p, C.c_int32]


def load_library(path: Optional[str] = None):
    """Loads libleap_hip.so.  There is no fallback: a missing library is an error."""
    global _lib
    if path is None and _lib is not None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError(
            f"{p} is missing: build it first (python -m paper_2307_05801_amd.build or __graft_entry__.build()); "
            "this package has no CPU or PyTorch fallback")
    lib = C.CDLL(p)
    declare(lib)
    if path is None:
        _lib = lib
    return lib


def _check(lib, status: int) -> None:
    if status != LEAP_OK:
        detail = lib.leap_last_error().decode() or lib.leap_status_string(status).decode()
        raise LeapError(status, detail)


def make_desc(*, type: int, nviews: int, nrows: int, ncols: int, nx: int, ny: int, nz: int,
              pixel_v: float, pixel_u: float, voxel_xy: float, voxel_z: float, angles_rad: Sequence[float],
              shift_v: float = 0.0, shift_u: float = 0.0, sod: float = 0.0, sdd: float = 0.0,
              center_x: float = 0.0, center_y: float = 0.0, center_z: float = 0.0, model: int = LEAP_MODEL_SF,
              poses=None):
    """(desc, keep-alive) from keyword arguments named like the C struct's fields; poses: nviews rows of 12 numbers."""
    ang = (C.c_double * len(angles_rad))(*[float(a) for a in angles_rad])
    if len(angles_rad) != nviews:
        raise ValueError("angles_rad must hold nviews entries")
    pp, flat = C.POINTER(C.c_double)(), None
    if poses is not None:
        vals = [float(v) for row in poses for v in row]
        if len(vals) != 12 * nviews:
            raise ValueError("poses must hold nviews rows of 12 numbers")
        flat = (C.c_double * len(vals))(*vals)
        pp = C.cast(flat, C.POINTER(C.c_double))
    d = leap_geometry_desc(type, nviews, nrows, ncols, nx, ny, nz, pixel_v, pixel_u, shift_v, shift_u,
                           sod, sdd, voxel_xy, voxel_z, center_x, center_y, center_z,
                           C.cast(ang, C.POINTER(C.c_double)), model, pp)
    return d, (ang, flat)


def desc_from_config(cfg, model: int = LEAP_MODEL_SF):
    """(desc, keep-alive) from an object with the fields of synthetic.CTConfig."""
    return make_desc(type=cfg.geom, nviews=cfg.nviews, nrows=cfg.nrows, ncols=cfg.ncols, nx=cfg.nx, ny=cfg.ny,
                     nz=cfg.nz, pixel_v=cfg.pixel_v, pixel_u=cfg.pixel_u, voxel_xy=cfg.voxel_xy,
                     voxel_z=cfg.voxel_z, angles_rad=list(cfg.angles()), shift_v=cfg.shift_v, shift_u=cfg.shift_u,
                     sod=cfg.sod, sdd=cfg.sdd, center_x=cfg.center_x, center_y=cfg.center_y, center_z=cfg.center_z,
                     model=model, poses=getattr(cfg, "poses", None) if cfg.geom == LEAP_MODULAR else None)


def leap_geometry_create(desc: leap_geometry_desc, lib=None) -> int:
    """Returns the opaque handle (an integer address).  Needs a current HIP device."""
    lib = lib or load_library()
    handle = C.c_void_p()
    _check(lib, lib.leap_geometry_create(C.byref(desc), C.byref(handle)))
    return handle.value


def leap_geometry_destroy(handle: int, lib=None) -> None:
    lib = lib or load_library()
    lib.leap_geometry_destroy(C.c_void_p(handle))


def leap_geometry_describe(handle: int, lib=None) -> str:
    lib = lib or load_library()
    buf = C.create_string_buffer(256)
    _check(lib, lib.leap_geometry_describe(C.c_void_p(handle), buf, 256))
    return buf.value.decode()


def leap_project(handle: int, d_vol: int, d_sino: int, batch: int, stream: int = 0, lib=None) -> None:
    """d_vol, d_sino: device addresses (tensor.data_ptr()); stream: hipStream_t as an integer."""
    lib = lib or load_library()
    _check(lib, lib.leap_project(C.c_void_p(handle), C.c_void_p(d_vol), C.c_void_p(d_sino), batch, C.c_void_p(stream)))


def leap_project_static_scratch(handle: int, d_vol: int, d_sino: int, batch: int, stream: int = 0, lib=None) -> None:
    """leap_project on the library's fixed scratch array (allocates nothing; see include/leap.h for its limits)."""
    lib = lib or load_library()
    _check(lib, lib.leap_project_static_scratch(C.c_void_p(handle), C.c_void_p(d_vol), C.c_void_p(d_sino), batch,
                                                C.c_void_p(stream)))


def leap_project_host(handle: int, h_vol: int, h_sino: int, batch: int, lib=None) -> None:
    """h_vol, h_sino: HOST addresses (numpy `.ctypes.data`, a pinned tensor's data_ptr()); returns when h_sino is written."""
    lib = lib or load_library()
    _check(lib, lib.leap_project_host(C.c_void_p(handle), C.c_void_p(h_vol), C.c_void_p(h_sino), batch))


def leap_backproject_host(handle: int, h_sino: int, h_vol: int, batch: int, lib=None) -> None:
    lib = lib or load_library()
    _check(lib, lib.leap_backproject_host(C.c_void_p(handle), C.c_void_p(h_sino), C.c_void_p(h_vol), batch))


def leap_backproject(handle: int, d_sino: int, d_vol: int, batch: int, stream: int = 0, lib=None) -> None:
    lib = lib or load_library()
    _check(lib, lib.leap_backproject(C.c_void_p(handle), C.c_void_p(d_sino), C.c_void_p(d_vol), batch, C.c_void_p(stream)))


def leap_recon_workspace_floats(handle: int, lib=None) -> int:
    lib = lib or load_library()
    n = C.c_int64()
    _check(lib, lib.leap_recon_workspace_floats(C.c_void_p(handle), C.byref(n)))
    return n.value


def leap_sirt(handle: int, d_sino: int, d_vol: int, d_work: int, iterations: int, relaxation: float = 1.0,
              nonneg: bool = False, stream: int = 0, lib=None) -> None:
    lib = lib or load_library()
    _check(lib, lib.leap_sirt(C.c_void_p(handle), C.c_void_p(d_sino), C.c_void_p(d_vol), C.c_void_p(d_work), iterations,
                              relaxation, int(bool(nonneg)), C.c_void_p(stream)))


def leap_least_squares_descent(handle: int, d_sino: int, d_vol: int, d_work: int, iterations: int, stream: int = 0,
                               lib=None) -> None:
    lib = lib or load_library()
    _check(lib, lib.leap_least_squares_descent(C.c_void_p(handle), C.c_void_p(d_sino), C.c_void_p(d_vol),
                                               C.c_void_p(d_work), iterations, C.c_void_p(stream)))
