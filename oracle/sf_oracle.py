"""ctypes front end of the C oracle (oracle/sf_oracle.c).  Test infrastructure only.

Marshals a synthetic.CTConfig into the oracle's own struct and numpy arrays into
pointers; no arithmetic of the method happens here.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sf_oracle.c")
_HDR = os.path.join(_HERE, "sf_oracle.h")
_LIB = os.path.join(_HERE, "libsf_oracle.so")
_lock = threading.Lock()
_lib = None


class _Scan(C.Structure):
    _fields_ = [
        ("geom", C.c_int32),
        ("nviews", C.c_int32), ("nrows", C.c_int32), ("ncols", C.c_int32),
        ("nx", C.c_int32), ("ny", C.c_int32), ("nz", C.c_int32),
        ("pu", C.c_double), ("pv", C.c_double),
        ("shift_u", C.c_double), ("shift_v", C.c_double),
        ("sod", C.c_double), ("sdd", C.c_double),
        ("T", C.c_double), ("Tz", C.c_double),
        ("cx", C.c_double), ("cy", C.c_double), ("cz", C.c_double),
        ("phi", C.POINTER(C.c_double)),
        ("poses", C.POINTER(C.c_double)),
    ]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP, -O2, strict IEEE: no fast-math)."""
    stale = (not os.path.exists(_LIB)) or any(
        os.path.getmtime(p) > os.path.getmtime(_LIB) for p in (_SRC, _HDR))
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = C.CDLL(build())
            dp, fp, ip = C.POINTER(C.c_double), C.POINTER(C.c_float), C.POINTER(C.c_int64)
            sp = C.POINTER(_Scan)
            lib.sfo_weight.restype = C.c_double
            lib.sfo_weight.argtypes = [sp] + [C.c_int] * 6 + [dp, dp, dp]
            lib.sfo_knots.restype = None
            lib.sfo_knots.argtypes = [sp, C.c_int, C.c_int, C.c_int, dp, dp]
            lib.sfo_trapezoid_integral.restype = C.c_double
            lib.sfo_trapezoid_integral.argtypes = [dp, C.c_double]
            lib.sfo_project.argtypes = [sp, fp, dp]
            lib.sfo_backproject.argtypes = [sp, fp, dp]
            lib.sfo_backproject_voxels.argtypes = [sp, fp, C.c_int64, ip, dp]
            lib.sfo_project_rays.argtypes = [sp, fp, C.c_int64, ip, dp]
            lib.sfo_dense_matrix.argtypes = [sp, dp]
            lib.sfo_nnz.restype = C.c_int64
            lib.sfo_nnz.argtypes = [sp, C.c_int, C.c_int]
            lib.sfo_num_threads.restype = C.c_int
            lib.sfo_set_num_threads.argtypes = [C.c_int]
            _lib = lib
    return _lib


def _scan(cfg):
    """(struct, keep-alive) for a synthetic.CTConfig-like object."""
    phi = np.ascontiguousarray(cfg.angles(), dtype=np.float64)
    assert phi.shape == (cfg.nviews,)
    poses = None
    if cfg.geom == 4:
        poses = np.ascontiguousarray(cfg.poses, dtype=np.float64).reshape(cfg.nviews, 12)
        pp = poses.ctypes.data_as(C.POINTER(C.c_double))
    else:
        pp = C.POINTER(C.c_double)()
    s = _Scan(cfg.geom, cfg.nviews, cfg.nrows, cfg.ncols, cfg.nx, cfg.ny, cfg.nz,
              cfg.pixel_u, cfg.pixel_v, cfg.shift_u, cfg.shift_v, cfg.sod, cfg.sdd,
              cfg.voxel_xy, cfg.voxel_z, cfg.center_x, cfg.center_y, cfg.center_z,
              phi.ctypes.data_as(C.POINTER(C.c_double)), pp)
    return s, (phi, poses)


def _f32(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def project(cfg, vol) -> np.ndarray:
    """A x for one volume [nz][ny][nx] (float32 in, float64 out [nviews][nrows][ncols])."""
    lib = _load()
    s, _keep = _scan(cfg)
    vol = _f32(vol, cfg.vol_shape)
    out = np.empty(cfg.sino_shape, dtype=np.float64)
    rc = lib.sfo_project(C.byref(s), _ptr(vol, C.c_float), _ptr(out, C.c_double))
    assert rc == 0
    return out


def backproject(cfg, sino) -> np.ndarray:
    """A^T y for one sinogram (float32 in, float64 out [nz][ny][nx])."""
    lib = _load()
    s, _keep = _scan(cfg)
    sino = _f32(sino, cfg.sino_shape)
    out = np.empty(cfg.vol_shape, dtype=np.float64)
    rc = lib.sfo_backproject(C.byref(s), _ptr(sino, C.c_float), _ptr(out, C.c_double))
    assert rc == 0
    return out


def backproject_voxels(cfg, sino, voxel_index) -> np.ndarray:
    """A^T y at the listed linear voxel indices ((k*ny+j)*nx+i)."""
    lib = _load()
    s, _keep = _scan(cfg)
    sino = _f32(sino, cfg.sino_shape)
    idx = np.ascontiguousarray(voxel_index, dtype=np.int64)
    assert idx.ndim == 1 and (idx >= 0).all() and (idx < cfg.nx * cfg.ny * cfg.nz).all()
    out = np.empty(idx.shape, dtype=np.float64)
    rc = lib.sfo_backproject_voxels(C.byref(s), _ptr(sino, C.c_float), idx.size, _ptr(idx, C.c_int64),
                                    _ptr(out, C.c_double))
    assert rc == 0
    return out


def project_rays(cfg, vol, ray_index) -> np.ndarray:
    """A x at the listed linear ray indices ((view*nrows+r)*ncols+c)."""
    lib = _load()
    s, _keep = _scan(cfg)
    vol = _f32(vol, cfg.vol_shape)
    idx = np.ascontiguousarray(ray_index, dtype=np.int64)
    assert idx.ndim == 1 and (idx >= 0).all() and (idx < cfg.nviews * cfg.nrows * cfg.ncols).all()
    out = np.empty(idx.shape, dtype=np.float64)
    rc = lib.sfo_project_rays(C.byref(s), _ptr(vol, C.c_float), idx.size, _ptr(idx, C.c_int64),
                              _ptr(out, C.c_double))
    assert rc == 0
    return out


def dense_matrix(cfg) -> np.ndarray:
    """Dense A [nrays][nvoxels], every pair evaluated from the single-weight routine."""
    lib = _load()
    s, _keep = _scan(cfg)
    m = cfg.nviews * cfg.nrows * cfg.ncols
    n = cfg.nx * cfg.ny * cfg.nz
    assert m * n <= 50_000_000, "dense matrix is for tiny grids"
    out = np.empty((m, n), dtype=np.float64)
    rc = lib.sfo_dense_matrix(C.byref(s), _ptr(out, C.c_double))
    assert rc == 0
    return out


def nnz(cfg, view_begin: int = 0, view_end=None) -> int:
    lib = _load()
    s, _keep = _scan(cfg)
    if view_end is None:
        view_end = cfg.nviews
    return int(lib.sfo_nnz(C.byref(s), view_begin, view_end))


def weight(cfg, view, r, c, i, j, k):
    """(w, F_u, F_v, amp) of one ray-voxel pair."""
    lib = _load()
    s, _keep = _scan(cfg)
    fu, fv, am = C.c_double(), C.c_double(), C.c_double()
    w = lib.sfo_weight(C.byref(s), view, r, c, i, j, k, C.byref(fu), C.byref(fv), C.byref(am))
    return w, fu.value, fv.value, am.value


def knots(cfg, view, i, j):
    """(tau[4] sorted, magnification) of voxel column (i,j) in a view."""
    lib = _load()
    s, _keep = _scan(cfg)
    tau = (C.c_double * 4)()
    mag = C.c_double()
    lib.sfo_knots(C.byref(s), view, i, j, tau, C.byref(mag))
    return np.array(list(tau)), mag.value


def trapezoid_integral(tau, u) -> float:
    lib = _load()
    t = (C.c_double * 4)(*[float(v) for v in tau])
    return float(lib.sfo_trapezoid_integral(t, float(u)))


def num_threads() -> int:
    return int(_load().sfo_num_threads())


def set_num_threads(n: int) -> None:
    _load().sfo_set_num_threads(int(n))
