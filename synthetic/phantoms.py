"""Seeded random phantoms and random test vectors (float32).

Recipe (fixed draw order, numpy.random.default_rng):
  stream [seed, 0]  ellipsoid parameters; per ellipsoid, in this order:
                    centre (x, y[, z]) ~ U over the inner 70 % of each field axis,
                    semi-axes ~ U[lo, hi] (one per axis),
                    orientation: 2-D an angle ~ U[0, pi); 3-D a quaternion of 4 standard
                    normals, normalised,
                    density ~ U[rho_lo, rho_hi].
  stream [seed, 1]  additive per-voxel Gaussian noise (when asked for).
  stream [seed, 2]  uniform [0,1) test sinograms;  stream [seed, 3]  uniform [0,1) test volumes.

An ellipsoid adds its density to every voxel whose CENTRE lies inside it
(no anti-aliasing).  World coordinates of voxel centres follow
x_i = center_x + (i - (nx-1)/2) * voxel_xy, likewise y and z; arrays are
[z][y][x], x fastest.
"""
from __future__ import annotations

import dataclasses
from typing import List, Sequence

import numpy as np

from .configs import CTConfig


@dataclasses.dataclass(frozen=True)
class Ellipsoid:
    center: tuple      # (x, y, z) mm
    semi: tuple        # (a, b, c) mm, along the columns of `rot`
    rot: tuple         # 3x3 row-major rotation matrix, columns are the axes' directions
    rho: float         # additive density (1/mm)

    def quadric(self) -> np.ndarray:
        """Q with (X-c)^T Q (X-c) <= 1 inside."""
        r = np.asarray(self.rot, dtype=np.float64).reshape(3, 3)
        d = np.diag(1.0 / np.asarray(self.semi, dtype=np.float64) ** 2)
        return r @ d @ r.T


def _field(cfg: CTConfig):
    return (cfg.nx * cfg.voxel_xy, cfg.ny * cfg.voxel_xy, cfg.nz * cfg.voxel_z)


def draw_ellipses_2d(cfg: CTConfig, seed: int, count: int, semi_range, rho_range) -> List[Ellipsoid]:
    """In-plane ellipses extruded along z (third semi-axis effectively infinite)."""
    rng = np.random.default_rng([seed, 0])
    fx, fy, _ = _field(cfg)
    out = []
    for _ in range(count):
        cx = cfg.center_x + rng.uniform(-0.35, 0.35) * fx
        cy = cfg.center_y + rng.uniform(-0.35, 0.35) * fy
        a = rng.uniform(*semi_range)
        b = rng.uniform(*semi_range)
        th = rng.uniform(0.0, np.pi)
        rho = rng.uniform(*rho_range)
        c, s = np.cos(th), np.sin(th)
        rot = (c, -s, 0.0, s, c, 0.0, 0.0, 0.0, 1.0)
        out.append(Ellipsoid((cx, cy, cfg.center_z), (a, b, 1e9), rot, rho))
    return out


def draw_ellipsoids_3d(cfg: CTConfig, seed: int, count: int, semi_range, rho_range) -> List[Ellipsoid]:
    rng = np.random.default_rng([seed, 0])
    fx, fy, fz = _field(cfg)
    out = []
    for _ in range(count):
        cx = cfg.center_x + rng.uniform(-0.35, 0.35) * fx
        cy = cfg.center_y + rng.uniform(-0.35, 0.35) * fy
        cz = cfg.center_z + rng.uniform(-0.35, 0.35) * fz
        semi = tuple(rng.uniform(*semi_range) for _ in range(3))
        q = rng.standard_normal(4)
        q /= np.linalg.norm(q)
        w, x, y, z = q
        rot = (1 - 2 * (y * y + z * z), 2 * (x * y - z * w), 2 * (x * z + y * w),
               2 * (x * y + z * w), 1 - 2 * (x * x + z * z), 2 * (y * z - x * w),
               2 * (x * z - y * w), 2 * (y * z + x * w), 1 - 2 * (x * x + y * y))
        rho = rng.uniform(*rho_range)
        out.append(Ellipsoid((cx, cy, cz), semi, rot, rho))
    return out


def rasterize(cfg: CTConfig, ellipsoids: Sequence[Ellipsoid]) -> np.ndarray:
    """Sum of densities of the ellipsoids containing each voxel centre, float32 [nz][ny][nx]."""
    vol = np.zeros(cfg.vol_shape, dtype=np.float32)
    xs = cfg.center_x + (np.arange(cfg.nx) - (cfg.nx - 1) / 2.0) * cfg.voxel_xy
    ys = cfg.center_y + (np.arange(cfg.ny) - (cfg.ny - 1) / 2.0) * cfg.voxel_xy
    zs = cfg.center_z + (np.arange(cfg.nz) - (cfg.nz - 1) / 2.0) * cfg.voxel_z
    for e in ellipsoids:
        q = e.quadric()
        # half extents of the axis-aligned bounding box: sqrt of the diagonal of Q^{-1}
        r = np.asarray(e.rot, dtype=np.float64).reshape(3, 3)
        ext = np.sqrt(np.sum((r * np.asarray(e.semi)[None, :]) ** 2, axis=1))
        c = np.asarray(e.center)
        ix = np.nonzero(np.abs(xs - c[0]) <= ext[0])[0]
        iy = np.nonzero(np.abs(ys - c[1]) <= ext[1])[0]
        iz = np.nonzero(np.abs(zs - c[2]) <= ext[2])[0]
        if len(ix) == 0 or len(iy) == 0 or len(iz) == 0:
            continue
        dx = (xs[ix[0]:ix[-1] + 1] - c[0])[None, :]
        dy = (ys[iy[0]:iy[-1] + 1] - c[1])[:, None]
        # in-plane part once, then one z-slice at a time to bound memory
        pxy = q[0, 0] * dx * dx + 2 * q[0, 1] * dx * dy + q[1, 1] * dy * dy
        lxy_x = 2 * q[0, 2] * dx
        lxy_y = 2 * q[1, 2] * dy
        rho = np.float32(e.rho)
        for k in range(iz[0], iz[-1] + 1):
            dz = zs[k] - c[2]
            inside = (pxy + (lxy_x + lxy_y) * dz + q[2, 2] * dz * dz) <= 1.0
            sub = vol[k, iy[0]:iy[-1] + 1, ix[0]:ix[-1] + 1]
            sub[inside] += rho
    return vol


def make_volume(cfg: CTConfig, seed: int, count: int, semi_range, rho_range, *, two_d=False,
                noise_sigma: float = 0.0, clip_min=None) -> np.ndarray:
    draw = draw_ellipses_2d if two_d else draw_ellipsoids_3d
    vol = rasterize(cfg, draw(cfg, seed, count, semi_range, rho_range))
    if noise_sigma > 0.0:
        rng = np.random.default_rng([seed, 1])
        for k in range(cfg.nz):                 # slice-wise: same values as one big draw, less memory
            vol[k] += rng.standard_normal((cfg.ny, cfg.nx), dtype=np.float32) * np.float32(noise_sigma)
    if clip_min is not None:
        np.maximum(vol, np.float32(clip_min), out=vol)
    return vol


def standard_volume(cfg_number: int, cfg: CTConfig, item: int = 0) -> np.ndarray:
    """The phantom of benchmark case `cfg_number`, rasterised on `cfg`'s grid (full or reduced)."""
    seed = 1000 + cfg_number + 100 * item
    if cfg_number == 1:
        return make_volume(cfg, seed, 10, (4.0, 24.0), (-0.3, 1.0), two_d=True, clip_min=0.0)
    if cfg_number == 2:
        return make_volume(cfg, seed, 20, (8.0, 80.0), (0.0, 1.0))
    if cfg_number == 3:
        return make_volume(cfg, seed, 30, (8.0, 80.0), (0.0, 0.05), noise_sigma=1e-4)
    if cfg_number == 4:
        return make_volume(cfg, seed, 20, (8.0, 80.0), (0.0, 0.02))
    if cfg_number == 5:
        return make_volume(cfg, seed, 50, (8.0, 80.0), (0.0, 0.05))
    raise ValueError(cfg_number)


def uniform_sinogram(cfg: CTConfig, seed: int, batch: int = 1) -> np.ndarray:
    rng = np.random.default_rng([seed, 2])
    return rng.random((batch,) + cfg.sino_shape, dtype=np.float32)


def uniform_volume(cfg: CTConfig, seed: int, batch: int = 1) -> np.ndarray:
    rng = np.random.default_rng([seed, 3])
    return rng.random((batch,) + cfg.vol_shape, dtype=np.float32)


def measured_sinogram(ideal: np.ndarray, seed: int, photons: float = 1e5) -> np.ndarray:
    """Photon-counting measurement of ideal line integrals (input preparation of the training-step case):
    counts ~ Poisson(photons * exp(-ideal)), y = -ln(max(counts, 1) / photons).  Stream [seed, 4]."""
    rng = np.random.default_rng([seed, 4])
    counts = rng.poisson(photons * np.exp(-np.asarray(ideal, dtype=np.float64)))
    return (-np.log(np.maximum(counts, 1) / photons)).astype(np.float32)


def perturbed_volume(vol: np.ndarray, seed: int, sigma: float = 1e-3) -> np.ndarray:
    """Current estimate of the training-step case: the phantom plus N(0, sigma) per voxel.  Stream [seed, 5]."""
    rng = np.random.default_rng([seed, 5])
    return (vol + rng.standard_normal(vol.shape, dtype=np.float32) * np.float32(sigma)).astype(np.float32)
