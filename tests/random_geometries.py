"""Seeded random scanner set-ups for fuzzing kernel selection, window limits and parity (sizes the oracle finishes
in about a second)."""
import numpy as np

from synthetic import CTConfig, perturbed_poses
from synthetic.configs import CONE, PARALLEL


def random_config(seed: int) -> CTConfig:
    rng = np.random.default_rng([777, seed])
    geom = CONE if rng.random() < 0.7 else PARALLEL
    nx, ny, nz = (int(rng.integers(9, 72)) for _ in range(3))
    voxel_xy = float(rng.uniform(0.3, 2.0))
    voxel_z = float(voxel_xy * rng.uniform(0.5, 2.0))
    half_diag = 0.5 * voxel_xy * float(np.hypot(nx, ny))
    cx, cy = (float(rng.uniform(-0.15, 0.15) * half_diag) for _ in range(2))
    cz = float(rng.uniform(-0.2, 0.2) * nz * voxel_z)
    reach = half_diag + float(np.hypot(cx, cy))
    sod = float(reach * rng.uniform(1.6, 8.0))
    sdd = float(sod * rng.uniform(1.1, 2.5))
    mag = sdd / sod if geom == CONE else 1.0
    pixel_u = float(voxel_xy * mag * rng.uniform(0.45, 2.5))
    pixel_v = float(voxel_z * mag * rng.uniform(0.45, 2.5))
    # detector somewhat smaller or larger than the shadow, sometimes shifted
    ncols = int(np.clip(2 * reach * mag / pixel_u * rng.uniform(0.6, 1.3), 8, 160))
    nrows = int(np.clip(nz * voxel_z * mag / pixel_v * rng.uniform(0.6, 1.4), 4, 160))
    if seed % 3:                       # two thirds of the cases: enough rows for the column-wise forward kernel
        nrows = max(nrows, int(rng.integers(32, 100)))
    shift_u = float(rng.uniform(-3, 3)) if rng.random() < 0.5 else 0.0
    shift_v = float(rng.uniform(-3, 3)) if rng.random() < 0.5 else 0.0
    nviews = int(rng.integers(3, 14))
    angles = tuple(float(a) for a in np.sort(rng.uniform(0.0, 2 * np.pi, nviews)))
    return CTConfig(f"random_{seed}", geom, nviews=nviews, arc_deg=360.0, nrows=nrows, ncols=ncols, pixel_v=pixel_v,
                    pixel_u=pixel_u, nx=nx, ny=ny, nz=nz, voxel_xy=voxel_xy, voxel_z=voxel_z, sod=sod, sdd=sdd,
                    shift_v=shift_v, shift_u=shift_u, center_x=cx, center_y=cy, center_z=cz, angles_override=angles)


def random_tilted_scan(seed: int) -> CTConfig:
    """A modular scan with tilted modules (up to 0.5 rad about every axis) whose sources keep more than a hundred voxels
    from the volume: random shifts, voxel aspect ratios and sizes."""
    rng = np.random.default_rng([seed, 91])
    base = CTConfig("far", CONE, nviews=5, arc_deg=360.0, nrows=48, ncols=56, pixel_v=1.5, pixel_u=1.5,
                    nx=int(rng.integers(17, 40)), ny=int(rng.integers(17, 40)), nz=int(rng.integers(9, 34)), voxel_xy=1.0,
                    voxel_z=float(rng.uniform(0.6, 1.8)), sod=160.0, sdd=240.0, shift_u=float(rng.uniform(-2, 2)),
                    shift_v=float(rng.uniform(-2, 2)), center_x=1.0, center_y=-2.0, center_z=0.5, start_deg=3.0)
    return perturbed_poses(base, 100 + seed, shift_mm=float(rng.uniform(0, 12)), tilt_rad=float(rng.uniform(0.02, 0.5)))
