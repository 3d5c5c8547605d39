"""Workload descriptions: scanner parameters and array shapes of the five benchmark cases.

A CTConfig is plain data (the CT parameter set the paper lists in its
"PyTorch Interfaces and CT Parameters" subsection).  Both the oracle wrapper
and the HIP binding translate it into their own structs.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np

PARALLEL, FAN, CONE, CONE_CURVED, MODULAR = 0, 1, 2, 3, 4
GEOM_NAMES = {PARALLEL: "parallel", FAN: "fan", CONE: "cone", CONE_CURVED: "cone_curved", MODULAR: "modular"}


@dataclasses.dataclass(frozen=True)
class CTConfig:
    name: str
    geom: int                 # PARALLEL / FAN / CONE (flat detector) / CONE_CURVED (cylindrical detector)
    nviews: int
    arc_deg: float            # views are a*arc/nviews, end point excluded
    nrows: int
    ncols: int
    pixel_v: float            # mm, detector pixel height
    pixel_u: float            # mm, detector pixel width
    nx: int
    ny: int
    nz: int
    voxel_xy: float           # mm
    voxel_z: float            # mm
    sod: float = 0.0          # mm, source to rotation axis (ignored for parallel)
    sdd: float = 0.0          # mm, source to detector     (ignored for parallel)
    shift_v: float = 0.0      # detector shift in pixels, + moves pixel centres to +v
    shift_u: float = 0.0      # detector shift in pixels, + moves pixel centres to +u
    center_x: float = 0.0     # mm, volume centre
    center_y: float = 0.0
    center_z: float = 0.0
    batch: int = 1
    start_deg: float = 0.0
    angles_override: Optional[tuple] = None   # explicit radian list (non-equispaced views)
    poses: Optional[tuple] = None             # MODULAR only: per view (S[3], C[3], ucol[3], vrow[3]) as 12 floats

    def angles(self) -> np.ndarray:
        if self.angles_override is not None:
            return np.asarray(self.angles_override, dtype=np.float64)
        a = np.arange(self.nviews, dtype=np.float64)
        return np.deg2rad(self.start_deg + a * (self.arc_deg / self.nviews))

    @property
    def vol_shape(self):
        return (self.nz, self.ny, self.nx)

    @property
    def sino_shape(self):
        return (self.nviews, self.nrows, self.ncols)

    @property
    def voxel_views(self) -> int:
        """Voxel-view pairs of one batch item (the usual projector update count)."""
        return self.nviews * self.nx * self.ny * self.nz

    def with_views(self, view_indices) -> "CTConfig":
        """Same scanner, only the listed views (a subset is just another angle list)."""
        ang = self.angles()[np.asarray(view_indices, dtype=np.int64)]
        poses = None if self.poses is None else tuple(self.poses[int(v)] for v in view_indices)
        return dataclasses.replace(self, nviews=len(ang), angles_override=tuple(float(v) for v in ang), poses=poses)

    def replace(self, **kw) -> "CTConfig":
        return dataclasses.replace(self, **kw)


CONFIGS = {
    # 2D parallel-beam: one slice, one detector row.
    1: CTConfig("c1_parallel2d_64", PARALLEL, nviews=90, arc_deg=180.0, nrows=1, ncols=96,
                pixel_v=1.0, pixel_u=1.0, nx=64, ny=64, nz=1, voxel_xy=1.0, voxel_z=1.0),
    2: CTConfig("c2_parallel3d_256", PARALLEL, nviews=180, arc_deg=180.0, nrows=256, ncols=256,
                pixel_v=1.0, pixel_u=1.0, nx=256, ny=256, nz=256, voxel_xy=1.0, voxel_z=1.0),
    3: CTConfig("c3_cone_512", CONE, nviews=720, arc_deg=360.0, nrows=512, ncols=512,
                pixel_v=1.0, pixel_u=1.0, nx=512, ny=512, nz=512, voxel_xy=0.5, voxel_z=0.5,
                sod=1000.0, sdd=1500.0),
    4: CTConfig("c4_cone_limited_batch8_256", CONE, nviews=60, arc_deg=90.0, nrows=384, ncols=384,
                pixel_v=1.2, pixel_u=1.2, nx=256, ny=256, nz=256, voxel_xy=1.0, voxel_z=1.0,
                sod=600.0, sdd=1000.0, batch=8),
    5: CTConfig("c5_cone_1024", CONE, nviews=1440, arc_deg=360.0, nrows=1024, ncols=1024,
                pixel_v=0.4, pixel_u=0.4, nx=1024, ny=1024, nz=1024, voxel_xy=0.25, voxel_z=0.25,
                sod=800.0, sdd=1200.0, shift_u=2.5),
}


def config(n: int) -> CTConfig:
    return CONFIGS[n]


def reduced(cfg: CTConfig, factor: int, nviews: Optional[int] = None, batch: Optional[int] = None) -> CTConfig:
    """Same physical scanner sampled `factor` times coarser (fewer, larger voxels and pixels).

    Used for parity cases the oracle finishes in seconds.  Detector shifts stay
    the same physical distance, so they shrink in pixel units.
    """
    def div(n):
        return max(1, int(math.ceil(n / factor)))
    return dataclasses.replace(
        cfg,
        name=f"{cfg.name}_div{factor}",
        nviews=cfg.nviews if nviews is None else nviews,
        nrows=div(cfg.nrows), ncols=div(cfg.ncols),
        pixel_v=cfg.pixel_v * factor, pixel_u=cfg.pixel_u * factor,
        nx=div(cfg.nx), ny=div(cfg.ny), nz=div(cfg.nz),
        voxel_xy=cfg.voxel_xy * factor, voxel_z=cfg.voxel_z * factor,
        shift_u=cfg.shift_u / factor, shift_v=cfg.shift_v / factor,
        batch=cfg.batch if batch is None else batch,
    )


def modular_from(cfg: CTConfig) -> CTConfig:
    """The flat-panel cone-beam scan `cfg` written as a modular one: the same sources, detector centres and axes, view
    by view (a description of the scanner, no projector arithmetic)."""
    assert cfg.geom == CONE
    poses = []
    for phi in cfg.angles():
        es = np.array([np.cos(phi), np.sin(phi), 0.0])
        eu = np.array([-np.sin(phi), np.cos(phi), 0.0])
        ev = np.array([0.0, 0.0, 1.0])
        poses.append(tuple(float(v) for v in np.concatenate([cfg.sod * es, (cfg.sod - cfg.sdd) * es, eu, ev])))
    return cfg.replace(geom=MODULAR, name=cfg.name + "_modular", poses=tuple(poses))


def perturbed_poses(cfg: CTConfig, seed: int, shift_mm: float = 3.0, tilt_rad: float = 0.08, upright: bool = False) -> CTConfig:
    """A modular scan near `cfg` (cone-beam or modular): every view's source and detector centre moved by up to
    shift_mm per axis and the detector rotated by up to tilt_rad about each of its own axes and its normal
    (upright=True: about the vertical only, and no vertical component in the column axis)."""
    base = cfg if cfg.geom == MODULAR else modular_from(cfg)
    rng = np.random.default_rng([seed, 6])
    out = []
    for p in base.poses:
        p = np.asarray(p, dtype=np.float64)
        S, C, eu, ev = p[0:3].copy(), p[3:6].copy(), p[6:9].copy(), p[9:12].copy()
        S += rng.uniform(-shift_mm, shift_mm, 3)
        C += rng.uniform(-shift_mm, shift_mm, 3)
        n = np.cross(eu, ev)
        angles = rng.uniform(-tilt_rad, tilt_rad, 3)
        axes = [ev] if upright else [ev, eu, n]
        for axis, ang in zip(axes, angles):
            k = axis / np.linalg.norm(axis)
            rot = lambda w: w * np.cos(ang) + np.cross(k, w) * np.sin(ang) + k * np.dot(k, w) * (1 - np.cos(ang))
            eu, ev = rot(eu), rot(ev)
        ev = ev - np.dot(ev, eu) * eu
        eu, ev = eu / np.linalg.norm(eu), ev / np.linalg.norm(ev)
        out.append(tuple(float(v) for v in np.concatenate([S, C, eu, ev])))
    return base.replace(name=base.name + f"_perturbed{seed}", poses=tuple(out))
