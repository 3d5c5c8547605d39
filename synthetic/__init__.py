"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

Holds workload descriptions (scanner parameters, array shapes) and random
phantoms only.  Nothing here evaluates a projector weight, a footprint or a
line integral: the method's arithmetic lives in the oracle and in the HIP
library, separately.
"""
from .configs import CTConfig, CONFIGS, config, reduced, modular_from, perturbed_poses  # noqa: F401
from .phantoms import (  # noqa: F401
    Ellipsoid,
    draw_ellipses_2d,
    draw_ellipsoids_3d,
    rasterize,
    make_volume,
    standard_volume,
    uniform_sinogram,
    uniform_volume,
    measured_sinogram,
    perturbed_volume,
)
