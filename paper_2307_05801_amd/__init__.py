"""MI355X-native separable-footprint CT projector pair (forward A, matched transpose A^T).

The compute path is the HIP library libleap_hip.so (C ABI in include/leap.h); this package only
marshals arguments.  There is no CPU or PyTorch fallback: a missing library raises.
"""
from .binding import (  # noqa: F401
    LEAP_PARALLEL, LEAP_FAN, LEAP_CONE, LeapError, leap_geometry_desc, make_desc, desc_from_config, load_library,
    leap_geometry_create, leap_geometry_destroy, leap_geometry_describe, leap_project, leap_backproject,
)


def __getattr__(name):
    # torch is imported only when the tensor-level classes are asked for
    if name in ("Geometry", "Projector"):
        from . import projector
        return getattr(projector, name)
    raise AttributeError(name)
