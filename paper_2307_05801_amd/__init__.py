"""MI355X-native CT projector pairs (forward A, matched transpose A^T; separable-footprint and Siddon models).

The compute path is the HIP library libleap_hip.so (C ABI in include/leap.h); this package only
marshals arguments.  There is no CPU or PyTorch fallback: a missing library raises.
"""
from .binding import (  # noqa: F401
    LEAP_PARALLEL, LEAP_FAN, LEAP_CONE, LEAP_CONE_CURVED, LEAP_MODEL_SF, LEAP_MODEL_SIDDON, LeapError, leap_geometry_desc, make_desc, desc_from_config, load_library,
    leap_geometry_create, leap_geometry_destroy, leap_geometry_describe, leap_project, leap_backproject,
    leap_recon_workspace_floats, leap_sirt, leap_least_squares_descent,
)


def __getattr__(name):
    # torch is imported only when the tensor-level classes are asked for
    if name in ("Geometry", "Projector"):
        from . import projector
        return getattr(projector, name)
    if name == "recon":
        import importlib
        return importlib.import_module(".recon", __name__)
    raise AttributeError(name)
