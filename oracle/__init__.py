"""CPU oracles of the projector pairs: separable footprint (the functions of this package) and Siddon
(`oracle.siddon`).  Test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product (paper_2307_05801_amd) never does.
"""
from . import siddon_oracle as siddon  # noqa: F401
from .sf_oracle import build as _build_sf
from .sf_oracle import (  # noqa: F401
    project,
    backproject,
    backproject_voxels,
    project_rays,
    dense_matrix,
    nnz,
    weight,
    knots,
    trapezoid_integral,
    num_threads,
    set_num_threads,
)


def build(force: bool = False):
    """Compile both C oracles (gcc); returns the paths of the two libraries."""
    return _build_sf(force), siddon.build(force)
