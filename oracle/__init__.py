"""CPU oracle of the separable-footprint projector pair.  Test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product (paper_2307_05801_amd) never does.
"""
from .sf_oracle import (  # noqa: F401
    build,
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
