"""Iterative reconstruction on top of the projector pair: thin wrappers of leap_sirt / leap_least_squares_descent.

Argument marshalling only: the iterations (projector calls, elementwise updates, reductions) run inside
libleap_hip.so on the current HIP stream.  PyTorch supplies the volume, the sinogram and the workspace memory.
"""
from __future__ import annotations

import torch

from . import binding as B
from .projector import Geometry


def _workspace(geo: Geometry) -> torch.Tensor:
    return torch.empty(B.leap_recon_workspace_floats(geo.handle), dtype=torch.float32, device=geo.device)


def _prepare(geo: Geometry, sino: torch.Tensor, x0):
    geo._check(sino, geo.sino_shape, "sinogram")
    if sino.dim() != 3:
        raise ValueError("the solvers take one sinogram [nviews, nrows, ncols]")
    x = torch.zeros(geo.vol_shape, dtype=torch.float32, device=geo.device) if x0 is None else x0.clone()
    geo._check(x, geo.vol_shape, "start volume")
    return x


def sirt(geo: Geometry, sino: torch.Tensor, iterations: int, x0: torch.Tensor = None, relaxation: float = 1.0,
         nonneg: bool = False, workspace: torch.Tensor = None) -> torch.Tensor:
    """x <- x + relaxation * C A^T (R (y - A x)), `iterations` times; returns the volume."""
    x = _prepare(geo, sino, x0)
    work = _workspace(geo) if workspace is None else workspace
    with torch.cuda.device(geo.device):
        B.leap_sirt(geo.handle, sino.data_ptr(), x.data_ptr(), work.data_ptr(), iterations, relaxation, nonneg,
                    torch.cuda.current_stream().cuda_stream)
    return x


def least_squares_descent(geo: Geometry, sino: torch.Tensor, iterations: int, x0: torch.Tensor = None,
                          workspace: torch.Tensor = None) -> torch.Tensor:
    """Steepest descent on 1/2 ||A x - y||^2 with the exact line search; returns the volume."""
    x = _prepare(geo, sino, x0)
    work = _workspace(geo) if workspace is None else workspace
    with torch.cuda.device(geo.device):
        B.leap_least_squares_descent(geo.handle, sino.data_ptr(), x.data_ptr(), work.data_ptr(), iterations,
                                     torch.cuda.current_stream().cuda_stream)
    return x
