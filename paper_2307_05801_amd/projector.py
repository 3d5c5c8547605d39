"""PyTorch face of the library: tensors in, tensors out, autograd pairing backward(A) = A^T.

PyTorch supplies device memory and the HIP stream only; both operators run in libleap_hip.so
("PyTorch Interfaces and CT Parameters": a Projector module derived from torch.nn.Module; "CT Projection
Models and Geometries": the gradient of 1/2 |Ax - y|^2 is A^T (Ax - y), hence the matched transpose).
"""
from __future__ import annotations

import torch

from . import binding as B


class Geometry:
    """Owns one leap_geometry handle on one GPU."""

    def __init__(self, cfg=None, device="cuda:0", model="sf", **desc_kwargs):
        self.device = torch.device(device)
        if self.device.type != "cuda":
            raise RuntimeError("the projector runs on a GPU only (device must be cuda:N); there is no CPU path")
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible to PyTorch; the projector has no CPU path")
        if model not in B.MODELS:
            raise ValueError(f"model must be one of {sorted(B.MODELS)}")
        self.model = model
        if cfg is not None:
            desc, keep = B.desc_from_config(cfg, B.MODELS[model])
        else:
            desc, keep = B.make_desc(model=B.MODELS[model], **desc_kwargs)
        self.nviews, self.nrows, self.ncols = desc.nviews, desc.nrows, desc.ncols
        self.nx, self.ny, self.nz = desc.nx, desc.ny, desc.nz
        with torch.cuda.device(self.device):
            self.handle = B.leap_geometry_create(desc)
        del keep

    @property
    def vol_shape(self):
        return (self.nz, self.ny, self.nx)

    @property
    def sino_shape(self):
        return (self.nviews, self.nrows, self.ncols)

    def describe(self) -> str:
        return B.leap_geometry_describe(self.handle)

    def close(self):
        if getattr(self, "handle", None):
            with torch.cuda.device(self.device):
                torch.cuda.synchronize()
            B.leap_geometry_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- raw operators on contiguous float32 CUDA tensors --------------------------------------

    def _check(self, t: torch.Tensor, shape, what: str) -> int:
        if t.device != self.device or t.dtype != torch.float32 or not t.is_contiguous():
            raise ValueError(f"{what} must be a contiguous float32 tensor on {self.device}")
        if tuple(t.shape[-3:]) != tuple(shape):
            raise ValueError(f"{what} must end in shape {tuple(shape)}, got {tuple(t.shape)}")
        batch = 1
        for n in t.shape[:-3]:
            batch *= n
        if batch < 1:
            raise ValueError("empty batch")
        return batch

    def project(self, vol: torch.Tensor, out: torch.Tensor = None) -> torch.Tensor:
        """A vol; vol [..., nz, ny, nx] -> [..., nviews, nrows, ncols]."""
        batch = self._check(vol, self.vol_shape, "volume")
        if out is None:
            out = torch.empty(tuple(vol.shape[:-3]) + self.sino_shape, dtype=torch.float32, device=self.device)
        elif self._check(out, self.sino_shape, "output sinogram") != batch:
            raise ValueError("output batch mismatch")
        with torch.cuda.device(self.device):
            B.leap_project(self.handle, vol.data_ptr(), out.data_ptr(), batch, torch.cuda.current_stream().cuda_stream)
        return out

    def backproject(self, sino: torch.Tensor, out: torch.Tensor = None) -> torch.Tensor:
        """A^T sino; sino [..., nviews, nrows, ncols] -> [..., nz, ny, nx]."""
        batch = self._check(sino, self.sino_shape, "sinogram")
        if out is None:
            out = torch.empty(tuple(sino.shape[:-3]) + self.vol_shape, dtype=torch.float32, device=self.device)
        elif self._check(out, self.vol_shape, "output volume") != batch:
            raise ValueError("output batch mismatch")
        with torch.cuda.device(self.device):
            B.leap_backproject(self.handle, sino.data_ptr(), out.data_ptr(), batch, torch.cuda.current_stream().cuda_stream)
        return out


    # ---- the same operators on arrays in host memory (numpy arrays or CPU tensors, pinned or not) --------

    def _host_array(self, a, shape, what: str):
        """(address, batch, keep-alive) of a C-contiguous float32 host array ending in `shape`."""
        if isinstance(a, torch.Tensor):
            if a.device.type != "cpu" or a.dtype != torch.float32 or not a.is_contiguous():
                raise ValueError(f"{what} must be a contiguous float32 CPU tensor or numpy array")
            addr, dims = a.data_ptr(), tuple(a.shape)
        else:
            import numpy as np
            if not isinstance(a, np.ndarray) or a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"]:
                raise ValueError(f"{what} must be a C-contiguous float32 numpy array or CPU tensor")
            addr, dims = a.ctypes.data, tuple(a.shape)
        if dims[-3:] != tuple(shape):
            raise ValueError(f"{what} must end in shape {tuple(shape)}, got {dims}")
        batch = 1
        for n in dims[:-3]:
            batch *= n
        if batch < 1:
            raise ValueError("empty batch")
        return addr, batch

    def project_host(self, vol, out):
        """out = A vol with both arrays in host memory; the library uploads, projects and downloads, overlapping the
        three over the items of a batch.  Returns `out`."""
        a_in, batch = self._host_array(vol, self.vol_shape, "volume")
        a_out, batch_out = self._host_array(out, self.sino_shape, "output sinogram")
        if batch != batch_out:
            raise ValueError("output batch mismatch")
        with torch.cuda.device(self.device):
            B.leap_project_host(self.handle, a_in, a_out, batch)
        return out

    def backproject_host(self, sino, out):
        """out = A^T sino with both arrays in host memory.  Returns `out`."""
        a_in, batch = self._host_array(sino, self.sino_shape, "sinogram")
        a_out, batch_out = self._host_array(out, self.vol_shape, "output volume")
        if batch != batch_out:
            raise ValueError("output batch mismatch")
        with torch.cuda.device(self.device):
            B.leap_backproject_host(self.handle, a_in, a_out, batch)
        return out


class _ProjectFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, vol, geom):
        ctx.geom = geom
        return geom.project(vol.contiguous())

    @staticmethod
    def backward(ctx, grad_sino):
        return _BackprojectFn.apply(grad_sino.contiguous(), ctx.geom), None


class _BackprojectFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, sino, geom):
        ctx.geom = geom
        return geom.backproject(sino.contiguous())

    @staticmethod
    def backward(ctx, grad_vol):
        return _ProjectFn.apply(grad_vol.contiguous(), ctx.geom), None


class Projector(torch.nn.Module):
    """y = A x as a differentiable module; `backproject` gives A^T (also differentiable)."""

    def __init__(self, cfg=None, device="cuda:0", model="sf", **desc_kwargs):
        super().__init__()
        self.geometry = Geometry(cfg, device=device, model=model, **desc_kwargs)

    def forward(self, vol: torch.Tensor) -> torch.Tensor:
        return _ProjectFn.apply(vol, self.geometry)

    def backproject(self, sino: torch.Tensor) -> torch.Tensor:
        return _BackprojectFn.apply(sino, self.geometry)
