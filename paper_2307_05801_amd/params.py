"""Plain-text parameter files for the CT parameter set ("PyTorch Interfaces and CT Parameters": geometry type, number
of projections, angular range or list of projection angles, detector pixel width and height, source-to-detector and
source-to-object distance, horizontal and vertical detector shift, number of voxels per dimension, voxel width and
height, position of the volume centre).

One `key = value` per line; `#` starts a comment; keys in any order, case-insensitive.  Lengths in mm, angles in
degrees, detector shifts in pixels.

    geometry     = parallel | fan | cone | cone_curved | modular
    model        = sf | siddon                      (optional, default sf)
    nviews       = 720
    angular_range = 360        start_angle = 0      (equally spaced views over the range, end point excluded)
    angles       = 0, 0.5, 1.0, ...                 (or)   angles_file = angles.txt   (one list of nviews numbers)
    nrows, ncols, pixel_height, pixel_width, shift_vertical, shift_horizontal
    sdd, sod                                        (not for parallel and modular)
    nx, ny, nz, voxel_width, voxel_height           (voxel_height defaults to voxel_width)
    center_x, center_y, center_z                    (default 0)
    poses_file   = poses.txt                        (modular: nviews rows of 12 numbers: source, detector centre,
                                                     column axis, row axis)

Relative file names are taken from the parameter file's folder.  `load_parameters` returns the keyword arguments of
`binding.make_desc` / `Geometry(**kwargs)` plus "model" as a string; `save_parameters` writes them back.
"""
from __future__ import annotations

import math
import os
from typing import Dict

from . import binding as B

GEOMETRIES = {"parallel": B.LEAP_PARALLEL, "fan": B.LEAP_FAN, "cone": B.LEAP_CONE, "cone_curved": B.LEAP_CONE_CURVED,
              "modular": B.LEAP_MODULAR}
_INT_KEYS = ("nviews", "nrows", "ncols", "nx", "ny", "nz")
_FLOAT_KEYS = {"pixel_height": "pixel_v", "pixel_width": "pixel_u", "shift_vertical": "shift_v", "shift_horizontal": "shift_u",
               "sdd": "sdd", "sod": "sod", "voxel_width": "voxel_xy", "voxel_height": "voxel_z",
               "center_x": "center_x", "center_y": "center_y", "center_z": "center_z"}
_OTHER_KEYS = ("geometry", "model", "angular_range", "start_angle", "angles", "angles_file", "poses_file")


def _numbers(text: str):
    return [float(t) for t in text.replace(",", " ").split()]


def parse_parameters(text: str, folder: str = ".") -> Dict:
    raw = {}
    for lineno, line in enumerate(text.splitlines(), 1):
        line = line.split("#", 1)[0].strip()
        if not line:
            continue
        if "=" not in line:
            raise ValueError(f"line {lineno}: expected 'key = value'")
        key, value = (t.strip() for t in line.split("=", 1))
        key = key.lower()
        if key not in _INT_KEYS and key not in _FLOAT_KEYS and key not in _OTHER_KEYS:
            raise ValueError(f"line {lineno}: unknown key '{key}'")
        if key in raw:
            raise ValueError(f"line {lineno}: '{key}' given twice")
        raw[key] = value
    for need in ("geometry", "nviews", "nrows", "ncols", "nx", "ny", "nz", "pixel_height", "pixel_width", "voxel_width"):
        if need not in raw:
            raise ValueError(f"'{need}' is missing")
    geometry = raw["geometry"].lower()
    if geometry not in GEOMETRIES:
        raise ValueError(f"geometry must be one of {sorted(GEOMETRIES)}")
    out = {"type": GEOMETRIES[geometry], "model": raw.get("model", "sf").lower()}
    if out["model"] not in B.MODELS:
        raise ValueError(f"model must be one of {sorted(B.MODELS)}")
    for key in _INT_KEYS:
        out[key] = int(raw[key])
    for key, field in _FLOAT_KEYS.items():
        if key in raw:
            out[field] = float(raw[key])
    out.setdefault("voxel_z", out["voxel_xy"])
    n = out["nviews"]
    if geometry == "modular":
        if "poses_file" not in raw:
            raise ValueError("a modular geometry needs poses_file")
        with open(os.path.join(folder, raw["poses_file"])) as f:
            vals = _numbers(f.read())
        if len(vals) != 12 * n:
            raise ValueError(f"poses_file must hold nviews x 12 = {12 * n} numbers, found {len(vals)}")
        out["poses"] = [vals[12 * a:12 * a + 12] for a in range(n)]
        out["angles_rad"] = [0.0] * n
    else:
        given = [k for k in ("angular_range", "angles", "angles_file") if k in raw]
        if len(given) != 1:
            raise ValueError("give exactly one of angular_range, angles, angles_file")
        if given[0] == "angular_range":
            start, span = float(raw.get("start_angle", 0.0)), float(raw["angular_range"])
            degs = [start + span * a / n for a in range(n)]
        elif given[0] == "angles":
            degs = _numbers(raw["angles"])
        else:
            with open(os.path.join(folder, raw["angles_file"])) as f:
                degs = _numbers(f.read())
        if len(degs) != n:
            raise ValueError(f"nviews = {n} but {len(degs)} angles given")
        out["angles_rad"] = [math.radians(d) for d in degs]
        if geometry != "parallel":
            for need in ("sdd", "sod"):
                if need not in out:
                    raise ValueError(f"'{need}' is missing")
    return out


def load_parameters(path: str) -> Dict:
    with open(path) as f:
        return parse_parameters(f.read(), os.path.dirname(os.path.abspath(path)))


def save_parameters(path: str, params: Dict) -> None:
    """Writes `params` (as returned by load_parameters) to `path`; view angles as a list, poses to `<path>.poses`."""
    names = {v: k for k, v in GEOMETRIES.items()}
    lines = [f"geometry = {names[params['type']]}", f"model = {params.get('model', 'sf')}"]
    lines += [f"{key} = {int(params[key])}" for key in _INT_KEYS]
    for key, field in _FLOAT_KEYS.items():
        if field in params:
            lines.append(f"{key} = {float(params[field])!r}")
    if params["type"] == B.LEAP_MODULAR:
        poses_path = path + ".poses"
        with open(poses_path, "w") as f:
            for row in params["poses"]:
                f.write(" ".join(repr(float(v)) for v in row) + "\n")
        lines.append(f"poses_file = {os.path.basename(poses_path)}")
    else:
        lines.append("angles = " + ", ".join(repr(math.degrees(a)) for a in params["angles_rad"]))
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")


def geometry_from_file(path: str, device="cuda:0"):
    """A Geometry (one handle on one GPU) for the scanner described by the parameter file."""
    from .projector import Geometry
    params = load_parameters(path)
    model = params.pop("model")
    return Geometry(None, device=device, model=model, **params)
