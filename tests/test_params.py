"""The plain-text parameter files of the Python package (no GPU): every field of the CT parameter set arrives in the
descriptor as written, the three ways of giving view angles agree, modular poses come from their own file, files
written by save_parameters read back identically, and malformed files are refused with a message."""
import math

import numpy as np
import pytest

from paper_2307_05801_amd import binding as B
from paper_2307_05801_amd import params as P
from synthetic import config, perturbed_poses, reduced

TEXT = """
# a flat-panel cone-beam scanner
geometry = cone
nviews = 8
angular_range = 180     # degrees
start_angle = 10
nrows = 20
ncols = 30
pixel_height = 1.5
pixel_width  = 1.25
shift_vertical = -0.5
shift_horizontal = 0.25
sdd = 900
sod = 600
nx = 16
ny = 18
nz = 12
voxel_width = 0.8
voxel_height = 1.1
center_x = 1
center_y = -2
center_z = 0.5
model = siddon
"""


def test_every_field_arrives_as_written():
    p = P.parse_parameters(TEXT)
    assert p["type"] == B.LEAP_CONE and p["model"] == "siddon"
    assert (p["nviews"], p["nrows"], p["ncols"], p["nx"], p["ny"], p["nz"]) == (8, 20, 30, 16, 18, 12)
    assert (p["pixel_v"], p["pixel_u"], p["shift_v"], p["shift_u"]) == (1.5, 1.25, -0.5, 0.25)
    assert (p["sdd"], p["sod"], p["voxel_xy"], p["voxel_z"]) == (900.0, 600.0, 0.8, 1.1)
    assert (p["center_x"], p["center_y"], p["center_z"]) == (1.0, -2.0, 0.5)
    np.testing.assert_allclose(np.degrees(p["angles_rad"]), 10 + 22.5 * np.arange(8), atol=1e-12)
    model = p.pop("model")
    d, keep = B.make_desc(model=B.MODELS[model], **p)
    assert d.nviews == 8 and d.sdd == 900.0 and d.model == B.LEAP_MODEL_SIDDON and d.angles_rad[7] == p["angles_rad"][7]


def test_three_ways_of_giving_angles_agree(tmp_path):
    base = TEXT.replace("angular_range = 180     # degrees\nstart_angle = 10\n", "")
    degs = [10 + 22.5 * a for a in range(8)]
    listed = P.parse_parameters(base + "angles = " + ", ".join(str(d) for d in degs))
    (tmp_path / "ang.txt").write_text("\n".join(str(d) for d in degs))
    (tmp_path / "scan.txt").write_text(base + "angles_file = ang.txt\n")
    from_file = P.load_parameters(str(tmp_path / "scan.txt"))
    assert listed["angles_rad"] == from_file["angles_rad"]
    np.testing.assert_allclose(listed["angles_rad"], P.parse_parameters(TEXT)["angles_rad"], atol=1e-15)


@pytest.mark.parametrize("make", [lambda: reduced(config(3), 16, nviews=11), lambda: reduced(config(2), 16, nviews=7),
                                  lambda: perturbed_poses(reduced(config(3), 16, nviews=5), 2)],
                         ids=["cone", "parallel", "modular"])
def test_written_files_read_back_identically(tmp_path, make):
    cfg = make()
    params = dict(type=cfg.geom, model="sf", nviews=cfg.nviews, nrows=cfg.nrows, ncols=cfg.ncols, nx=cfg.nx, ny=cfg.ny,
                  nz=cfg.nz, pixel_v=cfg.pixel_v, pixel_u=cfg.pixel_u, shift_v=cfg.shift_v, shift_u=cfg.shift_u,
                  sod=cfg.sod, sdd=cfg.sdd, voxel_xy=cfg.voxel_xy, voxel_z=cfg.voxel_z, center_x=cfg.center_x,
                  center_y=cfg.center_y, center_z=cfg.center_z, angles_rad=[float(a) for a in cfg.angles()])
    if cfg.geom == B.LEAP_MODULAR:
        params["poses"] = [list(p) for p in cfg.poses]
    path = str(tmp_path / "scan.txt")
    P.save_parameters(path, params)
    back = P.load_parameters(path)
    for key, value in params.items():
        if key == "angles_rad":
            if cfg.geom != B.LEAP_MODULAR:
                np.testing.assert_allclose(back[key], value, rtol=0, atol=1e-15)
        elif key == "poses":
            assert back[key] == value
        else:
            assert back[key] == value, key
    # the descriptor the library would see is the one the configuration gives directly
    d1, k1 = B.desc_from_config(cfg)
    model = back.pop("model")
    d2, k2 = B.make_desc(model=B.MODELS[model], **back)
    for name, _ in B.leap_geometry_desc._fields_:
        if name not in ("angles_rad", "poses"):
            assert getattr(d1, name) == getattr(d2, name), name


@pytest.mark.parametrize("bad,what", [
    (TEXT.replace("nx = 16", ""), "'nx' is missing"),
    (TEXT.replace("geometry = cone", "geometry = helical"), "geometry must be"),
    (TEXT + "nx = 17\n", "given twice"),
    (TEXT + "colour = blue\n", "unknown key"),
    (TEXT + "angles = 1, 2, 3\n", "exactly one of"),
    (TEXT.replace("sod = 600", ""), "'sod' is missing"),
    (TEXT.replace("angular_range = 180     # degrees", "angles = 1 2 3"), "8 but 3 angles"),
    (TEXT.replace("nrows = 20", "nrows 20"), "expected 'key = value'"),
])
def test_malformed_files_are_refused(bad, what):
    with pytest.raises(ValueError, match=what):
        P.parse_parameters(bad)
