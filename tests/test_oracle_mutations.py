"""The pins must be able to fail: plant one plausible mistake at a time into a COPY of the oracle's C source
(dropped term, wrong sign, transposed index, wrong magnification, ...) and check that tests/test_oracle_pins.py
rejects every one of them.  Everything happens on the CPU in a temporary directory; the real oracle is untouched."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = [
    ("magnification taken at the axis instead of the voxel centre",
     "*mag = s->sdd / (s->sod - (x * cphi + y * sphi));", "*mag = s->sdd / s->sod;"),
    ("amplitude divides by the smaller direction component",
     "fmax(fabs(dx), fabs(dy))", "fmin(fabs(dx), fabs(dy))"),
    ("parallel amplitude ignores the view angle",
     "return s->T / fmax(fabs(cphi), fabs(sphi));", "return s->T;"),
    ("sign of the detector axis",
     "double t = -x * sphi + y * cphi;", "double t = x * sphi + y * cphi;"),
    ("source on the wrong side",
     "return s->sdd * t / (s->sod - l);", "return s->sdd * t / (s->sod + l);"),
    ("sign of the horizontal detector shift",
     "(c - 0.5 * (s->ncols - 1) + s->shift_u) * s->pu", "(c - 0.5 * (s->ncols - 1) - s->shift_u) * s->pu"),
    ("row centres off by half a pixel",
     "(r - 0.5 * (s->nrows - 1) + s->shift_v) * s->pv", "(r - 0.5 * (s->nrows) + s->shift_v) * s->pv"),
    ("axial extent uses the in-plane voxel size",
     "double vlo = mag * (z - 0.5 * s->Tz), vhi = mag * (z + 0.5 * s->Tz);",
     "double vlo = mag * (z - 0.5 * s->T), vhi = mag * (z + 0.5 * s->T);"),
    ("ramp area counted twice",
     "if (u <= tau[2]) return 0.5 * (tau[1] - tau[0]) + (u - tau[1]);",
     "if (u <= tau[2]) return (tau[1] - tau[0]) + (u - tau[1]);"),
    ("ray length ignores the cone angle",
     "double len = sqrt(dx * dx + dy * dy + v * v);", "double len = sqrt(dx * dx + dy * dy);"),
    ("candidate range drops the last pixel",
     "double f = floor(ilo - 0.5), l = ceil(ihi + 0.5);", "double f = floor(ilo - 0.5), l = floor(ihi - 0.5);"),
    ("amplitude table indexed transposed in A",
     "y[(int64_t)r * s->ncols + c] += amp[(int64_t)r * s->ncols + c] * fu * fv * x;",
     "y[(int64_t)r * s->ncols + c] += amp[(int64_t)c * s->ncols + r] * fu * fv * x;"),
    ("amplitude arguments swapped in A^T",
     "acc += amplitude(s, s->phi[a], r, c) * fu * fv * y[(int64_t)r * s->ncols + c];",
     "acc += amplitude(s, s->phi[a], c, r) * fu * fv * y[(int64_t)r * s->ncols + c];"),
    ("sign of the axial volume offset",
     "static double vox_z(const sfo_scan *s, int k) { return s->cz + (k - 0.5 * (s->nz - 1)) * s->Tz; }",
     "static double vox_z(const sfo_scan *s, int k) { return -s->cz + (k - 0.5 * (s->nz - 1)) * s->Tz; }"),
]


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_reject_a_planted_mistake(tmp_path, what, old, new):
    shutil.copytree(os.path.join(ROOT, "oracle"), tmp_path / "oracle",
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    src = tmp_path / "oracle" / "sf_oracle.c"
    text = src.read_text()
    assert text.count(old) >= 1, "mutation site not found: the oracle changed, update this list"
    src.write_text(text.replace(old, new, 1))
    env = dict(os.environ, PYTHONPATH=os.pathsep.join([str(tmp_path), ROOT, os.path.join(ROOT, "tests")]))
    check = subprocess.run([sys.executable, "-c", "import oracle, os; print(os.path.dirname(oracle.__file__))"],
                           env=env, cwd=str(tmp_path), capture_output=True, text=True)
    assert check.stdout.strip() == str(tmp_path / "oracle"), check.stdout + check.stderr
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                          "-p", "no:cacheprovider", "--rootdir", str(tmp_path), "-c", os.devnull],
                         env=env, cwd=str(tmp_path), capture_output=True, text=True)
    assert run.returncode != 0, f"the pins accepted: {what}"
    assert "FAILED" in run.stdout, run.stdout[-400:] + run.stderr[-400:]
