"""The pins must be able to fail: plant one plausible mistake at a time into a COPY of the oracle's C source
(dropped term, wrong sign, transposed index, wrong magnification, ...) and check that the pin tests of that oracle
(tests/test_oracle_pins.py, tests/test_siddon_pins.py) reject every one of them.  Everything happens on the CPU in a temporary directory; the real oracle is untouched."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = [
    ("magnification taken at the axis instead of the voxel centre",
     "else *mag = f.sdd / (f.lS - l);", "else *mag = f.sdd / f.lS;"),
    ("amplitude divides by the smaller direction component",
     "fmax(fabs(dx), fabs(dy))", "fmin(fabs(dx), fabs(dy))"),
    ("parallel amplitude ignores the view angle",
     "return s->T / fmax(fabs(cphi), fabs(sphi));", "return s->T;"),
    ("sign of the detector axis",
     "double t = -x * f->sphi + y * f->cphi;", "double t = x * f->sphi + y * f->cphi;"),
    ("source on the wrong side",
     "return f->tS + f->sdd * (t - f->tS) / (f->lS - l) - f->tC;", "return f->tS + f->sdd * (t - f->tS) / (f->lS + l) - f->tC;"),
    ("sign of the horizontal detector shift",
     "(c - 0.5 * (s->ncols - 1) + s->shift_u) * s->pu", "(c - 0.5 * (s->ncols - 1) - s->shift_u) * s->pu"),
    ("row centres off by half a pixel",
     "(r - 0.5 * (s->nrows - 1) + s->shift_v) * s->pv", "(r - 0.5 * (s->nrows) + s->shift_v) * s->pv"),
    ("axial extent uses the in-plane voxel size",
     "*vhi = f.zS + mag * (z + 0.5 * s->Tz - f.zS) - f.zC;", "*vhi = f.zS + mag * (z + 0.5 * s->T - f.zS) - f.zC;"),
    ("ramp area counted twice",
     "if (u <= tau[2]) return 0.5 * (tau[1] - tau[0]) + (u - tau[1]);",
     "if (u <= tau[2]) return (tau[1] - tau[0]) + (u - tau[1]);"),
    ("ray length ignores the cone angle",
     "double len = sqrt(dx * dx + dy * dy + dz * dz);", "double len = sqrt(dx * dx + dy * dy);"),
    ("candidate range drops the last pixel",
     "double f = floor(ilo - 0.5), l = ceil(ihi + 0.5);", "double f = floor(ilo - 0.5), l = floor(ihi - 0.5);"),
    ("amplitude table indexed transposed in A",
     "y[(int64_t)r * s->ncols + c] += amp[(int64_t)r * s->ncols + c] * fu * fv * x;",
     "y[(int64_t)r * s->ncols + c] += amp[(int64_t)c * s->ncols + r] * fu * fv * x;"),
    ("amplitude arguments swapped in A^T",
     "acc += amplitude(s, a, r, c) * fu * fv * y[(int64_t)r * s->ncols + c];",
     "acc += amplitude(s, a, c, r) * fu * fv * y[(int64_t)r * s->ncols + c];"),
    ("sign of the axial volume offset",
     "static double vox_z(const sfo_scan *s, int k) { return s->cz + (k - 0.5 * (s->nz - 1)) * s->Tz; }",
     "static double vox_z(const sfo_scan *s, int k) { return -s->cz + (k - 0.5 * (s->nz - 1)) * s->Tz; }"),
]


SIDDON_MUTATIONS = [
    ("face plane given to the lower voxel",
     "if (!(lo[a] <= ray->o[a] && ray->o[a] < hi[a])) return 0.0;",
     "if (!(lo[a] < ray->o[a] && ray->o[a] <= hi[a])) return 0.0;"),
    ("ray length measured in the plane only",
     "for (int a = 0; a < ray->ndim; ++a) q += ray->d[a] * ray->d[a];",
     "for (int a = 0; a < 2; ++a) q += ray->d[a] * ray->d[a];"),
    ("parameter length not converted to mm",
     "return t1 > t0 ? (t1 - t0) * ray->len : 0.0;", "return t1 > t0 ? (t1 - t0) : 0.0;"),
    ("parallel rays ignore the detector row",
     "ray->o[a] = u * eu[a] + v * ez[a];", "ray->o[a] = u * eu[a];"),
    ("sign of the detector axis",
     "eu[3] = { -sphi, cphi, 0.0 }", "eu[3] = { sphi, cphi, 0.0 }"),
    ("detector placed at the source-to-detector distance behind the axis",
     "ray->d[a] = -s->sdd * es[a] + u * eu[a] + v * ez[a];",
     "ray->d[a] = -(s->sdd + s->sod) * es[a] + u * eu[a] + v * ez[a];"),
    ("grid shifted by half a voxel",
     "return centre - 0.5 * n * pitch;", "return centre - 0.5 * (n - 1) * pitch;"),
    ("ray walk keeps only the first cell of a slab",
     "fb = floor((hi - g0) / p + 1e-9);", "fb = floor((lo - g0) / p + 1e-9);"),
    ("sign of the horizontal shift in the voxel's pixel search",
     "0.5 * (s->ncols - 1) - s->shift_u, s->ncols", "0.5 * (s->ncols - 1) + s->shift_u, s->ncols"),
    ("pixel search forgets the axial magnification",
     "double u = mag * t, v = mag * z;", "double u = mag * t, v = z;"),
    ("volume indexed transposed in A",
     "sum += w * (double)vol[((int64_t)k * s->ny + j) * s->nx + i];",
     "sum += w * (double)vol[((int64_t)k * s->nx + i) * s->ny + j];"),
    ("sinogram indexed transposed in A^T",
     "sum += w * (double)sino[((int64_t)view * s->nrows + r) * s->ncols + c];",
     "sum += w * (double)sino[((int64_t)view * s->ncols + c) * s->nrows + r];"),
]

CURVED_SF_MUTATIONS = [
    ("curved detector: arc length replaced by the tangent",
     "return s->sdd * atan2(t, s->sod - l);", "return s->sdd * t / (s->sod - l);"),
    ("curved detector: axial magnification taken along the central ray",
     "else if (s->geom == SFO_CONE_CURVED) *mag = s->sdd / hypot(s->sod - l, t);",
     "else if (s->geom == SFO_CONE_CURVED) *mag = s->sdd / (s->sod - l);"),
    ("curved detector: amplitude of the flat detector's ray",
     "double gam = u / s->sdd;", "double gam = atan(u / s->sdd);"),
    ("curved detector: fan angle counted the other way in the amplitude",
     "dy = s->sdd * (-cos(gam) * sphi + sin(gam) * cphi);", "dy = s->sdd * (-cos(gam) * sphi - sin(gam) * cphi);"),
]
CURVED_SIDDON_MUTATIONS = [
    ("curved detector: pixels placed at flat-detector angles",
     "double gam = u / s->sdd;", "double gam = atan(u / s->sdd);"),
    ("curved detector: fan angle counted the other way",
     "ray->d[a] = s->sdd * (-cos(gam) * es[a] + sin(gam) * eu[a]) + v * ez[a];",
     "ray->d[a] = s->sdd * (-cos(gam) * es[a] - sin(gam) * eu[a]) + v * ez[a];"),
    ("curved detector: voxel's pixel search uses flat-detector columns",
     "u = s->sdd * atan2(t, s->sod - l);", "u = s->sdd * t / (s->sod - l);"),
]

MODULAR_SIDDON_MUTATIONS = [
    ("modular: detector axes swapped",
     "ray->d[a] = C[a] + pu_ * uc[a] + pv_ * vr[a] - S[a];", "ray->d[a] = C[a] + pu_ * vr[a] + pv_ * uc[a] - S[a];"),
    ("modular: rays leave from the detector centre",
     "ray->o[a] = S[a];\n            ray->d[a] = C[a]", "ray->o[a] = C[a];\n            ray->d[a] = C[a]"),
    ("modular: voxel's pixel search swaps the detector axes",
     "u += H * uc[a]; v += H * vr[a];", "u += H * vr[a]; v += H * uc[a];"),
    ("ray walk never takes z as its marching axis",
     "if (ray->ndim == 3 && fabs(ray->d[2]) > fabs(ray->d[major])) major = 2;", ";"),
]

MODULAR_SF_MUTATIONS = [
    ("modular: axial interval magnified about z = 0 instead of the source height",
     "*vlo = f.zS + mag * (z - 0.5 * s->Tz - f.zS) - f.zC;", "*vlo = mag * (z - 0.5 * s->Tz) - f.zC;"),
    ("modular: detector centre offset added instead of subtracted",
     "return f->tS + f->sdd * (t - f->tS) / (f->lS - l) - f->tC;", "return f->tS + f->sdd * (t - f->tS) / (f->lS - l) + f->tC;"),
    ("modular: amplitude of the ray of a centred module",
     "double du = u + f.tC - f.tS, dz = v + f.zC - f.zS;", "double du = u, dz = v;"),
    ("modular: source distance taken from the world origin",
     "f->lS = S[0] * f->cphi + S[1] * f->sphi;", "f->lS = sqrt(S[0] * S[0] + S[1] * S[1]);"),
]

TILTED_SF_MUTATIONS = [
    ("tilted module: row coordinate measured along z instead of the module's row axis",
     "*v = q[0] * p->ev[0] + q[1] * p->ev[1] + q[2] * p->ev[2];\n    return 0;", "*v = q[2];\n    return 0;"),
    ("tilted module: column coordinate ignores the column axis' vertical part",
     "*u = q[0] * p->eu[0] + q[1] * p->eu[1] + q[2] * p->eu[2];\n    *v", "*u = q[0] * p->eu[0] + q[1] * p->eu[1];\n    *v"),
    ("tilted module: one component of the plane's normal with the wrong sign",
     "p->n[1] = p->eu[2] * p->ev[0] - p->eu[0] * p->ev[2];", "p->n[1] = p->eu[0] * p->ev[2] - p->eu[2] * p->ev[0];"),
    ("tilted module: corners projected from the upper face instead of the centre's height",
     "bad |= module_project(&p, x - h, y - h, z, &tau[0], &v);",
     "bad |= module_project(&p, x - h, y - h, z + 0.5 * s->Tz, &tau[0], &v);"),
    ("tilted module: amplitude of a ray to an upright module's pixel",
     "d[q] = p.C[q] + u * p.eu[q] + v * p.ev[q] - p.S[q];", "d[q] = p.C[q] + u * p.eu[q] + v * (q == 2) - p.S[q];"),
    ("tilted module: upper face a whole voxel above the centre",
     "bad |= module_project(&p, x, y, z + 0.5 * s->Tz, &u, &vb);", "bad |= module_project(&p, x, y, z + 1.0 * s->Tz, &u, &vb);"),
    ("tilted module: sample index transposed in A",
     "int64_t pixel = (int64_t)r * s->ncols + c;", "int64_t pixel = (int64_t)c * s->nrows + r;"),
    ("tilted module: plane hit slightly short of the plane",
     "double lam = p->gap / along;\n    double q[3]", "double lam = p->gap / (along + 0.01);\n    double q[3]"),
]

CASES = ([("sf_oracle.c", "test_oracle_pins.py") + m for m in MUTATIONS]
         + [("siddon_oracle.c", "test_siddon_pins.py") + m for m in SIDDON_MUTATIONS]
         + [("sf_oracle.c", "test_curved_pins.py") + m for m in CURVED_SF_MUTATIONS]
         + [("siddon_oracle.c", "test_curved_pins.py") + m for m in CURVED_SIDDON_MUTATIONS]
         + [("siddon_oracle.c", "test_modular_pins.py") + m for m in MODULAR_SIDDON_MUTATIONS]
         + [("sf_oracle.c", "test_modular_pins.py") + m for m in MODULAR_SF_MUTATIONS]
         + [("sf_oracle.c", "test_modular_pins.py") + m for m in TILTED_SF_MUTATIONS])


@pytest.mark.parametrize("source,pins,what,old,new", CASES, ids=[c[0][:-9] + ": " + c[2] for c in CASES])
def test_pins_reject_a_planted_mistake(tmp_path, source, pins, what, old, new):
    shutil.copytree(os.path.join(ROOT, "oracle"), tmp_path / "oracle",
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    src = tmp_path / "oracle" / source
    text = src.read_text()
    assert text.count(old) >= 1, "mutation site not found: the oracle changed, update this list"
    src.write_text(text.replace(old, new, 1))
    env = dict(os.environ, PYTHONPATH=os.pathsep.join([str(tmp_path), ROOT, os.path.join(ROOT, "tests")]))
    check = subprocess.run([sys.executable, "-c", "import oracle, os; print(os.path.dirname(oracle.__file__))"],
                           env=env, cwd=str(tmp_path), capture_output=True, text=True)
    assert check.stdout.strip() == str(tmp_path / "oracle"), check.stdout + check.stderr
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", pins), "-x", "-q",
                          "-p", "no:cacheprovider", "--rootdir", str(tmp_path), "-c", os.devnull],
                         env=env, cwd=str(tmp_path), capture_output=True, text=True)
    assert run.returncode != 0, f"the pins accepted: {what}"
    assert "FAILED" in run.stdout, run.stdout[-400:] + run.stderr[-400:]
