// Siddon projector pair on the modular geometry ("CT Projection Models and Geometries": a flexible cone-beam geometry
// with sources and detectors at any position and orientation): view a has its own source S_a, detector centre C_a and
// orthonormal detector axes (along the column index, along the row index); the ray of pixel (r, c) runs from S_a to
// C_a + u_c ucol_a + v_r vrow_a.  Weight = length of that ray inside the half-open voxel box.
//
// General bodies, one output per call, double precision along the ray (a ray may advance fastest along any axis, so
// the slab formulation of the circular scanners does not apply):
//   forward : incremental traversal of the voxel grid (the next face crossing per axis, smallest first);
//   back    : the voxel's eight corners are projected onto the detector plane; every pixel of their bounding
//             rectangle is tested with the slab clip of its ray against the voxel box.
#pragma once

#include "sf_footprint.h"

struct MdPose {
    double S[3], C[3], ucol[3], vrow[3];
};

struct MdRay {
    double o[3], d[3], len;
};

SF_HD MdRay md_ray(const SfGeom &g, const MdPose &P, int r, int c)
{
    MdRay R;
    const double u = ((double)c - g.col_offd) * (double)g.pu_d, v = fma((double)r, g.pvd, g.v0d);
    double q = 0.0;
    for (int a = 0; a < 3; ++a) {
        R.o[a] = P.S[a];
        R.d[a] = P.C[a] + u * P.ucol[a] + v * P.vrow[a] - P.S[a];
        q = fma(R.d[a], R.d[a], q);
    }
    R.len = sqrt(q);
    return R;
}

// Parameter range [t0, t1] of the ray inside the half-open box [lo, hi); returns false when it misses.
SF_HD bool md_clip(const MdRay &R, const double lo[3], const double hi[3], double &t0, double &t1)
{
    t0 = -1e300;
    t1 = 1e300;
    for (int a = 0; a < 3; ++a) {
        if (R.d[a] == 0.0) {
            if (!(lo[a] <= R.o[a] && R.o[a] < hi[a])) return false;
        } else {
            const double inv = 1.0 / R.d[a];
            double ta = (lo[a] - R.o[a]) * inv, tb = (hi[a] - R.o[a]) * inv;
            if (ta > tb) { const double w = ta; ta = tb; tb = w; }
            t0 = ta > t0 ? ta : t0;
            t1 = tb < t1 ? tb : t1;
        }
    }
    return t1 > t0;
}

SF_HD float md_project_ray(const SfGeom &g, const MdPose &P, const float *__restrict__ vol, int r, int c)
{
    const MdRay R = md_ray(g, P, r, c);
    const int n[3] = {g.nx, g.ny, g.nz};
    const double pitch[3] = {g.Td, g.Td, g.Tzd};
    const double lo[3] = {g.x0d - 0.5 * g.Td, g.y0d - 0.5 * g.Td, g.zlo0d};
    const double hi[3] = {lo[0] + n[0] * pitch[0], lo[1] + n[1] * pitch[1], lo[2] + n[2] * pitch[2]};
    double t, t1;
    if (!md_clip(R, lo, hi, t, t1)) return 0.0f;
    int cell[3], step[3];
    double tmax[3], tdelta[3];
    for (int a = 0; a < 3; ++a) {
        // the entry point lies on a face of the volume up to rounding: clamp the cell found there into the grid
        double idx = floor((fma(t, R.d[a], R.o[a]) - lo[a]) / pitch[a]);
        idx = idx < 0.0 ? 0.0 : (idx > (double)(n[a] - 1) ? (double)(n[a] - 1) : idx);
        cell[a] = (int)idx;
        if (R.d[a] > 0.0) {
            step[a] = 1;
            tmax[a] = (lo[a] + (idx + 1.0) * pitch[a] - R.o[a]) / R.d[a];
            tdelta[a] = pitch[a] / R.d[a];
        } else if (R.d[a] < 0.0) {
            step[a] = -1;
            tmax[a] = (lo[a] + idx * pitch[a] - R.o[a]) / R.d[a];
            tdelta[a] = -pitch[a] / R.d[a];
        } else {
            step[a] = 0;
            tmax[a] = 1e300;
            tdelta[a] = 0.0;
        }
    }
    double sum = 0.0;
    const int max_steps = n[0] + n[1] + n[2] + 3;       // every step leaves one cell through one face
    for (int it = 0; it < max_steps && t < t1; ++it) {
        const int a = tmax[0] <= tmax[1] ? (tmax[0] <= tmax[2] ? 0 : 2) : (tmax[1] <= tmax[2] ? 1 : 2);
        const double tn = tmax[a] < t1 ? tmax[a] : t1;
        if (tn > t) sum = fma(tn - t, (double)vol[((size_t)cell[2] * g.ny + cell[1]) * g.nx + cell[0]], sum);
        t = tn;
        cell[a] += step[a];
        tmax[a] += tdelta[a];
        if (cell[a] < 0 || cell[a] >= n[a]) break;
    }
    return (float)(sum * R.len);
}

SF_HD float md_backproject_voxel(const SfGeom &g, const MdPose *__restrict__ poses, const float *__restrict__ sino, int i,
                                 int j, int k)
{
    const double lo[3] = {g.x0d + ((double)i - 0.5) * g.Td, g.y0d + ((double)j - 0.5) * g.Td, fma((double)k, g.Tzd, g.zlo0d)};
    const double hi[3] = {lo[0] + g.Td, lo[1] + g.Td, lo[2] + g.Tzd};
    const double ipu = 1.0 / g.pu_d, ipv = 1.0 / g.pvd;
    double acc = 0.0;
    for (int a = 0; a < g.nviews; ++a) {
        const MdPose P = poses[a];
        const double nrm[3] = {P.ucol[1] * P.vrow[2] - P.ucol[2] * P.vrow[1], P.ucol[2] * P.vrow[0] - P.ucol[0] * P.vrow[2],
                               P.ucol[0] * P.vrow[1] - P.ucol[1] * P.vrow[0]};
        const double num = (P.C[0] - P.S[0]) * nrm[0] + (P.C[1] - P.S[1]) * nrm[1] + (P.C[2] - P.S[2]) * nrm[2];
        double umin = 1e300, umax = -1e300, vmin = 1e300, vmax = -1e300;
        bool all_in_front = true;
        for (int corner = 0; corner < 8; ++corner) {
            const double X[3] = {(corner & 1) ? hi[0] : lo[0], (corner & 2) ? hi[1] : lo[1], (corner & 4) ? hi[2] : lo[2]};
            const double den = (X[0] - P.S[0]) * nrm[0] + (X[1] - P.S[1]) * nrm[1] + (X[2] - P.S[2]) * nrm[2];
            if (!(num * den > 0.0)) { all_in_front = false; break; }
            const double s = num / den;
            double u = 0.0, v = 0.0;
            for (int q = 0; q < 3; ++q) {
                const double H = fma(s, X[q] - P.S[q], P.S[q]) - P.C[q];
                u = fma(H, P.ucol[q], u);
                v = fma(H, P.vrow[q], v);
            }
            umin = u < umin ? u : umin; umax = u > umax ? u : umax;
            vmin = v < vmin ? v : vmin; vmax = v > vmax ? v : vmax;
        }
        int c0 = 0, c1 = g.ncols - 1, r0 = 0, r1 = g.nrows - 1;
        if (all_in_front) {           // otherwise every pixel of the view is tested
            const double fc0 = ceil(umin * ipu + g.col_offd - 1e-6), fc1 = floor(umax * ipu + g.col_offd + 1e-6);
            const double fr0 = ceil((vmin - g.v0d) * ipv - 1e-6), fr1 = floor((vmax - g.v0d) * ipv + 1e-6);
            if (fc1 < 0.0 || fr1 < 0.0 || fc0 > (double)c1 || fr0 > (double)r1) continue;
            c0 = fc0 < 0.0 ? 0 : (int)fc0; c1 = fc1 > (double)c1 ? c1 : (int)fc1;
            r0 = fr0 < 0.0 ? 0 : (int)fr0; r1 = fr1 > (double)r1 ? r1 : (int)fr1;
        }
        const float *__restrict__ ya = sino + (size_t)a * g.nrows * g.ncols;
        for (int r = r0; r <= r1; ++r)
            for (int c = c0; c <= c1; ++c) {
                const MdRay R = md_ray(g, P, r, c);
                double t0, t1;
                if (md_clip(R, lo, hi, t0, t1)) acc = fma((t1 - t0) * R.len, (double)ya[(size_t)r * g.ncols + c], acc);
            }
    }
    return (float)acc;
}
