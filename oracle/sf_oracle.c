/*
 * CPU oracle for the separable-footprint projector pair.  TEST INFRASTRUCTURE ONLY.
 * See sf_oracle.h for the weight definition (steps 1-4) this file writes out, and for
 * which statements of the paper it serves.  Everything is double precision; inputs are
 * the same float32 arrays the HIP library receives.  Loops are over views (A) or voxels
 * (A^T) in the plainest order; OpenMP only splits the outermost loop.
 */
#include "sf_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- coordinates ------------------------------------------------------------------ */

static double vox_x(const sfo_scan *s, int i) { return s->cx + (i - 0.5 * (s->nx - 1)) * s->T; }
static double vox_y(const sfo_scan *s, int j) { return s->cy + (j - 0.5 * (s->ny - 1)) * s->T; }
static double vox_z(const sfo_scan *s, int k) { return s->cz + (k - 0.5 * (s->nz - 1)) * s->Tz; }
static double pix_u(const sfo_scan *s, int c) { return (c - 0.5 * (s->ncols - 1) + s->shift_u) * s->pu; }
static double pix_v(const sfo_scan *s, int r) { return (r - 0.5 * (s->nrows - 1) + s->shift_v) * s->pv; }

/* The frame of one view: unit vectors e_s = (cphi, sphi, 0) (towards the source side) and e_u = (-sphi, cphi, 0), the
 * source at l = lS along e_s, t = tS along e_u, height zS; the detector plane at l = lS - sdd with its centre at
 * t = tC, height zC.  The circular scanners have tS = zS = tC = zC = 0, lS = SOD.  Modular scans (upright modules
 * only: column axis horizontal, row axis +z) read these from the view's pose. */
typedef struct { double cphi, sphi, lS, tS, zS, sdd, tC, zC; } view_frame;

static int frame_of(const sfo_scan *s, int view, view_frame *f)
{
    if (s->geom == SFO_MODULAR) {
        const double *S = s->poses + 12 * (int64_t)view, *C = S + 3, *uc = S + 6, *vr = S + 9;
        if (fabs(uc[2]) > 1e-12 || fabs(vr[0]) > 1e-12 || fabs(vr[1]) > 1e-12 || fabs(vr[2] - 1.0) > 1e-12) return -1;
        f->cphi = uc[1]; f->sphi = -uc[0];
        f->lS = S[0] * f->cphi + S[1] * f->sphi;
        f->tS = -S[0] * f->sphi + S[1] * f->cphi;
        f->zS = S[2];
        f->sdd = f->lS - (C[0] * f->cphi + C[1] * f->sphi);
        f->tC = -C[0] * f->sphi + C[1] * f->cphi;
        f->zC = C[2];
        return f->sdd > 0.0 ? 0 : -1;
    }
    f->cphi = cos(s->phi[view]); f->sphi = sin(s->phi[view]);
    f->lS = s->sod; f->tS = 0.0; f->zS = 0.0; f->sdd = s->sdd; f->tC = 0.0; f->zC = 0.0;
    return 0;
}

/* detector-u coordinate (measured from the detector centre) of the in-plane point (x,y) in a view */
static double project_u(const sfo_scan *s, const view_frame *f, double x, double y)
{
    double t = -x * f->sphi + y * f->cphi;
    if (s->geom == SFO_PARALLEL) return t;
    double l = x * f->cphi + y * f->sphi;
    if (s->geom == SFO_CONE_CURVED) return s->sdd * atan2(t, s->sod - l);     /* arc length on the cylinder */
    return f->tS + f->sdd * (t - f->tS) / (f->lS - l) - f->tC;
}

static void sort4(double a[4])
{
    for (int p = 1; p < 4; ++p) {
        double v = a[p];
        int q = p - 1;
        while (q >= 0 && a[q] > v) { a[q + 1] = a[q]; --q; }
        a[q + 1] = v;
    }
}

/* ---- tilted modules ---------------------------------------------------------------------------------------------
 * A module of a modular scan whose axes are not (horizontal, +z).  The paper says only that detectors may sit at any
 * position and orientation; the reading here keeps the separable footprint on the module's own (u, v) axes:
 *   step 1  the knots are the u coordinates of the central projections (from the source onto the module's plane) of
 *           the voxel's four in-plane corners, taken at the height of the voxel's centre;
 *   step 3  [v-, v+] spans the v coordinates of the central projections of the centres of the voxel's lower and upper
 *           face;
 *   steps 2 and 4 as before (D = pixel - source).
 * For an upright module these are exactly the expressions of the frame above (u does not depend on the height, v is
 * the height magnified about the source), so the two readings meet as the tilt goes to zero. */
typedef struct { const double *S, *C, *eu, *ev; double n[3], gap; } module_pose;   /* n = eu x ev, gap = (C - S).n */

static int view_is_tilted(const sfo_scan *s, int view)
{
    if (s->geom != SFO_MODULAR) return 0;
    const double *uc = s->poses + 12 * (int64_t)view + 6, *vr = uc + 3;
    return fabs(uc[2]) > 1e-12 || fabs(vr[0]) > 1e-12 || fabs(vr[1]) > 1e-12 || fabs(vr[2] - 1.0) > 1e-12;
}

static void pose_of(const sfo_scan *s, int view, module_pose *p)
{
    p->S = s->poses + 12 * (int64_t)view; p->C = p->S + 3; p->eu = p->S + 6; p->ev = p->S + 9;
    p->n[0] = p->eu[1] * p->ev[2] - p->eu[2] * p->ev[1];
    p->n[1] = p->eu[2] * p->ev[0] - p->eu[0] * p->ev[2];
    p->n[2] = p->eu[0] * p->ev[1] - p->eu[1] * p->ev[0];
    p->gap = (p->C[0] - p->S[0]) * p->n[0] + (p->C[1] - p->S[1]) * p->n[1] + (p->C[2] - p->S[2]) * p->n[2];
}

/* central projection of the point (x,y,z) onto the module's plane; (u,v) measured from the detector centre.
 * Returns -1 if the point is not in front of the source (on the detector's side). */
static int module_project(const module_pose *p, double x, double y, double z, double *u, double *v)
{
    double d[3] = {x - p->S[0], y - p->S[1], z - p->S[2]};
    double along = d[0] * p->n[0] + d[1] * p->n[1] + d[2] * p->n[2];
    if (!(along * p->gap > 0.0)) return -1;
    double lam = p->gap / along;
    double q[3] = {p->S[0] + lam * d[0] - p->C[0], p->S[1] + lam * d[1] - p->C[1], p->S[2] + lam * d[2] - p->C[2]};
    *u = q[0] * p->eu[0] + q[1] * p->eu[1] + q[2] * p->eu[2];
    *v = q[0] * p->ev[0] + q[1] * p->ev[1] + q[2] * p->ev[2];
    return 0;
}

/* footprint of voxel centre (x,y,z) on a tilted module: sorted knots and the axial interval */
static int tilted_footprint(const sfo_scan *s, int view, double x, double y, double z, double tau[4], double *vlo, double *vhi)
{
    module_pose p;
    pose_of(s, view, &p);
    double h = 0.5 * s->T, v, va, vb, u;
    int bad = 0;
    bad |= module_project(&p, x - h, y - h, z, &tau[0], &v);
    bad |= module_project(&p, x + h, y - h, z, &tau[1], &v);
    bad |= module_project(&p, x - h, y + h, z, &tau[2], &v);
    bad |= module_project(&p, x + h, y + h, z, &tau[3], &v);
    bad |= module_project(&p, x, y, z - 0.5 * s->Tz, &u, &va);
    bad |= module_project(&p, x, y, z + 0.5 * s->Tz, &u, &vb);
    if (bad) return -1;
    sort4(tau);
    *vlo = fmin(va, vb);
    *vhi = fmax(va, vb);
    return 0;
}

/* A tilted view is usable if the whole volume lies in front of its source and no pixel's ray runs along z (such a ray
 * has no amplitude): the vertical line through the source must miss the detector's rectangle, edge pixels included. */
static int tilted_view_ok(const sfo_scan *s, int view)
{
    module_pose p;
    pose_of(s, view, &p);
    double u, v;
    for (int c = 0; c < 8; ++c) {
        double x = s->cx + ((c & 1) ? 0.5 : -0.5) * s->nx * s->T, y = s->cy + ((c & 2) ? 0.5 : -0.5) * s->ny * s->T;
        double z = s->cz + ((c & 4) ? 0.5 : -0.5) * s->nz * s->Tz;
        if (module_project(&p, x, y, z, &u, &v)) return 0;
    }
    if (fabs(p.n[2]) > 1e-12) {                  /* the vertical line meets the module's plane */
        double lam = p.gap / p.n[2];
        double q[3] = {p.S[0] - p.C[0], p.S[1] - p.C[1], p.S[2] + lam - p.C[2]};
        u = q[0] * p.eu[0] + q[1] * p.eu[1] + q[2] * p.eu[2];
        v = q[0] * p.ev[0] + q[1] * p.ev[1] + q[2] * p.ev[2];
        double ulo = pix_u(s, 0) - 0.5 * s->pu, uhi = pix_u(s, s->ncols - 1) + 0.5 * s->pu;
        double vlo = pix_v(s, 0) - 0.5 * s->pv, vhi = pix_v(s, s->nrows - 1) + 0.5 * s->pv;
        if (u >= ulo && u <= uhi && v >= vlo && v <= vhi) return 0;
    }
    return 1;
}

/* ---- step 1: knots ---------------------------------------------------------------- */

static void knots_xy(const sfo_scan *s, int view, double x, double y, double tau[4], double *mag)
{
    view_frame f;
    frame_of(s, view, &f);
    double h = 0.5 * s->T;
    tau[0] = project_u(s, &f, x - h, y - h);
    tau[1] = project_u(s, &f, x + h, y - h);
    tau[2] = project_u(s, &f, x - h, y + h);
    tau[3] = project_u(s, &f, x + h, y + h);
    sort4(tau);
    if (mag) {
        double l = x * f.cphi + y * f.sphi, t = -x * f.sphi + y * f.cphi;
        if (s->geom == SFO_PARALLEL) *mag = 1.0;
        else if (s->geom == SFO_CONE_CURVED) *mag = s->sdd / hypot(s->sod - l, t);
        else *mag = f.sdd / (f.lS - l);
    }
}

void sfo_knots(const sfo_scan *s, int view, int i, int j, double tau[4], double *mag)
{
    knots_xy(s, view, vox_x(s, i), vox_y(s, j), tau, mag);
}

/* ---- step 2: trapezoid and F_u ---------------------------------------------------- */

double sfo_trapezoid_integral(const double tau[4], double u)
{
    double total = 0.5 * ((tau[3] - tau[0]) + (tau[2] - tau[1]));
    if (u <= tau[0]) return 0.0;
    if (u < tau[1]) return (u - tau[0]) * (u - tau[0]) / (2.0 * (tau[1] - tau[0]));
    if (u <= tau[2]) return 0.5 * (tau[1] - tau[0]) + (u - tau[1]);
    if (u < tau[3]) return total - (tau[3] - u) * (tau[3] - u) / (2.0 * (tau[3] - tau[2]));
    return total;
}

static double footprint_u(const sfo_scan *s, const double tau[4], int c)
{
    double uc = pix_u(s, c);
    return (sfo_trapezoid_integral(tau, uc + 0.5 * s->pu) - sfo_trapezoid_integral(tau, uc - 0.5 * s->pu)) / s->pu;
}

/* ---- step 3: F_v ------------------------------------------------------------------ */

/* axial interval of voxel k on the detector (v measured from the detector centre): the voxel's faces magnified about
 * the source height */
static void axial_interval(const sfo_scan *s, int view, double mag, int k, double *vlo, double *vhi)
{
    view_frame f;
    frame_of(s, view, &f);
    double z = vox_z(s, k);
    *vlo = f.zS + mag * (z - 0.5 * s->Tz - f.zS) - f.zC;
    *vhi = f.zS + mag * (z + 0.5 * s->Tz - f.zS) - f.zC;
}

static double overlap_v(const sfo_scan *s, double vlo, double vhi, int r)
{
    double vr = pix_v(s, r);
    double lo = fmax(vr - 0.5 * s->pv, vlo), hi = fmin(vr + 0.5 * s->pv, vhi);
    return fmax(0.0, hi - lo) / s->pv;
}

static double footprint_v(const sfo_scan *s, int view, double mag, int k, int r)
{
    if (s->geom == SFO_FAN) return 1.0;
    double vlo, vhi;
    axial_interval(s, view, mag, k, &vlo, &vhi);
    return overlap_v(s, vlo, vhi, r);
}

/* ---- step 4: amplitude ------------------------------------------------------------ */

static double amplitude(const sfo_scan *s, int view, int r, int c)
{
    if (view_is_tilted(s, view)) {               /* D = pixel - source, the pixel on the module's plane */
        module_pose p;
        pose_of(s, view, &p);
        double u = pix_u(s, c), v = pix_v(s, r), d[3];
        for (int q = 0; q < 3; ++q) d[q] = p.C[q] + u * p.eu[q] + v * p.ev[q] - p.S[q];
        return s->T * sqrt(d[0] * d[0] + d[1] * d[1] + d[2] * d[2]) / fmax(fabs(d[0]), fabs(d[1]));
    }
    view_frame f;
    frame_of(s, view, &f);
    double cphi = f.cphi, sphi = f.sphi;
    if (s->geom == SFO_PARALLEL) return s->T / fmax(fabs(cphi), fabs(sphi));
    double u = pix_u(s, c);
    double v = (s->geom == SFO_FAN) ? 0.0 : pix_v(s, r);
    /* pixel minus source in the view's frame: -sdd along e_s, (u + tC - tS) along e_u, (v + zC - zS) along z */
    double du = u + f.tC - f.tS, dz = v + f.zC - f.zS;
    double dx = -f.sdd * cphi - du * sphi;
    double dy = -f.sdd * sphi + du * cphi;
    if (s->geom == SFO_CONE_CURVED) {            /* pixel at fan angle gamma = u / SDD on the cylinder */
        double gam = u / s->sdd;
        dx = s->sdd * (-cos(gam) * cphi - sin(gam) * sphi);
        dy = s->sdd * (-cos(gam) * sphi + sin(gam) * cphi);
    }
    double len = sqrt(dx * dx + dy * dy + dz * dz);
    return s->T * len / fmax(fabs(dx), fabs(dy));
}

static int scan_ok(const sfo_scan *s);

/* ---- one weight ------------------------------------------------------------------- */

double sfo_weight(const sfo_scan *s, int view, int r, int c, int i, int j, int k,
                  double *Fu, double *Fv, double *amp)
{
    double tau[4], mag, fu, fv;
    if (view_is_tilted(s, view)) {
        double vlo, vhi;
        if (tilted_footprint(s, view, vox_x(s, i), vox_y(s, j), vox_z(s, k), tau, &vlo, &vhi)) return 0.0;
        fu = footprint_u(s, tau, c);
        fv = overlap_v(s, vlo, vhi, r);
    } else {
        sfo_knots(s, view, i, j, tau, &mag);
        fu = footprint_u(s, tau, c);
        fv = footprint_v(s, view, mag, k, r);
    }
    double am = amplitude(s, view, r, c);
    if (Fu) *Fu = fu;
    if (Fv) *Fv = fv;
    if (amp) *amp = am;
    return am * fu * fv;
}

int sfo_dense_matrix(const sfo_scan *s, double *A)
{
    int64_t n = (int64_t)s->nx * s->ny * s->nz;
    if (scan_ok(s)) return -1;
    for (int a = 0; a < s->nviews; ++a)
        for (int r = 0; r < s->nrows; ++r)
            for (int c = 0; c < s->ncols; ++c) {
                double *row = A + (((int64_t)a * s->nrows + r) * s->ncols + c) * n;
                for (int k = 0; k < s->nz; ++k)
                    for (int j = 0; j < s->ny; ++j)
                        for (int i = 0; i < s->nx; ++i)
                            row[((int64_t)k * s->ny + j) * s->nx + i] = sfo_weight(s, a, r, c, i, j, k, 0, 0, 0);
            }
    return 0;
}

/* ---- candidate pixels: a superset of those an interval [lo,hi] (mm) can touch ------ */

static void candidates(double lo, double hi, double pitch, double shift, int n, int *first, int *last)
{
    /* pixel m covers index coordinates [m-1/2, m+1/2], index(u) = u/pitch - shift + (n-1)/2 */
    double ilo = lo / pitch - shift + 0.5 * (n - 1);
    double ihi = hi / pitch - shift + 0.5 * (n - 1);
    double f = floor(ilo - 0.5), l = ceil(ihi + 0.5);
    if (f < 0) f = 0;
    if (l > n - 1) l = n - 1;
    *first = (int)f;
    *last = (int)l;          /* empty when last < first */
}

/* ---- tilted views: every voxel has its own knots; one voxel against its candidate pixels ---------------------------- */

/* forward: adds voxel (i,j,k)'s contributions x w to the view's samples y (amp: the view's amplitudes) */
static void tilted_scatter(const sfo_scan *s, int view, int i, int j, int k, double x, const double *amp, double *y)
{
    double tau[4], vlo, vhi;
    if (tilted_footprint(s, view, vox_x(s, i), vox_y(s, j), vox_z(s, k), tau, &vlo, &vhi)) return;
    int c0, c1, r0, r1;
    candidates(tau[0], tau[3], s->pu, s->shift_u, s->ncols, &c0, &c1);
    candidates(vlo, vhi, s->pv, s->shift_v, s->nrows, &r0, &r1);
    for (int c = c0; c <= c1; ++c) {
        double fu = footprint_u(s, tau, c);
        if (fu <= 0.0) continue;
        for (int r = r0; r <= r1; ++r) {
            double fv = overlap_v(s, vlo, vhi, r);
            int64_t pixel = (int64_t)r * s->ncols + c;
            if (fv > 0.0) y[pixel] += amp[pixel] * fu * fv * x;
        }
    }
}

/* back: voxel (i,j,k)'s sum over the view's samples y; *count (if given) receives the number of nonzero weights */
static double tilted_gather(const sfo_scan *s, int view, int i, int j, int k, const float *y, int64_t *count)
{
    double tau[4], vlo, vhi, acc = 0.0;
    if (tilted_footprint(s, view, vox_x(s, i), vox_y(s, j), vox_z(s, k), tau, &vlo, &vhi)) return 0.0;
    int c0, c1, r0, r1;
    candidates(tau[0], tau[3], s->pu, s->shift_u, s->ncols, &c0, &c1);
    candidates(vlo, vhi, s->pv, s->shift_v, s->nrows, &r0, &r1);
    for (int c = c0; c <= c1; ++c) {
        double fu = footprint_u(s, tau, c);
        if (fu <= 0.0) continue;
        for (int r = r0; r <= r1; ++r) {
            double fv = overlap_v(s, vlo, vhi, r);
            if (fv <= 0.0) continue;
            if (y) acc += amplitude(s, view, r, c) * fu * fv * y[(int64_t)r * s->ncols + c];
            if (count) ++*count;
        }
    }
    return acc;
}

/* 0 if every view of the scan has a reading */
static int scan_ok(const sfo_scan *s)
{
    if (s->geom != SFO_MODULAR) return 0;
    for (int a = 0; a < s->nviews; ++a) {
        view_frame f;
        if (view_is_tilted(s, a) ? !tilted_view_ok(s, a) : frame_of(s, a, &f)) return -1;
    }
    return 0;
}

/* ---- A ---------------------------------------------------------------------------- */

int sfo_project(const sfo_scan *s, const float *vol, double *sino)
{
    int64_t per_view = (int64_t)s->nrows * s->ncols;
    if (scan_ok(s)) return -1;
    memset(sino, 0, sizeof(double) * per_view * s->nviews);
#pragma omp parallel for schedule(dynamic, 1)
    for (int a = 0; a < s->nviews; ++a) {
        double *y = sino + a * per_view;
        double *amp = (double *)malloc(sizeof(double) * per_view);   /* amp depends on the ray only */
        for (int r = 0; r < s->nrows; ++r)
            for (int c = 0; c < s->ncols; ++c) amp[(int64_t)r * s->ncols + c] = amplitude(s, a, r, c);
        if (view_is_tilted(s, a)) {
            for (int k = 0; k < s->nz; ++k)
                for (int j = 0; j < s->ny; ++j)
                    for (int i = 0; i < s->nx; ++i)
                        tilted_scatter(s, a, i, j, k, vol[((int64_t)k * s->ny + j) * s->nx + i], amp, y);
            free(amp);
            continue;
        }
        for (int j = 0; j < s->ny; ++j)
            for (int i = 0; i < s->nx; ++i) {
                double tau[4], mag;
                sfo_knots(s, a, i, j, tau, &mag);
                int c0, c1;
                candidates(tau[0], tau[3], s->pu, s->shift_u, s->ncols, &c0, &c1);
                for (int c = c0; c <= c1; ++c) {
                    double fu = footprint_u(s, tau, c);
                    if (fu <= 0.0) continue;
                    for (int k = 0; k < s->nz; ++k) {
                        double x = vol[((int64_t)k * s->ny + j) * s->nx + i];
                        int r0 = 0, r1 = 0;
                        if (s->geom != SFO_FAN) {
                            double vlo, vhi;
                            axial_interval(s, a, mag, k, &vlo, &vhi);
                            candidates(vlo, vhi, s->pv, s->shift_v, s->nrows, &r0, &r1);
                        }
                        for (int r = r0; r <= r1; ++r) {
                            double fv = footprint_v(s, a, mag, k, r);
                            if (fv <= 0.0) continue;
                            y[(int64_t)r * s->ncols + c] += amp[(int64_t)r * s->ncols + c] * fu * fv * x;
                        }
                    }
                }
            }
        free(amp);
    }
    return 0;
}

int sfo_project_rays(const sfo_scan *s, const float *vol, int64_t n, const int64_t *ray, double *out)
{
    if (scan_ok(s)) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < n; ++q) {
        int64_t id = ray[q];
        int c = (int)(id % s->ncols);
        int r = (int)((id / s->ncols) % s->nrows);
        int a = (int)(id / ((int64_t)s->ncols * s->nrows));
        double am = amplitude(s, a, r, c), acc = 0.0;
        if (view_is_tilted(s, a)) {
            for (int k = 0; k < s->nz; ++k)
                for (int j = 0; j < s->ny; ++j)
                    for (int i = 0; i < s->nx; ++i) {
                        double tau[4], vlo, vhi;
                        if (tilted_footprint(s, a, vox_x(s, i), vox_y(s, j), vox_z(s, k), tau, &vlo, &vhi)) continue;
                        double fu = footprint_u(s, tau, c);
                        if (fu <= 0.0) continue;
                        double fv = overlap_v(s, vlo, vhi, r);
                        if (fv > 0.0) acc += am * fu * fv * vol[((int64_t)k * s->ny + j) * s->nx + i];
                    }
            out[q] = acc;
            continue;
        }
        for (int j = 0; j < s->ny; ++j)
            for (int i = 0; i < s->nx; ++i) {
                double tau[4], mag;
                sfo_knots(s, a, i, j, tau, &mag);
                double fu = footprint_u(s, tau, c);
                if (fu <= 0.0) continue;
                for (int k = 0; k < s->nz; ++k) {
                    double fv = footprint_v(s, a, mag, k, r);
                    if (fv > 0.0) acc += am * fu * fv * vol[((int64_t)k * s->ny + j) * s->nx + i];
                }
            }
        out[q] = acc;
    }
    return 0;
}

/* ---- A^T -------------------------------------------------------------------------- */

static double backproject_one(const sfo_scan *s, const float *sino, int i, int j, int k)
{
    double acc = 0.0;
    for (int a = 0; a < s->nviews; ++a) {
        const float *y = sino + (int64_t)a * s->nrows * s->ncols;
        if (view_is_tilted(s, a)) {
            acc += tilted_gather(s, a, i, j, k, y, NULL);
            continue;
        }
        double tau[4], mag;
        sfo_knots(s, a, i, j, tau, &mag);
        int c0, c1, r0 = 0, r1 = 0;
        candidates(tau[0], tau[3], s->pu, s->shift_u, s->ncols, &c0, &c1);
        if (s->geom != SFO_FAN) {
            double vlo, vhi;
            axial_interval(s, a, mag, k, &vlo, &vhi);
            candidates(vlo, vhi, s->pv, s->shift_v, s->nrows, &r0, &r1);
        }
        for (int c = c0; c <= c1; ++c) {
            double fu = footprint_u(s, tau, c);
            if (fu <= 0.0) continue;
            for (int r = r0; r <= r1; ++r) {
                double fv = footprint_v(s, a, mag, k, r);
                if (fv <= 0.0) continue;
                acc += amplitude(s, a, r, c) * fu * fv * y[(int64_t)r * s->ncols + c];
            }
        }
    }
    return acc;
}

int sfo_backproject(const sfo_scan *s, const float *sino, double *vol)
{
    if (scan_ok(s)) return -1;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
    for (int k = 0; k < s->nz; ++k)
        for (int j = 0; j < s->ny; ++j)
            for (int i = 0; i < s->nx; ++i)
                vol[((int64_t)k * s->ny + j) * s->nx + i] = backproject_one(s, sino, i, j, k);
    return 0;
}

int sfo_backproject_voxels(const sfo_scan *s, const float *sino, int64_t n, const int64_t *voxel, double *out)
{
    if (scan_ok(s)) return -1;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t q = 0; q < n; ++q) {
        int64_t id = voxel[q];
        int i = (int)(id % s->nx);
        int j = (int)((id / s->nx) % s->ny);
        int k = (int)(id / ((int64_t)s->nx * s->ny));
        out[q] = backproject_one(s, sino, i, j, k);
    }
    return 0;
}

/* ---- counting --------------------------------------------------------------------- */

int64_t sfo_nnz(const sfo_scan *s, int view_begin, int view_end)
{
    int64_t total = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : total)
    for (int a = view_begin; a < view_end; ++a)
        for (int j = 0; j < s->ny; ++j)
            for (int i = 0; i < s->nx; ++i) {
                if (view_is_tilted(s, a)) {
                    int64_t cnt = 0;
                    for (int k = 0; k < s->nz; ++k) tilted_gather(s, a, i, j, k, NULL, &cnt);
                    total += cnt;
                    continue;
                }
                double tau[4], mag;
                sfo_knots(s, a, i, j, tau, &mag);
                int c0, c1;
                candidates(tau[0], tau[3], s->pu, s->shift_u, s->ncols, &c0, &c1);
                int64_t nu = 0;
                for (int c = c0; c <= c1; ++c) nu += footprint_u(s, tau, c) > 0.0;
                if (!nu) continue;
                for (int k = 0; k < s->nz; ++k) {
                    int r0 = 0, r1 = 0;
                    if (s->geom != SFO_FAN) {
                        double vlo, vhi;
                        axial_interval(s, a, mag, k, &vlo, &vhi);
                        candidates(vlo, vhi, s->pv, s->shift_v, s->nrows, &r0, &r1);
                    }
                    int64_t nv = 0;
                    for (int r = r0; r <= r1; ++r) nv += footprint_v(s, a, mag, k, r) > 0.0;
                    total += nu * nv;
                }
            }
    return total;
}

int sfo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void sfo_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
