/*
 * CPU oracle for the Siddon projector pair.  TEST INFRASTRUCTURE ONLY.  See siddon_oracle.h for the definition
 * (weight = length of the pixel-centre ray inside the half-open voxel box) and for the statement of the paper it
 * serves.  Every weight that enters a sum comes from ONE routine, chord(), which clips the ray's parameter range
 * against the box one axis at a time (the textbook slab test).  The loops around it only enumerate a superset of the
 * voxels (A) or pixels (A^T) that can have a non-zero weight; tests compare them with the dense matrix, which calls
 * the same routine for every (ray, voxel) pair.  Double precision throughout; OpenMP splits the outermost loop only.
 */
#include "siddon_oracle.h"

#include <math.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- coordinates -------------------------------------------------------------------------------------------- */

static double grid_lo(double centre, int n, double pitch) { return centre - 0.5 * n * pitch; }   /* lower face of voxel 0 */
static double pix_u(const sdo_scan *s, int c) { return (c - 0.5 * (s->ncols - 1) + s->shift_u) * s->pu; }
static double pix_v(const sdo_scan *s, int r) { return (r - 0.5 * (s->nrows - 1) + s->shift_v) * s->pv; }

/* the line o + t d (t real) of ray (view, r, c); len = |d| converts parameter length to mm */
typedef struct { double o[3], d[3], len; int ndim; } ray_t;

static void ray_of(const sdo_scan *s, int view, int r, int c, ray_t *ray)
{
    if (s->geom == SDO_MODULAR) {
        const double *S = s->poses + 12 * (int64_t)view, *C = S + 3, *uc = S + 6, *vr = S + 9;
        double pu_ = pix_u(s, c), pv_ = pix_v(s, r), q = 0.0;
        ray->ndim = 3;
        for (int a = 0; a < 3; ++a) {
            ray->o[a] = S[a];
            ray->d[a] = C[a] + pu_ * uc[a] + pv_ * vr[a] - S[a];
            q += ray->d[a] * ray->d[a];
        }
        ray->len = sqrt(q);
        return;
    }
    double cphi = cos(s->phi[view]), sphi = sin(s->phi[view]);
    double es[3] = { cphi, sphi, 0.0 }, eu[3] = { -sphi, cphi, 0.0 }, ez[3] = { 0.0, 0.0, 1.0 };
    double u = pix_u(s, c), v = (s->geom == SDO_FAN) ? 0.0 : pix_v(s, r);
    ray->ndim = (s->geom == SDO_FAN) ? 2 : 3;
    for (int a = 0; a < 3; ++a) {
        if (s->geom == SDO_PARALLEL) {
            ray->o[a] = u * eu[a] + v * ez[a];
            ray->d[a] = es[a];
        } else if (s->geom == SDO_CONE_CURVED) {
            double gam = u / s->sdd;
            ray->o[a] = s->sod * es[a];
            ray->d[a] = s->sdd * (-cos(gam) * es[a] + sin(gam) * eu[a]) + v * ez[a];
        } else {
            ray->o[a] = s->sod * es[a];                                   /* source */
            ray->d[a] = -s->sdd * es[a] + u * eu[a] + v * ez[a];          /* pixel centre minus source */
        }
    }
    double q = 0.0;
    for (int a = 0; a < ray->ndim; ++a) q += ray->d[a] * ray->d[a];
    ray->len = sqrt(q);
}

/* length of the line inside the half-open box [lo, hi) */
static double chord(const ray_t *ray, const double lo[3], const double hi[3])
{
    double t0 = -INFINITY, t1 = INFINITY;
    for (int a = 0; a < ray->ndim; ++a) {
        if (ray->d[a] == 0.0) {
            if (!(lo[a] <= ray->o[a] && ray->o[a] < hi[a])) return 0.0;
        } else {
            double ta = (lo[a] - ray->o[a]) / ray->d[a], tb = (hi[a] - ray->o[a]) / ray->d[a];
            if (ta > tb) { double w = ta; ta = tb; tb = w; }
            if (ta > t0) t0 = ta;
            if (tb < t1) t1 = tb;
        }
    }
    return t1 > t0 ? (t1 - t0) * ray->len : 0.0;
}

static void voxel_box(const sdo_scan *s, int i, int j, int k, double lo[3], double hi[3])
{
    lo[0] = grid_lo(s->cx, s->nx, s->T) + i * s->T;   hi[0] = lo[0] + s->T;
    lo[1] = grid_lo(s->cy, s->ny, s->T) + j * s->T;   hi[1] = lo[1] + s->T;
    lo[2] = grid_lo(s->cz, s->nz, s->Tz) + k * s->Tz; hi[2] = lo[2] + s->Tz;
}

double sdo_weight(const sdo_scan *s, int view, int r, int c, int i, int j, int k)
{
    ray_t ray;
    double lo[3], hi[3];
    ray_of(s, view, r, c, &ray);
    voxel_box(s, i, j, k, lo, hi);
    return chord(&ray, lo, hi);
}

/* ---- A: one ray ----------------------------------------------------------------------------------------------- */

/* Index range [*a, *b] of the cells (pitch p, first lower face g0, n cells) that the closed interval between x0 and
 * x1 can touch, widened by a hair so that rounding never loses a cell; clipped to the grid. */
static void cell_range(double x0, double x1, double g0, double p, int n, int *a, int *b)
{
    double lo = fmin(x0, x1), hi = fmax(x0, x1);
    double fa = floor((lo - g0) / p - 1e-9), fb = floor((hi - g0) / p + 1e-9);
    *a = fa < 0.0 ? 0 : (fa > n ? n : (int)fa);
    *b = fb > n - 1 ? n - 1 : (fb < -1.0 ? -1 : (int)fb);
}

/* Visits every voxel the ray can cross: walks the slabs of the axis along which the ray advances fastest, and
 * inside each slab tries every voxel of the bounding box of the ray's piece in that slab.  `vol` may be NULL
 * (then only non-zero weights are counted into *count). */
static double ray_sum(const sdo_scan *s, const ray_t *ray, const float *vol, int64_t *count)
{
    /* the axis the ray advances fastest on (any of the three for a modular scan; fan-beam rays live in the plane) */
    int major = fabs(ray->d[0]) >= fabs(ray->d[1]) ? 0 : 1;
    if (ray->ndim == 3 && fabs(ray->d[2]) > fabs(ray->d[major])) major = 2;
    int n[3] = { s->nx, s->ny, s->nz };
    double pitch[3] = { s->T, s->T, s->Tz };
    double g0[3] = { grid_lo(s->cx, s->nx, s->T), grid_lo(s->cy, s->ny, s->T), grid_lo(s->cz, s->nz, s->Tz) };
    double sum = 0.0;
    for (int m = 0; m < n[major]; ++m) {
        double ta = (g0[major] + m * pitch[major] - ray->o[major]) / ray->d[major];
        double tb = (g0[major] + (m + 1) * pitch[major] - ray->o[major]) / ray->d[major];
        int lo_[3], hi_[3];
        for (int a = 0; a < 3; ++a) {
            if (a == major) { lo_[a] = hi_[a] = m; }
            else if (a == 2 && ray->ndim == 2) { lo_[a] = hi_[a] = 0; }
            else cell_range(ray->o[a] + ta * ray->d[a], ray->o[a] + tb * ray->d[a], g0[a], pitch[a], n[a], &lo_[a], &hi_[a]);
        }
        for (int k = lo_[2]; k <= hi_[2]; ++k)
            for (int j = lo_[1]; j <= hi_[1]; ++j)
                for (int i = lo_[0]; i <= hi_[0]; ++i) {
                    double lo[3], hi[3];
                    voxel_box(s, i, j, k, lo, hi);
                    double w = chord(ray, lo, hi);
                    if (w > 0.0) {
                        if (vol) sum += w * (double)vol[((int64_t)k * s->ny + j) * s->nx + i];
                        if (count) ++*count;
                    }
                }
    }
    return sum;
}

int sdo_project(const sdo_scan *s, const float *vol, double *sino)
{
    int64_t lines = (int64_t)s->nviews * s->nrows;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t l = 0; l < lines; ++l) {
        int view = (int)(l / s->nrows), r = (int)(l % s->nrows);
        for (int c = 0; c < s->ncols; ++c) {
            ray_t ray;
            ray_of(s, view, r, c, &ray);
            sino[l * s->ncols + c] = ray_sum(s, &ray, vol, NULL);
        }
    }
    return 0;
}

int sdo_project_rays(const sdo_scan *s, const float *vol, int64_t n, const int64_t *rayidx, double *out)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t m = 0; m < n; ++m) {
        int c = (int)(rayidx[m] % s->ncols);
        int r = (int)((rayidx[m] / s->ncols) % s->nrows);
        int view = (int)(rayidx[m] / ((int64_t)s->ncols * s->nrows));
        ray_t ray;
        ray_of(s, view, r, c, &ray);
        out[m] = ray_sum(s, &ray, vol, NULL);
    }
    return 0;
}

int64_t sdo_nnz(const sdo_scan *s, int view_begin, int view_end)
{
    int64_t total = 0;
    int64_t lines = (int64_t)(view_end - view_begin) * s->nrows;
#pragma omp parallel for schedule(dynamic, 4) reduction(+ : total)
    for (int64_t l = 0; l < lines; ++l) {
        int view = view_begin + (int)(l / s->nrows), r = (int)(l % s->nrows);
        for (int c = 0; c < s->ncols; ++c) {
            ray_t ray;
            int64_t cnt = 0;
            ray_of(s, view, r, c, &ray);
            ray_sum(s, &ray, NULL, &cnt);
            total += cnt;
        }
    }
    return total;
}

/* ---- A^T: one voxel ------------------------------------------------------------------------------------------- */

/* Pixel-index range whose centres can lie between detector coordinates a and b (pitch p, `off` = index of coordinate
 * 0), widened by a hair; clipped to [0, n-1]. */
static void pixel_range(double a, double b, double p, double off, int n, int *i0, int *i1)
{
    double lo = fmin(a, b) / p + off, hi = fmax(a, b) / p + off;
    double fa = ceil(lo - 1e-9), fb = floor(hi + 1e-9);
    *i0 = fa < 0.0 ? 0 : (fa > n ? n : (int)fa);
    *i1 = fb > n - 1 ? n - 1 : (fb < -1.0 ? -1 : (int)fb);
}

/* Only rays whose pixel centre lies inside the bounding rectangle of the voxel's eight projected corners can meet
 * the voxel (a perspective or parallel image of a box is the hull of its projected corners; on a cylindrical
 * detector the rectangle is bounded separately, see below). */
static double voxel_sum(const sdo_scan *s, int i, int j, int k, const float *sino)
{
    double lo[3], hi[3], sum = 0.0;
    voxel_box(s, i, j, k, lo, hi);
    for (int view = 0; view < s->nviews; ++view) {
        double cphi = 1.0, sphi = 0.0;
        if (s->geom != SDO_MODULAR) { cphi = cos(s->phi[view]); sphi = sin(s->phi[view]); }
        double umin = INFINITY, umax = -INFINITY, vmin = INFINITY, vmax = -INFINITY;
        for (int corner = 0; corner < 8 && s->geom == SDO_MODULAR; ++corner) {
            /* central projection of the corner onto the detector plane; a corner that is not in front of the source
             * (seen from the detector) makes the search cover the whole detector */
            const double *S = s->poses + 12 * (int64_t)view, *C = S + 3, *uc = S + 6, *vr = S + 9;
            double X[3] = { (corner & 1) ? hi[0] : lo[0], (corner & 2) ? hi[1] : lo[1], (corner & 4) ? hi[2] : lo[2] };
            double nrm[3] = { uc[1] * vr[2] - uc[2] * vr[1], uc[2] * vr[0] - uc[0] * vr[2], uc[0] * vr[1] - uc[1] * vr[0] };
            double num = 0.0, den = 0.0;
            for (int a = 0; a < 3; ++a) { num += (C[a] - S[a]) * nrm[a]; den += (X[a] - S[a]) * nrm[a]; }
            if (!(num * den > 0.0)) { umin = vmin = -INFINITY; umax = vmax = INFINITY; break; }
            double u = 0.0, v = 0.0;
            for (int a = 0; a < 3; ++a) {
                double H = S[a] + (num / den) * (X[a] - S[a]) - C[a];
                u += H * uc[a]; v += H * vr[a];
            }
            umin = fmin(umin, u); umax = fmax(umax, u);
            vmin = fmin(vmin, v); vmax = fmax(vmax, v);
        }
        for (int corner = 0; corner < 8 && s->geom != SDO_MODULAR; ++corner) {
            double x = (corner & 1) ? hi[0] : lo[0], y = (corner & 2) ? hi[1] : lo[1], z = (corner & 4) ? hi[2] : lo[2];
            double t = -x * sphi + y * cphi, l = x * cphi + y * sphi;
            double mag = (s->geom == SDO_PARALLEL) ? 1.0 : s->sdd / (s->sod - l);
            double u = mag * t, v = mag * z;
            if (s->geom == SDO_CONE_CURVED) {
                /* on the cylinder: the fan angle is extreme at a corner; the height z SDD / (in-plane distance from
                 * the source) is bounded with the distance of the voxel centre -+ half a diagonal */
                double xc = 0.5 * (lo[0] + hi[0]), yc = 0.5 * (lo[1] + hi[1]);
                double rc = hypot(s->sod - (xc * cphi + yc * sphi), -xc * sphi + yc * cphi), hd = s->T * 0.70710678118654757;
                u = s->sdd * atan2(t, s->sod - l);
                v = z * s->sdd / (z >= 0.0 ? rc - hd : rc + hd);
                vmin = fmin(vmin, z * s->sdd / (z >= 0.0 ? rc + hd : rc - hd));
            }
            umin = fmin(umin, u); umax = fmax(umax, u);
            vmin = fmin(vmin, v); vmax = fmax(vmax, v);
        }
        int c0, c1, r0 = 0, r1 = 0;
        pixel_range(umin, umax, s->pu, 0.5 * (s->ncols - 1) - s->shift_u, s->ncols, &c0, &c1);
        if (s->geom != SDO_FAN)
            pixel_range(vmin, vmax, s->pv, 0.5 * (s->nrows - 1) - s->shift_v, s->nrows, &r0, &r1);
        for (int r = r0; r <= r1; ++r)
            for (int c = c0; c <= c1; ++c) {
                ray_t ray;
                ray_of(s, view, r, c, &ray);
                double w = chord(&ray, lo, hi);
                if (w > 0.0) sum += w * (double)sino[((int64_t)view * s->nrows + r) * s->ncols + c];
            }
    }
    return sum;
}

int sdo_backproject(const sdo_scan *s, const float *sino, double *vol)
{
    int64_t lines = (int64_t)s->nz * s->ny;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t l = 0; l < lines; ++l) {
        int k = (int)(l / s->ny), j = (int)(l % s->ny);
        for (int i = 0; i < s->nx; ++i) vol[l * s->nx + i] = voxel_sum(s, i, j, k, sino);
    }
    return 0;
}

int sdo_backproject_voxels(const sdo_scan *s, const float *sino, int64_t n, const int64_t *voxel, double *out)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t m = 0; m < n; ++m) {
        int i = (int)(voxel[m] % s->nx);
        int j = (int)((voxel[m] / s->nx) % s->ny);
        int k = (int)(voxel[m] / ((int64_t)s->nx * s->ny));
        out[m] = voxel_sum(s, i, j, k, sino);
    }
    return 0;
}

/* ---- dense matrix: every pair from the single-weight routine --------------------------------------------------- */

int sdo_dense_matrix(const sdo_scan *s, double *A)
{
    int64_t nvox = (int64_t)s->nx * s->ny * s->nz;
    int64_t nray = (int64_t)s->nviews * s->nrows * s->ncols;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < nray; ++m) {
        int c = (int)(m % s->ncols), r = (int)((m / s->ncols) % s->nrows);
        int view = (int)(m / ((int64_t)s->ncols * s->nrows));
        for (int k = 0; k < s->nz; ++k)
            for (int j = 0; j < s->ny; ++j)
                for (int i = 0; i < s->nx; ++i)
                    A[m * nvox + ((int64_t)k * s->ny + j) * s->nx + i] = sdo_weight(s, view, r, c, i, j, k);
    }
    return 0;
}

int sdo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
