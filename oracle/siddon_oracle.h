/*
 * CPU oracle for the Siddon projector pair (exact ray/voxel intersection lengths).  TEST INFRASTRUCTURE ONLY:
 * slow, double precision, independent of the HIP library (no shared code; the HIP library never calls it).
 *
 * What it follows: the paper's Method section ("CT Projection Models and Geometries") lists the Siddon method as
 * the second projector model it implements: line integrals along infinitely thin rays, without modelling the width
 * of voxels or detector pixels.  The weight of voxel j for ray i is the textbook quantity
 *
 *     w(i; j) = length of { points of ray i inside voxel j }          (mm)
 *
 * with one ray per detector pixel, through the pixel CENTRE:
 *     parallel : { u_c e_u + v_r e_v + s e_s , s real }
 *     cone     : the line through the source S = SOD e_s and the pixel centre P = (SOD-SDD) e_s + u_c e_u + v_r e_v
 *     fan      : the cone formula with v = 0 in the plane z = center_z; the voxel is its in-plane square
 *     curved   : cone-beam with a cylindrical detector of radius SDD around the source's vertical axis, columns equally
 *                spaced in arc length: P = S + SDD (-cos g e_s + sin g e_u) + v_r e_v with g = u_c / SDD
 *     modular  : the paper's flexible geometry ("the 3D location of every source-detector pair, as well as an arbitrary
 *                orientation of the detector"): view a has its own source position S_a, detector centre C_a and
 *                orthonormal detector axes ucol_a (along columns' index) and vrow_a (along rows' index), 12 doubles per
 *                view in `poses`; the ray of pixel (r, c) runs from S_a to C_a + u_c ucol_a + v_r vrow_a
 * (same world frame, voxel and pixel centres as the separable-footprint oracle, see sf_oracle.h).  A voxel is the
 * half-open box [lo, hi) on every axis, which only matters for a ray that runs exactly inside a face plane: it then
 * belongs to the voxel on the upper side.  A = sum over voxels, A^T = exact transpose.
 *
 * Parity pins: tests/test_siddon_pins.py (brute-force slab-method chords in numpy, total chord through the volume
 * box, analytic ellipsoids, hand-worked rays, dense transpose, symmetries, unit scaling, parallel limit).
 */
#ifndef SIDDON_ORACLE_H
#define SIDDON_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SDO_PARALLEL = 0, SDO_FAN = 1, SDO_CONE = 2, SDO_CONE_CURVED = 3, SDO_MODULAR = 4 };

typedef struct {
    int32_t geom;
    int32_t nviews, nrows, ncols;
    int32_t nx, ny, nz;
    double  pu, pv;
    double  shift_u, shift_v;
    double  sod, sdd;
    double  T, Tz;
    double  cx, cy, cz;
    const double *phi;
    const double *poses;   /* SDO_MODULAR only: nviews x {S[3], C[3], ucol[3], vrow[3]}; phi is not read then */
} sdo_scan;

/* chord length (mm) of ray (view, r, c) in voxel (i, j, k) */
double sdo_weight(const sdo_scan *s, int view, int r, int c, int i, int j, int k);

int sdo_project(const sdo_scan *s, const float *vol, double *sino);
int sdo_backproject(const sdo_scan *s, const float *sino, double *vol);
int sdo_project_rays(const sdo_scan *s, const float *vol, int64_t n, const int64_t *ray, double *out);
int sdo_backproject_voxels(const sdo_scan *s, const float *sino, int64_t n, const int64_t *voxel, double *out);
int sdo_dense_matrix(const sdo_scan *s, double *A);
int64_t sdo_nnz(const sdo_scan *s, int view_begin, int view_end);
int sdo_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
