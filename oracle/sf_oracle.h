/*
 * CPU oracle for the separable-footprint (SF) forward projector A and its exact
 * transpose A^T.  TEST INFRASTRUCTURE ONLY: slow, double precision, written for
 * checking by eye against the weight definition below.  It shares no code with the
 * HIP library and the HIP library never calls it.
 *
 * What it follows: the paper's Method section states the operator (y = A x, the X-ray
 * transform of a voxelised volume, "CT Projection Models and Geometries"), names the
 * SF model that accounts for finite voxel and detector-pixel width, requires the back
 * projector to be the exact transpose, and requires quantitative mm / 1/mm scaling.
 * The paper prints no formula for the SF weights; the reading used here is the
 * trapezoid (transaxial) x rectangle (axial) footprint with a ray-dependent amplitude:
 *
 *   world:  voxel centres  x_i = cx + (i-(nx-1)/2) T,  y_j likewise,  z_k = cz + (k-(nz-1)/2) Tz
 *           pixel centres  u_c = (c-(ncols-1)/2+shift_u) pu,  v_r = (r-(nrows-1)/2+shift_v) pv
 *           view angle phi: e_s=(cos,sin,0) points at the source, e_u=(-sin,cos,0), e_v=(0,0,1)
 *           for a point X:  t = X.e_u,  l = X.e_s
 *           parallel ray (r,c) = { u_c e_u + v_r e_v + s e_s };  cone/fan: source S = SOD e_s,
 *           detector plane at l = SOD-SDD, pixel P = (SOD-SDD) e_s + u_c e_u + v_r e_v
 *   step 1  knots tau_0<=..<=tau_3: the detector-u coordinates of the voxel's four in-plane
 *           corners (x+-T/2, y+-T/2), sorted.  parallel u = t;  cone/fan u = SDD t/(SOD-l)
 *   step 2  unit-height trapezoid on those knots, G its running integral,
 *           F_u = [G(u_c+pu/2) - G(u_c-pu/2)] / pu
 *   step 3  axial interval [v-,v+] = m (z_k -+ Tz/2) with m = 1 (parallel) or the magnification
 *           SDD/(SOD-l) at the voxel CENTRE (cone);  F_v = overlap([v_r-pv/2, v_r+pv/2],[v-,v+]) / pv;
 *           fan: F_v = 1
 *   step 4  amp = T |D| / max(|D_x|,|D_y|), D the ray direction (parallel -e_s; cone P-S; fan: v_r:=0)
 *   weight  w(view,r,c; i,j,k) = amp * F_u * F_v      (mm)
 *   A       y[view][r][c] = sum_voxels w x[k][j][i];     A^T  x[k][j][i] = sum_rays w y[view][r][c]
 *
 * Curved detector (SFO_CONE_CURVED; the paper's "axial cone-beam (planar or curved)"): the detector is the cylinder
 * of radius SDD around the vertical line through the source; its columns are equally spaced in arc length, so pixel
 * (r,c) sits at the fan angle gamma_c = u_c / SDD:  P = S + SDD (-cos gamma e_s + sin gamma e_u) + v_r e_v.  The same
 * four steps apply with the detector coordinate of a point taken on the cylinder: u = SDD atan2(t, SOD-l) (arc
 * length) in step 1, and the magnification in step 3 is SDD over the in-plane distance of the voxel centre from the
 * source, SDD / hypot(SOD-l, t).  Step 4 uses D = P - S as before.
 *
 * Modular geometry (SFO_MODULAR; the paper's flexible geometry with a pose per view).  The paper gives no footprint
 * construction for it.  UPRIGHT modules (column axis horizontal, row axis +z): the cone-beam construction carried out in
 * each view's own frame: e_u = the module's column axis, e_s = the horizontal unit vector orthogonal to it on the
 * source's side, source at (l, t, z) = (lS, tS, zS), detector plane at l = lS - sdd_a with its centre at (tC, zC).
 * Step 1: u = tS + sdd_a (t - tS)/(lS - l) - tC; step 3: magnification sdd_a/(lS - l) about the source height,
 * [v-,v+] = zS + m (z_k -+ Tz/2 - zS) - zC; step 4: D = pixel - source.
 * TILTED modules (any other orthonormal axes): the same separable footprint on the module's own (u, v) axes.  Step 1: the
 * knots are the u coordinates of the central projections (from the source onto the module's plane) of the voxel's four
 * in-plane corners, taken at the height of the voxel's centre; step 3: [v-,v+] spans the v coordinates of the central
 * projections of the centres of the voxel's lower and upper face; steps 2 and 4 unchanged.  For an upright module
 * these are the expressions above, so the readings meet as the tilt goes to zero.  The whole volume must lie in front of
 * the source (else the calls return -1).
 *
 * Footprints partly off the detector are truncated; rays that miss the volume give 0.
 * For parallel-beam w * pu * pv equals the volume of (pixel beam  intersect  voxel) exactly.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (hand-worked
 * values, mass invariants, brute-force chord quadrature, analytic ellipsoids, dense
 * transpose, symmetries, the parallel limit, unit scaling).
 */
#ifndef SF_ORACLE_H
#define SF_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SFO_PARALLEL = 0, SFO_FAN = 1, SFO_CONE = 2, SFO_CONE_CURVED = 3, SFO_MODULAR = 4 };

typedef struct {
    int32_t geom;
    int32_t nviews, nrows, ncols;
    int32_t nx, ny, nz;
    double  pu, pv;              /* pixel width (u) and height (v), mm */
    double  shift_u, shift_v;    /* detector shifts, pixels */
    double  sod, sdd;            /* mm */
    double  T, Tz;               /* voxel size in-plane and axial, mm */
    double  cx, cy, cz;          /* volume centre, mm */
    const double *phi;           /* nviews angles, radians */
    const double *poses;         /* SFO_MODULAR only: nviews x {S[3], C[3], ucol[3], vrow[3]}; phi is not read then */
} sfo_scan;

/* One weight and its factors, straight from the definition (any of the out pointers may be NULL). */
double sfo_weight(const sfo_scan *s, int view, int r, int c, int i, int j, int k,
                  double *Fu, double *Fv, double *amp);

/* The four sorted knots (mm on the detector u axis) and the axial magnification of voxel column (i,j). */
void sfo_knots(const sfo_scan *s, int view, int i, int j, double tau[4], double *mag);

/* Running integral G of the unit-height trapezoid with the given knots, at u. */
double sfo_trapezoid_integral(const double tau[4], double u);

/* y = A x.  vol: float32 [nz][ny][nx];  sino: double [nviews][nrows][ncols], overwritten. */
int sfo_project(const sfo_scan *s, const float *vol, double *sino);

/* x = A^T y.  sino: float32 [nviews][nrows][ncols];  vol: double [nz][ny][nx], overwritten. */
int sfo_backproject(const sfo_scan *s, const float *sino, double *vol);

/* A^T y at n listed voxels only (linear index (k*ny+j)*nx+i), one by one. */
int sfo_backproject_voxels(const sfo_scan *s, const float *sino, int64_t n, const int64_t *voxel, double *out);

/* A x at n listed rays only (linear index (view*nrows+r)*ncols+c), one by one. */
int sfo_project_rays(const sfo_scan *s, const float *vol, int64_t n, const int64_t *ray, double *out);

/* Dense A, row-major [nviews*nrows*ncols][nz*ny*nx], every (ray,voxel) pair from sfo_weight: tiny grids only. */
int sfo_dense_matrix(const sfo_scan *s, double *A);

/* Number of (ray,voxel) pairs with w > 0 over views [view_begin, view_end). */
int64_t sfo_nnz(const sfo_scan *s, int view_begin, int view_end);

/* Threads the parallel loops will use. */
int sfo_num_threads(void);
void sfo_set_num_threads(int n);

#ifdef __cplusplus
}
#endif
#endif
