/*
 * leap.h - C ABI of the MI355X CT projector pairs (separable footprint and Siddon).
 *
 * The library computes, on one GPU, the forward projector A (line integrals of a voxel
 * volume along every source-detector ray) and its exact transpose A^T for parallel-,
 * fan- and flat-panel cone-beam scanners.  The operator and its transpose are the ones
 * the paper states in its Method section ("CT Projection Models and Geometries":
 * y = A x, back projection as the exact transpose, quantities in mm and 1/mm), for the two
 * projector models named there: separable-footprint weights, which model finite voxel and
 * detector-pixel width, and Siddon weights, the exact length of the thin ray through each
 * pixel centre inside each voxel.  The calling
 * convention follows "Core CUDA Implementation" (the user hands over pointers to
 * contiguous 32-bit float arrays) and "PyTorch Interfaces and CT Parameters" (the list
 * of scanner parameters).
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *     frees or keeps them.  Host arrays are not staged (the caller copies).
 *   - volume   : float32 [batch][nz][ny][nx], x fastest.
 *     sinogram : float32 [batch][nviews][nrows][ncols], column fastest.
 *   - Outputs are OVERWRITTEN, never accumulated into.
 *   - Calls are asynchronous on the given HIP stream (hipStream_t passed as void*, NULL =
 *     the default stream) and allocate nothing.  Per-view tables are uploaded once, in
 *     leap_geometry_create.  Device memory beyond the caller's arrays ("Performance and
 *     Memory Usage" asks for one copy of each array only): the fast forward kernels read the
 *     volume through a z-fastest scratch copy, one SLAB of the volume at a time, so the handle
 *     owns a scratch of at most max(64 MiB, an eighth of one volume) -- leap_geometry_describe
 *     reports its size as "scratch=<bytes>"; small volumes share it between the items of a batch.
 *     If it cannot be allocated the handle works without it on a slower kernel, says so in
 *     leap_last_error at creation and in a "note=" of leap_geometry_describe.  A
 *     LEAP_MODEL_SIDDON handle also keeps a table of 48 bytes per (view, detector column): the
 *     constants of each ray's line; a LEAP_CONE_CURVED footprint handle 24 bytes per (16x16
 *     voxel-column tile, view).  leap_project calls on one handle share its scratch; the library
 *     orders them on the device (a call arriving on another stream than the previous one first
 *     waits for that one's kernels), so any stream may be used; distinct handles are independent.
 *   - World frame: voxel centres x_i = center_x + (i-(nx-1)/2) voxel_xy (y, z alike); view
 *     angle phi counter-clockwise from +x, the source sits at sod*(cos phi, sin phi, 0);
 *     detector columns grow along (-sin phi, cos phi, 0), rows along +z; pixel centres
 *     u_c = (c-(ncols-1)/2+shift_u) pixel_u, v_r = (r-(nrows-1)/2+shift_v) pixel_v.
 *   - Every function returns LEAP_OK (0) or a negative status; nothing throws or aborts.
 */
#ifndef LEAP_H
#define LEAP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Scanner families ("CT Projection Models and Geometries": parallel-beam, axial cone-beam with a planar or a curved
 * detector; fan-beam is the one-row, one-slice case of the flat-panel cone-beam scanner).  LEAP_CONE_CURVED: the
 * detector is the cylinder of radius sdd around the vertical line through the source; columns are equally spaced in
 * arc length (pixel_u mm), so pixel (r, c) sits at fan angle u_c / sdd and height v_r on the cylinder.
 * LEAP_MODULAR: the flexible geometry of the same section (sources and detectors at any position and orientation):
 * every view has its own pose, 12 doubles in `poses`: source position S, detector centre C, unit vector along the
 * column index, unit vector along the row index (orthogonal to each other); pixel (r, c) sits at
 * C + u_c ucol + v_r vrow.  sod, sdd and angles_rad are not read.  LEAP_MODEL_SIDDON takes any pose (one limit: a scan
 * of more than 5e11 voxel-pixel pairs in views whose volume reaches behind the plane through the source parallel to the
 * module is LEAP_UNSUPPORTED; the back projection of such views has no bound on a voxel's pixel search).
 * LEAP_MODEL_SF on upright modules (ucol horizontal, vrow = +z): the cone-beam footprint construction is carried out
 * in each view's own frame.  On any other module (the paper gives no construction) the footprint stays separable on
 * the module's own axes: the trapezoid's knots are the column coordinates of the central projections, from the source
 * onto the module's plane, of the voxel's four in-plane corners at the height of its centre; the axial interval lies
 * between the row coordinates of the central projections of the centres of its lower and upper face; the amplitude is
 * T |D| / max(|Dx|, |Dy|) with D = pixel - source.  A scan with one such module runs on one thread per few rays / per voxel
 * in double precision.  It needs the whole volume in front of every source (on the module's side of the plane through
 * the source parallel to the module) and no pixel whose ray runs along z, else LEAP_BAD_GEOMETRY; a source so close to
 * the volume that the nearest voxel's footprint spans more than 64 pixels is LEAP_UNSUPPORTED. */
enum { LEAP_PARALLEL = 0, LEAP_FAN = 1, LEAP_CONE = 2, LEAP_CONE_CURVED = 3, LEAP_MODULAR = 4 };

/* Projector models ("CT Projection Models and Geometries").  LEAP_MODEL_SF: separable footprints.
 * LEAP_MODEL_SIDDON: weight = length (mm) of the ray through the pixel centre inside the voxel; a voxel is
 * the half-open box [lo, hi) on every axis, so a ray running inside a face plane belongs to the voxel above. */
enum { LEAP_MODEL_SF = 0, LEAP_MODEL_SIDDON = 1 };

enum {
    LEAP_OK = 0,
    LEAP_INVALID_ARG = -1,   /* null pointer, non-positive size or count, unknown type or model, FAN with nrows != 1 or nz != 1 */
    LEAP_BAD_GEOMETRY = -2,  /* cone/fan: source not strictly outside the volume's bounding circle, sdd <= 0, curved fan wider than +-1.5 rad;
                                modular: a source inside the volume, a module with no footprints (see LEAP_MODULAR) */
    LEAP_HIP_ERROR = -3,     /* a HIP runtime call failed (the message is kept, see leap_last_error) */
    LEAP_UNSUPPORTED = -4    /* sizes beyond what the index arithmetic of the kernels covers; footprints of more than 64 pixels on a tilted module;
                                a volume beyond the fixed array of leap_project_static_scratch */
};

/* The CT parameter set of "PyTorch Interfaces and CT Parameters": geometry type, number of
 * projections, list of projection angles, detector pixel width and height, source-to-detector
 * and source-to-object distance, horizontal/vertical detector shift, voxel counts, voxel sizes,
 * volume centre.  Host memory; copied by leap_geometry_create. */
typedef struct {
    int32_t type;                 /* LEAP_PARALLEL / LEAP_FAN / LEAP_CONE / LEAP_CONE_CURVED / LEAP_MODULAR */
    int32_t nviews, nrows, ncols; /* projections, detector rows (v), detector columns (u) */
    int32_t nx, ny, nz;           /* voxels */
    double  pixel_v, pixel_u;     /* mm: pixel height, pixel width */
    double  shift_v, shift_u;     /* detector shift in PIXELS; positive moves pixel centres to +v / +u */
    double  sod, sdd;             /* mm: source to rotation axis, source to detector; ignored for PARALLEL */
    double  voxel_xy, voxel_z;    /* mm: in-plane voxels are square */
    double  center_x, center_y, center_z; /* mm: volume centre */
    const double *angles_rad;     /* nviews view angles, any spacing (not read for LEAP_MODULAR) */
    int32_t model;                /* LEAP_MODEL_SF (0, so a zero-filled struct keeps the footprint model) / LEAP_MODEL_SIDDON */
    const double *poses;          /* LEAP_MODULAR only: nviews x 12 doubles {S[3], C[3], ucol[3], vrow[3]}, mm; else ignored */
} leap_geometry_desc;

typedef struct leap_geometry leap_geometry;   /* opaque; owned by the library */

/* Validates `desc`, derives the per-view constant tables in double precision and uploads them to
 * the current HIP device.  On success *out receives a handle valid on that device until
 * leap_geometry_destroy.  Blocking (synchronous upload). */
int leap_geometry_create(const leap_geometry_desc *desc, leap_geometry **out);

/* Frees the handle's host and device tables.  NULL is ignored.  The caller must have
 * synchronised every stream that still uses the handle. */
void leap_geometry_destroy(leap_geometry *geom);

/* Forward projection y = A x ("CT Projection Models and Geometries", y = A x), ray-driven gather:
 * d_sino[b] = A d_vol[b] for b < batch.  d_vol: batch volumes, d_sino: batch sinograms (layouts above),
 * both device memory, not overlapping.  Asynchronous on hip_stream.  Uses the handle's scratch (see above). */
int leap_project(const leap_geometry *geom, const float *d_vol, float *d_sino, int32_t batch, void *hip_stream);

/* Back projection x = A^T y, the exact transpose of leap_project ("matched projectors"), voxel-driven
 * gather without atomics (bitwise reproducible): d_vol[b] = A^T d_sino[b].  Asynchronous on hip_stream. */
int leap_backproject(const leap_geometry *geom, const float *d_sino, float *d_vol, int32_t batch, void *hip_stream);

/* leap_project for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same result as leap_project, same kernels; the z-fastest copy of
 * the volume's slabs is kept in a fixed array of 72 MiB inside the library's device code (every GPU the library runs
 * on holds that array until the process ends) instead of the handle's own scratch.  The call allocates and frees
 * nothing and calls no allocating routine; the array's address is looked up once per device in leap_geometry_create.
 * Limit: four voxel layers of the copy, 4 * max(nx, ny) * (nz + 16) floats, must fit the array (volumes up to about
 * 2000^3 do; the fewer layers fit, the more passes the call makes), else LEAP_UNSUPPORTED with a message; geometries
 * whose forward kernel reads the caller's volume directly (fan-beam, tilted Siddon modules, very coarse detectors)
 * have no limit.  Items of a batch share the array, as many per launch as fit.  All calls on one GPU share the one
 * array, whatever the handle: calls that overlap in time on one GPU (two streams, two threads) race; order them.
 * The array keeps the last call's contents; each call restores the zeros it relies on. */
int leap_project_static_scratch(const leap_geometry *geom, const float *d_vol, float *d_sino, int32_t batch, void *hip_stream);

/* The pair on arrays in HOST memory ("Core CUDA Implementation": data may live on the CPU, the library moves it;
 * "Performance and Memory Usage" quotes times with and without that transfer).  h_vol, h_sino: host memory, layouts
 * as above, pageable or pinned, not overlapping.  Synchronous: the result is in place when the call returns.  The
 * items of a batch run through a three-stage pipeline: item b+1 is uploaded while item b is projected and item b-1
 * is downloaded, on three streams of the library's own (default priority).  Pageable memory is staged through four
 * pinned buffers of 32 MiB, so that the CPU's copy of one chunk overlaps the DMA of the previous one; pinned memory
 * (hipHostMalloc) goes to the DMA engines directly.  The first such call on a handle allocates, on the handle, two
 * device arrays per direction (one for batch 1) of max(volume, sinogram) size, the pinned buffers, streams and
 * events; leap_geometry_destroy frees them.  Calls on one handle are serialised.  The handle's device must be current.
 * Returns LEAP_HIP_ERROR if an allocation or a copy fails. */
int leap_project_host(const leap_geometry *geom, const float *h_vol, float *h_sino, int32_t batch);
int leap_backproject_host(const leap_geometry *geom, const float *h_sino, float *h_vol, int32_t batch);

/* ---- iterative reconstruction on top of the pair ------------------------------------------------------------
 * "CT Projection Models and Geometries" motivates the matched transpose with the least-squares cost
 * 1/2 ||A x - y||^2, whose gradient is A^T (A x - y), and with iterations that stay stable over a thousand or
 * more steps.  Both solvers below run entirely on the caller's stream (projector calls, streaming elementwise
 * kernels, reductions whose results stay on the device), allocate nothing and never synchronise with the host.
 * One volume and one sinogram (batch 1).  d_work: device memory of leap_recon_workspace_floats() floats, contents
 * undefined before and after. */

/* Number of floats the solvers need in d_work: 2 sinograms + 2 volumes + a small reduction scratch. */
int leap_recon_workspace_floats(const leap_geometry *geom, int64_t *n_floats);

/* SIRT: x <- x + relaxation * C .* A^T ( R .* (y - A x) ), `iterations` times, with R = 1 / (A 1) per ray and
 * C = 1 / (A^T 1) per voxel (0 where the sum is 0).  d_vol holds the start value on entry and the result on return;
 * nonneg != 0 clips every update at zero from below. */
int leap_sirt(const leap_geometry *geom, const float *d_sino, float *d_vol, float *d_work, int32_t iterations,
              float relaxation, int32_t nonneg, void *hip_stream);

/* Steepest descent on 1/2 ||A x - y||^2 with the exact line search: g = A^T (A x - y), x <- x - (|g|^2 / |A g|^2) g,
 * `iterations` times (the step length is formed on the device, in double). */
int leap_least_squares_descent(const leap_geometry *geom, const float *d_sino, float *d_vol, float *d_work,
                               int32_t iterations, void *hip_stream);

/* Static description of a status code. */
const char *leap_status_string(int status);

/* Message of the most recent failure on the calling thread (empty string if none). */
const char *leap_last_error(void);

/* Which kernel family the handle dispatches to: writes up to `cap` bytes of a short NUL-terminated
 * description (for logs and benchmarks): "A=..." and "AT=..." name the forward and the back projection kernel and
 * their instance, "scratch=<bytes>" the device memory the handle owns beyond its tables, "note=..." anything that went
 * differently from the plan at creation.  Returns LEAP_OK or LEAP_INVALID_ARG.
 *
 * Debugging aid: the environment variable LEAP_DEBUG, read by leap_geometry_create, overrides the choices shown
 * there.  Comma-separated key=value pairs: general=1 (no fast kernels), cw=1|2|4 (detector columns per wavefront),
 * rg=1|2|4|8 (row groups per wavefront), vb=N / tb=N (views per run / tiles per chunk of the block order), bp_shape=0..4
 * (first back-projection tile shape tried), slab=N (voxel layers per scratch slab), items=N (batch items per launch),
 * scratch_mib=N (scratch budget), stage_kib=N (size of a pinned staging buffer of the host-memory entry points). */
int leap_geometry_describe(const leap_geometry *geom, char *buf, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif
