// Library-private definitions shared by the host geometry module and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "../../include/leap.h"
#include "sf_types.h"
#include "sd_ray.h"
#include "md_siddon.h"

struct leap_geometry {
    leap_geometry_desc desc;            // caller's parameters (angles_rad re-pointed at `angles`)
    std::vector<double> angles;
    SfGeom g;                           // float parameter block handed to every kernel by value
    std::vector<SfView> views;          // host copy of the per-view table
    SfView *d_views = nullptr;          // device copy
    int device = -1;
    // static bounds of the footprints, derived in double at creation; they select the kernel family
    double max_cols_per_voxel = 0;      // widest transaxial footprint, in detector pixels
    double max_rows_per_voxel = 0;      // tallest axial footprint, in detector pixels
    double max_voxels_per_row = 0;      // tallest pixel, in voxels (at the smallest magnification)
    double max_minor_slope = 0;         // largest |d minor / d major| of any ray in its marching frame
    // tiled back projection: columns / rows read per voxel, half footprint width, and whether its limits hold
    int bp_nc = 0, bp_nv = 0, bp_shape = 0;   // bp_shape indexes BP_SHAPES
    float bp_wh = 0.f;
    bool bp_tiled = false;
    int bp_need_w = 0, bp_need_h = 0;   // largest staged window any (view, tile, chunk) asks for
    // column-wise forward projection: candidate slots per slab, voxels per detector row, row groups per wave
    int fp_nq = 0, fp_nk = 0, fp_rg = 0, fp_need_q = 0, fp_waves = 4, fp_cw = 4, fp_wv = 1, fp_vb = 128, fp_tb = 1;
    bool fp_columns = false;
    float *d_volz = nullptr;            // z-fastest padded copy of one volume (scratch)
    int nzp = 0;
    // Siddon model: per-(view, detector column) ray constants, host copy and device copy
    std::vector<SdRayCol> raycols;
    SdRayCol *d_raycols = nullptr;
    double sd_max_axial_slope = 0;      // largest |dZ/dX| of any ray: voxels of z crossed per slab
    // modular geometry: per-view poses, host copy and device copy
    std::vector<MdPose> poses;
    MdPose *d_poses = nullptr;
    // footprint model on upright modules: every view is a cone-beam view with its own parameter block
    std::vector<SfGeom> geoms;
    SfGeom *d_geoms = nullptr;
    void *d_colcs = nullptr;            // cylinder, tiled back projection: (cos, sin) of every column's fan angle, then the (tile, view) table
    int volz_items = 1;                 // scratch copies of the volume (items of a batch per forward launch)
    bool sd_columns = false;            // wave-per-column forward kernel (needs the scratch copy and slope <= 1)
};

void leap_set_error(const std::string &msg);
int leap_hip_fail(hipError_t e, const char *what);

#define LEAP_HIP_CHECK(expr)                                   \
    do {                                                       \
        hipError_t e__ = (expr);                               \
        if (e__ != hipSuccess) return leap_hip_fail(e__, #expr); \
    } while (0)

// Size of the file-scope device array behind leap_project_static_scratch (one per GPU the library runs on).
constexpr size_t LEAP_STATIC_SCRATCH_BYTES = (size_t)72 << 20;
// Looks up the array's address on `device` (which must be current) once; called from leap_geometry_create.
int leap_static_scratch_init(int device);

// kernel launchers (leap_kernels.hip); one batch item per call
int leap_launch_project(const leap_geometry *geom, const float *d_vol, float *d_sino, hipStream_t stream);
int leap_launch_project_batch(const leap_geometry *geom, const float *d_vol, float *d_sino, int batch, hipStream_t stream);
int leap_launch_backproject(const leap_geometry *geom, const float *d_sino, float *d_vol, hipStream_t stream);
int leap_launch_backproject_batch(const leap_geometry *geom, const float *d_sino, float *d_vol, int batch, hipStream_t stream);
