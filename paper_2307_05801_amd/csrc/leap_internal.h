// Library-private definitions shared by the host geometry module and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>

#include <mutex>
#include <string>
#include <vector>

#include "../../include/leap.h"
#include "sf_types.h"
#include "sd_ray.h"
#include "md_siddon.h"
#include "md_footprint.h"

struct MdBpView;                       // per-view table of the tiled Siddon back projection on tilted modules (md_backproject_tiled.h)
struct LeapHostStage;                  // streams, events, staging and device buffers of the host-memory entry points (leap_host.cpp)

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
    // column-wise forward projection (footprint and Siddon models): the volume goes through a z-fastest scratch copy
    // slab by slab (sf_project_columns.h)
    int fp_nq = 0, fp_need_q = 0;       // candidate slots per slab: instance / needed
    int fp_nkp = 0;                     // voxels a pair of adjacent detector rows can overlap
    int fp_rg = 0;                      // row groups per wave (footprints: groups of 128 rows; Siddon: of 64)
    int fp_cw = 4, fp_vb = 128, fp_tb = 1;   // detector columns per wave; block order: views per run, tiles per chunk
    bool fp_columns = false;
    float *d_volz = nullptr;            // the scratch: scratch_items copies of one slab
    size_t scratch_bytes = 0;           // bytes allocated at d_volz
    int slab_width = 0;                 // voxel layers across the marching axis per slab when one volume is projected
    int dbg_slab = 0, dbg_items = 0;    // debugging overrides of the slab width and the items per launch (0: none)
    int nzp = 0;                        // floats per padded z-column
    std::vector<unsigned char> major;   // footprints: [view][bundle of fp_cw columns] 1 if the bundle advances fastest along x
    unsigned char *d_major = nullptr;
    std::string note;                   // what went differently from the plan at creation (shown by leap_geometry_describe)
    // calls on one handle share its scratch: a call on another stream than the last first waits for that one's kernels
    mutable std::mutex scratch_mutex;
    mutable hipEvent_t scratch_event = nullptr;
    mutable hipStream_t scratch_stream = nullptr;
    mutable bool scratch_used = false;
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
    // footprint model on tilted modules: per-view table of the general kernels (md_footprint.h)
    std::vector<MfView> mfviews;
    MfView *d_mfviews = nullptr;
    void *d_colcs = nullptr;            // cylinder, tiled back projection: (cos, sin) of every column's fan angle, then the (tile, view) table
    // leap_project_host / leap_backproject_host: created by the first such call, freed with the handle
    mutable LeapHostStage *host_stage = nullptr;
    mutable std::mutex host_mutex;
    size_t stage_chunk = (size_t)32 << 20;   // bytes per pinned staging buffer
    MdBpView *d_mdbp = nullptr;         // Siddon model on tilted modules, tiled back projection: its per-view table
    bool md_tilted = false;             // Siddon model on tilted modules: the per-lane variants of the two fast kernels
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

// Slab width and batch items per launch that a scratch of `floats` floats affords (leap_geometry.cpp).
bool leap_plan_scratch(const leap_geometry *G, size_t floats, int batch, int &width, int &items);

// Frees what the host-memory entry points created on the handle (leap_host.cpp).
void leap_host_stage_free(leap_geometry *G);

// kernel launchers (leap_kernels.hip); one batch item per call
int leap_launch_project(const leap_geometry *geom, const float *d_vol, float *d_sino, hipStream_t stream);
int leap_launch_project_batch(const leap_geometry *geom, const float *d_vol, float *d_sino, int batch, hipStream_t stream);
int leap_launch_backproject(const leap_geometry *geom, const float *d_sino, float *d_vol, hipStream_t stream);
int leap_launch_backproject_batch(const leap_geometry *geom, const float *d_sino, float *d_vol, int batch, hipStream_t stream);
