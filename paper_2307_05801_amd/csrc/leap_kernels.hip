// HIP kernels (gfx950) and launchers of the projector pairs (separable footprint and Siddon).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <mutex>

#include "leap_internal.h"
#include "sf_general.h"
#include "sf_backproject_tiled.h"
#include "sf_project_columns.h"
#include "sd_project_columns.h"
#include "md_project_columns.h"
#include "sd_backproject_tiled.h"
#include "md_backproject_tiled.h"

// ------------------------------------------------------------------------------------------------
// General kernels: plain loop nests over global memory, valid for every validated geometry.
// ------------------------------------------------------------------------------------------------

constexpr int GEN_ZC = 8;   // voxels along z per back-projection thread
constexpr int GEN_RC = 8;   // detector rows per forward-projection thread

// grid: x = ceil(nx/64), y = ceil(ny/4), z = ceil(nz/GEN_ZC); block 64x4.
__global__ __launch_bounds__(256) void sf_backproject_general(SfGeom g, const SfView *__restrict__ views,
                                                              const float *__restrict__ sino, float *__restrict__ vol)
{
    const int i = blockIdx.x * 64 + threadIdx.x;
    const int j = blockIdx.y * 4 + threadIdx.y;
    const int k0 = blockIdx.z * GEN_ZC;
    if (i >= g.nx || j >= g.ny) return;
    float acc[GEN_ZC];
#pragma unroll
    for (int kk = 0; kk < GEN_ZC; ++kk) acc[kk] = 0.0f;
    sf_backproject_column_chunk<GEN_ZC>(g, views, sino, i, j, k0, acc);
#pragma unroll
    for (int kk = 0; kk < GEN_ZC; ++kk)
        if (k0 + kk < g.nz) vol[((size_t)(k0 + kk) * g.ny + j) * g.nx + i] = acc[kk];
}

// grid: x = ceil(ncols/64), y = ceil(ceil(nrows/GEN_RC)/4), z = nviews; block 64x4.
__global__ __launch_bounds__(256) void sf_project_general(SfGeom g, const SfView *__restrict__ views,
                                                          const float *__restrict__ vol, float *__restrict__ sino)
{
    const int c = blockIdx.x * 64 + threadIdx.x;
    const int r0 = (blockIdx.y * 4 + threadIdx.y) * GEN_RC;
    const int a = blockIdx.z;
    if (c >= g.ncols || r0 >= g.nrows) return;
    const SfView v = views[a];
    float out[GEN_RC];
    sf_project_ray_chunk<GEN_RC>(g, v, vol, c, r0, out);
    float *__restrict__ y = sino + ((size_t)a * g.nrows) * g.ncols + c;
#pragma unroll
    for (int rr = 0; rr < GEN_RC; ++rr)
        if (r0 + rr < g.nrows) y[(size_t)(r0 + rr) * g.ncols] = out[rr];
}

// Modular geometry, footprint model on upright modules: the general bodies with one parameter block per view.
__global__ __launch_bounds__(256) void sf_backproject_general_modular(SfGeom g, const SfGeom *__restrict__ geoms,
                                                                      const SfView *__restrict__ views,
                                                                      const float *__restrict__ sino, float *__restrict__ vol)
{
    const int i = blockIdx.x * 64 + threadIdx.x;
    const int j = blockIdx.y * 4 + threadIdx.y;
    const int k0 = blockIdx.z * GEN_ZC;
    if (i >= g.nx || j >= g.ny) return;
    float acc[GEN_ZC];
#pragma unroll
    for (int kk = 0; kk < GEN_ZC; ++kk) acc[kk] = 0.0f;
    sf_backproject_column_chunk<GEN_ZC>(g, views, sino, i, j, k0, acc, geoms);
#pragma unroll
    for (int kk = 0; kk < GEN_ZC; ++kk)
        if (k0 + kk < g.nz) vol[((size_t)(k0 + kk) * g.ny + j) * g.nx + i] = acc[kk];
}

__global__ __launch_bounds__(256) void sf_project_general_modular(const SfGeom *__restrict__ geoms,
                                                                  const SfView *__restrict__ views,
                                                                  const float *__restrict__ vol, float *__restrict__ sino)
{
    const int a = blockIdx.z;
    const SfGeom g = geoms[a];
    const int c = blockIdx.x * 64 + threadIdx.x;
    const int r0 = (blockIdx.y * 4 + threadIdx.y) * GEN_RC;
    if (c >= g.ncols || r0 >= g.nrows) return;
    const SfView v = views[a];
    float out[GEN_RC];
    sf_project_ray_chunk<GEN_RC>(g, v, vol, c, r0, out);
    float *__restrict__ y = sino + ((size_t)a * g.nrows) * g.ncols + c;
#pragma unroll
    for (int rr = 0; rr < GEN_RC; ++rr)
        if (r0 + rr < g.nrows) y[(size_t)(r0 + rr) * g.ncols] = out[rr];
}

// Modular geometry, footprint model on tilted modules (md_footprint.h): one thread per MF_RC rows of a detector column /
// per voxel.  Forward grid: x = ceil(ncols/64), y = ceil(ceil(nrows/MF_RC)/4), z = nviews; back grid as for the general
// Siddon kernel below.
#ifndef MF_RC_VALUE
#define MF_RC_VALUE 8
#endif
constexpr int MF_RC = MF_RC_VALUE;
__global__ __launch_bounds__(256) void mf_project_general(SfGeom g, const MfView *__restrict__ views,
                                                          const float *__restrict__ vol, float *__restrict__ sino)
{
    const int c = blockIdx.x * 64 + threadIdx.x;
    const int r0 = (blockIdx.y * 4 + threadIdx.y) * MF_RC;
    const int a = blockIdx.z;
    if (c >= g.ncols || r0 >= g.nrows) return;
    float out[MF_RC];
    mf_project_rows<MF_RC>(g, views[a], vol, r0, c, out);
    float *__restrict__ y = sino + ((size_t)a * g.nrows) * g.ncols + c;
#pragma unroll
    for (int rr = 0; rr < MF_RC; ++rr)
        if (r0 + rr < g.nrows) y[(size_t)(r0 + rr) * g.ncols] = out[rr];
}

__global__ __launch_bounds__(256) void mf_backproject_general(SfGeom g, const MfView *__restrict__ views,
                                                              const float *__restrict__ sino, float *__restrict__ vol)
{
    const int i = blockIdx.x * 64 + threadIdx.x;
    const int j = blockIdx.y * 4 + threadIdx.y;
    const int k = blockIdx.z;
    if (i >= g.nx || j >= g.ny) return;
    vol[((size_t)k * g.ny + j) * g.nx + i] = mf_backproject_voxel(g, views, sino, i, j, k);
}

// Siddon model, general kernels: one thread per ray / per voxel.
// grid: x = ceil(ncols/64), y = ceil(nrows/4), z = nviews; block 64x4.
__global__ __launch_bounds__(256) void sd_project_general(SfGeom g, const SdRayCol *__restrict__ rays,
                                                          const float *__restrict__ vol, float *__restrict__ sino)
{
    const int c = blockIdx.x * 64 + threadIdx.x;
    const int r = blockIdx.y * 4 + threadIdx.y;
    const int a = blockIdx.z;
    if (c >= g.ncols || r >= g.nrows) return;
    const SdRayCol R = rays[(size_t)a * g.ncols + c];
    sino[((size_t)a * g.nrows + r) * g.ncols + c] = sd_project_ray(g, R, vol, r);
}

// grid: x = ceil(nx/64), y = ceil(ny/4), z = nz; block 64x4.
__global__ __launch_bounds__(256) void sd_backproject_general(SfGeom g, const SfView *__restrict__ views,
                                                              const SdRayCol *__restrict__ rays,
                                                              const float *__restrict__ sino, float *__restrict__ vol)
{
    const int i = blockIdx.x * 64 + threadIdx.x;
    const int j = blockIdx.y * 4 + threadIdx.y;
    const int k = blockIdx.z;
    if (i >= g.nx || j >= g.ny) return;
    vol[((size_t)k * g.ny + j) * g.nx + i] = sd_backproject_voxel(g, views, rays, sino, i, j, k);
}

// Modular geometry, Siddon model: one thread per ray / per voxel.  Same grids as the general Siddon kernels.
__global__ __launch_bounds__(256) void md_project_general(SfGeom g, const MdPose *__restrict__ poses,
                                                          const float *__restrict__ vol, float *__restrict__ sino)
{
    const int c = blockIdx.x * 64 + threadIdx.x;
    const int r = blockIdx.y * 4 + threadIdx.y;
    const int a = blockIdx.z;
    if (c >= g.ncols || r >= g.nrows) return;
    const MdPose P = poses[a];
    sino[((size_t)a * g.nrows + r) * g.ncols + c] = md_project_ray(g, P, vol, r, c);
}

__global__ __launch_bounds__(256) void md_backproject_general(SfGeom g, const MdPose *__restrict__ poses,
                                                              const float *__restrict__ sino, float *__restrict__ vol)
{
    const int i = blockIdx.x * 64 + threadIdx.x;
    const int j = blockIdx.y * 4 + threadIdx.y;
    const int k = blockIdx.z;
    if (i >= g.nx || j >= g.ny) return;
    vol[((size_t)k * g.ny + j) * g.nx + i] = md_backproject_voxel(g, poses, sino, i, j, k);
}

static inline unsigned cdiv(unsigned a, unsigned b) { return (a + b - 1) / b; }

constexpr int SD_WAVES = 4;   // adjacent detector columns per workgroup of the Siddon forward kernel

// Where the column-wise forward kernels find their z-fastest copy of a slab: the handle's own scratch, or the library's
// fixed array (leap_project_static_scratch).
struct FwdScratch {
    float *volz;
    size_t item_floats;     // floats per copy (one per item of a batch in flight): (columns of a slab + 1) * nzp
    int width;              // voxel layers across the marching axis per slab
    int items;              // copies
};

template <int RG>
static void launch_sd_columns(const leap_geometry *G, const FwdScratch &S, const SfSlab &slab, float *d_sino, hipStream_t stream, int items)
{
    const SfGeom &g = G->g;
    const int col_tiles = (int)cdiv(g.ncols, SD_WAVES), bands = (int)cdiv(g.nrows, RG * 64);
    const int vb = G->fp_vb, tb = G->fp_tb;
    const int views_pad = (int)cdiv(g.nviews, vb) * vb;
    const int tiles_per_xcd_pad = (int)cdiv(cdiv(col_tiles, 8), tb) * tb;
    const unsigned zero_col = (unsigned)(S.item_floats - (size_t)G->nzp);      // the copy's last column stays zero
    dim3 grid((unsigned)(8 * tiles_per_xcd_pad * views_pad * bands), (unsigned)items, 1);
    if (G->md_tilted) {
        if constexpr (RG <= 4)        // (the selection offers the per-lane kernel 1, 2 or 4 row groups)
            hipLaunchKernelGGL((md_project_columns<RG, SD_WAVES>), grid, dim3(SD_WAVES * 64, 1, 1), 0, stream, g,
                               (const MdPose *)G->d_poses, S.volz, d_sino, G->nzp, S.item_floats, zero_col, col_tiles, bands, vb, tb,
                               views_pad, tiles_per_xcd_pad, slab);
    } else if (g.type == SF_MODULAR)
        hipLaunchKernelGGL((sd_project_columns<RG, SD_WAVES, true>), grid, dim3(SD_WAVES * 64, 1, 1), 0, stream, g, G->d_raycols,
                           S.volz, d_sino, G->nzp, S.item_floats, zero_col, col_tiles, bands, vb, tb, views_pad, tiles_per_xcd_pad,
                           slab, (const SfGeom *)G->d_geoms);
    else
        hipLaunchKernelGGL((sd_project_columns<RG, SD_WAVES, false>), grid, dim3(SD_WAVES * 64, 1, 1), 0, stream, g, G->d_raycols,
                           S.volz, d_sino, G->nzp, S.item_floats, zero_col, col_tiles, bands, vb, tb, views_pad, tiles_per_xcd_pad,
                           slab, (const SfGeom *)nullptr);
}

static bool launch_sd_slab(const leap_geometry *G, const FwdScratch &S, const SfSlab &slab, float *d_sino, hipStream_t stream, int items)
{
    switch (G->fp_rg) {
    case 1: launch_sd_columns<1>(G, S, slab, d_sino, stream, items); return true;
    case 2: launch_sd_columns<2>(G, S, slab, d_sino, stream, items); return true;
    case 4: launch_sd_columns<4>(G, S, slab, d_sino, stream, items); return true;
    case 8: launch_sd_columns<8>(G, S, slab, d_sino, stream, items); return true;
    default: return false;
    }
}

static int run_forward_columns(const leap_geometry *G, const FwdScratch &S, const float *d_vol, float *d_sino, int batch,
                               hipStream_t stream);

static int launch_sd_project(const leap_geometry *G, const float *d_vol, float *d_sino, hipStream_t stream)
{
    const SfGeom &g = G->g;
    if (g.type == SF_MODULAR && !G->sd_columns) {     // sizes were checked against the grid limits at creation
        dim3 grid(cdiv(g.ncols, 64), cdiv(g.nrows, 4), g.nviews);
        hipLaunchKernelGGL(md_project_general, grid, dim3(64, 4, 1), 0, stream, g, G->d_poses, d_vol, d_sino);
        LEAP_HIP_CHECK(hipGetLastError());
        return LEAP_OK;
    }
    if (G->sd_columns) return leap_launch_project_batch(G, d_vol, d_sino, 1, stream);
    dim3 grid(cdiv(g.ncols, 64), cdiv(g.nrows, 4), g.nviews);
    if (grid.y > 65535u) {
        leap_set_error("detector has too many rows for one launch");
        return LEAP_UNSUPPORTED;
    }
    hipLaunchKernelGGL(sd_project_general, grid, dim3(64, 4, 1), 0, stream, g, G->d_raycols, d_vol, d_sino);
    LEAP_HIP_CHECK(hipGetLastError());
    return LEAP_OK;
}

template <int NCS, int SH>
static void launch_sd_tiled(const leap_geometry *G, const float *d_sino, float *d_vol, hipStream_t stream, int items)
{
    constexpr SfBpShape S = BP_SHAPES[SH];
    const SfGeom &g = G->g;
    const unsigned tiles_x = cdiv(g.nx, BP_T), tiles_y = cdiv(g.ny, BP_T);
    dim3 grid(tiles_x * tiles_y, cdiv(g.nz, S.zc), (unsigned)items);
    if (g.type == SF_MODULAR)
        hipLaunchKernelGGL((sd_backproject_tiled<NCS, S.zc, S.pw, S.ph, true>), grid, dim3(256, 1, 1), 0, stream, g, G->d_views,
                           G->d_raycols, d_sino, d_vol, (int)tiles_x, (const SfGeom *)G->d_geoms);
    else
        hipLaunchKernelGGL((sd_backproject_tiled<NCS, S.zc, S.pw, S.ph, false>), grid, dim3(256, 1, 1), 0, stream, g, G->d_views,
                           G->d_raycols, d_sino, d_vol, (int)tiles_x, (const SfGeom *)nullptr);
}

template <int NCS>
static bool launch_sd_shape(const leap_geometry *G, const float *d_sino, float *d_vol, hipStream_t stream, int items)
{
    switch (G->bp_shape) {
    case 1: launch_sd_tiled<NCS, 1>(G, d_sino, d_vol, stream, items); return true;
    case 2: launch_sd_tiled<NCS, 2>(G, d_sino, d_vol, stream, items); return true;
    case 3: launch_sd_tiled<NCS, 3>(G, d_sino, d_vol, stream, items); return true;
    case 4: launch_sd_tiled<NCS, 4>(G, d_sino, d_vol, stream, items); return true;
    default: return false;
    }
}

template <int SH>
static void launch_md_tiled(const leap_geometry *G, const float *d_sino, float *d_vol, hipStream_t stream, int items)
{
    constexpr SfBpShape S = MD_BP_SHAPES[SH];
    const SfGeom &g = G->g;
    const unsigned tiles_x = cdiv(g.nx, BP_T), tiles_y = cdiv(g.ny, BP_T);
    dim3 grid(tiles_x * tiles_y, cdiv(g.nz, S.zc), (unsigned)items);
    hipLaunchKernelGGL((md_backproject_tiled<S.zc, S.pw, S.ph>), grid, dim3(256, 1, 1), 0, stream, g, (const MdBpView *)G->d_mdbp,
                       d_sino, d_vol, (int)tiles_x);
}

// The tiled Siddon back projection on `items` consecutive sinograms of a batch in one launch.
static int launch_sd_bp_items(const leap_geometry *G, const float *d_sino, float *d_vol, int items, hipStream_t stream)
{
    bool ok = false;
    if (G->md_tilted || G->d_mdbp) {
        switch (G->d_mdbp ? G->bp_shape : -1) {
        case 0: launch_md_tiled<0>(G, d_sino, d_vol, stream, items); ok = true; break;
        case 1: launch_md_tiled<1>(G, d_sino, d_vol, stream, items); ok = true; break;
        case 2: launch_md_tiled<2>(G, d_sino, d_vol, stream, items); ok = true; break;
        case 3: launch_md_tiled<3>(G, d_sino, d_vol, stream, items); ok = true; break;
        case 4: launch_md_tiled<4>(G, d_sino, d_vol, stream, items); ok = true; break;
        case 5: launch_md_tiled<5>(G, d_sino, d_vol, stream, items); ok = true; break;
        default: break;
        }
    } else
    switch (G->bp_nc) {
    case 2: ok = launch_sd_shape<2>(G, d_sino, d_vol, stream, items); break;
    case 3: ok = launch_sd_shape<3>(G, d_sino, d_vol, stream, items); break;
    case 4: ok = launch_sd_shape<4>(G, d_sino, d_vol, stream, items); break;
    default: break;
    }
    if (!ok) {
        leap_set_error("internal: no tiled Siddon back-projection instance for this geometry");
        return LEAP_UNSUPPORTED;
    }
    LEAP_HIP_CHECK(hipGetLastError());
    return LEAP_OK;
}

static int launch_sd_backproject(const leap_geometry *G, const float *d_sino, float *d_vol, hipStream_t stream)
{
    const SfGeom &g = G->g;
    if (g.type == SF_MODULAR && !G->bp_tiled) {
        dim3 grid(cdiv(g.nx, 64), cdiv(g.ny, 4), g.nz);
        hipLaunchKernelGGL(md_backproject_general, grid, dim3(64, 4, 1), 0, stream, g, G->d_poses, d_sino, d_vol);
        LEAP_HIP_CHECK(hipGetLastError());
        return LEAP_OK;
    }
    if (G->bp_tiled) return launch_sd_bp_items(G, d_sino, d_vol, 1, stream);
    dim3 grid(cdiv(g.nx, 64), cdiv(g.ny, 4), g.nz);
    if (grid.y > 65535u || grid.z > 65535u) {
        leap_set_error("volume has too many voxels along y or z for one launch");
        return LEAP_UNSUPPORTED;
    }
    hipLaunchKernelGGL(sd_backproject_general, grid, dim3(64, 4, 1), 0, stream, g, G->d_views, G->d_raycols, d_sino, d_vol);
    LEAP_HIP_CHECK(hipGetLastError());
    return LEAP_OK;
}

template <int NKP, int RG, int CW, int GT>
static void launch_fp_columns(const leap_geometry *G, const FwdScratch &S, const SfSlab &slab, float *d_sino, hipStream_t stream, int items)
{
    const SfGeom &g = G->g;
    const int col_tiles = (int)cdiv(g.ncols, FP_WAVES * CW), bands = (int)cdiv(g.nrows, RG * 128);
    // XCD-aware block order (see the kernel): pad views to blocks of vb and each XCD's tiles to chunks of tb
    const int vb = G->fp_vb, tb = G->fp_tb;
    const int vgroups_pad = (int)cdiv(g.nviews, vb) * vb;
    const int tiles_per_xcd_pad = (int)cdiv(cdiv(col_tiles, 8), tb) * tb;
    int nq_log2 = 2;
    while ((1 << nq_log2) < G->fp_nq) ++nq_log2;
    dim3 grid((unsigned)(8 * tiles_per_xcd_pad * vgroups_pad * bands), (unsigned)items, 1);
    hipLaunchKernelGGL((sf_project_columns<NKP, RG, CW, GT>), grid, dim3(FP_WAVES * 64, 1, 1), 0, stream, g, G->d_views, S.volz,
                       d_sino, G->d_major, G->nzp, S.item_floats, nq_log2, col_tiles, bands, vb, tb, vgroups_pad, tiles_per_xcd_pad,
                       slab, (const SfGeom *)G->d_geoms);
}

template <int NKP, int RG>
static bool launch_fp_w(const leap_geometry *G, const FwdScratch &S, const SfSlab &slab, float *d_sino, hipStream_t stream, int items)
{
    const int gt = G->g.type == SF_CONE_CURVED ? 1 : (G->g.type == SF_MODULAR ? 2 : 0);
    switch (gt * 10 + G->fp_cw) {
    case 1: launch_fp_columns<NKP, RG, 1, 0>(G, S, slab, d_sino, stream, items); return true;
    case 2: launch_fp_columns<NKP, RG, 2, 0>(G, S, slab, d_sino, stream, items); return true;
    case 4: launch_fp_columns<NKP, RG, 4, 0>(G, S, slab, d_sino, stream, items); return true;
    case 12: launch_fp_columns<NKP, RG, 2, 1>(G, S, slab, d_sino, stream, items); return true;
    case 14: launch_fp_columns<NKP, RG, 4, 1>(G, S, slab, d_sino, stream, items); return true;
    case 22: launch_fp_columns<NKP, RG, 2, 2>(G, S, slab, d_sino, stream, items); return true;
    case 24: launch_fp_columns<NKP, RG, 4, 2>(G, S, slab, d_sino, stream, items); return true;
    default: return false;
    }
}

template <int NKP>
static bool launch_fp_rg(const leap_geometry *G, const FwdScratch &S, const SfSlab &slab, float *d_sino, hipStream_t stream, int items)
{
    switch (G->fp_rg) {
    case 1: return launch_fp_w<NKP, 1>(G, S, slab, d_sino, stream, items);
    case 2: return launch_fp_w<NKP, 2>(G, S, slab, d_sino, stream, items);
    case 3: return launch_fp_w<NKP, 3>(G, S, slab, d_sino, stream, items);
    case 4: return launch_fp_w<NKP, 4>(G, S, slab, d_sino, stream, items);
    default: return false;
    }
}

static bool launch_fp_slab(const leap_geometry *G, const FwdScratch &S, const SfSlab &slab, float *d_sino, hipStream_t stream, int items)
{
    switch (G->fp_nkp) {
    case 2: return launch_fp_rg<2>(G, S, slab, d_sino, stream, items);
    case 3: return launch_fp_rg<3>(G, S, slab, d_sino, stream, items);
    case 4: return launch_fp_rg<4>(G, S, slab, d_sino, stream, items);
    case 5: return launch_fp_rg<5>(G, S, slab, d_sino, stream, items);
    case 6: return launch_fp_rg<6>(G, S, slab, d_sino, stream, items);
    case 7: return launch_fp_rg<7>(G, S, slab, d_sino, stream, items);
    default: return false;
    }
}

// The column-wise forward projection (footprint or Siddon weights) of a batch: up to S.items volumes at a time, each
// walked slab by slab -- first the slabs across x for the rays that advance fastest along x, then the slabs across y
// for the others.  Per slab: copy it z-fastest into the scratch, then every ray adds the slab's share to its sample.
static int run_forward_columns(const leap_geometry *G, const FwdScratch &S, const float *d_vol, float *d_sino, int batch,
                               hipStream_t stream)
{
    const SfGeom &g = G->g;
    const size_t nvol = (size_t)g.nx * g.ny * g.nz, nsino = (size_t)g.nviews * g.nrows * g.ncols;
    const bool siddon = g.model == SF_MODEL_SIDDON;
    for (int b = 0; b < batch; b += S.items) {
        const int items = batch - b < S.items ? batch - b : S.items;
        const float *vol = d_vol + (size_t)b * nvol;
        float *sino = d_sino + (size_t)b * nsino;
        for (int xmajor = 1; xmajor >= 0; --xmajor) {
            const int n_major = xmajor ? g.nx : g.ny;
            for (int n0 = 0; n0 < n_major; n0 += S.width) {
                const int n1 = n0 + S.width < n_major ? n0 + S.width : n_major;
                const SfSlab slab = {n0, n1, xmajor, n0 == 0 ? 1 : 0, S.width};
                const int i0 = xmajor ? n0 : 0, ni = xmajor ? S.width : g.nx, nj = xmajor ? g.ny : n1 - n0;
                dim3 tgrid(cdiv(xmajor ? n1 - n0 : g.nx, 32), cdiv(g.nz, 32), (unsigned)(nj * items));
                hipLaunchKernelGGL(sf_volume_to_columns, tgrid, dim3(32, 8, 1), 0, stream, vol, S.volz, g.nx, g.ny, g.nz, G->nzp, i0,
                                   xmajor ? 0 : n0, ni, nj, S.item_floats);
                const bool ok = siddon ? launch_sd_slab(G, S, slab, sino, stream, items) : launch_fp_slab(G, S, slab, sino, stream, items);
                if (!ok) {
                    leap_set_error("internal: no column-wise forward instance for this geometry");
                    return LEAP_UNSUPPORTED;
                }
            }
        }
    }
    LEAP_HIP_CHECK(hipGetLastError());
    return LEAP_OK;
}

int leap_launch_project_batch(const leap_geometry *G, const float *d_vol, float *d_sino, int batch, hipStream_t stream)
{
    const SfGeom &g = G->g;
    const size_t nvol = (size_t)g.nx * g.ny * g.nz, nsino = (size_t)g.nviews * g.nrows * g.ncols;
    const bool footprint_fast = g.model != SF_MODEL_SIDDON && G->fp_columns;
    const bool siddon_fast = g.model == SF_MODEL_SIDDON && G->sd_columns;
    if (footprint_fast || siddon_fast) {
        // Calls on one handle share its scratch.  They are ordered on the device: a call that arrives on another stream
        // than the last one first waits for that one's kernels.
        std::lock_guard<std::mutex> lock(G->scratch_mutex);
        if (G->scratch_used && G->scratch_stream != stream) LEAP_HIP_CHECK(hipStreamWaitEvent(stream, G->scratch_event, 0));
        FwdScratch S;
        S.volz = G->d_volz;
        if (!leap_plan_scratch(G, G->scratch_bytes / sizeof(float), batch, S.width, S.items)) {
            leap_set_error("internal: the handle's scratch holds no slab");
            return LEAP_UNSUPPORTED;
        }
        S.item_floats = ((size_t)S.width * (size_t)(g.nx > g.ny ? g.nx : g.ny) + 1) * (size_t)G->nzp;
        const int rc = run_forward_columns(G, S, d_vol, d_sino, batch, stream);
        if (rc != LEAP_OK) return rc;
        LEAP_HIP_CHECK(hipEventRecord(G->scratch_event, stream));
        G->scratch_stream = stream;
        G->scratch_used = true;
        return LEAP_OK;
    }
    for (int b = 0; b < batch; ++b) {
        const int rc = leap_launch_project(G, d_vol + b * nvol, d_sino + b * nsino, stream);
        if (rc != LEAP_OK) return rc;
    }
    return LEAP_OK;
}

int leap_launch_project(const leap_geometry *G, const float *d_vol, float *d_sino, hipStream_t stream)
{
    const SfGeom &g = G->g;
    if (g.model == SF_MODEL_SIDDON) return launch_sd_project(G, d_vol, d_sino, stream);
    if (G->fp_columns) return leap_launch_project_batch(G, d_vol, d_sino, 1, stream);
    if (G->d_mfviews) {                     // sizes were checked against the grid limits at creation
        dim3 grid(cdiv(g.ncols, 64), cdiv(cdiv(g.nrows, MF_RC), 4), g.nviews);
        hipLaunchKernelGGL(mf_project_general, grid, dim3(64, 4, 1), 0, stream, g, G->d_mfviews, d_vol, d_sino);
        LEAP_HIP_CHECK(hipGetLastError());
        return LEAP_OK;
    }
    dim3 block(64, 4, 1);
    dim3 grid(cdiv(g.ncols, 64), cdiv(cdiv(g.nrows, GEN_RC), 4), g.nviews);
    if (grid.y > 65535u) {
        leap_set_error("detector has too many rows for one launch");
        return LEAP_UNSUPPORTED;
    }
    if (g.type == SF_MODULAR)
        hipLaunchKernelGGL(sf_project_general_modular, grid, block, 0, stream, G->d_geoms, G->d_views, d_vol, d_sino);
    else
        hipLaunchKernelGGL(sf_project_general, grid, block, 0, stream, g, G->d_views, d_vol, d_sino);
    LEAP_HIP_CHECK(hipGetLastError());
    return LEAP_OK;
}

template <int NC, int NV, int SH, int GT>
static void launch_bp_tiled_gt(const leap_geometry *G, const float *d_sino, float *d_vol, hipStream_t stream, int items)
{
    constexpr SfBpShape S = BP_SHAPES[SH];
    const SfGeom &g = G->g;
    const unsigned tiles_x = cdiv(g.nx, BP_T), tiles_y = cdiv(g.ny, BP_T);
    dim3 grid(tiles_x * tiles_y, cdiv(g.nz, S.zc), (unsigned)items);
    hipLaunchKernelGGL((sf_backproject_tiled<NC, NV, S.zc, S.pw, S.ph, GT>), grid, dim3(256, 1, 1), 0, stream, g, G->d_views,
                       d_sino, d_vol, (int)tiles_x, G->bp_wh, GT == 1 ? (const void *)G->d_colcs : (const void *)G->d_geoms);
}

template <int NC, int NV, int SH>
static void launch_bp_tiled(const leap_geometry *G, const float *d_sino, float *d_vol, hipStream_t stream, int items)
{
    if (G->g.type == SF_CONE_CURVED) launch_bp_tiled_gt<NC, NV, SH, 1>(G, d_sino, d_vol, stream, items);
    else if (G->g.type == SF_MODULAR) launch_bp_tiled_gt<NC, NV, SH, 2>(G, d_sino, d_vol, stream, items);
    else launch_bp_tiled_gt<NC, NV, SH, 0>(G, d_sino, d_vol, stream, items);
}

template <int NC, int NV>
static bool launch_bp_shape(const leap_geometry *G, const float *d_sino, float *d_vol, hipStream_t stream, int items)
{
    switch (G->bp_shape) {
    case 0:      // 64 voxels per thread: instances for two-row footprints only (taller ones would spill registers)
        if constexpr (NV == 2) {
            launch_bp_tiled<NC, NV, 0>(G, d_sino, d_vol, stream, items);
            return true;
        } else {
            return false;
        }
    case 1: launch_bp_tiled<NC, NV, 1>(G, d_sino, d_vol, stream, items); return true;
    case 2: launch_bp_tiled<NC, NV, 2>(G, d_sino, d_vol, stream, items); return true;
    case 3: launch_bp_tiled<NC, NV, 3>(G, d_sino, d_vol, stream, items); return true;
    case 4: launch_bp_tiled<NC, NV, 4>(G, d_sino, d_vol, stream, items); return true;
    case BP_TALL_SHAPE:      // 64 voxels per thread under a taller window: two- and three-row instances
        if constexpr (NV <= 3) {
            launch_bp_tiled<NC, NV, BP_TALL_SHAPE>(G, d_sino, d_vol, stream, items);
            return true;
        } else {
            return false;
        }
    default: return false;
    }
}

// The tiled footprint back projection on `items` consecutive sinograms of a batch in one launch.
static int launch_bp_items(const leap_geometry *G, const float *d_sino, float *d_vol, int items, hipStream_t stream)
{
    bool ok = false;
    switch (G->bp_nc * 10 + G->bp_nv) {
    case 22: ok = launch_bp_shape<2, 2>(G, d_sino, d_vol, stream, items); break;
    case 23: ok = launch_bp_shape<2, 3>(G, d_sino, d_vol, stream, items); break;
    case 32: ok = launch_bp_shape<3, 2>(G, d_sino, d_vol, stream, items); break;
    case 33: ok = launch_bp_shape<3, 3>(G, d_sino, d_vol, stream, items); break;
    case 24: ok = launch_bp_shape<2, 4>(G, d_sino, d_vol, stream, items); break;
    case 34: ok = launch_bp_shape<3, 4>(G, d_sino, d_vol, stream, items); break;
    case 42: ok = launch_bp_shape<4, 2>(G, d_sino, d_vol, stream, items); break;
    case 43: ok = launch_bp_shape<4, 3>(G, d_sino, d_vol, stream, items); break;
    case 44: ok = launch_bp_shape<4, 4>(G, d_sino, d_vol, stream, items); break;
    case 52: ok = launch_bp_shape<5, 2>(G, d_sino, d_vol, stream, items); break;
    case 53: ok = launch_bp_shape<5, 3>(G, d_sino, d_vol, stream, items); break;
    case 54: ok = launch_bp_shape<5, 4>(G, d_sino, d_vol, stream, items); break;
    default: break;
    }
    if (!ok) {
        leap_set_error("internal: no tiled back-projection instance for this footprint");
        return LEAP_UNSUPPORTED;
    }
    LEAP_HIP_CHECK(hipGetLastError());
    return LEAP_OK;
}

int leap_launch_backproject_batch(const leap_geometry *G, const float *d_sino, float *d_vol, int batch, hipStream_t stream)
{
    const SfGeom &g = G->g;
    const size_t nvol = (size_t)g.nx * g.ny * g.nz, nsino = (size_t)g.nviews * g.nrows * g.ncols;
    if (G->bp_tiled) {
        // up to 16 items per launch (a batch of small training volumes fills the chip better that way)
        for (int b = 0; b < batch; b += 16) {
            const int items = batch - b < 16 ? batch - b : 16;
            const int rc = g.model != SF_MODEL_SIDDON ? launch_bp_items(G, d_sino + b * nsino, d_vol + b * nvol, items, stream)
                                                      : launch_sd_bp_items(G, d_sino + b * nsino, d_vol + b * nvol, items, stream);
            if (rc != LEAP_OK) return rc;
        }
        return LEAP_OK;
    }
    for (int b = 0; b < batch; ++b) {
        const int rc = leap_launch_backproject(G, d_sino + b * nsino, d_vol + b * nvol, stream);
        if (rc != LEAP_OK) return rc;
    }
    return LEAP_OK;
}

int leap_launch_backproject(const leap_geometry *G, const float *d_sino, float *d_vol, hipStream_t stream)
{
    const SfGeom &g = G->g;
    if (g.model == SF_MODEL_SIDDON) return launch_sd_backproject(G, d_sino, d_vol, stream);
    if (G->bp_tiled) return launch_bp_items(G, d_sino, d_vol, 1, stream);
    if (G->d_mfviews) {
        dim3 grid(cdiv(g.nx, 64), cdiv(g.ny, 4), g.nz);
        hipLaunchKernelGGL(mf_backproject_general, grid, dim3(64, 4, 1), 0, stream, g, G->d_mfviews, d_sino, d_vol);
        LEAP_HIP_CHECK(hipGetLastError());
        return LEAP_OK;
    }
    dim3 block(64, 4, 1);
    dim3 grid(cdiv(g.nx, 64), cdiv(g.ny, 4), cdiv(g.nz, GEN_ZC));
    if (grid.y > 65535u || grid.z > 65535u) {
        leap_set_error("volume has too many voxels along y or z for one launch");
        return LEAP_UNSUPPORTED;
    }
    if (g.type == SF_MODULAR)
        hipLaunchKernelGGL(sf_backproject_general_modular, grid, block, 0, stream, g, G->d_geoms, G->d_views, d_sino, d_vol);
    else
        hipLaunchKernelGGL(sf_backproject_general, grid, block, 0, stream, g, G->d_views, d_sino, d_vol);
    LEAP_HIP_CHECK(hipGetLastError());
    return LEAP_OK;
}

// ------------------------------------------------------------------------------------------------
// Forward projection on a fixed scratch array, for callers that must not allocate.
// ------------------------------------------------------------------------------------------------
//
// The column-wise forward kernels read a z-fastest copy of the volume.  A handle normally owns that copy (allocated
// in leap_geometry_create).  leap_project_static_scratch keeps it in the file-scope device array below instead, so
// the call itself, and everything it launches, touches no allocator.  In host code the array's name is only a
// stand-in for the symbol: its device address is asked for once per device (hipGetSymbolAddress, with that device
// current) and only that address is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[LEAP_STATIC_SCRATCH_BYTES];

constexpr int LEAP_MAX_DEVICES = 64;
static float *g_static_scratch[LEAP_MAX_DEVICES];     // device address of `scratch`, per device (nullptr: not asked yet)
static std::mutex g_static_scratch_mutex;

int leap_static_scratch_init(int device)
{
    if (device < 0 || device >= LEAP_MAX_DEVICES) {
        leap_set_error("device index beyond the static scratch table");
        return LEAP_UNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (g_static_scratch[device]) return LEAP_OK;
    int current = -1;
    LEAP_HIP_CHECK(hipGetDevice(&current));
    if (current != device) {
        leap_set_error("the handle's device is not the current device");
        return LEAP_INVALID_ARG;
    }
    void *p = nullptr;
    LEAP_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    g_static_scratch[device] = static_cast<float *>(p);
    return LEAP_OK;
}

extern "C" int leap_project_static_scratch(const leap_geometry *G, const float *d_vol, float *d_sino, int32_t batch, void *hip_stream)
{
    if (!G || !d_vol || !d_sino) {
        leap_set_error("null handle or data pointer");
        return LEAP_INVALID_ARG;
    }
    if (batch <= 0) {
        leap_set_error("batch must be positive");
        return LEAP_INVALID_ARG;
    }
    if ((const void *)d_vol == (const void *)d_sino) {
        leap_set_error("input and output must not alias");
        return LEAP_INVALID_ARG;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    const SfGeom &g = G->g;
    const bool footprint_fast = g.model != SF_MODEL_SIDDON && G->fp_columns;
    const bool siddon_fast = g.model == SF_MODEL_SIDDON && G->sd_columns;
    if (!footprint_fast && !siddon_fast) {
        // this geometry runs on kernels that read the caller's volume directly: no scratch is involved at all
        const size_t nvol = (size_t)g.nx * g.ny * g.nz, nsino = (size_t)g.nviews * g.nrows * g.ncols;
        for (int b = 0; b < batch; ++b) {
            const int rc = leap_launch_project(G, d_vol + b * nvol, d_sino + b * nsino, stream);
            if (rc != LEAP_OK) return rc;
        }
        return LEAP_OK;
    }
    const int n_side = g.nx > g.ny ? g.nx : g.ny;
    FwdScratch S;
    if (!leap_plan_scratch(G, LEAP_STATIC_SCRATCH_BYTES / sizeof(float), batch, S.width, S.items)) {
        char msg[200];
        std::snprintf(msg, sizeof msg, "volume too large for the static scratch: four voxel layers of its z-fastest copy need %.0f bytes, "
                      "the array holds %zu", 4.0 * G->nzp * (4.0 * n_side + 1.0), (size_t)LEAP_STATIC_SCRATCH_BYTES);
        leap_set_error(msg);
        return LEAP_UNSUPPORTED;
    }
    float *volz = (G->device >= 0 && G->device < LEAP_MAX_DEVICES) ? g_static_scratch[G->device] : nullptr;
    if (!volz) {
        leap_set_error("static scratch address unknown for the handle's device");
        return LEAP_HIP_ERROR;
    }
    S.volz = volz;
    S.item_floats = ((size_t)S.width * n_side + 1) * (size_t)G->nzp;
    const int width = S.width, per = S.items;
    // the array keeps what the last call (of any handle) left in it: restore the zeros around this geometry's columns
    const unsigned ncolumns = (unsigned)width * (unsigned)n_side;
    const unsigned nthreads = ncolumns * 2u * FP_PAD > (unsigned)G->nzp ? ncolumns * 2u * FP_PAD : (unsigned)G->nzp;
    for (int it = 0; it < per; ++it)
        hipLaunchKernelGGL(sf_clear_column_pads, dim3(cdiv(nthreads, 256)), dim3(256), 0, stream, volz + (size_t)it * S.item_floats,
                           ncolumns, g.nz, G->nzp);
    LEAP_HIP_CHECK(hipGetLastError());
    return run_forward_columns(G, S, d_vol, d_sino, batch, stream);
}
