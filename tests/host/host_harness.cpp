// Host-side harness for the HIP library's host/device code (test infrastructure; built with g++, no GPU).
//
// It links the library's real host geometry module against stubs of the few HIP runtime calls that module makes,
// and supplies CPU versions of the two launchers that step the general kernel bodies thread by thread.  On top of
// that it re-enacts, on the CPU, the index arithmetic of the tiled back projection (does every LDS access of every
// thread of every workgroup stay inside the staged window?) and the arithmetic of the column-wise forward kernel
// (candidate slots, padded z-columns, axial overlap cascade), so that mistakes in them show up without a GPU.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../paper_2307_05801_amd/csrc/leap_internal.h"
#include "../../paper_2307_05801_amd/csrc/sf_general.h"
#define SF_NO_KERNELS
#include "../../paper_2307_05801_amd/csrc/sf_backproject_tiled.h"
#include "../../paper_2307_05801_amd/csrc/sf_project_columns.h"
#include "../../paper_2307_05801_amd/csrc/md_project_columns.h"
#include "../../paper_2307_05801_amd/csrc/md_backproject_tiled.h"

// ---- stubs of the HIP runtime calls made by leap_geometry.cpp: "device" memory is host memory ---------------
extern "C" {
hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
hipError_t hipMalloc(void **p, size_t n) { *p = std::malloc(n); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipMemcpy(void *d, const void *s, size_t n, hipMemcpyKind) { std::memcpy(d, s, n); return hipSuccess; }
hipError_t hipMemset(void *p, int v, size_t n) { std::memset(p, v, n); return hipSuccess; }
hipError_t hipFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipDeviceSynchronize() { return hipSuccess; }
hipError_t hipGetLastError() { return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = nullptr; return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
const char *hipGetErrorString(hipError_t) { return "stub"; }
// the host-memory entry points (leap_host.cpp): every asynchronous call happens at once, so the pipeline's buffer
// rotation and chunk arithmetic are checked, not its overlap
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned) { *s = nullptr; return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t) { return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, hipMemcpyKind, hipStream_t) { std::memcpy(d, s, n); return hipSuccess; }
hipError_t hipHostMalloc(void **p, size_t n, unsigned) { *p = std::malloc(n); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipHostFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipPointerGetAttributes(hipPointerAttribute_t *, const void *) { return hipErrorInvalidValue; }
}

int leap_static_scratch_init(int) { return LEAP_OK; }   // the fixed device array exists on a GPU only

// ---- CPU launchers: the general kernel bodies, one "thread" at a time ----------------------------------------
int leap_launch_project(const leap_geometry *G, const float *vol, float *sino, hipStream_t)
{
    const SfGeom &g = G->g;
    constexpr int RC = 8;
    if (g.type == SF_MODULAR && g.model == SF_MODEL_SIDDON) {
#pragma omp parallel for collapse(2)
        for (int a = 0; a < g.nviews; ++a)
            for (int r = 0; r < g.nrows; ++r)
                for (int c = 0; c < g.ncols; ++c)
                    sino[((size_t)a * g.nrows + r) * g.ncols + c] = md_project_ray(g, G->d_poses[a], vol, r, c);
        return LEAP_OK;
    }
    if (G->d_mfviews) {
#pragma omp parallel for collapse(2)
        for (int a = 0; a < g.nviews; ++a)
            for (int r0 = 0; r0 < g.nrows; r0 += RC)
                for (int c = 0; c < g.ncols; ++c) {
                    float out[RC];
                    mf_project_rows<RC>(g, G->d_mfviews[a], vol, r0, c, out);
                    for (int rr = 0; rr < RC && r0 + rr < g.nrows; ++rr) sino[((size_t)a * g.nrows + r0 + rr) * g.ncols + c] = out[rr];
                }
        return LEAP_OK;
    }
    if (g.model == SF_MODEL_SIDDON) {
#pragma omp parallel for collapse(2)
        for (int a = 0; a < g.nviews; ++a)
            for (int r = 0; r < g.nrows; ++r)
                for (int c = 0; c < g.ncols; ++c)
                    sino[((size_t)a * g.nrows + r) * g.ncols + c] = sd_project_ray(g, G->d_raycols[(size_t)a * g.ncols + c], vol, r);
        return LEAP_OK;
    }
#pragma omp parallel for collapse(2)
    for (int a = 0; a < g.nviews; ++a)
        for (int r0 = 0; r0 < g.nrows; r0 += RC)
            for (int c = 0; c < g.ncols; ++c) {
                float out[RC];
                sf_project_ray_chunk<RC>(G->d_geoms ? G->d_geoms[a] : g, G->d_views[a], vol, c, r0, out);
                for (int rr = 0; rr < RC && r0 + rr < g.nrows; ++rr) sino[((size_t)a * g.nrows + r0 + rr) * g.ncols + c] = out[rr];
            }
    return LEAP_OK;
}

int leap_launch_project_batch(const leap_geometry *G, const float *vol, float *sino, int batch, hipStream_t st)
{
    const SfGeom &g = G->g;
    const size_t nvol = (size_t)g.nx * g.ny * g.nz, nsino = (size_t)g.nviews * g.nrows * g.ncols;
    for (int b = 0; b < batch; ++b) {
        const int rc = leap_launch_project(G, vol + b * nvol, sino + b * nsino, st);
        if (rc != LEAP_OK) return rc;
    }
    return LEAP_OK;
}

int leap_launch_backproject(const leap_geometry *G, const float *sino, float *vol, hipStream_t)
{
    const SfGeom &g = G->g;
    constexpr int ZC = 8;
    if (g.type == SF_MODULAR && g.model == SF_MODEL_SIDDON) {
#pragma omp parallel for collapse(2)
        for (int k = 0; k < g.nz; ++k)
            for (int j = 0; j < g.ny; ++j)
                for (int i = 0; i < g.nx; ++i) vol[((size_t)k * g.ny + j) * g.nx + i] = md_backproject_voxel(g, G->d_poses, sino, i, j, k);
        return LEAP_OK;
    }
    if (G->d_mfviews) {
#pragma omp parallel for collapse(2)
        for (int k = 0; k < g.nz; ++k)
            for (int j = 0; j < g.ny; ++j)
                for (int i = 0; i < g.nx; ++i) vol[((size_t)k * g.ny + j) * g.nx + i] = mf_backproject_voxel(g, G->d_mfviews, sino, i, j, k);
        return LEAP_OK;
    }
    if (g.model == SF_MODEL_SIDDON) {
#pragma omp parallel for collapse(2)
        for (int k = 0; k < g.nz; ++k)
            for (int j = 0; j < g.ny; ++j)
                for (int i = 0; i < g.nx; ++i)
                    vol[((size_t)k * g.ny + j) * g.nx + i] = sd_backproject_voxel(g, G->d_views, G->d_raycols, sino, i, j, k);
        return LEAP_OK;
    }
#pragma omp parallel for collapse(2)
    for (int k0 = 0; k0 < g.nz; k0 += ZC)
        for (int j = 0; j < g.ny; ++j)
            for (int i = 0; i < g.nx; ++i) {
                float acc[ZC] = {0};
                sf_backproject_column_chunk<ZC>(g, G->d_views, sino, i, j, k0, acc, G->d_geoms);
                for (int kk = 0; kk < ZC && k0 + kk < g.nz; ++kk) vol[((size_t)(k0 + kk) * g.ny + j) * g.nx + i] = acc[kk];
            }
    return LEAP_OK;
}

int leap_launch_backproject_batch(const leap_geometry *G, const float *sino, float *vol, int batch, hipStream_t st)
{
    const SfGeom &g = G->g;
    const size_t nvol = (size_t)g.nx * g.ny * g.nz, nsino = (size_t)g.nviews * g.nrows * g.ncols;
    for (int b = 0; b < batch; ++b) {
        const int rc = leap_launch_backproject(G, sino + b * nsino, vol + b * nvol, st);
        if (rc != LEAP_OK) return rc;
    }
    return LEAP_OK;
}

// ---- tiled back projection: every thread's LDS reads against the staged window --------------------------------
// report[0..7] = {tiled?, nc, nv, zc, max column index read, max row index read, widest footprint in pixels, violations}
extern "C" int host_check_backproject_windows(const leap_geometry *G, int64_t *report)
{
    const SfGeom &g = G->g;
    std::fill(report, report + 8, 0);
    report[0] = G->bp_tiled;
    if (!G->bp_tiled) return 0;
    const int NC = G->bp_nc, NV = G->bp_nv;
    const SfBpShape S = BP_SHAPES[G->bp_shape];
    const int tiles_x = (g.nx + BP_T - 1) / BP_T, tiles_y = (g.ny + BP_T - 1) / BP_T, chunks = (g.nz + S.zc - 1) / S.zc;
    int maxc = -1, maxr = -1, maxspan = 0;
    long bad = 0;
#pragma omp parallel for collapse(2) reduction(max : maxc, maxr, maxspan) reduction(+ : bad)
    for (int a = 0; a < g.nviews; ++a)
        for (int ty = 0; ty < tiles_y; ++ty)
            for (int tx = 0; tx < tiles_x; ++tx)
                for (int ch = 0; ch < chunks; ++ch) {
                    const SfGeom &g = G->geoms.empty() ? G->g : G->geoms[a];      // modular: the view's own parameter block
                    const int i0 = tx * BP_T, j0 = ty * BP_T, k0 = ch * S.zc;
                    const double zlo = fma((double)k0, g.Tzd, g.zlo0d);
                    const float z0 = (float)zlo, z1 = z0 + (float)S.zc * g.Tz;
                    const float hx = 0.5f * (float)(BP_T - 1) * g.T;
                    const float xc = (float)(g.x0d + ((double)i0 + 0.5 * (BP_T - 1)) * g.Td);
                    const float yc = (float)(g.y0d + ((double)j0 + 0.5 * (BP_T - 1)) * g.Td);
                    const SfWindow w = sf_bp_window(g, G->views[a], xc, yc, hx, z0, z1, G->bp_wh, NC, NV);
                    for (int tj = 0; tj < BP_T; ++tj)
                        for (int ti = 0; ti < BP_T; ++ti) {
                            const int i = std::min(i0 + ti, g.nx - 1), j = std::min(j0 + tj, g.ny - 1);
                            SfColumn f;
                            if (g.type == SF_CONE_CURVED) {      // as the kernel: relative to the tile centre
                                const double xcd = g.x0d + ((double)i0 + 0.5 * (BP_T - 1)) * g.Td;
                                const double ycd = g.y0d + ((double)j0 + 0.5 * (BP_T - 1)) * g.Td;
                                const SfView &v = G->views[a];
                                const double tref = fma(ycd, v.cd, -xcd * v.sd), dnref = g.sodd - fma(xcd, v.cd, ycd * v.sd);
                                f = sf_column_curved_ref(g, v, i, j, tref, dnref, atan2(tref, dnref));
                            } else {
                                f = sf_column(g, G->views[a], i, j);
                            }
                            int cf, cl;
                            sf_col_range(f, cf, cl);
                            const SfRowsOfVoxels ax = sf_rows_of_voxels(g, f, zlo);
                            const int c_lo = cf - w.c0, c_hi = c_lo + NC - 1;
                            const int r_lo = ax.rb - w.r0;
                            // last row read: first row of the last voxel plus NV-1 (the shared-row variant reads the same set)
                            const int r_hi = r_lo + (int)std::floor(fmaf(ax.av, (float)(S.zc - 1), ax.phi0)) + NV - 1;
                            maxc = std::max(maxc, c_hi);
                            maxr = std::max(maxr, r_hi);
                            maxspan = std::max(maxspan, cl - cf + 1);
                            if (c_lo < 0 || c_hi >= S.pw || r_lo < 0 || r_hi >= S.ph) ++bad;   // read outside the staged window
                            if (cl - cf + 1 > NC) ++bad;                                          // footprint wider than NC columns
                            if (ax.av > (float)(NV - 1) * 1.000001f) ++bad;                       // voxel taller than NV-1 rows
                        }
                }
    report[1] = NC; report[2] = NV; report[3] = S.zc; report[4] = maxc; report[5] = maxr; report[6] = maxspan; report[7] = bad;
    return bad != 0;
}

// ---- cylinder: the tile-relative column function of the tiled kernel against the general one ------------------------
// out[0] = largest |difference| of the column coordinate (pixels), out[1] = of the four knot offsets, over every view,
// tile and voxel column; out[2] = largest corner angle met (rad).
extern "C" int host_curved_column_deviation(const leap_geometry *G, double *out)
{
    const SfGeom &g = G->g;
    out[0] = out[1] = out[2] = 0.0;
    if (g.type != SF_CONE_CURVED) return -1;
    const int tiles_x = (g.nx + BP_T - 1) / BP_T, tiles_y = (g.ny + BP_T - 1) / BP_T;
    double dxi = 0.0, dof = 0.0, ang = 0.0;
#pragma omp parallel for collapse(2) reduction(max : dxi, dof, ang)
    for (int a = 0; a < g.nviews; ++a)
        for (int ty = 0; ty < tiles_y; ++ty)
            for (int tx = 0; tx < tiles_x; ++tx) {
                const SfView &v = G->views[a];
                const double xcd = g.x0d + ((double)(tx * BP_T) + 0.5 * (BP_T - 1)) * g.Td;
                const double ycd = g.y0d + ((double)(ty * BP_T) + 0.5 * (BP_T - 1)) * g.Td;
                const double tref = fma(ycd, v.cd, -xcd * v.sd), dnref = g.sodd - fma(xcd, v.cd, ycd * v.sd);
                const double gref = atan2(tref, dnref);
                for (int tj = 0; tj < BP_T; ++tj)
                    for (int ti = 0; ti < BP_T; ++ti) {
                        const int i = std::min(tx * BP_T + ti, g.nx - 1), j = std::min(ty * BP_T + tj, g.ny - 1);
                        const SfColumn p = sf_column(g, v, i, j), q = sf_column_curved_ref(g, v, i, j, tref, dnref, gref);
                        dxi = std::max(dxi, std::fabs(p.xi - q.xi));
                        dof = std::max(dof, (double)std::max(std::max(std::fabs(p.o0 - q.o0), std::fabs(p.o1 - q.o1)),
                                                             std::max(std::fabs(p.o2 - q.o2), std::fabs(p.o3 - q.o3))));
                        ang = std::max(ang, (double)std::max(std::fabs(p.o0), std::fabs(p.o3)) / g.ku);
                    }
            }
    out[0] = dxi; out[1] = dof; out[2] = ang;
    return 0;
}

// ---- column-wise forward projection: the kernel's own per-lane functions, stepped serially ------------------------------
// One (view, bundle of CW detector columns) at a time, the way a wavefront of sf_project_columns works through it: the
// host's marching axis for the bundle, candidate slots per slab, sf_candidate_record for every candidate, then for every
// pair of adjacent rows sf_place_row, a window of P voxels read from the z-fastest copy (zero outside the padded
// column, as the kernel's buffer loads return) and sf_pair_sums.  The whole volume stands in for one slab.
template <int CW, int P>
static void host_pairs_of_candidate(const SfGeom &g, const float *col, int nzp, double mu, double zkp, const float (&fa)[CW],
                                    std::vector<float> &acc)
{
    const SfPairConsts<P> k = sf_pair_consts<P>((float)mu);      // per candidate, as the kernel's lanes work them out
    for (int r = 0; r < g.nrows; r += 2) {
        float fr1;
        unsigned hi;
        sf_place_row((double)r - g.row_offd, mu, zkp, fr1, hi);
        const int kf = (int)(hi - FP_KAP_HI);
        float x[P];
        for (int t = 0; t < P; ++t) x[t] = (kf + t >= 0 && kf + t < nzp) ? col[kf + t] : 0.0f;
        float sa, sb;
        sf_pair_sums<P>(x, fr1, k, sa, sb);
        for (int cw = 0; cw < CW; ++cw) {
            acc[(size_t)r * CW + cw] = fmaf(fa[cw], sa, acc[(size_t)r * CW + cw]);
            if (r + 1 < g.nrows) acc[(size_t)(r + 1) * CW + cw] = fmaf(fa[cw], sb, acc[(size_t)(r + 1) * CW + cw]);
        }
    }
}

template <int CW>
static long host_project_bundles(const leap_geometry *G, const std::vector<float> (&volz)[2], int nzp, float *sino)
{
    const int NQ = G->fp_nq, NKP = G->fp_nkp;
    const int nbundles = (G->g.ncols + CW - 1) / CW;
    long uncovered = 0;
#pragma omp parallel for collapse(2) reduction(+ : uncovered)
    for (int a = 0; a < G->g.nviews; ++a)
        for (int b = 0; b < nbundles; ++b) {
            const int c0 = b * CW;
            const SfGeom &g = G->geoms.empty() ? G->g : G->geoms[a];      // modular: the view's own parameter block
            const double zkp = sf_kappa_const(g);
            const SfView v = G->views[a];
            const int xmajor = G->major[(size_t)a * nbundles + b];
            const SfRayLines L = sf_ray_lines(g, v, c0, CW, xmajor);
            const int n_major = xmajor ? g.nx : g.ny, n_minor = xmajor ? g.ny : g.nx;
            const SfSlab slab = {0, n_major, xmajor, 1, n_major};
            std::vector<float> acc((size_t)g.nrows * CW, 0.f);
            for (int n = 0; n < n_major; ++n) {
                int qf, ql;
                sf_candidates(L, n, qf, ql);
                if (ql - qf + 1 > NQ) ++uncovered;
                for (int s = 0; s < NQ; ++s) {
                    const int q = qf + s;
                    if (q < 0 || q >= n_minor || q > ql) continue;
                    const int i = xmajor ? n : q, j = xmajor ? q : n;
                    float fa[CW];
                    double mu;
                    if (!sf_candidate_record<CW, -1>(g, v, i, j, c0, true, fa, mu)) continue;
                    const float *col = &volz[xmajor][(size_t)sf_slab_column(slab, g.nx, i, j) * nzp];
                    const int P = (NKP > 4 && (float)mu <= 1.4999f) ? 4 : NKP;
                    switch (P) {
                    case 2: host_pairs_of_candidate<CW, 2>(g, col, nzp, mu, zkp, fa, acc); break;
                    case 3: host_pairs_of_candidate<CW, 3>(g, col, nzp, mu, zkp, fa, acc); break;
                    case 4: host_pairs_of_candidate<CW, 4>(g, col, nzp, mu, zkp, fa, acc); break;
                    case 5: host_pairs_of_candidate<CW, 5>(g, col, nzp, mu, zkp, fa, acc); break;
                    case 6: host_pairs_of_candidate<CW, 6>(g, col, nzp, mu, zkp, fa, acc); break;
                    default: host_pairs_of_candidate<CW, 7>(g, col, nzp, mu, zkp, fa, acc); break;
                    }
                }
            }
            for (int cw = 0; cw < CW && c0 + cw < g.ncols; ++cw) {
                const SfAmpCol ac = sf_amp_col(g, v, c0 + cw);
                for (int r = 0; r < g.nrows; ++r)
                    sino[((size_t)a * g.nrows + r) * g.ncols + c0 + cw] = sf_amp(g, v, ac, r) * acc[(size_t)r * CW + cw];
            }
        }
    return uncovered;
}

// Returns -1 when the handle does not use the column kernel, else the number of (view, bundle, slab) cases in which the
// candidate slots do not cover the candidate range (must be 0).
extern "C" long host_project_columns(const leap_geometry *G, const float *vol, float *sino)
{
    const SfGeom &g = G->g;
    if (!G->fp_columns) return -1;
    const int nzp = g.nz + 2 * FP_PAD;
    // the z-fastest copy in both slab layouts (a slab across x is laid out differently from one across y)
    std::vector<float> volz[2];
    for (int xmajor = 0; xmajor < 2; ++xmajor) {
        const SfSlab slab = {0, xmajor ? g.nx : g.ny, xmajor, 1, xmajor ? g.nx : g.ny};
        volz[xmajor].assign((size_t)g.nx * g.ny * nzp, 0.f);
        for (int k = 0; k < g.nz; ++k)
            for (int j = 0; j < g.ny; ++j)
                for (int i = 0; i < g.nx; ++i)
                    volz[xmajor][(size_t)sf_slab_column(slab, g.nx, i, j) * nzp + FP_PAD + k] = vol[((size_t)k * g.ny + j) * g.nx + i];
    }
    switch (G->fp_cw) {
    case 1: return host_project_bundles<1>(G, volz, nzp, sino);
    case 2: return host_project_bundles<2>(G, volz, nzp, sino);
    default: return host_project_bundles<4>(G, volz, nzp, sino);
    }
}

// ---- Siddon column-wise forward projection: the kernel's own functions, serially, with every read of the padded copy
// checked ----
// Returns -1 when the handle does not use that kernel, else the number of reads that would leave the scratch array.
extern "C" long host_sd_project_columns(const leap_geometry *G, const float *vol, float *sino)
{
    const SfGeom &gk = G->g;
    const SfGeom &g = gk;
    if (!G->sd_columns) return -1;
    const int nzp = g.nz + 2 * FP_PAD, kmax = nzp - 2;
    const size_t total = ((size_t)g.nx * g.ny + 1) * nzp;
    const unsigned zero_col = (unsigned)g.nx * (unsigned)g.ny * (unsigned)nzp;
    std::vector<float> volz(total, 0.f);
    for (int k = 0; k < g.nz; ++k)
        for (int j = 0; j < g.ny; ++j)
            for (int i = 0; i < g.nx; ++i) volz[((size_t)j * g.nx + i) * nzp + FP_PAD + k] = vol[((size_t)k * g.ny + j) * g.nx + i];
    long bad = 0;
#pragma omp parallel for collapse(2) reduction(+ : bad)
    for (int a = 0; a < g.nviews; ++a)
        for (int c = 0; c < g.ncols; ++c) {
            const SfGeom &g = G->geoms.empty() ? gk : G->geoms[a];        // modular: the view's own parameter block
            const SdRayCol R = G->raycols[(size_t)a * g.ncols + c];
            const int n_major = R.xmajor ? g.nx : g.ny, n_minor = R.xmajor ? g.ny : g.nx;
            for (int r = 0; r < g.nrows; ++r) {
                const SdAxial A = sd_axial(g, R, r);
                float acc = 0.f;
                for (int n = 0; n < n_major; ++n) {
                    const SdSplit s = sd_slab_split(R, n);
                    const bool a_ok = s.qa >= 0 && s.qa < n_minor, b_ok = s.qa != s.qb && s.qb >= 0 && s.qb < n_minor;
                    const unsigned base_a = a_ok ? (unsigned)(R.xmajor ? s.qa * g.nx + n : n * g.nx + s.qa) * (unsigned)nzp : zero_col;
                    const unsigned base_b = b_ok ? (unsigned)(R.xmajor ? s.qb * g.nx + n : n * g.nx + s.qb) * (unsigned)nzp : zero_col;
                    int kf;
                    float tlow;
                    sd_axial_place(A, fma((double)n, R.dh, R.h0), kmax, kf, tlow);
                    if (kf < 0 || (size_t)base_a + kf + 1 >= total || (size_t)base_b + kf + 1 >= total) { ++bad; continue; }
                    const float *xa = &volz[(size_t)base_a + kf], *xb = &volz[(size_t)base_b + kf];
                    acc = s.qa != s.qb ? sd_gather_two(xa, xb, A.inc, s.f, 1.0f - s.f, tlow, acc) : sd_gather_one(xa, tlow, acc);
                }
                sino[((size_t)a * g.nrows + r) * g.ncols + c] = sd_ray_length(R, A.vr) * acc;
            }
        }
    return bad;
}

// ---- Siddon model on tilted modules: the per-lane forward kernel, slab by slab, with the kernel's own functions ---------
// Returns -1 when the handle does not use that kernel, else the number of samples that came out non-finite (the slab
// copies sit between guard bands of NaN, so a gather outside a copy shows).
extern "C" long host_md_project_columns(const leap_geometry *G, const float *vol, float *sino, int width)
{
    const SfGeom &g = G->g;
    if (!G->md_tilted) return -1;
    const int nzp = g.nz + 2 * FP_PAD;
    const size_t guard = 4096;
    std::vector<float> acc((size_t)g.nviews * g.nrows * g.ncols, 0.f);
    for (int xmajor = 1; xmajor >= 0; --xmajor) {
        const int n_major = xmajor ? g.nx : g.ny, n_side = xmajor ? g.ny : g.nx;
        for (int n0 = 0; n0 < n_major; n0 += width) {
            const int n1 = std::min(n0 + width, n_major);
            const SfSlab slab = {n0, n1, xmajor, n0 == 0 ? 1 : 0, width};
            const size_t columns = (size_t)width * n_side;
            std::vector<float> buf(2 * guard + (columns + 1) * nzp, NAN);
            float *volz = buf.data() + guard;
            std::fill(volz, volz + (columns + 1) * nzp, 0.f);
            for (int n = n0; n < n1; ++n)
                for (int q = 0; q < n_side; ++q) {
                    const int i = xmajor ? n : q, j = xmajor ? q : n;
                    float *col = volz + (size_t)sf_slab_column(slab, g.nx, i, j) * nzp + FP_PAD;
                    for (int k = 0; k < g.nz; ++k) col[k] = vol[((size_t)k * g.ny + j) * g.nx + i];
                }
            const unsigned zero_col = (unsigned)(columns * nzp);
#pragma omp parallel for collapse(2)
            for (int a = 0; a < g.nviews; ++a)
                for (int r = 0; r < g.nrows; ++r)
                    for (int c = 0; c < g.ncols; ++c) {
                        const MdSlabRay M = md_slab_ray(g, G->poses[a], r, c);
                        const MdAxial A = md_axial(M);
                        const bool mine = M.R.xmajor == xmajor;
                        float t = 0.f;
                        for (int n = n0; n < n1; ++n) t = md_slab_step(g, M, A, n, slab, volz, nzp, zero_col, mine, t);
                        if (mine) acc[((size_t)a * g.nrows + r) * g.ncols + c] += M.len * t;
                    }
        }
    }
    long bad = 0;
    for (size_t q = 0; q < acc.size(); ++q) {
        sino[q] = acc[q];
        bad += !std::isfinite(acc[q]);
    }
    return bad;
}

// ---- Siddon model on tilted modules: the tiled back projection, tile by tile, with the kernel's own functions ------------
// report[0]: (view, tile, chunk) windows wider or taller than the instance stages; report[1]: reads outside the staged
// window; report[2]: slots outside the per-thread sums.  Returns -1 when the handle does not use that kernel.
template <int ZC, int PW, int PH>
static void host_md_bp_shape(const leap_geometry *G, const float *sino, float *vol, int64_t *report)
{
    const SfGeom &g = G->g;
    constexpr int PS = PW + 1, NSLOT = ZC + 4;
    const int tiles_x = (g.nx + BP_T - 1) / BP_T, tiles_y = (g.ny + BP_T - 1) / BP_T, chunks = (g.nz + ZC - 1) / ZC;
    int64_t wide = 0, outside = 0, badslot = 0;
#pragma omp parallel for collapse(2) reduction(+ : wide, outside, badslot)
    for (int ch = 0; ch < chunks; ++ch)
        for (int tile = 0; tile < tiles_x * tiles_y; ++tile) {
            const int i0 = (tile % tiles_x) * BP_T, j0 = (tile / tiles_x) * BP_T, k0 = ch * ZC;
            std::vector<float> sums((size_t)NSLOT * 256, 0.f);
            std::vector<MdBpPixel> px((size_t)PH * PS);
            for (int a = 0; a < g.nviews; ++a) {
                const MdBpView &V = G->d_mdbp[a];
                const SfWindow win = md_bp_window(g, V, i0, j0, k0, ZC);
                wide += win.need_w > PW || win.need_h > PH;
                const bool xmajor = md_bp_tile_xmajor(g, V, i0, j0);
                for (int sc = 0; sc < PW; ++sc) {
                    const int c = win.c0 + sc;
                    for (int row = 0; row < PH; ++row) {
                        const int r = win.r0 + row;
                        const bool in = c >= 0 && c < g.ncols && r >= 0 && r < g.nrows;
                        const float y = in ? sino[((size_t)a * g.nrows + r) * g.ncols + c] : 0.f;
                        px[(size_t)row * PS + sc] = md_bp_pixel(md_bp_slopes(g, V, xmajor, r, c), y);
                    }
                }
                const int H = std::min(win.need_h, PH);
                for (int tid = 0; tid < 256; ++tid) {
                    const int i = i0 + (tid & (BP_T - 1)), j = j0 + (tid >> 4);
                    const int ic = std::min(i, g.nx - 1), jc = std::min(j, g.ny - 1);
                    const MdBpColumn C = md_bp_column<ZC>(g, V, xmajor, ic, jc, k0);
                    const int cbeg = std::max(C.cfirst, win.c0), cend = std::min(C.clast, win.c0 + PW - 1);
                    for (int c = cbeg; c <= cend; ++c) {
                        const int wc = c - win.c0;
                        if (c < 0 || c >= g.ncols) continue;
                        int rs, re;
                        md_bp_rows(C, c, win.r0, H, rs, re);
                        for (int row = rs; row < re; ++row) {
                            if (row < 0 || row >= PH) { ++outside; continue; }
                            int slot;
                            float w_low, w_high;
                            if (!md_bp_row<ZC>(C, px[(size_t)row * PS + wc], slot, w_low, w_high)) continue;
                            if (slot < 0 || slot + 1 >= NSLOT) { ++badslot; continue; }
                            sums[(size_t)slot * 256 + tid] += w_low;
                            sums[(size_t)(slot + 1) * 256 + tid] += w_high;
                        }
                    }
                }
            }
            for (int tid = 0; tid < 256; ++tid) {
                const int i = i0 + (tid & (BP_T - 1)), j = j0 + (tid >> 4);
                if (i >= g.nx || j >= g.ny) continue;
                for (int kk = 0; kk < ZC && k0 + kk < g.nz; ++kk)
                    vol[((size_t)(k0 + kk) * g.ny + j) * g.nx + i] = sums[(size_t)(kk + 2) * 256 + tid];
            }
        }
    report[0] = wide; report[1] = outside; report[2] = badslot;
}

extern "C" long host_md_backproject_tiled(const leap_geometry *G, const float *sino, float *vol, int64_t *report)
{
    if (!G->d_mdbp || !G->bp_tiled) return -1;
    switch (G->bp_shape) {
    case 0: host_md_bp_shape<MD_BP_SHAPES[0].zc, MD_BP_SHAPES[0].pw, MD_BP_SHAPES[0].ph>(G, sino, vol, report); break;
    case 1: host_md_bp_shape<MD_BP_SHAPES[1].zc, MD_BP_SHAPES[1].pw, MD_BP_SHAPES[1].ph>(G, sino, vol, report); break;
    case 2: host_md_bp_shape<MD_BP_SHAPES[2].zc, MD_BP_SHAPES[2].pw, MD_BP_SHAPES[2].ph>(G, sino, vol, report); break;
    case 3: host_md_bp_shape<MD_BP_SHAPES[3].zc, MD_BP_SHAPES[3].pw, MD_BP_SHAPES[3].ph>(G, sino, vol, report); break;
    case 4: host_md_bp_shape<MD_BP_SHAPES[4].zc, MD_BP_SHAPES[4].pw, MD_BP_SHAPES[4].ph>(G, sino, vol, report); break;
    case 5: host_md_bp_shape<MD_BP_SHAPES[5].zc, MD_BP_SHAPES[5].pw, MD_BP_SHAPES[5].ph>(G, sino, vol, report); break;
    default: return -1;
    }
    return report[0] + report[1] + report[2];
}
