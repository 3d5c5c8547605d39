// Host geometry module: validates the CT parameter set ("PyTorch Interfaces and CT Parameters") and turns
// it into the constant tables the kernels read.  All derivations run in double; the tables are rounded to
// float once, here.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <cstring>
#include <new>

#include "leap_internal.h"
#define SF_NO_KERNELS   // this file needs the kernels' host-side limit functions only
#include "sf_backproject_tiled.h"
#include "sf_project_columns.h"
#include "sd_backproject_tiled.h"

static thread_local std::string g_last_error;

void leap_set_error(const std::string &msg) { g_last_error = msg; }

int leap_hip_fail(hipError_t e, const char *what)
{
    g_last_error = std::string(what) + ": " + hipGetErrorString(e);
    return LEAP_HIP_ERROR;
}

extern "C" const char *leap_last_error(void) { return g_last_error.c_str(); }

extern "C" const char *leap_status_string(int status)
{
    switch (status) {
    case LEAP_OK: return "ok";
    case LEAP_INVALID_ARG: return "invalid argument";
    case LEAP_BAD_GEOMETRY: return "geometry not supported: source must lie strictly outside the volume";
    case LEAP_HIP_ERROR: return "HIP runtime error";
    case LEAP_UNSUPPORTED: return "size not supported";
    default: return "unknown status";
    }
}

static int invalid(const char *why)
{
    leap_set_error(why);
    return LEAP_INVALID_ARG;
}

static bool finite_pos(double v) { return std::isfinite(v) && v > 0.0; }

// Siddon model: constants of the line of every (view, detector column), in double ("sd_ray.h" states the formulation).
static void build_ray_table(leap_geometry *G)
{
    const leap_geometry_desc &d = G->desc;
    const double T = d.voxel_xy, Tz = d.voxel_z;
    G->raycols.resize((size_t)d.nviews * d.ncols);
    double max_slope = 0.0;
    for (int a = 0; a < d.nviews; ++a) {
        // modular scans with upright modules bring one parameter block per view: a circular cone-beam view of the
        // translated scene, with its own source distance, detector distance and column offset
        const bool per_view = !G->geoms.empty();
        const SfGeom &g = per_view ? G->geoms[a] : G->g;
        const int type = per_view ? (int)LEAP_CONE : d.type;
        const double sod = per_view ? g.sodd : d.sod, sdd = per_view ? g.kud * d.pixel_u : d.sdd;
        const double xlo = g.x0d - 0.5 * T, ylo = g.y0d - 0.5 * T;      // lower faces of voxel (0, 0)
        const double c = G->views[a].cd, s = G->views[a].sd;
        double max_dh = 0.0;
        for (int col = 0; col < d.ncols; ++col) {
            const double u = ((double)col - g.col_offd) * d.pixel_u;
            double ox, oy, dx, dy;
            if (type == LEAP_PARALLEL) {
                ox = -u * s; oy = u * c; dx = c; dy = s;
            } else if (type == LEAP_CONE_CURVED) {    // pixel at fan angle u / sdd on the cylinder
                const double cg = std::cos(u / sdd), sg = std::sin(u / sdd);
                ox = sod * c; oy = sod * s;
                dx = -sdd * (cg * c + sg * s); dy = sdd * (sg * c - cg * s);
            } else {
                ox = sod * c; oy = sod * s;
                dx = -sdd * c - u * s; dy = -sdd * s + u * c;
            }
            SdRayCol R;
            R.xmajor = std::fabs(dx) >= std::fabs(dy) ? 1 : 0;
            const double dmaj = R.xmajor ? dx : dy, dmin = R.xmajor ? dy : dx;
            const double omaj = R.xmajor ? ox : oy, omin = R.xmajor ? oy : ox;
            const double lomaj = R.xmajor ? xlo : ylo, lomin = R.xmajor ? ylo : xlo;
            R.m = dmin / dmaj;
            R.b = (omin - lomin) / T - R.m * (omaj - lomaj) / T;
            const double inv_m = R.m != 0.0 ? 1.0 / R.m : 1e30;
            R.inv_m = (float)std::fmin(std::fmax(inv_m, -1e30), 1e30);
            R.lxy = (float)(T * std::sqrt(dx * dx + dy * dy) / std::fabs(dmaj));
            if (type == LEAP_CONE || type == LEAP_CONE_CURVED) {
                R.h0 = (lomaj - omaj) / (dmaj * Tz);
                R.dh = T / (dmaj * Tz);
                R.vscale = (float)(T / std::fabs(dmaj));
            } else if (type == LEAP_PARALLEL) {
                R.h0 = 1.0 / Tz; R.dh = 0.0; R.vscale = 0.0f;
            } else {
                R.h0 = 0.0; R.dh = 0.0; R.vscale = 0.0f;
            }
            max_dh = std::fmax(max_dh, std::fabs(R.dh));
            G->raycols[(size_t)a * d.ncols + col] = R;
        }
        const double vmax = std::fmax(std::fabs(g.v0d), std::fabs(g.v0d + (d.nrows - 1) * g.pvd));
        max_slope = std::fmax(max_slope, max_dh * vmax);
    }
    G->sd_max_axial_slope = max_slope;
}

// Modular geometry, footprint model: static limits of the two fast kernels, checked view by view on each view's own
// parameter block (the same checks the circular scanners get in leap_geometry_create).
static void select_modular_fast_kernels(leap_geometry *G)
{
    const leap_geometry_desc *d = &G->desc;
    const double T = d->voxel_xy, half_x = 0.5 * d->nx * T, half_y = 0.5 * d->ny * T;
    double cols = 0.0, rows = 0.0, vpr = 0.0;
    for (int a = 0; a < d->nviews; ++a) {
        const SfGeom &ga = G->geoms[a];
        const double cx = ga.x0d + 0.5 * (d->nx - 1) * T, cy = ga.y0d + 0.5 * (d->ny - 1) * T;
        const double rx = std::fabs(cx) + half_x, ry = std::fabs(cy) + half_y;
        const double reach = std::sqrt(rx * rx + ry * ry) + T;
        const double sdd = ga.kud * d->pixel_u, lS = ga.sodd;
        if (!(lS > reach)) return;
        const double mag_max = sdd / (lS - reach), mag_min = sdd / (lS + reach);
        const double umax = std::fmax(std::fabs(-2.0 - ga.col_offd), std::fabs(d->ncols + 1.0 - ga.col_offd)) * d->pixel_u;
        const double stretch = 1.02 / std::cos(std::atan(umax / sdd));
        cols = std::fmax(cols, mag_max * T * std::sqrt(2.0) / d->pixel_u * stretch);
        rows = std::fmax(rows, mag_max * d->voxel_z / d->pixel_v);
        vpr = std::fmax(vpr, d->pixel_v / (mag_min * d->voxel_z));
    }
    G->max_cols_per_voxel = cols; G->max_rows_per_voxel = rows; G->max_voxels_per_row = vpr;
    if (const char *env = std::getenv("LEAP_FORCE_GENERAL"))
        if (env[0] == '1') return;

    if (d->nz >= 8 && std::isfinite(cols) && cols <= 4.0 && rows <= 3.0 && (double)d->nrows * d->ncols < 1073741824.0) {
        G->bp_nc = std::max(2, (int)std::ceil(cols) + 1);
        G->bp_nv = std::max(2, (int)std::ceil(rows - 1e-6) + 1);
        G->bp_wh = (float)(0.5 * cols);
        const int tiles_x = (d->nx + BP_T - 1) / BP_T, tiles_y = (d->ny + BP_T - 1) / BP_T;
        const float hx = 0.5f * (float)(BP_T - 1) * G->g.T;
        for (int sh = d->nz >= 128 ? 0 : 1; sh < BP_NSHAPES && !G->bp_tiled; ++sh) {
            const int zc = BP_SHAPES[sh].zc, chunks = (d->nz + zc - 1) / zc;
            int need_w = 0, need_h = 0;
            for (int a = 0; a < d->nviews; ++a)
                for (int ty = 0; ty < tiles_y; ++ty)
                    for (int tx = 0; tx < tiles_x; ++tx)
                        for (int ch = 0; ch < chunks; ch += (chunks > 1 ? chunks - 1 : 1)) {
                            const SfGeom &ga = G->geoms[a];
                            const float xc = (float)(ga.x0d + ((double)(tx * BP_T) + 0.5 * (BP_T - 1)) * ga.Td);
                            const float yc = (float)(ga.y0d + ((double)(ty * BP_T) + 0.5 * (BP_T - 1)) * ga.Td);
                            const float z0 = (float)(ga.zlo0d + (double)(ch * zc) * ga.Tzd), z1 = z0 + (float)zc * ga.Tz;
                            const SfWindow w = sf_bp_window(ga, G->views[a], xc, yc, hx, z0, z1, G->bp_wh, G->bp_nc, G->bp_nv);
                            need_w = std::max(need_w, w.need_w);
                            need_h = std::max(need_h, w.need_h);
                        }
            G->bp_need_w = need_w; G->bp_need_h = need_h; G->bp_shape = sh;
            G->bp_tiled = need_w <= BP_SHAPES[sh].pw - 1 && need_h <= BP_SHAPES[sh].ph - 1;
        }
    }
    if (d->nrows >= 32 && std::isfinite(vpr) && vpr <= 3.0 && (double)d->nx * d->ny * (d->nz + 2.0 * FP_PAD) < 4294967296.0 &&
        d->ny <= 65535) {
        auto slots_needed = [&](int cw) {
            int need = 0;
            for (int a = 0; a < d->nviews && need <= 16; ++a)
                for (int c = 0; c < d->ncols; c += cw) {
                    const SfRayLines L = sf_ray_lines(G->geoms[a], G->views[a], c, cw);
                    const int n_major = L.xmajor ? d->nx : d->ny;
                    const float d0 = std::fabs(L.b0 - L.b1);
                    const float d1 = std::fabs(fmaf(L.m0 - L.m1, (float)(n_major - 1), L.b0 - L.b1));
                    const float dm = d0 > d1 ? d0 : d1;
                    if (!(dm < 1e6f)) return 1 << 20;
                    need = std::max(need, (int)std::floor(dm + 2.0f * L.spread + 1e-3f) + 2);
                }
            return need;
        };
        G->fp_cw = 4;                              // the modular instances exist for bundles of 4 and 2 columns
        if (const char *env = std::getenv("LEAP_FP_CW")) {
            const int v = std::atoi(env);
            if (v == 2 || v == 4) G->fp_cw = v;
        }
        G->fp_nk = std::max(2, (int)std::ceil(vpr - 1e-6) + 1);
        const int groups = (d->nrows + 63) / 64;
        G->fp_rg = groups >= 8 ? 8 : (groups >= 4 ? 4 : (groups >= 2 ? 2 : 1));
        if (G->fp_rg < 4 && !std::getenv("LEAP_FP_CW")) G->fp_cw = 2;      // short detectors: see leap_geometry_create
        int need = slots_needed(G->fp_cw);
        if (need > 16 && G->fp_cw == 4) {
            G->fp_cw = 2;
            need = slots_needed(2);
        }
        G->fp_need_q = need;
        G->fp_nq = need <= 4 ? 4 : (need <= 8 ? 8 : 16);
        G->fp_columns = need <= 16 && G->fp_nk <= 4;
    }
}

// Siddon model: static limits of the two fast kernels.  With per-view parameter blocks (upright modular scans) every
// view is checked on its own block.
static void select_siddon_fast_kernels(leap_geometry *G)
{
    const leap_geometry_desc *d = &G->desc;
    const bool per_view = !G->geoms.empty();
    if (d->type == LEAP_FAN || !(G->sd_max_axial_slope <= 0.999)) return;
    if (const char *env = std::getenv("LEAP_FORCE_GENERAL"))
        if (env[0] == '1') return;

    // wave-per-column forward projection: no ray may cross more than one z-face per slab
    if (d->nrows >= 32 && ((double)d->nx * d->ny + 1.0) * (d->nz + 2.0 * FP_PAD) < 4294967296.0 && d->ny <= 65535) {
        G->sd_columns = true;
        const int groups = (d->nrows + 63) / 64;
        G->fp_rg = groups >= 8 ? 8 : (groups >= 4 ? 4 : (groups >= 2 ? 2 : 1));
        if (const char *env = std::getenv("LEAP_FP_VB")) {
            const int v = std::atoi(env);
            if (v >= 1 && v <= 1024) G->fp_vb = v;
        }
        if (const char *env = std::getenv("LEAP_FP_TB")) {
            const int v = std::atoi(env);
            if (v >= 1 && v <= 1024) G->fp_tb = v;
        }
        if (const char *env = std::getenv("LEAP_FP_RG")) {
            const int v = std::atoi(env);
            if (v == 1 || v == 2 || v == 4 || v == 8) G->fp_rg = v;
        }
    }

    // tiled back projection: at most 4 pixel centres inside a voxel's footprint, and the staged window of every
    // (view, tile, z-chunk) must fit the instance (checked with the kernel's own function)
    if (d->nz >= 8 && std::isfinite(G->max_cols_per_voxel) && G->max_cols_per_voxel > 0.0 && G->max_cols_per_voxel < 3.9 &&
        (double)d->nrows * d->ncols < 1073741824.0) {      // the staging loads use 32-bit byte offsets within a view
        G->bp_nc = (int)std::floor(G->max_cols_per_voxel + 0.01) + 1;
        if (G->bp_nc < 2) G->bp_nc = 2;
        const int tiles_x = (d->nx + BP_T - 1) / BP_T, tiles_y = (d->ny + BP_T - 1) / BP_T;
        const float hx = 0.5f * (float)BP_T * G->g.T;
        int first_shape = 1;                          // the 64-voxel shape does not fit: the sums live in LDS
        if (const char *env = std::getenv("LEAP_BP_SHAPE")) {
            first_shape = std::atoi(env) % BP_NSHAPES;
            if (first_shape < 1) first_shape = 1;
        }
        for (int sh = first_shape; sh < BP_NSHAPES && !G->bp_tiled; ++sh) {
            const int zc = BP_SHAPES[sh].zc;
            const int chunks = (d->nz + zc - 1) / zc;
            int need_w = 0, need_h = 0;
            for (int a = 0; a < d->nviews; ++a) {
                const SfGeom &g = per_view ? G->geoms[a] : G->g;
                for (int ty = 0; ty < tiles_y; ++ty)
                    for (int tx = 0; tx < tiles_x; ++tx) {
                        const float xc = (float)(g.x0d + ((double)(tx * BP_T) + 0.5 * (BP_T - 1)) * g.Td);
                        const float yc = (float)(g.y0d + ((double)(ty * BP_T) + 0.5 * (BP_T - 1)) * g.Td);
                        for (int ch = 0; ch < chunks; ch += (chunks > 1 ? chunks - 1 : 1)) {
                            const float z0 = (float)(g.zlo0d + (double)(ch * zc) * g.Tzd), z1 = z0 + (float)zc * g.Tz;
                            const SfWindow w = sd_bp_window(g, G->views[a], xc, yc, hx, z0, z1);
                            need_w = w.need_w > need_w ? w.need_w : need_w;
                            need_h = w.need_h > need_h ? w.need_h : need_h;
                        }
                    }
            }
            G->bp_need_w = need_w;
            G->bp_need_h = need_h;
            G->bp_shape = sh;
            G->bp_tiled = need_w <= BP_SHAPES[sh].pw - 1 && need_h <= BP_SHAPES[sh].ph - 1;
        }
    }
}

// Modular geometry: per-view poses instead of the angle list; only the fields the modular kernels read are filled.
static int create_modular(const leap_geometry_desc *d, leap_geometry **out)
{
    if (!d->poses) return invalid("poses is null");
    if (d->nviews > 65535 || (double)d->nx * d->ny * d->nz >= 4294967296.0 ||
        (double)d->nviews * d->nrows * d->ncols >= 4294967296.0 || d->ny > 262140 || d->nz > 65535 || d->nrows > 262140) {
        leap_set_error("sizes beyond what one launch covers");
        return LEAP_UNSUPPORTED;
    }
    const double half[3] = {0.5 * d->nx * d->voxel_xy, 0.5 * d->ny * d->voxel_xy, 0.5 * d->nz * d->voxel_z};
    const double ctr[3] = {d->center_x, d->center_y, d->center_z};
    for (int a = 0; a < d->nviews; ++a) {
        const double *p = d->poses + 12 * (size_t)a;
        for (int q = 0; q < 12; ++q)
            if (!std::isfinite(p[q])) return invalid("poses must be finite");
        const double uu = p[6] * p[6] + p[7] * p[7] + p[8] * p[8], vv = p[9] * p[9] + p[10] * p[10] + p[11] * p[11];
        const double uv = p[6] * p[9] + p[7] * p[10] + p[8] * p[11];
        if (std::fabs(uu - 1.0) > 1e-9 || std::fabs(vv - 1.0) > 1e-9 || std::fabs(uv) > 1e-9)
            return invalid("detector axes must be orthonormal");
        bool inside = true;
        for (int q = 0; q < 3; ++q) inside = inside && std::fabs(p[q] - ctr[q]) <= half[q];
        if (inside) {
            leap_set_error("a source lies inside the volume");
            return LEAP_BAD_GEOMETRY;
        }
    }
    // Upright modules (column axis horizontal, row axis +z, detector behind the volume as seen from the source, source
    // clear of the volume's bounding circle in the module's frame) are circular cone-beam views of a translated scene:
    // the footprint construction needs them, the Siddon model uses them for its fast kernels.
    bool upright = true;
    const char *why_not = "";
    int why_status = LEAP_OK;
    for (int a = 0; a < d->nviews && upright; ++a) {
        const double *p = d->poses + 12 * (size_t)a;
        if (std::fabs(p[8]) > 1e-9 || std::fabs(p[9]) > 1e-9 || std::fabs(p[10]) > 1e-9 || std::fabs(p[11] - 1.0) > 1e-9) {
            upright = false;
            why_not = "the footprint model needs upright modules (column axis horizontal, row axis +z); "
                      "use LEAP_MODEL_SIDDON for tilted ones";
            why_status = LEAP_UNSUPPORTED;
            break;
        }
        const double c = p[7], s = -p[6];
        const double lS = p[0] * c + p[1] * s, lD = p[3] * c + p[4] * s, tS = -p[0] * s + p[1] * c;
        // the volume as this view sees it: moved by -tS along the column axis
        const double mx = std::fabs(d->center_x - tS * p[6]) + half[0], my = std::fabs(d->center_y - tS * p[7]) + half[1];
        const double reach_a = std::sqrt(mx * mx + my * my);
        if (!(lS - lD > 0.0) || !(lS > reach_a) || !(d->pixel_u < 0.25 * (lS - lD))) {
            upright = false;
            why_not = "module does not face its source across the volume";
            why_status = LEAP_BAD_GEOMETRY;
        }
    }
    if (d->model == LEAP_MODEL_SF && !upright) {
        leap_set_error(why_not);
        return why_status;
    }
    leap_geometry *G = new (std::nothrow) leap_geometry;
    if (!G) return invalid("out of host memory");
    G->desc = *d;
    G->desc.angles_rad = nullptr;
    SfGeom &g = G->g;
    std::memset(&g, 0, sizeof(g));
    g.type = d->type; g.model = d->model;
    g.nviews = d->nviews; g.nrows = d->nrows; g.ncols = d->ncols;
    g.nx = d->nx; g.ny = d->ny; g.nz = d->nz;
    g.Td = d->voxel_xy; g.Tzd = d->voxel_z;
    g.x0d = d->center_x - 0.5 * (d->nx - 1) * d->voxel_xy;
    g.y0d = d->center_y - 0.5 * (d->ny - 1) * d->voxel_xy;
    g.zlo0d = d->center_z - 0.5 * d->nz * d->voxel_z;
    g.col_offd = 0.5 * (d->ncols - 1) - d->shift_u;
    g.row_offd = 0.5 * (d->nrows - 1) - d->shift_v + 0.5;
    g.v0d = (-0.5 * (d->nrows - 1) + d->shift_v) * d->pixel_v;
    g.pvd = d->pixel_v;
    g.pu_d = d->pixel_u;
    g.T = (float)d->voxel_xy; g.Tz = (float)d->voxel_z; g.pu = (float)d->pixel_u; g.pv = (float)d->pixel_v;
    G->poses.resize(d->nviews);
    std::memcpy(G->poses.data(), d->poses, sizeof(MdPose) * (size_t)d->nviews);
    G->desc.poses = reinterpret_cast<const double *>(G->poses.data());
    if (upright) {
        // per view: the same scene translated so that the source sits on the frame's axis at height 0
        g.iTzd = 1.0 / d->voxel_z;
        G->views.resize(d->nviews);
        G->geoms.resize(d->nviews);
        const double h = 0.5 * d->voxel_xy;
        for (int a = 0; a < d->nviews; ++a) {
            const MdPose &P = G->poses[a];
            const double c = P.ucol[1], s = -P.ucol[0];
            const double lS = P.S[0] * c + P.S[1] * s, tS = -P.S[0] * s + P.S[1] * c, zS = P.S[2];
            const double sdd = lS - (P.C[0] * c + P.C[1] * s), tC = -P.C[0] * s + P.C[1] * c, zC = P.C[2];
            SfView &v = G->views[a];
            std::memset(&v, 0, sizeof(v));
            v.cd = c; v.sd = s; v.c = (float)c; v.s = (float)s;
            v.p = (float)(h * c); v.q = (float)(h * s);
            v.xmajor = std::fabs(c) >= std::fabs(s) ? 1 : 0;
            SfGeom &ga = G->geoms[a];
            ga = g;
            ga.type = SF_CONE;
            ga.x0d = g.x0d - tS * P.ucol[0];
            ga.y0d = g.y0d - tS * P.ucol[1];
            ga.zlo0d = g.zlo0d - zS;
            ga.sodd = lS;
            ga.kud = sdd / d->pixel_u; ga.kvd = sdd / d->pixel_v; ga.ikvd = 1.0 / ga.kvd;
            ga.col_offd = g.col_offd - (tC - tS) / d->pixel_u;
            ga.row_offd = g.row_offd - (zC - zS) / d->pixel_v;
            ga.v0d = g.v0d + (zC - zS);
            ga.zk0d = -ga.zlo0d / d->voxel_z;
            ga.sod = (float)lS; ga.sdd = (float)sdd; ga.ku = (float)ga.kud;
            ga.col_off = (float)ga.col_offd; ga.v0 = (float)ga.v0d;
        }
    }
    if (d->model == LEAP_MODEL_SF) select_modular_fast_kernels(G);
    if (d->model == LEAP_MODEL_SIDDON && upright) {
        build_ray_table(G);
        select_modular_fast_kernels(G);      // footprint bounds (columns per voxel) are what the Siddon limits need too
        G->bp_tiled = G->fp_columns = false;
        G->bp_shape = 0;
        select_siddon_fast_kernels(G);
    }
    hipError_t e = hipGetDevice(&G->device);
    if (e == hipSuccess) (void)leap_static_scratch_init(G->device);   // set-up for leap_project_static_scratch; it reports a failure itself
    if (e == hipSuccess && (G->fp_columns || G->sd_columns)) {
        G->nzp = d->nz + 2 * FP_PAD;
        const size_t bytes = sizeof(float) * ((size_t)d->nx * d->ny + 1) * G->nzp;
        hipError_t es = hipMalloc((void **)&G->d_volz, bytes);
        if (es == hipSuccess) es = hipMemset(G->d_volz, 0, bytes);
        if (es == hipSuccess) es = hipDeviceSynchronize();
        if (es != hipSuccess) {
            if (G->d_volz) (void)hipFree(G->d_volz);
            G->d_volz = nullptr;
            G->fp_columns = G->sd_columns = false;
            (void)hipGetLastError();
        }
    }
    if (e == hipSuccess && (G->sd_columns || (G->bp_tiled && d->model == LEAP_MODEL_SIDDON))) {
        const size_t bytes = sizeof(SdRayCol) * G->raycols.size();
        e = hipMalloc((void **)&G->d_raycols, bytes);
        if (e == hipSuccess) e = hipMemcpy(G->d_raycols, G->raycols.data(), bytes, hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && !G->geoms.empty()) {
        e = hipMalloc((void **)&G->d_geoms, sizeof(SfGeom) * G->geoms.size());
        if (e == hipSuccess) e = hipMemcpy(G->d_geoms, G->geoms.data(), sizeof(SfGeom) * G->geoms.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMalloc((void **)&G->d_views, sizeof(SfView) * G->views.size());
        if (e == hipSuccess) e = hipMemcpy(G->d_views, G->views.data(), sizeof(SfView) * G->views.size(), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipMalloc((void **)&G->d_poses, sizeof(MdPose) * (size_t)d->nviews);
    if (e == hipSuccess) e = hipMemcpy(G->d_poses, G->poses.data(), sizeof(MdPose) * (size_t)d->nviews, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (G->d_poses) (void)hipFree(G->d_poses);
        if (G->d_geoms) (void)hipFree(G->d_geoms);
        if (G->d_views) (void)hipFree(G->d_views);
        if (G->d_volz) (void)hipFree(G->d_volz);
        if (G->d_raycols) (void)hipFree(G->d_raycols);
        delete G;
        return leap_hip_fail(e, "uploading the pose table");
    }
    *out = G;
    return LEAP_OK;
}

extern "C" int leap_geometry_create(const leap_geometry_desc *d, leap_geometry **out)
{
    if (out) *out = nullptr;
    if (!d || !out) return invalid("null descriptor or output pointer");
    if (d->type != LEAP_PARALLEL && d->type != LEAP_FAN && d->type != LEAP_CONE && d->type != LEAP_CONE_CURVED &&
        d->type != LEAP_MODULAR)
        return invalid("unknown geometry type");
    if (d->model != LEAP_MODEL_SF && d->model != LEAP_MODEL_SIDDON) return invalid("unknown projector model");
    if (d->nviews <= 0 || d->nrows <= 0 || d->ncols <= 0) return invalid("nviews, nrows and ncols must be positive");
    if (d->nx <= 0 || d->ny <= 0 || d->nz <= 0) return invalid("nx, ny and nz must be positive");
    if (!finite_pos(d->pixel_u) || !finite_pos(d->pixel_v)) return invalid("pixel sizes must be positive");
    if (!finite_pos(d->voxel_xy) || !finite_pos(d->voxel_z)) return invalid("voxel sizes must be positive");
    if (!std::isfinite(d->shift_u) || !std::isfinite(d->shift_v)) return invalid("detector shifts must be finite");
    if (!std::isfinite(d->center_x) || !std::isfinite(d->center_y) || !std::isfinite(d->center_z))
        return invalid("volume centre must be finite");
    if (d->type == LEAP_MODULAR) return create_modular(d, out);
    if (!d->angles_rad) return invalid("angles_rad is null");
    for (int a = 0; a < d->nviews; ++a)
        if (!std::isfinite(d->angles_rad[a])) return invalid("view angles must be finite");
    if (d->type == LEAP_FAN && (d->nrows != 1 || d->nz != 1)) return invalid("fan-beam needs nrows == 1 and nz == 1");
    if (d->nviews > 65535) {
        leap_set_error("more than 65535 views in one geometry");
        return LEAP_UNSUPPORTED;
    }
    if ((double)d->nx * d->ny * d->nz >= 2147483648.0 * 2.0 || (double)d->nviews * d->nrows * d->ncols >= 2147483648.0 * 2.0) {
        leap_set_error("array of more than 2^32 elements");
        return LEAP_UNSUPPORTED;
    }

    const double T = d->voxel_xy, h = 0.5 * T;
    const double half_x = 0.5 * d->nx * T, half_y = 0.5 * d->ny * T;
    if (d->type != LEAP_PARALLEL) {
        if (!finite_pos(d->sdd) || !finite_pos(d->sod)) {
            leap_set_error("sod and sdd must be positive");
            return LEAP_BAD_GEOMETRY;
        }
        // farthest in-plane corner of the volume from the rotation axis
        const double rx = std::fabs(d->center_x) + half_x, ry = std::fabs(d->center_y) + half_y;
        const double reach = std::sqrt(rx * rx + ry * ry);
        if (!(d->sod > reach)) {
            leap_set_error("source orbit radius (sod) does not clear the volume's bounding circle");
            return LEAP_BAD_GEOMETRY;
        }
        if (!(d->pixel_u < 0.25 * d->sdd)) {
            leap_set_error("detector pixel wider than a quarter of sdd");
            return LEAP_BAD_GEOMETRY;
        }
        if (d->type == LEAP_CONE_CURVED && !((0.5 * d->ncols + std::fabs(d->shift_u) + 1.0) * d->pixel_u < 1.5 * d->sdd)) {
            leap_set_error("curved detector spans a fan of more than +-1.5 rad");
            return LEAP_BAD_GEOMETRY;
        }
    }

    leap_geometry *G = new (std::nothrow) leap_geometry;
    if (!G) return invalid("out of host memory");
    G->desc = *d;
    G->angles.assign(d->angles_rad, d->angles_rad + d->nviews);
    G->desc.angles_rad = G->angles.data();

    SfGeom &g = G->g;
    std::memset(&g, 0, sizeof(g));
    const bool par = d->type == LEAP_PARALLEL;
    g.type = d->type;
    g.nviews = d->nviews; g.nrows = d->nrows; g.ncols = d->ncols;
    g.nx = d->nx; g.ny = d->ny; g.nz = d->nz;
    g.Td = T; g.Tzd = d->voxel_z;
    g.x0d = d->center_x - 0.5 * (d->nx - 1) * T;
    g.y0d = d->center_y - 0.5 * (d->ny - 1) * T;
    g.zlo0d = d->center_z - 0.5 * d->nz * d->voxel_z;
    g.sodd = par ? 0.0 : d->sod;
    g.kud = par ? 1.0 / d->pixel_u : d->sdd / d->pixel_u;
    g.kvd = par ? 1.0 / d->pixel_v : d->sdd / d->pixel_v;
    g.ikvd = 1.0 / g.kvd;
    g.iTzd = 1.0 / d->voxel_z;
    g.col_offd = 0.5 * (d->ncols - 1) - d->shift_u;
    g.row_offd = 0.5 * (d->nrows - 1) - d->shift_v + 0.5;
    g.T = (float)T; g.Tz = (float)d->voxel_z;
    g.sod = (float)g.sodd; g.sdd = par ? 0.0f : (float)d->sdd;
    g.pu = (float)d->pixel_u; g.pv = (float)d->pixel_v;
    g.ku = (float)g.kud;
    g.col_off = (float)g.col_offd;
    g.v0 = (float)((-0.5 * (d->nrows - 1) + d->shift_v) * d->pixel_v);
    g.model = d->model;
    g.v0d = (-0.5 * (d->nrows - 1) + d->shift_v) * d->pixel_v;
    g.pvd = d->pixel_v;
    g.pu_d = d->pixel_u;
    g.zk0d = d->type == LEAP_FAN ? 0.5 : -g.zlo0d / d->voxel_z;

    G->views.resize(d->nviews);
    for (int a = 0; a < d->nviews; ++a) {
        const double c = std::cos(G->angles[a]), s = std::sin(G->angles[a]);
        SfView &v = G->views[a];
        v.cd = c; v.sd = s;
        v.c = (float)c; v.s = (float)s;
        v.p = (float)(h * c); v.q = (float)(h * s);
        v.par_out = (float)(h * (std::fabs(c) + std::fabs(s)) / d->pixel_u);
        v.par_in = (float)(h * std::fabs(std::fabs(c) - std::fabs(s)) / d->pixel_u);
        v.par_amp = (float)(T / std::fmax(std::fabs(c), std::fabs(s)));
        v.xmajor = std::fabs(c) >= std::fabs(s) ? 1 : 0;
    }

    if (d->model == LEAP_MODEL_SIDDON) build_ray_table(G);

    // Footprint bounds over the whole volume (double).  Magnification is extreme at the corner of the volume's
    // bounding circle; a flat detector stretches a footprint seen at fan angle gamma by 1/cos(gamma).
    {
        const double rx = std::fabs(d->center_x) + half_x, ry = std::fabs(d->center_y) + half_y;
        const double reach = std::sqrt(rx * rx + ry * ry) + T;
        double mag_max = 1.0, mag_min = 1.0, stretch = 1.0, slope = 1.0;
        if (!par) {
            mag_max = d->sdd / std::fmax(d->sod - reach, 1e-9 * d->sod);
            mag_min = d->sdd / (d->sod + reach);
            const double umax = (0.5 * d->ncols + std::fabs(d->shift_u) + 2.0) * d->pixel_u;
            const double gam = d->type == LEAP_CONE_CURVED ? std::fmin(umax / d->sdd, 1.57) : std::atan(umax / d->sdd);
            stretch = d->type == LEAP_CONE_CURVED ? 1.02 : 1.02 / std::cos(gam);     // no stretch on the cylinder
            slope = (gam < 0.78) ? std::tan(0.7853981633974483 + gam) : 1e30;
        }
        G->max_cols_per_voxel = mag_max * T * std::sqrt(2.0) / d->pixel_u * stretch;
        G->max_rows_per_voxel = (d->type == LEAP_FAN) ? 1.0 : mag_max * d->voxel_z / d->pixel_v;
        G->max_voxels_per_row = (d->type == LEAP_FAN) ? 1.0 : d->pixel_v / (mag_min * d->voxel_z);
        G->max_minor_slope = slope;
    }

    // Tiled back projection: pick the template instance and verify its staged window against every
    // (view, tile, z-chunk) with the very function the kernel evaluates.
    if (d->model == LEAP_MODEL_SF && d->type != LEAP_FAN && d->nz >= 8 && std::isfinite(G->max_cols_per_voxel) && G->max_cols_per_voxel <= 4.0 &&
        G->max_rows_per_voxel <= 3.0 && (double)d->nrows * d->ncols < 1073741824.0) {     // 32-bit byte offsets within a view
        G->bp_nc = (int)std::ceil(G->max_cols_per_voxel) + 1;
        if (G->bp_nc < 2) G->bp_nc = 2;
        G->bp_nv = (int)std::ceil(G->max_rows_per_voxel - 1e-6) + 1;
        if (G->bp_nv < 2) G->bp_nv = 2;
        G->bp_wh = (float)(0.5 * G->max_cols_per_voxel);
        const int tiles_x = (d->nx + BP_T - 1) / BP_T, tiles_y = (d->ny + BP_T - 1) / BP_T;
        const float hx = 0.5f * (float)(BP_T - 1) * g.T;
        int first_shape = d->nz >= 128 ? 0 : 1;       // 64-voxel chunks only pay off on tall volumes
        if (const char *env = std::getenv("LEAP_BP_SHAPE")) first_shape = std::atoi(env) % BP_NSHAPES;
        for (int sh = first_shape; sh < BP_NSHAPES && !G->bp_tiled; ++sh) {
            const int zc = BP_SHAPES[sh].zc;
            const int chunks = (d->nz + zc - 1) / zc;
            int need_w = 0, need_h = 0;
            for (int a = 0; a < d->nviews; ++a)
                for (int ty = 0; ty < tiles_y; ++ty)
                    for (int tx = 0; tx < tiles_x; ++tx) {
                        const float xc = (float)(g.x0d + ((double)(tx * BP_T) + 0.5 * (BP_T - 1)) * g.Td);
                        const float yc = (float)(g.y0d + ((double)(ty * BP_T) + 0.5 * (BP_T - 1)) * g.Td);
                        for (int ch = 0; ch < chunks; ch += (chunks > 1 ? chunks - 1 : 1)) {   // extremes: first and last chunk
                            const float z0 = (float)(g.zlo0d + (double)(ch * zc) * g.Tzd), z1 = z0 + (float)zc * g.Tz;
                            const SfWindow w = sf_bp_window(g, G->views[a], xc, yc, hx, z0, z1, G->bp_wh, G->bp_nc, G->bp_nv);
                            need_w = w.need_w > need_w ? w.need_w : need_w;
                            need_h = w.need_h > need_h ? w.need_h : need_h;
                        }
                    }
            G->bp_need_w = need_w;
            G->bp_need_h = need_h;
            G->bp_shape = sh;
            // one spare row and column: host and device floats may round apart
            G->bp_tiled = need_w <= BP_SHAPES[sh].pw - 1 && need_h <= BP_SHAPES[sh].ph - 1;
        }
        // Cylinder: the tiled kernel takes the angle between a voxel's centre and its corners from a short series,
        // good to 3e-9 rad below 0.08 rad.
        if (d->type == LEAP_CONE_CURVED) {
            const double rx = std::fabs(d->center_x) + 0.5 * d->nx * d->voxel_xy, ry = std::fabs(d->center_y) + 0.5 * d->ny * d->voxel_xy;
            const double nearest = d->sod - std::sqrt(rx * rx + ry * ry);
            if (!(0.7072 * d->voxel_xy <= 0.08 * nearest)) G->bp_tiled = false;
        }
    }

    // Column-wise forward projection: static limits, then its scratch copy of the volume.
    if (d->model == LEAP_MODEL_SF && d->type != LEAP_FAN && d->nrows >= 32 && std::isfinite(G->max_voxels_per_row) && G->max_voxels_per_row <= 3.0 &&
        (double)d->nx * d->ny * (d->nz + 2.0 * FP_PAD) < 4294967296.0 && d->ny <= 65535) {
        // tuning aids (read once per handle)
        if (const char *env = std::getenv("LEAP_FP_CW")) {
            const int v = std::atoi(env);
            if (v == 1 || v == 2 || v == 4) G->fp_cw = v;
        }
        if (d->type == LEAP_CONE_CURVED && G->fp_cw == 1) G->fp_cw = 2;      // the cylinder has instances for 4 and 2 columns
        // candidate slots per slab: widest range of voxel columns any bundle of cw detector columns can see
        auto slots_needed = [&](int cw) {
            int need = 0;
            for (int a = 0; a < d->nviews; ++a)
                for (int c = 0; c < d->ncols; c += cw) {
                    const SfRayLines L = sf_ray_lines(g, G->views[a], c, cw);
                    const int n_major = L.xmajor ? d->nx : d->ny;
                    const float d0 = std::fabs(L.b0 - L.b1);
                    const float d1 = std::fabs(fmaf(L.m0 - L.m1, (float)(n_major - 1), L.b0 - L.b1));
                    const float dm = d0 > d1 ? d0 : d1;
                    if (!(dm < 1e6f)) return 1 << 20;
                    const int cnt = (int)std::floor(dm + 2.0f * L.spread + 1e-3f) + 2;
                    need = cnt > need ? cnt : need;
                }
            return need;
        };
        G->fp_nk = (int)std::ceil(G->max_voxels_per_row - 1e-6) + 1;
        if (G->fp_nk < 2) G->fp_nk = 2;
        const int groups = (d->nrows + 63) / 64;
        G->fp_rg = groups >= 8 ? 8 : (groups >= 4 ? 4 : (groups >= 2 ? 2 : 1));
        if (const char *env = std::getenv("LEAP_FP_RG")) {
            const int v = std::atoi(env);
            if (v == 1 || v == 2 || v == 4 || v == 8) G->fp_rg = v;
        }
        // Short detectors (fewer than 256 rows) have too few bundles of four to fill the chip: two columns measured
        // 5 to 12 % faster there, four columns 5 to 10 % faster from 256 rows on.
        if (G->fp_cw == 4 && G->fp_rg < 4 && !std::getenv("LEAP_FP_CW")) G->fp_cw = 2;
        // the cylinder's record phase is heavier: four columns only pay off from 512 rows on (64.4 against 70.5 ms at 512^3)
        if (G->fp_cw == 4 && d->type == LEAP_CONE_CURVED && G->fp_rg < 8 && !std::getenv("LEAP_FP_CW")) G->fp_cw = 2;
        int need = slots_needed(G->fp_cw);
        while (need > 16 && G->fp_cw > 1) {
            G->fp_cw /= 2;
            need = slots_needed(G->fp_cw);
        }
        G->fp_need_q = need;
        G->fp_nq = need <= 4 ? 4 : (need <= 8 ? 8 : 16);
        G->fp_columns = need <= 16 && G->fp_nk <= 4 && (d->type != LEAP_CONE_CURVED || G->fp_cw >= 2);
        if (const char *env = std::getenv("LEAP_FP_VB")) {
            const int v = std::atoi(env);
            if (v >= 1 && v <= 1024) G->fp_vb = v;
        }
        if (const char *env = std::getenv("LEAP_FP_TB")) {
            const int v = std::atoi(env);
            if (v >= 1 && v <= 1024) G->fp_tb = v;
        }
    }

    if (d->model == LEAP_MODEL_SIDDON) select_siddon_fast_kernels(G);

    // Testing aid: LEAP_FORCE_GENERAL=1 keeps every call on the general kernels.
    if (const char *env = std::getenv("LEAP_FORCE_GENERAL"))
        if (env[0] == '1') G->bp_tiled = G->fp_columns = G->sd_columns = false;

    hipError_t e = hipGetDevice(&G->device);
    if (e == hipSuccess) (void)leap_static_scratch_init(G->device);   // set-up for leap_project_static_scratch; it reports a failure itself
    if (e == hipSuccess) e = hipMalloc((void **)&G->d_views, sizeof(SfView) * (size_t)d->nviews);
    if (e == hipSuccess) e = hipMemcpy(G->d_views, G->views.data(), sizeof(SfView) * (size_t)d->nviews, hipMemcpyHostToDevice);
    if (e == hipSuccess && (G->fp_columns || G->sd_columns)) {
        G->nzp = d->nz + 2 * FP_PAD;
        // one more column than the volume has: it stays zero and stands for cells outside the volume (Siddon kernel)
        const size_t item_bytes = sizeof(float) * ((size_t)d->nx * d->ny + 1) * G->nzp;
        // Small volumes (a batch of training volumes): up to 16 scratch copies within 1 GiB, so that the footprint
        // kernel can take that many items of a batch in one launch.
        {
            const size_t fit = ((size_t)1 << 30) / item_bytes;
            G->volz_items = (int)(fit < 1 ? 1 : (fit > 16 ? 16 : fit));
        }
        size_t bytes = item_bytes * (size_t)G->volz_items;
        hipError_t es = hipMalloc((void **)&G->d_volz, bytes);
        if (es != hipSuccess && G->volz_items > 1) {                      // one copy at least
            (void)hipGetLastError();
            G->volz_items = 1;
            bytes = item_bytes;
            es = hipMalloc((void **)&G->d_volz, bytes);
        }
        if (es == hipSuccess) es = hipMemset(G->d_volz, 0, bytes);       // the pads stay zero for the handle's life
        if (es == hipSuccess) es = hipDeviceSynchronize();
        if (es != hipSuccess) {                                           // no room for the copy: use the general kernel
            if (G->d_volz) (void)hipFree(G->d_volz);
            G->d_volz = nullptr;
            G->fp_columns = G->sd_columns = false;
            (void)hipGetLastError();
        }
    }
    if (e == hipSuccess && !G->raycols.empty()) {
        const size_t bytes = sizeof(SdRayCol) * G->raycols.size();
        e = hipMalloc((void **)&G->d_raycols, bytes);
        if (e == hipSuccess) e = hipMemcpy(G->d_raycols, G->raycols.data(), bytes, hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && d->type == LEAP_CONE_CURVED && d->model == LEAP_MODEL_SF && G->bp_tiled) {
        // For the tiled back projection: cosine and sine of every detector column's fan angle (ray amplitudes), then
        // per (tile, view) the tile centre's fan angle and the tile's window bounds.
        const int tiles_x = (d->nx + BP_T - 1) / BP_T, tiles_y = (d->ny + BP_T - 1) / BP_T;
        const size_t head = 2 * sizeof(float) * (size_t)d->ncols;
        const size_t bytes = head + sizeof(SfCurvedBounds) * (size_t)tiles_x * tiles_y * d->nviews;
        std::vector<unsigned char> blob(bytes);
        float *cs = reinterpret_cast<float *>(blob.data());
        for (int c = 0; c < d->ncols; ++c) {
            const double gam = ((double)c - g.col_offd) * d->pixel_u / d->sdd;
            cs[2 * (size_t)c] = (float)std::cos(gam);
            cs[2 * (size_t)c + 1] = (float)std::sin(gam);
        }
        SfCurvedBounds *tab = reinterpret_cast<SfCurvedBounds *>(blob.data() + head);
        const float hx = 0.5f * (float)(BP_T - 1) * g.T;
        for (int ty = 0; ty < tiles_y; ++ty)
            for (int tx = 0; tx < tiles_x; ++tx) {
                const double xcd = g.x0d + ((double)(tx * BP_T) + 0.5 * (BP_T - 1)) * g.Td;
                const double ycd = g.y0d + ((double)(ty * BP_T) + 0.5 * (BP_T - 1)) * g.Td;
                SfCurvedBounds *row = tab + ((size_t)ty * tiles_x + tx) * d->nviews;
                for (int a = 0; a < d->nviews; ++a) {
                    const SfView &v = G->views[a];
                    row[a].gref = std::atan2(std::fma(ycd, v.cd, -xcd * v.sd), g.sodd - std::fma(xcd, v.cd, ycd * v.sd));
                    sf_curved_tile_bounds(g, v, (float)xcd, (float)ycd, hx, row[a].xi_lo, row[a].xi_hi, row[a].ilo, row[a].ihi);
                }
            }
        hipError_t et = hipMalloc((void **)&G->d_colcs, bytes);
        if (et == hipSuccess) et = hipMemcpy(G->d_colcs, blob.data(), bytes, hipMemcpyHostToDevice);
        if (et != hipSuccess) {                       // no room for the tables: the general kernel needs none
            if (G->d_colcs) (void)hipFree(G->d_colcs);
            G->d_colcs = nullptr;
            G->bp_tiled = false;
            (void)hipGetLastError();
        }
    }
    if (e != hipSuccess) {
        if (G->d_colcs) (void)hipFree(G->d_colcs);
        if (G->d_views) (void)hipFree(G->d_views);
        if (G->d_volz) (void)hipFree(G->d_volz);
        if (G->d_raycols) (void)hipFree(G->d_raycols);
        delete G;
        return leap_hip_fail(e, "uploading the view table");
    }
    *out = G;
    return LEAP_OK;
}

extern "C" void leap_geometry_destroy(leap_geometry *G)
{
    if (!G) return;
    if (G->d_views) (void)hipFree(G->d_views);
    if (G->d_volz) (void)hipFree(G->d_volz);
    if (G->d_raycols) (void)hipFree(G->d_raycols);
    if (G->d_poses) (void)hipFree(G->d_poses);
    if (G->d_geoms) (void)hipFree(G->d_geoms);
    if (G->d_colcs) (void)hipFree(G->d_colcs);
    delete G;
}

extern "C" int leap_geometry_describe(const leap_geometry *G, char *buf, int32_t cap)
{
    if (!G || !buf || cap <= 0) return invalid("null handle or buffer");
    if (G->g.type == SF_MODULAR) {
        if (G->g.model == SF_MODEL_SIDDON)
            std::snprintf(buf, (size_t)cap, "type=4 model=siddon A=%s(rg=%d) AT=%s(nc=%d,zc=%d,window=%dx%d) %s",
                          G->sd_columns ? "columns" : "general", G->fp_rg, G->bp_tiled ? "tiled" : "general", G->bp_nc,
                          BP_SHAPES[G->bp_shape].zc, G->bp_need_w, G->bp_need_h,
                          G->geoms.empty() ? "(tilted modules: one thread per ray / per voxel)" : "(upright modules)");
        else
            std::snprintf(buf, (size_t)cap, "type=4 model=sf A=%s(nq=%d/%d,nk=%d,rg=%d) AT=%s(nc=%d,nv=%d,zc=%d,window=%dx%d) "
                          "cols/voxel<=%.2f rows/voxel<=%.2f voxels/row<=%.2f", G->fp_columns ? "columns" : "general", G->fp_need_q,
                          G->fp_nq, G->fp_nk, G->fp_rg, G->bp_tiled ? "tiled" : "general", G->bp_nc, G->bp_nv,
                          BP_SHAPES[G->bp_shape].zc, G->bp_need_w, G->bp_need_h, G->max_cols_per_voxel, G->max_rows_per_voxel,
                          G->max_voxels_per_row);
        return LEAP_OK;
    }
    if (G->g.model == SF_MODEL_SIDDON) {
        std::snprintf(buf, (size_t)cap, "type=%d model=siddon A=%s(rg=%d) AT=%s(nc=%d,zc=%d,window=%dx%d) axial-slope<=%.3f "
                      "cols/voxel<=%.2f", G->g.type, G->sd_columns ? "columns" : "general", G->fp_rg,
                      G->bp_tiled ? "tiled" : "general", G->bp_nc, BP_SHAPES[G->bp_shape].zc, G->bp_need_w, G->bp_need_h,
                      G->sd_max_axial_slope, G->max_cols_per_voxel);
        return LEAP_OK;
    }
    std::snprintf(buf, (size_t)cap,
                  "type=%d A=%s(nq=%d/%d,nk=%d,rg=%d,w=%d,cw=%d,wv=%d) AT=%s(nc=%d,nv=%d,zc=%d,window=%dx%d) cols/voxel<=%.2f rows/voxel<=%.2f "
                  "voxels/row<=%.2f slope<=%.2f",
                  G->g.type, G->fp_columns ? "columns" : "general", G->fp_need_q, G->fp_nq, G->fp_nk, G->fp_rg, G->fp_waves, G->fp_cw, G->fp_wv, G->bp_tiled ? "tiled" : "general", G->bp_nc, G->bp_nv, BP_SHAPES[G->bp_shape].zc, G->bp_need_w, G->bp_need_h,
                  G->max_cols_per_voxel, G->max_rows_per_voxel, G->max_voxels_per_row, G->max_minor_slope);
    return LEAP_OK;
}

static int check_call(const leap_geometry *G, const void *in, const void *out, int32_t batch)
{
    if (!G || !in || !out) return invalid("null handle or data pointer");
    if (batch <= 0) return invalid("batch must be positive");
    if (in == out) return invalid("input and output must not alias");
    return LEAP_OK;
}

extern "C" int leap_project(const leap_geometry *G, const float *d_vol, float *d_sino, int32_t batch, void *hip_stream)
{
    int rc = check_call(G, d_vol, d_sino, batch);
    if (rc != LEAP_OK) return rc;
    const size_t nvol = (size_t)G->g.nx * G->g.ny * G->g.nz, nsino = (size_t)G->g.nviews * G->g.nrows * G->g.ncols;
    (void)nvol; (void)nsino;
    return leap_launch_project_batch(G, d_vol, d_sino, batch, (hipStream_t)hip_stream);
}

extern "C" int leap_backproject(const leap_geometry *G, const float *d_sino, float *d_vol, int32_t batch, void *hip_stream)
{
    int rc = check_call(G, d_sino, d_vol, batch);
    if (rc != LEAP_OK) return rc;
    const size_t nvol = (size_t)G->g.nx * G->g.ny * G->g.nz, nsino = (size_t)G->g.nviews * G->g.nrows * G->g.ncols;
    (void)nvol; (void)nsino;
    return leap_launch_backproject_batch(G, d_sino, d_vol, batch, (hipStream_t)hip_stream);
}
